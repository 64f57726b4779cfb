"""Counter-based random numbers for the synthetic inputs.

Every value is a pure function of (seed, stream, index), so a tensor can be
generated in chunks, on the CPU or on a GPU, and comes out the same.  The
mixer is the SplitMix64 finaliser (Steele, Lea, Flood 2014), evaluated on
torch int64 tensors: int64 multiplication wraps like uint64, and the logical
right shifts are done as an arithmetic shift followed by a mask.

This module is input generation only.  It holds nothing of the method.
"""
import math

import torch


def _s64(x: int) -> int:
    """Reinterpret an unsigned 64-bit constant as a signed Python int."""
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    return (z >> k) & ((1 << (64 - k)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = z + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _mix_int(z: int) -> int:
    m = (1 << 64) - 1
    z = (z + 0x9E3779B97F4A7C15) & m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """Scalar key of one random stream (signed 64-bit)."""
    return _s64(_mix_int(_mix_int(seed & ((1 << 64) - 1)) ^ (stream & ((1 << 64) - 1))))


def bits(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """64 random bits (as int64) for every entry of `index` (int64)."""
    return _mix(index.to(torch.int64) + stream_key(seed, stream))


def uniform01(seed: int, stream: int, index: torch.Tensor) -> torch.Tensor:
    """float64 in [0, 1) with 53 random bits."""
    return _lsr(bits(seed, stream, index), 11).to(torch.float64) * (2.0 ** -53)


def randint(seed: int, stream: int, index: torch.Tensor, n) -> torch.Tensor:
    """int64 in [0, n); `n` is an int or an int64 tensor broadcastable to index."""
    return _lsr(bits(seed, stream, index), 1) % n


def normal(seed: int, stream: int, start: int, count: int, device="cpu",
           dtype=torch.float32) -> torch.Tensor:
    """`count` N(0,1) samples for indices start..start+count-1 (Box-Muller,
    one sample per index, evaluated in float32)."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    b1 = _lsr(bits(seed, stream, idx * 2), 40)          # 24 bits
    b2 = _lsr(bits(seed, stream, idx * 2 + 1), 40)
    u1 = (b1.to(torch.float32) + 1.0) * (2.0 ** -24)    # (0, 1]
    u2 = b2.to(torch.float32) * (2.0 ** -24)            # [0, 1)
    z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
    return z.to(dtype)


def normal_matrix(seed: int, stream: int, rows: int, cols: int, device="cpu",
                  dtype=torch.float32, chunk_rows: int = 1 << 20) -> torch.Tensor:
    """[rows, cols] N(0,1), entry (i, j) drawn at index i*cols+j, rounded to `dtype`."""
    out = torch.empty((rows, cols), dtype=dtype, device=device)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = normal(seed, stream, r0 * cols, (r1 - r0) * cols, device, dtype).view(r1 - r0, cols)
    return out


def glorot_uniform(seed: int, stream: int, fan_in: int, fan_out: int, device="cpu",
                   dtype=torch.float32) -> torch.Tensor:
    """[fan_in, fan_out] uniform in +-sqrt(6/(fan_in+fan_out)), row-major."""
    idx = torch.arange(fan_in * fan_out, dtype=torch.int64, device=device)
    a = math.sqrt(6.0 / (fan_in + fan_out))
    u = uniform01(seed, stream, idx)
    return ((2.0 * u - 1.0) * a).to(dtype).view(fan_in, fan_out)


def permutation(seed: int, stream: int, n: int) -> torch.Tensor:
    """Seeded permutation of 0..n-1 (argsort of hashes, ties by index)."""
    idx = torch.arange(n, dtype=torch.int64)
    h = _lsr(bits(seed, stream, idx), 1)
    return torch.argsort(h * 1, stable=True)


def ball_matrix(seed: int, stream: int, n: int, f: int, radius: float, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """n points drawn uniformly from the closed ball of the given radius in R^f, one per row: a Gaussian
    direction scaled to length radius * u^(1/f)."""
    g = normal_matrix(seed, stream, n, f, device, torch.float32).double()
    u = uniform01(seed, stream + 1, torch.arange(n, dtype=torch.int64, device=device))
    r = radius * u ** (1.0 / f)
    return (g / g.norm(dim=1, keepdim=True).clamp_min(1e-300) * r[:, None]).to(dtype)
