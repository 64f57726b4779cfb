"""The entry point that allocates nothing (gas_linear_bwd_weight_static: slab partials in a static device array of
the library) against the entry point it is a variant of (gas_linear_bwd_weight with a caller's workspace), through
the C ABI: two calls in a row, the second on a smaller input, then the size limit."""
import numpy as np
import pytest
import torch

from gas_inputs import rng
from oracle import ops as oops
from tests.util import to_np, max_rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_static_scratch_variant_matches_the_workspace_variant(dtype):
    import paper_2106_05609_amd as gas
    gas.lib()
    # large first (its partials stay behind in the shared array), then smaller and ragged shapes
    for M, K, N in [(70000, 256, 256), (4097, 128, 256), (300, 15, 20), (9000, 72, 200), (1, 8, 8)]:
        z = rng.normal_matrix(9, 620, M, K, dtype=dtype).to("cuda")
        gp = rng.normal_matrix(9, 621, M, N, dtype=dtype).to("cuda")
        nbytes = gas.gas_linear_bwd_weight_workspace(M, K, N)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        want_dev = torch.full((K, N), float("nan"), device="cuda")
        gas.gas_linear_bwd_weight(z, gp, want_dev, ws, c_weight=0.5)
        got = torch.full((K, N), float("nan"), device="cuda")
        gas.gas_linear_bwd_weight_static(z, gp, got, c_weight=0.5)
        torch.cuda.synchronize()
        assert torch.equal(got, want_dev), (M, K, N)                   # same kernels, same slabs: same bits
        want = oops.linear_bwd_weight(to_np(z), to_np(gp), c_weight=0.5)
        assert max_rel_err(to_np(got), want) <= 1e-5, (M, K, N)
    # an empty sum is a zero matrix
    got = torch.full((8, 8), float("nan"), device="cuda")
    gas.gas_linear_bwd_weight_static(torch.empty((0, 8), dtype=dtype, device="cuda"),
                                     torch.empty((0, 8), dtype=dtype, device="cuda"), got)
    assert not got.any()


def test_static_scratch_variant_rejects_shapes_beyond_its_array():
    import paper_2106_05609_amd as gas
    M = 1_200_000                                                      # 293 slabs of 256 KiB > 64 MiB
    assert gas.gas_linear_bwd_weight_workspace(M, 256, 256) > 64 << 20
    z = torch.zeros((M, 256), dtype=torch.bfloat16, device="cuda")
    dw = torch.full((256, 256), 3.0, device="cuda")
    with pytest.raises(gas.GasError) as e:
        gas.gas_linear_bwd_weight_static(z, z, dw)
    assert e.value.status == -1 and "64" in str(e.value) or "67108864" in str(e.value)
    torch.cuda.synchronize()
    assert (dw == 3.0).all()                                           # nothing was launched
