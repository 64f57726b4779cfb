/*
 * A trace-driven model of the eight L2 caches under the aggregation's launch order (bench/l2_model.py drives it).
 * Each XCD is a set-associative LRU cache of `slots` feature rows.  An XCD's work items (begin, end: a range of the
 * gathered index array) are taken in the order given; `nconc` of them are in flight at once and advance in turn,
 * `step` gathers each, which is how wavefronts of one XCD interleave.  An access flagged in `cold` is inserted at
 * the old end of its set's ages (a gather that is not meant to displace anything).  Returns the misses; hits in *hits.
 */
#include <stdint.h>
#include <stdlib.h>

typedef struct { int32_t* tag; uint32_t* age; int sets, ways; uint32_t clock; } cache_t;

static void cache_init(cache_t* c, int slots, int ways) {
    c->ways = ways;
    c->sets = slots / ways;
    c->tag = (int32_t*)malloc(sizeof(int32_t) * (size_t)slots);
    c->age = (uint32_t*)calloc((size_t)slots, 4);
    for (int i = 0; i < slots; ++i) c->tag[i] = -1;
    c->clock = 0;
}

static int cache_access(cache_t* c, int32_t row, int cold) {
    const uint32_t h = (uint32_t)row * 2654435761u;
    const int s = (int)((h >> 8) % (uint32_t)c->sets);
    int32_t* t = c->tag + (size_t)s * c->ways;
    uint32_t* a = c->age + (size_t)s * c->ways;
    c->clock++;
    int old = 0;
    for (int w = 0; w < c->ways; ++w) {
        if (t[w] == row) {
            if (!cold) a[w] = c->clock;
            return 1;
        }
        if (a[w] < a[old]) old = w;
    }
    t[old] = row;
    a[old] = cold ? (c->clock > 4096 ? c->clock - 4096 : 1) : c->clock;
    return 0;
}

long long l2_model(const int32_t* index, const int32_t* items, const int32_t* xcd_start, int slots, int ways, int nconc,
                   int step, const uint8_t* cold, long long* hits) {
    long long miss = 0, hit = 0;
    for (int x = 0; x < 8; ++x) {
        cache_t c;
        cache_init(&c, slots, ways);
        const int hi = xcd_start[x + 1];
        int next = xcd_start[x];
        int* cur = (int*)malloc(sizeof(int) * (size_t)nconc);
        int* end = (int*)malloc(sizeof(int) * (size_t)nconc);
        int active = 0;
        for (int i = 0; i < nconc && next < hi; ++i, ++next) { cur[active] = items[2 * next]; end[active] = items[2 * next + 1]; ++active; }
        while (active > 0) {
            for (int i = 0; i < active;) {
                for (int k = 0; k < step && cur[i] < end[i]; ++k, ++cur[i]) {
                    if (cache_access(&c, index[cur[i]], cold ? cold[cur[i]] : 0)) ++hit;
                    else ++miss;
                }
                if (cur[i] < end[i]) { ++i; continue; }
                if (next < hi) { cur[i] = items[2 * next]; end[i] = items[2 * next + 1]; ++next; ++i; }
                else { cur[i] = cur[active - 1]; end[i] = end[active - 1]; --active; }
            }
        }
        free(cur); free(end); free(c.tag); free(c.age);
    }
    *hits = hit;
    return miss;
}
