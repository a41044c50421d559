// Per-key aggregation structure of a step (the "aggregate per key" stage): from the list of keys
// a step accesses in one table, build the distinct keys in ascending order, their access counts
// and the accesses grouped by key.  Keys are bounded by the table size, so the distinct set is a
// bitmap over the key space and a key's position among the distinct keys is a prefix population
// count; no comparison sort is needed.  Up to two tables are planned by the same launches
// (blockIdx.y selects the table).
#include <algorithm>
#include <initializer_list>

#include "device_utils.h"

namespace nups {

struct PlanPair {
    PlanArgs p[2];
};

// Marks the keys of the step in the bitmap; flags keys outside the table.
__global__ void __launch_bounds__(kBlock) k_plan_mark(PlanPair pp)
{
    const PlanArgs &a = pp.p[blockIdx.y];
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i == 0) a.meta[kMetaNumLong] = 0;
    if (i >= a.n) return;
    const uint32_t key = source_key(a.src, i);
    if (key >= a.num_keys) { atomicOr(a.error_flag, 1u); return; }
    atomicOr(&a.bitmap[key >> 5], 1u << (key & 31));
}

// Population count of each tile of kScanTile bitmap words.
__global__ void __launch_bounds__(kBlock) k_plan_bitmap_tiles(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.bitmap_tiles) return;
    const uint32_t w0 = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j)
        if (w0 + j < a.words) c += __popc(a.bitmap[w0 + j]);
    const uint32_t s = block_sum(c, lds);
    if (threadIdx.x == 0) a.tile_sum[blockIdx.x] = s;
}

// Rank of every bitmap word among the distinct keys; emits the distinct keys and clears their counts.
__global__ void __launch_bounds__(kBlock) k_plan_bitmap_scan(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.bitmap_tiles) return;
    uint32_t before = 0;
    for (uint32_t t = threadIdx.x; t < blockIdx.x; t += kBlock) before += a.tile_sum[t];
    before = block_sum(before, lds);
    const uint32_t w0 = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t bits[kScanItems];
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        bits[j] = (w0 + j < a.words) ? a.bitmap[w0 + j] : 0u;
        c += __popc(bits[j]);
    }
    uint32_t total;
    uint32_t run = before + block_exclusive_scan(c, lds, &total);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (w0 + j < a.words) a.word_rank[w0 + j] = run;
        uint32_t b = bits[j];
        while (b) {
            const uint32_t bit = __ffs(b) - 1;
            b &= b - 1;
            a.uniq[run] = (w0 + j) * 32 + bit;
            a.count[run] = 0;
            ++run;
        }
    }
    if (blockIdx.x == a.bitmap_tiles - 1 && threadIdx.x == 0) a.meta[kMetaNumUniq] = before + total;
}

// Per access: which distinct key it belongs to and its position inside that key's segment.
__global__ void __launch_bounds__(kBlock) k_plan_rank(PlanPair pp)
{
    const PlanArgs &a = pp.p[blockIdx.y];
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= a.n) return;
    const uint32_t key = source_key(a.src, i);
    if (key >= a.num_keys) { a.slot[i] = kBadIndex; return; }
    const uint32_t w = key >> 5, b = key & 31;
    const uint32_t u = a.word_rank[w] + __popc(a.bitmap[w] & ((1u << b) - 1u));
    a.slot[i] = u;
    a.rank[i] = atomicAdd(&a.count[u], 1u);
}

// Sum of each tile of kScanTile access counts.
__global__ void __launch_bounds__(kBlock) k_plan_count_tiles(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.count_tiles) return;
    const uint32_t nu = a.meta[kMetaNumUniq];
    const uint32_t u0 = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j)
        if (u0 + j < nu) c += a.count[u0 + j];
    const uint32_t s = block_sum(c, lds);
    if (threadIdx.x == 0) a.tile_sum[blockIdx.x] = s;
}

// Segment offsets = exclusive prefix sums of the counts; lists the long segments.
__global__ void __launch_bounds__(kBlock) k_plan_count_scan(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.count_tiles) return;
    const uint32_t nu = a.meta[kMetaNumUniq];
    const uint32_t u0 = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    if (blockIdx.x * kScanTile >= nu && blockIdx.x != 0) return;
    uint32_t before = 0;
    for (uint32_t t = threadIdx.x; t < blockIdx.x; t += kBlock) before += a.tile_sum[t];
    before = block_sum(before, lds);
    uint32_t cnt[kScanItems];
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        cnt[j] = (u0 + j < nu) ? a.count[u0 + j] : 0u;
        c += cnt[j];
    }
    uint32_t total;
    uint32_t run = before + block_exclusive_scan(c, lds, &total);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (u0 + j < nu) {
            a.seg[u0 + j] = run;
            if (cnt[j] > kLongSegment) a.long_list[atomicAdd(&a.meta[kMetaNumLong], 1u)] = u0 + j;
        }
        run += cnt[j];
        if (u0 + j + 1 == nu || (nu == 0 && u0 + j == 0)) {   // end marker seg[nu]
            a.seg[nu] = run;
            a.meta[kMetaTotal] = run;
        }
    }
}

// Groups the accesses by key and returns the bitmap to all-zero for the next step.
__global__ void __launch_bounds__(kBlock) k_plan_scatter(PlanPair pp)
{
    const PlanArgs &a = pp.p[blockIdx.y];
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= a.n) return;
    const uint32_t u = a.slot[i];
    if (u == kBadIndex) return;
    a.perm[a.seg[u] + a.rank[i]] = i;
    a.bitmap[source_key(a.src, i) >> 5] = 0u;
}

static nups_status grow_u32(uint32_t **buf, size_t n, bool zero, hipStream_t stream)
{
    if (*buf) NUPS_HIP(hipFree(*buf));
    *buf = nullptr;
    NUPS_HIP(hipMalloc((void **)buf, sizeof(uint32_t) * (n ? n : 1)));
    if (zero) NUPS_HIP(hipMemsetAsync(*buf, 0, sizeof(uint32_t) * (n ? n : 1), stream));
    return NUPS_OK;
}

nups_status ensure_plan_capacity(nups_ctx *ctx, Table &t, size_t n)
{
    Plan &pl = t.plan;
    PlanArgs &a = pl.a;
    const size_t words = (size_t)((t.num_keys + 31) / 32);
    if (pl.cap_words < words) {
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        nups_status st;
        if ((st = grow_u32(&a.bitmap, words, true, ctx->stream)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.word_rank, words, false, ctx->stream)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.meta, kMetaWords, true, ctx->stream)) != NUPS_OK) return st;
        pl.cap_words = words;
    }
    if (pl.cap_n < n || pl.cap_n == 0) {
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        const size_t cap = n + n / 4 + 1024;
        nups_status st;
        for (uint32_t **b : {&a.uniq, &a.count, &a.slot, &a.rank, &a.perm})
            if ((st = grow_u32(b, cap, false, ctx->stream)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.seg, cap + 1, false, ctx->stream)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.long_list, cap / kLongSegment + 2, false, ctx->stream)) != NUPS_OK) return st;
        pl.cap_n = cap;
    }
    const size_t tiles = std::max((words + kScanTile - 1) / kScanTile, (pl.cap_n + kScanTile - 1) / kScanTile);
    if (pl.cap_tiles < tiles) {
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        nups_status st;
        if ((st = grow_u32(&a.tile_sum, tiles, false, ctx->stream)) != NUPS_OK) return st;
        pl.cap_tiles = tiles;
    }
    a.num_keys = (uint32_t)t.num_keys;
    a.words = (uint32_t)words;
    a.bitmap_tiles = (uint32_t)((words + kScanTile - 1) / kScanTile);
    a.error_flag = ctx->error_flag;
    return NUPS_OK;
}

// Enqueues the plan construction for one or two tables (a.src, a.n already set by the caller).
nups_status build_plans(nups_ctx *ctx, Plan **plans, int n_plans)
{
    if (n_plans < 1 || n_plans > 2) return fail(NUPS_ERR_ARG, "build_plans: one or two plans");
    PhaseScope scope(ctx, NUPS_PHASE_PLAN);
    PlanPair pp;
    uint32_t max_n = 0, max_btiles = 0, max_ctiles = 0;
    for (int k = 0; k < n_plans; ++k) {
        PlanArgs &a = plans[k]->a;
        a.count_tiles = (a.n + kScanTile - 1) / kScanTile;
        if (a.count_tiles == 0) a.count_tiles = 1;   // still writes seg[0] and the totals for an empty step
        pp.p[k] = a;
        max_n = std::max(max_n, a.n);
        max_btiles = std::max(max_btiles, a.bitmap_tiles);
        max_ctiles = std::max(max_ctiles, a.count_tiles);
        plans[k]->valid = true;
    }
    if (n_plans == 1) pp.p[1] = pp.p[0];
    const dim3 blk(kBlock);
    const uint32_t nblocks = std::max(1u, (max_n + kBlock - 1) / kBlock);
    hipStream_t s = ctx->stream;
    hipLaunchKernelGGL(k_plan_mark, dim3(nblocks, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_bitmap_tiles, dim3(max_btiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_bitmap_scan, dim3(max_btiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_rank, dim3(nblocks, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_count_tiles, dim3(max_ctiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_count_scan, dim3(max_ctiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_scatter, dim3(nblocks, n_plans), blk, 0, s, pp);
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

}  // namespace nups
