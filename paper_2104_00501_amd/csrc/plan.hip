// Per-key aggregation structure of a step (the "aggregate per key" stage): from the list of keys
// a step accesses in one table, build the distinct keys in ascending order, their access counts
// and the accesses grouped by key.  Keys are bounded by the table size, so the distinct set is a
// bitmap over the key space and a key's position among the distinct keys is a prefix population
// count; no comparison sort is needed.  Up to two tables are planned by the same launches
// (blockIdx.y selects the table).
//
// Hot keys (Section 3.2: a few keys take a large share of the accesses) would serialise global
// atomics, so every workgroup first combines its own accesses to a key in LDS and issues one
// global atomic per distinct key; segments that are too long for one row group are cut into
// chunks that separate workgroups sum.
#include <algorithm>
#include <initializer_list>

#include "device_utils.h"

namespace nups {

struct PlanPair {
    PlanArgs p[2];
};

constexpr int kRankItems = 1;                       // accesses per thread in k_plan_mark / k_plan_rank
constexpr int kRankTile = kBlock * kRankItems;
constexpr int kHashBits = 9;
constexpr uint32_t kHashSlots = 1u << kHashBits;    // open-addressing table in LDS, at most half full
static_assert(kHashSlots >= 2 * kRankTile, "the LDS hash table must stay at most half full");

// Marks the keys of the step in the bitmap; flags keys outside the table.
__global__ void __launch_bounds__(kBlock) k_plan_mark(PlanPair pp)
{
    // The bits of one workgroup's keys are first OR-ed together per bitmap word in an LDS hash table,
    // so that a hot word receives one global atomic per workgroup instead of one per access.
    __shared__ uint32_t hword[kHashSlots], hbits[kHashSlots];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        a.meta[kMetaNumChunks] = 0;
        if (a.zero_loss) *a.zero_loss = 0.0;   // the step's loss accumulator starts from zero
    }
    if (blockIdx.x * kRankTile >= a.n) return;
    for (uint32_t s = threadIdx.x; s < kHashSlots; s += kBlock) { hword[s] = kBadIndex; hbits[s] = 0; }
    __syncthreads();
    bool bad = false;
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        const uint32_t i = blockIdx.x * kRankTile + j * kBlock + threadIdx.x;
        if (i < a.n) {
            const uint32_t key = source_key(a.src, i);
            if (key >= a.num_keys) { bad = true; continue; }
            const uint32_t w = key >> 5;
            uint32_t s = (w * 2654435761u) >> (32 - kHashBits);
            for (;;) {   // ends: at most kRankTile distinct words in 2 * kRankTile slots
                const uint32_t old = atomicCAS(&hword[s], kBadIndex, w);
                if (old == kBadIndex || old == w) break;
                s = (s + 1) & (kHashSlots - 1);
            }
            atomicOr(&hbits[s], 1u << (key & 31));
        }
    }
    if (bad) atomicOr(a.error_flag, 1u);
    __syncthreads();
    for (uint32_t s = threadIdx.x; s < kHashSlots; s += kBlock)
        if (hbits[s]) atomicOr(&a.bitmap[hword[s]], hbits[s]);
}

// Sum of `items[0 .. end)` (popcounts if POPC) over the whole workgroup; every thread gets the result.
// `items` is 16-byte aligned; whole uint4 are read, four per thread and iteration, then the tail.
template <bool POPC>
__device__ __forceinline__ uint32_t block_sum_range(const uint32_t *items, uint32_t end, uint32_t *lds)
{
    uint32_t c = 0;
    const uint4 *v = reinterpret_cast<const uint4 *>(items);
    const uint32_t n4 = end / 4;
    auto add = [&](const uint4 x) {
        c += POPC ? (__popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w)) : (x.x + x.y + x.z + x.w);
    };
    uint32_t q = threadIdx.x;
    for (; q + 3 * kBlock < n4; q += 4 * kBlock) {
        const uint4 x0 = v[q], x1 = v[q + kBlock], x2 = v[q + 2 * kBlock], x3 = v[q + 3 * kBlock];
        add(x0); add(x1); add(x2); add(x3);
    }
    for (; q < n4; q += kBlock) add(v[q]);
    for (uint32_t w = n4 * 4 + threadIdx.x; w < end; w += kBlock) c += POPC ? __popc(items[w]) : items[w];
    return block_sum(c, lds);
}

// Population count of each tile of kScanTile bitmap words (large key spaces only).
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
// With `direct` set each workgroup counts the bits below its tile itself (small key spaces) and
// k_plan_bitmap_tiles is not needed.
__global__ void __launch_bounds__(kBlock) k_plan_bitmap_scan(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.bitmap_tiles) return;
    uint32_t before;
    if (a.direct_bitmap) before = block_sum_range<true>(a.bitmap, blockIdx.x * kScanTile, lds);
    else before = block_sum_range<false>(a.tile_sum, blockIdx.x, lds);
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
// The workgroup's accesses are first grouped by key in an LDS hash table; one global atomic per
// distinct key and workgroup reserves a run of positions, which the LDS counts subdivide.
__global__ void __launch_bounds__(kBlock) k_plan_rank(PlanPair pp)
{
    __shared__ uint32_t hkey[kHashSlots], hcnt[kHashSlots], hbase[kHashSlots];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x * kRankTile >= a.n) return;
    for (uint32_t s = threadIdx.x; s < kHashSlots; s += kBlock) { hkey[s] = kBadIndex; hcnt[s] = 0; }
    __syncthreads();
    uint32_t slot_of[kRankItems], local[kRankItems], uidx[kRankItems];
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        const uint32_t i = blockIdx.x * kRankTile + j * kBlock + threadIdx.x;
        uidx[j] = kBadIndex;
        if (i < a.n) {
            const uint32_t key = source_key(a.src, i);
            if (key < a.num_keys) {
                const uint32_t w = key >> 5, b = key & 31;
                const uint32_t u = a.word_rank[w] + __popc(a.bitmap[w] & ((1u << b) - 1u));
                uidx[j] = u;
                uint32_t s = (u * 2654435761u) >> (32 - kHashBits);
                for (;;) {   // ends: at most kRankTile distinct keys in 2 * kRankTile slots
                    const uint32_t old = atomicCAS(&hkey[s], kBadIndex, u);
                    if (old == kBadIndex || old == u) break;
                    s = (s + 1) & (kHashSlots - 1);
                }
                slot_of[j] = s;
                local[j] = atomicAdd(&hcnt[s], 1u);
            }
        }
    }
    __syncthreads();
    for (uint32_t s = threadIdx.x; s < kHashSlots; s += kBlock)
        if (hcnt[s]) hbase[s] = atomicAdd(&a.count[hkey[s]], hcnt[s]);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        const uint32_t i = blockIdx.x * kRankTile + j * kBlock + threadIdx.x;
        if (i < a.n) {
            a.slot[i] = uidx[j];
            if (uidx[j] != kBadIndex) a.rank[i] = hbase[slot_of[j]] + local[j];
        }
    }
}

// Sum of each tile of kScanTile access counts (large steps only).
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

// Segment offsets = exclusive prefix sums of the counts; cuts long segments into chunks.
__global__ void __launch_bounds__(kBlock) k_plan_count_scan(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.count_tiles) return;
    const uint32_t nu = a.meta[kMetaNumUniq];
    const uint32_t u0 = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    if (blockIdx.x * kScanTile >= nu && blockIdx.x != 0) return;
    uint32_t before;
    if (a.direct_count) before = block_sum_range<false>(a.count, min(blockIdx.x * kScanTile, nu), lds);
    else before = block_sum_range<false>(a.tile_sum, blockIdx.x, lds);
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
            if (cnt[j] > kLongSegment) {
                const uint32_t nch = (cnt[j] + kChunk - 1) / kChunk;
                const uint32_t base = atomicAdd(&a.meta[kMetaNumChunks], nch);
                for (uint32_t ch = 0; ch < nch; ++ch) {
                    a.chunk_seg[base + ch] = u0 + j;
                    a.chunk_base[base + ch] = base;
                }
            }
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

size_t max_chunks(size_t n) { return n / kChunk + n / (kLongSegment + 1) + 2; }

void free_plan_arrays(Plan &pl)
{
    PlanArgs &a = pl.a;
    for (uint32_t *p : {a.uniq, a.count, a.seg, a.perm, a.chunk_seg, a.chunk_base, a.chunk_done, a.meta})
        if (p) (void)hipFree(p);
    pl = Plan{};
}

void free_plan_scratch(PlanScratch &sc)
{
    for (uint32_t *p : {sc.bitmap, sc.word_rank, sc.tile_sum, sc.slot, sc.rank})
        if (p) (void)hipFree(p);
    sc = PlanScratch{};
}

// Both streams are idle after this (buffers may then be replaced).
static nups_status quiesce(nups_ctx *ctx)
{
    NUPS_HIP(hipStreamSynchronize(ctx->side));
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    return NUPS_OK;
}

// Makes the table's build scratch and the plan's result arrays large enough for n accesses and
// fills in the plan's pointers and shape fields.  Growing waits for both streams.
nups_status ensure_plan_capacity(nups_ctx *ctx, Table &t, Plan &pl, size_t n)
{
    PlanScratch &sc = t.scratch;
    PlanArgs &a = pl.a;
    nups_status st;
    const size_t words = (size_t)((t.num_keys + 31) / 32);
    if (sc.cap_words < words) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.bitmap, words, true, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.word_rank, words, false, ctx->side)) != NUPS_OK) return st;
        sc.cap_words = words;
    }
    if (sc.cap_n < n || sc.cap_n == 0) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        const size_t cap = n + n / 4 + 1024;
        if ((st = grow_u32(&sc.slot, cap, false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.rank, cap, false, ctx->side)) != NUPS_OK) return st;
        sc.cap_n = cap;
    }
    if (pl.cap_n < n || pl.cap_n == 0) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        const size_t cap = n + n / 4 + 1024;
        for (uint32_t **b : {&a.uniq, &a.count, &a.perm})
            if ((st = grow_u32(b, cap, false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.seg, cap + 1, false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_seg, max_chunks(cap), false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_base, max_chunks(cap), false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_done, max_chunks(cap), true, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.meta, kMetaWords, true, ctx->side)) != NUPS_OK) return st;
        pl.cap_n = cap;
    }
    const size_t tiles = std::max((words + kScanTile - 1) / kScanTile, (sc.cap_n + kScanTile - 1) / kScanTile);
    if (sc.cap_tiles < tiles) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.tile_sum, tiles, false, ctx->side)) != NUPS_OK) return st;
        sc.cap_tiles = tiles;
    }
    // partial rows of chunked segments (one buffer per context: the tables' updates run one after another)
    const size_t need_partial = max_chunks(pl.cap_n) * (size_t)t.stride;
    if (ctx->partial_cap < need_partial) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        if ((st = ensure_f32(&ctx->partial, &ctx->partial_cap, need_partial, ctx->stream)) != NUPS_OK) return st;
    }
    a.bitmap = sc.bitmap; a.word_rank = sc.word_rank; a.tile_sum = sc.tile_sum; a.slot = sc.slot; a.rank = sc.rank;
    a.num_keys = (uint32_t)t.num_keys;
    a.words = (uint32_t)words;
    a.bitmap_tiles = (uint32_t)((words + kScanTile - 1) / kScanTile);
    a.direct_bitmap = words <= 65536 ? 1u : 0u;            // up to 2M keys: 256 KB of bitmap per workgroup at most
    a.error_flag = ctx->error_flag;
    return NUPS_OK;
}

// Enqueues, on the side stream, the plan construction for one or two tables (a.src, a.n set by the caller).
nups_status build_plans(nups_ctx *ctx, Plan *plans, int n_plans)
{
    if (n_plans < 1 || n_plans > 2) return fail(NUPS_ERR_ARG, "build_plans: one or two plans");
    PhaseScope scope(ctx, NUPS_PHASE_PLAN, ctx->side);
    PlanPair pp;
    uint32_t max_n = 0, max_btiles = 0, max_ctiles = 0;
    bool need_bitmap_tiles = false, need_count_tiles = false;
    for (int k = 0; k < n_plans; ++k) {
        PlanArgs &a = plans[k].a;
        a.count_tiles = (a.n + kScanTile - 1) / kScanTile;
        if (a.count_tiles == 0) a.count_tiles = 1;   // still writes seg[0] and the totals for an empty step
        a.direct_count = a.n <= 131072 ? 1u : 0u;
        need_bitmap_tiles |= !a.direct_bitmap;
        need_count_tiles |= !a.direct_count;
        pp.p[k] = a;
        max_n = std::max(max_n, a.n);
        max_btiles = std::max(max_btiles, a.bitmap_tiles);
        max_ctiles = std::max(max_ctiles, a.count_tiles);
    }
    if (n_plans == 1) pp.p[1] = pp.p[0];
    const dim3 blk(kBlock);
    const uint32_t nblocks = std::max(1u, (max_n + kBlock - 1) / kBlock);
    const uint32_t rblocks = std::max(1u, (max_n + kRankTile - 1) / kRankTile);
    hipStream_t s = ctx->side;
    hipLaunchKernelGGL(k_plan_mark, dim3(rblocks, n_plans), blk, 0, s, pp);
    if (need_bitmap_tiles) hipLaunchKernelGGL(k_plan_bitmap_tiles, dim3(max_btiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_bitmap_scan, dim3(max_btiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_rank, dim3(rblocks, n_plans), blk, 0, s, pp);
    if (need_count_tiles) hipLaunchKernelGGL(k_plan_count_tiles, dim3(max_ctiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_count_scan, dim3(max_ctiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_scatter, dim3(nblocks, n_plans), blk, 0, s, pp);
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

}  // namespace nups
