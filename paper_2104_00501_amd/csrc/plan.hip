// Per-key aggregation structure of a step (the "aggregate per key" stage): from the list of keys
// a step accesses in one table, build the distinct keys in ascending order, their access counts
// and the accesses grouped by key.  Keys are bounded by the table size, so the distinct set is a
// map over the key space and a key's position among the distinct keys is a prefix population
// count; no comparison sort is needed.  Up to two tables are planned by the same launches
// (blockIdx.y selects the table).
//
// Marking uses one byte per key, and one byte per group of 32 keys, and plain stores (idempotent, so no
// atomics and no contention on hot keys); only the groups that hold a marked key are then packed into
// bitmap words, so a build reads 1/32 byte per key of the table plus 32 bytes per group in use.  Hot keys (Section 3.2: a few keys take a
// large share of the accesses) would serialise the global atomics that hand out positions inside
// a segment, so every workgroup first combines its own accesses to a key in LDS and issues one
// global atomic per distinct key; segments that are too long for one row group are cut into
// chunks that separate workgroups sum.
#include <algorithm>
#include <initializer_list>

#include "device_utils.h"

namespace nups {

struct PlanPair {
    PlanArgs p[2];
};

constexpr int kRankItems = 4;                       // accesses per thread in k_plan_rank
constexpr int kRankTile = kBlock * kRankItems;
constexpr int kHashBits = 11;
constexpr uint32_t kHashSlots = 1u << kHashBits;    // open-addressing table in LDS, at most half full
constexpr uint32_t kLdsTiles = 2048;                // tile counts that k_plan_rank scans by itself (64M keys)
static_assert(kHashSlots >= 2 * kRankTile, "the LDS hash table must stay at most half full");

// Marks the keys of the step in the byte map; flags keys outside the table.
__global__ void __launch_bounds__(kBlock) k_plan_mark(PlanPair pp)
{
    const PlanArgs &a = pp.p[blockIdx.y];
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i == 0) {
        a.meta[kMetaNumChunks] = 0;
    }
    if (i < kLossSlots && a.zero_loss) a.zero_loss[i * kLossStride] = 0.0;   // the step's loss starts from zero
    if (i >= a.n) return;
    const uint32_t key = source_key(a.src, i);
    if (key >= a.num_keys) { atomicOr(a.error_flag, 1u); return; }
    a.bytemap[key] = 1;
    a.wordmap[key >> 5] = 1;
}

// Sum of `items[0 .. end)` over the whole workgroup; every thread gets the result.
// `items` is 16-byte aligned; whole uint4 are read, four per thread and iteration, then the tail.
__device__ __forceinline__ uint32_t block_sum_range(const uint32_t *items, uint32_t end, uint32_t *lds)
{
    uint32_t c = 0;
    const uint4 *v = reinterpret_cast<const uint4 *>(items);
    const uint32_t n4 = end / 4;
    uint32_t q = threadIdx.x;
    for (; q + 3 * kBlock < n4; q += 4 * kBlock) {
        const uint4 x0 = v[q], x1 = v[q + kBlock], x2 = v[q + 2 * kBlock], x3 = v[q + 3 * kBlock];
        c += (x0.x + x0.y + x0.z + x0.w) + (x1.x + x1.y + x1.z + x1.w) + (x2.x + x2.y + x2.z + x2.w)
             + (x3.x + x3.y + x3.z + x3.w);
    }
    for (; q < n4; q += kBlock) { const uint4 x = v[q]; c += x.x + x.y + x.z + x.w; }
    for (uint32_t w = n4 * 4 + threadIdx.x; w < end; w += kBlock) c += items[w];
    return block_sum(c, lds);
}

// Four marker bytes (0 or 1 each) -> four bits.
__device__ __forceinline__ uint32_t pack4(uint32_t x)
{
    return (x & 1u) | ((x >> 7) & 2u) | ((x >> 14) & 4u) | ((x >> 21) & 8u);
}

// For every tile of kScanTile bitmap words: packs the marked groups of the byte map into bitmap words, ranks each
// word's distinct keys inside the tile and counts the tile's distinct keys.
__global__ void __launch_bounds__(kBlock) k_plan_bitmap_tiles(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x >= a.bitmap_tiles) return;
    const uint32_t w0 = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
    uint32_t bits[kScanItems];
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        bits[j] = 0;
        if (w0 + j < a.words && a.wordmap[w0 + j]) {   // the byte map is allocated in whole words of 32 keys
            const uint4 *src = reinterpret_cast<const uint4 *>(a.bytemap + (size_t)(w0 + j) * 32);
            const uint4 lo = src[0], hi = src[1];
            bits[j] = pack4(lo.x) | (pack4(lo.y) << 4) | (pack4(lo.z) << 8) | (pack4(lo.w) << 12)
                      | (pack4(hi.x) << 16) | (pack4(hi.y) << 20) | (pack4(hi.z) << 24) | (pack4(hi.w) << 28);
            a.bitmap[w0 + j] = bits[j];
            a.wordmap[w0 + j] = 0;
            c += __popc(bits[j]);
        }
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan(c, lds, &total);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (bits[j]) a.word_rank[w0 + j] = run;
        run += __popc(bits[j]);
    }
    if (threadIdx.x == 0) a.tile_sum[blockIdx.x] = total;
}

// Exclusive prefix sums of the tile counts into `prefix` (LDS or global); returns the number of distinct keys.
__device__ __forceinline__ uint32_t scan_tile_sums(const PlanArgs &a, uint32_t *prefix, uint32_t *lds)
{
    uint32_t carry = 0;
    for (uint32_t base = 0; base < a.bitmap_tiles; base += kBlock) {
        const uint32_t t = base + threadIdx.x;
        const uint32_t v = t < a.bitmap_tiles ? a.tile_sum[t] : 0u;
        uint32_t sum;
        const uint32_t before = block_exclusive_scan(v, lds, &sum);
        if (t < a.bitmap_tiles) prefix[t] = carry + before;
        carry += sum;
    }
    return carry;
}

// Tables with more tiles than k_plan_rank scans by itself: the number of distinct keys below each tile, in memory.
__global__ void __launch_bounds__(kBlock) k_plan_tile_prefix(PlanPair pp)
{
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (a.bitmap_tiles <= kLdsTiles) return;
    const uint32_t nu = scan_tile_sums(a, a.tile_prefix, lds);
    if (threadIdx.x == 0) a.meta[kMetaNumUniq] = nu;
}

// Per access: which distinct key it belongs to and its position inside that key's segment.
// The workgroup's accesses are first grouped by key in an LDS hash table; one global atomic per
// distinct key and workgroup reserves a run of positions, which the LDS counts subdivide.  Also
// emits the distinct keys (every workgroup writes the keys it met; equal values where they meet).
__global__ void __launch_bounds__(kBlock) k_plan_rank(PlanPair pp)
{
    __shared__ uint32_t hkey[kHashSlots], hcnt[kHashSlots], hbase[kHashSlots], hval[kHashSlots];
    __shared__ uint32_t tile_prefix_lds[kLdsTiles];
    __shared__ uint32_t lds[kBlock / 64 + 1];
    const PlanArgs &a = pp.p[blockIdx.y];
    if (blockIdx.x * kRankTile >= a.n && blockIdx.x != 0) return;
    uint32_t slot_of[kRankItems], local[kRankItems], uidx[kRankItems], key[kRankItems];
    // all loads are issued before the first use (keys, then their bitmap words and word ranks), and before the
    // scan below, which hides their latency
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        const uint32_t i = blockIdx.x * kRankTile + j * kBlock + threadIdx.x;
        key[j] = i < a.n ? source_key(a.src, i) : kBadIndex;
        if (key[j] >= a.num_keys) key[j] = kBadIndex;     // outside the table: flagged when it was marked
    }
    uint32_t below[kRankItems], bits[kRankItems];
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        const uint32_t w = key[j] >> 5;
        below[j] = key[j] != kBadIndex ? a.word_rank[w] : 0u;
        bits[j] = key[j] != kBadIndex ? a.bitmap[w] : 0u;
    }
    // distinct keys below each bitmap tile: every workgroup scans the tile counts for itself
    const uint32_t *tile_prefix = a.tile_prefix;
    if (a.bitmap_tiles <= kLdsTiles) {
        const uint32_t nu = scan_tile_sums(a, tile_prefix_lds, lds);
        if (blockIdx.x == 0 && threadIdx.x == 0) a.meta[kMetaNumUniq] = nu;
        tile_prefix = tile_prefix_lds;
    }
    for (uint32_t s = threadIdx.x; s < kHashSlots; s += kBlock) { hkey[s] = kBadIndex; hcnt[s] = 0; }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        uidx[j] = kBadIndex;
        if (key[j] != kBadIndex) {
            const uint32_t w = key[j] >> 5, b = key[j] & 31;
            const uint32_t u = tile_prefix[w / kScanTile] + below[j] + __popc(bits[j] & ((1u << b) - 1u));
            uidx[j] = u;
            uint32_t s = (u * 2654435761u) >> (32 - kHashBits);
            for (;;) {   // ends: at most kRankTile distinct keys in 2 * kRankTile slots
                const uint32_t old = atomicCAS(&hkey[s], kBadIndex, u);
                if (old == kBadIndex || old == u) break;
                s = (s + 1) & (kHashSlots - 1);
            }
            slot_of[j] = s;
            hval[s] = key[j];
            local[j] = atomicAdd(&hcnt[s], 1u);
        }
    }
    __syncthreads();
    {   // one global atomic per distinct key of the workgroup; all of a thread's atomics are in flight together
        constexpr int kPerThread = kHashSlots / kBlock;
        uint32_t base[kPerThread], cnt[kPerThread];
#pragma unroll
        for (int q = 0; q < kPerThread; ++q) {
            const uint32_t s = q * kBlock + threadIdx.x;
            cnt[q] = hcnt[s];
            base[q] = 0;
            if (cnt[q]) {
                base[q] = atomicAdd(&a.cnt_work[hkey[s]], cnt[q]);
                a.uniq[hkey[s]] = hval[s];
            }
        }
#pragma unroll
        for (int q = 0; q < kPerThread; ++q)
            if (cnt[q]) hbase[q * kBlock + threadIdx.x] = base[q];
    }
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
        if (u0 + j < nu) c += a.cnt_work[u0 + j];
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
    if (a.direct_count) before = block_sum_range(a.cnt_work, min(blockIdx.x * kScanTile, nu), lds);
    else before = block_sum_range(a.tile_sum, blockIdx.x, lds);
    uint32_t cnt[kScanItems];
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        cnt[j] = (u0 + j < nu) ? a.cnt_work[u0 + j] : 0u;
        c += cnt[j];
    }
    uint32_t total;
    uint32_t run = before + block_exclusive_scan(c, lds, &total);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (u0 + j < nu) {
            a.seg[u0 + j] = run;
            a.count[u0 + j] = cnt[j];
            if (takes_hot_path(cnt[j], a.uniq[u0 + j], a.hot_bits)) {
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

// Groups the accesses by key and returns the byte map and the position counters to all-zero for the next step.
__global__ void __launch_bounds__(kBlock) k_plan_scatter(PlanPair pp)
{
    const PlanArgs &a = pp.p[blockIdx.y];
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= a.n) return;
    const uint32_t u = a.slot[i];
    if (u == kBadIndex) return;
    const uint32_t r = a.rank[i];
    const uint32_t first = a.seg[u], next = a.seg[u + 1];
    a.perm[first + r] = i;
    a.bytemap[source_key(a.src, i)] = 0;
    if (r == 0) {
        a.cnt_work[u] = 0;
        if (next - first == 1) a.rank[i] = kSingleAccess;   // lets the update skip the segment lookup
    }
}

// (Re)allocates; all streams are idle when this is called, and the clearing has finished when it returns.
static nups_status grow_u32(uint32_t **buf, size_t n, bool zero, hipStream_t)
{
    if (*buf) NUPS_HIP(hipFree(*buf));
    *buf = nullptr;
    NUPS_HIP(hipMalloc((void **)buf, sizeof(uint32_t) * (n ? n : 1)));
    if (zero) NUPS_HIP(hipMemset(*buf, 0, sizeof(uint32_t) * (n ? n : 1)));
    return NUPS_OK;
}

size_t max_chunks(size_t n) { return n / kChunk + n / (kLongSegment + 1) + 2; }

// Room for `need` floats of partial rows of chunked segments; growing waits for both streams.
nups_status ensure_partial(nups_ctx *ctx, size_t need)
{
    if (ctx->partial_cap >= need && ctx->partial) return NUPS_OK;
    nups_status st = sync_side(ctx);
    if (st != NUPS_OK) return st;
    return ensure_f32(&ctx->partial, &ctx->partial_cap, need, ctx->stream);
}

void free_plan_arrays(Plan &pl)
{
    PlanArgs &a = pl.a;
    for (uint32_t *p : {a.uniq, a.count, a.seg, a.perm, a.slot, a.rank, a.chunk_seg, a.chunk_base, a.chunk_done, a.meta})
        if (p) (void)hipFree(p);
    pl = Plan{};
}

void free_plan_scratch(PlanScratch &sc)
{
    for (uint32_t *p : {sc.bitmap, sc.word_rank, sc.tile_sum, sc.tile_prefix, sc.cnt_work})
        if (p) (void)hipFree(p);
    if (sc.bytemap) (void)hipFree(sc.bytemap);
    if (sc.wordmap) (void)hipFree(sc.wordmap);
    sc = PlanScratch{};
}

// Both streams are idle after this (buffers may then be replaced).
static nups_status quiesce(nups_ctx *ctx)
{
    nups_status st = sync_side(ctx);
    if (st != NUPS_OK) return st;
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    return NUPS_OK;
}

// Makes the table's build scratch and the plan's result arrays large enough for n accesses and
// fills in the plan's pointers and shape fields.  Growing waits for both streams.
nups_status ensure_plan_capacity(nups_ctx *ctx, Table &t, Plan &pl, size_t n, int lane)
{
    PlanScratch &sc = t.scratch[lane];
    PlanArgs &a = pl.a;
    nups_status st;
    const size_t words = (size_t)((t.num_keys + 31) / 32);
    if (sc.cap_words < words) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.bitmap, words, true, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32((uint32_t **)&sc.bytemap, words * 8, true, ctx->side)) != NUPS_OK) return st;   // 32 bytes per word
        if ((st = grow_u32((uint32_t **)&sc.wordmap, (words + 3) / 4, true, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.word_rank, words, false, ctx->side)) != NUPS_OK) return st;
        sc.cap_words = words;
    }
    if (sc.cap_n < n || sc.cap_n == 0) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        sc.cap_n = n + n / 4 + 1024;                       // also sizes the tile sums below
        if ((st = grow_u32(&sc.cnt_work, sc.cap_n, true, ctx->side)) != NUPS_OK) return st;
    }
    if (pl.cap_n < n || pl.cap_n == 0) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        const size_t cap = n + n / 4 + 1024;
        for (uint32_t **b : {&a.uniq, &a.count, &a.perm, &a.slot, &a.rank})
            if ((st = grow_u32(b, cap, false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.seg, cap + 1, false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_seg, max_chunks(cap), false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_base, max_chunks(cap), false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_done, max_chunks(cap), true, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.meta, kMetaWords, true, ctx->side)) != NUPS_OK) return st;
        pl.cap_n = cap;
    }
    const size_t tiles = std::max((words + kScanTile - 1) / kScanTile,
                                  (std::max(sc.cap_n, pl.cap_n) + kScanTile - 1) / kScanTile);
    if (sc.cap_tiles < tiles) {
        if ((st = quiesce(ctx)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.tile_sum, tiles, false, ctx->side)) != NUPS_OK) return st;
        if ((st = grow_u32(&sc.tile_prefix, tiles, false, ctx->side)) != NUPS_OK) return st;
        sc.cap_tiles = tiles;
    }
    a.bytemap = sc.bytemap; a.wordmap = sc.wordmap;
    a.bitmap = sc.bitmap; a.word_rank = sc.word_rank; a.tile_sum = sc.tile_sum; a.tile_prefix = sc.tile_prefix;
    a.cnt_work = sc.cnt_work;
    a.num_keys = (uint32_t)t.num_keys;
    a.words = (uint32_t)words;
    a.bitmap_tiles = (uint32_t)((words + kScanTile - 1) / kScanTile);
    a.error_flag = ctx->error_flag;
    a.hot_bits = t.hot_bits_dev;
    return NUPS_OK;
}

// Enqueues, on side stream `s`, the plan construction for one or two tables (a.src, a.n set by the caller).
nups_status build_plans(nups_ctx *ctx, hipStream_t s, Plan *plans, int n_plans)
{
    if (n_plans < 1 || n_plans > 2) return fail(NUPS_ERR_ARG, "build_plans: one or two plans");
    PhaseScope scope(ctx, NUPS_PHASE_PLAN, s);
    PlanPair pp;
    uint32_t max_n = 0, max_btiles = 0, max_ctiles = 0;
    bool need_count_tiles = false;
    for (int k = 0; k < n_plans; ++k) {
        PlanArgs &a = plans[k].a;
        a.count_tiles = (a.n + kScanTile - 1) / kScanTile;
        if (a.count_tiles == 0) a.count_tiles = 1;   // still writes seg[0] and the totals for an empty step
        a.direct_count = a.n <= 131072 ? 1u : 0u;
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
    hipLaunchKernelGGL(k_plan_mark, dim3(nblocks, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_bitmap_tiles, dim3(max_btiles, n_plans), blk, 0, s, pp);
    if (max_btiles > kLdsTiles) hipLaunchKernelGGL(k_plan_tile_prefix, dim3(1, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_rank, dim3(rblocks, n_plans), blk, 0, s, pp);
    if (need_count_tiles) hipLaunchKernelGGL(k_plan_count_tiles, dim3(max_ctiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_count_scan, dim3(max_ctiles, n_plans), blk, 0, s, pp);
    hipLaunchKernelGGL(k_plan_scatter, dim3(nblocks, n_plans), blk, 0, s, pp);
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

}  // namespace nups
