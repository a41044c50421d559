// Preparatory work of a step (Section 4.3: drawing the samples; and the per-key aggregation structure that the
// update needs) as device functions that run in spare workgroups of other kernels' launches.
//
// The work of one step is a chain of phases, each of which needs everything the previous one wrote:
//   draw    the step's own sample keys (Section 4.4 schemes) + marks every key the step accesses
//   tiles   packs the marked key groups into bitmap words, ranks the words inside tiles, counts per tile
//   slot    per access: index of its key among the distinct keys (tile counts scanned by every workgroup; tables
//           with very many tiles get a phase of their own for that scan before)
//   rank    per access: position inside its key's segment; the distinct keys
//   counts  segment offsets (prefix sums of the per-key counts), chunk lists of long segments
//   scatter accesses grouped by key; the scratch maps return to all-zero
//   sort    (deterministic mode only) every segment's accesses in ascending order
// A launch of a gradient or update kernel carries, in its first workgroups, one phase each of up to kMaxSide later
// steps: the phases depend on key arrays and random numbers only, never on table values, so they may run while
// earlier steps still update the tables, and kernel boundaries on one stream order consecutive phases.
//
// Keys are bounded by the table size, so the distinct set is a map over the key space and a key's position among
// the distinct keys is a prefix population count; no comparison sort is needed.  Marking uses one byte per key,
// and one byte per group of 32 keys, and plain stores (idempotent, so no atomics and no contention on hot keys);
// only the groups that hold a marked key are then packed into bitmap words.  Hot keys (Section 3.2: a few keys
// take a large share of the accesses) would serialise the global atomics that hand out positions inside a
// segment, so every workgroup first combines its own accesses to a key in an LDS hash table and issues one global
// atomic per distinct key; segments that are too long for one row group are cut into chunks.
#pragma once

#include "device_utils.h"

namespace nups {

// ---- drawing ---------------------------------------------------------------------------------------------------

// One fresh draw from pi: bucket = floor((x0 + 2^32 x1) * V / 2^64); keep it if x2 < thresh[bucket].
__device__ __forceinline__ uint32_t fresh_key(const SampleArgs &d, uint64_t step, uint64_t draw)
{
    const Words w = draw_words(d.seed, kStreamFresh, d.dist_id, step, draw);
    const uint64_t u = (uint64_t)w.x0 | ((uint64_t)w.x1 << 32);
    const uint32_t b = (uint32_t)__umul64hi(u, d.num_keys);
    if (d.thresh == nullptr) return b;
    return (w.x2 < d.thresh[b]) ? b : d.alias[b];
}

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x85EBCA6Bu;
    x ^= x >> 13; x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

// Stores sample `pos` and, if the drawing feeds a step directly, marks its key in that step's maps.
__device__ __forceinline__ void emit_sample(const SampleArgs &d, uint64_t pos, uint32_t key)
{
    d.out[pos] = key;
    if (d.bytemap == nullptr) return;
    if (key >= d.rep.base_keys) { atomicOr(d.error_flag, 1u); return; }   // batch-local keys can be anything
    const uint32_t k = replica_key(d.rep, key, (uint32_t)pos / (d.per_sample ? d.per_sample : 1u));
    if (k >= d.mark_keys) return;
    d.bytemap[k] = 1;
    d.wordmap[k >> 5] = 1;
}

// Workgroup `vb` of a drawing of d.n samples; `word` is LDS for kMaxPool + 8 words, 16-byte aligned.
__device__ __forceinline__ void draw_block(const SampleArgs &d, uint32_t vb, uint32_t *word)
{
    const uint32_t i = vb * kBlock + threadIdx.x;
    switch (d.scheme) {
    case NUPS_CONFORM:      // independent sampling: sample i is draw i of the step
        if (i < d.n) emit_sample(d, i, fresh_key(d, d.step, i));
        break;
    case NUPS_BOUNDED: {    // sample reuse: one workgroup emits one pass over one pool.  The order of the pass is the
                            // ascending order of (first ORDER-stream word at (fresh id, pass), slot); rank by counting.
        const uint32_t pool = vb / d.U, pass = vb % d.U;
        const uint32_t first = pool * d.G;
        const uint32_t g = min(d.G, d.F - first);
        // position of this pass in the sequence: full pools emit U * G samples each
        const uint64_t base = (uint64_t)pool * d.U * d.G + (uint64_t)pass * g;
        if (base >= d.n) return;
        const uint32_t g8 = (g + 7) & ~7u;    // padded with words that rank after every real one
        for (uint32_t s = threadIdx.x; s < g8; s += kBlock)
            word[s] = s < g ? draw_words(d.seed, kStreamOrder, d.dist_id, d.step,
                                         (uint64_t)(first + s) | ((uint64_t)pass << 32)).x0
                            : 0xFFFFFFFFu;
        __syncthreads();
        const uint4 *word4 = reinterpret_cast<const uint4 *>(word);
        for (uint32_t s = threadIdx.x; s < g; s += kBlock) {
            const uint32_t w = word[s];
            uint32_t rank = 0;
#pragma unroll 4
            for (uint32_t j = 0; j < g8; j += 8) {   // eight words per turn: the reads' latency overlaps
                const uint4 a = word4[j / 4], b = word4[j / 4 + 1];
                rank += (a.x < w || (a.x == w && j + 0 < s)) ? 1u : 0u;
                rank += (a.y < w || (a.y == w && j + 1 < s)) ? 1u : 0u;
                rank += (a.z < w || (a.z == w && j + 2 < s)) ? 1u : 0u;
                rank += (a.w < w || (a.w == w && j + 3 < s)) ? 1u : 0u;
                rank += (b.x < w || (b.x == w && j + 4 < s)) ? 1u : 0u;
                rank += (b.y < w || (b.y == w && j + 5 < s)) ? 1u : 0u;
                rank += (b.z < w || (b.z == w && j + 6 < s)) ? 1u : 0u;
                rank += (b.w < w || (b.w == w && j + 7 < s)) ? 1u : 0u;
            }
            const uint64_t pos = base + rank;
            if (pos < d.n) emit_sample(d, pos, fresh_key(d, d.step, first + s));   // every pass redraws the pool's keys
        }
        break;
    }
    case NUPS_LONGTERM: {   // reuse over a long-lived pool: the sample at global position g is slot perm(rank) of the
                            // pool of its epoch, perm a four-round Feistel permutation of 0..P-1 (cycle walking)
        if (i >= d.n) return;
        const uint64_t g = d.cursor + i;
        const uint64_t per_epoch = d.P * (uint64_t)d.R;
        const uint64_t epoch = g / per_epoch, within = g % per_epoch;
        const uint64_t pass = within / d.P;
        uint64_t x = within % d.P;
        const int half = d.half;
        const uint32_t mask = (half >= 32) ? 0xFFFFFFFFu : ((1u << half) - 1u);
        const Words k = draw_words(d.seed, kStreamRoundKey, d.dist_id, epoch, pass);
        const uint32_t rk[4] = {k.x0, k.x1, k.x2, k.x3};
        do {   // ends: the walk follows a cycle of a permutation of the 2^(2 half) domain that contains x < P
            uint32_t L = (uint32_t)(x >> half) & mask, Rr = (uint32_t)x & mask;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t nR = L ^ (mix32(Rr ^ rk[t]) & mask);
                L = Rr; Rr = nR;
            }
            x = ((uint64_t)L << half) | Rr;
        } while (x >= d.P);
        emit_sample(d, i, fresh_key(d, epoch, x));
        break;
    }
    case NUPS_NONCONFORM: { // direct-access repurposing: sample p takes the key that a uniformly chosen example of
                            // its tile contributes
        if (i >= d.n) return;
        const uint32_t e = i / d.per_example;
        const uint32_t base = (e / d.tile) * d.tile;
        const uint32_t t = min(d.tile, d.local_n - base);
        const Words w = draw_words(d.seed, kStreamLocal, d.dist_id, d.step, i);
        const uint32_t pick = base + __umulhi(w.x0, t);
        emit_sample(d, i, ((i % d.per_example) < d.split) ? d.local_a[pick] : d.local_b[pick]);
        break;
    }
    default:
        break;
    }
}

// ---- the aggregation structure -----------------------------------------------------------------------------------

// Marks the first mark_n keys of the step in the maps (the rest were marked when they were drawn); flags keys
// outside the table.  Workgroup 0 also resets the step's counters.
__device__ __forceinline__ void mark_block(const PlanArgs &a, uint32_t vb)
{
    const uint32_t i = vb * kBlock + threadIdx.x;
    if (i == 0) a.meta[kMetaNumChunks] = 0;
    if (i < kLossSlots && a.zero_loss) a.zero_loss[i * kLossStride] = 0.0;   // the step's loss starts from zero
    if (i >= a.mark_n) return;
    const uint32_t key = plan_key(a.src, a.rep, i);
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

// Tile `vb` of kScanTile bitmap words: packs the marked groups of the byte map into bitmap words, ranks each
// word's distinct keys inside the tile and counts the tile's distinct keys.
__device__ __forceinline__ void tiles_block(const PlanArgs &a, uint32_t vb, uint32_t *lds)
{
    if (vb >= a.bitmap_tiles) return;
    const uint32_t w0 = vb * kScanTile + threadIdx.x * kScanItems;
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
    if (threadIdx.x == 0) a.tile_sum[vb] = total;
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

// Tables with more tiles than a workgroup scans by itself: one workgroup writes the distinct keys below each tile
// to memory, and the number of distinct keys.
__device__ __forceinline__ void prefix_block(const PlanArgs &a, uint32_t *lds)
{
    if (a.bitmap_tiles <= kLdsTiles) return;
    const uint32_t nu = scan_tile_sums(a, a.tile_prefix, lds);
    if (threadIdx.x == 0) a.meta[kMetaNumUniq] = nu;
}

// Accesses [vb * kSlotTile, ...): the index of each access's key among the distinct keys = distinct keys below
// its tile + below its word inside the tile + below its bit inside the word.  `scan`: LDS for kLdsTiles words.
__device__ __forceinline__ void slot_block(const PlanArgs &a, uint32_t vb, uint32_t *scan, uint32_t *lds)
{
    if (vb * kSlotTile >= a.n && vb != 0) return;
    uint32_t key[kSlotItems], below[kSlotItems], bits[kSlotItems];
    // the keys and their bitmap words are requested before the scan, which hides their latency
#pragma unroll
    for (int j = 0; j < kSlotItems; ++j) {
        const uint32_t i = vb * kSlotTile + j * kBlock + threadIdx.x;
        key[j] = i < a.n ? plan_key(a.src, a.rep, i) : kBadIndex;
        if (key[j] >= a.num_keys) key[j] = kBadIndex;     // outside the table: flagged when it was marked
    }
#pragma unroll
    for (int j = 0; j < kSlotItems; ++j) {
        const uint32_t w = key[j] >> 5;
        below[j] = key[j] != kBadIndex ? a.word_rank[w] : 0u;
        bits[j] = key[j] != kBadIndex ? a.bitmap[w] : 0u;
    }
    const uint32_t *tile_prefix = a.tile_prefix;
    if (a.bitmap_tiles <= kLdsTiles) {
        const uint32_t nu = scan_tile_sums(a, scan, lds);
        if (vb == 0 && threadIdx.x == 0) a.meta[kMetaNumUniq] = nu;
        tile_prefix = scan;
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < kSlotItems; ++j) {
        const uint32_t i = vb * kSlotTile + j * kBlock + threadIdx.x;
        if (i < a.n) {
            const uint32_t w = key[j] >> 5;
            uint32_t u = kBadIndex;
            if (key[j] != kBadIndex) {
                u = tile_prefix[w / kScanTile] + below[j] + __popc(bits[j] & ((1u << (key[j] & 31)) - 1u));
                // at most n distinct keys.  More means that a key array changed after the step was prepared: such
                // accesses are dropped and reported like keys outside the table, never used as an index.
                if (u >= a.n) { u = kBadIndex; atomicOr(a.error_flag, 1u); }
            }
            a.slot[i] = u;
        }
    }
}

// Where the position counter of distinct key number u lives.  Keys that are neighbours in key order are often hot
// together (ids sorted by frequency), and the atomics of all workgroups on counters in one cache line queue up
// behind each other (measured: 13 us of a 20 us phase), so the counters of 16 consecutive keys sit in 16 different
// lines.  The map permutes within blocks of kScanTile counters, which keeps the sums over whole tiles unchanged.
__device__ __forceinline__ uint32_t counter_index(uint32_t u)
{
    static_assert(kScanTile == 512, "the permutation is written for tiles of 512 counters");
    return (u & ~511u) | ((u & 15u) << 5) | ((u >> 4) & 31u);
}

// Accesses [vb * kRankTile, ...): the position of each inside its key's segment.  The workgroup's accesses are
// first grouped by key in an LDS hash table (`hash`: 4 * kHashSlots words, open addressing, at most half full); one
// global atomic per distinct key and workgroup reserves a run of positions, which the LDS counts subdivide.  Also
// emits the distinct keys (every workgroup writes the keys it met; equal values where they meet).
template <int kRankItems>
__device__ __forceinline__ void rank_block(const PlanArgs &a, uint32_t vb, uint32_t *hash)
{
    constexpr uint32_t kRankTile = kBlock * kRankItems, kHashSlots = 2 * kRankTile;
    constexpr int kHashBits = kRankItems == 4 ? 11 : kRankItems == 2 ? 10 : 9;
    static_assert(kHashSlots == 1u << kHashBits, "accesses per thread: 1, 2 or 4");
    if (vb * kRankTile >= a.n) return;
    uint32_t *hkey = hash, *hcnt = hash + kHashSlots, *hbase = hash + 2 * kHashSlots, *hval = hash + 3 * kHashSlots;
    uint32_t slot_of[kRankItems], local[kRankItems], uidx[kRankItems], key[kRankItems];
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        const uint32_t i = vb * kRankTile + j * kBlock + threadIdx.x;
        uidx[j] = i < a.n ? a.slot[i] : kBadIndex;
        key[j] = i < a.n ? plan_key(a.src, a.rep, i) : kBadIndex;
    }
    for (uint32_t s = threadIdx.x; s < kHashSlots; s += kBlock) { hkey[s] = kBadIndex; hcnt[s] = 0; }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kRankItems; ++j) {
        if (uidx[j] != kBadIndex) {
            const uint32_t u = uidx[j];
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
                base[q] = atomicAdd(&a.cnt_work[counter_index(hkey[s])], cnt[q]);
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
        const uint32_t i = vb * kRankTile + j * kBlock + threadIdx.x;
        if (i < a.n && uidx[j] != kBadIndex) a.rank[i] = hbase[slot_of[j]] + local[j];
    }
}

// Sum of each tile of kScanTile access counts (large steps only).
__device__ __forceinline__ void count_tiles_block(const PlanArgs &a, uint32_t vb, uint32_t *lds)
{
    if (vb >= a.count_tiles) return;
    const uint32_t nu = a.meta[kMetaNumUniq];
    const uint32_t u0 = vb * kScanTile + threadIdx.x * kScanItems;
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j)
        if (u0 + j < nu) c += a.cnt_work[counter_index(u0 + j)];
    const uint32_t s = block_sum(c, lds);
    if (threadIdx.x == 0) a.tile_sum[vb] = s;
}

// Segment offsets = exclusive prefix sums of the counts; cuts long segments into chunks.
__device__ __forceinline__ void counts_block(const PlanArgs &a, uint32_t vb, uint32_t *lds)
{
    if (vb >= a.count_tiles) return;
    const uint32_t nu = a.meta[kMetaNumUniq];
    const uint32_t u0 = vb * kScanTile + threadIdx.x * kScanItems;
    if (vb * kScanTile >= nu && vb != 0) return;
    uint32_t before;
    if (a.direct_count) before = block_sum_range(a.cnt_work, min(vb * kScanTile, nu), lds);
    else before = block_sum_range(a.tile_sum, vb, lds);
    uint32_t cnt[kScanItems];
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        cnt[j] = (u0 + j < nu) ? a.cnt_work[counter_index(u0 + j)] : 0u;
        c += cnt[j];
    }
    uint32_t total;
    uint32_t run = before + block_exclusive_scan(c, lds, &total);
    // chunks of this workgroup's long segments: one reservation per workgroup in the step's chunk list (a
    // reservation per hot key would queue up on that one counter)
    uint32_t nch[kScanItems], my_chunks = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        nch[j] = (u0 + j < nu && takes_hot_path(cnt[j], a.uniq[u0 + j], a.hot_bits, a.rep.base_keys)) ? (cnt[j] + kChunk - 1) / kChunk : 0u;
        my_chunks += nch[j];
    }
    uint32_t block_chunks;
    uint32_t chunk = block_exclusive_scan(my_chunks, lds, &block_chunks);
    __shared__ uint32_t chunk_base_of_block;
    if (threadIdx.x == 0) chunk_base_of_block = block_chunks ? atomicAdd(&a.meta[kMetaNumChunks], block_chunks) : 0u;
    __syncthreads();
    chunk += chunk_base_of_block;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (u0 + j < nu) {
            a.seg[u0 + j] = run;
            a.count[u0 + j] = cnt[j];
            for (uint32_t ch = 0; ch < nch[j] && chunk + ch < a.max_chunks; ++ch) {   // in range by construction
                a.chunk_of[chunk + ch] = make_uint4(u0 + j, chunk, run, run + cnt[j]);
            }
            chunk += nch[j];
        }
        run += cnt[j];
        if (u0 + j + 1 == nu || (nu == 0 && u0 + j == 0)) {   // end marker seg[nu]
            a.seg[nu] = run;
            a.meta[kMetaTotal] = run;
        }
    }
}

// Groups the accesses by key and returns the byte map and the position counters to all-zero for the next step.
__device__ __forceinline__ void scatter_block(const PlanArgs &a, uint32_t vb)
{
    const uint32_t i = vb * kBlock + threadIdx.x;
    if (i >= a.n) return;
    const uint32_t key = plan_key(a.src, a.rep, i);
    if (key < a.num_keys) a.bytemap[key] = 0;   // also for an access that is dropped below
    a.pos[i] = kBadIndex;
    const uint32_t u = a.slot[i];
    if (u == kBadIndex) return;
    const uint32_t r = a.rank[i];
    const uint32_t first = a.seg[u], next = a.seg[u + 1];
    if (first + r >= a.n) return;   // cannot happen with unchanged key arrays
    a.perm[first + r] = i;
    a.pos[i] = first + r;
    if (r == 0) {
        a.cnt_work[counter_index(u)] = 0;
        if (next - first == 1) a.rank[i] = kSingleAccess;   // the key's only access: a gradient kernel may update the row itself
    }
}

// Deterministic mode: every segment's accesses once more, in ascending order, free of any dependence on the order
// in which the rank phase's atomics were served.  Two phases over blocks of kBlock consecutive positions of perm.
// First: the piece of each segment that lies inside the block, sorted by counting, for every access, the smaller
// access numbers of its piece (from LDS).  A position that is not consistent with the structure (possible only if
// a key array was changed behind a prepared step) keeps what it holds.
__device__ __forceinline__ void sort_pieces_block(const PlanArgs &a, uint32_t vb, uint32_t *held)
{
    const uint32_t total = min(a.meta[kMetaTotal], a.n);
    const uint32_t block0 = vb * kBlock, t = block0 + threadIdx.x;
    uint32_t v = kBadIndex, first = 0, last = 0;
    bool placed = false;
    if (t < total) {
        v = a.perm[t];
        const uint32_t u = v < a.n ? a.slot[v] : kBadIndex;
        if (u != kBadIndex && u < a.meta[kMetaNumUniq]) {
            first = a.seg[u];
            last = min(a.seg[u + 1], total);
            placed = first <= t && t < last;
        }
    }
    held[threadIdx.x] = v;
    __syncthreads();
    if (t >= total) return;
    if (!placed) { a.perm_pieces[t] = v < a.n ? v : 0u; return; }
    const uint32_t lo = max(first, block0) - block0, hi = min(last, block0 + kBlock) - block0;
    uint32_t below = 0;
    for (uint32_t j = lo; j < hi; ++j) below += held[j] < v ? 1u : 0u;
    a.perm_pieces[block0 + lo + below] = v;
}

// Second: the position of an access in its segment is its position in its own piece plus, for every other piece
// of the segment, the number of smaller access numbers there (a binary search: the pieces are sorted).  Most
// segments have one piece and end here with their first phase's result.
__device__ __forceinline__ void merge_pieces_block(const PlanArgs &a, uint32_t vb)
{
    const uint32_t total = min(a.meta[kMetaTotal], a.n);
    const uint32_t block0 = vb * kBlock, t = block0 + threadIdx.x;
    if (t >= total) return;
    const uint32_t v = a.perm_pieces[t];       // below a.n by the first phase
    const uint32_t u = a.slot[v];
    uint32_t first = 0, last = 0;
    if (u != kBadIndex && u < a.meta[kMetaNumUniq]) {
        first = a.seg[u];
        last = min(a.seg[u + 1], total);
    }
    if (!(first <= t && t < last)) { a.perm_sorted[t] = v; return; }
    uint32_t below = t - max(first, block0);
    for (uint32_t q = first / kBlock; q <= (last - 1) / kBlock; ++q) {
        if (q == vb) continue;
        const uint32_t lo = max(first, q * kBlock);
        uint32_t l = lo, h = min(last, q * kBlock + kBlock);
        while (l < h) {
            const uint32_t m = (l + h) >> 1;
            if (a.perm_pieces[m] < v) l = m + 1;
            else h = m;
        }
        below += l - lo;
    }
    a.perm_sorted[first + below] = v;
    a.pos[v] = first + below;
}

// ---- dispatch ------------------------------------------------------------------------------------------------------

// Unit `vb` of one phase.  Dynamic LDS of the launch: at least side_lds_bytes(item.phase).
__device__ __forceinline__ void side_item_unit(const SideItem &it, uint32_t vb)
{
    extern __shared__ __align__(16) uint32_t side_dyn[];
    __shared__ uint32_t side_lds[kBlock / 64 + 1];
    vb += it.block0;
    if (it.phase == kSideDraw) {
        if (vb < it.draw.blocks) { draw_block(it.draw, vb, side_dyn); return; }
        vb -= it.draw.blocks;
    }
    const uint32_t plan = vb / it.blocks_per_plan;
    if (plan >= (uint32_t)it.n_plans) return;
    const PlanArgs &a = it.plan[plan];
    vb -= plan * it.blocks_per_plan;
    switch (it.phase) {
    case kSideDraw: mark_block(a, vb); break;
    case kSideTiles: tiles_block(a, vb, side_lds); break;
    case kSidePrefix: prefix_block(a, side_lds); break;
    case kSideSlot: slot_block(a, vb, side_dyn, side_lds); break;
    case kSideRank:
        if (a.rank_items == 4) rank_block<4>(a, vb, side_dyn);
        else rank_block<2>(a, vb, side_dyn);
        break;
    case kSideCountTiles: count_tiles_block(a, vb, side_lds); break;
    case kSideCounts: counts_block(a, vb, side_lds); break;
    case kSideScatter: scatter_block(a, vb); break;
    case kSideSort: sort_pieces_block(a, vb, side_dyn); break;
    case kSideMerge: merge_pieces_block(a, vb); break;
    default: break;
    }
}

// True if this workgroup belongs to the side work of the launch (and has done it).  The remaining workgroups,
// numbered from sw.blocks on, are the launch's own.
__device__ __forceinline__ bool side_work_block(const SideWork &sw)
{
    if (blockIdx.x >= sw.blocks) return false;
    uint32_t vb = blockIdx.x;
#pragma unroll
    for (int k = 0; k < kMaxSide; ++k) {
        if (k < sw.n) {
            if (vb < sw.item[k].wgs) {
                for (uint32_t unit = vb; unit < sw.item[k].blocks; unit += sw.item[k].wgs) {
                    side_item_unit(sw.item[k], unit);
                    __syncthreads();   // LDS is reused by the next unit
                }
                return true;
            }
            vb -= sw.item[k].wgs;
        }
    }
    return true;   // padding workgroup
}

// Preparatory work on its own (a step that is run before later launches could carry all of its phases; push).
__global__ void __launch_bounds__(kBlock) k_side(SideWork sw) { (void)side_work_block(sw); }

}  // namespace nups
