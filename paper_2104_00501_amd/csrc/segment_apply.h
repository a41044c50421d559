// "Aggregate per key, then push": for every distinct key of a plan, sum the gradient
// contributions of its accesses and update the row once.  A contribution is a coefficient times
// a source row (a staged gradient row, or a row of another table); the sum is kept in registers
// by a 16-lane row group, so each touched row is read once and written once.
// Short segments take one row group each; long segments (the hot keys of Section 3.2) are cut into
// chunks, one workgroup per chunk, whose partial rows are combined by the workgroup that finishes last.
//
// The order of the additions is a fixed function of a segment's length, whichever path sums it.  Up to
// kLongSegment = 16 accesses: one after the other.  Longer: kTreeBlock = 16 consecutive accesses are added one
// after the other (a block), sixteen consecutive block sums one after the other (a super-block of kChunk = 256
// accesses: what one workgroup sums of a chunked segment), and the super-block sums one after the other.  (Blocks
// of 4 and chunks of 64 make a chunk's workgroup finish in 4 instead of 7 us, but there are then more workgroups
// than the device holds at once: 38.8 against 37.6 us per step of the large skip-gram configuration.)  A long
// chain of fp32 additions never forms, and with the accesses of a segment in ascending order (a plan built in
// deterministic mode) the result does not depend on the run or on which keys are declared hot.
#pragma once

#include <algorithm>

#include "side_work.h"

namespace nups {

// ---- contribution sources: access i -> (coefficient, source row) ---------------------------

// An access that contributes nothing to its key's sum has this source row number (sources whose kSkips is true may
// return it from fetch): its row is neither read nor added.  Leaving a term of zero out of a sum that starts at +0
// changes no bit of the result.
constexpr uint32_t kNoRow = 0xFFFFFFFFu;

// Row i of a staging array, coefficient one (KGE relations, push).
struct SrcStaged {
    static constexpr bool kSkips = false;   // every access contributes a row
    static constexpr bool kDoneInRows = false;
    const float *stage;
    bool singles_done = false;   // the gradient kernel has updated the keys with a single access itself
    __device__ __forceinline__ bool done_already(uint32_t) const { return singles_done; }
    __device__ __forceinline__ bool segment_done(const uint32_t *perm, uint32_t first, uint32_t last, int) const
    {
        return last - first == 1 && done_already(perm[first]);
    }
    __device__ __forceinline__ float coef(uint32_t) const { return 1.0f; }
    __device__ __forceinline__ const float *rows() const { return stage; }
    __device__ __forceinline__ uint32_t row_number(uint32_t i) const { return i; }
    // coefficient and source row number of the access at position t of the plan's access order
    __device__ __forceinline__ void fetch(const uint32_t *perm, uint32_t t, float &c, uint32_t &r) const
    {
        const uint32_t i = perm[t];
        c = coef(i);
        r = row_number(i);
    }
};

// The row that example i's key lives in (its replica for the example's part of the minibatch if the key is hot and
// the table has replicas); kBadIndex for a key outside the table.  Runs of examples are runs of equal rows.
__device__ __forceinline__ uint32_t run_row(const uint32_t *keys, const ReplicaMap &rep, uint32_t i)
{
    const uint32_t key = keys[i];
    return key < rep.base_keys ? replica_key(rep, key, i) : kBadIndex;
}

// Staged rows whose numbers the gradient kernel has left where the accesses stand in the plan's access order (it
// knows the positions from the structure), so the update reads them in order, with no look-up through access
// numbers or keys in between.  An entry is a row of `stage`; kNoRow for an access that contributes nothing more
// (an example inside a run whose gradients the gradient kernel has added up and staged at the run's first example:
// SGNS input side, where 2 x window consecutive pairs of a stream share their center word, and the column side of a
// factorisation whose workers walk their cells column by column); or kRowDone for an access whose key the gradient
// kernel has updated itself (a key with a single access, or with all its accesses in one run: it had the sum and
// the row in registers).  Nine of ten SGNS accesses of this source are pairs inside a run: the update kernel's L1
// traffic, which bounds it, is spared their rows.
constexpr uint32_t kRowDone = 0xFFFFFFFEu;

struct SrcStagedAt {
    static constexpr bool kSkips = true;
    // Whether a short segment is done shows in the row numbers that its sum fetches anyway: the update of a short
    // segment fetches them once and asks done_in_rows, instead of segment_done and a second read.
    static constexpr bool kDoneInRows = true;
    const float *stage;
    const uint32_t *row_at;   // [accesses] in the plan's access order
    bool singles_done;        // the gradient kernel updates keys by itself where it can: a key with one access is then
                              // done, which its segment's length says without a read
    // Every lane of the group calls it; r: the row number of the segment's access number `lane` (any value in lanes
    // beyond the segment's n <= kGroup accesses).  Only a segment of at most kGroupsPerBlock accesses can be done (a
    // run lies inside one workgroup of the gradient kernel); it is done iff one of its accesses says so.
    __device__ __forceinline__ bool done_in_rows(uint32_t r, uint32_t n, int lane) const
    {
        return group_max(((uint32_t)lane < n && r == kRowDone) ? 1u : 0u) != 0u;
    }
    __device__ __forceinline__ bool segment_done(const uint32_t *, uint32_t first, uint32_t last, int lane) const
    {
        const uint32_t n = last - first;
        if (n > (uint32_t)kGroupsPerBlock) return false;
        if (n == 1 && singles_done) return true;
        return done_in_rows((uint32_t)lane < n ? row_at[first + lane] : 0u, n, lane);
    }
    __device__ __forceinline__ const float *rows() const { return stage; }
    __device__ __forceinline__ void fetch(const uint32_t *, uint32_t t, float &c, uint32_t &r) const
    {
        c = 1.0f;
        r = row_at[t];
    }
};

// SGNS output side: the gradient of a scored row (the pair's context word or one of its negatives) is
// coef * (input vector of the pair's center word, as it was at the start of the step).  Those vectors are read from
// a staged copy, one row per distinct center word, so that the input table may be updated at the same time.  The
// gradient kernel leaves coefficient and row number of every access where the access stands in the output table's
// access order (it knows the positions from the structure), so the update reads them in order, with no look-up
// through the access numbers in between.
struct SrcSgnsOut {
    static constexpr bool kSkips = false;
    static constexpr bool kDoneInRows = false;
    const float *center_rows;   // [distinct centers][stride]
    const float *coef_at;       // [accesses] in the plan's access order
    const uint32_t *row_at;     // [accesses] row of center_rows (the center word's index among the distinct ones)
    __device__ __forceinline__ bool segment_done(const uint32_t *, uint32_t, uint32_t, int) const { return false; }
    __device__ __forceinline__ const float *rows() const { return center_rows; }
    __device__ __forceinline__ void fetch(const uint32_t *, uint32_t t, float &c, uint32_t &r) const
    {
        c = coef_at[t];
        r = row_at[t];
    }
};

// KGE entity table: accesses [0,B) subjects and [B,2B) objects take their staged gradient rows;
// access 2B + p is negative p of triple p / nn and takes coef * (staged direction row of that
// triple: rows 2B.. for replaced subjects, rows 3B.. for replaced objects).  A negative that is its entity's only
// access of the step was updated by the gradient kernel.
struct SrcKgeEntity {
    static constexpr bool kSkips = false;
    static constexpr bool kDoneInRows = false;
    const float *stage;
    const float *coefs;   // [B, nn]
    uint32_t B, nn, nh;
    // i: the only access of its key
    __device__ __forceinline__ bool done_already(uint32_t i) const { return i >= 2 * B; }
    __device__ __forceinline__ bool segment_done(const uint32_t *perm, uint32_t first, uint32_t last, int) const
    {
        return last - first == 1 && done_already(perm[first]);
    }
    __device__ __forceinline__ float coef(uint32_t i) const { return i < 2 * B ? 1.0f : coefs[i - 2 * B]; }
    __device__ __forceinline__ const float *rows() const { return stage; }
    __device__ __forceinline__ uint32_t row_number(uint32_t i) const
    {
        if (i < 2 * B) return i;
        const uint32_t p = i - 2 * B, e = p / nn;
        return ((p % nn) < nh ? 2 * B : 3 * B) + e;
    }
    // coefficient and source row number of the access at position t of the plan's access order
    __device__ __forceinline__ void fetch(const uint32_t *perm, uint32_t t, float &c, uint32_t &r) const
    {
        const uint32_t i = perm[t];
        c = coef(i);
        r = row_number(i);
    }
};

// ---- update rules ----------------------------------------------------------------------------
// An update is split in two so that the row (and its state) can be requested from memory before the
// gradient contributions are summed: load() issues the reads, finish() combines and writes back.

struct OptSgd {          // theta <- theta - lr * delta
    float lr;
    // Norm clipping of the updates of hot keys (Section 5.1: updates of replicated parameters that exceed the
    // average norm by more than a factor are clipped).  clip_bound: factor x the mean norm of the hot-key updates
    // of earlier steps (+inf while there are none), computed before the launch; null: no clipping.  clip_stats:
    // kLossSlots pairs {sum of norms, number of norms}, kLossStride doubles apart, which this step adds to.
    const float *clip_bound = nullptr;
    double *clip_stats = nullptr;
    static constexpr bool kHasState = false;
    __device__ __forceinline__ bool clips() const { return clip_bound != nullptr; }
    // d: the summed gradient of a hot key, held by one row group.  Records its norm and shortens it to the bound.
    template <int NV4>
    __device__ __forceinline__ void clip(Row<NV4> &d, int lane) const
    {
        float sq = 0.0f;
#pragma unroll
        for (int q = 0; q < NV4; ++q) sq += d.v[q].x * d.v[q].x + d.v[q].y * d.v[q].y + d.v[q].z * d.v[q].z + d.v[q].w * d.v[q].w;
        const float norm = sqrtf(group_sum(sq));
        if (lane == 0) {
            double *slot = clip_stats + (blockIdx.x % kLossSlots) * kLossStride;
            atomicAdd(slot, (double)norm);
            atomicAdd(slot + 1, 1.0);
        }
        const float bound = *clip_bound;
        if (norm > bound) {
            const float shrink = bound / norm;
#pragma unroll
            for (int q = 0; q < NV4; ++q) {
                d.v[q].x *= shrink;
                d.v[q].y *= shrink;
                d.v[q].z *= shrink;
                d.v[q].w *= shrink;
            }
        }
    }
    template <int NV4>
    __device__ __forceinline__ void load(Row<NV4> &t, Row<NV4> &, const float *row, const float *, int lane) const
    {
        load_row(t, row, lane);
    }
    template <int NV4>
    __device__ __forceinline__ void finish(Row<NV4> &t, Row<NV4> &, float *row, float *, const Row<NV4> &d,
                                           int lane) const
    {
#pragma unroll
        for (int q = 0; q < NV4; ++q) axpy4(t.v[q], -lr, d.v[q]);
        store_row_through(row, t, lane);
    }
};

struct OptAdd {          // theta <- theta + delta   (push)
    static constexpr bool kHasState = false;
    __device__ __forceinline__ bool clips() const { return false; }
    template <int NV4>
    __device__ __forceinline__ void clip(Row<NV4> &, int) const {}
    template <int NV4>
    __device__ __forceinline__ void load(Row<NV4> &t, Row<NV4> &, const float *row, const float *, int lane) const
    {
        load_row(t, row, lane);
    }
    template <int NV4>
    __device__ __forceinline__ void finish(Row<NV4> &t, Row<NV4> &, float *row, float *, const Row<NV4> &d,
                                           int lane) const
    {
#pragma unroll
        for (int q = 0; q < NV4; ++q) axpy4(t.v[q], 1.0f, d.v[q]);
        store_row_through(row, t, lane);
    }
};

struct OptAdagrad {      // G <- G + delta^2 ; theta <- theta - lr * delta / (sqrt(G) + eps)
    float lr, eps;
    static constexpr bool kHasState = true;
    __device__ __forceinline__ bool clips() const { return false; }
    template <int NV4>
    __device__ __forceinline__ void clip(Row<NV4> &, int) const {}
    // The hardware square root and reciprocal (one unit in the last place each) instead of the correctly rounded
    // sequences: the update is a product of rounded factors anyway, and the row update is arithmetic-bound otherwise
    // (a 2 KB row is 512 square roots and divisions).
    __device__ __forceinline__ void one(float &t, float &g, float d) const
    {
        g += d * d;
        t -= lr * d * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(g) + eps);
    }
    template <int NV4>
    __device__ __forceinline__ void load(Row<NV4> &t, Row<NV4> &g, const float *row, const float *state_row,
                                         int lane) const
    {
        load_row(t, row, lane);
        load_row(g, state_row, lane);
    }
    template <int NV4>
    __device__ __forceinline__ void finish(Row<NV4> &t, Row<NV4> &g, float *row, float *state_row,
                                           const Row<NV4> &d, int lane) const
    {
#pragma unroll
        for (int q = 0; q < NV4; ++q) {
            one(t.v[q].x, g.v[q].x, d.v[q].x);
            one(t.v[q].y, g.v[q].y, d.v[q].y);
            one(t.v[q].z, g.v[q].z, d.v[q].z);
            one(t.v[q].w, g.v[q].w, d.v[q].w);
        }
        store_row_through(state_row, g, lane);
        store_row_through(row, t, lane);
    }
};

// ---- kernels ---------------------------------------------------------------------------------

struct ApplyArgs {
    float *table;
    float *state;
    const uint32_t *hot_bits; // the table's declared hot-key set or null (see takes_hot_path)
    const uint32_t *uniq, *seg, *perm, *meta;
    const uint4 *chunk_of; // per chunk: {segment, the segment's first chunk, the segment's first position, its end}
    uint32_t *chunk_done;
    float *partial;        // [max_chunks][stride] partial sums of chunked segments
    int stride;
    uint32_t n;            // accesses of the plan
    uint32_t max_chunks;   // capacity of the chunk lists and of `partial`
    uint32_t deterministic; // the chunks' partial rows are added in chunk order by one group, however many
    float *replica_rows;   // rows of the keys from base_keys on (replicas of hot keys), or null
    uint32_t base_keys;    // keys below are rows of `table`
    float *totals;         // [workgroups of the launch][kGroupsPerBlock][stride] running totals of segments of more
                           // than kChunk accesses that one group sums by itself
};

// LDS of the update kernels: one row per row group.  Row `group` holds a group's block sum while a chunk is
// combined, or the running super-block sum of a long segment that one group sums by itself (that segment's running
// total over super-blocks, needed beyond kChunk accesses only, lives in global memory: ApplyArgs::totals).
__host__ __device__ constexpr size_t apply_lds_bytes(int stride) { return sizeof(float) * kGroupsPerBlock * (size_t)stride; }

// Rows that a group requests together while it sums a block.  More rows in flight hide more latency per group but
// cost a row of registers each; with rows of 320 floats and more, two in flight keep the update kernels at four
// wavefronts per SIMD, so that every work item of a step of the large skip-gram configuration is resident at once;
// rows of 1,024 floats (64 registers each) one at a time: two wavefronts per SIMD instead of one (update kernel of
// the 1.9M-word, d = 1000 workload: 39.7 -> 35.3 us).
template <int NV4>
constexpr int kRowsInFlight = NV4 >= 16 ? 1 : NV4 >= 5 ? 2 : 4;

// Does the access in lane kLane of the group (source row number r there) take part in a block of m accesses?
template <int kLane, bool kSkips>
__device__ __forceinline__ bool takes_part(uint32_t r, uint32_t m)
{
    if constexpr (kLane >= kGroup) {
        return false;
    } else {
        if ((uint32_t)kLane >= m) return false;
        return !kSkips || group_share<kLane>(r) < kRowDone;   // neither kNoRow nor kRowDone: a row of the source
    }
}

template <int NV4, int kLane>
__device__ __forceinline__ void load_shared_row(Row<NV4> &x, const float *rows, uint32_t r, int stride, int lane)
{
    if constexpr (kLane < kGroup) load_row(x, rows + (size_t)group_share<kLane>(r) * stride, lane);
}

template <int NV4, int kLane>
__device__ __forceinline__ void add_shared_row(Row<NV4> &acc, float c, const Row<NV4> &x)
{
    if constexpr (kLane < kGroup) axpy_row(acc, group_share<kLane>(c), x);
}

// kRows accesses of a block of sixteen: their coefficients and source row numbers sit in lanes kFirst .. kFirst +
// kRows - 1 of the group (c, r); m = accesses in the block, kFirst < m.  The rows are requested together and added
// in order.
template <int NV4, int kFirst, int kRows, bool kSkips>
__device__ __forceinline__ void sum_rows(Row<NV4> &acc, const float *rows, uint32_t r, float c, uint32_t m, int stride,
                                         int lane)
{
    static_assert(kRows >= 1 && kRows <= 4, "one to four rows in flight");
    Row<NV4> x[kRows];
    const bool on0 = takes_part<kFirst, kSkips>(r, m), on1 = kRows > 1 && takes_part<kFirst + 1, kSkips>(r, m),
               on2 = kRows > 2 && takes_part<kFirst + 2, kSkips>(r, m), on3 = kRows > 3 && takes_part<kFirst + 3, kSkips>(r, m);
    if (on0) load_shared_row<NV4, kFirst>(x[0], rows, r, stride, lane);
    if constexpr (kRows > 1) if (on1) load_shared_row<NV4, kFirst + 1>(x[1], rows, r, stride, lane);
    if constexpr (kRows > 2) if (on2) load_shared_row<NV4, kFirst + 2>(x[2], rows, r, stride, lane);
    if constexpr (kRows > 3) if (on3) load_shared_row<NV4, kFirst + 3>(x[3], rows, r, stride, lane);
    if (on0) add_shared_row<NV4, kFirst>(acc, c, x[0]);
    if constexpr (kRows > 1) if (on1) add_shared_row<NV4, kFirst + 1>(acc, c, x[1]);
    if constexpr (kRows > 2) if (on2) add_shared_row<NV4, kFirst + 2>(acc, c, x[2]);
    if constexpr (kRows > 3) if (on3) add_shared_row<NV4, kFirst + 3>(acc, c, x[3]);
}

template <int NV4, int kFirst, int kMost, bool kSkips>
__device__ __forceinline__ void sum_rows_from(Row<NV4> &acc, const float *rows, uint32_t r, float c, uint32_t m,
                                              int stride, int lane)
{
    constexpr int kRows = kRowsInFlight<NV4>;
    if constexpr (kFirst < kMost) {
        if (kFirst == 0 || (uint32_t)kFirst < m) {
            sum_rows<NV4, kFirst, kRows, kSkips>(acc, rows, r, c, m, stride, lane);
            sum_rows_from<NV4, kFirst + kRows, kMost, kSkips>(acc, rows, r, c, m, stride, lane);
        }
    }
}

// acc += the contributions of accesses t0 .. min(t0 + kMost, last) - 1 of a segment, in that order:
// lane l of the group fetches the l-th access's coefficient and source row number, so the dependent reads
// that lead to a row's address are paid once for all of them rather than once per access; the rows are then
// read a few at a time.  Every lane of the group must call it with the same arguments; t0 < last.
template <int NV4, uint32_t kMost, class Src>
__device__ __forceinline__ void sum_block(Row<NV4> &acc, const Src &src, const uint32_t *perm, uint32_t t0,
                                          uint32_t last, int stride, int lane)
{
    static_assert(kMost <= (uint32_t)kGroup, "one access per lane");
    const float *rows = src.rows();
    const uint32_t m = min(kMost, last - t0);
    uint32_t r = 0;
    float c = 0.0f;
    if ((uint32_t)lane < m) src.fetch(perm, t0 + (uint32_t)lane, c, r);
    sum_rows_from<NV4, 0, (int)kMost, Src::kSkips>(acc, rows, r, c, m, stride, lane);
}

// row <- x if `first`, else row + x (LDS or global memory); each lane touches its own words only, so neither a
// barrier nor a fence is involved.
template <int NV4>
__device__ __forceinline__ void accumulate_row(float *row, const Row<NV4> &x, bool first, int lane)
{
    if (first) {
        store_row(row, x, lane);
    } else {
        Row<NV4> t;
        load_row(t, row, lane);
        axpy_row(t, 1.0f, x);
        store_row(row, t, lane);
    }
}

// acc = sum of the whole segment [first, last) by one group, in the fixed tree (blocks, super-blocks, total).
// super_row: this group's row of LDS; total_row: this group's row of running totals in global memory.
template <int NV4, class Src>
__device__ __forceinline__ void sum_segment(Row<NV4> &acc, const Src &src, const uint32_t *perm, uint32_t first,
                                            uint32_t last, int stride, int lane, float *super_row, float *total_row)
{
    zero_row(acc);
    if (last - first <= kLongSegment) {
        if (first < last) sum_block<NV4, kLongSegment>(acc, src, perm, first, last, stride, lane);
        return;
    }
    const bool several = last - first > kChunk;
    for (uint32_t s0 = first; s0 < last; s0 += kChunk) {
        const uint32_t s1 = min(s0 + kChunk, last);
        for (uint32_t t0 = s0; t0 < s1; t0 += kTreeBlock) {
            zero_row(acc);
            sum_block<NV4, kTreeBlock>(acc, src, perm, t0, s1, stride, lane);
            accumulate_row(super_row, acc, t0 == s0, lane);
        }
        if (several) {
            load_row(acc, super_row, lane);
            accumulate_row(total_row, acc, s0 == first, lane);
        }
    }
    load_row(acc, several ? total_row : super_row, lane);
}

// Work items of a plan: one per chunk (kChunk accesses) of a long segment, and the short segments (at most
// kLongSegment accesses, or any length if the key is not in a declared hot set), one 16-lane group each, in key
// order: rows are then visited in ascending address order and every group of an item has a segment.  (Walking
// the accesses instead, with the key straight from the key array, saves two dependent reads per row but leaves
// the groups of repeated accesses idle and visits rows in batch order; it measured slower on every workload.)
struct ApplyShape {
    uint32_t nu, chunk_items, short_items;
};

// Segments per row group in an item of short segments (two, one after the other, measured slower: 40.9 instead of
// 38.8 us per step of the large skip-gram configuration; the items get twice as long).
constexpr int kSegmentsPerGroup = 1;
constexpr uint32_t kSegmentsPerItem = kGroupsPerBlock * kSegmentsPerGroup;

__device__ __forceinline__ ApplyShape apply_shape(const ApplyArgs &a)
{
    ApplyShape sh;
    sh.nu = a.meta[kMetaNumUniq];
    sh.chunk_items = min(a.meta[kMetaNumChunks], a.max_chunks);
    sh.short_items = (sh.nu + kSegmentsPerItem - 1) / kSegmentsPerItem;
    return sh;
}

// src.done_in_rows for the sources that have it (kDoneInRows); never called for the others.
template <class Src>
__device__ __forceinline__ bool done_in_rows_of(const Src &src, uint32_t r, uint32_t n, int lane)
{
    if constexpr (Src::kDoneInRows) return src.done_in_rows(r, n, lane);
    else return false;
}

template <class Src>
__device__ __forceinline__ bool single_is_done(const Src &src)
{
    if constexpr (Src::kDoneInRows) return src.singles_done;
    else return false;
}

// One item of short segments: this group's segments, if it has any (segment numbers item * kSegmentsPerItem +
// group + k * kGroupsPerBlock: neighbouring groups update neighbouring rows).
template <int NV4, class Src, class Opt>
__device__ __forceinline__ void apply_short_item(const ApplyArgs &a, const Src &src, const Opt &opt,
                                                 const ApplyShape &sh, uint32_t item, float *lds, uint32_t workgroup,
                                                 int lane, int group)
{
    uint32_t key[kSegmentsPerGroup], first[kSegmentsPerGroup], last[kSegmentsPerGroup];
#pragma unroll
    for (int k = 0; k < kSegmentsPerGroup; ++k) {
        const uint32_t u = item * kSegmentsPerItem + (uint32_t)k * kGroupsPerBlock + group;
        key[k] = 0;
        first[k] = last[k] = 0;          // an empty range: nothing to do
        if (u < sh.nu) {
            key[k] = a.uniq[u];
            first[k] = a.seg[u];
            last[k] = a.seg[u + 1];
        }
    }
#pragma unroll
    for (int k = 0; k < kSegmentsPerGroup; ++k) {
        if (first[k] >= last[k]) continue;
        if (takes_hot_path(last[k] - first[k], key[k], a.hot_bits, a.base_keys)) continue;   // summed by chunk items
        Row<NV4> acc, t, g;
        const uint32_t n = last[k] - first[k];
        if (Src::kDoneInRows && n <= kLongSegment) {   // one fetch serves the question and the sum
            static_assert(kLongSegment <= (uint32_t)kGroup, "one access per lane");
            if (n == 1 && single_is_done(src)) continue;
            uint32_t r = 0;
            float c = 0.0f;
            if ((uint32_t)lane < n) src.fetch(a.perm, first[k] + (uint32_t)lane, c, r);
            if (done_in_rows_of(src, r, n, lane)) continue;      // the gradient kernel has updated this row itself
            zero_row(acc);
            sum_rows_from<NV4, 0, (int)kLongSegment, Src::kSkips>(acc, src.rows(), r, c, n, a.stride, lane);
        } else {
            if (src.segment_done(a.perm, first[k], last[k], lane)) continue;    // the gradient kernel has updated this row itself
            sum_segment<NV4>(acc, src, a.perm, first[k], last[k], a.stride, lane, lds + (size_t)group * a.stride,
                             a.totals + ((size_t)workgroup * kGroupsPerBlock + group) * a.stride);
        }
        float *row = extended_row(a.table, a.replica_rows, a.base_keys, key[k], a.stride);
        float *state_row = Opt::kHasState ? a.state + (size_t)key[k] * a.stride : nullptr;   // tables with state have no replicas
        opt.template load<NV4>(t, g, row, state_row, lane);   // after the sum: results are waited for in issue order, an early request of the cold row holds up the sum's first reads
        if (opt.clips() && a.hot_bits != nullptr && in_hot_set(key[k], a.hot_bits, a.base_keys)) opt.template clip<NV4>(acc, lane);
        opt.template finish<NV4>(t, g, row, state_row, acc, lane);
    }
}

// The counter of a chunked segment: how many of its chunks have left their partial row.  The partial rows travel
// as device-scope word accesses (device_utils.h), which are performed at the memory side of the dies' caches; the
// storing wavefront waits for their acknowledgement before it counts itself in, and the workgroup that sees the
// last count reads them with device-scope loads after its barrier: no cache write-back or invalidation is needed
// (a release fence at device scope writes back the whole L2 of the die, which holds the step's updated rows:
// measured at 8.6 us of a 32 us launch).  NUPS_HANDOFF_RELEASE_ACQUIRE builds the formally ordered variant.
__device__ __forceinline__ uint32_t count_chunk_in(uint32_t *counter)
{
#if defined(NUPS_HANDOFF_RELEASE_ACQUIRE)
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
#else
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#endif
}

// One chunk (super-block) of a long segment, by the whole workgroup: group g sums block g of the chunk, the
// block sums are added in block order through LDS, and the workgroup that finishes a segment's last outstanding
// chunk adds the chunks' partial rows and updates the row.  Contains workgroup barriers: every thread of the
// workgroup must call it with the same `id`.
template <int NV4, class Src, class Opt>
__device__ __forceinline__ void apply_chunk_item(const ApplyArgs &a, const Src &src, const Opt &opt, uint32_t id,
                                                 const uint4 chunk, float *part, uint32_t *last_arrival, int lane,
                                                 int group)
{
    const uint32_t u = chunk.x, base = chunk.y, first = chunk.z, last = chunk.w;   // chunk = a.chunk_of[id]
    const uint32_t nch = (last - first + kChunk - 1) / kChunk;
    const uint32_t cf = first + (id - base) * kChunk, cl = min(cf + kChunk, last);
    const uint32_t blocks = (cl - cf + kTreeBlock - 1) / kTreeBlock;     // non-empty blocks of this chunk
    Row<NV4> acc;
    zero_row(acc);
    if ((uint32_t)group < blocks)
        sum_block<NV4, kTreeBlock>(acc, src, a.perm, cf + (uint32_t)group * kTreeBlock, cl, a.stride, lane);
    __syncthreads();                  // LDS of the previous item has been read
    if (group > 0 && (uint32_t)group < blocks) store_row(part + (size_t)group * a.stride, acc, lane);
    __syncthreads();
    if (group == 0) {
        for (uint32_t g = 1; g < blocks; ++g) {
            Row<NV4> r;
            load_row(r, part + (size_t)g * a.stride, lane);
            axpy_row(acc, 1.0f, r);
        }
        if (nch > 1) {
            store_row_device_scope(a.partial + (size_t)id * a.stride, acc, lane);
            all_stores_performed();   // the partial row is in place before the arrival is counted (same wavefront)
        }
    }
    bool update = true;
    if (nch > 1) {
        __syncthreads();
        if (threadIdx.x == 0) *last_arrival = (count_chunk_in(&a.chunk_done[base]) == nch - 1) ? 1u : 0u;
        __syncthreads();
        update = *last_arrival != 0;
        if (update) {
            const float *prow = a.partial + (size_t)base * a.stride;
            if (!a.deterministic) {   // every group adds an interleaved share of the partial rows, combined in group order
                zero_row(acc);
                for (uint32_t ch = group; ch < nch; ch += kGroupsPerBlock) {
                    Row<NV4> r;
                    load_row_device_scope(r, prow + (size_t)ch * a.stride, lane);
                    axpy_row(acc, 1.0f, r);
                }
                const uint32_t shares = min(nch, (uint32_t)kGroupsPerBlock);
                if (group > 0 && (uint32_t)group < shares) store_row(part + (size_t)group * a.stride, acc, lane);   // LDS is free again
                __syncthreads();
                if (group == 0) {
                    for (uint32_t g = 1; g < shares; ++g) {
                        Row<NV4> r;
                        load_row(r, part + (size_t)g * a.stride, lane);
                        axpy_row(acc, 1.0f, r);
                    }
                }
            } else if (group == 0) { // chunk order, by one group: the fixed tree's last level; every chunk has arrived
                zero_row(acc);
                uint32_t ch = 0;
                for (; ch + 1 < nch; ch += 2) {
                    Row<NV4> r0, r1;
                    load_row_device_scope(r0, prow + (size_t)ch * a.stride, lane);
                    load_row_device_scope(r1, prow + (size_t)(ch + 1) * a.stride, lane);
                    axpy_row(acc, 1.0f, r0);
                    axpy_row(acc, 1.0f, r1);
                }
                if (ch < nch) {
                    Row<NV4> r;
                    load_row_device_scope(r, prow + (size_t)ch * a.stride, lane);
                    axpy_row(acc, 1.0f, r);
                }
            }
            if (threadIdx.x == 0) a.chunk_done[base] = 0u;   // ready for the next step
        }
    }
    if (update && group == 0) {
        const uint32_t key = a.uniq[u];
        float *row = extended_row(a.table, a.replica_rows, a.base_keys, key, a.stride);
        float *state_row = Opt::kHasState ? a.state + (size_t)key * a.stride : nullptr;
        Row<NV4> t, g;
        opt.template load<NV4>(t, g, row, state_row, lane);
        if (opt.clips() && a.hot_bits != nullptr) opt.template clip<NV4>(acc, lane);   // chunked and declared: a hot key
        opt.template finish<NV4>(t, g, row, state_row, acc, lane);
    }
    __syncthreads();                  // the block sums in LDS have been read: the groups' rows are theirs again
}

// Updates one table.  A fixed-size grid walks over the items, chunks first (they are the long poles); every
// workgroup leaves the loop after at most ceil(items / gridDim) turns.
// Updates one table.  A fixed-size grid walks over the items, chunks first (they are the long poles); every
// workgroup leaves the loop after at most ceil(items / gridDim) turns.  (Handing the items beyond the first round
// out through a counter, so that whichever workgroup finishes first carries on, was measured: the atomics of all
// workgroups on the one counter and the barriers around them cost far more than the idle slots they fill: 44 instead
// of 39 us per step of the large skip-gram configuration, 126 instead of 64 us for the factorisation.)
template <int NV4, class Src, class Opt>
__global__ void __launch_bounds__(kBlock) k_apply(ApplyArgs a, Src src, Opt opt)
{
    extern __shared__ float part[];   // apply_lds_bytes(stride)
    __shared__ uint32_t last_arrival;
    const int lane = threadIdx.x & (kGroup - 1), group = threadIdx.x / kGroup;
    const ApplyShape sh = apply_shape(a);
    const uint32_t items = sh.chunk_items + sh.short_items;
    for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
        if (item < sh.chunk_items) apply_chunk_item<NV4>(a, src, opt, item, a.chunk_of[item], part, &last_arrival, lane, group);
        else apply_short_item<NV4>(a, src, opt, sh, item - sh.chunk_items, part, blockIdx.x, lane, group);
    }
}

// Updates the two tables of a step in one launch (their updates are independent of each other: both read
// staged rows only).  Item order: chunks of table 0, chunks of table 1, short segments of 0, of 1.  The first
// sw.blocks workgroups do preparatory work of later steps instead.
// Wavefronts per SIMD that the update of both tables is compiled for.  Rows of 320 floats sit a register or two
// above the limit for four; with four, the work items of a step of the large skip-gram configuration are (nearly)
// all resident at once.  Other widths: whatever the code needs.
template <int NV4>
constexpr int kApply2WavesPerSimd = NV4 == 5 ? 4 : 1;

template <int NV4, class Src0, class Opt0, class Src1, class Opt1>
__global__ void __launch_bounds__(kBlock, kApply2WavesPerSimd<NV4>) k_apply2(ApplyArgs a0, Src0 src0, Opt0 opt0, ApplyArgs a1, Src1 src1,
                                                   Opt1 opt1, SideWork sw)
{
    extern __shared__ float part[];   // apply_lds_bytes(stride)
    __shared__ uint32_t last_arrival;
    if (side_work_block(sw)) return;
    const uint32_t first_item = blockIdx.x - sw.blocks, item_step = gridDim.x - sw.blocks;
    const int lane = threadIdx.x & (kGroup - 1), group = threadIdx.x / kGroup;
    // The first items are the chunks of the first table, the longest of the launch: a workgroup asks for the chunk
    // that its number stands for together with the item counts (one dependent read fewer in front of the rows; the
    // entry is inside the array whatever it holds, and is used only if the counts confirm it).  Not for rows of up
    // to 128 floats, whose launches have four times as many workgroups with little to do each: there the extra
    // read costs more than it saves (factorisation at rank 100: 64.9 against 63.2 us per step).
    constexpr bool kAskAhead = NV4 >= 3;
    uint4 own_chunk = make_uint4(0u, 0u, 0u, 0u);
    if (kAskAhead && first_item < a0.max_chunks) own_chunk = a0.chunk_of[first_item];
    const ApplyShape s0 = apply_shape(a0), s1 = apply_shape(a1);
    const uint32_t e0 = s0.chunk_items, e1 = e0 + s1.chunk_items, e2 = e1 + s0.short_items,
                   e3 = e2 + s1.short_items;
    for (uint32_t item = first_item; item < e3; item += item_step) {
        if (item < e0) apply_chunk_item<NV4>(a0, src0, opt0, item, (kAskAhead && item == first_item) ? own_chunk : a0.chunk_of[item], part, &last_arrival, lane, group);
        else if (item < e1) apply_chunk_item<NV4>(a1, src1, opt1, item - e0, a1.chunk_of[item - e0], part, &last_arrival, lane, group);
        else if (item < e2) apply_short_item<NV4>(a0, src0, opt0, s0, item - e1, part, first_item, lane, group);
        else apply_short_item<NV4>(a1, src1, opt1, s1, item - e2, part, first_item, lane, group);
    }
}

// Workgroups of the update kernels: 8 per compute unit; narrow rows (many short items, little state per
// workgroup) do better with one item per workgroup, up to 32 per compute unit.
template <int NV4>
constexpr uint32_t kApplyGrid = NV4 <= 2 ? 8192 : 2048;

static inline uint32_t apply_grid_of_stride(int stride) { return stride / 64 <= 2 ? kApplyGrid<2> : kApplyGrid<8>; }

// Where an update launch keeps its workgroups' running totals and how many workgroups it may use at most.
struct ApplyScratch {
    float *totals;       // [grid_cap][kGroupsPerBlock][stride]
    uint32_t grid_cap;
};

static inline size_t apply_totals_floats(uint32_t grid_cap, int stride) { return (size_t)grid_cap * kGroupsPerBlock * stride; }

static inline ApplyArgs make_apply_args(const Plan &pl, float *partial, float *table, float *state, int stride,
                                        float *totals, float *replica_rows = nullptr)
{
    const PlanArgs &p = pl.a;
    return ApplyArgs{table, state, p.hot_bits, p.uniq, p.seg, p.deterministic ? p.perm_sorted : p.perm, p.meta,
                     p.chunk_of, p.chunk_done, partial, stride, p.n, p.max_chunks, p.deterministic,
                     replica_rows, p.rep.base_keys, totals};
}

static inline uint32_t max_apply_items(const Plan &pl)
{
    return (pl.a.n + kGroupsPerBlock - 1) / kGroupsPerBlock + (uint32_t)max_chunks(pl.a.n);
}

// Workgroups that ask for more dynamic LDS than the default limit of 64 KB (wide rows) say so first; the device
// has 160 KB per compute unit.  `allowed`: what this kernel has been granted so far (one variable per kernel).
template <class Kernel>
static void allow_lds(Kernel kernel, size_t lds, size_t *allowed)
{
    if (lds <= 48 * 1024 || lds <= *allowed) return;
    if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess)
        *allowed = lds;
}

template <int NV4, class Src, class Opt>
static void launch_apply_nv(hipStream_t s, const Plan &pl, float *partial, const ApplyScratch &scratch, float *table,
                            float *state, int stride, const Src &src, const Opt &opt)
{
    if (pl.a.n == 0) return;
    const ApplyArgs a = make_apply_args(pl, partial, table, state, stride, scratch.totals);
    const size_t lds = apply_lds_bytes(stride);
    static size_t allowed = 0;
    allow_lds(k_apply<NV4, Src, Opt>, lds, &allowed);
    const uint32_t grid = std::min({max_apply_items(pl), kApplyGrid<NV4>, scratch.grid_cap});
    hipLaunchKernelGGL((k_apply<NV4, Src, Opt>), dim3(grid), dim3(kBlock), lds, s, a, src, opt);
}

#define NUPS_FOR_EACH_ROW_WIDTH(stride, CALL)                                                     \
    switch ((stride) / 64) {                                                                      \
    case 1: CALL(1); break;                                                                       \
    case 2: CALL(2); break;                                                                       \
    case 3: CALL(3); break;                                                                       \
    case 4: CALL(4); break;                                                                       \
    case 5: CALL(5); break;                                                                       \
    case 6: CALL(6); break;                                                                       \
    case 8: CALL(8); break;                                                                       \
    case 16: CALL(16); break;                                                                     \
    default:                                                                                      \
        return fail(NUPS_ERR_UNIMPLEMENTED,                                                       \
                    "row_stride must be 64, 128, 192, 256, 320, 384, 512 or 1024 floats");        \
    }

// One table: dispatch on the row length (stride / 64 float4 per lane).
template <class Src, class Opt>
static nups_status launch_apply(hipStream_t s, const Plan &pl, float *partial, const ApplyScratch &scratch,
                                float *table, float *state, int stride, const Src &src, const Opt &opt)
{
#define NUPS_CALL(N) launch_apply_nv<N>(s, pl, partial, scratch, table, state, stride, src, opt)
    NUPS_FOR_EACH_ROW_WIDTH(stride, NUPS_CALL)
#undef NUPS_CALL
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

// What one table's update needs besides its plan.
template <class Src, class Opt>
struct TableUpdate {
    const Plan *plan;
    float *partial, *table, *state;
    Src src;
    Opt opt;
    float *replica_rows = nullptr;   // of the table's hot keys, if it has replicas
};

template <int NV4, class U0, class U1>
static void launch_apply2_nv(hipStream_t s, int stride, const U0 &u0, const U1 &u1, const ApplyScratch &scratch,
                             const SideWork &sw, size_t side_lds)
{
    const ApplyArgs a0 = make_apply_args(*u0.plan, u0.partial, u0.table, u0.state, stride, scratch.totals, u0.replica_rows);
    const ApplyArgs a1 = make_apply_args(*u1.plan, u1.partial, u1.table, u1.state, stride, scratch.totals, u1.replica_rows);
    const uint32_t items = max_apply_items(*u0.plan) + max_apply_items(*u1.plan);
    const size_t lds = std::max(apply_lds_bytes(stride), side_lds);
    static size_t allowed = 0;
    const auto kernel = k_apply2<NV4, decltype(u0.src), decltype(u0.opt), decltype(u1.src), decltype(u1.opt)>;
    allow_lds(kernel, lds, &allowed);
    const uint32_t grid = std::max(1u, std::min({items, kApplyGrid<NV4>, scratch.grid_cap}));
    hipLaunchKernelGGL(kernel, dim3(sw.blocks + grid), dim3(kBlock), lds, s,
                       a0, u0.src,
                       u0.opt, a1, u1.src, u1.opt, sw);
}

// Both tables of a step in one launch (both strides are equal), plus the side work `sw`.
template <class U0, class U1>
static nups_status launch_apply2(hipStream_t s, int stride, const U0 &u0, const U1 &u1, const ApplyScratch &scratch,
                                 const SideWork &sw, size_t side_lds)
{
#define NUPS_CALL(N) launch_apply2_nv<N>(s, stride, u0, u1, scratch, sw, side_lds)
    NUPS_FOR_EACH_ROW_WIDTH(stride, NUPS_CALL)
#undef NUPS_CALL
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

}  // namespace nups
