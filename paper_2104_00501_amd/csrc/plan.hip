// Host side of a step's preparatory work (device side: side_work.h): the arrays of a per-key aggregation
// structure ("plan"), and the list of phases that builds it.
#include <algorithm>
#include <initializer_list>

#include "nups_internal.h"

namespace nups {

// (Re)allocates; the stream is idle when this is called, and the clearing has finished when it returns.
static nups_status grow_u32(uint32_t **buf, size_t n, bool zero)
{
    if (*buf) NUPS_HIP(hipFree(*buf));
    *buf = nullptr;
    NUPS_HIP(hipMalloc((void **)buf, sizeof(uint32_t) * (n ? n : 1)));
    if (zero) NUPS_HIP(hipMemset(*buf, 0, sizeof(uint32_t) * (n ? n : 1)));
    return NUPS_OK;
}

// Keys of a table's extended key space: its rows, then the replica rows of its hot keys.
int64_t extended_keys(const nups_ctx *ctx, const Table &t)
{
    return t.num_keys + (ctx->replicas > 0 && t.hot_slot_dev ? (int64_t)ctx->replicas * (int64_t)t.hot_keys.size() : 0);
}

size_t max_chunks(size_t n) { return n / kChunk + n / (kLongSegment + 1) + 2; }

// Room for `need` floats of partial rows of chunked segments; growing waits for the stream.
nups_status ensure_partial(nups_ctx *ctx, size_t need)
{
    return ensure_f32(&ctx->partial, &ctx->partial_cap, need, ctx->stream);
}

// Room for the running totals of an update launch over rows of `stride` floats (its largest grid).
nups_status ensure_totals(nups_ctx *ctx, int stride)
{
    const size_t grid = stride / 64 <= 2 ? 8192 : 2048;   // apply_grid_of_stride (segment_apply.h)
    return ensure_f32(&ctx->totals, &ctx->totals_cap, grid * kGroupsPerBlock * (size_t)stride, ctx->stream);
}

void free_plan_arrays(Plan &pl)
{
    PlanArgs &a = pl.a;
    for (uint32_t *p : {a.uniq, a.count, a.seg, a.perm, a.perm_sorted, a.perm_pieces, a.slot, a.pos, a.rank, (uint32_t *)a.chunk_of, a.chunk_done, a.meta,
                        a.bitmap, a.word_rank, a.tile_sum, a.tile_prefix, a.cnt_work})
        if (p) (void)hipFree(p);
    if (a.bytemap) (void)hipFree(a.bytemap);
    if (a.wordmap) (void)hipFree(a.wordmap);
    pl = Plan{};
}

// Makes the plan's arrays large enough for n accesses to table t and fills in the plan's pointers and shape
// fields.  Growing waits for the stream: kernels in flight may still read the arrays that are replaced.
nups_status ensure_plan_capacity(nups_ctx *ctx, Table &t, Plan &pl, size_t n)
{
    PlanArgs &a = pl.a;
    nups_status st;
    const size_t words = (size_t)((extended_keys(ctx, t) + 31) / 32);
    if (pl.cap_words < words) {
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        if ((st = grow_u32(&a.bitmap, words, true)) != NUPS_OK) return st;
        if ((st = grow_u32((uint32_t **)&a.bytemap, words * 8, true)) != NUPS_OK) return st;   // 32 bytes per word
        if ((st = grow_u32((uint32_t **)&a.wordmap, (words + 3) / 4, true)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.word_rank, words, false)) != NUPS_OK) return st;
        pl.cap_words = words;
    }
    if (pl.cap_n < n || pl.cap_n == 0) {
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        const size_t cap = n + n / 4 + 1024;
        for (uint32_t **b : {&a.uniq, &a.count, &a.slot, &a.rank})
            if ((st = grow_u32(b, cap, false)) != NUPS_OK) return st;
        // zeroed: a position that a build leaves out (a key array changed behind a prepared step) then holds an
        // access number of an earlier build or zero, never an arbitrary word
        for (uint32_t **b : {&a.perm, &a.perm_sorted, &a.perm_pieces, &a.pos})
            if ((st = grow_u32(b, cap, true)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.cnt_work, (cap + kScanTile - 1) / kScanTile * kScanTile, true)) != NUPS_OK) return st;   // whole tiles
        if ((st = grow_u32(&a.seg, cap + 1, false)) != NUPS_OK) return st;
        if ((st = grow_u32((uint32_t **)&a.chunk_of, 4 * max_chunks(cap), false)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.chunk_done, max_chunks(cap), true)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.meta, kMetaWords, true)) != NUPS_OK) return st;
        pl.cap_n = cap;
    }
    const size_t tiles = std::max((words + kScanTile - 1) / kScanTile, (pl.cap_n + kScanTile - 1) / kScanTile);
    if (pl.cap_tiles < tiles) {
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        if ((st = grow_u32(&a.tile_sum, tiles, false)) != NUPS_OK) return st;
        if ((st = grow_u32(&a.tile_prefix, tiles, false)) != NUPS_OK) return st;
        pl.cap_tiles = tiles;
    }
    set_plan_shape(ctx, t, pl);
    return NUPS_OK;
}

// The shape fields of a plan whose arrays are in place (cap_n set) for table t.
void set_plan_shape(const nups_ctx *ctx, const Table &t, Plan &pl)
{
    PlanArgs &a = pl.a;
    const size_t words = (size_t)((extended_keys(ctx, t) + 31) / 32);
    a.num_keys = (uint32_t)extended_keys(ctx, t);
    a.rep = ReplicaMap{nullptr, (uint32_t)t.num_keys, 0u, 0u, 1u};
    if (ctx->replicas > 0 && t.hot_slot_dev)   // rep.batch: set with the step's batch size
        a.rep = ReplicaMap{t.hot_slot_dev, (uint32_t)t.num_keys, (uint32_t)t.hot_keys.size(), (uint32_t)ctx->replicas, 1u};
    a.max_chunks = (uint32_t)max_chunks(pl.cap_n);
    a.rank_items = 4u;   // accesses per thread of the rank phase (2 measured slower, also in narrow-row carriers)
    a.words = (uint32_t)words;
    a.bitmap_tiles = (uint32_t)((words + kScanTile - 1) / kScanTile);
    a.error_flag = ctx->error_flag;
    a.hot_bits = t.hot_bits_dev;
    a.deterministic = ctx->deterministic ? 1u : 0u;
}

// Dynamic LDS that the launch carrying this phase must provide.
size_t side_lds_bytes(const SideItem &it)
{
    if (it.phase == kSideRank) return rank_lds_bytes((int)it.plan[0].rank_items);
    if (it.phase == kSideSlot) return kSlotLdsBytes;
    if (it.phase == kSideSort) return sizeof(uint32_t) * kBlock;
    if (it.phase == kSideDraw && it.draw.scheme == NUPS_BOUNDED) return kDrawLdsBytes;
    return 0;
}

// The phases that build the step's plans (a.src, a.n, a.mark_n set by the caller).  `draw`: the samples that the
// step draws itself (scheme 0: none); they are marked in plan `mark_plan` as they are drawn.
void build_phases(nups_prepared &p, const SampleArgs &draw, int mark_plan)
{
    uint32_t max_mark = 0, max_n = 0, max_btiles = 0, max_ctiles = 0;
    bool need_count_tiles = false;
    for (int k = 0; k < p.n_plans; ++k) {
        PlanArgs &a = p.plan[k].a;
        a.count_tiles = std::max(1u, (a.n + kScanTile - 1) / kScanTile);   // also for an empty step: seg[0], totals
        a.direct_count = a.n <= 131072 ? 1u : 0u;
        need_count_tiles |= !a.direct_count;
        max_mark = std::max(max_mark, a.mark_n);
        max_n = std::max(max_n, a.n);
        max_btiles = std::max(max_btiles, a.bitmap_tiles);
        max_ctiles = std::max(max_ctiles, a.count_tiles);
    }
    SideItem it{};
    it.n_plans = p.n_plans;
    for (int k = 0; k < p.n_plans; ++k) it.plan[k] = p.plan[k].a;
    p.phases.clear();
    p.next_phase = 0;
    auto add = [&](int32_t phase, uint32_t per_plan, uint32_t extra) {
        it.phase = phase;
        it.block0 = 0;
        it.blocks_per_plan = per_plan;
        it.blocks = extra + per_plan * (uint32_t)p.n_plans;
        p.phases.push_back(it);
    };
    it.draw = draw;
    if (draw.scheme != 0 && mark_plan >= 0) {
        it.draw.bytemap = p.plan[mark_plan].a.bytemap;
        it.draw.wordmap = p.plan[mark_plan].a.wordmap;
        it.draw.mark_keys = p.plan[mark_plan].a.num_keys;
        it.draw.rep = p.plan[mark_plan].a.rep;
        it.draw.per_sample = (uint32_t)(p.batch.n_neg + p.batch.n_neg2);
    }
    const uint32_t draw_blocks = draw.scheme != 0 ? draw.blocks : 0u;
    it.draw.blocks = draw_blocks;
    add(kSideDraw, std::max(1u, (max_mark + kBlock - 1) / kBlock), draw_blocks);
    it.draw = SampleArgs{};
    add(kSideTiles, max_btiles, 0);
    if (max_btiles > kLdsTiles) add(kSidePrefix, 1, 0);   // else every workgroup of the next phase scans the tile counts
    add(kSideSlot, std::max(1u, (max_n + kSlotTile - 1) / kSlotTile), 0);
    const uint32_t rank_tile = kBlock * p.plan[0].a.rank_items;
    for (int k = 1; k < p.n_plans; ++k) it.plan[k].rank_items = p.plan[0].a.rank_items;   // one tile size per launch
    add(kSideRank, std::max(1u, (max_n + rank_tile - 1) / rank_tile), 0);
    if (need_count_tiles) add(kSideCountTiles, max_ctiles, 0);
    add(kSideCounts, max_ctiles, 0);
    add(kSideScatter, std::max(1u, (max_n + kBlock - 1) / kBlock), 0);
    if (p.plan[0].a.deterministic) {
        add(kSideSort, std::max(1u, (max_n + kBlock - 1) / kBlock), 0);
        add(kSideMerge, std::max(1u, (max_n + kBlock - 1) / kBlock), 0);
    }
}

}  // namespace nups
