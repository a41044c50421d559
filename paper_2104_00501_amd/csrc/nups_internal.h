// Internal declarations shared by the translation units of libnups (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <deque>
#include <string>
#include <vector>

#include "../../include/nups.h"

namespace nups {

constexpr int kGroup = 16;            // lanes that cooperate on one row (one DPP row of a wavefront)
constexpr int kBlock = 256;           // threads per workgroup (4 wavefronts, 16 row groups)
constexpr int kGroupsPerBlock = kBlock / kGroup;
constexpr int kMaxTables = 4;
constexpr int kMaxSide = 4;            // later steps whose preparatory work one launch can carry (one phase each)
constexpr int kMaxStride = 1024;
constexpr int kScanItems = 2;         // items per thread in the tile scans
constexpr int kScanTile = kBlock * kScanItems;
// A step's loss is accumulated in kLossSlots partial sums, each on a cache line of its own (kLossStride doubles
// apart): thousands of workgroups adding to one address would queue up behind each other.  The host adds the slots.
constexpr int kLossSlots = 64;
constexpr int kLossStride = 16;
// Flag in rank[i]: access i is the only access of its key in this step (its position is then 0).
constexpr uint32_t kSingleAccess = 0x80000000u;
constexpr uint32_t kLongSegment = 16; // segments with more accesses are summed by whole workgroups, in chunks
constexpr uint32_t kChunk = 256;      // accesses of a long segment that one workgroup sums (a super-block)
constexpr uint32_t kTreeBlock = kChunk / kGroupsPerBlock;   // accesses of a long segment that are added one after the other (a block: what one row group sums of a chunk)
constexpr uint32_t kBadIndex = 0xFFFFFFFFu;
constexpr int kSlotItems = 2;                       // accesses per thread in the slot phase of the preparatory work
constexpr int kSlotTile = kBlock * kSlotItems;
// Rank phase: accesses per thread, 2 or 4 (PlanArgs::rank_items).  More per workgroup means fewer global atomics
// on hot keys (each workgroup combines its accesses to a key first) but four LDS words per slot of a hash table
// with two slots per access: 16 KB or 32 KB that every workgroup of the carrying launch is charged for.
constexpr size_t rank_lds_bytes(int items) { return (size_t)4 * 2 * kBlock * items * sizeof(uint32_t); }
constexpr uint32_t kLdsTiles = 2048;                // tile counts that a workgroup scans in LDS by itself (64M keys)
constexpr size_t kSlotLdsBytes = kLdsTiles * sizeof(uint32_t);
constexpr uint32_t kMaxPool = 1024;                 // BOUNDED: largest pool (its order words are kept in LDS)
constexpr size_t kDrawLdsBytes = (kMaxPool + 8) * sizeof(uint32_t);

// meta words of a plan (device)
enum { kMetaNumUniq = 0, kMetaNumChunks = 1, kMetaTotal = 2, kMetaWords = 4 };

// Random streams of the counter-based generator.
enum { kStreamFresh = 1, kStreamOrder = 2, kStreamLocal = 3, kStreamRoundKey = 4 };

void set_error(const std::string &msg);
nups_status fail(nups_status st, const std::string &msg);
bool hip_ok(hipError_t e, const char *what);

#define NUPS_HIP(call)                                                  \
    do {                                                                \
        if (!::nups::hip_ok((call), #call)) return NUPS_ERR_DEVICE;     \
    } while (0)

// Up to three key arrays that together list the accesses to one table in one step.
struct KeySource {
    const uint32_t *ptr[3];
    uint32_t len[3];
    uint32_t per[3];       // entries of each array per example (0 is read as 1): entry j belongs to example j / per
};

// Stale replicas of a table's hot keys (Section 3.2: hot-spot keys are replicated on every node, and a node's workers
// read and update the node's replica).  The nodes are `replicas` contiguous parts of the minibatch: example e of
// `batch` belongs to part e * replicas / batch.  Replica r of hot key number s is row r * hot_count + s of a buffer
// of the library's, addressed as key base_keys + r * hot_count + s of an extended key space; keys below base_keys
// are the table's own rows.  hot_slot == null: the table has no replicas.
struct ReplicaMap {
    const uint32_t *hot_slot;   // [base_keys] number of the key in the hot list, kBadIndex if it is not hot
    uint32_t base_keys;         // keys of the table itself
    uint32_t hot_count, replicas, batch;
};

// Device-side description of the per-key aggregation structure of one table for one step:
// distinct keys in ascending order, the number of accesses of each, and the accesses grouped by key.
struct PlanArgs {
    KeySource src;
    uint32_t n;            // accesses (sum of src.len)
    uint32_t mark_n;       // the first mark_n accesses are marked by the structure's own first phase; the rest
                           // (samples that the step draws itself) are marked as they are drawn
    uint32_t num_keys;     // V, plus the replica rows of the hot keys if the table has replicas (rep)
    ReplicaMap rep;        // rep.base_keys = V also without replicas: a key of the batch is valid below it
    uint32_t words;        // bitmap words = ceil(V / 32)
    uint32_t bitmap_tiles; // ceil(words / kScanTile)
    uint32_t count_tiles;  // ceil(n / kScanTile)
    uint32_t direct_count;  // 1: the count scan sums the counts below its tile itself
    uint32_t max_chunks;   // capacity of the chunk lists
    uint32_t rank_items;   // accesses per thread in the rank phase (2: narrow rows, 4: others)
    uint32_t deterministic; // 1: the accesses of a segment are also listed in ascending order (perm_sorted)
    // build scratch, owned by the plan (the structures of several later steps are under construction at a time)
    uint8_t *bytemap;      // [32 * words] one byte per key, all zero between builds
    uint8_t *wordmap;      // [words]     one byte per bitmap word: some key of the word is marked; zero between builds
    uint32_t *bitmap;      // [words]     one bit per key; only the words with a marked key are written by a build
    uint32_t *word_rank;   // [words]     distinct keys below the word inside its tile (written for the same words)
    uint32_t *tile_sum;    // [max(bitmap_tiles, count_tiles)]
    uint32_t *tile_prefix; // [bitmap_tiles] distinct keys below each tile (tables with more than kLdsTiles tiles only)
    uint32_t *cnt_work;    // [n]         per distinct key: positions handed out so far, zero between builds
    // result, owned by the plan
    uint32_t *uniq;        // [n]         distinct keys, ascending
    uint32_t *count;       // [n]         accesses per distinct key
    uint32_t *seg;         // [n + 1]     exclusive prefix sums of count
    uint32_t *perm;        // [n]         accesses grouped by key (inside a segment: in the order positions were handed out)
    uint32_t *perm_sorted; // [n]         the same with every segment in ascending order (deterministic mode only)
    uint32_t *perm_pieces; // [n]         on the way there: ascending inside every piece of a segment (a piece: the part of
                           //             the segment inside one block of kBlock consecutive positions)
    uint32_t *slot;        // [n]         per access: index of its key among the distinct keys
    uint32_t *pos;         // [n]         per access: where it stands in perm (perm_sorted in deterministic mode)
    uint32_t *rank;        // [n]         per access: position inside its key's segment (| kSingleAccess)
    uint4 *chunk_of;       // [max_chunks]  per chunk of a long segment: {distinct-key index of the segment, number of the
                           //               segment's first chunk, first position of the segment, position after its last}
    uint32_t *chunk_done;  // [max_chunks]  arrival counter per long segment (at its first chunk), zero between steps
    uint32_t *meta;        // [kMetaWords]
    uint32_t *error_flag;  // shared by the context: bit 0 = key out of range
    double *zero_loss;     // if not null: loss accumulator (kLossSlots slots) that the build resets
    const uint32_t *hot_bits; // explicit hot-key set of the table (one bit per key), or null: decide by segment length
};

struct Plan {
    PlanArgs a{};
    size_t cap_n = 0;      // capacity (accesses) of the result arrays and of cnt_work
    size_t cap_words = 0;  // capacity (bitmap words) of the maps
    size_t cap_tiles = 0;  // capacity of the tile arrays
    int table = -1;
};

struct Table {
    float *data = nullptr;
    float *state = nullptr;
    int64_t num_keys = 0;
    int32_t dim = 0;
    int32_t stride = 0;
    std::vector<uint32_t> hot_keys;   // hottest first (as declared by the caller)
    uint32_t *hot_bits_dev = nullptr; // [ceil(V/32)] membership bitmap of the declared set; null = none declared
    // stale replicas of the hot keys (nups_set_replicas); all null / 0 while they are off
    uint32_t *hot_slot_dev = nullptr; // [V] number of the key in hot_keys, kBadIndex if it is not hot
    uint32_t *hot_list_dev = nullptr; // [hot keys] the hot keys
    float *replica_rows = nullptr;    // [replicas x hot keys][stride]
    Plan *last_plan = nullptr;        // structure of the last step / push on this table (owned by a prepared step)
};

// Everything the drawing of one batch of samples needs (device-side view, filled in when the call is made: the
// distribution object may change afterwards: cursor, batch-local key arrays).
struct SampleArgs {
    int32_t scheme;                   // nups_scheme; 0: nothing to draw
    const uint32_t *thresh, *alias;   // null thresh: uniform
    uint64_t num_keys, seed, step, cursor, P;
    uint32_t dist_id, n, U, G, F, R;
    int32_t half;                     // LONG-TERM: bits per half of the Feistel domain
    const uint32_t *local_a, *local_b;
    uint32_t local_n, per_example, split, tile;
    uint32_t per_sample;              // samples per example of the step that draws them (marking only; 0 is read as 1)
    uint32_t *out;                    // [n] sample keys
    uint32_t blocks;                  // workgroups that the drawing needs
    uint8_t *bytemap, *wordmap;       // maps of the step's structure to mark the keys in, or null
    uint32_t mark_keys;               // size of that structure's (extended) key space
    ReplicaMap rep;                   // the replicas of that structure's table, to mark a drawn hot key's replica
    uint32_t *error_flag;
};

// Phases of a step's preparatory work, in order (side_work.h).
enum SidePhase : int32_t {
    kSideDraw = 0, kSideTiles, kSidePrefix, kSideSlot, kSideRank, kSideCountTiles, kSideCounts, kSideScatter, kSideSort, kSideMerge
};

// One phase of one step: units block0 .. block0 + blocks - 1 of it.
struct SideItem {
    int32_t phase;
    int32_t n_plans;
    uint32_t block0, blocks;          // units of work, each sized for one workgroup
    uint32_t wgs;                     // workgroups that share them (unit w, w + wgs, ... to workgroup w); set per launch
    uint32_t blocks_per_plan;         // units per plan (after the drawing's own, in kSideDraw)
    PlanArgs plan[2];
    SampleArgs draw;                  // kSideDraw only
};

// What a launch carries in its first `blocks` workgroups.
struct SideWork {
    int32_t n;
    uint32_t blocks;                  // sum of the items' wgs, rounded up to a multiple of the die count
    SideItem item[kMaxSide];
};

struct Phase {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;
    std::vector<hipEvent_t> free_events;
    double ms = 0.0;
    int64_t launches = 0;
};

}  // namespace nups

// A step that has been handed to the library: its preparatory work is a list of phases, carried one per launch by
// the gradient and update kernels of the steps that run before it (or launched on their own when it runs sooner).
struct nups_prepared {
    nups_ctx *ctx = nullptr;
    nups_batch batch{};
    nups::Plan plan[2];
    int n_plans = 0;
    std::vector<nups::SideItem> phases;
    size_t next_phase = 0;         // phases before this one have been enqueued
    int lead_launches = 0;         // launches that pass before the first phase rides in one (see nups_prepare_step)
    double *loss_dev = nullptr;    // this step's loss accumulator: kLossSlots partial sums, kLossStride doubles apart
    uint32_t *negs_buf = nullptr;  // negatives drawn by the step itself (batch.dist)
    size_t negs_cap = 0;
    bool live = false;             // prepared, not yet run
    bool retired = false;          // run, still referenced by a table's structure query
};

struct nups_ctx {
    int n_tables = 0;
    nups::Table tab[nups::kMaxTables];
    hipStream_t stream = nullptr;   // the caller's stream: all device work is enqueued here
    int device = 0;
    std::deque<nups_prepared *> pending;   // prepared steps with phases left, oldest first
    // step workspace
    float *coef = nullptr;      size_t coef_cap = 0;      // per (example, scored row) loss derivative
    float *stage = nullptr;     size_t stage_cap = 0;     // staged gradient rows
    float *partial = nullptr;   size_t partial_cap = 0;   // partial sums of the chunks of long segments
    float *totals = nullptr;    size_t totals_cap = 0;    // running totals of long segments summed by single row groups
    double *loss_cur = nullptr;                            // loss accumulator of the step being run
    bool want_loss = true;                                 // the caller of the step being run asked for its loss
    uint32_t *error_flag = nullptr;                        // device word
    double *loss_pinned = nullptr;                         // pinned host copies for read-back
    uint32_t *flag_pinned = nullptr;
    // norm clipping of hot-key updates (Section 5.1); factor 0: off
    float clip_factor = 0.0f;
    double *clip_stats = nullptr;   // [kMaxTables][kLossSlots * kLossStride]: per slot {sum of norms, number of norms}
    float *clip_bound = nullptr;    // [kMaxTables] factor x mean norm, refreshed before each update launch
    int replicas = 0;               // parts of the minibatch with replicas of their own of the hot keys; 0: off
    bool deterministic = false;     // structures built from now on list every segment's accesses in ascending order
    bool profiling = false;
    nups::Phase phase[NUPS_PHASE_COUNT];
    std::vector<nups_dist *> dists;
    std::vector<nups_prepared *> prepared_all;   // every prepared-step object ever created (owned)
    std::vector<nups_prepared *> prepared_free;  // run and no longer referenced by a structure query
    nups_prepared *static_push = nullptr;        // the structure of nups_push_static: its arrays are the static scratch
};

struct nups_dist {
    nups_ctx *ctx = nullptr;
    int table = 0;
    uint32_t id = 0;
    nups_scheme scheme = NUPS_CONFORM;
    bool uniform = true;
    uint32_t *thresh_dev = nullptr;
    uint32_t *alias_dev = nullptr;
    int32_t U = 1, G = 1, R = 1;
    int64_t P = 1;
    uint64_t seed = 0;
    uint64_t cursor = 0;           // LONG-TERM: samples handed to earlier handles
    // LONG-TERM with postponing (Section 4.4): samples of keys that are not resident move to the end of their handle
    bool postpone = false;
    uint32_t *first_pos_dev = nullptr;      // [num_keys] first position of a key in the handle being built, else ~0
    uint32_t *tile_counts_dev = nullptr;   size_t tile_cap = 0;
    // NON-CONFORM
    const uint32_t *local_a = nullptr, *local_b = nullptr;
    int64_t local_n = 0;
    int32_t per_example = 0, split = 0, tile = 0;
    std::vector<nups_sample *> live;       // handles not yet released
    std::vector<nups_sample *> recycled;   // released handles whose buffers are reused
};

struct nups_sample {
    nups_dist *dist = nullptr;
    uint32_t *keys_dev = nullptr;   size_t cap = 0;
    uint32_t *raw_dev = nullptr;    size_t raw_cap = 0;   // the pool's sequence before postponing
    int64_t n = 0;
    int64_t pulled = 0;
    bool live = false;
};

namespace nups {

// RAII bracket that records HIP events around the launches of one phase when profiling is on.
struct PhaseScope {
    nups_ctx *ctx;
    int phase;
    hipStream_t stream;
    hipEvent_t start = nullptr;
    PhaseScope(nups_ctx *c, int p, hipStream_t s);
    ~PhaseScope();
};

// host-side helpers and launchers (defined in the .hip files)
SampleArgs sample_args(const nups_dist *d, uint32_t *keys_out, int64_t n_samples, uint64_t step);
nups_status launch_postpone(nups_dist *d, const uint32_t *raw, uint32_t *out, int64_t n_samples);
nups_status ensure_plan_capacity(nups_ctx *ctx, Table &t, Plan &pl, size_t n);
void set_plan_shape(const nups_ctx *ctx, const Table &t, Plan &pl);
int64_t extended_keys(const nups_ctx *ctx, const Table &t);
nups_status static_scratch_setup(int device);   // once per device, with that device current
void build_phases(nups_prepared &p, const SampleArgs &draw, int mark_plan);
size_t side_lds_bytes(const SideItem &it);
SideWork take_side_work(nups_ctx *ctx, size_t *lds_bytes, uint32_t max_wgs_per_phase);
nups_status flush_side_work(nups_ctx *ctx, nups_prepared *p);
nups_status launch_side(nups_ctx *ctx, const SideItem &it);
void free_plan_arrays(Plan &pl);
nups_status launch_replicas(nups_ctx *ctx, Table &t, bool sync);   // false: replicas <- rows; true: synchronise
nups_status launch_pull(nups_ctx *ctx, const Table &t, const uint32_t *keys, int64_t n, float *values);
nups_status launch_push_apply(nups_ctx *ctx, Table &t, const Plan &pl, float *partial, float *totals,
                              uint32_t grid_cap, const float *updates);
nups_status plan_step_sgns(nups_ctx *ctx, nups_prepared &p);   // capacity + plan arguments
nups_status plan_step_mf(nups_ctx *ctx, nups_prepared &p);
nups_status plan_step_kge(nups_ctx *ctx, nups_prepared &p);
nups_status run_step_sgns(nups_ctx *ctx, nups_prepared &p);
nups_status run_step_mf(nups_ctx *ctx, nups_prepared &p);
nups_status run_step_kge(nups_ctx *ctx, nups_prepared &p);
nups_status ensure_f32(float **buf, size_t *cap, size_t need, hipStream_t stream);
size_t max_chunks(size_t n);
nups_status ensure_partial(nups_ctx *ctx, size_t need);
nups_status ensure_totals(nups_ctx *ctx, int stride);   // room for an update launch of rows of `stride` floats

}  // namespace nups
