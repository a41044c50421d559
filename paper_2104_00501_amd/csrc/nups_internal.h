// Internal declarations shared by the translation units of libnups (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/nups.h"

namespace nups {

constexpr int kGroup = 16;            // lanes that cooperate on one row (one DPP row of a wavefront)
constexpr int kBlock = 256;           // threads per workgroup (4 wavefronts, 16 row groups)
constexpr int kGroupsPerBlock = kBlock / kGroup;
constexpr int kMaxTables = 4;
constexpr int kMaxStride = 1024;
constexpr int kScanItems = 8;         // items per thread in the tile scans
constexpr int kScanTile = kBlock * kScanItems;
constexpr uint32_t kLongSegment = 48; // segments with more accesses are summed by a whole workgroup
constexpr uint32_t kBadIndex = 0xFFFFFFFFu;

// meta words of a plan (device)
enum { kMetaNumUniq = 0, kMetaNumLong = 1, kMetaTotal = 2, kMetaWords = 4 };

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
};

// Device-side description of the per-key aggregation structure of one table for one step:
// distinct keys in ascending order, the number of accesses of each, and the accesses grouped by key.
struct PlanArgs {
    KeySource src;
    uint32_t n;            // accesses (sum of src.len)
    uint32_t num_keys;     // V
    uint32_t words;        // bitmap words = ceil(V / 32)
    uint32_t bitmap_tiles; // ceil(words / kScanTile)
    uint32_t count_tiles;  // ceil(n / kScanTile)
    uint32_t *bitmap;      // [words]     one bit per key, all zero between steps
    uint32_t *word_rank;   // [words]     number of distinct keys below each bitmap word
    uint32_t *tile_sum;    // [max(bitmap_tiles, count_tiles)]
    uint32_t *uniq;        // [n]         distinct keys, ascending
    uint32_t *count;       // [n]         accesses per distinct key
    uint32_t *seg;         // [n + 1]     exclusive prefix sums of count
    uint32_t *slot;        // [n]         per access: index of its key among the distinct keys
    uint32_t *rank;        // [n]         per access: position inside its key's segment
    uint32_t *perm;        // [n]         accesses grouped by key
    uint32_t *long_list;   // [n / kLongSegment + 1] distinct-key indices of long segments
    uint32_t *meta;        // [kMetaWords]
    uint32_t *error_flag;  // shared by the context: bit 0 = key out of range
};

struct Plan {
    PlanArgs a{};
    size_t cap_n = 0;      // capacity (accesses) of the per-access arrays
    size_t cap_words = 0;
    size_t cap_tiles = 0;
    bool valid = false;    // arrays describe the last build
};

struct Table {
    float *data = nullptr;
    float *state = nullptr;
    int64_t num_keys = 0;
    int32_t dim = 0;
    int32_t stride = 0;
    std::vector<uint32_t> hot_keys;   // hottest first
    uint32_t *hot_slot_dev = nullptr; // [num_keys] slot of a hot key, kBadIndex otherwise (built on demand)
    Plan plan;
};

struct Phase {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;
    std::vector<hipEvent_t> free_events;
    double ms = 0.0;
    int64_t launches = 0;
};

}  // namespace nups

struct nups_ctx {
    int n_tables = 0;
    nups::Table tab[nups::kMaxTables];
    hipStream_t stream = nullptr;
    int device = 0;
    // step workspace
    float *coef = nullptr;      size_t coef_cap = 0;      // per (example, scored row) loss derivative
    float *stage = nullptr;     size_t stage_cap = 0;     // staged gradient rows
    double *loss_dev = nullptr;                            // batch loss accumulator
    uint32_t *error_flag = nullptr;                        // device word
    double *loss_pinned = nullptr;                         // pinned host copies for read-back
    uint32_t *flag_pinned = nullptr;
    bool profiling = false;
    nups::Phase phase[NUPS_PHASE_COUNT];
    std::vector<nups_dist *> dists;
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
    uint32_t *fresh_dev = nullptr;  size_t fresh_cap = 0;   // BOUNDED: the fresh draws of the handle
    int64_t n = 0;
    int64_t pulled = 0;
    bool live = false;
};

namespace nups {

// RAII bracket that records HIP events around the launches of one phase when profiling is on.
struct PhaseScope {
    nups_ctx *ctx;
    int phase;
    hipEvent_t start = nullptr;
    PhaseScope(nups_ctx *c, int p);
    ~PhaseScope();
};

// kernels' host-side launchers (defined in the .hip files)
nups_status launch_sample(nups_dist *d, nups_sample *h, uint64_t step);
nups_status build_plans(nups_ctx *ctx, Plan **plans, int n_plans);
nups_status ensure_plan_capacity(nups_ctx *ctx, Table &t, size_t n);
nups_status launch_pull(nups_ctx *ctx, const Table &t, const uint32_t *keys, int64_t n, float *values);
nups_status launch_push_apply(nups_ctx *ctx, Table &t, const float *updates);
nups_status launch_step_sgns(nups_ctx *ctx, const nups_batch &b);
nups_status launch_step_mf(nups_ctx *ctx, const nups_batch &b);
nups_status launch_step_kge(nups_ctx *ctx, const nups_batch &b);
nups_status ensure_f32(float **buf, size_t *cap, size_t need, hipStream_t stream);

}  // namespace nups
