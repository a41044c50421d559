// Host side of the C ABI declared in include/nups.h: argument checks, workspace, object lifetimes, and the
// schedule of preparatory work (Section 4.3: sampling and what else a step needs before it can run).  All device
// work goes to the caller's stream.  The preparatory work of a prepared step is a list of phases; each launch of
// a gradient or update kernel carries one phase of each of the next few prepared steps in spare workgroups, so a
// step that was prepared three steps ahead finds its samples drawn and its structure built when it runs, and
// nothing but the steps' own two launches is ever enqueued.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "nups_internal.h"

namespace nups {

static thread_local std::string g_error;

void set_error(const std::string &msg) { g_error = msg; }

nups_status fail(nups_status st, const std::string &msg)
{
    g_error = msg;
    return st;
}

bool hip_ok(hipError_t e, const char *what)
{
    if (e == hipSuccess) return true;
    g_error = std::string(what) + ": " + hipGetErrorString(e);
    return false;
}

nups_status ensure_f32(float **buf, size_t *cap, size_t need, hipStream_t stream)
{
    if (*cap >= need && *buf) return NUPS_OK;
    NUPS_HIP(hipStreamSynchronize(stream));
    if (*buf) NUPS_HIP(hipFree(*buf));
    *buf = nullptr;
    const size_t n = need + need / 4 + 1024;
    NUPS_HIP(hipMalloc((void **)buf, sizeof(float) * n));
    *cap = n;
    return NUPS_OK;
}

PhaseScope::PhaseScope(nups_ctx *c, int p, hipStream_t s) : ctx(c), phase(p), stream(s)
{
    if (!ctx->profiling) return;
    Phase &ph = ctx->phase[phase];
    if (!ph.free_events.empty()) { start = ph.free_events.back(); ph.free_events.pop_back(); }
    else if (hipEventCreate(&start) != hipSuccess) start = nullptr;
    if (start) (void)hipEventRecord(start, stream);
}

PhaseScope::~PhaseScope()
{
    if (!start) return;
    Phase &ph = ctx->phase[phase];
    hipEvent_t stop = nullptr;
    if (!ph.free_events.empty()) { stop = ph.free_events.back(); ph.free_events.pop_back(); }
    else if (hipEventCreate(&stop) != hipSuccess) stop = nullptr;
    if (!stop) { ph.free_events.push_back(start); return; }
    (void)hipEventRecord(stop, stream);
    ph.pending.emplace_back(start, stop);
}

static void free_sample(nups_sample *h)
{
    if (h->keys_dev) (void)hipFree(h->keys_dev);
    if (h->raw_dev) (void)hipFree(h->raw_dev);
    delete h;
}

static void free_dist(nups_dist *d)
{
    for (nups_sample *h : d->live) free_sample(h);
    for (nups_sample *h : d->recycled) free_sample(h);
    if (d->thresh_dev) (void)hipFree(d->thresh_dev);
    if (d->alias_dev) (void)hipFree(d->alias_dev);
    if (d->first_pos_dev) (void)hipFree(d->first_pos_dev);
    if (d->tile_counts_dev) (void)hipFree(d->tile_counts_dev);
    delete d;
}

static void free_prepared(nups_prepared *p)
{
    free_plan_arrays(p->plan[0]);
    free_plan_arrays(p->plan[1]);
    if (p->loss_dev) (void)hipFree(p->loss_dev);
    if (p->negs_buf) (void)hipFree(p->negs_buf);
    delete p;
}

// After a bad key (or a key array changed behind a prepared step) the scratch maps of a structure may hold marks
// of accesses that were dropped, which the phases do not find again to clear.  Returns the maps and counters of
// every structure that is not under construction to all-zero, the state that the next build starts from.
static nups_status reset_idle_plans(nups_ctx *ctx)
{
    for (nups_prepared *q : ctx->prepared_all) {
        if (q->live) continue;   // under construction or waiting to run: its marks are in use
        for (Plan &pl : q->plan) {
            PlanArgs &a = pl.a;
            if (pl.cap_words) {
                NUPS_HIP(hipMemsetAsync(a.bytemap, 0, pl.cap_words * 32, ctx->stream));
                NUPS_HIP(hipMemsetAsync(a.wordmap, 0, pl.cap_words, ctx->stream));
            }
            if (pl.cap_n) {
                NUPS_HIP(hipMemsetAsync(a.cnt_work, 0, sizeof(uint32_t) * ((pl.cap_n + kScanTile - 1) / kScanTile * kScanTile), ctx->stream));
                NUPS_HIP(hipMemsetAsync(a.chunk_done, 0, sizeof(uint32_t) * max_chunks(pl.cap_n), ctx->stream));
            }
        }
    }
    return NUPS_OK;
}

// Waits for the stream and turns a raised device flag into an error.
static nups_status sync_and_check(nups_ctx *ctx)
{
    NUPS_HIP(hipMemcpyAsync(ctx->flag_pinned, ctx->error_flag, sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    if (*ctx->flag_pinned != 0) {
        NUPS_HIP(hipMemsetAsync(ctx->error_flag, 0, sizeof(uint32_t), ctx->stream));
        nups_status st = reset_idle_plans(ctx);
        if (st != NUPS_OK) return st;
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        return fail(NUPS_ERR_KEY_RANGE, "a key was outside its table (it was skipped)");
    }
    return NUPS_OK;
}

static void free_replicas(Table &t)
{
    if (t.hot_slot_dev) (void)hipFree(t.hot_slot_dev);
    if (t.hot_list_dev) (void)hipFree(t.hot_list_dev);
    if (t.replica_rows) (void)hipFree(t.replica_rows);
    t.hot_slot_dev = t.hot_list_dev = nullptr;
    t.replica_rows = nullptr;
}

static bool valid_table(const nups_ctx *ctx, int t) { return ctx && t >= 0 && t < ctx->n_tables; }

static nups_status get_prepared(nups_ctx *ctx, nups_prepared **out)
{
    nups_prepared *p = nullptr;
    if (!ctx->prepared_free.empty()) { p = ctx->prepared_free.back(); ctx->prepared_free.pop_back(); }
    else {
        p = new nups_prepared();
        p->ctx = ctx;
        ctx->prepared_all.push_back(p);
    }
    nups_status st = NUPS_OK;
    p->phases.clear();
    p->next_phase = 0;
    p->lead_launches = 0;
    if (!p->loss_dev && !hip_ok(hipMalloc((void **)&p->loss_dev, sizeof(double) * kLossSlots * kLossStride), "loss accumulator"))
        st = NUPS_ERR_DEVICE;
    if (st != NUPS_OK) { ctx->prepared_free.push_back(p); return st; }
    *out = p;
    return NUPS_OK;
}

// A consumed step is recycled once no table's structure query refers to it any more.  Its arrays may still be
// read by kernels in flight; whatever reuses them is enqueued behind those on the same stream.
static void retire_prepared(nups_ctx *ctx, nups_prepared *p)
{
    p->live = false;
    p->retired = true;
    for (int j = 0; j < p->n_plans; ++j) ctx->tab[p->plan[j].table].last_plan = &p->plan[j];
    for (nups_prepared *q : ctx->prepared_all) {
        if (!q->retired) continue;
        bool referenced = false;
        for (int t = 0; t < kMaxTables; ++t)
            for (int k = 0; k < 2; ++k) referenced |= (ctx->tab[t].last_plan == &q->plan[k]);
        if (!referenced) { q->retired = false; ctx->prepared_free.push_back(q); }
    }
}

static nups_status check_batch(nups_ctx *ctx, const nups_batch *b)
{
    if (!ctx || !b) return fail(NUPS_ERR_ARG, "nups_step: null argument");
    if (ctx->n_tables < 2) return fail(NUPS_ERR_STATE, "nups_step: the context needs two tables");
    if (b->B < 0 || b->B > (1ll << 24)) return fail(NUPS_ERR_ARG, "nups_step: batch size out of range");
    if (b->n_neg < 0 || b->n_neg2 < 0 || b->n_neg > 4096 || b->n_neg2 > 4096)
        return fail(NUPS_ERR_ARG, "nups_step: negative counts out of range");
    if (b->B > 0 && (!b->k0 || !b->k1)) return fail(NUPS_ERR_ARG, "nups_step: null key array");
    const int64_t nn = (int64_t)b->n_neg + b->n_neg2;
    if (b->B * (nn + 2) > 0x7FFFFFFFll) return fail(NUPS_ERR_ARG, "nups_step: too many accesses for one step");
    if (ctx->tab[0].stride != ctx->tab[1].stride)
        return fail(NUPS_ERR_ARG, "nups_step: tables 0 and 1 need equal row_stride");
    if ((b->sample != nullptr) + (b->negs != nullptr) + (b->dist != nullptr) > 1)
        return fail(NUPS_ERR_ARG, "nups_step: give only one of negs, sample and dist");
    if (b->dist) {
        if (b->dist->ctx != ctx) return fail(NUPS_ERR_ARG, "nups_step: the distribution is of another context");
        // the drawn keys index the table that the task's negatives live in (Section 2.2: output vectors; entities)
        if (b->task == NUPS_TASK_SGNS && b->dist->table != 1)
            return fail(NUPS_ERR_ARG, "nups_step: SGNS negatives index table 1: register the distribution there");
        if (b->task == NUPS_TASK_KGE && b->dist->table != 0)
            return fail(NUPS_ERR_ARG, "nups_step: KGE negatives index table 0: register the distribution there");
        if (b->dist->postpone)
            return fail(NUPS_ERR_UNIMPLEMENTED, "nups_step: a distribution with postponing is drawn from through "
                                                "nups_prepare_sample; pass the handle as batch.sample");
        if (b->dist->scheme == NUPS_NONCONFORM && !b->dist->local_a)
            return fail(NUPS_ERR_STATE, "nups_step: call nups_set_local_keys first");
        if (b->dist->scheme == NUPS_NONCONFORM && b->B * nn > b->dist->local_n * (int64_t)b->dist->per_example)
            return fail(NUPS_ERR_ARG, "nups_step: more samples than examples * per_example");
        if (b->sample_step >> 48) return fail(NUPS_ERR_ARG, "nups_step: sample_step must be below 2^48");
    }
    if (b->sample) {
        if (!b->sample->live) return fail(NUPS_ERR_STATE, "nups_step: the sample handle was released");
        if (b->sample->dist->ctx != ctx) return fail(NUPS_ERR_ARG, "nups_step: the sample handle is of another context");
        if (b->sample->n < b->B * nn) return fail(NUPS_ERR_ARG, "nups_step: the sample handle holds too few keys");
    }
    switch (b->task) {
    case NUPS_TASK_SGNS:
        if (b->n_neg2 != 0) return fail(NUPS_ERR_ARG, "nups_step: SGNS uses n_neg only");
        if (b->B > 0 && b->n_neg > 0 && !b->negs && !b->sample && !b->dist) return fail(NUPS_ERR_ARG, "nups_step: null negatives");
        break;
    case NUPS_TASK_MF:
        if (b->B > 0 && !b->val) return fail(NUPS_ERR_ARG, "nups_step: null cell values");
        if (nn != 0) return fail(NUPS_ERR_ARG, "nups_step: MF has no sampling access");
        break;
    case NUPS_TASK_KGE:
        if (b->B > 0 && !b->k2) return fail(NUPS_ERR_ARG, "nups_step: null object keys");
        if (b->B > 0 && nn > 0 && !b->negs && !b->sample && !b->dist) return fail(NUPS_ERR_ARG, "nups_step: null negatives");
        if (!ctx->tab[0].state || !ctx->tab[1].state)
            return fail(NUPS_ERR_STATE, "nups_step: KGE needs AdaGrad state on tables 0 and 1 (nups_set_state)");
        break;
    default:
        return fail(NUPS_ERR_ARG, "nups_step: unknown task");
    }
    return NUPS_OK;
}

}  // namespace nups

using namespace nups;

extern "C" {

const char *nups_last_error(void) { return g_error.c_str(); }

const char *nups_phase_name(int phase)
{
    static const char *names[NUPS_PHASE_COUNT] = {"sample", "plan", "grad", "apply0", "apply1", "pull", "push"};
    return (phase >= 0 && phase < NUPS_PHASE_COUNT) ? names[phase] : "";
}

nups_status nups_init(nups_ctx **out, int n_tables, float *const *tables_dev, const int64_t *num_keys,
                      const int32_t *dim, const int32_t *row_stride, void *hip_stream)
{
    if (!out) return fail(NUPS_ERR_ARG, "nups_init: out is null");
    *out = nullptr;
    if (!tables_dev || !num_keys || !dim || !row_stride) return fail(NUPS_ERR_ARG, "nups_init: null array");
    if (n_tables < 1 || n_tables > kMaxTables) return fail(NUPS_ERR_ARG, "nups_init: n_tables must be 1..4");
    for (int t = 0; t < n_tables; ++t) {
        if (!tables_dev[t]) return fail(NUPS_ERR_ARG, "nups_init: null table");
        if (num_keys[t] < 1 || num_keys[t] > 0xFFFFFFFFll) return fail(NUPS_ERR_ARG, "nups_init: num_keys out of range");
        if (dim[t] < 1 || dim[t] > row_stride[t]) return fail(NUPS_ERR_ARG, "nups_init: need 1 <= dim <= row_stride");
        const int w = row_stride[t] / 64;   // float4 per lane of a row group: the widths that kernels are built for
        if (row_stride[t] % 64 != 0 || !(w == 1 || w == 2 || w == 3 || w == 4 || w == 5 || w == 6 || w == 8 || w == 16))
            return fail(NUPS_ERR_ARG, "nups_init: row_stride must be 64, 128, 192, 256, 320, 384, 512 or 1024 floats");
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(NUPS_ERR_DEVICE, "nups_init: no HIP device");
    nups_ctx *ctx = new nups_ctx();
    NUPS_HIP(hipGetDevice(&ctx->device));
    ctx->n_tables = n_tables;
    ctx->stream = (hipStream_t)hip_stream;
    for (int t = 0; t < n_tables; ++t) {
        ctx->tab[t].data = tables_dev[t];
        ctx->tab[t].num_keys = num_keys[t];
        ctx->tab[t].dim = dim[t];
        ctx->tab[t].stride = row_stride[t];
    }
    hipError_t e = hipMalloc((void **)&ctx->error_flag, sizeof(uint32_t));
    if (e == hipSuccess) e = hipHostMalloc((void **)&ctx->loss_pinned, sizeof(double) * kLossSlots * kLossStride, hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void **)&ctx->flag_pinned, sizeof(uint32_t), hipHostMallocDefault);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->error_flag, 0, sizeof(uint32_t), ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) {
        hip_ok(e, "nups_init: workspace allocation");
        nups_destroy(ctx);
        return NUPS_ERR_DEVICE;
    }
    if (static_scratch_setup(ctx->device) != NUPS_OK) {   // the address of this device's copy of the static scratch
        nups_destroy(ctx);
        return NUPS_ERR_DEVICE;
    }
    *out = ctx;
    return NUPS_OK;
}

nups_status nups_destroy(nups_ctx *ctx)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_destroy: null context");
    (void)hipStreamSynchronize(ctx->stream);
    for (nups_dist *d : ctx->dists) free_dist(d);
    for (nups_prepared *p : ctx->prepared_all) free_prepared(p);
    delete ctx->static_push;   // its arrays are not its own
    for (int t = 0; t < kMaxTables; ++t) {
        if (ctx->tab[t].hot_bits_dev) (void)hipFree(ctx->tab[t].hot_bits_dev);
        free_replicas(ctx->tab[t]);
    }
    if (ctx->clip_stats) (void)hipFree(ctx->clip_stats);
    if (ctx->clip_bound) (void)hipFree(ctx->clip_bound);
    if (ctx->coef) (void)hipFree(ctx->coef);
    if (ctx->stage) (void)hipFree(ctx->stage);
    if (ctx->partial) (void)hipFree(ctx->partial);
    if (ctx->totals) (void)hipFree(ctx->totals);
    if (ctx->error_flag) (void)hipFree(ctx->error_flag);
    if (ctx->loss_pinned) (void)hipHostFree(ctx->loss_pinned);
    if (ctx->flag_pinned) (void)hipHostFree(ctx->flag_pinned);
    for (Phase &ph : ctx->phase) {
        for (auto &pr : ph.pending) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
        for (hipEvent_t ev : ph.free_events) (void)hipEventDestroy(ev);
    }
    delete ctx;
    return NUPS_OK;
}

nups_status nups_set_state(nups_ctx *ctx, int table, float *state_dev)
{
    if (!valid_table(ctx, table)) return fail(NUPS_ERR_ARG, "nups_set_state: bad context or table");
    if (!state_dev) return fail(NUPS_ERR_ARG, "nups_set_state: null state");
    ctx->tab[table].state = state_dev;
    return NUPS_OK;
}

nups_status nups_set_hot_keys(nups_ctx *ctx, int table, const uint32_t *keys_host, int64_t k)
{
    if (!valid_table(ctx, table)) return fail(NUPS_ERR_ARG, "nups_set_hot_keys: bad context or table");
    if (k < 0 || (k > 0 && !keys_host)) return fail(NUPS_ERR_ARG, "nups_set_hot_keys: bad key list");
    Table &t = ctx->tab[table];
    if (ctx->replicas > 0) return fail(NUPS_ERR_STATE, "nups_set_hot_keys: switch the replicas off first (nups_set_replicas)");
    std::vector<uint32_t> keys(keys_host, keys_host + k);
    std::vector<uint32_t> sorted(keys);
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end())
        return fail(NUPS_ERR_ARG, "nups_set_hot_keys: keys must be distinct");
    if (k > 0 && (int64_t)sorted.back() >= t.num_keys) return fail(NUPS_ERR_KEY_RANGE, "nups_set_hot_keys: key out of range");
    // membership bitmap on the device; plans built from now on consult it
    const size_t words = (size_t)((t.num_keys + 31) / 32);
    std::vector<uint32_t> bits(words, 0u);
    for (uint32_t key : keys) bits[key >> 5] |= 1u << (key & 31);
    for (nups_prepared *q : ctx->prepared_all)
        if (q->live) return fail(NUPS_ERR_STATE, "nups_set_hot_keys: prepared steps are outstanding");
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    if (!t.hot_bits_dev) NUPS_HIP(hipMalloc((void **)&t.hot_bits_dev, sizeof(uint32_t) * words));
    NUPS_HIP(hipMemcpy(t.hot_bits_dev, bits.data(), sizeof(uint32_t) * words, hipMemcpyHostToDevice));
    t.hot_keys.swap(keys);
    return NUPS_OK;
}

nups_status nups_set_replicas(nups_ctx *ctx, int32_t replicas)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_set_replicas: null context");
    if (replicas < 0 || replicas > 64) return fail(NUPS_ERR_ARG, "nups_set_replicas: 0 (off) to 64 replicas");
    if (ctx->n_tables < 2) return fail(NUPS_ERR_STATE, "nups_set_replicas: the context needs two tables");
    for (nups_prepared *q : ctx->prepared_all)
        if (q->live) return fail(NUPS_ERR_STATE, "nups_set_replicas: prepared steps are outstanding");
    if (replicas > 0 && ctx->clip_factor > 0.0f)
        return fail(NUPS_ERR_STATE, "nups_set_replicas: not together with update clipping");
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    if (ctx->replicas > 0) {             // what the replicas have accumulated goes into the tables first
        for (int k = 0; k < 2; ++k) {
            nups_status st = launch_replicas(ctx, ctx->tab[k], true);
            if (st != NUPS_OK) return st;
        }
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
    }
    for (int k = 0; k < 2; ++k) free_replicas(ctx->tab[k]);
    ctx->replicas = 0;
    if (replicas == 0) return NUPS_OK;
    for (int k = 0; k < 2; ++k) {
        Table &t = ctx->tab[k];
        const size_t H = t.hot_keys.size();
        if (H == 0) continue;            // no declared hot keys: no replicas for this table
        if ((uint64_t)t.num_keys + (uint64_t)replicas * H > 0xFFFFFFF0ull)
            return fail(NUPS_ERR_ARG, "nups_set_replicas: too many replica rows for 32-bit keys");
        std::vector<uint32_t> slot((size_t)t.num_keys, kBadIndex);
        for (size_t i = 0; i < H; ++i) slot[t.hot_keys[i]] = (uint32_t)i;
        hipError_t e = hipMalloc((void **)&t.hot_slot_dev, sizeof(uint32_t) * slot.size());
        if (e == hipSuccess) e = hipMalloc((void **)&t.hot_list_dev, sizeof(uint32_t) * H);
        if (e == hipSuccess) e = hipMalloc((void **)&t.replica_rows, sizeof(float) * (size_t)replicas * H * t.stride);
        if (e == hipSuccess) e = hipMemcpy(t.hot_slot_dev, slot.data(), sizeof(uint32_t) * slot.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(t.hot_list_dev, t.hot_keys.data(), sizeof(uint32_t) * H, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            hip_ok(e, "nups_set_replicas: replica buffers");
            for (int j = 0; j < 2; ++j) free_replicas(ctx->tab[j]);
            return NUPS_ERR_DEVICE;
        }
    }
    ctx->replicas = replicas;
    for (int k = 0; k < 2; ++k) {
        nups_status st = launch_replicas(ctx, ctx->tab[k], false);
        if (st != NUPS_OK) return st;
    }
    return NUPS_OK;
}

nups_status nups_sync_replicas(nups_ctx *ctx)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_sync_replicas: null context");
    for (int k = 0; k < 2 && k < ctx->n_tables; ++k) {
        nups_status st = launch_replicas(ctx, ctx->tab[k], true);
        if (st != NUPS_OK) return st;
    }
    return NUPS_OK;
}

nups_status nups_replica_rows(nups_ctx *ctx, int table, float **rows_dev, int64_t *n_rows)
{
    if (!valid_table(ctx, table) || !rows_dev || !n_rows) return fail(NUPS_ERR_ARG, "nups_replica_rows: bad arguments");
    const Table &t = ctx->tab[table];
    *rows_dev = t.replica_rows;
    *n_rows = t.replica_rows ? (int64_t)ctx->replicas * (int64_t)t.hot_keys.size() : 0;
    return NUPS_OK;
}

nups_status nups_set_deterministic(nups_ctx *ctx, int enable)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_set_deterministic: null context");
    for (nups_prepared *q : ctx->prepared_all)
        if (q->live) return fail(NUPS_ERR_STATE, "nups_set_deterministic: prepared steps are outstanding");
    ctx->deterministic = enable != 0;
    return NUPS_OK;
}

nups_status nups_set_update_clipping(nups_ctx *ctx, float factor)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_set_update_clipping: null context");
    if (!(factor >= 0.0f) || !std::isfinite(factor))
        return fail(NUPS_ERR_ARG, "nups_set_update_clipping: factor must be finite and not negative");
    if (factor > 0.0f && ctx->replicas > 0)
        return fail(NUPS_ERR_STATE, "nups_set_update_clipping: not together with replicas");
    const size_t stats_bytes = sizeof(double) * kMaxTables * kLossSlots * kLossStride;
    if (factor > 0.0f && !(ctx->clip_factor > 0.0f)) {   // switched on: statistics start from nothing
        if (!ctx->clip_stats) {
            NUPS_HIP(hipMalloc((void **)&ctx->clip_stats, stats_bytes));
            NUPS_HIP(hipMalloc((void **)&ctx->clip_bound, sizeof(float) * kMaxTables));
        }
        NUPS_HIP(hipStreamSynchronize(ctx->stream));
        NUPS_HIP(hipMemset(ctx->clip_stats, 0, stats_bytes));
    }
    ctx->clip_factor = factor;
    return NUPS_OK;
}

nups_status nups_get_update_clipping(nups_ctx *ctx, int table, double *norm_sum, double *norm_count)
{
    if (!valid_table(ctx, table)) return fail(NUPS_ERR_ARG, "nups_get_update_clipping: bad context or table");
    if (!ctx->clip_stats) return fail(NUPS_ERR_STATE, "nups_get_update_clipping: clipping was never switched on");
    std::vector<double> slots((size_t)kLossSlots * kLossStride);
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    NUPS_HIP(hipMemcpy(slots.data(), ctx->clip_stats + (size_t)table * slots.size(), sizeof(double) * slots.size(),
                       hipMemcpyDeviceToHost));
    double sum = 0.0, count = 0.0;
    for (int s = 0; s < kLossSlots; ++s) {
        sum += slots[(size_t)s * kLossStride];
        count += slots[(size_t)s * kLossStride + 1];
    }
    if (norm_sum) *norm_sum = sum;
    if (norm_count) *norm_count = count;
    return NUPS_OK;
}

nups_status nups_pull(nups_ctx *ctx, int table, const uint32_t *keys_dev, int64_t n, float *values_dev)
{
    if (!valid_table(ctx, table)) return fail(NUPS_ERR_ARG, "nups_pull: bad context or table");
    if (n < 0 || (n > 0 && (!keys_dev || !values_dev))) return fail(NUPS_ERR_ARG, "nups_pull: bad arguments");
    return launch_pull(ctx, ctx->tab[table], keys_dev, n, values_dev);
}

nups_status nups_push(nups_ctx *ctx, int table, const uint32_t *keys_dev, int64_t n, const float *updates_dev)
{
    if (!valid_table(ctx, table)) return fail(NUPS_ERR_ARG, "nups_push: bad context or table");
    if (n < 0 || n > 0x7FFFFFFFll || (n > 0 && (!keys_dev || !updates_dev)))
        return fail(NUPS_ERR_ARG, "nups_push: bad arguments");
    Table &t = ctx->tab[table];
    if (t.replica_rows) return fail(NUPS_ERR_STATE, "nups_push: the table has replicas of its hot keys (nups_set_replicas)");
    nups_prepared *p = nullptr;
    nups_status st = get_prepared(ctx, &p);
    if (st != NUPS_OK) return st;
    p->n_plans = 1;
    p->plan[0].table = table;
    if ((st = ensure_plan_capacity(ctx, t, p->plan[0], (size_t)n)) == NUPS_OK)
        st = ensure_partial(ctx, max_chunks(p->plan[0].cap_n) * (size_t)t.stride);
    if (st == NUPS_OK) st = ensure_totals(ctx, t.stride);
    if (st != NUPS_OK) { ctx->prepared_free.push_back(p); return st; }   // nothing was enqueued: the object is free again
    p->plan[0].a.src = KeySource{{keys_dev, nullptr, nullptr}, {(uint32_t)n, 0, 0}};
    p->plan[0].a.n = p->plan[0].a.mark_n = (uint32_t)n;
    p->plan[0].a.zero_loss = nullptr;
    build_phases(*p, SampleArgs{}, -1);
    st = flush_side_work(ctx, p);
    if (st == NUPS_OK && n > 0) st = launch_push_apply(ctx, t, p->plan[0], ctx->partial, ctx->totals, 0xFFFFFFFFu, updates_dev);
    retire_prepared(ctx, p);
    return st;
}

nups_status nups_register_distribution(nups_ctx *ctx, int table, const double *weights_host, nups_scheme scheme,
                                       int32_t U, int32_t G, int64_t P, int32_t R, uint64_t seed, nups_dist **out)
{
    if (!out) return fail(NUPS_ERR_ARG, "nups_register_distribution: out is null");
    *out = nullptr;
    if (!valid_table(ctx, table)) return fail(NUPS_ERR_ARG, "nups_register_distribution: bad context or table");
    if (scheme < NUPS_CONFORM || scheme > NUPS_NONCONFORM)
        return fail(NUPS_ERR_ARG, "nups_register_distribution: unknown scheme");
    if (scheme == NUPS_BOUNDED && (U < 1 || G < 1 || G > 1024))
        return fail(NUPS_ERR_ARG, "nups_register_distribution: BOUNDED needs U >= 1 and 1 <= G <= 1024");
    if (scheme == NUPS_LONGTERM && (P < 1 || R < 1 || P > (1ll << 40)))
        return fail(NUPS_ERR_ARG, "nups_register_distribution: LONG-TERM needs P >= 1 and R >= 1");
    if (ctx->dists.size() >= 255) return fail(NUPS_ERR_STATE, "nups_register_distribution: too many distributions");
    const int64_t V = ctx->tab[table].num_keys;
    std::vector<uint32_t> thresh, alias;
    if (weights_host) {
        thresh.resize((size_t)V);
        alias.resize((size_t)V);
        nups_status st = nups_build_alias_table(weights_host, V, thresh.data(), alias.data());
        if (st != NUPS_OK) return st;
    }
    nups_dist *d = new nups_dist();
    d->ctx = ctx;
    d->table = table;
    d->id = (uint32_t)ctx->dists.size();
    d->scheme = scheme;
    d->uniform = (weights_host == nullptr);
    d->U = U; d->G = G; d->P = P; d->R = R;
    d->seed = seed;
    if (weights_host) {
        hipError_t e = hipMalloc((void **)&d->thresh_dev, sizeof(uint32_t) * (size_t)V);
        if (e == hipSuccess) e = hipMalloc((void **)&d->alias_dev, sizeof(uint32_t) * (size_t)V);
        if (e == hipSuccess) e = hipMemcpy(d->thresh_dev, thresh.data(), sizeof(uint32_t) * (size_t)V, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(d->alias_dev, alias.data(), sizeof(uint32_t) * (size_t)V, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            hip_ok(e, "nups_register_distribution: alias table upload");
            free_dist(d);
            return NUPS_ERR_DEVICE;
        }
    }
    ctx->dists.push_back(d);
    *out = d;
    return NUPS_OK;
}

nups_status nups_register_distribution_at_level(nups_ctx *ctx, int table, const double *weights_host,
                                                nups_scheme level, uint64_t seed, nups_dist **out)
{
    // the untuned configuration's parameters (Section 5.1): use frequency 16, pools of 250
    return nups_register_distribution(ctx, table, weights_host, level, 16, 250, 1000000, 16, seed, out);
}

nups_status nups_select_hot_keys(const double *frequency_host, int64_t num_keys, double factor,
                                 uint32_t *keys_out_host, int64_t capacity, int64_t *k_out)
{
    if (!frequency_host || !k_out || num_keys < 1 || num_keys > 0xFFFFFFFFll || capacity < 0
        || (capacity > 0 && !keys_out_host) || !(factor > 0.0) || !std::isfinite(factor))
        return fail(NUPS_ERR_ARG, "nups_select_hot_keys: bad arguments");
    double total = 0.0;
    for (int64_t k = 0; k < num_keys; ++k) {
        if (!(frequency_host[k] >= 0.0) || !std::isfinite(frequency_host[k]))
            return fail(NUPS_ERR_ARG, "nups_select_hot_keys: frequencies must be finite and not negative");
        total += frequency_host[k];
    }
    const double bar = factor * (total / (double)num_keys);
    std::vector<uint32_t> hot;
    for (int64_t k = 0; k < num_keys; ++k)
        if (frequency_host[k] > bar) hot.push_back((uint32_t)k);
    std::stable_sort(hot.begin(), hot.end(),
                     [&](uint32_t a, uint32_t b) { return frequency_host[a] > frequency_host[b]; });
    *k_out = (int64_t)hot.size();
    for (int64_t i = 0; i < std::min<int64_t>(capacity, (int64_t)hot.size()); ++i) keys_out_host[i] = hot[(size_t)i];
    return NUPS_OK;
}

nups_status nups_set_local_keys(nups_dist *dist, const uint32_t *keys_a_dev, const uint32_t *keys_b_dev,
                                int64_t n_examples, int32_t per_example, int32_t split, int32_t tile)
{
    if (!dist) return fail(NUPS_ERR_ARG, "nups_set_local_keys: null distribution");
    if (dist->scheme != NUPS_NONCONFORM) return fail(NUPS_ERR_STATE, "nups_set_local_keys: scheme is not NON-CONFORM");
    if (!keys_a_dev || !keys_b_dev || n_examples < 1 || n_examples > 0x7FFFFFFFll || per_example < 1 || split < 0
        || split > per_example || tile < 1)
        return fail(NUPS_ERR_ARG, "nups_set_local_keys: bad arguments");
    dist->local_a = keys_a_dev;
    dist->local_b = keys_b_dev;
    dist->local_n = n_examples;
    dist->per_example = per_example;
    dist->split = split;
    dist->tile = tile;
    return NUPS_OK;
}

nups_status nups_set_postponing(nups_dist *dist, int enable)
{
    if (!dist) return fail(NUPS_ERR_ARG, "nups_set_postponing: null distribution");
    if (dist->scheme != NUPS_LONGTERM) return fail(NUPS_ERR_STATE, "nups_set_postponing: scheme is not LONG-TERM");
    if (enable && !dist->first_pos_dev) {
        const size_t bytes = sizeof(uint32_t) * (size_t)dist->ctx->tab[dist->table].num_keys;
        hipError_t e = hipMalloc((void **)&dist->first_pos_dev, bytes);
        if (e == hipSuccess) e = hipMemset(dist->first_pos_dev, 0xFF, bytes);    // "not seen" everywhere
        if (e != hipSuccess) {
            hip_ok(e, "nups_set_postponing: first-occurrence array");
            if (dist->first_pos_dev) (void)hipFree(dist->first_pos_dev);
            dist->first_pos_dev = nullptr;
            return NUPS_ERR_DEVICE;
        }
    }
    dist->postpone = enable != 0;
    return NUPS_OK;
}

nups_status nups_prepare_sample(nups_dist *dist, int64_t n, uint64_t step, nups_sample **out)
{
    if (!out) return fail(NUPS_ERR_ARG, "nups_prepare_sample: out is null");
    *out = nullptr;
    if (!dist) return fail(NUPS_ERR_ARG, "nups_prepare_sample: null distribution");
    if (n < 0 || n > 0x7FFFFFFFll) return fail(NUPS_ERR_ARG, "nups_prepare_sample: n out of range");
    if (step >> 48) return fail(NUPS_ERR_ARG, "nups_prepare_sample: step must be below 2^48");
    if (dist->scheme == NUPS_NONCONFORM) {
        if (!dist->local_a) return fail(NUPS_ERR_STATE, "nups_prepare_sample: call nups_set_local_keys first");
        if (n > dist->local_n * (int64_t)dist->per_example)
            return fail(NUPS_ERR_ARG, "nups_prepare_sample: more samples than examples * per_example");
    }
    nups_ctx *ctx = dist->ctx;
    nups_sample *h = nullptr;
    if (!dist->recycled.empty()) { h = dist->recycled.back(); dist->recycled.pop_back(); }
    else { h = new nups_sample(); h->dist = dist; }
    nups_status st = NUPS_OK;
    if (h->cap < (size_t)n || !h->keys_dev) {
        hipError_t e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess && h->keys_dev) e = hipFree(h->keys_dev);
        h->keys_dev = nullptr;
        h->cap = (size_t)n + (size_t)n / 4 + 1024;
        if (e == hipSuccess) e = hipMalloc((void **)&h->keys_dev, sizeof(uint32_t) * h->cap);
        if (e != hipSuccess) { hip_ok(e, "nups_prepare_sample: key buffer"); h->cap = 0; st = NUPS_ERR_DEVICE; }
    }
    if (st == NUPS_OK && dist->postpone && h->raw_cap < (size_t)n) {
        hipError_t e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess && h->raw_dev) e = hipFree(h->raw_dev);
        h->raw_dev = nullptr;
        h->raw_cap = h->cap;
        if (e == hipSuccess) e = hipMalloc((void **)&h->raw_dev, sizeof(uint32_t) * h->raw_cap);
        if (e != hipSuccess) { hip_ok(e, "nups_prepare_sample: key buffer"); h->raw_cap = 0; st = NUPS_ERR_DEVICE; }
    }
    if (st != NUPS_OK) { dist->recycled.push_back(h); return st; }
    h->n = n;
    h->pulled = 0;
    h->live = true;
    if (n > 0) {   // the drawing alone, enqueued now: PullSample and steps that use the handle follow it on the stream
        SideItem it{};
        it.phase = kSideDraw;
        it.n_plans = 0;
        it.blocks_per_plan = 1;
        it.draw = sample_args(dist, dist->postpone ? h->raw_dev : h->keys_dev, n, step);
        it.blocks = it.draw.blocks;
        PhaseScope scope(ctx, NUPS_PHASE_SAMPLE, ctx->stream);
        st = launch_side(ctx, it);
        if (st == NUPS_OK && dist->postpone) st = launch_postpone(dist, h->raw_dev, h->keys_dev, n);
    }
    if (dist->scheme == NUPS_LONGTERM) dist->cursor += (uint64_t)n;
    if (st != NUPS_OK) { h->live = false; dist->recycled.push_back(h); return st; }
    dist->live.push_back(h);
    *out = h;
    return NUPS_OK;
}

nups_status nups_pull_sample(nups_sample *h, int64_t n_j, uint32_t *keys_dev, float *values_dev)
{
    if (!h) return fail(NUPS_ERR_ARG, "nups_pull_sample: null handle");
    if (!h->live) return fail(NUPS_ERR_STATE, "nups_pull_sample: handle was released");
    if (n_j < 0) return fail(NUPS_ERR_ARG, "nups_pull_sample: negative count");
    if (h->pulled + n_j > h->n) return fail(NUPS_ERR_OVERPULL, "nups_pull_sample: more samples requested than prepared");
    if (n_j == 0) return NUPS_OK;
    nups_ctx *ctx = h->dist->ctx;
    const uint32_t *src = h->keys_dev + h->pulled;
    if (keys_dev)
        NUPS_HIP(hipMemcpyAsync(keys_dev, src, sizeof(uint32_t) * (size_t)n_j, hipMemcpyDeviceToDevice, ctx->stream));
    if (values_dev) {
        nups_status st = launch_pull(ctx, ctx->tab[h->dist->table], src, n_j, values_dev);
        if (st != NUPS_OK) return st;
    }
    h->pulled += n_j;
    return NUPS_OK;
}

nups_status nups_sample_keys(nups_sample *h, const uint32_t **keys_dev, int64_t *n)
{
    if (!h || !keys_dev) return fail(NUPS_ERR_ARG, "nups_sample_keys: null argument");
    if (!h->live) return fail(NUPS_ERR_STATE, "nups_sample_keys: handle was released");
    *keys_dev = h->keys_dev;
    if (n) *n = h->n;
    return NUPS_OK;
}

nups_status nups_release_sample(nups_sample *h)
{
    if (!h) return fail(NUPS_ERR_ARG, "nups_release_sample: null handle");
    if (!h->live) return fail(NUPS_ERR_STATE, "nups_release_sample: handle already released");
    nups_dist *d = h->dist;
    h->live = false;
    d->live.erase(std::remove(d->live.begin(), d->live.end(), h), d->live.end());
    d->recycled.push_back(h);
    return NUPS_OK;
}

nups_status nups_prepare_step(nups_ctx *ctx, const nups_batch *b, nups_prepared **out)
{
    if (!out) return fail(NUPS_ERR_ARG, "nups_prepare_step: out is null");
    *out = nullptr;
    nups_status st = check_batch(ctx, b);
    if (st != NUPS_OK) return st;
    nups_prepared *p = nullptr;
    if ((st = get_prepared(ctx, &p)) != NUPS_OK) return st;
    p->batch = *b;
    if (b->sample) {   // drawn when the handle was prepared, i.e. earlier on the stream
        p->batch.negs = b->sample->keys_dev;
        p->batch.sample = nullptr;
    }
    const int64_t n_draw = b->dist ? b->B * ((int64_t)b->n_neg + b->n_neg2) : 0;
    if (n_draw > 0 && p->negs_cap < (size_t)n_draw) {   // the step draws its own negatives into its own buffer
        hipError_t e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess && p->negs_buf) e = hipFree(p->negs_buf);
        p->negs_buf = nullptr;
        p->negs_cap = (size_t)n_draw + (size_t)n_draw / 4 + 1024;
        if (e == hipSuccess) e = hipMalloc((void **)&p->negs_buf, sizeof(uint32_t) * p->negs_cap);
        if (e != hipSuccess) {
            hip_ok(e, "nups_prepare_step: negatives buffer");
            p->negs_cap = 0;
            ctx->prepared_free.push_back(p);
            return NUPS_ERR_DEVICE;
        }
    }
    SampleArgs draw{};
    int mark_plan = -1;
    if (n_draw > 0) {
        draw = sample_args(b->dist, p->negs_buf, n_draw, b->sample_step);
        if (b->dist->scheme == NUPS_LONGTERM) b->dist->cursor += (uint64_t)n_draw;
        p->batch.negs = p->negs_buf;
        p->batch.dist = nullptr;
    }
    switch (b->task) {   // capacities and plan arguments
    case NUPS_TASK_SGNS: st = plan_step_sgns(ctx, *p); mark_plan = 1; break;
    case NUPS_TASK_MF: st = plan_step_mf(ctx, *p); break;
    default: st = plan_step_kge(ctx, *p); mark_plan = 0; break;
    }
    if (st != NUPS_OK) { ctx->prepared_free.push_back(p); return st; }
    // the drawn keys are marked as they are drawn (check_batch: they index the table that plan `mark_plan` is for);
    // the plan's own first phase marks the keys before them
    if (n_draw > 0) p->plan[mark_plan].a.mark_n -= (uint32_t)n_draw;
    else mark_plan = -1;
    build_phases(*p, draw, mark_plan);
    p->live = true;
    if (ctx->profiling) {   // every phase as a launch of its own, timed
        if ((st = flush_side_work(ctx, p)) != NUPS_OK) { p->live = false; ctx->prepared_free.push_back(p); return st; }
    } else {
        // Which launch carries which phase matters.  A factorisation step's update kernel is much shorter than the
        // rank phase, which by default rides in the update launch of the next step but one; when the caller prepares
        // four steps ahead (three are still under construction), the chain starts one launch later, so that the long
        // phases (tiles, rank, scatter) ride in the gradient launches and the short ones in the update launches.
        p->lead_launches = (b->task == NUPS_TASK_MF && ctx->pending.size() >= 3) ? 1 : 0;
        ctx->pending.push_back(p);
    }
    *out = p;
    return NUPS_OK;
}

nups_status nups_step_prepared(nups_ctx *ctx, nups_prepared *p, double *loss_sum_host)
{
    if (!ctx || !p) return fail(NUPS_ERR_ARG, "nups_step_prepared: null argument");
    if (p->ctx != ctx) return fail(NUPS_ERR_ARG, "nups_step_prepared: the step was prepared on another context");
    if (!p->live) return fail(NUPS_ERR_STATE, "nups_step_prepared: the prepared step was already run");
    nups_status st = flush_side_work(ctx, p);   // whatever earlier launches have not carried
    ctx->want_loss = loss_sum_host != nullptr;
    if (st == NUPS_OK) {
        switch (p->batch.task) {
        case NUPS_TASK_SGNS: st = run_step_sgns(ctx, *p); break;
        case NUPS_TASK_MF: st = run_step_mf(ctx, *p); break;
        default: st = run_step_kge(ctx, *p); break;
        }
    }
    retire_prepared(ctx, p);
    if (st != NUPS_OK) return st;
    if (loss_sum_host) {
        NUPS_HIP(hipMemcpyAsync(ctx->loss_pinned, p->loss_dev, sizeof(double) * kLossSlots * kLossStride,
                                hipMemcpyDeviceToHost, ctx->stream));
        st = sync_and_check(ctx);
        double total = 0.0;
        for (int s = 0; s < kLossSlots; ++s) total += ctx->loss_pinned[s * kLossStride];
        *loss_sum_host = total;
        return st;
    }
    return NUPS_OK;
}

nups_status nups_step(nups_ctx *ctx, const nups_batch *b, double *loss_sum_host)
{
    nups_prepared *p = nullptr;
    nups_status st = nups_prepare_step(ctx, b, &p);
    if (st != NUPS_OK) return st;
    return nups_step_prepared(ctx, p, loss_sum_host);
}

nups_status nups_debug_structure(nups_ctx *ctx, int table, uint32_t *uniq_keys_dev, uint32_t *counts_dev,
                                 int64_t *n_uniq_host)
{
    if (!valid_table(ctx, table) || !n_uniq_host) return fail(NUPS_ERR_ARG, "nups_debug_structure: bad arguments");
    const Plan *pl = ctx->tab[table].last_plan;
    if (!pl) return fail(NUPS_ERR_STATE, "nups_debug_structure: no step or push has run on this table");
    uint32_t meta[kMetaWords];
    NUPS_HIP(hipMemcpyAsync(meta, pl->a.meta, sizeof(meta), hipMemcpyDeviceToHost, ctx->stream));
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    const size_t nu = meta[kMetaNumUniq];
    if (uniq_keys_dev)
        NUPS_HIP(hipMemcpyAsync(uniq_keys_dev, pl->a.uniq, sizeof(uint32_t) * nu, hipMemcpyDeviceToDevice, ctx->stream));
    if (counts_dev)
        NUPS_HIP(hipMemcpyAsync(counts_dev, pl->a.count, sizeof(uint32_t) * nu, hipMemcpyDeviceToDevice, ctx->stream));
    *n_uniq_host = (int64_t)nu;
    return sync_and_check(ctx);
}

nups_status nups_check(nups_ctx *ctx)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_check: null context");
    return sync_and_check(ctx);
}

nups_status nups_profile(nups_ctx *ctx, int enable)
{
    if (!ctx) return fail(NUPS_ERR_ARG, "nups_profile: null context");
    ctx->profiling = enable != 0;
    return NUPS_OK;
}

nups_status nups_profile_read(nups_ctx *ctx, int phase, double *ms_total, int64_t *launches)
{
    if (!ctx || phase < 0 || phase >= NUPS_PHASE_COUNT) return fail(NUPS_ERR_ARG, "nups_profile_read: bad arguments");
    NUPS_HIP(hipStreamSynchronize(ctx->stream));
    Phase &ph = ctx->phase[phase];
    for (auto &pr : ph.pending) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) { ph.ms += ms; ph.launches += 1; }
        ph.free_events.push_back(pr.first);
        ph.free_events.push_back(pr.second);
    }
    ph.pending.clear();
    if (ms_total) *ms_total = ph.ms;
    if (launches) *launches = ph.launches;
    ph.ms = 0.0;
    ph.launches = 0;
    return NUPS_OK;
}

}  // extern "C"
