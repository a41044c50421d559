// Direct access (pull / push), the per-task gradient kernels of the minibatch step and the scheduling of
// preparatory work:
// skip-gram with negative sampling, matrix factorisation, ComplEx (Section 5.1).  Every
// kernel reads the tables as they are at the start of the step and writes only coefficients
// and staged gradient rows; the tables are updated afterwards, once per distinct key
// (segment_apply.h).
#include <mutex>

#include "segment_apply.h"

namespace nups {

// ------------------------------------------------------------------------------------------------
// Preparatory work of prepared steps: carried by the launches below, or launched on its own.
// ------------------------------------------------------------------------------------------------

// Workgroups per phase of side work in a carrier with many resident workgroups (narrow rows) or few (wide rows).
constexpr uint32_t kSideWgsNarrow = 1024, kSideWgsWide = 64;

// One phase on its own.
nups_status launch_side(nups_ctx *ctx, const SideItem &it)
{
    if (it.blocks == 0) return NUPS_OK;
    SideWork sw{};
    sw.n = 1;
    sw.blocks = it.blocks;
    sw.item[0] = it;
    sw.item[0].wgs = it.blocks;
    hipLaunchKernelGGL(k_side, dim3(it.blocks), dim3(kBlock), side_lds_bytes(it), ctx->stream, sw);
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

// The next phase of each of the oldest prepared steps (at most kMaxSide), for the launch that is about to be
// enqueued; *lds_bytes: dynamic LDS that the phases need.  A phase gets at most max_wgs_per_phase workgroups:
// a side workgroup takes the registers of one of the carrier's own, so carriers with few resident workgroups
// (wide rows) give the side work a few workgroups that loop, and have the time for it.
SideWork take_side_work(nups_ctx *ctx, size_t *lds_bytes, uint32_t max_wgs_per_phase)
{
    SideWork sw{};
    size_t lds = 0;
    for (auto it = ctx->pending.begin(); it != ctx->pending.end() && sw.n < kMaxSide;) {
        nups_prepared *p = *it;
        if (p->lead_launches > 0) {   // this step's phases start one launch later
            --p->lead_launches;
            ++it;
            continue;
        }
        const SideItem &ph = p->phases[p->next_phase++];
        sw.item[sw.n] = ph;
        sw.item[sw.n].wgs = std::min(ph.blocks, max_wgs_per_phase);
        sw.blocks += sw.item[sw.n].wgs;
        ++sw.n;
        lds = std::max(lds, side_lds_bytes(ph));
        if (p->next_phase == p->phases.size()) it = ctx->pending.erase(it);
        else ++it;
    }
    sw.blocks = (sw.blocks + kNumXcd - 1) / kNumXcd * kNumXcd;   // keeps the carrier's own workgroups die-aligned
    *lds_bytes = lds;
    return sw;
}

// Enqueues, as launches of their own, the phases of p that no launch has carried yet.
nups_status flush_side_work(nups_ctx *ctx, nups_prepared *p)
{
    for (auto it = ctx->pending.begin(); it != ctx->pending.end(); ++it)
        if (*it == p) { ctx->pending.erase(it); break; }
    if (p->next_phase >= p->phases.size()) return NUPS_OK;
    nups_status st = NUPS_OK;
    const SideItem &first = p->phases[p->next_phase];
    // when phases are timed, the drawing is a launch (and a timed phase) of its own, apart from the marking that
    // otherwise shares its launch
    const bool draws = ctx->profiling && first.phase == kSideDraw && first.draw.blocks > 0;
    if (draws) {
        SideItem draw = first;
        draw.blocks = first.draw.blocks;
        PhaseScope scope(ctx, NUPS_PHASE_SAMPLE, ctx->stream);
        st = launch_side(ctx, draw);
    }
    PhaseScope scope(ctx, NUPS_PHASE_PLAN, ctx->stream);
    if (draws && st == NUPS_OK) {
        SideItem mark = first;
        mark.block0 = first.draw.blocks;
        mark.blocks = first.blocks - first.draw.blocks;
        st = launch_side(ctx, mark);
        ++p->next_phase;
    }
    while (st == NUPS_OK && p->next_phase < p->phases.size()) st = launch_side(ctx, p->phases[p->next_phase++]);
    return st;
}

// ------------------------------------------------------------------------------------------------
// Norm clipping of hot-key updates (Section 5.1).  Before the update launch of a step, one wavefront per table
// adds up the table's slots of {sum of norms, number of norms} and leaves the bound for this step: factor x
// mean, +inf while no norm has been recorded.  The update kernel then adds this step's norms to the slots.
// ------------------------------------------------------------------------------------------------
static_assert(kLossSlots == 64, "one lane per slot");

__global__ void __launch_bounds__(64) k_clip_bounds(const double *stats, float factor, float *bound)
{
    const double *slot = stats + ((size_t)blockIdx.x * kLossSlots + threadIdx.x) * kLossStride;
    double sum = slot[0], seen = slot[1];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        sum += __shfl_xor(sum, o, 64);
        seen += __shfl_xor(seen, o, 64);
    }
    if (threadIdx.x == 0) bound[blockIdx.x] = seen > 0.0 ? (float)((double)factor * (sum / seen)) : INFINITY;
}

// The update rule of table `table` for a step with learning rate lr; with clipping on, the bounds of tables
// 0 and 1 must have been refreshed on the stream (refresh_clip_bounds) before the update kernel runs.
static OptSgd sgd_rule(const nups_ctx *ctx, int table, float lr)
{
    OptSgd opt{lr};
    if (ctx->clip_factor > 0.0f) {
        opt.clip_bound = ctx->clip_bound + table;
        opt.clip_stats = ctx->clip_stats + (size_t)table * kLossSlots * kLossStride;
    }
    return opt;
}

static nups_status refresh_clip_bounds(nups_ctx *ctx)
{
    if (!(ctx->clip_factor > 0.0f)) return NUPS_OK;
    hipLaunchKernelGGL(k_clip_bounds, dim3(2), dim3(64), 0, ctx->stream, (const double *)ctx->clip_stats,
                       ctx->clip_factor, ctx->clip_bound);
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

// ------------------------------------------------------------------------------------------------
// pull: values[i, :] = table[keys[i], :] (Section 3.1).  One 16-lane group per row: a load instruction of a group
// reads 256 contiguous bytes, a wavefront keeps four rows in flight; zero rows for keys out of range.
// ------------------------------------------------------------------------------------------------
template <int NV4>
__global__ void __launch_bounds__(kBlock) k_pull(const float *table, uint32_t num_keys, int stride,
                                                 const uint32_t *keys, uint32_t n, float *values,
                                                 uint32_t *error_flag)
{
    const int lane = threadIdx.x & (kGroup - 1);
    const uint32_t i = (blockIdx.x * kBlock + threadIdx.x) / kGroup;
    if (i >= n) return;
    const uint32_t key = keys[i];
    Row<NV4> r;
    if (key < num_keys) {
        load_row(r, table + (size_t)key * stride, lane);
    } else {
        zero_row(r);
        if (lane == 0) atomicOr(error_flag, 1u);
    }
    store_row(values + (size_t)i * stride, r, lane);
}

nups_status launch_pull(nups_ctx *ctx, const Table &t, const uint32_t *keys, int64_t n, float *values)
{
    if (n == 0) return NUPS_OK;
    PhaseScope scope(ctx, NUPS_PHASE_PULL, ctx->stream);
    if (n > 0x7FFFFFFFll) return fail(NUPS_ERR_ARG, "nups_pull: too many rows for one call");
    const uint32_t blocks = (uint32_t)((n + kGroupsPerBlock - 1) / kGroupsPerBlock);
#define CALL(N)                                                                                                   \
    hipLaunchKernelGGL(k_pull<N>, dim3(blocks), dim3(kBlock), 0, ctx->stream, (const float *)t.data,              \
                       (uint32_t)t.num_keys, t.stride, keys, (uint32_t)n, values, ctx->error_flag)
    NUPS_FOR_EACH_ROW_WIDTH(t.stride, CALL)
#undef CALL
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

// push: table[k] += sum of the update rows sent for k (plan already built over the keys).
nups_status launch_push_apply(nups_ctx *ctx, Table &t, const Plan &pl, float *partial, float *totals, uint32_t grid_cap,
                              const float *updates)
{
    PhaseScope scope(ctx, NUPS_PHASE_PUSH, ctx->stream);
    return launch_apply(ctx->stream, pl, partial, ApplyScratch{totals, grid_cap}, t.data, nullptr, t.stride,
                        SrcStaged{updates}, OptAdd{});
}

// Where the rows of a table live for the gradient kernels: the table, and the replicas of its hot keys if it has
// any (Section 3.2).  row(key, example): the row that the example's access to `key` reads (and updates).
struct RowSpace {
    float *table;
    float *replica_rows;
    ReplicaMap rep;          // rep.base_keys: keys of the table
    __device__ __forceinline__ uint32_t keys() const { return rep.base_keys; }
    // kReplicas false: the caller knows that neither table of the step has replicas (a kernel compiled for that
    // case carries none of the look-ups)
    template <bool kReplicas = true>
    __device__ __forceinline__ float *row(uint32_t key, uint32_t example, int stride) const
    {
        const uint32_t valid = min(key, rep.base_keys - 1);   // keys outside the table are flagged by the structure
        if (!kReplicas) return table + (size_t)valid * stride;
        return extended_row(table, replica_rows, rep.base_keys, replica_key(rep, valid, example), stride);
    }
};

static RowSpace row_space(const Table &t, const Plan &pl) { return RowSpace{t.data, t.replica_rows, pl.a.rep}; }

// ------------------------------------------------------------------------------------------------
// Skip-gram with negative sampling.  One 16-lane group per (center, context) pair:
//   z_j = <v, u_j>, g_j = sigma(z_j) - label_j, input-side gradient of the pair = sum_j g_j u_j.
// The input-side gradients of a run of consecutive pairs with the same center word (in stream order a word's 2 x
// window pairs follow each other) are added up inside the workgroup, through LDS, by the group of the run's first
// pair, in pair order.  If the run holds every pair of its center word in this step (the word's segment in the
// input table's structure is as long as the run), that group updates the input row right away: it has the row in
// registers, nobody else reads it in this step, and the output side works from the staged copy of the row.
// Otherwise the run's sum is staged at the row of its first pair and the update kernel adds the runs of the word.
// So a staged gradient row is written per run that shares its word with other runs, not per pair.
// What the update kernel needs it finds where the accesses stand in the tables' segment orders (out_pos, center_pos:
// the structure's positions): per scored row its coefficient and the number of the pair's staged center row; per
// pair the staged row of its run's sum, "none" inside a run, "done" for a word updated here (SrcStagedAt).
// ------------------------------------------------------------------------------------------------
template <int NV4, bool kWithLoss, bool kReplicas>
__global__ void __launch_bounds__(kBlock) k_sgns_grad(RowSpace in_rows, RowSpace out_rows, int stride,
                                                      const uint32_t *center, const uint32_t *context,
                                                      const uint32_t *negs, uint32_t B, int K, float lr,
                                                      const uint32_t *out_pos, float *coef_at, uint32_t *row_at,
                                                      float *stage, int update_whole_runs,
                                                      const uint32_t *center_slot, const uint32_t *center_rank,
                                                      const uint32_t *center_seg, const uint32_t *center_pos,
                                                      uint32_t *in_row_at, float *center_rows, double *loss,
                                                      SideWork sw)
{
    extern __shared__ float run_rows[];   // [kGroupsPerBlock][stride]: the pairs' input-side gradients
    __shared__ float lds[kBlock / 64];
    __shared__ uint32_t run_key[kGroupsPerBlock];
    if (side_work_block(sw)) return;   // the first sw.blocks workgroups prepare later steps
    const int lane = threadIdx.x & (kGroup - 1), group = threadIdx.x / kGroup;
    const uint32_t own_block = blockIdx.x - sw.blocks;
    const uint32_t e_raw = (xcd_block(own_block, gridDim.x - sw.blocks) * kBlock + threadIdx.x) / kGroup;
    const bool active = e_raw < B;
    const uint32_t e = active ? e_raw : B - 1;
    // the row (or replica row) of the center word
    const uint32_t crow = kReplicas ? run_row(center, in_rows.rep, e)
                                    : (center[e] < in_rows.keys() ? center[e] : kBadIndex);
    const uint32_t slot = center_slot[e];          // kBadIndex: the center key is outside the table
    const uint32_t in_pos = center_pos[e];         // where the pair's access stands in the input table's order
    uint32_t seg_len = 0;
    if (slot != kBadIndex) seg_len = center_seg[slot + 1] - center_seg[slot];
    Row<NV4> v, acc;
    float *v_row = in_rows.template row<kReplicas>(center[e], e, stride);
    load_row(v, v_row, lane);
    // the first pair of every distinct center word keeps a copy of the input vector for the output-side update
    if (active && slot != kBadIndex && (center_rank[e] & ~kSingleAccess) == 0)
        store_row(center_rows + (size_t)slot * stride, v, lane);
    zero_row(acc);
    float loss_acc = 0.f;
    // rows in flight per group: all of a pair's scored rows at three negatives; rows of 1,024 floats take 64
    // registers each, and two of them in flight leave room for two wavefronts per SIMD instead of one (gradient kernel
    // of the 1.9M-word, d = 1000 workload: 60 -> 33 us)
    constexpr int JU = NV4 >= 16 ? 2 : 4;
    const uint32_t n_out = B * (uint32_t)(K + 1);
    for (int j0 = 0; j0 <= K; j0 += JU) {
        // lane jj of the group looks after scored row j0 + jj: where its access stands in the output table's order
        uint32_t my_pos = kBadIndex;
        if (active && lane < JU && j0 + lane <= K)
            my_pos = out_pos[(j0 + lane == 0) ? e : B + e * (uint32_t)K + (uint32_t)(j0 + lane - 1)];
        Row<NV4> u[JU];
#pragma unroll
        for (int jj = 0; jj < JU; ++jj) {
            const int j = min(j0 + jj, K);
            const uint32_t key = (j == 0) ? context[e] : negs[(size_t)e * K + (j - 1)];
            load_row(u[jj], out_rows.template row<kReplicas>(key, e, stride), lane);
        }
        float g_mine = 0.f;   // lane jj of the group keeps coefficient j0 + jj: one store for the JU of them
#pragma unroll
        for (int jj = 0; jj < JU; ++jj) {
            const int j = j0 + jj;
            if (j <= K) {
                const float z = group_sum(partial_dot(v, u[jj]));
                const float g = sigmoidf(z) - (j == 0 ? 1.0f : 0.0f);
                if (kWithLoss) loss_acc += softplusf(j == 0 ? -z : z);   // only when the caller asked for the loss
                if (lane == jj) g_mine = g;
                axpy_row(acc, g, u[jj]);
            }
        }
        if (my_pos < n_out) {   // an access that the structure dropped (key outside the table) has no position
            coef_at[my_pos] = g_mine;
            row_at[my_pos] = slot == kBadIndex ? 0u : slot;   // bad center key: flagged, row 0 used
        }
    }
    // runs of equal center words inside the workgroup (pairs beyond the batch belong to no run)
    if (lane == 0) run_key[group] = active ? crow : kBadIndex;
    store_row(run_rows + (size_t)group * stride, acc, lane);
    if (kWithLoss) {   // the wavefronts' loss sums cross the same barrier as the runs' rows
        const float wave_loss = wave_sum((active && lane == 0) ? loss_acc : 0.f);
        if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = wave_loss;
    }
    __syncthreads();
    if (kWithLoss && threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < kBlock / 64; ++w) s += (double)lds[w];
        atomicAdd(loss + (blockIdx.x % kLossSlots) * kLossStride, s);
    }
    if (active && slot != kBadIndex) {
        uint32_t source = kNoRow;   // what the update kernel finds at this access: nothing more, inside a run
        if (group == 0 || run_key[group - 1] != crow) {
            uint32_t len = 1;
            while (group + len < (uint32_t)kGroupsPerBlock && run_key[group + len] == crow) {
                Row<NV4> r;
                load_row(r, run_rows + (size_t)(group + len) * stride, lane);
                axpy_row(acc, 1.0f, r);
                ++len;
            }
            if (update_whole_runs && len == seg_len) {
#pragma unroll
                for (int q = 0; q < NV4; ++q) axpy4(v.v[q], -lr, acc.v[q]);
                store_row(v_row, v, lane);
                source = kRowDone;
            } else {
                store_row(stage + (size_t)e * stride, acc, lane);
                source = e;
            }
        }
        if (lane == 0 && in_pos < B) in_row_at[in_pos] = source;
    }
}

template <int NV4>
static void launch_sgns_grad(nups_ctx *ctx, const nups_batch &b, const Plan &in_plan, const Plan &out_plan,
                             float *center_rows, uint32_t *row_at, uint32_t *in_row_at, bool update_whole_runs,
                             const SideWork &sw, size_t side_lds)
{
    const Table &tin = ctx->tab[0], &tout = ctx->tab[1];
    const uint32_t blocks = xcd_grid((uint32_t)((b.B + kGroupsPerBlock - 1) / kGroupsPerBlock));
    const size_t lds = std::max(sizeof(float) * kGroupsPerBlock * (size_t)tin.stride, side_lds);
    static size_t allowed[4] = {0, 0, 0, 0};
    const auto launch = [&](auto kernel, size_t *granted) {
        allow_lds(kernel, lds, granted);
        hipLaunchKernelGGL(kernel, dim3(sw.blocks + blocks), dim3(kBlock), lds, ctx->stream, row_space(tin, in_plan),
                           row_space(tout, out_plan), tin.stride, b.k0, b.k1, b.negs, (uint32_t)b.B, (int)b.n_neg, b.lr, (const uint32_t *)out_plan.a.pos, ctx->coef,
                           row_at, ctx->stage, update_whole_runs ? 1 : 0, (const uint32_t *)in_plan.a.slot,
                           (const uint32_t *)in_plan.a.rank, (const uint32_t *)in_plan.a.seg,
                           (const uint32_t *)in_plan.a.pos, in_row_at, center_rows, ctx->loss_cur, sw);
    };
    const bool replicas = in_plan.a.rep.hot_slot != nullptr || out_plan.a.rep.hot_slot != nullptr;
    if (ctx->want_loss && replicas) launch(k_sgns_grad<NV4, true, true>, &allowed[3]);
    else if (ctx->want_loss) launch(k_sgns_grad<NV4, true, false>, &allowed[2]);
    else if (replicas) launch(k_sgns_grad<NV4, false, true>, &allowed[1]);
    else launch(k_sgns_grad<NV4, false, false>, &allowed[0]);
}

// Plan side of a step: which keys each table is accessed with (plan 0: table 0, plan 1: table 1).  Sizes the
// arrays and fills in the arguments; the caller then lists the phases of the construction (build_phases).
static nups_status plan_two_tables(nups_ctx *ctx, nups_prepared &p, const KeySource &s0, uint32_t n0,
                                   const KeySource &s1, uint32_t n1)
{
    nups_status st;
    p.n_plans = 2;
    p.plan[0].table = 0;
    p.plan[1].table = 1;
    if ((st = ensure_plan_capacity(ctx, ctx->tab[0], p.plan[0], n0)) != NUPS_OK) return st;
    if ((st = ensure_plan_capacity(ctx, ctx->tab[1], p.plan[1], n1)) != NUPS_OK) return st;
    p.plan[0].a.src = s0;
    p.plan[0].a.n = p.plan[0].a.mark_n = n0;
    p.plan[1].a.src = s1;
    p.plan[1].a.n = p.plan[1].a.mark_n = n1;
    p.plan[0].a.zero_loss = p.loss_dev;
    p.plan[1].a.zero_loss = nullptr;
    p.plan[0].a.rep.batch = p.plan[1].a.rep.batch = (uint32_t)std::max<int64_t>(p.batch.B, 1);
    // partial rows of chunked segments: one region per table, the two updates run in the same launch
    const size_t need = (max_chunks(p.plan[0].cap_n) + max_chunks(p.plan[1].cap_n)) * (size_t)ctx->tab[0].stride;
    if ((st = ensure_partial(ctx, need)) != NUPS_OK) return st;
    return ensure_totals(ctx, ctx->tab[0].stride);
}

nups_status plan_step_sgns(nups_ctx *ctx, nups_prepared &p)
{
    const nups_batch &b = p.batch;
    const uint32_t B = (uint32_t)b.B, K = (uint32_t)b.n_neg;
    return plan_two_tables(ctx, p, KeySource{{b.k0, nullptr, nullptr}, {B, 0, 0}, {1, 0, 0}}, B,
                           KeySource{{b.k1, b.negs, nullptr}, {B, B * K, 0}, {1, K, 0}}, B * (K + 1));
}

static ApplyScratch update_scratch(nups_ctx *ctx, int stride) { return ApplyScratch{ctx->totals, apply_grid_of_stride(stride)}; }

// Where table 1's partial rows start inside the context's partial buffer.
static float *partial_of(nups_ctx *ctx, const nups_prepared &p, int k)
{
    return k == 0 ? ctx->partial : ctx->partial + max_chunks(p.plan[0].cap_n) * (size_t)ctx->tab[0].stride;
}

nups_status run_step_sgns(nups_ctx *ctx, nups_prepared &p)
{
    const nups_batch &b = p.batch;
    Table &tin = ctx->tab[0], &tout = ctx->tab[1];
    const uint32_t B = (uint32_t)b.B, K = (uint32_t)b.n_neg;
    nups_status st;
    // per access of the output table, in the order of its structure: the coefficient, then (as integers) the row
    // of the center word among the staged center rows; then per access of the input table, in the order of its
    // structure: the staged row of its run's sum (SrcStagedAt)
    if ((st = ensure_f32(&ctx->coef, &ctx->coef_cap, (size_t)2 * B * (K + 1) + B, ctx->stream)) != NUPS_OK) return st;
    uint32_t *row_at = reinterpret_cast<uint32_t *>(ctx->coef + (size_t)B * (K + 1));
    uint32_t *in_row_at = row_at + (size_t)B * (K + 1);
    // staged rows: [0, B) input-side gradient sums of runs of pairs (at the runs' first pairs), [B, 2B) input
    // vectors of the distinct center words
    if ((st = ensure_f32(&ctx->stage, &ctx->stage_cap, (size_t)2 * B * tin.stride, ctx->stream)) != NUPS_OK) return st;
    ctx->loss_cur = p.loss_dev;   // zeroed by the step's plan construction
    if (B == 0) return NUPS_OK;
    float *center_rows = ctx->stage + (size_t)B * tin.stride;
    // With norm clipping on, every update goes through the update kernel, which measures and clips the hot keys'.
    const bool update_whole_runs = !(ctx->clip_factor > 0.0f);
    size_t side_lds = 0;
    {
        const SideWork sw = take_side_work(ctx, &side_lds, kSideWgsNarrow);
        PhaseScope scope(ctx, NUPS_PHASE_GRAD, ctx->stream);
#define CALL(N) launch_sgns_grad<N>(ctx, b, p.plan[0], p.plan[1], center_rows, row_at, in_row_at, update_whole_runs, sw, side_lds)
        NUPS_FOR_EACH_ROW_WIDTH(tin.stride, CALL)
#undef CALL
        NUPS_HIP(hipGetLastError());
    }
    {   // both tables in one launch: the output side reads the staged center rows, not the input table
        const SideWork sw = take_side_work(ctx, &side_lds, kSideWgsNarrow);
        PhaseScope scope(ctx, NUPS_PHASE_APPLY0, ctx->stream);
        if ((st = refresh_clip_bounds(ctx)) != NUPS_OK) return st;
        const TableUpdate<SrcStagedAt, OptSgd> uin{&p.plan[0], partial_of(ctx, p, 0), tin.data, nullptr,
                                                   SrcStagedAt{ctx->stage, in_row_at, update_whole_runs}, sgd_rule(ctx, 0, b.lr),
                                                   tin.replica_rows};
        const TableUpdate<SrcSgnsOut, OptSgd> uout{&p.plan[1], partial_of(ctx, p, 1), tout.data, nullptr,
                                                   SrcSgnsOut{center_rows, ctx->coef, row_at}, sgd_rule(ctx, 1, b.lr),
                                                   tout.replica_rows};
        // the output table first: its items are the many, the input table's few remaining ones fill in behind
        if ((st = launch_apply2(ctx->stream, tin.stride, uout, uin, update_scratch(ctx, tin.stride), sw, side_lds)) != NUPS_OK) return st;
    }
    return NUPS_OK;
}

// ------------------------------------------------------------------------------------------------
// Replicas of hot keys (Section 3.2).  init: every replica starts as a copy of its key's row.  sync: the periodic
// synchronisation, an exchange of the updates accumulated since the last one: the key's row (the value at the
// last synchronisation) gains every replica's difference from it, in replica order, and row and replicas are set
// to the result.  One 16-lane group per hot key.
// ------------------------------------------------------------------------------------------------
template <int NV4, bool kSync>
__global__ void __launch_bounds__(kBlock) k_replicas(float *table, float *replica_rows, const uint32_t *hot_list,
                                                     uint32_t hot_count, uint32_t replicas, int stride)
{
    const int lane = threadIdx.x & (kGroup - 1);
    const uint32_t s = (blockIdx.x * kBlock + threadIdx.x) / kGroup;
    if (s >= hot_count) return;
    float *base_row = table + (size_t)hot_list[s] * stride;
    Row<NV4> base, total;
    load_row(base, base_row, lane);
    total = base;
    if (kSync) {
        for (uint32_t r = 0; r < replicas; ++r) {
            Row<NV4> v;
            load_row(v, replica_rows + ((size_t)r * hot_count + s) * stride, lane);
#pragma unroll
            for (int q = 0; q < NV4; ++q) {
                total.v[q].x += v.v[q].x - base.v[q].x;
                total.v[q].y += v.v[q].y - base.v[q].y;
                total.v[q].z += v.v[q].z - base.v[q].z;
                total.v[q].w += v.v[q].w - base.v[q].w;
            }
        }
        store_row(base_row, total, lane);
    }
    for (uint32_t r = 0; r < replicas; ++r) store_row(replica_rows + ((size_t)r * hot_count + s) * stride, total, lane);
}

nups_status launch_replicas(nups_ctx *ctx, Table &t, bool sync)
{
    const uint32_t H = (uint32_t)t.hot_keys.size();
    if (!t.replica_rows || H == 0) return NUPS_OK;
    const uint32_t blocks = (H + kGroupsPerBlock - 1) / kGroupsPerBlock;
#define CALL(N)                                                                                                      \
    if (sync)                                                                                                        \
        hipLaunchKernelGGL((k_replicas<N, true>), dim3(blocks), dim3(kBlock), 0, ctx->stream, t.data, t.replica_rows,  \
                           (const uint32_t *)t.hot_list_dev, H, (uint32_t)ctx->replicas, t.stride);                  \
    else                                                                                                             \
        hipLaunchKernelGGL((k_replicas<N, false>), dim3(blocks), dim3(kBlock), 0, ctx->stream, t.data, t.replica_rows, \
                           (const uint32_t *)t.hot_list_dev, H, (uint32_t)ctx->replicas, t.stride)
    NUPS_FOR_EACH_ROW_WIDTH(t.stride, CALL)
#undef CALL
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

// ------------------------------------------------------------------------------------------------
// Matrix factorisation.  One group per cell: err = x - <w, h>; staged rows
//   dW = -2 err h + 2 l2 w   (rows [0, B))      dH = -2 err w + 2 l2 h   (rows [B, 2B)).
// A row whose only access of the step is this cell is updated here instead, theta <- theta - lr d, while it is in
// registers: nobody else reads it in this step, so every gradient is still taken at the values of the step's start,
// and the row is read once and written once in all, with no staged copy (most rows of a long tail are of this
// kind).  rank_w: the row plan's per-access flags (kSingleAccess); null: stage everything.
// Columns: the task's workers walk their cells column by column (Section 5.1), so consecutive cells share their
// column.  As for the center words of skip-gram pairs, the column gradients of a run of consecutive cells with one
// column are added up inside the workgroup, through LDS, by the group of the run's first cell, in cell order; a
// column whose cells of this step all sit in the run (a single cell included) is updated right away, otherwise the
// run's sum is staged at the row of its first cell: one staged row per run instead of one per cell.
// slot_h, seg_h: the column plan's per-access key numbers and segment bounds.  kRuns false (narrow rows, see
// kMfRunsFromNV4): columns are treated like rows (rank_h: the column plan's flags), nothing goes through LDS, and the
// update kernel finds the staged rows through the plans' access numbers (SrcStaged).
// ------------------------------------------------------------------------------------------------
// Row width (in units of 64 floats) from which the column gradients of runs are added up in the gradient kernel.
// Measured on 10M x 1M factors, 65,536 cells per step: rows of 128 floats: the look-ups and the round trip through
// LDS cost more than the staged rows they save (cells in generation order 68.8 against 64.5 us per step, visited by
// column 59.6 against 55.9); rows of 1,024 floats visited by column: 210 against 301 us.
constexpr int kMfRunsFromNV4 = 4;

template <int NV4, bool kRuns>
__global__ void __launch_bounds__(kBlock) k_mf_grad(RowSpace W, RowSpace H, int stride, const uint32_t *row, const uint32_t *col,
                                                    const float *val, uint32_t B, float l2, float lr,
                                                    const uint32_t *rank_w, const uint32_t *rank_h,
                                                    const uint32_t *slot_h, const uint32_t *seg_h, const uint32_t *pos_w, const uint32_t *pos_h, uint32_t *row_at_w,
                                                    uint32_t *row_at_h, int update_whole_runs, float *stage, double *loss,
                                                    SideWork sw)
{
    extern __shared__ float run_rows[];   // [kGroupsPerBlock][stride]: the cells' column gradients
    __shared__ float lds[kBlock / 64];
    __shared__ uint32_t run_key[kGroupsPerBlock];
    if (side_work_block(sw)) return;   // the first sw.blocks workgroups prepare later steps
    const int lane = threadIdx.x & (kGroup - 1), group = threadIdx.x / kGroup;
    const uint32_t c_raw = (xcd_block(blockIdx.x - sw.blocks, gridDim.x - sw.blocks) * kBlock + threadIdx.x) / kGroup;
    const bool active = c_raw < B;
    const uint32_t c = active ? c_raw : B - 1;
    Row<NV4> w, h;
    const uint32_t rk = row[c], ck = col[c];
    const bool alone_w = rank_w != nullptr && rk < W.keys() && (rank_w[c] & kSingleAccess) != 0;
    const bool alone_h = !kRuns && rank_h != nullptr && ck < H.keys() && (rank_h[c] & kSingleAccess) != 0;
    uint32_t h_id = kBadIndex, h_slot = kBadIndex, h_seg_len = 0, at_w = kBadIndex, at_h = kBadIndex;
    if (kRuns) {
        h_id = run_row(col, H.rep, c);   // the column's row (or replica row); kBadIndex: outside the table
        h_slot = slot_h[c];              // kBadIndex: dropped by the structure
        if (h_slot != kBadIndex) h_seg_len = seg_h[h_slot + 1] - seg_h[h_slot];
        at_w = pos_w[c];                 // where the cell's accesses stand in the plans' orders
        at_h = pos_h[c];
    }
    float *w_row = W.row(rk, c, stride), *h_row = H.row(ck, c, stride);
    load_row(w, w_row, lane);
    load_row(h, h_row, lane);
    const float dot = group_sum(partial_dot(w, h));
    const float nw = group_sum(partial_dot(w, w));
    const float nh = group_sum(partial_dot(h, h));
    const float err = val[c] - dot;
    Row<NV4> dw, dh;
#pragma unroll
    for (int q = 0; q < NV4; ++q) {
        dw.v[q] = make_float4(-2.f * err * h.v[q].x + 2.f * l2 * w.v[q].x, -2.f * err * h.v[q].y + 2.f * l2 * w.v[q].y,
                              -2.f * err * h.v[q].z + 2.f * l2 * w.v[q].z, -2.f * err * h.v[q].w + 2.f * l2 * w.v[q].w);
        dh.v[q] = make_float4(-2.f * err * w.v[q].x + 2.f * l2 * h.v[q].x, -2.f * err * w.v[q].y + 2.f * l2 * h.v[q].y,
                              -2.f * err * w.v[q].z + 2.f * l2 * h.v[q].z, -2.f * err * w.v[q].w + 2.f * l2 * h.v[q].w);
    }
    if (active) {
        if (alone_w) {
#pragma unroll
            for (int q = 0; q < NV4; ++q) axpy4(w.v[q], -lr, dw.v[q]);
            store_row(w_row, w, lane);
        } else {
            store_row(stage + (size_t)c * stride, dw, lane);
        }
        if (kRuns && lane == 0 && at_w < B) row_at_w[at_w] = alone_w ? kRowDone : c;   // what the update kernel finds (SrcStagedAt)
        if (!kRuns) {
            if (alone_h) {
#pragma unroll
                for (int q = 0; q < NV4; ++q) axpy4(h.v[q], -lr, dh.v[q]);
                store_row(h_row, h, lane);
            } else {
                store_row(stage + ((size_t)B + c) * stride, dh, lane);
            }
        }
    }
    if (!kRuns) {
        block_add_loss((active && lane == 0) ? err * err + l2 * (nw + nh) : 0.f, loss, lds);
        return;
    }
    // runs of equal columns inside the workgroup (cells beyond the batch and keys outside the table belong to none)
    if (lane == 0) run_key[group] = active ? h_id : kBadIndex;
    store_row(run_rows + (size_t)group * stride, dh, lane);
    block_add_loss((active && lane == 0) ? err * err + l2 * (nw + nh) : 0.f, loss, lds);   // its barrier serves the runs too
    if (active && h_slot != kBadIndex) {
        uint32_t source = kNoRow;   // inside a run: nothing more to add
        if (group == 0 || run_key[group - 1] != h_id) {
            uint32_t len = 1;
            while (group + len < (uint32_t)kGroupsPerBlock && run_key[group + len] == h_id) {
                Row<NV4> r;
                load_row(r, run_rows + (size_t)(group + len) * stride, lane);
                axpy_row(dh, 1.0f, r);
                ++len;
            }
            if (update_whole_runs && len == h_seg_len) {
#pragma unroll
                for (int q = 0; q < NV4; ++q) axpy4(h.v[q], -lr, dh.v[q]);
                store_row(h_row, h, lane);
                source = kRowDone;
            } else {
                store_row(stage + ((size_t)B + c) * stride, dh, lane);
                source = c;
            }
        }
        if (lane == 0 && at_h < B) row_at_h[at_h] = source;
    }
}

template <int NV4>
static void launch_mf_grad(nups_ctx *ctx, const nups_batch &b, const nups_prepared &p, const uint32_t *rank_w,
                           uint32_t *row_at, bool update_whole_runs, const SideWork &sw, size_t side_lds)
{
    const Table &tw = ctx->tab[0], &th = ctx->tab[1];
    const uint32_t blocks = xcd_grid((uint32_t)((b.B + kGroupsPerBlock - 1) / kGroupsPerBlock));
    constexpr bool kRuns = NV4 >= kMfRunsFromNV4;
    const size_t lds = kRuns ? std::max(sizeof(float) * kGroupsPerBlock * (size_t)tw.stride, side_lds) : side_lds;
    static size_t allowed = 0;
    allow_lds(k_mf_grad<NV4, kRuns>, lds, &allowed);
    const uint32_t *rank_h = rank_w ? (const uint32_t *)p.plan[1].a.rank : nullptr;
    hipLaunchKernelGGL((k_mf_grad<NV4, kRuns>), dim3(sw.blocks + blocks), dim3(kBlock), lds, ctx->stream,
                       row_space(tw, p.plan[0]), row_space(th, p.plan[1]), tw.stride, b.k0, b.k1, b.val, (uint32_t)b.B, b.l2,
                       b.lr, rank_w, rank_h, (const uint32_t *)p.plan[1].a.slot, (const uint32_t *)p.plan[1].a.seg,
                       (const uint32_t *)p.plan[0].a.pos, (const uint32_t *)p.plan[1].a.pos, row_at,
                       row_at + (size_t)b.B, update_whole_runs ? 1 : 0, ctx->stage, ctx->loss_cur, sw);
}

nups_status plan_step_mf(nups_ctx *ctx, nups_prepared &p)
{
    const nups_batch &b = p.batch;
    const uint32_t B = (uint32_t)b.B;
    return plan_two_tables(ctx, p, KeySource{{b.k0, nullptr, nullptr}, {B, 0, 0}}, B,
                           KeySource{{b.k1, nullptr, nullptr}, {B, 0, 0}}, B);
}

nups_status run_step_mf(nups_ctx *ctx, nups_prepared &p)
{
    const nups_batch &b = p.batch;
    Table &tw = ctx->tab[0], &th = ctx->tab[1];
    const uint32_t B = (uint32_t)b.B;
    nups_status st;
    if ((st = ensure_f32(&ctx->stage, &ctx->stage_cap, (size_t)2 * B * tw.stride, ctx->stream)) != NUPS_OK) return st;
    // per access of either table, in the order of its structure: the staged row to add (SrcStagedAt)
    if ((st = ensure_f32(&ctx->coef, &ctx->coef_cap, (size_t)2 * B, ctx->stream)) != NUPS_OK) return st;
    uint32_t *row_at = reinterpret_cast<uint32_t *>(ctx->coef);
    ctx->loss_cur = p.loss_dev;   // zeroed by the step's plan construction
    if (B == 0) return NUPS_OK;
    size_t side_lds = 0;
    // Rows with a single access and columns whose cells are all in one run are updated by the gradient kernel; with
    // norm clipping on, every update goes through the update kernel, which measures and clips the hot keys' updates.
    const bool singles_in_place = !(ctx->clip_factor > 0.0f);
    const uint32_t *rank_w = singles_in_place ? p.plan[0].a.rank : nullptr;
    {
        const SideWork sw = take_side_work(ctx, &side_lds, kSideWgsNarrow);
        PhaseScope scope(ctx, NUPS_PHASE_GRAD, ctx->stream);
#define CALL(N) launch_mf_grad<N>(ctx, b, p, rank_w, row_at, singles_in_place, sw, side_lds)
        NUPS_FOR_EACH_ROW_WIDTH(tw.stride, CALL)
#undef CALL
        NUPS_HIP(hipGetLastError());
    }
    {
        const SideWork sw = take_side_work(ctx, &side_lds, kSideWgsNarrow);
        PhaseScope scope(ctx, NUPS_PHASE_APPLY0, ctx->stream);
        if ((st = refresh_clip_bounds(ctx)) != NUPS_OK) return st;
        if (tw.stride / 64 >= kMfRunsFromNV4) {
            const TableUpdate<SrcStagedAt, OptSgd> uw{&p.plan[0], partial_of(ctx, p, 0), tw.data, nullptr,
                                                      SrcStagedAt{ctx->stage, row_at, singles_in_place}, sgd_rule(ctx, 0, b.lr),
                                                      tw.replica_rows};
            const TableUpdate<SrcStagedAt, OptSgd> uh{&p.plan[1], partial_of(ctx, p, 1), th.data, nullptr,
                                                      SrcStagedAt{ctx->stage + (size_t)B * tw.stride, row_at + (size_t)B, singles_in_place},
                                                      sgd_rule(ctx, 1, b.lr), th.replica_rows};
            st = launch_apply2(ctx->stream, tw.stride, uw, uh, update_scratch(ctx, tw.stride), sw, side_lds);
        } else {
            const TableUpdate<SrcStaged, OptSgd> uw{&p.plan[0], partial_of(ctx, p, 0), tw.data, nullptr,
                                                    SrcStaged{ctx->stage, singles_in_place}, sgd_rule(ctx, 0, b.lr),
                                                    tw.replica_rows};
            const TableUpdate<SrcStaged, OptSgd> uh{&p.plan[1], partial_of(ctx, p, 1), th.data, nullptr,
                                                    SrcStaged{ctx->stage + (size_t)B * tw.stride, singles_in_place},
                                                    sgd_rule(ctx, 1, b.lr), th.replica_rows};
            st = launch_apply2(ctx->stream, tw.stride, uw, uh, update_scratch(ctx, tw.stride), sw, side_lds);
        }
        if (st != NUPS_OK) return st;
    }
    return NUPS_OK;
}

// ------------------------------------------------------------------------------------------------
// ComplEx with logistic loss.  A stored row is two halves: real parts from float 0, imaginary parts
// from float stride / 2; with stride a multiple of 128 a lane owns float4 q of the real half and
// float4 q + NV4/2 of the imaginary half, i.e. both parts of the same four components.
//
// score(s, r, o) = Re(sum s r conj(o)) is linear in each argument:
//   score = <s, A> with A = d score / d s  (a function of r and o),
//   score = <o, C> with C = d score / d o  (a function of s and r).
// One workgroup per triple: every negative is one dot product with A (replaced subject) or C
// (replaced object); its own gradient is coef * A or coef * C; the triple's subject, object and
// relation gradients follow from the coefficient-weighted sums of the negatives' rows.
// Staged rows: [0,B) subject gradient, [B,2B) object gradient, [2B,3B) A, [3B,4B) C, [4B,5B) relation gradient.
// ------------------------------------------------------------------------------------------------
// out = d score / d s  given r (conjugate-linear pairing with o):  re = r_re o_re + r_im o_im ; im = r_re o_im - r_im o_re
template <int NV4>
__device__ __forceinline__ void grad_subject(Row<NV4> &out, const Row<NV4> &r, const Row<NV4> &o)
{
    constexpr int H = NV4 / 2;
#pragma unroll
    for (int q = 0; q < H; ++q) {
        const float4 rr = r.v[q], ri = r.v[q + H], orr = o.v[q], oi = o.v[q + H];
        out.v[q] = make_float4(rr.x * orr.x + ri.x * oi.x, rr.y * orr.y + ri.y * oi.y, rr.z * orr.z + ri.z * oi.z,
                               rr.w * orr.w + ri.w * oi.w);
        out.v[q + H] = make_float4(rr.x * oi.x - ri.x * orr.x, rr.y * oi.y - ri.y * orr.y, rr.z * oi.z - ri.z * orr.z,
                                   rr.w * oi.w - ri.w * orr.w);
    }
}

// out = d score / d o  given s, r:  re = s_re r_re - s_im r_im ; im = s_im r_re + s_re r_im
template <int NV4>
__device__ __forceinline__ void grad_object(Row<NV4> &out, const Row<NV4> &s, const Row<NV4> &r)
{
    constexpr int H = NV4 / 2;
#pragma unroll
    for (int q = 0; q < H; ++q) {
        const float4 sr = s.v[q], si = s.v[q + H], rr = r.v[q], ri = r.v[q + H];
        out.v[q] = make_float4(sr.x * rr.x - si.x * ri.x, sr.y * rr.y - si.y * ri.y, sr.z * rr.z - si.z * ri.z,
                               sr.w * rr.w - si.w * ri.w);
        out.v[q + H] = make_float4(si.x * rr.x + sr.x * ri.x, si.y * rr.y + sr.y * ri.y, si.z * rr.z + sr.z * ri.z,
                                   si.w * rr.w + sr.w * ri.w);
    }
}

// out += d score / d r  given s, o:  re = s_re o_re + s_im o_im ; im = s_re o_im - s_im o_re
template <int NV4>
__device__ __forceinline__ void add_grad_relation(Row<NV4> &out, const Row<NV4> &s, const Row<NV4> &o)
{
    constexpr int H = NV4 / 2;
#pragma unroll
    for (int q = 0; q < H; ++q) {
        const float4 sr = s.v[q], si = s.v[q + H], orr = o.v[q], oi = o.v[q + H];
        out.v[q].x += sr.x * orr.x + si.x * oi.x; out.v[q].y += sr.y * orr.y + si.y * oi.y;
        out.v[q].z += sr.z * orr.z + si.z * oi.z; out.v[q].w += sr.w * orr.w + si.w * oi.w;
        out.v[q + H].x += sr.x * oi.x - si.x * orr.x; out.v[q + H].y += sr.y * oi.y - si.y * orr.y;
        out.v[q + H].z += sr.z * oi.z - si.z * orr.z; out.v[q + H].w += sr.w * oi.w - si.w * orr.w;
    }
}

// GB = row groups per triple (GB * 16 threads); a workgroup of kBlock threads takes kBlock / (GB * 16) triples.
// IF = negative rows that a group has in flight.  The first sw.blocks workgroups prepare later steps instead.
//
// A negative whose entity nothing else accesses in this step (the plan flags it: a segment of one access) is
// updated right here: its row is in registers, its gradient is coef * direction, nobody else reads the row, so the
// AdaGrad step is exact under the step's snapshot semantics and the row is not read a second time by the update
// kernel, which skips these accesses.  With uniform negatives over millions of entities that is nearly all of them.
template <int NV4, int GB, int IF>
__global__ void __launch_bounds__(kBlock) k_kge_grad(float *E, const float *R, uint32_t n_ent, uint32_t n_rel,
                                                     int stride, const uint32_t *subj, const uint32_t *rel,
                                                     const uint32_t *obj, const uint32_t *negs, uint32_t B, int nh,
                                                     int nt, float *coefs, float *stage, double *loss,
                                                     float *E_state, const uint32_t *entity_rank, OptAdagrad opt,
                                                     SideWork sw)
{
    extern __shared__ float part_all[];   // [triples per workgroup][GB][stride]: per-group weighted row sums
    __shared__ float lds[kBlock / 64];
    if (side_work_block(sw)) return;
    constexpr int kHalf = GB / 2;
    constexpr int kTriples = kBlock / (GB * kGroup);
    static_assert(GB >= 8 && GB % 8 == 0, "whole wavefronts per role, at least five groups for the last stage");
    static_assert(kTriples >= 1 && kBlock % (GB * kGroup) == 0, "whole triples per workgroup");
    const int lane = threadIdx.x & (kGroup - 1), group = (threadIdx.x / kGroup) % GB, which = threadIdx.x / (GB * kGroup);
    const uint32_t e_raw = (blockIdx.x - sw.blocks) * kTriples + which;
    const bool active = e_raw < B;      // a workgroup's last triples may be beyond the batch: they repeat triple B - 1
    const uint32_t e = active ? e_raw : B - 1;   // and write nothing
    float *part = part_all + (size_t)which * GB * stride;
    const int nn = nh + nt;
    // The first half of the groups scores the replaced subjects (dot products with A), the second half the
    // replaced objects (with C).  Group number gi of a role takes that role's negatives gi, gi + kHalf, ...;
    // lane l of the group fetches the key of the l-th of them up front, so that the row reads wait for no index.
    const bool head = group < kHalf;
    const int gi = group % kHalf;
    const int lo = head ? 0 : nh, cnt = head ? nh : nt;
    const int mine = cnt > gi ? (cnt - gi + kHalf - 1) / kHalf : 0;
    const uint32_t *my_negs = negs + (size_t)e * nn + lo + gi;
    const uint32_t *my_rank = entity_rank + (size_t)2 * B + (size_t)e * nn + lo + gi;   // negatives follow s and o
    uint32_t early = 0u, early_alone = 0u;
    if (lane < mine) {
        const uint32_t raw = my_negs[(size_t)lane * kHalf];
        early = min(raw, n_ent - 1);
        early_alone = (active && raw < n_ent && (my_rank[(size_t)lane * kHalf] & kSingleAccess)) ? 1u : 0u;
    }
    const float *s_ptr = E + (size_t)min(subj[e], n_ent - 1) * stride;
    const float *o_ptr = E + (size_t)min(obj[e], n_ent - 1) * stride;
    const float *r_ptr = R + (size_t)min(rel[e], n_rel - 1) * stride;
    Row<NV4> dir;
    {
        Row<NV4> s, r, o;
        load_row(r, r_ptr, lane);
        if (head) { load_row(o, o_ptr, lane); grad_subject<NV4>(dir, r, o); }
        else { load_row(s, s_ptr, lane); grad_object<NV4>(dir, s, r); }
    }
    Row<NV4> wsum;                     // sum of coef * negative row over this group's negatives
    zero_row(wsum);
    float loss_acc = 0.f;
    for (int j0 = 0; j0 < mine; j0 += IF) {
        Row<NV4> x[IF], gs[IF];
        uint32_t key[IF];
        bool alone[IF];
#pragma unroll
        for (int k = 0; k < IF; ++k) {
            const int j = j0 + k;
            alone[k] = false;
            if (j < mine) {
                if (j < kGroup) {
                    key[k] = __shfl(early, j, kGroup);
                    alone[k] = __shfl(early_alone, j, kGroup) != 0u;
                } else {
                    const uint32_t raw = my_negs[(size_t)j * kHalf];
                    key[k] = min(raw, n_ent - 1);
                    alone[k] = active && raw < n_ent && (my_rank[(size_t)j * kHalf] & kSingleAccess);
                }
                load_row(x[k], E + (size_t)key[k] * stride, lane);
                if (alone[k]) load_row(gs[k], E_state + (size_t)key[k] * stride, lane);
            }
        }
#pragma unroll
        for (int k = 0; k < IF; ++k) {
            const int j = j0 + k;
            if (j < mine) {
                const float phi = group_sum(partial_dot(x[k], dir));
                const float g = sigmoidf(phi);           // label -1: d softplus(phi) / d phi
                loss_acc += softplusf(phi);
                if (active && lane == 0) coefs[(size_t)e * nn + lo + gi + j * kHalf] = g;
                axpy_row(wsum, g, x[k]);                 // the row as it was at the start of the step
                if (alone[k]) {                          // its whole update: gradient g * direction
                    Row<NV4> delta;
                    zero_row(delta);
                    axpy_row(delta, g, dir);
                    float *row = E + (size_t)key[k] * stride, *state_row = E_state + (size_t)key[k] * stride;
                    opt.template finish<NV4>(x[k], gs[k], row, state_row, delta, lane);
                }
            }
        }
    }
    store_row(part + (size_t)group * stride, wsum, lane);
    __syncthreads();
    if (group < 5 && active) {
        Row<NV4> s, r, o, A;
        load_row(s, s_ptr, lane);
        load_row(r, r_ptr, lane);
        load_row(o, o_ptr, lane);
        grad_subject<NV4>(A, r, o);
        const float phi = group_sum(partial_dot(s, A));
        const float gp = -sigmoidf(-phi);            // label +1: d softplus(-phi) / d phi
        if (group == 0) loss_acc += softplusf(-phi);
        // weighted sums of the replaced-subject rows (first half of the groups) and replaced-object rows, fixed order
        Row<NV4> ws, wo;
        zero_row(ws);
        zero_row(wo);
        if (group == 1 || group == 4)
            for (int g2 = 0; g2 < kHalf; ++g2) {
                Row<NV4> t;
                load_row(t, part + (size_t)g2 * stride, lane);
                axpy_row(ws, 1.0f, t);
            }
        if (group == 0 || group == 4)
            for (int g2 = kHalf; g2 < GB; ++g2) {
                Row<NV4> t;
                load_row(t, part + (size_t)g2 * stride, lane);
                axpy_row(wo, 1.0f, t);
            }
        Row<NV4> out;
        if (group == 0) {            // subject gradient: d score/d s is linear in o
            axpy_row(wo, gp, o);
            grad_subject<NV4>(out, r, wo);
            store_row(stage + (size_t)e * stride, out, lane);
        } else if (group == 1) {     // object gradient: linear in s
            axpy_row(ws, gp, s);
            grad_object<NV4>(out, ws, r);
            store_row(stage + ((size_t)B + e) * stride, out, lane);
        } else if (group == 2) {
            store_row(stage + ((size_t)2 * B + e) * stride, A, lane);
        } else if (group == 3) {
            grad_object<NV4>(out, s, r);
            store_row(stage + ((size_t)3 * B + e) * stride, out, lane);
        } else {                     // relation gradient: bilinear in (s, o)
            zero_row(out);
            axpy_row(wo, gp, o);
            add_grad_relation<NV4>(out, s, wo);      // positive + replaced objects (subject fixed)
            add_grad_relation<NV4>(out, ws, o);      // replaced subjects (object fixed)
            store_row(stage + ((size_t)4 * B + e) * stride, out, lane);
        }
    }
    block_add_loss((active && lane == 0) ? loss_acc : 0.f, loss, lds);
}

template <int NV4>
static void launch_kge_grad(nups_ctx *ctx, const nups_batch &b, const Plan &entity_plan, const SideWork &sw,
                            size_t side_lds)
{
    // Eight groups per triple, two negative rows in flight per group.  More groups per triple or more rows in
    // flight change nothing: the kernel runs at the speed at which memory delivers the negatives' rows.
    constexpr int GB = 8, IF = 2;
    constexpr int kTriples = kBlock / (GB * kGroup);
    const Table &te = ctx->tab[0], &tr = ctx->tab[1];
    const size_t lds = std::max(sizeof(float) * kTriples * GB * (size_t)te.stride, side_lds);
    const uint32_t blocks = (uint32_t)((b.B + kTriples - 1) / kTriples);
    hipLaunchKernelGGL((k_kge_grad<NV4, GB, IF>), dim3(sw.blocks + blocks), dim3(kBlock), lds, ctx->stream, te.data,
                       (const float *)tr.data, (uint32_t)te.num_keys, (uint32_t)tr.num_keys, te.stride, b.k0, b.k1,
                       b.k2, b.negs, (uint32_t)b.B, (int)b.n_neg, (int)b.n_neg2, ctx->coef, ctx->stage, ctx->loss_cur,
                       te.state, (const uint32_t *)entity_plan.a.rank, OptAdagrad{b.lr, b.eps}, sw);
}

nups_status plan_step_kge(nups_ctx *ctx, nups_prepared &p)
{
    const nups_batch &b = p.batch;
    const uint32_t B = (uint32_t)b.B, nn = (uint32_t)(b.n_neg + b.n_neg2);
    if (ctx->replicas > 0)
        return fail(NUPS_ERR_UNIMPLEMENTED, "NUPS_TASK_KGE has no replicas (AdaGrad state): switch nups_set_replicas off");
    if (ctx->tab[0].stride % 128 != 0 || ctx->tab[0].stride > 512)
        return fail(NUPS_ERR_UNIMPLEMENTED, "KGE tables need a row_stride of 128, 256, 384 or 512 floats");
    return plan_two_tables(ctx, p, KeySource{{b.k0, b.k2, b.negs}, {B, B, B * nn}}, B * (2 + nn),
                           KeySource{{b.k1, nullptr, nullptr}, {B, 0, 0}}, B);
}

nups_status run_step_kge(nups_ctx *ctx, nups_prepared &p)
{
    const nups_batch &b = p.batch;
    Table &te = ctx->tab[0], &tr = ctx->tab[1];
    const uint32_t B = (uint32_t)b.B, nh = (uint32_t)b.n_neg, nn = (uint32_t)(b.n_neg + b.n_neg2);
    nups_status st;
    if ((st = ensure_f32(&ctx->coef, &ctx->coef_cap, (size_t)B * nn + 1, ctx->stream)) != NUPS_OK) return st;
    if ((st = ensure_f32(&ctx->stage, &ctx->stage_cap, (size_t)5 * B * te.stride, ctx->stream)) != NUPS_OK) return st;
    ctx->loss_cur = p.loss_dev;   // zeroed by the step's plan construction
    if (B == 0) return NUPS_OK;
    size_t side_lds = 0;
    {
        const SideWork sw = take_side_work(ctx, &side_lds, kSideWgsWide);
        PhaseScope scope(ctx, NUPS_PHASE_GRAD, ctx->stream);
        switch (te.stride / 64) {
        case 2: launch_kge_grad<2>(ctx, b, p.plan[0], sw, side_lds); break;
        case 4: launch_kge_grad<4>(ctx, b, p.plan[0], sw, side_lds); break;
        case 6: launch_kge_grad<6>(ctx, b, p.plan[0], sw, side_lds); break;
        case 8: launch_kge_grad<8>(ctx, b, p.plan[0], sw, side_lds); break;
        default: return fail(NUPS_ERR_UNIMPLEMENTED, "KGE row_stride");
        }
        NUPS_HIP(hipGetLastError());
    }
    {
        const SideWork sw = take_side_work(ctx, &side_lds, kSideWgsWide);
        PhaseScope scope(ctx, NUPS_PHASE_APPLY0, ctx->stream);
        const TableUpdate<SrcKgeEntity, OptAdagrad> ue{&p.plan[0], partial_of(ctx, p, 0), te.data, te.state,
                                                       SrcKgeEntity{ctx->stage, ctx->coef, B, nn, nh},
                                                       OptAdagrad{b.lr, b.eps}};
        const TableUpdate<SrcStaged, OptAdagrad> ur{&p.plan[1], partial_of(ctx, p, 1), tr.data, tr.state,
                                                    SrcStaged{ctx->stage + (size_t)4 * B * te.stride},
                                                    OptAdagrad{b.lr, b.eps}};
        if ((st = launch_apply2(ctx->stream, te.stride, ue, ur, update_scratch(ctx, te.stride), sw, side_lds)) != NUPS_OK) return st;
    }
    return NUPS_OK;
}

}  // namespace nups

// ------------------------------------------------------------------------------------------------
// nups_push_static: the push for callers that cannot allocate.  Everything that nups_push keeps in allocated
// workspace (the scratch maps and result arrays of the per-key structure, the partial rows of chunked segments)
// lives in one file-scope device array of a fixed size.  Host code never uses the array's name as an address: the
// address of a device's copy is asked for once (static_scratch_setup) and kept per device.
// ------------------------------------------------------------------------------------------------
namespace nups {

constexpr size_t kStaticKeys = NUPS_STATIC_MAX_KEYS, kStaticPush = NUPS_STATIC_MAX_PUSH;
constexpr size_t kStaticWordsOfMap = (kStaticKeys + 31) / 32;
constexpr size_t kStaticChunks = kStaticPush / kChunk + kStaticPush / (kLongSegment + 1) + 2;   // max_chunks(kStaticPush)
constexpr size_t kStaticTiles = (kStaticWordsOfMap > kStaticPush ? kStaticWordsOfMap : kStaticPush) / kScanTile + 1;
constexpr uint32_t kStaticGrid = 128;   // workgroups of the update launch (its running totals are part of the array)
constexpr size_t align64(size_t words) { return (words + 63) / 64 * 64; }   // regions start on 256-byte boundaries

// Offsets (in 32-bit words) of the regions.  The first kStaticZeroWords words are what a build expects to be zero.
struct StaticLayout {
    size_t bytemap, wordmap, cnt_work, chunk_done, meta, zero_end, bitmap, word_rank, tile_sum, tile_prefix, uniq, count,
        seg, perm, perm_sorted, perm_pieces, slot, pos, rank, chunk_of, partial, totals, end;
};

constexpr StaticLayout static_layout()
{
    StaticLayout l{};
    size_t at = 0;
    auto take = [&at](size_t words) { const size_t start = at; at += align64(words); return start; };
    l.bytemap = take(kStaticWordsOfMap * 8);
    l.wordmap = take((kStaticWordsOfMap + 3) / 4);
    l.cnt_work = take((kStaticPush + kScanTile - 1) / kScanTile * kScanTile);
    l.chunk_done = take(kStaticChunks);
    l.meta = take(kMetaWords);
    l.zero_end = at;
    l.bitmap = take(kStaticWordsOfMap);
    l.word_rank = take(kStaticWordsOfMap);
    l.tile_sum = take(kStaticTiles);
    l.tile_prefix = take(kStaticTiles);
    l.uniq = take(kStaticPush);
    l.count = take(kStaticPush);
    l.seg = take(kStaticPush + 1);
    l.perm = take(kStaticPush);
    l.perm_sorted = take(kStaticPush);
    l.perm_pieces = take(kStaticPush);
    l.slot = take(kStaticPush);
    l.pos = take(kStaticPush);
    l.rank = take(kStaticPush);
    l.chunk_of = take(4 * kStaticChunks);
    l.partial = take(kStaticChunks * (size_t)kMaxStride);
    l.totals = take((size_t)kStaticGrid * kGroupsPerBlock * kMaxStride);
    l.end = at;
    return l;
}

constexpr StaticLayout kStaticLayout = static_layout();

static __device__ __align__(256) uint32_t scratch[kStaticLayout.end];   // about 14 MB per device, for the life of the process

constexpr int kMaxDevices = 64;
static uint32_t *g_scratch_of_device[kMaxDevices];   // device address of each device's copy; null: not asked for yet
static std::mutex g_scratch_mutex;

nups_status static_scratch_setup(int device)
{
    if (device < 0 || device >= kMaxDevices) return fail(NUPS_ERR_DEVICE, "device ordinal out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_of_device[device]) return NUPS_OK;
    uint32_t *ptr = nullptr;
    NUPS_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));   // of the current device's copy
    if (!ptr) return fail(NUPS_ERR_DEVICE, "no address for the static scratch");
    g_scratch_of_device[device] = ptr;
    return NUPS_OK;
}

__global__ void __launch_bounds__(kBlock) k_fill_zero(uint32_t *words, uint32_t n)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i < n) words[i] = 0u;
}

}  // namespace nups

extern "C" nups_status nups_push_static(nups_ctx *ctx, int table, const uint32_t *keys_dev, int64_t n,
                                        const float *updates_dev)
{
    using namespace nups;
    if (!ctx || table < 0 || table >= ctx->n_tables) return fail(NUPS_ERR_ARG, "nups_push_static: bad context or table");
    if (n < 0 || (n > 0 && (!keys_dev || !updates_dev))) return fail(NUPS_ERR_ARG, "nups_push_static: bad arguments");
    Table &t = ctx->tab[table];
    if (t.replica_rows) return fail(NUPS_ERR_STATE, "nups_push_static: the table has replicas of its hot keys");
    if (n > (int64_t)kStaticPush)
        return fail(NUPS_ERR_ARG, "nups_push_static: at most NUPS_STATIC_MAX_PUSH keys per call (use nups_push)");
    if (t.num_keys > (int64_t)kStaticKeys)
        return fail(NUPS_ERR_ARG, "nups_push_static: tables of at most NUPS_STATIC_MAX_KEYS keys (use nups_push)");
    uint32_t *base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        base = (ctx->device >= 0 && ctx->device < kMaxDevices) ? g_scratch_of_device[ctx->device] : nullptr;
    }
    if (!base) return fail(NUPS_ERR_STATE, "nups_push_static: the static scratch of this device was not set up");
    if (!ctx->static_push) {          // host-side object only
        ctx->static_push = new nups_prepared();
        ctx->static_push->ctx = ctx;
    }
    nups_prepared *p = ctx->static_push;
    constexpr StaticLayout L = kStaticLayout;
    Plan &pl = p->plan[0];
    PlanArgs &a = pl.a;
    a.bytemap = (uint8_t *)(base + L.bytemap);
    a.wordmap = (uint8_t *)(base + L.wordmap);
    a.cnt_work = base + L.cnt_work;
    a.chunk_done = base + L.chunk_done;
    a.meta = base + L.meta;
    a.bitmap = base + L.bitmap;
    a.word_rank = base + L.word_rank;
    a.tile_sum = base + L.tile_sum;
    a.tile_prefix = base + L.tile_prefix;
    a.uniq = base + L.uniq;
    a.count = base + L.count;
    a.seg = base + L.seg;
    a.perm = base + L.perm;
    a.perm_sorted = base + L.perm_sorted;
    a.perm_pieces = base + L.perm_pieces;
    a.slot = base + L.slot;
    a.pos = base + L.pos;
    a.rank = base + L.rank;
    a.chunk_of = reinterpret_cast<uint4 *>(base + L.chunk_of);   // regions start on 256-byte boundaries
    pl.cap_n = kStaticPush;
    pl.cap_words = kStaticWordsOfMap;
    pl.cap_tiles = kStaticTiles;
    pl.table = table;
    p->n_plans = 1;
    set_plan_shape(ctx, t, pl);
    a.src = KeySource{{keys_dev, nullptr, nullptr}, {(uint32_t)n, 0, 0}};
    a.n = a.mark_n = (uint32_t)n;
    a.zero_loss = nullptr;
    // The array is shared by every call on this device and keeps the last call's contents: what a build expects
    // to be zero is cleared first, by a kernel (a memset node would not do for callers that capture the stream).
    hipLaunchKernelGGL(k_fill_zero, dim3((uint32_t)((L.zero_end + kBlock - 1) / kBlock)), dim3(kBlock), 0, ctx->stream, base,
                       (uint32_t)L.zero_end);
    NUPS_HIP(hipGetLastError());
    build_phases(*p, SampleArgs{}, -1);
    nups_status st = flush_side_work(ctx, p);
    if (st == NUPS_OK && n > 0)
        st = launch_push_apply(ctx, t, pl, (float *)(base + L.partial), (float *)(base + L.totals), kStaticGrid, updates_dev);
    t.last_plan = &pl;                // nups_debug_structure describes this call until the next step or push
    return st;
}
