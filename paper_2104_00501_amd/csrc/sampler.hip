// Sampling access (Sections 4.3, 4.4): device kernels that draw the sample keys of one
// PrepareSample call under the four schemes, and the host-side alias-table build.
#include <cmath>

#include "device_utils.h"

namespace nups {

struct DistArgs {
    const uint32_t *thresh;   // null: uniform target distribution
    const uint32_t *alias;
    uint64_t num_keys;
    uint64_t seed;
    uint32_t dist;
};

// One fresh draw from pi: bucket = floor((x0 + 2^32 x1) * V / 2^64); keep it if x2 < thresh[bucket].
__device__ __forceinline__ uint32_t fresh_key(const DistArgs &d, uint64_t step, uint64_t draw)
{
    const Words w = draw_words(d.seed, kStreamFresh, d.dist, step, draw);
    const uint64_t u = (uint64_t)w.x0 | ((uint64_t)w.x1 << 32);
    const uint32_t b = (uint32_t)__umul64hi(u, d.num_keys);
    if (d.thresh == nullptr) return b;
    return (w.x2 < d.thresh[b]) ? b : d.alias[b];
}

// Independent sampling: sample i is draw draw0 + i of the step.
__global__ void __launch_bounds__(kBlock) k_sample_fresh(DistArgs d, uint64_t step, uint64_t draw0, uint32_t n,
                                                         uint32_t *out)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i < n) out[i] = fresh_key(d, step, draw0 + i);
}

// Sample reuse: one workgroup emits one pass over one pool.  The order of the pass is the
// ascending order of (first ORDER-stream word at (fresh id, pass), slot); rank by counting.
__global__ void __launch_bounds__(kBlock) k_sample_pool_pass(DistArgs d, uint64_t step, uint32_t F, uint32_t G,
                                                             uint32_t U, uint32_t N, uint32_t *out)
{
    __shared__ uint32_t word[1024];
    const uint32_t pool = blockIdx.x / U, pass = blockIdx.x % U;
    const uint32_t first = pool * G;
    const uint32_t g = min(G, F - first);
    // position of this pass in the sequence: full pools emit U * G samples each
    const uint64_t base = (uint64_t)pool * U * G + (uint64_t)pass * g;
    if (base >= N) return;
    for (uint32_t i = threadIdx.x; i < g; i += kBlock)
        word[i] = draw_words(d.seed, kStreamOrder, d.dist, step, (uint64_t)(first + i) | ((uint64_t)pass << 32)).x0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < g; i += kBlock) {
        const uint32_t w = word[i];
        uint32_t rank = 0;
        for (uint32_t j = 0; j < g; ++j) {
            const uint32_t wj = word[j];
            rank += (wj < w || (wj == w && j < i)) ? 1u : 0u;
        }
        const uint64_t pos = base + rank;
        if (pos < N) out[pos] = fresh_key(d, step, first + i);   // every pass redraws the pool's keys itself
    }
}

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x85EBCA6Bu;
    x ^= x >> 13; x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

// Sample reuse over a long-lived pool: sample at global position g is slot perm(rank) of the pool
// of its epoch, perm a four-round Feistel permutation of 0..P-1 (cycle walking) keyed per pass.
__global__ void __launch_bounds__(kBlock) k_sample_longterm(DistArgs d, uint64_t P, uint32_t R, uint64_t cursor,
                                                            uint32_t n, int half, uint32_t *out)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint64_t g = cursor + i;
    const uint64_t per_epoch = P * (uint64_t)R;
    const uint64_t epoch = g / per_epoch, within = g % per_epoch;
    const uint64_t pass = within / P;
    uint64_t x = within % P;
    const uint32_t mask = (half >= 32) ? 0xFFFFFFFFu : ((1u << half) - 1u);
    const Words k = draw_words(d.seed, kStreamRoundKey, d.dist, epoch, pass);
    const uint32_t rk[4] = {k.x0, k.x1, k.x2, k.x3};
    do {   // ends: the walk follows a cycle of a permutation of the 2^(2 half) domain that contains x < P
        uint32_t L = (uint32_t)(x >> half) & mask, Rr = (uint32_t)x & mask;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t nR = L ^ (mix32(Rr ^ rk[t]) & mask);
            L = Rr; Rr = nR;
        }
        x = ((uint64_t)L << half) | Rr;
    } while (x >= P);
    out[i] = fresh_key(d, epoch, x);
}

// Direct-access repurposing: sample p takes the key that a uniformly chosen example of its tile contributes.
__global__ void __launch_bounds__(kBlock) k_sample_local(const uint32_t *keys_a, const uint32_t *keys_b,
                                                         uint32_t n_examples, uint32_t per_example, uint32_t split,
                                                         uint32_t tile, uint64_t seed, uint32_t dist, uint64_t step,
                                                         uint32_t n, uint32_t *out)
{
    const uint32_t p = blockIdx.x * kBlock + threadIdx.x;
    if (p >= n) return;
    const uint32_t e = p / per_example;
    const uint32_t base = (e / tile) * tile;
    const uint32_t t = min(tile, n_examples - base);
    const Words w = draw_words(seed, kStreamLocal, dist, step, p);
    const uint32_t pick = base + __umulhi(w.x0, t);
    out[p] = ((p % per_example) < split) ? keys_a[pick] : keys_b[pick];
}

static int feistel_half_bits(uint64_t P)
{
    int half = 1;
    while (half < 32 && ((uint64_t)1 << (2 * half)) < P) ++half;
    return half;
}

SampleSpec sample_spec(const nups_dist *d)
{
    SampleSpec sp{};
    sp.scheme = d->scheme;
    sp.thresh = d->uniform ? nullptr : d->thresh_dev;
    sp.alias = d->alias_dev;
    sp.num_keys = (uint64_t)d->ctx->tab[d->table].num_keys;
    sp.seed = d->seed;
    sp.cursor = d->cursor;
    sp.dist_id = d->id;
    sp.U = d->U; sp.G = d->G; sp.R = d->R; sp.P = d->P;
    sp.local_a = d->local_a; sp.local_b = d->local_b; sp.local_n = d->local_n;
    sp.per_example = d->per_example; sp.split = d->split; sp.tile = d->tile;
    return sp;
}

// Enqueues the drawing of n_samples keys on `stream`.
nups_status launch_sample(nups_ctx *ctx, hipStream_t stream, const SampleSpec &d, uint32_t *keys_out, int64_t n_samples,
                          uint64_t step)
{
    const uint32_t n = (uint32_t)n_samples;
    if (n == 0) return NUPS_OK;
    PhaseScope scope(ctx, NUPS_PHASE_SAMPLE, stream);
    DistArgs a{d.thresh, d.alias, d.num_keys, d.seed, d.dist_id};
    const uint32_t blocks = (n + kBlock - 1) / kBlock;
    switch (d.scheme) {
    case NUPS_CONFORM:
        hipLaunchKernelGGL(k_sample_fresh, dim3(blocks), dim3(kBlock), 0, stream, a, step, (uint64_t)0, n,
                           keys_out);
        break;
    case NUPS_BOUNDED: {
        const uint32_t U = (uint32_t)d.U, G = (uint32_t)d.G;
        const uint32_t F = (n + U - 1) / U;
        const uint32_t pools = (F + G - 1) / G;
        hipLaunchKernelGGL(k_sample_pool_pass, dim3(pools * U), dim3(kBlock), 0, stream, a, step, F, G, U, n,
                           keys_out);
        break;
    }
    case NUPS_LONGTERM:
        hipLaunchKernelGGL(k_sample_longterm, dim3(blocks), dim3(kBlock), 0, stream, a, (uint64_t)d.P,
                           (uint32_t)d.R, d.cursor, n, feistel_half_bits((uint64_t)d.P), keys_out);
        break;
    case NUPS_NONCONFORM:
        hipLaunchKernelGGL(k_sample_local, dim3(blocks), dim3(kBlock), 0, stream, d.local_a, d.local_b,
                           (uint32_t)d.local_n, (uint32_t)d.per_example, (uint32_t)d.split, (uint32_t)d.tile,
                           d.seed, d.dist_id, step, n, keys_out);
        break;
    default:
        return fail(NUPS_ERR_ARG, "unknown sampling scheme");
    }
    NUPS_HIP(hipGetLastError());
    return NUPS_OK;
}

}  // namespace nups

// Alias table of pi_k = w_k / sum(w) (Walker's method in Vose's formulation).  The order of
// operations is part of the definition so that any two builds agree bit for bit: masses are
// (w_k / sum) * V with the sum taken in key order; keys below one go on a "small" stack, the
// others on a "large" stack, both filled in ascending key order and popped from the back; the
// large key donates to the small bucket, keeps (q_l + q_s) - 1 and is pushed back where its new
// mass belongs; leftovers keep themselves.  Thresholds are floor(mass * 2^32), saturated.
extern "C" nups_status nups_build_alias_table(const double *w, int64_t V, uint32_t *thresh, uint32_t *alias)
{
    using namespace nups;
    if (!w || !thresh || !alias) return fail(NUPS_ERR_ARG, "nups_build_alias_table: null pointer");
    if (V <= 0 || V > 0xFFFFFFFFll) return fail(NUPS_ERR_ARG, "nups_build_alias_table: num_keys out of range");
    double sum = 0.0;
    for (int64_t k = 0; k < V; ++k) {
        if (!(w[k] >= 0.0) || std::isinf(w[k]))
            return fail(NUPS_ERR_ARG, "nups_build_alias_table: weights must be finite and non-negative");
        sum += w[k];
    }
    if (!(sum > 0.0) || std::isinf(sum)) return fail(NUPS_ERR_ARG, "nups_build_alias_table: weights sum to zero");
    std::vector<double> q((size_t)V);
    std::vector<uint32_t> small, large;
    small.reserve((size_t)V);
    large.reserve((size_t)V);
    for (int64_t k = 0; k < V; ++k) {
        const double p = w[k] / sum;
        q[(size_t)k] = p * (double)V;
        (q[(size_t)k] < 1.0 ? small : large).push_back((uint32_t)k);
    }
    std::vector<double> keep((size_t)V, 1.0);
    for (int64_t k = 0; k < V; ++k) alias[k] = (uint32_t)k;
    while (!small.empty() && !large.empty()) {
        const uint32_t s = small.back(); small.pop_back();
        const uint32_t l = large.back(); large.pop_back();
        keep[s] = q[s];
        alias[s] = l;
        const double donated = q[l] + q[s];
        q[l] = donated - 1.0;
        (q[l] < 1.0 ? small : large).push_back(l);
    }
    for (int64_t k = 0; k < V; ++k) {
        const double t = std::floor(keep[(size_t)k] * 4294967296.0);
        thresh[k] = t >= 4294967295.0 ? 0xFFFFFFFFu : (t <= 0.0 ? 0u : (uint32_t)t);
    }
    return NUPS_OK;
}
