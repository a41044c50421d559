// Sampling access (Sections 4.3, 4.4), host side: the description of one drawing that the device code
// (side_work.h) works from, and the alias-table build.
#include <cmath>

#include "nups_internal.h"

namespace nups {

static int feistel_half_bits(uint64_t P)
{
    int half = 1;
    while (half < 32 && ((uint64_t)1 << (2 * half)) < P) ++half;
    return half;
}

// Device-side description of the drawing of n_samples keys from d for step `step` (Section 4.4 schemes), taken
// from the distribution as it is now.  The caller advances a LONG-TERM cursor.
SampleArgs sample_args(const nups_dist *d, uint32_t *keys_out, int64_t n_samples, uint64_t step)
{
    SampleArgs a{};
    const uint32_t n = (uint32_t)n_samples;
    if (n == 0) return a;                 // scheme 0: nothing to draw
    a.scheme = (int32_t)d->scheme;
    a.thresh = d->uniform ? nullptr : d->thresh_dev;
    a.alias = d->alias_dev;
    a.num_keys = (uint64_t)d->ctx->tab[d->table].num_keys;
    a.seed = d->seed;
    a.step = step;
    a.cursor = d->cursor;
    a.P = (uint64_t)d->P;
    a.dist_id = d->id;
    a.n = n;
    a.U = (uint32_t)d->U;
    a.G = (uint32_t)d->G;
    a.R = (uint32_t)d->R;
    a.half = feistel_half_bits((uint64_t)d->P);
    a.local_a = d->local_a;
    a.local_b = d->local_b;
    a.local_n = (uint32_t)d->local_n;
    a.per_example = (uint32_t)d->per_example;
    a.split = (uint32_t)d->split;
    a.tile = (uint32_t)d->tile;
    a.out = keys_out;
    a.error_flag = d->ctx->error_flag;
    a.blocks = (n + kBlock - 1) / kBlock;
    if (d->scheme == NUPS_BOUNDED) {      // one workgroup per (pool, pass)
        a.F = (n + a.U - 1) / a.U;
        a.blocks = (a.F + a.G - 1) / a.G * a.U;
    }
    return a;
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
