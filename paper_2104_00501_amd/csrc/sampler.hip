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

// ---- sample reuse with postponing (Section 4.4), within the samples of one handle -------------------------------
// A sample whose key is not resident when the walk through the handle reaches it goes to the end of the handle's
// samples, once, and its key counts as resident from then on.  In closed form: the samples that move are exactly
// the first occurrences, within the handle, of the keys that are not resident at the start; the others keep their
// order in front, the moved ones follow in the order in which they were met.  Three passes over the raw samples:
// first occurrence per key (atomic minimum of the position), number of moving samples per tile of kBlock, and,
// after a scan of those numbers, the scatter to the final positions.
__device__ __forceinline__ bool resident_key(uint32_t key, const uint32_t *hot_bits)
{
    return hot_bits != nullptr && ((hot_bits[key >> 5] >> (key & 31)) & 1u) != 0;
}

__global__ void __launch_bounds__(kBlock)
k_postpone_first(const uint32_t *__restrict__ raw, uint32_t n, const uint32_t *__restrict__ hot_bits,
                 uint32_t num_keys, uint32_t *__restrict__ first_pos)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint32_t key = raw[i];
    if (key < num_keys && !resident_key(key, hot_bits)) atomicMin(&first_pos[key], i);
}

// Whether sample i moves, and (exclusive) how many samples of its tile before it move; the tile's total in *total.
__device__ __forceinline__ bool moves_and_rank(const uint32_t *raw, uint32_t n, const uint32_t *hot_bits,
                                               uint32_t num_keys, const uint32_t *first_pos, uint32_t i,
                                               uint32_t *key_out, uint32_t *rank, uint32_t *total)
{
    __shared__ uint32_t wave_count[kBlock / 64];
    const uint32_t key = i < n ? raw[i] : 0u;
    const bool moves = i < n && key < num_keys && !resident_key(key, hot_bits) && first_pos[key] == i;
    const uint64_t votes = __ballot(moves);
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    if (lane == 0) wave_count[wave] = (uint32_t)__popcll(votes);
    __syncthreads();
    uint32_t before = (uint32_t)__popcll(votes & (((uint64_t)1 << lane) - 1));
    uint32_t all = 0;
    for (uint32_t w = 0; w < kBlock / 64; ++w) {
        if (w < wave) before += wave_count[w];
        all += wave_count[w];
    }
    *key_out = key;
    *rank = before;
    *total = all;
    return moves;
}

__global__ void __launch_bounds__(kBlock)
k_postpone_count(const uint32_t *__restrict__ raw, uint32_t n, const uint32_t *__restrict__ hot_bits,
                 uint32_t num_keys, const uint32_t *__restrict__ first_pos, uint32_t *__restrict__ tile_counts)
{
    uint32_t key, rank, total;
    (void)moves_and_rank(raw, n, hot_bits, num_keys, first_pos, blockIdx.x * kBlock + threadIdx.x, &key, &rank, &total);
    if (threadIdx.x == 0) tile_counts[blockIdx.x] = total;
}

// One workgroup: tile_counts[0 .. tiles) become their exclusive prefix sums, tile_counts[tiles] the total.
__global__ void __launch_bounds__(kBlock) k_postpone_scan(uint32_t *__restrict__ tile_counts, uint32_t tiles)
{
    __shared__ uint32_t part[kBlock];
    uint32_t carry = 0;
    for (uint32_t base = 0; base < tiles; base += kBlock) {
        const uint32_t t = base + threadIdx.x;
        const uint32_t mine = t < tiles ? tile_counts[t] : 0u;
        part[threadIdx.x] = mine;
        __syncthreads();
        for (uint32_t step = 1; step < kBlock; step <<= 1) {
            const uint32_t add = threadIdx.x >= step ? part[threadIdx.x - step] : 0u;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        if (t < tiles) tile_counts[t] = carry + part[threadIdx.x] - mine;
        carry += part[kBlock - 1];
        __syncthreads();
    }
    if (threadIdx.x == 0) tile_counts[tiles] = carry;
}

__global__ void __launch_bounds__(kBlock)
k_postpone_scatter(const uint32_t *__restrict__ raw, uint32_t n, const uint32_t *__restrict__ hot_bits,
                   uint32_t num_keys, uint32_t *__restrict__ first_pos, const uint32_t *__restrict__ tile_counts,
                   uint32_t tiles, uint32_t *__restrict__ out)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    uint32_t key, rank, total;
    const bool moves = moves_and_rank(raw, n, hot_bits, num_keys, first_pos, i, &key, &rank, &total);
    if (i >= n) return;
    const uint32_t before = tile_counts[blockIdx.x] + rank;     // moving samples ahead of this one
    const uint32_t moving = tile_counts[tiles];
    out[moves ? (n - moving) + before : i - before] = key;
    // back to "not seen" for the next handle; positions of the same key elsewhere compare unequal to either value
    if (moves) first_pos[key] = 0xFFFFFFFFu;
}

nups_status launch_postpone(nups_dist *d, const uint32_t *raw, uint32_t *out, int64_t n_samples)
{
    nups_ctx *ctx = d->ctx;
    const uint32_t n = (uint32_t)n_samples;
    if (n == 0) return NUPS_OK;
    const uint32_t tiles = (n + kBlock - 1) / kBlock;
    if (d->tile_cap < (size_t)tiles + 1) {
        hipError_t e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess && d->tile_counts_dev) e = hipFree(d->tile_counts_dev);
        d->tile_counts_dev = nullptr;
        d->tile_cap = (size_t)tiles + (size_t)tiles / 4 + 64;
        if (e == hipSuccess) e = hipMalloc((void **)&d->tile_counts_dev, sizeof(uint32_t) * d->tile_cap);
        if (e != hipSuccess) {
            d->tile_cap = 0;
            hip_ok(e, "sample reuse with postponing: tile counters");
            return NUPS_ERR_DEVICE;
        }
    }
    const Table &t = ctx->tab[d->table];
    const uint32_t V = (uint32_t)t.num_keys;
    k_postpone_first<<<tiles, kBlock, 0, ctx->stream>>>(raw, n, t.hot_bits_dev, V, d->first_pos_dev);
    k_postpone_count<<<tiles, kBlock, 0, ctx->stream>>>(raw, n, t.hot_bits_dev, V, d->first_pos_dev, d->tile_counts_dev);
    k_postpone_scan<<<1, kBlock, 0, ctx->stream>>>(d->tile_counts_dev, tiles);
    k_postpone_scatter<<<tiles, kBlock, 0, ctx->stream>>>(raw, n, t.hot_bits_dev, V, d->first_pos_dev,
                                                          d->tile_counts_dev, tiles, out);
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
