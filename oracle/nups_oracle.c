/*
 * CPU oracle for the minibatch step of sparse-parameter SGD on the paper's three
 * workloads (knowledge-graph embeddings, word vectors, matrix factorisation;
 * Section 5.1, Table 1) and for the sampling primitive PrepareSample / PullSample
 * (Section 4.3) with the four schemes of Section 4.4.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, sequential, single-threaded
 * reference: every dot product, coefficient and per-key sum is carried in fp64 and
 * rounded to fp32 once, when the update is applied.  It shares no code, header,
 * table or constant generator with the GPU library and must never be called from
 * the product path; only tests, the smoke check and the CPU-baseline leg of the
 * benchmark use it.
 *
 * Step semantics (synchronous minibatch reading of the per-key working-copy
 * behaviour described in Section 5.8): all gradients of a step are computed
 * against the table values as they were when the step began; contributions to the
 * same key are summed; the sum is applied once per key.
 *
 * Where the paper leaves the arithmetic to its citations (skip-gram negative
 * sampling, ComplEx, AdaGrad, squared-loss factorisation), the textbook form is
 * used; each function says which.  Nothing here is pinned to itself: the tests
 * check finite differences, closed forms, the paper's worked pool-reuse example
 * (Section 4.4), distribution tests and brute-force enumeration.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NOR_OK 0
#define NOR_ERR_ARG (-1)
#define NOR_ERR_KEY (-2)
#define NOR_ERR_MEM (-7)

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers: Philox-4x32 with 10 rounds (Salmon, Moraes,   */
/* Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11).          */
/* The paper does not name a generator; a counter-based one makes every        */
/* sample a pure function of (seed, step, draw).                               */
/* ------------------------------------------------------------------------- */
void nor_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random streams: what a block of four words is used for. */
enum { STREAM_FRESH = 1, STREAM_ORDER = 2, STREAM_LOCAL = 3, STREAM_ROUNDKEY = 4 };

/*
 * The four words of draw number `draw` of step `step`:
 *   key     = (seed low word, seed high word)
 *   counter = (draw low, draw high, step low, stream | dist_id << 8 | step bits 32..47 << 16)
 */
static void words_of(uint64_t seed, uint32_t stream, uint32_t dist_id, uint64_t step, uint64_t draw,
                     uint32_t out[4])
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t ctr[4] = { (uint32_t)draw, (uint32_t)(draw >> 32), (uint32_t)step,
                        (stream & 0xFFu) | ((dist_id & 0xFFu) << 8) | ((uint32_t)((step >> 32) & 0xFFFFu) << 16) };
    nor_philox4x32_10(ctr, key, out);
}

void nor_words(uint64_t seed, uint32_t stream, uint32_t dist_id, uint64_t step, uint64_t draw, uint32_t out[4])
{
    words_of(seed, stream, dist_id, step, draw, out);
}

/* floor(a * n / 2^64) for a 64-bit a: maps a uniform 64-bit word onto 0..n-1. */
static uint64_t scale64(uint64_t a, uint64_t n)
{
    return (uint64_t)(((unsigned __int128)a * (unsigned __int128)n) >> 64);
}

static uint32_t scale32(uint32_t a, uint32_t n)
{
    return (uint32_t)(((uint64_t)a * (uint64_t)n) >> 32);
}

/* ------------------------------------------------------------------------- */
/* Target distribution pi over keys (Section 4.1): alias table (Walker / Vose). */
/* ------------------------------------------------------------------------- */
/*
 * Builds, from non-negative weights w[0..V), the table used to draw from
 * pi_k = w_k / sum(w) in O(1): bucket b keeps itself with probability
 * thresh[b] / 2^32 and otherwise yields alias[b].
 *
 * Construction order (fixed so that two independent builds agree bit for bit):
 * q_k = (w_k / sum) * V with the sum taken in key order; keys with q < 1 go on
 * the `small` stack and the others on the `large` stack, in ascending key order;
 * repeatedly pop one of each from the back, give the small bucket the large key
 * as alias, reduce the large key's mass by what it donated ((q_l + q_s) - 1) and
 * push it back on the stack its new mass belongs to; whatever is left keeps
 * itself with probability one.
 */
int nor_alias_build(const double *w, int64_t V, uint32_t *thresh, uint32_t *alias)
{
    if (!w || !thresh || !alias || V <= 0 || V > 0xFFFFFFFFll) return NOR_ERR_ARG;
    double sum = 0.0;
    for (int64_t k = 0; k < V; ++k) {
        if (!(w[k] >= 0.0) || isinf(w[k])) return NOR_ERR_ARG;   /* negative or NaN */
        sum += w[k];
    }
    if (!(sum > 0.0) || isinf(sum)) return NOR_ERR_ARG;
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    uint32_t *small = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)V);
    uint32_t *large = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)V);
    if (!q || !small || !large) { free(q); free(small); free(large); return NOR_ERR_MEM; }
    int64_t ns = 0, nl = 0;
    for (int64_t k = 0; k < V; ++k) {
        double p = w[k] / sum;
        q[k] = p * (double)V;
        if (q[k] < 1.0) small[ns++] = (uint32_t)k; else large[nl++] = (uint32_t)k;
    }
    double *mass = (double *)malloc(sizeof(double) * (size_t)V);
    if (!mass) { free(q); free(small); free(large); return NOR_ERR_MEM; }
    for (int64_t k = 0; k < V; ++k) { mass[k] = 1.0; alias[k] = (uint32_t)k; }
    while (ns > 0 && nl > 0) {
        uint32_t s = small[--ns];
        uint32_t l = large[--nl];
        mass[s] = q[s];
        alias[s] = l;
        q[l] = (q[l] + q[s]) - 1.0;
        if (q[l] < 1.0) small[ns++] = l; else large[nl++] = l;
    }
    for (int64_t k = 0; k < V; ++k) {
        double t = floor(mass[k] * 4294967296.0);
        thresh[k] = (t >= 4294967295.0) ? 0xFFFFFFFFu : (t <= 0.0 ? 0u : (uint32_t)t);
    }
    free(q); free(small); free(large); free(mass);
    return NOR_OK;
}

/*
 * One fresh draw from pi: words (x0..x3) of the draw; bucket = floor((x0 + 2^32 x1) V / 2^64);
 * keep the bucket if x2 < thresh[bucket], else take its alias.  With thresh == NULL the
 * target is the uniform distribution over keys (the KGE task of Section 5.1).
 */
static uint32_t fresh_key(const uint32_t *thresh, const uint32_t *alias, int64_t V,
                          uint64_t seed, uint32_t dist_id, uint64_t step, uint64_t draw)
{
    uint32_t x[4];
    words_of(seed, STREAM_FRESH, dist_id, step, draw, x);
    uint64_t u = (uint64_t)x[0] | ((uint64_t)x[1] << 32);
    uint32_t b = (uint32_t)scale64(u, (uint64_t)V);
    if (!thresh) return b;
    return (x[2] < thresh[b]) ? b : alias[b];
}

/* ------------------------------------------------------------------------- */
/* Sampling schemes (Section 4.4).  Each writes the sample sequence of one     */
/* PrepareSample call (one handle of N samples) into out[0..N).                */
/* ------------------------------------------------------------------------- */

/* Independent sampling (CONFORM): N i.i.d. draws, each used once.  Sample i is draw draw0 + i. */
int nor_sample_conform(const uint32_t *thresh, const uint32_t *alias, int64_t V,
                       uint64_t seed, uint32_t dist_id, uint64_t step, uint64_t draw0,
                       int64_t N, uint32_t *out)
{
    if (V <= 0 || N < 0 || (N > 0 && !out) || (thresh && !alias)) return NOR_ERR_ARG;
    for (int64_t i = 0; i < N; ++i)
        out[i] = fresh_key(thresh, alias, V, seed, dist_id, step, draw0 + (uint64_t)i);
    return NOR_OK;
}

typedef struct { uint32_t word; uint32_t slot; } order_item;

static int order_cmp(const void *a, const void *b)
{
    const order_item *x = (const order_item *)a, *y = (const order_item *)b;
    if (x->word != y->word) return x->word < y->word ? -1 : 1;
    if (x->slot != y->slot) return x->slot < y->slot ? -1 : 1;
    return 0;
}

/*
 * Sample reuse (BOUNDED): pools of G i.i.d. draws; each pool is traversed U times,
 * each time in a random order, before the next pool is started (Section 4.4).
 * For one handle of N samples: F = ceil(N / U) fresh draws (draw ids 0..F-1 of this
 * step), pool m holds draws m*G .. min((m+1)*G, F)-1 (the last pool may be short),
 * the order of pass r over a pool is the ascending order of (w, slot) where w is
 * the first word of the ORDER stream at draw id (fresh id, pass r); the sequence is
 * cut after N samples.  Pools do not span handles.
 */
int nor_sample_bounded(const uint32_t *thresh, const uint32_t *alias, int64_t V,
                       uint64_t seed, uint32_t dist_id, uint64_t step,
                       int64_t N, int32_t U, int32_t G, uint32_t *out)
{
    if (V <= 0 || N < 0 || U < 1 || G < 1 || (N > 0 && !out) || (thresh && !alias)) return NOR_ERR_ARG;
    int64_t F = (N + U - 1) / U;
    order_item *item = (order_item *)malloc(sizeof(order_item) * (size_t)G);
    uint32_t *pool = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)G);
    if (!item || !pool) { free(item); free(pool); return NOR_ERR_MEM; }
    int64_t emitted = 0;
    for (int64_t first = 0; first < F && emitted < N; first += G) {
        int64_t g = (F - first < G) ? (F - first) : G;
        for (int64_t i = 0; i < g; ++i)
            pool[i] = fresh_key(thresh, alias, V, seed, dist_id, step, (uint64_t)(first + i));
        for (int32_t r = 0; r < U && emitted < N; ++r) {
            for (int64_t i = 0; i < g; ++i) {
                uint32_t x[4];
                words_of(seed, STREAM_ORDER, dist_id, step, (uint64_t)(first + i) | ((uint64_t)r << 32), x);
                item[i].word = x[0];
                item[i].slot = (uint32_t)i;
            }
            qsort(item, (size_t)g, sizeof(order_item), order_cmp);
            for (int64_t i = 0; i < g && emitted < N; ++i) out[emitted++] = pool[item[i].slot];
        }
    }
    free(item); free(pool);
    return NOR_OK;
}

static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x85EBCA6Bu;
    x ^= x >> 13; x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

/*
 * A keyed permutation of 0..P-1: a four-round balanced Feistel network on the
 * smallest even-width bit domain that holds P, walked until the value falls
 * below P.  Round keys are the four words of the ROUNDKEY stream at (step = epoch,
 * draw = pass).
 */
uint64_t nor_permute(uint64_t x, uint64_t P, uint64_t seed, uint32_t dist_id, uint64_t epoch, uint64_t pass)
{
    int half = 1;
    while (half < 32 && ((uint64_t)1 << (2 * half)) < P) ++half;
    uint32_t mask = (half >= 32) ? 0xFFFFFFFFu : (((uint32_t)1 << half) - 1u);
    uint32_t k[4];
    words_of(seed, STREAM_ROUNDKEY, dist_id, epoch, pass, k);
    do {
        uint32_t L = (uint32_t)(x >> half) & mask, R = (uint32_t)x & mask;
        for (int t = 0; t < 4; ++t) {
            uint32_t nR = L ^ (mix32(R ^ k[t]) & mask);
            L = R; R = nR;
        }
        x = ((uint64_t)L << half) | R;
    } while (x >= P);
    return x;
}

/*
 * Sample reuse over a long-lived pool (LONG-TERM).  The scheme of Section 4.4 is
 * sample reuse plus postponing of samples whose parameters are not local; on one
 * device every parameter is local, so the postponing branch never fires.  What is
 * left is reuse of a pool that outlives a handle: a pool of P i.i.d. draws (draw ids
 * 0..P-1 of pseudo-step `epoch`) is traversed R times, each pass in the order given
 * by a keyed permutation, and then replaced by the pool of the next epoch, so that
 * long-run frequencies follow pi (Eq. 1) and not one pool's empirical frequencies.
 * `cursor` is the number of samples consumed by earlier handles.
 */
int nor_sample_longterm(const uint32_t *thresh, const uint32_t *alias, int64_t V,
                        uint64_t seed, uint32_t dist_id, int64_t P, int32_t R, uint64_t cursor,
                        int64_t N, uint32_t *out)
{
    if (V <= 0 || N < 0 || P < 1 || R < 1 || (N > 0 && !out) || (thresh && !alias)) return NOR_ERR_ARG;
    uint64_t per_epoch = (uint64_t)P * (uint64_t)R;
    for (int64_t i = 0; i < N; ++i) {
        uint64_t g = cursor + (uint64_t)i;
        uint64_t epoch = g / per_epoch, within = g % per_epoch;
        uint64_t pass = within / (uint64_t)P, rank = within % (uint64_t)P;
        uint64_t slot = nor_permute(rank, (uint64_t)P, seed, dist_id, epoch, pass);
        out[i] = fresh_key(thresh, alias, V, seed, dist_id, epoch, slot);
    }
    return NOR_OK;
}

/*
 * Direct-access repurposing / local sampling (NON-CONFORM, Sections 4.2 and 4.4):
 * negatives are taken from keys that the minibatch accesses anyway.  Sample p
 * belongs to example e = p / per_example; examples are grouped in tiles of T; the
 * sample is the key that a uniformly chosen example of e's tile contributes:
 * keys_a[e'] for the first `split` samples of an example, keys_b[e'] for the rest
 * (for word vectors both lists are the context words; for triples they are the
 * subjects and the objects).  The choice is floor(x0 * t / 2^32) with x0 the first
 * word of the LOCAL stream at draw id p and t the size of the tile.
 */
int nor_sample_nonconform(const uint32_t *keys_a, const uint32_t *keys_b, int64_t n_examples,
                          int32_t per_example, int32_t split, int32_t T,
                          uint64_t seed, uint32_t dist_id, uint64_t step,
                          int64_t N, uint32_t *out)
{
    if (!keys_a || !keys_b || n_examples < 1 || per_example < 1 || split < 0 || split > per_example || T < 1
        || N < 0 || (N > 0 && !out) || N > n_examples * (int64_t)per_example) return NOR_ERR_ARG;
    for (int64_t p = 0; p < N; ++p) {
        int64_t e = p / per_example;
        int64_t base = (e / T) * T;
        int64_t t = (n_examples - base < T) ? (n_examples - base) : T;
        uint32_t x[4];
        words_of(seed, STREAM_LOCAL, dist_id, step, (uint64_t)p, x);
        int64_t pick = base + (int64_t)scale32(x[0], (uint32_t)t);
        out[p] = ((p % per_example) < split) ? keys_a[pick] : keys_b[pick];
    }
    return NOR_OK;
}

/* ------------------------------------------------------------------------- */
/* Per-key aggregation structure: sorted distinct keys and how often each is   */
/* accessed in the step (one access per example and role, Section 2).          */
/* ------------------------------------------------------------------------- */
static int u32_cmp(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* Sorts a copy of keys[0..n); writes distinct keys ascending and their counts; returns how many. */
static int64_t distinct_keys(const uint32_t *keys, int64_t n, uint32_t *uniq, uint32_t *count)
{
    if (n == 0) return 0;
    uint32_t *s = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    if (!s) return -1;
    memcpy(s, keys, sizeof(uint32_t) * (size_t)n);
    qsort(s, (size_t)n, sizeof(uint32_t), u32_cmp);
    int64_t nu = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (nu > 0 && uniq[nu - 1] == s[i]) { count[nu - 1] += 1; }
        else { uniq[nu] = s[i]; count[nu] = 1; ++nu; }
    }
    free(s);
    return nu;
}

int64_t nor_distinct_keys(const uint32_t *keys, int64_t n, uint32_t *uniq, uint32_t *count)
{
    if (n < 0 || (n > 0 && (!keys || !uniq || !count))) return NOR_ERR_ARG;
    return distinct_keys(keys, n, uniq, count);
}

static int64_t slot_of(const uint32_t *uniq, int64_t nu, uint32_t key)
{
    int64_t lo = 0, hi = nu - 1;
    while (lo < hi) {
        int64_t mid = (lo + hi) / 2;
        if (uniq[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

static int keys_in_range(const uint32_t *keys, int64_t n, int64_t V)
{
    for (int64_t i = 0; i < n; ++i) if ((int64_t)keys[i] >= V) return 0;
    return 1;
}

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* log(1 + e^x) without overflow. */
static double softplus(double x) { return x > 0.0 ? x + log1p(exp(-x)) : log1p(exp(x)); }

/* ------------------------------------------------------------------------- */
/* Direct access: pull and push (Section 3.1).                                 */
/* ------------------------------------------------------------------------- */
/* pull: values[i, :] = table[keys[i], :] (whole stored row, padding included). */
int nor_pull(const float *table, int64_t V, int32_t stride, const uint32_t *keys, int64_t n, float *values)
{
    if (!table || V <= 0 || stride <= 0 || n < 0 || (n > 0 && (!keys || !values))) return NOR_ERR_ARG;
    if (!keys_in_range(keys, n, V)) return NOR_ERR_KEY;
    for (int64_t i = 0; i < n; ++i)
        memcpy(values + i * (int64_t)stride, table + (int64_t)keys[i] * stride, sizeof(float) * (size_t)stride);
    return NOR_OK;
}

/* push: table[k, :] += sum of the update rows sent for k (updates are additive, duplicates add up). */
int nor_push(float *table, int64_t V, int32_t stride, int32_t dim, const uint32_t *keys, int64_t n,
             const float *updates)
{
    if (!table || V <= 0 || stride <= 0 || dim <= 0 || dim > stride || n < 0 || (n > 0 && (!keys || !updates)))
        return NOR_ERR_ARG;
    if (!keys_in_range(keys, n, V)) return NOR_ERR_KEY;
    if (n == 0) return NOR_OK;
    uint32_t *uniq = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    uint32_t *cnt = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n);
    if (!uniq || !cnt) { free(uniq); free(cnt); return NOR_ERR_MEM; }
    int64_t nu = distinct_keys(keys, n, uniq, cnt);
    double *acc = (double *)calloc((size_t)nu * (size_t)dim, sizeof(double));
    if (nu < 0 || !acc) { free(uniq); free(cnt); free(acc); return NOR_ERR_MEM; }
    for (int64_t i = 0; i < n; ++i) {
        double *a = acc + slot_of(uniq, nu, keys[i]) * dim;
        for (int32_t m = 0; m < dim; ++m) a[m] += (double)updates[i * (int64_t)stride + m];
    }
    for (int64_t u = 0; u < nu; ++u) {
        float *row = table + (int64_t)uniq[u] * stride;
        for (int32_t m = 0; m < dim; ++m) row[m] = (float)((double)row[m] + acc[u * dim + m]);
    }
    free(uniq); free(cnt); free(acc);
    return NOR_OK;
}

/* theta <- fl32(theta - lr * delta), elementwise, for every distinct key. */
static void apply_sgd(float *table, int32_t stride, int32_t dim, const uint32_t *uniq, int64_t nu,
                      const double *acc, float lr)
{
    for (int64_t u = 0; u < nu; ++u) {
        float *row = table + (int64_t)uniq[u] * stride;
        for (int32_t m = 0; m < dim; ++m)
            row[m] = (float)((double)row[m] - (double)lr * acc[u * dim + m]);
    }
}

/*
 * Norm clipping of the updates of hot keys (Section 5.1, implementation paragraph: for the replicated
 * parameters of the word-vector and factorisation tasks, an update whose norm exceeds the average norm
 * by more than a factor is clipped; the construction is that of Pascanu, Mikolov, Bengio 2013: an update
 * that is too long keeps its direction and is shortened to the bound).
 *
 * Reading used here, the paper gives no more than that sentence:
 *  - "update" = the summed gradient of one key in one step, `acc` row u; its norm is Euclidean, over `dim`;
 *  - "replicated parameters" = the keys with hot[key] != 0 (one flag per key of the table);
 *  - "average norm" = the mean of the norms, before clipping, of all hot-key updates of this table in the
 *    steps before this one: stats[0] = their sum, stats[1] = their number.  A step never looks at its own
 *    norms, so its result does not depend on the order of its keys; while no norm has been seen nothing is clipped;
 *  - a hot key's update of norm n > factor * mean is multiplied by factor * mean / n.
 * After the step, stats include this step's norms (as they were before clipping).
 * hot == NULL, stats == NULL or factor <= 0: nothing happens.
 */
static void clip_hot_updates(double *acc, const uint32_t *uniq, int64_t nu, int32_t dim, const uint8_t *hot,
                             double factor, double *stats)
{
    if (!hot || !stats || !(factor > 0.0)) return;
    const double seen = stats[1];
    const double bound = seen > 0.0 ? factor * (stats[0] / seen) : INFINITY;
    for (int64_t u = 0; u < nu; ++u) {
        if (!hot[uniq[u]]) continue;
        double *a = acc + u * dim;
        double sq = 0.0;
        for (int32_t m = 0; m < dim; ++m) sq += a[m] * a[m];
        const double norm = sqrt(sq);
        stats[0] += norm;
        stats[1] += 1.0;
        if (norm > bound) {
            const double shrink = bound / norm;
            for (int32_t m = 0; m < dim; ++m) a[m] *= shrink;
        }
    }
}

/*
 * AdaGrad (Duchi, Hazan, Singer 2011) on the summed gradient of the step, elementwise:
 * G <- fl32(G + delta^2); theta <- fl32(theta - lr * delta / (sqrt(G) + eps)) with the new G.
 * Rows that the step does not touch keep value and state (sparse AdaGrad).
 */
/* `split` > 0: accumulator entries split.. are stored from float `split_at` on (complex rows); 0: contiguous. */
static void apply_adagrad(float *table, float *state, int32_t stride, int32_t dim, const uint32_t *uniq,
                          int64_t nu, const double *acc, float lr, float eps, int32_t split, int32_t split_at)
{
    for (int64_t u = 0; u < nu; ++u) {
        float *row = table + (int64_t)uniq[u] * stride;
        float *g2 = state + (int64_t)uniq[u] * stride;
        for (int32_t m = 0; m < dim; ++m) {
            int32_t at = (split > 0 && m >= split) ? split_at + (m - split) : m;
            double d = acc[u * dim + m];
            g2[at] = (float)((double)g2[at] + d * d);
            row[at] = (float)((double)row[at] - (double)lr * d / (sqrt((double)g2[at]) + (double)eps));
        }
    }
}

void nor_apply_adagrad_rows(float *table, float *state, int32_t stride, int32_t dim, const uint32_t *uniq,
                            int64_t nu, const double *acc, float lr, float eps)
{
    apply_adagrad(table, state, stride, dim, uniq, nu, acc, lr, eps, 0, 0);
}

/* ------------------------------------------------------------------------- */
/* Word vectors: skip-gram with negative sampling (Mikolov et al. 2013;        */
/* Section 5.1).  Negatives read and write the output table only (Section 2.2). */
/* ------------------------------------------------------------------------- */
/*
 * Example e: v = In[center_e]; rows u_0 = Out[context_e] (label 1) and
 * u_j = Out[negs[e*K + j-1]] (label 0), j = 1..K.
 *   z_j = <v, u_j>,  loss_e = -log sigma(z_0) - sum_{j>=1} log sigma(-z_j),
 *   g_j = dloss/dz_j = sigma(z_j) - label_j,
 *   dloss/dv = sum_j g_j u_j,   dloss/du_j = g_j v.
 * A negative that equals the context word, or repeats, is kept: it simply
 * contributes another term.  Batch gradients are summed, not averaged.
 *
 * Outputs (any may be NULL): loss summed over the batch; for each table the distinct
 * keys ascending with their access counts (buffers of B and B*(K+1) entries).
 */
static int step_sgns(float *In, float *Out, int64_t V_in, int64_t V_out, int32_t stride, int32_t dim,
                     const uint32_t *center, const uint32_t *context, const uint32_t *negs,
                     int64_t B, int32_t K, float lr, double *loss_out,
                     uint32_t *uniq_in, uint32_t *count_in, int64_t *n_uniq_in,
                     uint32_t *uniq_out, uint32_t *count_out, int64_t *n_uniq_out,
                     const uint8_t *hot_in, const uint8_t *hot_out, double clip_factor,
                     double *clip_stats_in, double *clip_stats_out)
{
    if (!In || !Out || V_in <= 0 || V_out <= 0 || stride <= 0 || dim <= 0 || dim > stride || B < 0 || K < 0
        || (B > 0 && (!center || !context)) || (B > 0 && K > 0 && !negs)) return NOR_ERR_ARG;
    if (!keys_in_range(center, B, V_in) || !keys_in_range(context, B, V_out)
        || !keys_in_range(negs, B * (int64_t)K, V_out)) return NOR_ERR_KEY;
    int64_t n_out = B * (int64_t)(K + 1);
    int rc = NOR_ERR_MEM;
    uint32_t *okeys = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_out + 1));
    uint32_t *ui = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    uint32_t *ci = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    uint32_t *uo = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_out + 1));
    uint32_t *co = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_out + 1));
    double *acc_in = NULL, *acc_out = NULL;
    if (!okeys || !ui || !ci || !uo || !co) goto done;
    for (int64_t e = 0; e < B; ++e) {
        okeys[e * (K + 1)] = context[e];
        for (int32_t j = 0; j < K; ++j) okeys[e * (K + 1) + 1 + j] = negs[e * K + j];
    }
    int64_t nui = distinct_keys(center, B, ui, ci);
    int64_t nuo = distinct_keys(okeys, n_out, uo, co);
    if (nui < 0 || nuo < 0) goto done;
    acc_in = (double *)calloc((size_t)(nui * dim + 1), sizeof(double));
    acc_out = (double *)calloc((size_t)(nuo * dim + 1), sizeof(double));
    if (!acc_in || !acc_out) goto done;

    double loss = 0.0;
    for (int64_t e = 0; e < B; ++e) {
        const float *v = In + (int64_t)center[e] * stride;
        double *av = acc_in + slot_of(ui, nui, center[e]) * dim;
        for (int32_t j = 0; j <= K; ++j) {
            uint32_t key = okeys[e * (K + 1) + j];
            const float *u = Out + (int64_t)key * stride;
            double z = 0.0;
            for (int32_t m = 0; m < dim; ++m) z += (double)v[m] * (double)u[m];
            double label = (j == 0) ? 1.0 : 0.0;
            double g = sigmoid(z) - label;
            loss += (j == 0) ? softplus(-z) : softplus(z);
            double *au = acc_out + slot_of(uo, nuo, key) * dim;
            for (int32_t m = 0; m < dim; ++m) {
                av[m] += g * (double)u[m];
                au[m] += g * (double)v[m];
            }
        }
    }
    clip_hot_updates(acc_in, ui, nui, dim, hot_in, clip_factor, clip_stats_in);
    clip_hot_updates(acc_out, uo, nuo, dim, hot_out, clip_factor, clip_stats_out);
    apply_sgd(In, stride, dim, ui, nui, acc_in, lr);
    apply_sgd(Out, stride, dim, uo, nuo, acc_out, lr);
    if (loss_out) *loss_out = loss;
    if (n_uniq_in) *n_uniq_in = nui;
    if (n_uniq_out) *n_uniq_out = nuo;
    if (uniq_in) memcpy(uniq_in, ui, sizeof(uint32_t) * (size_t)nui);
    if (count_in) memcpy(count_in, ci, sizeof(uint32_t) * (size_t)nui);
    if (uniq_out) memcpy(uniq_out, uo, sizeof(uint32_t) * (size_t)nuo);
    if (count_out) memcpy(count_out, co, sizeof(uint32_t) * (size_t)nuo);
    rc = NOR_OK;
done:
    free(okeys); free(ui); free(ci); free(uo); free(co); free(acc_in); free(acc_out);
    return rc;
}

int nor_step_sgns(float *In, float *Out, int64_t V_in, int64_t V_out, int32_t stride, int32_t dim,
                  const uint32_t *center, const uint32_t *context, const uint32_t *negs,
                  int64_t B, int32_t K, float lr, double *loss_out,
                  uint32_t *uniq_in, uint32_t *count_in, int64_t *n_uniq_in,
                  uint32_t *uniq_out, uint32_t *count_out, int64_t *n_uniq_out)
{
    return step_sgns(In, Out, V_in, V_out, stride, dim, center, context, negs, B, K, lr, loss_out, uniq_in, count_in,
                     n_uniq_in, uniq_out, count_out, n_uniq_out, NULL, NULL, 0.0, NULL, NULL);
}

/* The same step with the updates of hot keys clipped (see clip_hot_updates): hot_* are one byte per key of the
 * table (NULL: no hot keys), clip_stats_* the table's {sum of norms, number of norms} so far, updated in place. */
int nor_step_sgns_clipped(float *In, float *Out, int64_t V_in, int64_t V_out, int32_t stride, int32_t dim,
                          const uint32_t *center, const uint32_t *context, const uint32_t *negs,
                          int64_t B, int32_t K, float lr, double *loss_out,
                          const uint8_t *hot_in, const uint8_t *hot_out, double clip_factor,
                          double *clip_stats_in, double *clip_stats_out)
{
    return step_sgns(In, Out, V_in, V_out, stride, dim, center, context, negs, B, K, lr, loss_out, NULL, NULL, NULL,
                     NULL, NULL, NULL, hot_in, hot_out, clip_factor, clip_stats_in, clip_stats_out);
}

/* Loss of a batch at the current table values, nothing updated (for finite differences). */
double nor_loss_sgns(const float *In, const float *Out, int32_t stride, int32_t dim,
                     const uint32_t *center, const uint32_t *context, const uint32_t *negs,
                     int64_t B, int32_t K)
{
    double loss = 0.0;
    for (int64_t e = 0; e < B; ++e) {
        const float *v = In + (int64_t)center[e] * stride;
        for (int32_t j = 0; j <= K; ++j) {
            uint32_t key = (j == 0) ? context[e] : negs[e * K + j - 1];
            const float *u = Out + (int64_t)key * stride;
            double z = 0.0;
            for (int32_t m = 0; m < dim; ++m) z += (double)v[m] * (double)u[m];
            loss += (j == 0) ? softplus(-z) : softplus(z);
        }
    }
    return loss;
}

/* ------------------------------------------------------------------------- */
/* Matrix factorisation: squared loss with L2 regularisation, SGD              */
/* (Section 5.1; the form of Koren, Bell, Volinsky 2009).  No sampling access. */
/* ------------------------------------------------------------------------- */
/*
 * Cell c = (i, j, x): err = x - <W_i, H_j>;
 *   loss_c = err^2 + l2 (|W_i|^2 + |H_j|^2)   (the regulariser counts once per cell occurrence)
 *   dloss/dW_i = -2 err H_j + 2 l2 W_i,   dloss/dH_j = -2 err W_i + 2 l2 H_j.
 * Duplicate cells are kept.  Gradients are summed over the batch.
 */
static int step_mf(float *W, float *H, int64_t n_rows, int64_t n_cols, int32_t stride, int32_t dim,
                   const uint32_t *row, const uint32_t *col, const float *val, int64_t B,
                   float lr, float l2, double *loss_out,
                   uint32_t *uniq_w, uint32_t *count_w, int64_t *n_uniq_w,
                   uint32_t *uniq_h, uint32_t *count_h, int64_t *n_uniq_h,
                   const uint8_t *hot_w, const uint8_t *hot_h, double clip_factor,
                   double *clip_stats_w, double *clip_stats_h)
{
    if (!W || !H || n_rows <= 0 || n_cols <= 0 || stride <= 0 || dim <= 0 || dim > stride || B < 0
        || (B > 0 && (!row || !col || !val))) return NOR_ERR_ARG;
    if (!keys_in_range(row, B, n_rows) || !keys_in_range(col, B, n_cols)) return NOR_ERR_KEY;
    int rc = NOR_ERR_MEM;
    uint32_t *uw = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    uint32_t *cw = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    uint32_t *uh = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    uint32_t *ch = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    double *acc_w = NULL, *acc_h = NULL;
    if (!uw || !cw || !uh || !ch) goto done;
    int64_t nuw = distinct_keys(row, B, uw, cw);
    int64_t nuh = distinct_keys(col, B, uh, ch);
    if (nuw < 0 || nuh < 0) goto done;
    acc_w = (double *)calloc((size_t)(nuw * dim + 1), sizeof(double));
    acc_h = (double *)calloc((size_t)(nuh * dim + 1), sizeof(double));
    if (!acc_w || !acc_h) goto done;
    double loss = 0.0;
    for (int64_t c = 0; c < B; ++c) {
        const float *w = W + (int64_t)row[c] * stride;
        const float *h = H + (int64_t)col[c] * stride;
        double dot = 0.0, nw = 0.0, nh = 0.0;
        for (int32_t m = 0; m < dim; ++m) {
            dot += (double)w[m] * (double)h[m];
            nw += (double)w[m] * (double)w[m];
            nh += (double)h[m] * (double)h[m];
        }
        double err = (double)val[c] - dot;
        loss += err * err + (double)l2 * (nw + nh);
        double *aw = acc_w + slot_of(uw, nuw, row[c]) * dim;
        double *ah = acc_h + slot_of(uh, nuh, col[c]) * dim;
        for (int32_t m = 0; m < dim; ++m) {
            aw[m] += -2.0 * err * (double)h[m] + 2.0 * (double)l2 * (double)w[m];
            ah[m] += -2.0 * err * (double)w[m] + 2.0 * (double)l2 * (double)h[m];
        }
    }
    clip_hot_updates(acc_w, uw, nuw, dim, hot_w, clip_factor, clip_stats_w);
    clip_hot_updates(acc_h, uh, nuh, dim, hot_h, clip_factor, clip_stats_h);
    apply_sgd(W, stride, dim, uw, nuw, acc_w, lr);
    apply_sgd(H, stride, dim, uh, nuh, acc_h, lr);
    if (loss_out) *loss_out = loss;
    if (n_uniq_w) *n_uniq_w = nuw;
    if (n_uniq_h) *n_uniq_h = nuh;
    if (uniq_w) memcpy(uniq_w, uw, sizeof(uint32_t) * (size_t)nuw);
    if (count_w) memcpy(count_w, cw, sizeof(uint32_t) * (size_t)nuw);
    if (uniq_h) memcpy(uniq_h, uh, sizeof(uint32_t) * (size_t)nuh);
    if (count_h) memcpy(count_h, ch, sizeof(uint32_t) * (size_t)nuh);
    rc = NOR_OK;
done:
    free(uw); free(cw); free(uh); free(ch); free(acc_w); free(acc_h);
    return rc;
}

int nor_step_mf(float *W, float *H, int64_t n_rows, int64_t n_cols, int32_t stride, int32_t dim,
                const uint32_t *row, const uint32_t *col, const float *val, int64_t B,
                float lr, float l2, double *loss_out,
                uint32_t *uniq_w, uint32_t *count_w, int64_t *n_uniq_w,
                uint32_t *uniq_h, uint32_t *count_h, int64_t *n_uniq_h)
{
    return step_mf(W, H, n_rows, n_cols, stride, dim, row, col, val, B, lr, l2, loss_out, uniq_w, count_w, n_uniq_w,
                   uniq_h, count_h, n_uniq_h, NULL, NULL, 0.0, NULL, NULL);
}

/* The same step with the updates of hot rows and columns clipped (see clip_hot_updates). */
int nor_step_mf_clipped(float *W, float *H, int64_t n_rows, int64_t n_cols, int32_t stride, int32_t dim,
                        const uint32_t *row, const uint32_t *col, const float *val, int64_t B,
                        float lr, float l2, double *loss_out,
                        const uint8_t *hot_w, const uint8_t *hot_h, double clip_factor,
                        double *clip_stats_w, double *clip_stats_h)
{
    return step_mf(W, H, n_rows, n_cols, stride, dim, row, col, val, B, lr, l2, loss_out, NULL, NULL, NULL, NULL, NULL,
                   NULL, hot_w, hot_h, clip_factor, clip_stats_w, clip_stats_h);
}

double nor_loss_mf(const float *W, const float *H, int32_t stride, int32_t dim,
                   const uint32_t *row, const uint32_t *col, const float *val, int64_t B, float l2)
{
    double loss = 0.0;
    for (int64_t c = 0; c < B; ++c) {
        const float *w = W + (int64_t)row[c] * stride;
        const float *h = H + (int64_t)col[c] * stride;
        double dot = 0.0, nw = 0.0, nh = 0.0;
        for (int32_t m = 0; m < dim; ++m) {
            dot += (double)w[m] * (double)h[m];
            nw += (double)w[m] * (double)w[m];
            nh += (double)h[m] * (double)h[m];
        }
        double err = (double)val[c] - dot;
        loss += err * err + (double)l2 * (nw + nh);
    }
    return loss;
}

/* ------------------------------------------------------------------------- */
/* Knowledge-graph embeddings: ComplEx (Trouillon et al. 2016) with logistic   */
/* loss, negative sampling by corrupting subject and object, AdaGrad           */
/* (Section 5.1).  Storage layout of a complex row of `dim` values in a row of */
/* `stride` floats: the dim/2 real parts start at float 0, the dim/2 imaginary */
/* parts start at float stride/2 (so a stored row is two equal halves); the    */
/* paper does not prescribe a layout.                                          */
/* ------------------------------------------------------------------------- */
/* score(s, r, o) = Re( sum_m s_m r_m conj(o_m) ); `im` = offset of the imaginary half. */
static double complex_score(const float *s, const float *r, const float *o, int32_t half, int32_t im)
{
    double phi = 0.0;
    for (int32_t m = 0; m < half; ++m) {
        double sr = s[m], si = s[im + m], rr = r[m], ri = r[im + m], orr = o[m], oi = o[im + m];
        phi += sr * rr * orr + si * rr * oi + sr * ri * oi - si * ri * orr;
    }
    return phi;
}

double nor_complex_score(const float *s, const float *r, const float *o, int32_t stride, int32_t dim)
{
    return complex_score(s, r, o, dim / 2, stride / 2);
}

/* acc_* += g * dscore/d(row) for the three rows of one scored triple (accumulators are [dim]: re then im). */
static void complex_grad(const float *s, const float *r, const float *o, int32_t half, int32_t im, double g,
                         double *as, double *ar, double *ao)
{
    for (int32_t m = 0; m < half; ++m) {
        double sr = s[m], si = s[im + m], rr = r[m], ri = r[im + m], orr = o[m], oi = o[im + m];
        as[m]        += g * (rr * orr + ri * oi);
        as[half + m] += g * (rr * oi - ri * orr);
        ar[m]        += g * (sr * orr + si * oi);
        ar[half + m] += g * (sr * oi - si * orr);
        ao[m]        += g * (sr * rr - si * ri);
        ao[half + m] += g * (si * rr + sr * ri);
    }
}

/*
 * Triple e = (s, r, o) with label +1; its negatives (label -1) are
 *   (negs[e*(nh+nt) + i], r, o) for i < nh   (subject replaced) and
 *   (s, r, negs[e*(nh+nt) + nh + i]) for i < nt   (object replaced).
 * loss = sum over scored triples of softplus(-label * score); dloss/dscore =
 * -label * sigma(-label * score).  A negative equal to the true entity is kept.
 * Entity rows and relation rows live in separate tables E, R with AdaGrad state
 * GE, GR of the same shape.  Structure output for E counts one access per example
 * and role (subject, object, each negative); for R one per example.
 */
int nor_step_kge(float *E, float *GE, float *R, float *GR, int64_t n_ent, int64_t n_rel,
                 int32_t stride, int32_t dim,
                 const uint32_t *subj, const uint32_t *rel, const uint32_t *obj, const uint32_t *negs,
                 int64_t B, int32_t nh, int32_t nt, float lr, float eps, double *loss_out,
                 uint32_t *uniq_e, uint32_t *count_e, int64_t *n_uniq_e,
                 uint32_t *uniq_r, uint32_t *count_r, int64_t *n_uniq_r)
{
    if (!E || !GE || !R || !GR || n_ent <= 0 || n_rel <= 0 || stride <= 0 || dim <= 0 || dim > stride
        || (dim & 1) || B < 0 || nh < 0 || nt < 0 || (B > 0 && (!subj || !rel || !obj))
        || (B > 0 && nh + nt > 0 && !negs)) return NOR_ERR_ARG;
    int32_t nn = nh + nt, half = dim / 2, im = stride / 2;
    if ((stride & 1) || half > im) return NOR_ERR_ARG;
    if (!keys_in_range(subj, B, n_ent) || !keys_in_range(obj, B, n_ent) || !keys_in_range(rel, B, n_rel)
        || !keys_in_range(negs, B * (int64_t)nn, n_ent)) return NOR_ERR_KEY;
    int64_t n_acc = B * (int64_t)(2 + nn);
    int rc = NOR_ERR_MEM;
    uint32_t *ekeys = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_acc + 1));
    uint32_t *ue = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_acc + 1));
    uint32_t *ce = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(n_acc + 1));
    uint32_t *ur = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    uint32_t *cr = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(B + 1));
    double *acc_e = NULL, *acc_r = NULL;
    if (!ekeys || !ue || !ce || !ur || !cr) goto done;
    for (int64_t e = 0; e < B; ++e) {
        ekeys[e * (2 + nn)] = subj[e];
        ekeys[e * (2 + nn) + 1] = obj[e];
        for (int32_t i = 0; i < nn; ++i) ekeys[e * (2 + nn) + 2 + i] = negs[e * nn + i];
    }
    int64_t nue = distinct_keys(ekeys, n_acc, ue, ce);
    int64_t nur = distinct_keys(rel, B, ur, cr);
    if (nue < 0 || nur < 0) goto done;
    acc_e = (double *)calloc((size_t)(nue * dim + 1), sizeof(double));
    acc_r = (double *)calloc((size_t)(nur * dim + 1), sizeof(double));
    if (!acc_e || !acc_r) goto done;
    double loss = 0.0;
    for (int64_t e = 0; e < B; ++e) {
        const float *r = R + (int64_t)rel[e] * stride;
        double *ar = acc_r + slot_of(ur, nur, rel[e]) * dim;
        for (int32_t t = 0; t <= nn; ++t) {
            uint32_t ks = subj[e], ko = obj[e];
            double label = 1.0;
            if (t >= 1) {
                label = -1.0;
                if (t - 1 < nh) ks = negs[e * nn + (t - 1)]; else ko = negs[e * nn + (t - 1)];
            }
            const float *s = E + (int64_t)ks * stride;
            const float *o = E + (int64_t)ko * stride;
            double phi = complex_score(s, r, o, half, im);
            loss += softplus(-label * phi);
            double g = -label * sigmoid(-label * phi);
            complex_grad(s, r, o, half, im, g, acc_e + slot_of(ue, nue, ks) * dim, ar,
                         acc_e + slot_of(ue, nue, ko) * dim);
        }
    }
    apply_adagrad(E, GE, stride, dim, ue, nue, acc_e, lr, eps, half, im);
    apply_adagrad(R, GR, stride, dim, ur, nur, acc_r, lr, eps, half, im);
    if (loss_out) *loss_out = loss;
    if (n_uniq_e) *n_uniq_e = nue;
    if (n_uniq_r) *n_uniq_r = nur;
    if (uniq_e) memcpy(uniq_e, ue, sizeof(uint32_t) * (size_t)nue);
    if (count_e) memcpy(count_e, ce, sizeof(uint32_t) * (size_t)nue);
    if (uniq_r) memcpy(uniq_r, ur, sizeof(uint32_t) * (size_t)nur);
    if (count_r) memcpy(count_r, cr, sizeof(uint32_t) * (size_t)nur);
    rc = NOR_OK;
done:
    free(ekeys); free(ue); free(ce); free(ur); free(cr); free(acc_e); free(acc_r);
    return rc;
}

double nor_loss_kge(const float *E, const float *R, int32_t stride, int32_t dim,
                    const uint32_t *subj, const uint32_t *rel, const uint32_t *obj, const uint32_t *negs,
                    int64_t B, int32_t nh, int32_t nt)
{
    int32_t nn = nh + nt, half = dim / 2, im = stride / 2;
    double loss = 0.0;
    for (int64_t e = 0; e < B; ++e) {
        const float *r = R + (int64_t)rel[e] * stride;
        for (int32_t t = 0; t <= nn; ++t) {
            uint32_t ks = subj[e], ko = obj[e];
            double label = 1.0;
            if (t >= 1) {
                label = -1.0;
                if (t - 1 < nh) ks = negs[e * nn + (t - 1)]; else ko = negs[e * nn + (t - 1)];
            }
            loss += softplus(-label * complex_score(E + (int64_t)ks * stride, r, E + (int64_t)ko * stride, half, im));
        }
    }
    return loss;
}
