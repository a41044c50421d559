// Device-side helpers: counter-based random words, 16-lane row groups, workgroup scans.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nups_internal.h"

namespace nups {

struct Words {
    uint32_t x0, x1, x2, x3;
};

// Philox-4x32, 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).
__device__ __forceinline__ Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    return Words{c0, c1, c2, c3};
}

// The four words of draw `draw` of step `step`: key = seed halves,
// counter = (draw lo, draw hi, step lo, stream | dist << 8 | step bits 32..47 << 16).
__device__ __forceinline__ Words draw_words(uint64_t seed, uint32_t stream, uint32_t dist, uint64_t step,
                                            uint64_t draw)
{
    const uint32_t c3 = (stream & 0xFFu) | ((dist & 0xFFu) << 8) | ((uint32_t)((step >> 32) & 0xFFFFu) << 16);
    return philox4x32_10((uint32_t)draw, (uint32_t)(draw >> 32), (uint32_t)step, c3, (uint32_t)seed,
                         (uint32_t)(seed >> 32));
}

// x as lane `ctrl` of the same 16-lane row holds it (a data-parallel-primitive move inside the vector unit: no LDS
// traffic, unlike a general shuffle).
template <int kCtrl>
__device__ __forceinline__ float row_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xF, 0xF, false));
}

// Lane kLane's x of each 16-lane row, to every lane of that row.
template <int kLane>
__device__ __forceinline__ uint32_t group_share(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x150 + kLane, 0xF, 0xF, false);   // row_newbcast
}

template <int kLane>
__device__ __forceinline__ float group_share(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + kLane, 0xF, 0xF, false));
}

// Sum over the 16 lanes of a row group; every lane of the group receives the total.  Neighbour in the pair, other
// pair of the quad, mirror image in the half row (the other quad), mirror image in the row (the other half).
__device__ __forceinline__ float group_sum(float x)
{
    x += row_move<0xB1>(x);    // quad_perm [1,0,3,2]
    x += row_move<0x4E>(x);    // quad_perm [2,3,0,1]
    x += row_move<0x141>(x);   // row_half_mirror
    x += row_move<0x140>(x);   // row_mirror
    return x;
}

template <int kCtrl>
__device__ __forceinline__ uint32_t row_move(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kCtrl, 0xF, 0xF, false);
}

// Smallest and largest x over the 16 lanes of a row group, to every lane of the group (same moves as group_sum).
__device__ __forceinline__ uint32_t group_min(uint32_t x)
{
    x = min(x, row_move<0xB1>(x));
    x = min(x, row_move<0x4E>(x));
    x = min(x, row_move<0x141>(x));
    x = min(x, row_move<0x140>(x));
    return x;
}

__device__ __forceinline__ uint32_t group_max(uint32_t x)
{
    x = max(x, row_move<0xB1>(x));
    x = max(x, row_move<0x4E>(x));
    x = max(x, row_move<0x141>(x));
    x = max(x, row_move<0x140>(x));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

__device__ __forceinline__ float dot4(const float4 a, const float4 b)
{
    return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
}

__device__ __forceinline__ void axpy4(float4 &acc, float a, const float4 x)
{
    acc.x += a * x.x; acc.y += a * x.y; acc.z += a * x.z; acc.w += a * x.w;
}

// A row of NV4 * 64 floats held by a 16-lane group: lane l owns float4 number l + 16 q, q < NV4.
template <int NV4>
struct Row {
    float4 v[NV4];
};

template <int NV4>
__device__ __forceinline__ void load_row(Row<NV4> &r, const float *base, int lane)
{
    const float4 *p = reinterpret_cast<const float4 *>(base) + lane;
#pragma unroll
    for (int q = 0; q < NV4; ++q) r.v[q] = p[q * kGroup];
}

template <int NV4>
__device__ __forceinline__ void store_row(float *base, const Row<NV4> &r, int lane)
{
    float4 *p = reinterpret_cast<float4 *>(base) + lane;
#pragma unroll
    for (int q = 0; q < NV4; ++q) p[q * kGroup] = r.v[q];
}

// The final value of a table row: written through to memory.  A launch ends with the write-back of whatever its
// stores left dirty in the dies' L2 caches, and the next launch starts only after it; rows written through as they
// are produced drain while the launch still runs (measured: the launch that follows an update of 12,000 rows of
// 1,280 bytes starts about 4 us sooner).  Nothing in the same launch reads these rows again.
template <int NV4>
__device__ __forceinline__ void store_row_through(float *base, const Row<NV4> &r, int lane)
{
    typedef float vec4 __attribute__((ext_vector_type(4)));
    vec4 *p = reinterpret_cast<vec4 *>(base) + lane;
#pragma unroll
    for (int q = 0; q < NV4; ++q) {
        const vec4 x = {r.v[q].x, r.v[q].y, r.v[q].z, r.v[q].w};
        __builtin_nontemporal_store(x, p + q * kGroup);
    }
}

// A row that another workgroup of the same launch reads (or has written): every word moves as a device-scope
// atomic access, which is performed where all compute dies see it, so no cache write-back or invalidation is
// needed around it.  all_stores_performed() returns once this wavefront's earlier stores have been acknowledged;
// an arrival counter incremented after it orders them before the reader's loads.
template <int NV4>
__device__ __forceinline__ void store_row_device_scope(float *base, const Row<NV4> &r, int lane)
{
    float *p = base + 4 * lane;
#pragma unroll
    for (int q = 0; q < NV4; ++q) {
        float *w = p + q * 4 * kGroup;
        __hip_atomic_store(w + 0, r.v[q].x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(w + 1, r.v[q].y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(w + 2, r.v[q].z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(w + 3, r.v[q].w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int NV4>
__device__ __forceinline__ void load_row_device_scope(Row<NV4> &r, const float *base, int lane)
{
    const float *p = base + 4 * lane;
#pragma unroll
    for (int q = 0; q < NV4; ++q) {
        const float *w = p + q * 4 * kGroup;
        r.v[q].x = __hip_atomic_load(w + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        r.v[q].y = __hip_atomic_load(w + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        r.v[q].z = __hip_atomic_load(w + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        r.v[q].w = __hip_atomic_load(w + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__device__ __forceinline__ void all_stores_performed() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int NV4>
__device__ __forceinline__ void zero_row(Row<NV4> &r)
{
#pragma unroll
    for (int q = 0; q < NV4; ++q) r.v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
}

template <int NV4>
__device__ __forceinline__ float partial_dot(const Row<NV4> &a, const Row<NV4> &b)
{
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < NV4; ++q) s += dot4(a.v[q], b.v[q]);
    return s;
}

template <int NV4>
__device__ __forceinline__ void axpy_row(Row<NV4> &acc, float a, const Row<NV4> &x)
{
#pragma unroll
    for (int q = 0; q < NV4; ++q) axpy4(acc.v[q], a, x.v[q]);
}

// hardware exponential and reciprocal: a unit in the last place each
__device__ __forceinline__ float sigmoidf(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

// log(1 + e^x), stable.  Only the reported loss uses it: the hardware logarithm of 1 + t is within 1e-7 absolute
// of log1p(t), which is the rounding level of a loss term anyway.
__device__ __forceinline__ float softplusf(float x)
{
    const float t = __expf(-fabsf(x));
    return fmaxf(x, 0.f) + __logf(1.0f + t);
}

// Exclusive prefix sum of one value per thread over a workgroup of kBlock threads.
// Returns the exclusive prefix; *total receives the workgroup sum.  `lds` needs kBlock / 64 + 1 words.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t *lds, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
    }
    __syncthreads();                  // lds may still be read from a previous call
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) {
        const uint32_t s = lds[w];
        if (w < wave) base += s;
        sum += s;
    }
    *total = sum;
    return base + incl - x;
}

__device__ __forceinline__ uint32_t block_sum(uint32_t x, uint32_t *lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    __syncthreads();
    if (lane == 0) lds[wave] = x;
    __syncthreads();
    uint32_t sum = 0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) sum += lds[w];
    return sum;
}

// Adds one value per workgroup (of WAVES wavefronts) to the step's loss accumulator: the slot is chosen by workgroup number.
template <int WAVES = kBlock / 64>
__device__ __forceinline__ void block_add_loss(float x, double *loss, float *lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    x = wave_sum(x);
    if (lane == 0) lds[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < WAVES; ++w) s += (double)lds[w];
        atomicAdd(loss + (blockIdx.x % kLossSlots) * kLossStride, s);
    }
}

// Workgroups are handed to the eight accelerator dies (XCDs, each with its own L2) round-robin by
// workgroup number.  xcd_block() renumbers them so that each die works on one contiguous eighth of the
// logical workgroups: examples that are neighbours in the batch (same center word, same sample pool)
// then share an L2 instead of fetching the same rows into several.  The grid must come from xcd_grid(); a
// launch that carries side work in its first workgroups passes its own workgroup number and count, and pads the
// side work to a multiple of kNumXcd workgroups.
constexpr uint32_t kNumXcd = 8;

__device__ __forceinline__ uint32_t xcd_block(uint32_t block, uint32_t blocks)
{
    return (block % kNumXcd) * (blocks / kNumXcd) + block / kNumXcd;
}

__device__ __forceinline__ uint32_t xcd_block() { return xcd_block(blockIdx.x, gridDim.x); }

static inline uint32_t xcd_grid(uint32_t blocks) { return (blocks + kNumXcd - 1) / kNumXcd * kNumXcd; }

// Which technique a key gets (Section 3.2: hot spots and the long tail are managed differently).  A segment of
// `count` accesses is cut into chunks for several workgroups if it is long and, when the caller declared a
// hot-key set, the key is in it; every other segment is summed by a single row group.
__device__ __forceinline__ bool in_hot_set(uint32_t key, const uint32_t *hot_bits, uint32_t base_keys)
{
    if (key >= base_keys) return true;   // a replica row of a hot key
    return ((hot_bits[key >> 5] >> (key & 31)) & 1u) != 0;
}

__device__ __forceinline__ bool takes_hot_path(uint32_t count, uint32_t key, const uint32_t *hot_bits, uint32_t base_keys)
{
    if (count <= kLongSegment) return false;
    return hot_bits == nullptr || in_hot_set(key, hot_bits, base_keys);
}

// The row that example `example`'s access to `key` (a valid key of the table) goes to: the key's replica for the
// example's part of the minibatch if the table has replicas and the key is hot, the key itself otherwise.
__device__ __forceinline__ uint32_t replica_key(const ReplicaMap &m, uint32_t key, uint32_t example)
{
    if (m.hot_slot == nullptr) return key;
    const uint32_t s = m.hot_slot[key];
    if (s == kBadIndex) return key;
    const uint32_t part = (uint32_t)(((uint64_t)example * m.replicas) / m.batch);
    return m.base_keys + part * m.hot_count + s;
}

// Address of row `key` of an extended key space: a row of the table or a replica row.
__device__ __forceinline__ float *extended_row(float *table, float *replica_rows, uint32_t base_keys, uint32_t key,
                                               int stride)
{
    return key < base_keys ? table + (size_t)key * stride : replica_rows + (size_t)(key - base_keys) * stride;
}

// Access i of a step's accesses to one table: its key in the table's extended key space, kBadIndex if the batch's
// key is outside the table.
__device__ __forceinline__ uint32_t plan_key(const KeySource &s, const ReplicaMap &m, uint32_t i)
{
    int which = 0;
    if (i >= s.len[0]) {
        i -= s.len[0];
        which = 1;
        if (i >= s.len[1]) { i -= s.len[1]; which = 2; }
    }
    const uint32_t key = s.ptr[which][i];
    if (key >= m.base_keys) return kBadIndex;
    const uint32_t per = s.per[which] ? s.per[which] : 1u;
    return replica_key(m, key, i / per);
}

}  // namespace nups
