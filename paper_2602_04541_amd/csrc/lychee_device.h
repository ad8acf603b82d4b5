// Device-side building blocks of the work-unit kernels (included by lychee_units.hip and lychee_layer.hip):
// the LDS layout of a workgroup, global-memory accessors, the bf16 dot product, wavefront and
// workgroup reductions and scans.
#pragma once
#include "lychee_internal.h"

namespace lychee {
namespace {

// ------------------------------------------------------------------------------ LDS layout
struct SharedAttn {
    int32_t idx_s[kIdxChunk];
    float red_o[kWaves * kMaxGroup * kHeadDim];
    float red_ml[kWaves * kMaxGroup * 2];
    float pool_ml[kWaves * 2];
    union {
        unsigned long long cand[kWaves][kCandBuf];  // per wavefront: candidates not yet flushed
        uint32_t keys[kKeyBuf];                     // or: the ordered keys of the piece's last kKeyBuf rows,
    };                                              //     filtered once the row's threshold is known
    int32_t cand_left[kWaves];                  // what each wavefront still holds when a piece ends
    int32_t cand_base;                          // where the workgroup's last candidates go
    uint32_t late_thr;                          // the row's threshold, once a piece has fetched it
    int32_t late_have;
    uint32_t scan[kWaves + 1];                  // block_scan scratch of the key filter
};
struct SharedSelect {
    uint32_t hist[4096];                   // radix histograms; position bitmap of the ordered write
    uint32_t samp[kSampleTilesMax * 16];   // ordered keys of the threshold sample
    uint32_t found[2];
    uint32_t chunk_at[kThreads];           // ordered write: output rank of the first position of each
    uint16_t word_at[4096];                //   run of 16 bitmap words, and of each word within its run
};
struct SharedCombine {
    float w[kMaxWg];
    float red[kMaxGroup * (kThreads / 32) * kHeadDim];  // (combine_unit uses the first head's share)
    float l[kMaxGroup];
};
union SharedUnit {
    SharedSelect sel;
    SharedCombine comb;
};
struct SharedPool {
    int32_t ipre[kMaxItems + 1];         // first pooled block of every (layer, sequence) item
    int32_t upre[4][kMaxLayers + 1];     // first small unit of every layer, per unit kind
    int32_t len[kMaxBatch];
    uint32_t scan[kWaves + 1];
    unsigned long long scan64[kWaves + 1];
    float fred[kWaves + 1];
};

// ------------------------------------------------------------------------------ primitives
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), acc, false);
}

template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float x)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kCtrl, 0xF, 0xF, false));
}

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the same bits.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_f32<0xB1>(x);   // quad_perm [1,0,3,2]  : lane ^ 1
    x += dpp_f32<0x4E>(x);   // quad_perm [2,3,0,1]  : lane ^ 2
    x += dpp_f32<0x141>(x);  // row_half_mirror      : the other quad of the 8-lane half
    x += dpp_f32<0x140>(x);  // row_mirror           : the other half of the 16-lane row
    return x;
}

// x + (x of the lane 16 lanes away) and the same for 32 lanes, as x + __shfl_xor(x, 16 / 32) give
// them (bit for bit: one addition of the same two numbers), without the LDS crossbar: gfx950's row
// swaps are plain vector instructions.  v_permlane16_swap(a, b) exchanges the odd rows of 16 lanes of a
// with the even rows of b, v_permlane32_swap(a, b) the upper half of a with the lower half of b; with
// a = b = x the two results hold the even (lower) parts of x everywhere and the odd (upper) parts
// everywhere.
__device__ __forceinline__ float sum_rows16(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}
__device__ __forceinline__ float sum_halves32(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}
__device__ __forceinline__ float max_rows16(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float max_halves32(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xFFFF0000u); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x)
{
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Every buffer the units touch is device global memory, but most pointers reach the kernel
// through the descriptor table, where the compiler can no longer see that.  Generic-address
// ("flat") accesses make it wait for *all* outstanding loads before each use, which breaks the
// load pipeline of the streaming loop; so every access goes through these casts.
#define LYCHEE_GLOBAL __attribute__((address_space(1)))
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ T gload(const T *p)
{
    return *(const LYCHEE_GLOBAL T *)p;
}
template <typename T>
__device__ __forceinline__ void gstore(T *p, T v)
{
    *(LYCHEE_GLOBAL T *)p = v;
}
// Write-through store: the value goes through the XCD's L2 to device memory, and the store counts
// as outstanding (vmcnt) until it is there.  A workgroup on another XCD that learns, through an
// agent-scope atomic issued after wait_stores(), that the data exists reads it after an acquire
// fence.  This is what lets a workgroup hand a partial result to another one in the same launch
// without the agent-scope release fence, whose write-back of the whole L2 costs tens of
// microseconds when hundreds of workgroups execute it.
__device__ __forceinline__ void gstore_through(float *p, float v)
{
    __hip_atomic_store((LYCHEE_GLOBAL float *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void gstore_through(int32_t *p, int32_t v)
{
    __hip_atomic_store((LYCHEE_GLOBAL int32_t *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void gstore_through(uint32_t *p, uint32_t v)
{
    __hip_atomic_store((LYCHEE_GLOBAL uint32_t *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float4 gload_f4(const float *p)
{
    const f32x4_t r = *(const LYCHEE_GLOBAL f32x4_t *)p;
    return make_float4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ uint4 gload_u4(const void *p)
{
    const u32x4_t r = *(const LYCHEE_GLOBAL u32x4_t *)p;
    return make_uint4(r.x, r.y, r.z, r.w);
}

// 16-byte streaming load: cache rows are read once per step and never again.
__device__ __forceinline__ uint4 load_stream16(const uint16_t *p)
{
    const u32x4_t r = __builtin_nontemporal_load((const LYCHEE_GLOBAL u32x4_t *)p);
    return make_uint4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ uint32_t ordered_key(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int clamp_len(int L, int max_len) { return L < 1 ? 1 : (L > max_len ? max_len : L); }

// Selectable units of a sequence of L rows: its positions, or its blocks of 64 positions
// (the last one may be short) in the block-granular variant (App. C).
__device__ __forceinline__ int units_of(const Common &c, int L)
{
    return (L + (1 << c.block_shift) - 1) >> c.block_shift;
}

// Units selected for a sequence of L units: Eq. 2's fixed budget, min(k, L), or under the
// Ratio rule (Sec. 4.4.1: a budget proportional to the sequence length) the rounded-up share
// keep_ppm / 10^6 of L, at least 1 and at most the fixed budget.
__device__ __forceinline__ int budget_of(const Common &c, int L)
{
    int n = c.k < L ? c.k : L;
    if (c.keep_ppm > 0) {
        long long r = ((long long)L * c.keep_ppm + 999999) / 1000000;
        r = r < 1 ? 1 : r;
        n = r < n ? (int)r : n;
    }
    return n;
}

// Fields of a layer descriptor staged in LDS as 32-bit words.  The values are the same in
// every lane; reading them back through readfirstlane tells the compiler so (scalar registers,
// scalar address arithmetic in the streaming loop).
constexpr int kDescWords = (int)(sizeof(LayerDesc) / 4);
static_assert(sizeof(LayerDesc) % 4 == 0 && kDescWords <= kThreads, "one word per thread");

// A value that is the same in every lane, said so to the compiler (a scalar register).
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

__device__ __forceinline__ uint32_t desc_u32(const uint32_t *dw, size_t off)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)dw[off / 4]);
}
__device__ __forceinline__ uint32_t desc_u8(const uint32_t *dw, size_t off)
{
    return (desc_u32(dw, off & ~(size_t)3) >> (8 * (off & 3))) & 0xFFu;
}
template <typename T>
__device__ __forceinline__ T *desc_ptr(const uint32_t *dw, size_t off)
{
    const uint64_t lo = desc_u32(dw, off), hi = desc_u32(dw, off + 4);
    return reinterpret_cast<T *>(lo | (hi << 32));
}

// Largest i in [0, n) with pre[i] <= x, for a non-decreasing pre[0..n] with pre[0] <= x < pre[n].
__device__ __forceinline__ int find_item(const int32_t *pre, int n, int x)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (pre[mid] <= x) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Rows a sparse KV head gathers for a sequence of L cache rows (set entries that are -1 or
// name rows past L are skipped one by one), and how many of them make one pooled block.
__device__ __forceinline__ int gather_rows(const Common &c, int L)
{
    const int units = units_of(c, L);
    return (c.k < units ? c.k : units) << c.block_shift;
}
__device__ __forceinline__ int gather_block(const Common &c)
{
    return c.block_shift ? (1 << c.block_shift) : c.g_block_rows;  // whole blocks stream like R rows
}

// Inclusive prefix sum over the 256 threads of the workgroup; `total` = sum of all.
__device__ __forceinline__ uint32_t block_scan(uint32_t v, uint32_t *wave_tot, uint32_t &total)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();  // wave_tot may still be read by the previous call
    if (lane == 63) wave_tot[wave] = x;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = wave_tot[w];
        before += (w < wave) ? t : 0u;
        all += t;
    }
    total = all;
    return x + before;
}

// The same for four 16-bit counts packed in 64 bits (no field may overflow).
__device__ __forceinline__ unsigned long long block_scan64(unsigned long long v, unsigned long long *wave_tot,
                                                           unsigned long long &total)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    unsigned long long x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = x;
    __syncthreads();
    unsigned long long before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const unsigned long long t = wave_tot[w];
        before += (w < wave) ? t : 0ull;
        all += t;
    }
    total = all;
    return x + before;
}

__device__ __forceinline__ float block_max(float v, float *scratch)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = scratch[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = fmaxf(r, scratch[w]);
    return r;
}

__device__ __forceinline__ float block_sum(float v, float *scratch)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = scratch[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r += scratch[w];
    return r;
}



}  // namespace
}  // namespace lychee
