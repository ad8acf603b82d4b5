// Top-k selection kernel (Eq. 2): for every (sequence, KV head) whose group holds a
// retrieval head, the min(k, L) positions with the largest pooled selection score, ties to
// the lower position, written ascending by position and padded with -1.  KV heads without a
// retrieval head get a verbatim copy of their inherited set (Sec. 3.1: the set is
// propagated unchanged).
//
// The paper does not say how argsTopK is executed.  Here: an exact radix select on the
// order-preserving 32-bit image of the fp32 score (three digit passes of 12 + 10 + 10 bits
// with an LDS histogram each, no sort), which yields the k-th largest key T and the number r
// of keys equal to T that still fit, followed by one ordered compaction pass that keeps
// keys > T and the first r keys == T, using wavefront prefix sums to place every kept
// position directly at its final slot.
#include "lychee_internal.h"

namespace lychee {
namespace {

constexpr int kSelWaves = kSelectThreads / 64;
constexpr int kTile = kSelectThreads * 4;  // elements per sweep step

__device__ __forceinline__ uint32_t ordered_key(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the workgroup (thread order).  `wave_tot` is LDS scratch of
// kSelWaves + 1 words.  Also returns the workgroup total through `total`.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t *wave_tot,
                                                         uint32_t &total)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();  // protects wave_tot from the previous call's readers
    if (lane == 63) wave_tot[wave] = x;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const uint32_t t = wave_tot[w];
        before += (w < wave) ? t : 0u;
        all += t;
    }
    total = all;
    return x + before;
}

__global__ __launch_bounds__(kSelectThreads) void select_kernel(const SelectPlan p)
{
    __shared__ uint32_t hist[4096];
    __shared__ uint32_t wave_tot[kSelWaves + 1];
    __shared__ uint32_t found[2];  // digit, remaining rank

    const int bg = blockIdx.x;
    const int b = bg / p.n_kv_heads;
    const int g = bg % p.n_kv_heads;
    const int tid = threadIdx.x;
    int32_t *dst = p.idx_out + (int64_t)bg * p.k;

    const int rgi = p.rindex[g];
    if (rgi == 0xFF) {
        const int32_t *src = p.idx_in + (int64_t)bg * p.k;
        for (int i = tid; i < p.k; i += kSelectThreads) dst[i] = src[i];
        return;
    }
    int L = p.lengths[b];
    L = L < 1 ? 1 : (L > p.max_len ? p.max_len : L);
    const int n = p.k < L ? p.k : L;
    if (n == L) {  // everything is selected
        for (int i = tid; i < p.k; i += kSelectThreads) dst[i] = i < L ? i : -1;
        return;
    }
    const float *sel = p.sel + ((int64_t)b * p.n_rgroups + rgi) * p.sel_stride;
    const float4 *sel4 = reinterpret_cast<const float4 *>(sel);

    // ---- radix select: find the n-th largest key ---------------------------------------
    uint32_t prefix = 0, prefix_mask = 0, need = (uint32_t)n;
    const int shifts[3] = {20, 10, 0};
    const int widths[3] = {12, 10, 10};
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = shifts[pass];
        const int n_bins = 1 << widths[pass];
        const uint32_t digit_mask = (uint32_t)n_bins - 1u;
        for (int i = tid; i < n_bins; i += kSelectThreads) hist[i] = 0;
        __syncthreads();
        for (int i0 = tid * 4; i0 < L; i0 += kTile) {
            const float4 x = sel4[i0 >> 2];  // rows are padded to a multiple of 4 floats
            const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t key = ordered_key(xs[j]);
                if (i0 + j < L && (key & prefix_mask) == prefix)
                    atomicAdd(&hist[(key >> shift) & digit_mask], 1u);
            }
        }
        __syncthreads();
        // Thread t owns `per` bins, taken from the top: its j-th bin is
        // n_bins-1 - (t*per + j).  An exclusive prefix over that order counts the keys in
        // strictly higher bins.
        const int per = n_bins / kSelectThreads > 0 ? n_bins / kSelectThreads : 1;
        uint32_t mine[4] = {0, 0, 0, 0};
        uint32_t sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = tid * per + j;
            if (j < per && r < n_bins) {
                mine[j] = hist[n_bins - 1 - r];
                sum += mine[j];
            }
        }
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(sum, wave_tot, total);
        uint32_t above = incl - sum;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = tid * per + j;
            if (j < per && r < n_bins) {
                if (above < need && need <= above + mine[j]) {
                    found[0] = (uint32_t)(n_bins - 1 - r);
                    found[1] = need - above;
                }
                above += mine[j];
            }
        }
        __syncthreads();
        prefix |= found[0] << shift;
        prefix_mask |= digit_mask << shift;
        need = found[1];
        __syncthreads();
    }
    const uint32_t T = prefix;  // the n-th largest key
    const uint32_t r_eq = need; // how many keys == T are kept (the lowest positions)

    // ---- ordered compaction -------------------------------------------------------------
    uint32_t base_gt = 0, base_eq = 0;
    for (int t0 = 0; t0 < L; t0 += kTile) {
        const int i0 = t0 + tid * 4;
        uint32_t gt = 0, eq = 0;
        if (i0 < L) {
            const float4 x = sel4[i0 >> 2];
            const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t key = ordered_key(xs[j]);
                const bool in = i0 + j < L;
                gt |= (uint32_t)(in && key > T) << j;
                eq |= (uint32_t)(in && key == T) << j;
            }
        }
        const uint32_t packed = (uint32_t)__builtin_popcount(gt) | ((uint32_t)__builtin_popcount(eq) << 16);
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(packed, wave_tot, total);
        const uint32_t excl = incl - packed;
        uint32_t n_gt = base_gt + (excl & 0xFFFFu);
        uint32_t n_eq = base_eq + (excl >> 16);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if ((gt >> j) & 1u) {
                dst[n_gt + (n_eq < r_eq ? n_eq : r_eq)] = i0 + j;
                ++n_gt;
            } else if ((eq >> j) & 1u) {
                if (n_eq < r_eq) dst[n_gt + n_eq] = i0 + j;
                ++n_eq;
            }
        }
        base_gt += total & 0xFFFFu;
        base_eq += total >> 16;
    }
    for (int i = n + tid; i < p.k; i += kSelectThreads) dst[i] = -1;
}

}  // namespace

hipError_t launch_select(const SelectPlan &plan, hipStream_t stream)
{
    hipLaunchKernelGGL(select_kernel, dim3(plan.batch * plan.n_kv_heads), dim3(kSelectThreads), 0,
                       stream, plan);
    return hipGetLastError();
}

}  // namespace lychee
