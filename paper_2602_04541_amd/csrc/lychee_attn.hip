// Attention-units kernel for gfx950 (CDNA4): the retrieval branch (Eq. 1, o = A V, and the
// pooled selection score that Eq. 2 ranks) and the sparse branch (Eq. 3) of Alg. 1's per-head
// loop, in one launch over a pooled list of equally sized work units.
//
// Work decomposition.  The paper's kernel pools the block work of full and sparse heads
// and cuts it into uniform splits (App. C); here a unit is `unit_r` consecutive cache rows of
// one (sequence, KV head) for that group's retrieval heads, or `unit_s` entries of the
// inherited set for that group's sparse heads.  One 256-thread workgroup runs one unit and
// leaves an un-normalised partial (running maximum, sum, weighted V sum) per head; the
// combine kernel merges the partials.
//
// Data path.  The cache is read exactly once per unit, straight from HBM into registers:
// a 64-lane wavefront covers 4 rows per load instruction (16 lanes x 16 bytes = one 256-byte
// row), 16 rows per iteration, with the next iteration's K and V rows already in flight while
// the current ones are consumed.  A row is shared by all heads of the group in registers, so
// nothing is staged in LDS; LDS only holds the unit's slice of the index set and the
// end-of-unit reduction.  Dot products use the packed bf16 dot instruction with fp32
// accumulation; the 16 lanes of a row are summed with a fixed DPP butterfly, so a key row
// gives a bit-identical score wherever it is processed (exact ties stay exact ties).
#include "lychee_internal.h"

namespace lychee {
namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

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

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u)
{
    return __builtin_bit_cast(float, u & 0xFFFF0000u);
}

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte streaming load: the cache rows are read once per step and never again.
__device__ __forceinline__ uint4 load_stream16(const uint16_t *p)
{
    const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
}

struct Tile {
    uint4 k[4];
    uint4 v[4];
    int valid;  // bit j: row slot j of this lane holds a real row
};

// Per-wavefront running state of the online softmax, one copy per row slot (lane >> 4).
template <int NH>
struct Acc {
    float o[NH][8];
    float m[NH];  // running maximum, raw dot-product units
    float l[NH];  // running sum of exp
};

template <int NH>
__device__ __forceinline__ void consume_tile(const Tile &t, const uint4 (&qf)[NH], Acc<NH> &acc,
                                             float c_log2e, float (&sel_sum)[4])
{
    float s[NH][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool ok = (t.valid >> j) & 1;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float a = dot2_bf16(t.k[j].x, qf[h].x, 0.0f);
            a = dot2_bf16(t.k[j].y, qf[h].y, a);
            a = dot2_bf16(t.k[j].z, qf[h].z, a);
            a = dot2_bf16(t.k[j].w, qf[h].w, a);
            s[h][j] = row16_sum(a);
        }
        float pooled = s[0][j];
#pragma unroll
        for (int h = 1; h < NH; ++h) pooled += s[h][j];
        sel_sum[j] = pooled;
#pragma unroll
        for (int h = 0; h < NH; ++h) s[h][j] = ok ? s[h][j] : -INFINITY;
    }

    // Raise the running maxima only when some row beats them (rare after the first tiles).
    bool grow = false;
    float mx[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        mx[h] = fmaxf(fmaxf(s[h][0], s[h][1]), fmaxf(s[h][2], s[h][3]));
        grow |= mx[h] > acc.m[h];
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const float m_new = fmaxf(acc.m[h], mx[h]);
            const float alpha = fast_exp2((acc.m[h] - m_new) * c_log2e);
            acc.m[h] = m_new;
            acc.l[h] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc.o[h][e] *= alpha;
        }
    }

    float p[NH][4];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        const float mc = -acc.m[h] * c_log2e;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            p[h][j] = fast_exp2(fmaf(s[h][j], c_log2e, mc));
            acc.l[h] += p[h][j];
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t w[4] = {t.v[j].x, t.v[j].y, t.v[j].z, t.v[j].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float v0 = bf16_lo(w[i]), v1 = bf16_hi(w[i]);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                acc.o[h][2 * i] = fmaf(p[h][j], v0, acc.o[h][2 * i]);
                acc.o[h][2 * i + 1] = fmaf(p[h][j], v1, acc.o[h][2 * i + 1]);
            }
        }
    }
}

// Tile buffers per wavefront: fewer heads leave more registers for loads in flight.
__host__ __device__ constexpr int ring_depth(int nh) { return nh == 1 ? 6 : (nh == 2 ? 5 : (nh == 3 ? 4 : 3)); }

// One unit.  GATHER = false: rows [r0, r1) of the cache (retrieval heads); true: entries
// [r0, r1) of the inherited set, staged in `idx_s` (sparse heads).
template <int NH, bool GATHER>
__device__ __forceinline__ void run_unit(const AttnPlan &p, int b, int g, int rg_index,
                                         uint32_t hmask, int split, int L, int r0, int r1,
                                         const int32_t *idx_s, float *red_o, float *red_ml)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rs = lane >> 4;  // row slot: which of the 4 rows of a load this lane is in
    const int c = lane & 15;   // 16-byte chunk of the 256-byte row

    int heads[NH];
    {
        uint32_t mk = hmask;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const int bit = __builtin_ctz(mk);
            mk &= mk - 1;
            heads[h] = g * p.group + bit;
        }
    }
    uint4 qf[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h)
        qf[h] = reinterpret_cast<const uint4 *>(
            p.q + ((int64_t)b * p.n_q_heads + heads[h]) * kHeadDim)[c];

    Acc<NH> acc;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        acc.m[h] = kMinusBig;
        acc.l[h] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc.o[h][e] = 0.0f;
    }

    const uint16_t *kbase = p.k_cache + (int64_t)b * p.stride_b + (int64_t)g * p.stride_h;
    const uint16_t *vbase = p.v_cache + (int64_t)b * p.stride_b + (int64_t)g * p.stride_h;
    const float c_log2e = p.scale_log2e;
    const float sel_mul = p.scale / (float)NH;
    float *sel_row = nullptr;
    if (!GATHER && p.emit_sel)
        sel_row = p.sel + ((int64_t)b * p.n_rgroups + rg_index) * p.sel_stride;

    const int n_rows = r1 - r0;
    const int n_tiles = (n_rows + kTileRows - 1) / kTileRows;

    auto issue = [&](Tile &t, int tile) {
        const int base = r0 + tile * kTileRows;
        t.valid = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = base + 4 * j + rs;
            int row;
            bool ok;
            if (GATHER) {
                const int tpos = (r < r1) ? idx_s[r - r0] : -1;
                ok = (tpos >= 0) && (tpos < L);
                row = ok ? tpos : 0;
            } else {
                ok = r < r1;
                row = ok ? r : (r1 > 0 ? r1 - 1 : 0);
            }
            t.valid |= (ok ? 1 : 0) << j;
            const int64_t off = (int64_t)row * p.stride_t;
            t.k[j] = load_stream16(kbase + off + c * 8);
            t.v[j] = load_stream16(vbase + off + c * 8);
        }
    };
    auto consume = [&](const Tile &t, int tile) {
        float sel_sum[4];
        consume_tile<NH>(t, qf, acc, c_log2e, sel_sum);
        if (!GATHER && sel_row != nullptr) {
            // lane c (< 4) of each row slot stores the score of row 4*c + rs of the tile
            float mine = sel_sum[0];
            mine = (c == 1) ? sel_sum[1] : mine;
            mine = (c == 2) ? sel_sum[2] : mine;
            mine = (c == 3) ? sel_sum[3] : mine;
            const int r = r0 + tile * kTileRows + 4 * c + rs;
            if (c < 4 && r < r1) sel_row[r] = mine * sel_mul + 0.0f;  // +0 turns -0 into +0
        }
    };

    // Wavefront w takes tiles w, w+4, ...; a ring of kDepth tile buffers keeps kDepth-1
    // tiles' loads in flight while one tile is consumed.
    constexpr int kDepth = ring_depth(NH);
    Tile ring[kDepth];
    const int n_mine = n_tiles > wave ? (n_tiles - wave + kAttnWaves - 1) / kAttnWaves : 0;
    // Loads are issued unconditionally (a tile past the end re-reads the unit's last row and
    // is marked invalid): a conditional refill would make the ring registers loop-carried
    // through a copy, and the copy would have to wait for the load it copies.
#pragma unroll
    for (int d = 0; d < kDepth; ++d) issue(ring[d], wave + d * kAttnWaves);
    for (int i = 0; i < n_mine; i += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            if (i + d < n_mine) consume(ring[d], wave + (i + d) * kAttnWaves);
            __builtin_amdgcn_sched_barrier(0);
            issue(ring[d], wave + (i + d + kDepth) * kAttnWaves);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // Merge the 4 row slots of the wavefront (lanes l, l^16, l^32, l^48).
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        float mw = fmaxf(acc.m[h], __shfl_xor(acc.m[h], 16));
        mw = fmaxf(mw, __shfl_xor(mw, 32));
        const float a = fast_exp2((acc.m[h] - mw) * c_log2e);
        acc.m[h] = mw;
        float lw = acc.l[h] * a;
        lw += __shfl_xor(lw, 16);
        lw += __shfl_xor(lw, 32);
        acc.l[h] = lw;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float ow = acc.o[h][e] * a;
            ow += __shfl_xor(ow, 16);
            ow += __shfl_xor(ow, 32);
            acc.o[h][e] = ow;
        }
    }
    // Merge the 4 wavefronts through LDS and write the unit's partial.
    if (rs == 0) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float *dst = red_o + (wave * kMaxGroup + h) * kHeadDim + c * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e] = acc.o[h][e];
            if (c == 0) {
                red_ml[(wave * kMaxGroup + h) * 2 + 0] = acc.m[h];
                red_ml[(wave * kMaxGroup + h) * 2 + 1] = acc.l[h];
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < kHeadDim) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float M = kMinusBig;
#pragma unroll
            for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, red_ml[(w * kMaxGroup + h) * 2]);
            float o = 0.0f, l = 0.0f;
#pragma unroll
            for (int w = 0; w < kAttnWaves; ++w) {
                const float a = fast_exp2((red_ml[(w * kMaxGroup + h) * 2] - M) * c_log2e);
                o = fmaf(a, red_o[(w * kMaxGroup + h) * kHeadDim + threadIdx.x], o);
                l = fmaf(a, red_ml[(w * kMaxGroup + h) * 2 + 1], l);
            }
            const int64_t prow = ((int64_t)b * p.n_q_heads + heads[h]) * p.s_max + split;
            p.part_o[prow * kHeadDim + threadIdx.x] = o;
            if (threadIdx.x == 0) {
                p.part_ml[prow * 2 + 0] = M;
                p.part_ml[prow * 2 + 1] = l;
            }
        }
    }
}

__global__ __launch_bounds__(kAttnThreads) void attn_units_kernel(const AttnPlan p)
{
    __shared__ int32_t idx_s[kMaxSparseUnit];
    __shared__ float red_o[kAttnWaves * kMaxGroup * kHeadDim];
    __shared__ float red_ml[kAttnWaves * kMaxGroup * 2];

    int u = blockIdx.x;
    const int n_r_units = p.batch * p.n_rgroups * p.nsplit_r;
    const uint32_t gmask = (1u << p.group) - 1u;
    bool gather;
    int b, gi, split, g, unit;
    uint32_t hmask;
    if (u < n_r_units) {
        gather = false;
        split = u % p.nsplit_r;
        gi = (u / p.nsplit_r) % p.n_rgroups;
        b = u / (p.nsplit_r * p.n_rgroups);
        g = p.rgroup[gi];
        hmask = p.rmask[g] & gmask;
        unit = p.unit_r;
    } else {
        u -= n_r_units;
        gather = true;
        split = u % p.nsplit_s;
        gi = (u / p.nsplit_s) % p.n_sgroups;
        b = u / (p.nsplit_s * p.n_sgroups);
        g = p.sgroup[gi];
        hmask = ~(uint32_t)p.rmask[g] & gmask;
        unit = p.unit_s;
    }
    int L = p.lengths[b];
    L = L < 1 ? 1 : (L > p.max_len ? p.max_len : L);
    const int limit = gather ? (p.k < L ? p.k : L) : L;  // a set holds at most min(k, L) entries
    int r0 = split * unit;
    int r1 = r0 + unit;
    r1 = r1 < limit ? r1 : limit;
    if (r0 > r1) r0 = r1;  // an empty unit still writes its (empty) partial

    if (gather) {
        const int32_t *src = p.idx_in + ((int64_t)b * p.n_kv_heads + g) * p.k;
        for (int i = threadIdx.x; i < r1 - r0; i += kAttnThreads) idx_s[i] = src[r0 + i];
        __syncthreads();
    }

    const int nh = __builtin_popcount(hmask);
    if (gather) {
        switch (nh) {
        case 1: run_unit<1, true>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        case 2: run_unit<2, true>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        case 3: run_unit<3, true>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        default: run_unit<4, true>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        }
    } else {
        switch (nh) {
        case 1: run_unit<1, false>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        case 2: run_unit<2, false>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        case 3: run_unit<3, false>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        default: run_unit<4, false>(p, b, g, gi, hmask, split, L, r0, r1, idx_s, red_o, red_ml); break;
        }
    }
}

}  // namespace

hipError_t launch_attn_units(const AttnPlan &plan, hipStream_t stream)
{
    const int n_units = plan.batch * (plan.n_rgroups * plan.nsplit_r + plan.n_sgroups * plan.nsplit_s);
    if (n_units <= 0) return hipSuccess;
    hipLaunchKernelGGL(attn_units_kernel, dim3(n_units), dim3(kAttnThreads), 0, stream, plan);
    return hipGetLastError();
}

}  // namespace lychee
