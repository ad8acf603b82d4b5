// C, T, S and A units (included by lychee_units.hip and lychee_layer.hip): the log-sum-exp merge of partials, the
// sampled selection threshold, the exact radix select of Eq. 2 with the Ratio, Threshold and Top-p
// rules of Sec. 4.4.1, the set copies, and the cache append of Alg. 1.
#pragma once
#include "lychee_device.h"

namespace lychee {
namespace {

// ------------------------------------------------------------------------------ C
// out = (sum_s w_s o_s) / (sum_s w_s l_s),  w_s = 2^((m_s - M) log2(e)/sqrt(d)),  M = max_s m_s,
// over the head's partial slots in ascending order (a fixed summation tree).
// `known_count` >= 0: the number of partial slots, known to the caller; else it is read from part_count.
template <typename Pool>
__device__ __forceinline__ void combine_unit(const Common &c, const LayerDesc &p, int bh, SharedCombine &sh,
                                             Pool &pool, int known_count = -1)
{
    int count = known_count >= 0 ? known_count : gload(p.part_count + bh);
    count = count < 0 ? 0 : (count > c.part_stride ? c.part_stride : count);
    const float *ml = p.part_ml + (int64_t)bh * c.part_stride * 2;
    const float *po = p.part_o + (int64_t)bh * c.part_stride * kHeadDim;
    float m_loc = kMinusBig;
    for (int s = threadIdx.x; s < count; s += kThreads)
        if (gload(ml + 2 * s + 1) > 0.0f) m_loc = fmaxf(m_loc, gload(ml + 2 * s));
    const float M = block_max(m_loc, pool.fred);
    float l_loc = 0.0f;
    for (int s = threadIdx.x; s < count; s += kThreads) {
        const float ls = gload(ml + 2 * s + 1);
        const float w = ls > 0.0f ? fast_exp2((gload(ml + 2 * s) - M) * c.scale_log2e) : 0.0f;
        sh.w[s] = w;
        l_loc = fmaf(w, ls, l_loc);
    }
    const float lsum = block_sum(l_loc, pool.fred);  // also publishes sh.w
    constexpr int kLanes = kThreads / 32;  // interleaved slot subsets
    const int lane8 = threadIdx.x >> 5;
    const int c4 = threadIdx.x & 31;       // which 4 columns
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = lane8; s0 < count; s0 += 8 * kLanes) {
        // 8 slots per thread and round, all loads issued before the first use
        float wv[8];
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int s = s0 + kLanes * u;
            wv[u] = s < count ? sh.w[s] : 0.0f;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (wv[u] > 0.0f) v[u] = gload_f4(po + (int64_t)s * kHeadDim + c4 * 4);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc.x = fmaf(wv[u], v[u].x, acc.x);
            acc.y = fmaf(wv[u], v[u].y, acc.y);
            acc.z = fmaf(wv[u], v[u].z, acc.z);
            acc.w = fmaf(wv[u], v[u].w, acc.w);
        }
    }
    reinterpret_cast<float4 *>(sh.red + lane8 * kHeadDim)[c4] = acc;
    __syncthreads();
    if (threadIdx.x < kHeadDim) {
        float o = 0.0f;
#pragma unroll
        for (int i = 0; i < kLanes; ++i) o += sh.red[i * kHeadDim + threadIdx.x];
        const float r = lsum > 0.0f ? o / lsum : 0.0f;
        gstore(p.out + (int64_t)bh * kHeadDim + threadIdx.x, f32_to_bf16_rne(r));
    }
    __syncthreads();
}

// The same merge for all NH heads of a segment at once, by the workgroup that has just written the
// segment's last partial: every load of a group of slots - the (m, l) pairs and the partial
// outputs of all heads - is issued before the first one is used, so that a group costs about one
// round trip to memory however many heads it has (the heads one after the other, each with its
// own rounds of dependent loads, took 20 us for the four heads of a dense layer's segment).  A
// group is 64 slots for one or two heads and 32 for three or four: 64 registers of loads in
// flight either way.  Each wavefront keeps the running maximum and sum of every head itself
// (redundantly: no barrier between groups); thread (o8, c4) sums slots o8, o8 + 8, ... of a
// group for columns 4 c4 .. 4 c4 + 3, and the eight sums per column are added in a fixed order
// at the end.
template <int NH>
__device__ __forceinline__ void combine_segment(const Common &c, const LayerDesc &p, int b, int g, uint32_t hmask,
                                                int count, SharedCombine &sh)
{
    constexpr int kU = NH <= 2 ? 8 : 4;  // slots per thread and group
    constexpr int kSlots = 8 * kU;       // slots per group
    const int lane = threadIdx.x & 63;
    const int o8 = threadIdx.x >> 5;  // which eighth of a group's slots
    const int c4 = threadIdx.x & 31;  // which 4 columns
    int64_t bh[NH];
    {
        uint32_t mk = hmask;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            bh[h] = (int64_t)b * c.n_q_heads + g * c.group + __builtin_ctz(mk);
            mk &= mk - 1;
        }
    }
    float M[NH], Ls[NH];
    float4 acc[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        M[h] = kMinusBig;
        Ls[h] = 0.0f;
        acc[h] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int s0 = 0; s0 < count; s0 += kSlots) {
        float2 ml[NH];
        float4 v[NH][kU];
        const bool mine = lane < kSlots && s0 + lane < count;  // this lane holds a slot of the group
        const int sl = mine ? s0 + lane : count - 1;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const float *pm = p.part_ml + (bh[h] * c.part_stride + sl) * 2;
            ml[h] = make_float2(gload(pm), gload(pm + 1));
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                int s = s0 + o8 + 8 * u;
                s = s < count ? s : count - 1;
                v[h][u] = gload_f4(p.part_o + (bh[h] * c.part_stride + s) * kHeadDim + c4 * 4);
            }
        }
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const bool live = mine && ml[h].y > 0.0f;  // (a piece without a valid row leaves l = 0)
            float mg = live ? ml[h].x : kMinusBig;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) mg = fmaxf(mg, __shfl_xor(mg, d));
            const float m_new = fmaxf(M[h], mg);
            const float alpha = fast_exp2((M[h] - m_new) * c.scale_log2e);
            M[h] = m_new;
            const float wl = live ? fast_exp2((ml[h].x - m_new) * c.scale_log2e) : 0.0f;  // this lane's slot
            float lg = wl * ml[h].y;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) lg += __shfl_xor(lg, d);
            Ls[h] = Ls[h] * alpha + lg;
            acc[h].x *= alpha, acc[h].y *= alpha, acc[h].z *= alpha, acc[h].w *= alpha;
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const float wu = __shfl(wl, o8 + 8 * u);  // (slots past the end carry weight 0)
                acc[h].x = fmaf(wu, v[h][u].x, acc[h].x);
                acc[h].y = fmaf(wu, v[h][u].y, acc[h].y);
                acc[h].z = fmaf(wu, v[h][u].z, acc[h].z);
                acc[h].w = fmaf(wu, v[h][u].w, acc[h].w);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        reinterpret_cast<float4 *>(sh.red + (h * 8 + o8) * kHeadDim)[c4] = acc[h];
        if (threadIdx.x == 0) sh.l[h] = Ls[h];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < NH * kHeadDim; i += kThreads) {
        const int h = i / kHeadDim, col = i % kHeadDim;
        float o = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) o += sh.red[(h * 8 + j) * kHeadDim + col];
        const float l = sh.l[h];
        // (bh[h] with a run-time h: picked without indexing the register array)
        int64_t row = bh[0];
#pragma unroll
        for (int hh = 1; hh < NH; ++hh) row = h == hh ? bh[hh] : row;
        gstore(p.out + row * kHeadDim + col, f32_to_bf16_rne(l > 0.0f ? o / l : 0.0f));
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------ T and S
// In the histogram of `n_bins` digits, finds the highest digit d whose suffix count
// (keys with digit >= d) reaches `need`; returns d and need minus the count above d.
template <int kBins>
__device__ __forceinline__ void find_digit(const uint32_t *hist, uint32_t need, uint32_t *found,
                                           uint32_t *scan_scratch, uint32_t &digit, uint32_t &rest)
{
    constexpr int per = kBins / kThreads;
    uint32_t mine[per];
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {
        mine[j] = hist[kBins - 1 - (threadIdx.x * per + j)];  // bins taken from the top
        sum += mine[j];
    }
    uint32_t total;
    uint32_t above = block_scan(sum, scan_scratch, total) - sum;
    if (threadIdx.x == 0) {
        found[0] = 0;      // need > total: every key qualifies
        found[1] = need;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < per; ++j) {
        if (above < need && need <= above + mine[j]) {
            found[0] = (uint32_t)(kBins - 1 - (threadIdx.x * per + j));
            found[1] = need - above;
        }
        above += mine[j];
    }
    __syncthreads();
    digit = found[0];
    rest = found[1];
    __syncthreads();
}

template <int NH>
__device__ __forceinline__ void load_q(const Common &c, const uint16_t *q, int b, int g, uint32_t hmask,
                                       uint4 (&qf)[NH])
{
    const int ch = threadIdx.x & 15;
    uint32_t mk = hmask;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        const int bit = __builtin_ctz(mk);
        mk &= mk - 1;
        qf[h] = gload_u4(q + ((int64_t)b * c.n_q_heads + g * c.group + bit) * kHeadDim + ch * 8);
    }
}

// Pooled scores of the 16 rows base .. base+15 of one KV head (rows past L-1 repeat row L-1);
// afterwards lane (rs, ch) with ch < 4 holds the score of row base + 4*ch + rs.
template <int NH>
__device__ __forceinline__ float tile_pooled_score(const uint4 (&kr)[4], const uint4 (&qf)[NH], float sel_mul)
{
    const int ch = threadIdx.x & 15;
    float mine = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float pooled = row_score(kr[j], qf[0]);
#pragma unroll
        for (int h = 1; h < NH; ++h) pooled += row_score(kr[j], qf[h]);
        mine = (ch == j) ? sel_value(pooled, sel_mul) : mine;
    }
    return mine;
}

// T unit of score row (b, rgi): the ordered key that a row's pooled score has to reach to
// become a candidate.  The key is the target-th largest of a sample of the row's scores,
// to 22 bits, where target is the number of sampled rows expected among the top n = min(k, L)
// plus sel_margin (six, unless the caller changes it) standard deviations; the streamed rows
// that reach it are then very likely at least n and a few thousand more at most.  Whatever the sample yields, the select unit
// checks the candidate count and ranks the whole row itself when the list cannot be used.
// The sample is one row at a hashed offset inside each of 2048 to 4096 equal strata.
// `publish` != nullptr (launches whose streaming runs beside this unit): the threshold goes, with
// the launch's generation `gen` in the upper half, into *publish by one 64-bit atomic store, which
// the row's pieces poll; the candidate counter is not touched (it is zero between uses, and the
// pieces may already be counting).
// `split` (launches whose streaming waits for the threshold): the row's sample is dealt to n_sub
// units, each of which reads its share of the rows in one round of loads and leaves the keys in
// device memory; the unit that arrives last ranks them.  Nobody waits for anybody.
struct ThrSplit {
    int sub = 0, n_sub = 1;
    uint32_t *keys = nullptr;     // [sample size] scratch of this score row
    uint32_t *arrived = nullptr;  // units of this row that have left their keys (zero between launches)
};
template <int NH, typename Pool>
__device__ __forceinline__ void threshold_unit(const Common &c, const LayerDesc &p, int b, int rgi,
                                               SharedSelect &sh, Pool &pool, unsigned long long *publish = nullptr,
                                               uint32_t gen = 0, const ThrSplit split = ThrSplit())
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rs = lane >> 4;
    const int ch = lane & 15;
    const int L = pool.len[b];  // staged by the kernel, clamped
    const int n = budget_of(c, L);
    const int64_t row = (int64_t)b * p.n_rgroups + rgi;
    auto emit = [&](uint32_t key) {
        if (threadIdx.x != 0) return;
        if (publish != nullptr)
            __hip_atomic_store((LYCHEE_GLOBAL unsigned long long *)publish, ((unsigned long long)gen << 32) | key,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            gstore(p.thr + row, key);
    };
    if (publish == nullptr && threadIdx.x == 0) gstore(p.list_count + row, (int32_t)0);
    if (split.sub == 0 && p.q_keep != nullptr && (int)threadIdx.x < c.group * (kHeadDim / 8)) {
        // the group's query rows (consecutive heads, 16 chunks of 16 bytes each)
        const int64_t at = ((int64_t)b * c.n_q_heads + p.rgroup[rgi] * c.group) * kHeadDim + threadIdx.x * 8;
        *(LYCHEE_GLOBAL u32x4_t *)(p.q_keep + at) = *(const LYCHEE_GLOBAL u32x4_t *)(p.q + at);
    }
    if (n == L || L <= kDirectLen || 2 * (int64_t)n >= L) {
        // everything is selected anyway (no candidates wanted), or every row is a candidate
        // (a probability rule may keep fewer than everything: it still needs the candidates)
        if (split.sub == 0) emit(n == L && c.prob_rule == 0 ? 0xFFFFFFFFu : 0u);
        return;
    }
    int n_tiles = L / 1024;
    n_tiles = n_tiles < kSampleTilesMin ? kSampleTilesMin : (n_tiles > kSampleTilesMax ? kSampleTilesMax : n_tiles);
    const int n_sample = n_tiles * 16;
    const int g = p.rgroup[rgi];
    const uint32_t hmask = p.rmask[g] & ((1u << c.group) - 1u);
    uint4 qf[NH];
    load_q<NH>(c, p.q, b, g, hmask, qf);
    const uint16_t *kbase = p.k_cache + (int64_t)b * c.stride_b + (int64_t)g * c.stride_h;
    const float sel_mul = c.scale / (float)NH;
    for (int i = threadIdx.x; i < 4096; i += kThreads) sh.hist[i] = 0;
    __syncthreads();

    constexpr int kBatch = 8;  // groups of 16 sampled rows a wavefront has in flight
    // One row at a hashed offset in each of n_sample equal strata of rows 0 .. L-2 (the newest
    // row may be being appended in this very launch).  Row by row, not tile by tile: scores
    // come in runs (a passage that matters is hundreds of consecutive rows), and a sample of
    // contiguous tiles would over- or under-count such runs far beyond its nominal deviation.
    const int stratum = (L - 1) / n_sample;  // >= 2
    const int t_lo = n_tiles * split.sub / split.n_sub, t_hi = n_tiles * (split.sub + 1) / split.n_sub;
    for (int t0 = t_lo + wave * kBatch; t0 < t_hi; t0 += kWaves * kBatch) {
        uint4 kr[kBatch][4];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int t = t0 + u < t_hi ? t0 + u : t_hi - 1;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = t * 16 + 4 * j + rs;  // sample number
                const uint32_t hsh = ((uint32_t)i * 2654435761u + (uint32_t)row * 40503u) >> 12;
                const int pos = i * stratum + (int)(hsh % (uint32_t)stratum);
                kr[u][j] = gload_u4(kbase + (int64_t)pos * c.stride_t + ch * 8);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const uint32_t key = ordered_key(tile_pooled_score<NH>(kr[u], qf, sel_mul));
            if (t0 + u < t_hi && ch < 4) {
                if (split.n_sub > 1) {
                    gstore_through(split.keys + (t0 + u) * 16 + 4 * ch + rs, key);
                } else {
                    sh.samp[(t0 + u) * 16 + 4 * ch + rs] = key;
                    atomicAdd(&sh.hist[key >> 20], 1u);
                }
            }
        }
    }
    if (split.n_sub > 1) {
        // leave the keys, count this unit in; the last one to arrive goes on with all of them
        wait_stores();
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t old = __hip_atomic_fetch_add((LYCHEE_GLOBAL uint32_t *)split.arrived, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
            const bool last = old == (uint32_t)split.n_sub - 1u;
            if (last) __hip_atomic_store((LYCHEE_GLOBAL uint32_t *)split.arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh.found[0] = last;
        }
        __syncthreads();
        const bool last = sh.found[0] != 0;
        __syncthreads();
        if (!last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        for (int i = threadIdx.x; i < n_sample; i += kThreads) {
            const uint32_t key = gload(split.keys + i);
            sh.samp[i] = key;
            atomicAdd(&sh.hist[key >> 20], 1u);
        }
    }
    __syncthreads();
    const float f = (float)n_sample * (float)n / (float)L;
    const float want = f + c.sel_margin * sqrtf(f) + 6.0f;
    const uint32_t target = want < 1.0f ? 1u : (want > (float)n_sample ? (uint32_t)n_sample : (uint32_t)want);
    uint32_t t_key = 0;
    if (target < (uint32_t)n_sample) {
        // the sample's target-th largest key: top 12 bits, then the next 10
        uint32_t d1, rest1, d2, rest2;
        find_digit<4096>(sh.hist, target, sh.found, pool.scan, d1, rest1);
        for (int i = threadIdx.x; i < 1024; i += kThreads) sh.hist[i] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < n_sample; i += kThreads) {
            const uint32_t key = sh.samp[i];
            if ((key >> 20) == d1) atomicAdd(&sh.hist[(key >> 10) & 1023u], 1u);
        }
        __syncthreads();
        find_digit<1024>(sh.hist, rest1, sh.found, pool.scan, d2, rest2);
        t_key = (d1 << 20) | (d2 << 10);
    }
    emit(t_key);
}

// Writes the pooled score of every row of (b, g) into sel[0 .. L): what the select unit falls
// back on when a row's candidate list is short of n entries or has overflowed.
template <int NH>
__device__ __forceinline__ void score_row_unit(const Common &c, const LayerDesc &p, int b, int g, int L, float *sel)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rs = lane >> 4;
    const int ch = lane & 15;
    const uint32_t hmask = p.rmask[g] & ((1u << c.group) - 1u);
    uint4 qf[NH];
    load_q<NH>(c, p.q, b, g, hmask, qf);
    const uint16_t *kbase = p.k_cache + (int64_t)b * c.stride_b + (int64_t)g * c.stride_h;
    const float sel_mul = c.scale / (float)NH;
    const int n_tiles = (L + 15) / 16;
    constexpr int kBatch = 4;
    for (int t0 = wave * kBatch; t0 < n_tiles; t0 += kWaves * kBatch) {
        uint4 kr[kBatch][4];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int r = (t0 + u) * 16 + 4 * j + rs;
                r = r < L ? r : L - 1;
                kr[u][j] = gload_u4(kbase + (int64_t)r * c.stride_t + ch * 8);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float v = tile_pooled_score<NH>(kr[u], qf, sel_mul);
            const int r = (t0 + u) * 16 + 4 * ch + rs;
            if (ch < 4 && r < L) gstore(sel + r, v);
        }
    }
}

// The three sources of (ordered key, position) entries the select unit ranks.  for_each may
// also hand out "no entry" (position kNoEntry).  The visitors below fold everything that
// decides whether an entry counts into one flag, with bitwise operators, and guard a single
// LDS operation with it: short-circuit conditions made the compiler keep a lane mask per entry
// and condition, spill them, and branch several times per entry.
constexpr uint32_t kNoEntry = 0xFFFFFFFFu;
constexpr int kSelRegs = 40;  // entries one thread keeps in registers
struct RegEntries {           // up to kThreads * kSelRegs list entries, loaded once
    uint32_t key[kSelRegs], pos[kSelRegs];
    __device__ __forceinline__ void load(const unsigned long long *list, int total)
    {
#pragma unroll
        for (int e = 0; e < kSelRegs; ++e) {
            const int i = threadIdx.x + e * kThreads;
            const unsigned long long v = gload(list + (i < total ? i : 0));  // total >= 1
            key[e] = (uint32_t)v;
            pos[e] = i < total ? (uint32_t)(v >> 32) : kNoEntry;
        }
    }
    template <typename F>
    __device__ __forceinline__ void for_each(F f) const
    {
#pragma unroll
        for (int e = 0; e < kSelRegs; ++e) f(key[e], pos[e]);
    }
};
struct ListEntries {          // a longer list, read from memory on every pass
    const unsigned long long *list;
    int total;
    template <typename F>
    __device__ __forceinline__ void for_each(F f) const
    {
        for (int i0 = threadIdx.x; i0 < total; i0 += 8 * kThreads) {
            unsigned long long v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kThreads;
                v[u] = gload(list + (i < total ? i : total - 1));  // unconditional: the loads overlap
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                f((uint32_t)v[u], i0 + u * kThreads < total ? (uint32_t)(v[u] >> 32) : kNoEntry);
        }
    }
};
struct RowEntries {           // every row of the sequence, from its recomputed scores
    const float *sel;
    int total;
    template <typename F>
    __device__ __forceinline__ void for_each(F f) const
    {
        for (int i0 = threadIdx.x; i0 < total; i0 += 8 * kThreads) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kThreads;
                v[u] = gload(sel + (i < total ? i : total - 1));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * kThreads;
                f(ordered_key(v[u]), i < total ? (uint32_t)i : kNoEntry);
            }
        }
    }
};

// The `need`-th largest of the 32-bit values val(key, pos) over the entries that pass
// `among`, by radix select (12 + 10 + 10 bits); `rest` = how many entries equal to the
// result are among the `need` largest.
template <typename Entries, typename Val, typename Among, typename Pool>
__device__ __forceinline__ uint32_t radix_select(const Entries &E, uint32_t need, Val val, Among among,
                                                 uint32_t &rest, SharedSelect &sh, Pool &pool)
{
    uint32_t prefix = 0, prefix_mask = 0;
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
        const int n_bins = pass == 0 ? 4096 : 1024;
        const uint32_t digit_mask = (uint32_t)n_bins - 1u;
        for (int i = threadIdx.x; i < n_bins; i += kThreads) sh.hist[i] = 0;
        __syncthreads();
        E.for_each([&](uint32_t key, uint32_t pos) {
            const uint32_t v = val(key, pos);
            const bool in = (pos != kNoEntry) & among(key, pos) & ((v & prefix_mask) == prefix);
            if (in) atomicAdd(&sh.hist[(v >> shift) & digit_mask], 1u);
        });
        __syncthreads();
        uint32_t digit, left;
        if (pass == 0)
            find_digit<4096>(sh.hist, need, sh.found, pool.scan, digit, left);
        else
            find_digit<1024>(sh.hist, need, sh.found, pool.scan, digit, left);
        prefix |= digit << shift;
        prefix_mask |= digit_mask << shift;
        need = left;
    }
    rest = need;
    return prefix;
}

// Exact top-n of the entries by key, ties to the lower position (Eq. 2), written to dst in
// ascending position order.  The entries may come in any order: the n-th largest key T and the
// number r_eq of entries equal to T that belong to the top n come from a radix select; when
// more than r_eq entries equal T, a second radix select finds the r_eq-th lowest position
// among them; the chosen positions are then marked in an LDS bitmap, 131072 positions at a
// time, and read back in order.
template <typename Entries, typename Pool>
__device__ __forceinline__ void select_from(const Entries &E, int n, int L, int32_t *dst, SharedSelect &sh,
                                            Pool &pool)
{
    uint32_t r_eq;
    const uint32_t T = radix_select(
        E, (uint32_t)n, [](uint32_t key, uint32_t) { return key; }, [](uint32_t, uint32_t) { return true; }, r_eq,
        sh, pool);
    uint32_t my_eq = 0;
    E.for_each([&](uint32_t key, uint32_t pos) { my_eq += (uint32_t)((key == T) & (pos != kNoEntry)); });
    uint32_t n_eq;
    (void)block_scan(my_eq, pool.scan, n_eq);
    uint32_t pos_cut = 0xFFFFFFFEu;  // entries equal to T are taken up to this position
    if (r_eq < n_eq) {
        uint32_t unused;
        pos_cut = ~radix_select(
            E, r_eq, [](uint32_t, uint32_t pos) { return ~pos; }, [&](uint32_t key, uint32_t) { return key == T; },
            unused, sh, pool);
    }
    constexpr uint32_t kWindow = 4096u * 32u;
    constexpr int kPer = 4096 / kThreads;
    uint32_t base = 0;
    for (uint32_t w0 = 0; w0 < (uint32_t)L; w0 += kWindow) {
        for (int i = threadIdx.x; i < 4096; i += kThreads) sh.hist[i] = 0;
        __syncthreads();
        E.for_each([&](uint32_t key, uint32_t pos) {
            const uint32_t rel = pos - w0;  // "no entry" lies outside every window
            const bool take = ((key > T) | ((key == T) & (pos <= pos_cut))) & (rel < kWindow);
            if (take) atomicOr(&sh.hist[rel >> 5], 1u << (rel & 31u));
        });
        __syncthreads();
        // Thread t counts bitmap words 16 t .. 16 t + 15; the scan gives the output rank of every
        // run of 16 words and, inside a run, of every word.
        uint32_t cnt = 0;
#pragma unroll 4
        for (int j = 0; j < kPer; ++j) {
            sh.word_at[threadIdx.x * kPer + j] = (uint16_t)cnt;  // (at most 16 * 32 positions before it)
            cnt += (uint32_t)__builtin_popcount(sh.hist[threadIdx.x * kPer + j]);
        }
        uint32_t tot;
        const uint32_t at0 = base + block_scan(cnt, pool.scan, tot) - cnt;
        sh.chunk_at[threadIdx.x] = at0;
        __syncthreads();
        // The positions are put in order in LDS, kStage at a time, and copied out with coalesced
        // write-through stores: the set is in device memory once the unit's stores have
        // completed, whoever reads it next (a gather piece of the same launch, on another XCD,
        // after an acquire), and a store per position from every lane's own bit loop took four
        // times as long beside a streaming launch as it does alone.  Here thread t takes words
        // t, t + 256, ...: selected positions come in clusters (the newest rows, a few hot spans),
        // and a thread that held 16 neighbouring words would walk a cluster's hundreds of bits
        // alone while the others wait.
        constexpr uint32_t kStage = (uint32_t)(sizeof(sh.samp) / sizeof(sh.samp[0]));
        uint32_t end = base + tot;
        end = end < (uint32_t)n ? end : (uint32_t)n;
        for (uint32_t c0 = base; c0 < end; c0 += kStage) {
            // (eight words at a time: their LDS reads overlap instead of each waiting in its own branch)
#pragma unroll 1
            for (int j0 = 0; j0 < kPer; j0 += 8) {
                uint32_t wd[8], at[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint32_t wi = (uint32_t)(j0 + u) * kThreads + threadIdx.x;
                    wd[u] = sh.hist[wi];
                    at[u] = sh.chunk_at[wi / kPer] + sh.word_at[wi] - c0;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint32_t first = w0 + ((uint32_t)(j0 + u) * kThreads + threadIdx.x) * 32u;
                    while (wd[u] != 0) {
                        const uint32_t bit = (uint32_t)__builtin_ctz(wd[u]);
                        wd[u] &= wd[u] - 1u;
                        if (at[u] < kStage) sh.samp[at[u]] = first + bit;
                        ++at[u];
                    }
                }
            }
            __syncthreads();
            const uint32_t m = end - c0 < kStage ? end - c0 : kStage;
            for (uint32_t i = threadIdx.x; i < m; i += kThreads) gstore_through(dst + c0 + i, (int32_t)sh.samp[i]);
            __syncthreads();
        }
        base += tot;
    }
}

// A unit of one layer (Alg. 1, "C.append(k, v)"): the decoded token's key and value rows become
// row L_b - 1 of every KV head's cache.  16 lanes move one 256-byte row.
__device__ __forceinline__ void append_unit(const Common &c, const LayerDesc &p)
{
    const int ch = threadIdx.x & 15;
    const int n_rows = c.batch * c.n_kv_heads * 2;  // K rows, then V rows
    for (int r = threadIdx.x >> 4; r < n_rows; r += kThreads >> 4) {
        const int which = r / (c.batch * c.n_kv_heads);
        const int bg = r % (c.batch * c.n_kv_heads);
        const int b = bg / c.n_kv_heads, g = bg % c.n_kv_heads;
        const int L = clamp_len(c.lengths[b], c.max_len);
        const uint16_t *src = (which ? p.v_new : p.k_new) + (int64_t)bg * kHeadDim + ch * 8;
        const uint16_t *dst = (which ? p.v_cache : p.k_cache) + (int64_t)b * c.stride_b +
                              (int64_t)g * c.stride_h + (int64_t)(L - 1) * c.stride_t + ch * 8;
        const uint4 v = gload_u4(src);
        *(LYCHEE_GLOBAL u32x4_t *)const_cast<uint16_t *>(dst) = u32x4_t{v.x, v.y, v.z, v.w};
    }
}

// ---- the probability rules of Sec. 4.4.1 (Threshold, Top-p): how many entries to keep
// The pooled logit an ordered key stands for.
__device__ __forceinline__ float key_score(uint32_t key)
{
    return __builtin_bit_cast(float, (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

// Probability of a pooled logit under the softmax over the whole sequence, as a 40-bit
// fixed-point number: sums of these are integer sums, the same in any order.
constexpr float kMassOne = 1099511627776.0f;  // 2^40
__device__ __forceinline__ unsigned long long mass_of(uint32_t key, float lse)
{
    const float p = fast_exp2((key_score(key) - lse) * kLog2e);  // <= 1 up to rounding
    return (unsigned long long)(fminf(p, 1.0f) * kMassOne);
}

// In a histogram of probability mass per digit, finds the highest digit d at which the mass
// of the digits >= d reaches `need`; returns d and what is still needed inside d, or digit
// 0xFFFFFFFF when all the mass together does not reach it.
template <int kBins, typename Pool>
__device__ __forceinline__ void find_digit_mass(const unsigned long long *hist, unsigned long long need,
                                                Pool &pool, uint32_t &digit, unsigned long long &rest)
{
    constexpr int per = kBins / kThreads;
    unsigned long long mine[per], sum = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {
        mine[j] = hist[kBins - 1 - (threadIdx.x * per + j)];  // bins taken from the top
        sum += mine[j];
    }
    unsigned long long total;
    unsigned long long above = block_scan64(sum, pool.scan64, total) - sum;
    if (threadIdx.x == 0) {
        pool.scan64[kWaves] = 0xFFFFFFFFull << 32;  // "not reached"
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < per; ++j) {
        if (above < need && need <= above + mine[j]) {
            // digit in the high word, the remaining need (< 2^41) cannot be packed with it: two words
            pool.scan64[kWaves] = (unsigned long long)(uint32_t)(kBins - 1 - (threadIdx.x * per + j)) << 32;
            pool.scan64[kWaves - 1] = need - above;
        }
        above += mine[j];
    }
    __syncthreads();
    digit = (uint32_t)(pool.scan64[kWaves] >> 32);
    rest = pool.scan64[kWaves - 1];
    __syncthreads();
}

// Entries the rule keeps, before the clamp to [1, n]: Threshold counts the entries whose
// probability exceeds the parameter; Top-p finds, digit by digit, the key at which the
// probability mass of the descending order reaches the parameter (all entries with that key
// have the same mass, so a division says how many of them are needed).  `lse` is the
// log-sum-exp of the pooled logits of the whole sequence.  The entries hold at least the n best
// positions, and a rule that would go beyond them is capped at n anyway.
template <typename Entries, typename Pool>
__device__ __forceinline__ int rule_keeps(const Common &c, const Entries &E, int n, float lse, SharedSelect &sh,
                                          Pool &pool)
{
    uint32_t want;
    if (c.prob_rule == 1) {
        const uint32_t cut = ordered_key(lse + __logf(c.prob_param));
        uint32_t mine = 0;
        E.for_each([&](uint32_t key, uint32_t pos) { mine += (uint32_t)((pos != kNoEntry) & (key > cut)); });
        (void)block_scan(mine, pool.scan, want);
    } else {
        if (c.prob_param >= 1.0f) return n;  // all of the mass: everything, i.e. the cap
        unsigned long long *mh = reinterpret_cast<unsigned long long *>(sh.hist);  // 4096 x 8 bytes: hist + samp
        unsigned long long need = (unsigned long long)((double)c.prob_param * (double)kMassOne);
        need = need < 1 ? 1 : need;
        uint32_t prefix = 0, prefix_mask = 0;
        bool reached = true;
#pragma unroll
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
            const int n_bins = pass == 0 ? 4096 : 1024;
            const uint32_t digit_mask = (uint32_t)n_bins - 1u;
            for (int i = threadIdx.x; i < n_bins; i += kThreads) mh[i] = 0;
            __syncthreads();
            E.for_each([&](uint32_t key, uint32_t pos) {
                const bool in = (pos != kNoEntry) & ((key & prefix_mask) == prefix);
                if (in) atomicAdd(&mh[(key >> shift) & digit_mask], mass_of(key, lse));
            });
            __syncthreads();
            uint32_t digit;
            unsigned long long left;
            if (pass == 0)
                find_digit_mass<4096, Pool>(mh, need, pool, digit, left);
            else
                find_digit_mass<1024, Pool>(mh, need, pool, digit, left);
            if (digit == 0xFFFFFFFFu) {  // (uniform) not even all entries reach the mass: the cap decides
                reached = false;
                break;
            }
            prefix |= digit << shift;
            prefix_mask |= digit_mask << shift;
            need = left;
        }
        if (!reached) return n;
        const unsigned long long each = mass_of(prefix, lse);  // > 0: its digit held mass
        const uint32_t of_last = (uint32_t)((need + each - 1) / each);
        uint32_t mine = 0;
        E.for_each([&](uint32_t key, uint32_t pos) { mine += (uint32_t)((pos != kNoEntry) & (key > prefix)); });
        uint32_t above;
        (void)block_scan(mine, pool.scan, above);
        want = above + of_last;
    }
    return want < 1u ? 1 : (want > (uint32_t)n ? n : (int)want);
}

// Log-sum-exp of the pooled logits of score row `row`: the pieces' states, merged.
template <typename Pool>
__device__ __forceinline__ float pooled_lse(const Common &c, const LayerDesc &p, int64_t row, int count,
                                            Pool &pool)
{
    const float *ml = p.part_pool + row * (2 * (int64_t)c.part_stride);
    float m_loc = kMinusBig;
    for (int s = threadIdx.x; s < count; s += kThreads) m_loc = fmaxf(m_loc, gload(ml + 2 * s));
    const float M = block_max(m_loc, pool.fred);
    float l_loc = 0.0f;
    for (int s = threadIdx.x; s < count; s += kThreads)
        l_loc = fmaf(fast_exp2((gload(ml + 2 * s) - M) * kLog2e), gload(ml + 2 * s + 1), l_loc);
    const float l = block_sum(l_loc, pool.fred);
    return M + __logf(l);
}

// The set of a KV head (b, g) whose group holds no retrieval head is handed on unchanged
// (Sec. 3.1): a verbatim copy.
__device__ __forceinline__ void copy_set_unit(const Common &c, const LayerDesc &p, int b, int g)
{
    const int64_t bg = (int64_t)b * c.n_kv_heads + g;
    int32_t *dst = p.idx_out + bg * c.k;
    const int32_t *src = p.idx_src[g] + bg * c.k;
    for (int i = threadIdx.x; i < c.k; i += kThreads) gstore_through(dst + i, gload(src + i));
}

// S unit of KV head (b, g), whose group holds a retrieval head: the set the next layer's
// sparse heads of the group inherit.  PROB: the build that knows the probability rules (their
// 64-bit mass arithmetic over register-resident entries would cost the plain build registers).
template <bool PROB, typename Pool>
__device__ __forceinline__ void select_unit(const Common &c, const LayerDesc &p, int b, int g,
                                            SharedSelect &sh, Pool &pool)
{
    const int64_t bg = (int64_t)b * c.n_kv_heads + g;
    int32_t *dst = p.idx_out + bg * c.k;
    const int rgi = p.rindex[g];
    const int len = pool.len[b];  // staged by the kernel, clamped
    const int L = units_of(c, len);  // what is ranked: positions, or blocks of positions
    const int n = budget_of(c, L);
    const bool by_prob = PROB && c.prob_rule != 0;
    if (n == L && !by_prob) {  // everything is selected
        for (int i = threadIdx.x; i < c.k; i += kThreads) gstore_through(dst + i, (int32_t)(i < L ? i : -1));
        if (threadIdx.x == 0 && c.block_shift == 0 && rgi != 0xFF)
            gstore(p.list_count + ((int64_t)b * p.n_rgroups + rgi), (int32_t)0);  // (nothing was collected; see below)
        return;
    }
    const int64_t row = (int64_t)b * p.n_rgroups + rgi;
    const unsigned long long *list = p.list + row * (int64_t)c.list_row;
    // block-granular: the streaming left every block's score at its place in the list
    const int total = c.block_shift ? L : gload(p.list_count + row);
    // The select is the counter's only reader: it leaves it at zero for the next launch that
    // collects into it (a launch whose streaming runs beside its threshold units has nobody who
    // could clear it first).  Every thread has read it before any thread gets past the barriers
    // that follow, so one thread may clear it then.
    const bool clear_count = c.block_shift == 0;
    float lse = 0.0f;
    if (by_prob) {
        // the pieces of this KV head's segment, counted by its first retrieval head
        const int h = g * c.group + __builtin_ctz((uint32_t)p.rmask[g]);
        int count = gload(p.part_count + (int64_t)b * c.n_q_heads + h);
        count = count < 0 ? 0 : (count > c.part_stride ? c.part_stride : count);
        lse = pooled_lse(c, p, row, count, pool);
    }
    int keep = n;  // what is selected in the end: n, or fewer under a probability rule
    if (total >= n && total <= kThreads * kSelRegs && total <= c.list_row) {
        RegEntries E;
        E.load(list, total);
        if (PROB && by_prob) keep = rule_keeps(c, E, n, lse, sh, pool);
        select_from(E, keep, L, dst, sh, pool);
    } else if (total >= n && total <= c.list_row) {
        const ListEntries E{list, total};
        if (PROB && by_prob) keep = rule_keeps(c, E, n, lse, sh, pool);
        select_from(E, keep, L, dst, sh, pool);
    } else {
        // too few candidates reached the threshold, or too many for the list: rank the row
        // (token-granular only: a block list is always complete)
        if (threadIdx.x == 0) atomicAdd(c.stats + (total < n ? 0 : 1), 1u);
        float *sel = p.sel + row * c.sel_stride;
        switch (__builtin_popcount(p.rmask[g] & ((1u << c.group) - 1u))) {
        case 1: score_row_unit<1>(c, p, b, g, len, sel); break;
        case 2: score_row_unit<2>(c, p, b, g, len, sel); break;
        case 3: score_row_unit<3>(c, p, b, g, len, sel); break;
        default: score_row_unit<4>(c, p, b, g, len, sel); break;
        }
        __threadfence();
        __syncthreads();  // the scores are read back by other threads of the workgroup
        const RowEntries E{sel, len};
        if (PROB && by_prob) keep = rule_keeps(c, E, n, lse, sh, pool);
        select_from(E, keep, L, dst, sh, pool);
    }
    for (int i = keep + threadIdx.x; i < c.k; i += kThreads) gstore_through(dst + i, (int32_t)-1);
    if (clear_count && threadIdx.x == 0) gstore(p.list_count + row, (int32_t)0);
}


}  // namespace
}  // namespace lychee
