// The work-unit kernels of liblychee for gfx950 (CDNA4).
//
// One launch runs a pooled list of work for a fixed grid of workgroups (about two per CU):
//   A  cache append          Alg. 1's C.append(k, v): the decoded token's rows enter the caches
//   T  selection threshold   a score that somewhat more than k rows reach, read off a sample
//                            of the row's pooled scores (Eq. 2's ranking needs only those)
//   R  retrieval streaming   Eq. 1, o = A V; rows whose pooled score reaches the threshold
//                            are collected as candidates of Eq. 2's top-k (block-granular
//                            sets, App. C: every block's best score is written in place)
//   S  select                exact radix select over the candidates (ties to the lower
//                            position), ascending write of the set; verbatim copy for groups
//                            that keep theirs; the Ratio, Threshold and Top-p rules of
//                            Sec. 4.4.1 decide here how many are kept
//   G  sparse gather         Eq. 3 on the inherited set
//   C  combine               log-sum-exp merge of a head's partials into its bf16 output
// R and G rows run in lychee_pool_kernel, the other kinds in lychee_small_kernel.  A launch
// names, for each kind, the range of layers it covers in a table of layer descriptors in
// device memory.  The units of one launch are mutually independent;
// everything that depends on another unit's result runs in a later launch, so there are no
// device-side waits or fences; the only atomics on global memory are counters whose final
// value, not the order of the additions, is what later launches use.
//
// Why candidates and not scores: writing every pooled score (4 bytes per 516 streamed) cost
// the streaming launch 12 % of its time, most of it HBM write traffic interleaved with the
// read stream, and a later pass had to read the scores back.  With a threshold known before
// the rows stream by, only about 6 % of the scores leave the CU, in bursts.
//
// Pooling (App. C describes pooling full and sparse block work into uniform splits).  The R
// and G rows of a launch, over all its layers, sequences and KV heads, form one row space
// cut into blocks of 64 rows (fewer for gathered rows, which cost more); every workgroup
// takes an equal, contiguous run of blocks.  A run may cross from one (layer, sequence, KV
// head) segment into the next; each (workgroup, segment) piece leaves one partial per head in
// a slot that depends only on the shapes, never on timing.  Small units (T, S, C) are
// dealt round-robin.
//
// Data path of R and G.  Cache rows go from HBM to registers with 16-byte nontemporal loads:
// a 64-lane wavefront covers 4 rows per load instruction (16 lanes x 16 bytes = one 256-byte
// row) and 16 rows (K and V) per tile; a small ring of tiles keeps about one tile of loads in
// flight per wavefront, which is what saturates a CU's share of HBM bandwidth on this chip
// (deeper queues were measured to be slower).  A row is used by all heads of the GQA group
// from registers, so no K/V staging in LDS is needed.  Scores use the packed-bf16 dot
// instruction with fp32 accumulation; the 16 lanes of a row are summed by a fixed DPP
// butterfly, so a key row's score has the same bits wherever it is processed and exact ties
// stay exact ties.
#include "lychee_internal.h"

namespace lychee {
namespace {

// ------------------------------------------------------------------------------ LDS layout
struct SharedAttn {
    int32_t idx_s[kIdxChunk];
    float red_o[kWaves * kMaxGroup * kHeadDim];
    float red_ml[kWaves * kMaxGroup * 2];
    float pool_ml[kWaves * 2];
    unsigned long long cand[kWaves][kCandBuf];  // per wavefront: candidates not yet flushed
    int32_t cand_left[kWaves];                  // what each wavefront still holds when a piece ends
    int32_t cand_base;                          // where the workgroup's last candidates go
};
struct SharedSelect {
    uint32_t hist[4096];                   // radix histograms; position bitmap of the ordered write
    uint32_t samp[kSampleTilesMax * 16];   // ordered keys of the threshold sample
    uint32_t found[2];
};
struct SharedCombine {
    float w[kMaxWg];
    float red[(kThreads / 32) * kHeadDim];
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

#ifdef LYCHEE_TRACE
__device__ unsigned long long g_trace[kMaxWg * 8];
__device__ int g_trace_on = 1;
#define TRACE(slot) do { if (threadIdx.x == 0 && g_trace_on) g_trace[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
// Lap timer of a workgroup: adds the time since the previous lap to accumulator `which` (0..3);
// which < 0 only restarts it, which == -2 also clears the accumulators.
__device__ unsigned long long g_lap[kMaxWg * 4];
__device__ __forceinline__ void trace_lap(int which)
{
    __shared__ unsigned long long mark;
    if (threadIdx.x == 0) {
        const unsigned long long now = wall_clock64();
        if (which == -2)
            for (int i = 0; i < 4; ++i) g_lap[blockIdx.x * 4 + i] = 0;
        if (which >= 0) g_lap[blockIdx.x * 4 + which] += now - mark;
        mark = now;
    }
}
#define TRACE_LAP(which) trace_lap(which)
#else
#define TRACE(slot) do { } while (0)
#define TRACE_LAP(which) do { } while (0)
#endif

// ------------------------------------------------------------------------------ R and G
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

// q . k of one cache row: each of the row's 16 lanes holds 8 elements; all 16 end with the sum.
__device__ __forceinline__ float row_score(const uint4 &kr, const uint4 &qh)
{
    float a = dot2_bf16(kr.x, qh.x, 0.0f);
    a = dot2_bf16(kr.y, qh.y, a);
    a = dot2_bf16(kr.z, qh.z, a);
    a = dot2_bf16(kr.w, qh.w, a);
    return row16_sum(a);
}

// The pooled selection score of a row (App. F: the group's retrieval heads are averaged) from
// the sum of its heads' dot products; sel_mul = 1 / (sqrt(d) * heads).  Adding +0 turns a -0
// into +0, so equal scores have equal bits.
__device__ __forceinline__ float sel_value(float pooled_sum, float sel_mul) { return pooled_sum * sel_mul + 0.0f; }

template <int NH>
__device__ __forceinline__ void consume_tile(const Tile &t, const uint4 (&qf)[NH], Acc<NH> &acc,
                                             float c_log2e, float (&sel_sum)[4])
{
    float s[NH][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool ok = (t.valid >> j) & 1;
#pragma unroll
        for (int h = 0; h < NH; ++h) s[h][j] = row_score(t.k[j], qf[h]);
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

// Where the candidates of one segment's score row go.
struct Emit {
    unsigned long long *list;  // nullptr: the segment collects no candidates
    int32_t *count;
    uint32_t thr;              // a row is a candidate when its ordered key reaches this
    int32_t cap;
    int32_t direct;            // block-granular: entry b of the list is block b's best score,
                               // written in place; no threshold, no counter
    float *pool_ml;            // Threshold / Top-p rules: this score row's per-piece (maximum,
                               // sum of exp) of the pooled logits; nullptr otherwise
};

// Appends a wavefront's n buffered candidates to the row's list.  The counter keeps counting
// past the capacity, which is how the select unit learns that the list is incomplete.
// (Only a full buffer comes here.  What a wavefront holds when its piece ends is written by
// run_piece with one reservation per workgroup: a short launch has hundreds of workgroups
// per score row that all end at the same time, and their reservations on the row's one
// counter are served one after the other.)
__device__ __forceinline__ void flush_candidates(const unsigned long long *buf, int n, const Emit &em)
{
    const int lane = threadIdx.x & 63;
    int base = 0;
    if (lane == 0)
        base = __hip_atomic_fetch_add((LYCHEE_GLOBAL int32_t *)em.count, (int32_t)n, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
    base = __builtin_amdgcn_readfirstlane(base);
    for (int i = lane; i < n; i += 64)
        if (base + i < em.cap) gstore(em.list + base + i, buf[i]);
}

// Streams rows [r0, r1) of one segment through the accumulators.  GATHER = false: cache rows
// r0..r1-1; true: the cache rows named by set entries r0..r1-1, staged in idx_s[0 .. r1-r0).
//
// Rows are dealt in spans of 32 * kWaves: wavefront w owns rows 32w .. 32w+31 of every span,
// as two tiles of 16 rows (4 rows per load instruction, K and V).  The two tile buffers
// alternate: one tile's loads are in flight while the other is consumed.  After both tiles of
// a span the wavefront compares its 32 pooled scores with the threshold and puts the rows
// that reach it into its LDS buffer, which goes to the list in bursts.
template <int NH, bool GATHER>
__device__ __forceinline__ void stream_rows(const Common &c, const uint16_t *kbase,
                                            const uint16_t *vbase, const uint4 (&qf)[NH],
                                            Acc<NH> &acc, int L, int r0, int r1,
                                            const int32_t *idx_s, const Emit &em, float sel_mul,
                                            unsigned long long *cand_buf, int &cand_left,
                                            float &pool_m, float &pool_l)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rs = lane >> 4;  // row slot: which of the 4 rows of a load this lane is in
    const int ch = lane & 15;  // 16-byte chunk of the 256-byte row
    constexpr int kSpan = 32 * kWaves;
    const float c_log2e = c.scale_log2e;
    const int bshift = c.block_shift;
    // A span is 32 rows per wavefront.  Normally the wavefronts' rows interleave (wavefront w:
    // rows 32w .. 32w+31 of every 128).  When block scores are wanted a wavefront owns a whole
    // block instead: rows 64w .. 64w+63 of every 256, as two consecutive spans.
    const bool by_block = !GATHER && em.direct != 0;
    const int n_spans = by_block ? 2 * ((r1 - r0 + 2 * kSpan - 1) / (2 * kSpan)) : (r1 - r0 + kSpan - 1) / kSpan;
    auto span_base = [&](int span) {
        return by_block ? r0 + (span >> 1) * (2 * kSpan) + 64 * wave + 32 * (span & 1) : r0 + span * kSpan + 32 * wave;
    };
    float block_best = 0.0f;

    // tile `half` (0 or 1) of span `span`: rows base .. base+15 of this wavefront
    auto issue = [&](Tile &t, int span, int half) {
        const int base = span_base(span) + 16 * half;
        t.valid = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = base + 4 * j + rs;
            int row;
            bool ok;
            if (GATHER) {
                // set entry (r - r0) >> bshift names 2^bshift consecutive cache rows
                const int e = (r < r1) ? idx_s[(r - r0) >> bshift] : -1;
                const int tpos = (e << bshift) + (r & ((1 << bshift) - 1));
                ok = (e >= 0) && (tpos < L);
                row = ok ? tpos : 0;
            } else {
                ok = r < r1;
                row = ok ? r : (r1 > 0 ? r1 - 1 : 0);
            }
            t.valid |= (ok ? 1 : 0) << j;
            const int64_t off = (int64_t)row * c.stride_t + ch * 8;
            t.k[j] = load_stream16(kbase + off);
            t.v[j] = load_stream16(vbase + off);
        }
    };
    auto consume = [&](const Tile &t, float (&sel_sum)[4]) {
        consume_tile<NH>(t, qf, acc, c_log2e, sel_sum);
    };

    // Loads are issued unconditionally (a tile past the end re-reads the segment's last row
    // and is marked invalid): a conditional refill would make the tile registers loop-carried
    // through a copy that has to wait for its load.
    Tile t0, t1;
    int cand_n = 0;  // candidates in cand_buf; the same in every lane
    if (n_spans == 0) return;
    issue(t0, 0, 0);
    issue(t1, 0, 1);
    TRACE(5);
    TRACE_LAP(0);  // piece set-up, until its first loads are issued
    for (int span = 0; span < n_spans; ++span) {
        float sel0[4], sel1[4];
        consume(t0, sel0);
        if (span == 0) {
            TRACE(6);
            TRACE_LAP(1);  // until the first tile has arrived and is consumed
        }
        __builtin_amdgcn_sched_barrier(0);
        issue(t0, span + 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        consume(t1, sel1);
        __builtin_amdgcn_sched_barrier(0);
        issue(t1, span + 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (!GATHER && em.list != nullptr && em.direct != 0) {
            // the best pooled score of this span's valid rows: every lane of a row slot holds
            // its 8 rows' scores, the four row slots are merged by two exchanges
            const int rb = span_base(span);
            float m = -INFINITY;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = rb + 4 * j + rs;
                m = (r < r1) ? fmaxf(m, sel_value(sel0[j], sel_mul)) : m;
                m = (r + 16 < r1) ? fmaxf(m, sel_value(sel1[j], sel_mul)) : m;
            }
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            block_best = (span & 1) ? fmaxf(block_best, m) : m;
            const int first = rb - 32;  // of the block, when this is its second span
            if ((span & 1) && first < r1 && lane == 0) {
                const uint32_t blk = (uint32_t)(first >> 6);
                gstore(em.list + blk, (unsigned long long)ordered_key(block_best) | ((unsigned long long)blk << 32));
            }
        } else if (!GATHER && em.list != nullptr) {
            // lane ch (< 8) of each row slot holds the score of row 16*(ch/4) + 4*(ch%4) + rs
            const int j = ch & 3;
            float lo = sel0[0], hi = sel1[0];
            lo = (j == 1) ? sel0[1] : lo;
            hi = (j == 1) ? sel1[1] : hi;
            lo = (j == 2) ? sel0[2] : lo;
            hi = (j == 2) ? sel1[2] : hi;
            lo = (j == 3) ? sel0[3] : lo;
            hi = (j == 3) ? sel1[3] : hi;
            const float mine = (ch & 4) ? hi : lo;
            const int r = r0 + span * kSpan + 32 * wave + 16 * ((ch >> 2) & 1) + 4 * j + rs;
            const float score = sel_value(mine, sel_mul);
            const uint32_t key = ordered_key(score);
            if (em.pool_ml != nullptr && ch < 8 && r < r1) {
                // online log-sum-exp of the pooled logits, one row per lane and span
                const float m_new = fmaxf(pool_m, score);
                pool_l = pool_l * fast_exp2((pool_m - m_new) * kLog2e) + fast_exp2((score - m_new) * kLog2e);
                pool_m = m_new;
            }
            const bool hit = ch < 8 && r < r1 && key >= em.thr;
            const unsigned long long hits = __builtin_amdgcn_ballot_w64(hit);
            if (hits != 0) {  // wave-uniform
                const int before = (int)__builtin_amdgcn_mbcnt_hi(
                    (uint32_t)(hits >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hits, 0u));
                if (hit) cand_buf[cand_n + before] = (unsigned long long)key | ((unsigned long long)(uint32_t)r << 32);
                cand_n += __builtin_popcountll(hits);
                if (cand_n > kCandBuf - 32) {
                    flush_candidates(cand_buf, cand_n, em);
                    cand_n = 0;
                }
            }
        }
    }
    cand_left = cand_n;  // the caller writes these out, one reservation for the whole workgroup
}

// One (workgroup, segment) piece: rows/entries [r0, r1) of segment (b, g) for the heads in
// hmask.  Leaves one un-normalised partial per head in `slot`; the piece that ends the
// segment also records how many slots the segment has.
template <int NH, bool GATHER, typename Hook>
__device__ __forceinline__ void run_piece(const Common &c, const uint16_t *q, const uint16_t *k_cache,
                                          const uint16_t *v_cache, const int32_t *idx_src,
                                          const Emit &em, float *part_o, float *part_ml,
                                          int32_t *part_count, int b, int g, uint32_t hmask, int L,
                                          int r0, int r1, int slot, bool ends_segment,
                                          SharedAttn &sh, Hook &at_rows_done)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rs = lane >> 4;
    const int ch = lane & 15;

    int heads[NH];
    {
        uint32_t mk = hmask;
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const int bit = __builtin_ctz(mk);
            mk &= mk - 1;
            heads[h] = g * c.group + bit;
        }
    }
    uint4 qf[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h)
        qf[h] = gload_u4(q + ((int64_t)b * c.n_q_heads + heads[h]) * kHeadDim + ch * 8);

    Acc<NH> acc;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        acc.m[h] = kMinusBig;
        acc.l[h] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc.o[h][e] = 0.0f;
    }
    const uint16_t *kbase = k_cache + (int64_t)b * c.stride_b + (int64_t)g * c.stride_h;
    const uint16_t *vbase = v_cache + (int64_t)b * c.stride_b + (int64_t)g * c.stride_h;
    const float sel_mul = c.scale / (float)NH;
    float pool_m = kMinusBig, pool_l = 0.0f;  // per lane: log-sum-exp state of the pooled logits
    int cand_left = 0;                        // candidates still in this wavefront's LDS buffer

    if (GATHER) {
        // rows r0 .. r1-1 of the gathered sequence are row (r mod 2^shift) of set entry r >> shift
        const int shift = c.block_shift;
        const int chunk_rows = kIdxChunk << shift;
        for (int e0 = r0; e0 < r1; e0 += chunk_rows) {
            const int e1 = e0 + chunk_rows < r1 ? e0 + chunk_rows : r1;
            const int n_entries = (e1 - e0 + (1 << shift) - 1) >> shift;
            __syncthreads();  // the previous chunk's readers are done
            for (int i = threadIdx.x; i < n_entries; i += kThreads) sh.idx_s[i] = gload(idx_src + (e0 >> shift) + i);
            __syncthreads();
            stream_rows<NH, true>(c, kbase, vbase, qf, acc, L, e0, e1, sh.idx_s, em, 0.0f, nullptr, cand_left, pool_m, pool_l);
        }
    } else {
        stream_rows<NH, false>(c, kbase, vbase, qf, acc, L, r0, r1, nullptr, em, sel_mul, sh.cand[wave], cand_left, pool_m, pool_l);
    }
    const bool collects = !GATHER && em.list != nullptr && em.direct == 0;  // the same in every wavefront

    TRACE(7);
    TRACE_LAP(2);  // streaming
    at_rows_done();  // what the caller wants in flight while the partial is merged and written
    // Merge the 4 row slots of the wavefront (lanes l, l^16, l^32, l^48).
    const float c_log2e = c.scale_log2e;
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
    const bool pooled_lse = !GATHER && em.pool_ml != nullptr;
    if (pooled_lse) {  // wave-uniform: merge the lanes' pooled log-sum-exp states
        float mw = pool_m;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) mw = fmaxf(mw, __shfl_xor(mw, d));
        float lw = pool_l * fast_exp2((pool_m - mw) * kLog2e);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) lw += __shfl_xor(lw, d);
        pool_m = mw;
        pool_l = lw;
    }
    // Merge the 4 wavefronts through LDS and write the piece's partial.
    __syncthreads();  // red_o / idx_s readers of the previous piece are done
    if (pooled_lse && lane == 0) {
        sh.pool_ml[2 * wave] = pool_m;
        sh.pool_ml[2 * wave + 1] = pool_l;
    }
    if (collects && lane == 0) sh.cand_left[wave] = cand_left;
    if (rs == 0) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float *dst = sh.red_o + (wave * kMaxGroup + h) * kHeadDim + ch * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e] = acc.o[h][e];
            if (ch == 0) {
                sh.red_ml[(wave * kMaxGroup + h) * 2 + 0] = acc.m[h];
                sh.red_ml[(wave * kMaxGroup + h) * 2 + 1] = acc.l[h];
            }
        }
    }
    __syncthreads();
    if (collects && threadIdx.x == kThreads - 1) {
        // room for the workgroup's last candidates, asked for by a thread that writes no
        // partial: the answer is on its way while the others merge
        int n = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) n += sh.cand_left[w];
        int base = 0;
        if (n > 0)
            base = __hip_atomic_fetch_add((LYCHEE_GLOBAL int32_t *)em.count, (int32_t)n, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
        sh.cand_base = base;
    }
    if (threadIdx.x < kHeadDim) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float M = kMinusBig;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sh.red_ml[(w * kMaxGroup + h) * 2]);
            float o = 0.0f, l = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float a = fast_exp2((sh.red_ml[(w * kMaxGroup + h) * 2] - M) * c_log2e);
                o = fmaf(a, sh.red_o[(w * kMaxGroup + h) * kHeadDim + threadIdx.x], o);
                l = fmaf(a, sh.red_ml[(w * kMaxGroup + h) * 2 + 1], l);
            }
            const int64_t bh = (int64_t)b * c.n_q_heads + heads[h];
            const int64_t prow = bh * c.part_stride + slot;
            gstore(part_o + prow * kHeadDim + threadIdx.x, o);
            if (threadIdx.x == 0) {
                gstore(part_ml + prow * 2 + 0, M);
                gstore(part_ml + prow * 2 + 1, l);
                if (ends_segment) gstore(part_count + bh, (int32_t)(slot + 1));
            }
        }
    }
    if (pooled_lse && threadIdx.x == 0) {  // the piece's pooled log-sum-exp state, same slot
        float M = kMinusBig, l = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sh.pool_ml[2 * w]);
#pragma unroll
        for (int w = 0; w < kWaves; ++w) l = fmaf(fast_exp2((sh.pool_ml[2 * w] - M) * kLog2e), sh.pool_ml[2 * w + 1], l);
        gstore(em.pool_ml + 2 * slot, M);
        gstore(em.pool_ml + 2 * slot + 1, l);
    }
    if (collects) {
        __syncthreads();
        int base = sh.cand_base;
        for (int w = 0; w < wave; ++w) base += sh.cand_left[w];
        const unsigned long long *buf = sh.cand[wave];
        for (int i = lane; i < cand_left; i += 64)
            if (base + i < em.cap) gstore(em.list + base + i, buf[i]);
    }
}

template <bool GATHER, typename Hook>
__device__ __forceinline__ void dispatch_piece(int nh, const Common &c, const uint16_t *q,
                                               const uint16_t *k_cache, const uint16_t *v_cache,
                                               const int32_t *idx_src, const Emit &em, float *part_o,
                                               float *part_ml, int32_t *part_count, int b, int g,
                                               uint32_t hmask, int L, int r0, int r1, int slot,
                                               bool ends_segment, SharedAttn &sh, Hook &at_rows_done)
{
    switch (nh) {
    case 1: run_piece<1, GATHER>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    case 2: run_piece<2, GATHER>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    case 3: run_piece<3, GATHER>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    default: run_piece<4, GATHER>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    }
}

// ------------------------------------------------------------------------------ C
// out = (sum_s w_s o_s) / (sum_s w_s l_s),  w_s = 2^((m_s - M) log2(e)/sqrt(d)),  M = max_s m_s,
// over the head's partial slots in ascending order (a fixed summation tree).
__device__ __forceinline__ void combine_unit(const Common &c, const LayerDesc &p, int bh, SharedCombine &sh,
                                             SharedPool &pool)
{
    int count = gload(p.part_count + bh);
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
template <int NH>
__device__ __forceinline__ void threshold_unit(const Common &c, const LayerDesc &p, int b, int rgi,
                                               SharedSelect &sh, SharedPool &pool)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rs = lane >> 4;
    const int ch = lane & 15;
    const int L = pool.len[b];  // staged by the kernel, clamped
    const int n = budget_of(c, L);
    const int64_t row = (int64_t)b * p.n_rgroups + rgi;
    if (threadIdx.x == 0) gstore(p.list_count + row, (int32_t)0);
    if (p.q_keep != nullptr && (int)threadIdx.x < c.group * (kHeadDim / 8)) {
        // the group's query rows (consecutive heads, 16 chunks of 16 bytes each)
        const int64_t at = ((int64_t)b * c.n_q_heads + p.rgroup[rgi] * c.group) * kHeadDim + threadIdx.x * 8;
        *(LYCHEE_GLOBAL u32x4_t *)(p.q_keep + at) = *(const LYCHEE_GLOBAL u32x4_t *)(p.q + at);
    }
    if (n == L || L <= kDirectLen || 2 * (int64_t)n >= L) {
        // everything is selected anyway (no candidates wanted), or every row is a candidate
        // (a probability rule may keep fewer than everything: it still needs the candidates)
        if (threadIdx.x == 0) gstore(p.thr + row, n == L && c.prob_rule == 0 ? 0xFFFFFFFFu : 0u);
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
    for (int t0 = wave * kBatch; t0 < n_tiles; t0 += kWaves * kBatch) {
        uint4 kr[kBatch][4];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int t = t0 + u < n_tiles ? t0 + u : n_tiles - 1;
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
            if (t0 + u < n_tiles && ch < 4) {
                sh.samp[(t0 + u) * 16 + 4 * ch + rs] = key;
                atomicAdd(&sh.hist[key >> 20], 1u);
            }
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
    if (threadIdx.x == 0) gstore(p.thr + row, t_key);
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
template <typename Entries, typename Val, typename Among>
__device__ __forceinline__ uint32_t radix_select(const Entries &E, uint32_t need, Val val, Among among,
                                                 uint32_t &rest, SharedSelect &sh, SharedPool &pool)
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
template <typename Entries>
__device__ __forceinline__ void select_from(const Entries &E, int n, int L, int32_t *dst, SharedSelect &sh,
                                            SharedPool &pool)
{
    uint32_t r_eq;
    const uint32_t T = radix_select(
        E, (uint32_t)n, [](uint32_t key, uint32_t) { return key; }, [](uint32_t, uint32_t) { return true; }, r_eq,
        sh, pool);
    TRACE(7);
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
        TRACE(2);
        uint32_t words[kPer], cnt = 0;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            words[j] = sh.hist[threadIdx.x * kPer + j];
            cnt += (uint32_t)__builtin_popcount(words[j]);
        }
        uint32_t tot;
        uint32_t at = base + block_scan(cnt, pool.scan, tot) - cnt;
        TRACE(3);
        // (handing neighbouring words to neighbouring lanes, for store addresses that share
        // cache lines, was measured to be slower: the loop below is bound by its divergence)
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            uint32_t wd = words[j];
            while (wd != 0) {
                const uint32_t bit = (uint32_t)__builtin_ctz(wd);
                wd &= wd - 1u;
                if (at < (uint32_t)n) gstore(dst + at, (int32_t)(w0 + (uint32_t)(threadIdx.x * kPer + j) * 32u + bit));
                ++at;
            }
        }
        base += tot;
    }
    TRACE(4);
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
template <int kBins>
__device__ __forceinline__ void find_digit_mass(const unsigned long long *hist, unsigned long long need,
                                                SharedPool &pool, uint32_t &digit, unsigned long long &rest)
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
template <typename Entries>
__device__ __forceinline__ int rule_keeps(const Common &c, const Entries &E, int n, float lse, SharedSelect &sh,
                                          SharedPool &pool)
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
                find_digit_mass<4096>(mh, need, pool, digit, left);
            else
                find_digit_mass<1024>(mh, need, pool, digit, left);
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
__device__ __forceinline__ float pooled_lse(const Common &c, const LayerDesc &p, int64_t row, int count,
                                            SharedPool &pool)
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
    for (int i = threadIdx.x; i < c.k; i += kThreads) gstore(dst + i, gload(src + i));
}

// S unit of KV head (b, g), whose group holds a retrieval head: the set the next layer's
// sparse heads of the group inherit.  PROB: the build that knows the probability rules (their
// 64-bit mass arithmetic over register-resident entries would cost the plain build registers).
template <bool PROB>
__device__ __forceinline__ void select_unit(const Common &c, const LayerDesc &p, int b, int g,
                                            SharedSelect &sh, SharedPool &pool)
{
    const int64_t bg = (int64_t)b * c.n_kv_heads + g;
    int32_t *dst = p.idx_out + bg * c.k;
    const int rgi = p.rindex[g];
    const int len = pool.len[b];  // staged by the kernel, clamped
    const int L = units_of(c, len);  // what is ranked: positions, or blocks of positions
    const int n = budget_of(c, L);
    const bool by_prob = PROB && c.prob_rule != 0;
    if (n == L && !by_prob) {  // everything is selected
        for (int i = threadIdx.x; i < c.k; i += kThreads) gstore(dst + i, (int32_t)(i < L ? i : -1));
        return;
    }
    const int64_t row = (int64_t)b * p.n_rgroups + rgi;
    const unsigned long long *list = p.list + row * (int64_t)c.list_row;
    // block-granular: the streaming left every block's score at its place in the list
    const int total = c.block_shift ? L : gload(p.list_count + row);
    TRACE(5);
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
        TRACE(6);
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
    for (int i = keep + threadIdx.x; i < c.k; i += kThreads) gstore(dst + i, (int32_t)-1);
}

// ------------------------------------------------------------------------------ the kernels
// Fields of a layer descriptor staged in LDS as 32-bit words.  The values are the same in
// every lane; reading them back through readfirstlane tells the compiler so (scalar registers,
// scalar address arithmetic in the streaming loop).
constexpr int kDescWords = (int)(sizeof(LayerDesc) / 4);
static_assert(sizeof(LayerDesc) % 4 == 0 && kDescWords <= kThreads, "one word per thread");

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

// Launches that carry T, S and C units: unit j runs on workgroup j mod W.  SELECTS = 0 is
// the lighter build for launches without S units on retrieval groups (their candidates held
// in registers set this kernel's register budget, and spill code with it), 1 the build with
// them, 2 the one whose S units also know the probability rules.
template <int SELECTS>
__global__ __launch_bounds__(kThreads, 2) void lychee_small_kernel(const LaunchPlan P)
{
    __shared__ SharedUnit su;
    __shared__ SharedPool pool;
    __shared__ __align__(16) uint32_t small_desc[kDescWords];  // the current unit's layer descriptor
    const Common &c = P.c;
    const LayerDesc *layers = P.layers;
    const int w = blockIdx.x;
    const int W = c.n_wg;
    TRACE(0);
    if (w == 0 && (int)threadIdx.x < c.n_clear) c.tickets[c.clear_slot[threadIdx.x]] = 0u;
    // the sequence lengths: asked for now, in LDS by the time the unit tables below are built
    if ((int)threadIdx.x < c.batch) pool.len[threadIdx.x] = clamp_len(c.lengths[threadIdx.x], c.max_len);

    // Kinds in a fixed order (S on retrieval groups, C, T, S set copies, A); within a kind
    // layer by layer.
    {
        // (C and A units are the same number per layer: their tables are arithmetic.  The three
        // other kinds take two scans: S units and set copies range over the same layers.)
        const int t = threadIdx.x;
        unsigned long long cnt_s = 0;  // S units | set copies << 32
        uint32_t cnt_t = 0;
        if (t < P.s_count) {
            const int n_r = P.n_rseg[P.s_first + t];
            cnt_s = (unsigned long long)(c.batch * n_r);
            if (P.keeps[P.s_first + t]) cnt_s |= (unsigned long long)(c.batch * (c.n_kv_heads - n_r)) << 32;
        }
        if (t < P.t_count) cnt_t = (uint32_t)(c.batch * P.n_rseg[P.t_first + t]);
        uint32_t tot[5];
        unsigned long long tot_s;
        const unsigned long long incl_s = block_scan64(cnt_s, pool.scan64, tot_s);
        const uint32_t incl_t = block_scan(cnt_t, pool.scan, tot[2]);
        tot[0] = (uint32_t)tot_s;
        tot[3] = (uint32_t)(tot_s >> 32);
        tot[1] = (uint32_t)(P.c_count * c.batch * c.n_q_heads);
        tot[4] = (uint32_t)P.a_count;
        if (t < kMaxLayers) {
            pool.upre[0][t + 1] = (int32_t)(uint32_t)incl_s;
            pool.upre[3][t + 1] = (int32_t)(uint32_t)(incl_s >> 32);
            pool.upre[2][t + 1] = (int32_t)incl_t;
        }
        if (t == 0) pool.upre[0][0] = pool.upre[2][0] = pool.upre[3][0] = 0;
        __syncthreads();
        const int n_small = (int)(tot[0] + tot[1] + tot[2] + tot[3] + tot[4]);
        // A unit reads a dozen fields of its layer's descriptor, several of them pointers it
        // then loads through: read from the table that is a chain of dependent loads (4 to 5 us
        // before a select unit had its candidate count).  The workgroup fetches the whole
        // descriptor into LDS at once instead; which layer a unit belongs to follows from the
        // kernel arguments alone.
        int held = -1;
        auto stage = [&](int layer) -> const LayerDesc & {
            if (layer != held) {  // (the previous unit's readers are behind the barrier that ends a unit)
                if (threadIdx.x < kDescWords)
                    small_desc[threadIdx.x] = gload(reinterpret_cast<const uint32_t *>(layers + layer) + threadIdx.x);
                held = layer;
                __syncthreads();
            }
            return *reinterpret_cast<const LayerDesc *>(small_desc);
        };
        for (int j = w; j < n_small; j += W) {
            int u = j;
            if (u < (int)tot[0]) {
                const int li = find_item(pool.upre[0], P.s_count, u);
                const LayerDesc &L = stage(P.s_first + li);
                u -= pool.upre[0][li];
                const int b = u / L.n_rgroups;
                if (SELECTS == 1) select_unit<false>(c, L, b, L.rgroup[u % L.n_rgroups], su.sel, pool);
                if (SELECTS == 2) select_unit<true>(c, L, b, L.rgroup[u % L.n_rgroups], su.sel, pool);
            } else if ((u -= (int)tot[0]) < (int)tot[1]) {
                const int li = u / (c.batch * c.n_q_heads);
                combine_unit(c, stage(P.c_first + li), u % (c.batch * c.n_q_heads), su.comb, pool);
            } else if ((u -= (int)tot[1]) < (int)tot[2]) {
                const int li = find_item(pool.upre[2], P.t_count, u);
                const LayerDesc &L = stage(P.t_first + li);
                u -= pool.upre[2][li];
                const int rgi = u % L.n_rgroups;
                const int b = u / L.n_rgroups;
                switch (__builtin_popcount(L.rmask[L.rgroup[rgi]] & ((1u << c.group) - 1u))) {
                case 1: threshold_unit<1>(c, L, b, rgi, su.sel, pool); break;
                case 2: threshold_unit<2>(c, L, b, rgi, su.sel, pool); break;
                case 3: threshold_unit<3>(c, L, b, rgi, su.sel, pool); break;
                default: threshold_unit<4>(c, L, b, rgi, su.sel, pool); break;
                }
            } else if ((u -= (int)tot[2]) >= (int)tot[3]) {  // append: one unit per layer
                append_unit(c, stage(P.a_first + u - (int)tot[3]));
            } else {  // copy of the set of a KV head whose group holds no retrieval head
                const int li = find_item(pool.upre[3], P.s_count, u);
                const LayerDesc &L = stage(P.s_first + li);
                u -= pool.upre[3][li];
                const int n_keep = c.n_kv_heads - L.n_rgroups;
                const int b = u / n_keep;
                int want = u % n_keep, g = 0;
                for (int gg = 0; gg < c.n_kv_heads; ++gg)
                    if (L.rindex[gg] == 0xFF && want-- == 0) g = gg;
                copy_set_unit(c, L, b, g);
            }
            __syncthreads();
        }
    }
    TRACE(1);
}

// Launches that carry pooled R and G rows.  Two workgroups per CU must fit (the static shares
// assume that every workgroup runs from the start): at most 256 registers per lane.
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

// COLLECT = false is the dense baseline's streaming: no layer selects anything.
template <bool HAS_R, bool HAS_G, bool COLLECT>
__global__ __launch_bounds__(kThreads, 2) void lychee_pool_kernel(const LaunchPlan P)
{
    __shared__ SharedAttn sa;
    __shared__ SharedPool pool;
    __shared__ uint32_t desc_s[2][kDescWords];
    const Common &c = P.c;
    const LayerDesc *layers = P.layers;
    const int w = blockIdx.x;
    const int W = c.n_wg;
    TRACE(0);
    const int n_items = (P.r_count + P.g_count) * c.batch;
    if (n_items == 0) return;

    // ---- the pooled row space: R items (layer, sequence) then G items, each item holding
    // one segment per retrieval (sparse) KV head of the layer
    // (the sequence lengths go to LDS for the pieces; the item sizes below read them from memory
    // themselves, so that those loads are not behind a barrier)
    if (threadIdx.x < c.batch) pool.len[threadIdx.x] = clamp_len(c.lengths[threadIdx.x], c.max_len);
    // Most of the pooled blocks are dealt statically, an equal contiguous run per workgroup;
    // the last tail_permille/1000 of them are cut into chunks that workgroups claim through
    // a counter as they finish, which evens out CUs that stream at different speeds.  Runs
    // and chunks in ascending block order are the launch's *work items*; the pieces of a
    // segment sit in consecutive items, and a piece's partial slot is its item's distance to
    // the first item of the segment, whoever ran it.
    // A launch too short to hold several chunks per workgroup is dealt statically (the chunks'
    // start-up cost would outweigh what they level out), and then nothing evens out a
    // workgroup whose run crosses from one segment into the next and pays a second piece's
    // start-up and merge: such a launch pads every segment to a whole number of runs (`pad`),
    // so that each workgroup has one piece, when that lengthens the runs by little.
    int share, pad = 0;
    {
        constexpr int kPer = kMaxItems / kThreads;
        uint32_t nseg[kPer], nb[kPer];  // per item: segments, blocks per segment
        unsigned long long sum = 0;      // segments << 32 | blocks
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int it = threadIdx.x * kPer + i;
            nseg[i] = nb[i] = 0;
            if (it < n_items) {
                const int li = it / c.batch;
                const int L = clamp_len(c.lengths[it % c.batch], c.max_len);
                if (li < P.r_count) {
                    nseg[i] = (uint32_t)P.n_rseg[P.r_first + li];
                    nb[i] = (uint32_t)((L + kBlockRows - 1) / kBlockRows);
                } else {
                    nseg[i] = (uint32_t)P.n_gseg[P.g_first + li - P.r_count];
                    nb[i] = (uint32_t)((gather_rows(c, L) + gather_block(c) - 1) / gather_block(c));
                }
                if (nb[i] == 0) nseg[i] = 0;
            }
            sum += ((unsigned long long)nseg[i] << 32) | (unsigned long long)(nseg[i] * nb[i]);
        }
        unsigned long long total64;
        uint32_t at = (uint32_t)(block_scan64(sum, pool.scan64, total64) - sum);
        const int T_real = (int)(uint32_t)total64;
        const int n_segs = (int)(total64 >> 32);
        const int tail = (int64_t)T_real >= 8ll * c.chunk_blocks * W ? c.tail_permille : 0;
        share = (int)((int64_t)T_real * (1000 - tail) / (1000ll * W));
        if (tail == 0 && 8 * n_segs <= W && T_real > 0) {  // (few segments: else the padding would not pay)
            // the smallest run length whose padded segments fit the W workgroups, unless it is
            // much longer than the unpadded run: with many short segments the padding would
            // idle more than the second pieces cost
            const int s0 = (T_real + W - 1) / W;
            const int s_last = s0 + (s0 / 8 > 1 ? s0 / 8 : 1);
            int s = s0;
            for (; s <= s_last; ++s) {
                uint32_t runs = 0, all;
#pragma unroll
                for (int i = 0; i < kPer; ++i) runs += nseg[i] * ((nb[i] + s - 1) / s);
                (void)block_scan(runs, pool.scan, all);
                if ((int)all <= W) break;
            }
            if (s <= s_last) {
                share = s;
                pad = 1;
                uint32_t vsum = 0, vtot;
#pragma unroll
                for (int i = 0; i < kPer; ++i) vsum += nseg[i] * ((nb[i] + s - 1) / s) * s;
                at = block_scan(vsum, pool.scan, vtot) - vsum;
            }
        }
        if (threadIdx.x == 0) pool.ipre[0] = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            at += pad ? nseg[i] * ((nb[i] + share - 1) / share) * share : nseg[i] * nb[i];
            pool.ipre[threadIdx.x * kPer + i + 1] = (int32_t)at;
        }
    }
    __syncthreads();
    const int T = pool.ipre[n_items];  // padded blocks included
    const int T_static = pad ? T : share * W;
    const int n_static = share > 0 ? W : 0;
    const int chunk = c.chunk_blocks;
    const int n_chunks = pad ? 0 : (T - T_static + chunk - 1) / chunk;
    auto item_of = [&](int blk) { return blk < T_static ? blk / share : n_static + (blk - T_static) / chunk; };
    uint32_t *counter = c.tickets + c.ticket_slot;
    uint32_t next_ticket = 0;
    if (threadIdx.x == 0) {
        if (n_chunks > 0) next_ticket = atomicAdd(counter, 1u);  // asked for early, looked at after the static run
        if (w == 0) c.tickets[(c.ticket_slot + kTicketRing / 2) % kTicketRing] = 0u;
    }
    TRACE(2);
    TRACE_LAP(-2);

    // A piece needs its layer's descriptor before it can issue its first load.  Read through
    // the table pointer that is a chain of dependent loads; instead the descriptor is staged
    // in LDS, and the one for the piece after this one is fetched while this piece's partial is
    // merged and written, so that a piece starts with LDS reads only.
    auto layer_of_block = [&](int blk) {
        const int li = find_item(pool.ipre, n_items, blk) / c.batch;
        return HAS_G && (!HAS_R || li >= P.r_count) ? P.g_first + li - P.r_count : P.r_first + li;
    };
    auto fetch_desc = [&](int layer) {
        return threadIdx.x < kDescWords ? gload(reinterpret_cast<const uint32_t *>(layers + layer) + threadIdx.x) : 0u;
    };
    int cur = 0, held[2] = {-1, -1};  // which layer's descriptor each LDS buffer holds

    int item = w;
    int x = w * share;
    int x1 = x + share;
    x1 = x1 < T_static ? x1 : T_static;
    for (;;) {
        while (x < x1) {
            const int it = find_item(pool.ipre, n_items, x);
            const int li = it / c.batch;
            const int b = it % c.batch;
            const bool gather = HAS_G && (!HAS_R || li >= P.r_count);
            const int layer = gather ? P.g_first + li - P.r_count : P.r_first + li;
            __syncthreads();  // a descriptor stashed after the previous piece is visible
            if (held[cur] != layer) {
                if (held[cur ^ 1] == layer) {
                    cur ^= 1;
                } else {
                    const uint32_t v = fetch_desc(layer);
                    if (threadIdx.x < kDescWords) desc_s[cur][threadIdx.x] = v;
                    held[cur] = layer;
                    __syncthreads();
                }
            }
            const uint32_t *dw = desc_s[cur];
            const int len_b = pool.len[b];
            const int seg_rows = gather ? gather_rows(c, len_b) : len_b;
            const int brows = gather ? gather_block(c) : kBlockRows;
            const int nb = (seg_rows + brows - 1) / brows;  // blocks per segment of this item
            const int nbv = pad ? (nb + share - 1) / share * share : nb;  // and with its padding
            const int xo = x - pool.ipre[it];
            const int gi = xo / nbv;
            const int blk = xo % nbv;
            if (blk >= nb) break;  // the run lies in a segment's padding (the last run of a segment ends in it)
            const int seg_start = pool.ipre[it] + gi * nbv;
            int len = x1 - x;
            len = len < nb - blk ? len : nb - blk;
            const int r0 = blk * brows;
            int r1 = (blk + len) * brows;
            r1 = r1 < seg_rows ? r1 : seg_rows;
            const int slot = item - item_of(seg_start);
            const bool ends = blk + len == nb;
            const uint32_t gmask = (1u << c.group) - 1u;

            // where the next piece starts decides which descriptor to fetch meanwhile
            const bool run_ends = x + len >= x1;
            uint32_t ahead = 0;
            int ahead_layer = -1;
            auto at_rows_done = [&]() {
                int xn = x + len;
                if (run_ends) {  // the next piece is the chunk whose ticket is already here
                    __syncthreads();
                    if (threadIdx.x == 0) pool.scan[0] = next_ticket;
                    __syncthreads();
                    const int ticket = (int)pool.scan[0];
                    xn = ticket < n_chunks ? T_static + ticket * chunk : -1;
                }
                if (xn >= 0) {
                    const int ln = layer_of_block(xn);
                    if (ln != layer) {
                        ahead = fetch_desc(ln);
                        ahead_layer = ln;
                    }
                }
            };

            const uint16_t *dq = desc_ptr<const uint16_t>(dw, offsetof(LayerDesc, q));
            const uint16_t *dk = desc_ptr<const uint16_t>(dw, offsetof(LayerDesc, k_cache));
            const uint16_t *dv = desc_ptr<const uint16_t>(dw, offsetof(LayerDesc, v_cache));
            float *d_part_o = desc_ptr<float>(dw, offsetof(LayerDesc, part_o));
            float *d_part_ml = desc_ptr<float>(dw, offsetof(LayerDesc, part_ml));
            int32_t *d_part_count = desc_ptr<int32_t>(dw, offsetof(LayerDesc, part_count));
            if (!gather) {
                const int g = (int)desc_u8(dw, offsetof(LayerDesc, rgroup) + gi);
                const uint32_t hmask = desc_u8(dw, offsetof(LayerDesc, rmask) + g) & gmask;
                Emit em{nullptr, nullptr, 0u, 0, 0, nullptr};
                if (COLLECT && desc_u32(dw, offsetof(LayerDesc, emit_sel))) {
                    const int64_t row = (int64_t)b * (int)desc_u32(dw, offsetof(LayerDesc, n_rgroups)) + gi;
                    em.list = desc_ptr<unsigned long long>(dw, offsetof(LayerDesc, list)) + row * c.list_row;
                    em.count = desc_ptr<int32_t>(dw, offsetof(LayerDesc, list_count)) + row;
                    em.thr = c.block_shift ? 0u : gload(desc_ptr<uint32_t>(dw, offsetof(LayerDesc, thr)) + row);
                    em.cap = c.list_row;
                    em.direct = c.block_shift != 0;
                    if (c.prob_rule != 0)
                        em.pool_ml = desc_ptr<float>(dw, offsetof(LayerDesc, part_pool)) + row * (2 * (int64_t)c.part_stride);
                }
                dispatch_piece<false>(__builtin_popcount(hmask), c, dq, dk, dv, nullptr, em, d_part_o, d_part_ml,
                                      d_part_count, b, g, hmask, len_b, r0, r1, slot, ends, sa, at_rows_done);
            } else {
                const int g = (int)desc_u8(dw, offsetof(LayerDesc, sgroup) + gi);
                const uint32_t hmask = ~desc_u8(dw, offsetof(LayerDesc, rmask) + g) & gmask;
                const int32_t *idx_src = desc_ptr<const int32_t>(dw, offsetof(LayerDesc, idx_src) + 8 * (size_t)g) +
                                         ((int64_t)b * c.n_kv_heads + g) * c.k;
                dispatch_piece<true>(__builtin_popcount(hmask), c, dq, dk, dv, idx_src, Emit{nullptr, nullptr, 0u, 0, 0, nullptr},
                                     d_part_o, d_part_ml, d_part_count, b, g, hmask, len_b, r0, r1, slot, ends, sa,
                                     at_rows_done);
            }
            if (ahead_layer >= 0) {  // wave-uniform; readers of this buffer finished a piece ago
                if (threadIdx.x < kDescWords) desc_s[cur ^ 1][threadIdx.x] = ahead;
                held[cur ^ 1] = ahead_layer;
            }
            x += len;
            TRACE(3);
            TRACE_LAP(3);  // merging and writing the partial
        }
        // next chunk: every workgroup asks until it is told that none is left
        __syncthreads();
        if (threadIdx.x == 0) pool.scan[0] = next_ticket;
        __syncthreads();
        const int ticket = (int)pool.scan[0];
        __syncthreads();
        if (ticket >= n_chunks) break;
        if (threadIdx.x == 0) next_ticket = atomicAdd(counter, 1u);
        item = n_static + ticket;
        x = T_static + ticket * chunk;
        x1 = x + chunk;
        x1 = x1 < T ? x1 : T;
    }
    TRACE(4);
}

// ------------------------------------------------------------------------------ helpers
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4_t *src, size_t n_vec, uint32_t *sink)
{
    // every workgroup streams one contiguous share with 8 nontemporal 16-byte loads in flight
    const size_t share = (n_vec / gridDim.x) / (256 * 8) * (256 * 8);
    const u32x4_t *p = src + (size_t)blockIdx.x * share + threadIdx.x;
    uint32_t acc = 0;
    for (size_t r = 0; r < share; r += 256 * 8) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + r + (size_t)u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;  // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void probe_copy_kernel(uint4 *dst, const uint4 *src, size_t n_vec)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n_vec; i += stride) dst[i] = src[i];
}

__global__ void validate_idx_kernel(const int32_t *idx, const int32_t *lengths, int32_t n_kv_heads,
                                    int32_t k, int32_t max_len, int32_t block_shift,
                                    unsigned long long *n_bad)
{
    // one workgroup per (sequence, KV head); quadratic duplicate check, debug use only
    const int bg = blockIdx.x;
    const int b = bg / n_kv_heads;
    const int L = (clamp_len(lengths[b], max_len) + (1 << block_shift) - 1) >> block_shift;
    const int32_t *row = idx + (int64_t)bg * k;
    unsigned long long bad = 0;
    for (int i = threadIdx.x; i < k; i += blockDim.x) {
        const int32_t t = row[i];
        if (t < 0) {
            if (t != -1) ++bad;
            continue;
        }
        if (t >= L) ++bad;
        if (i > 0 && row[i - 1] < 0) ++bad;  // a valid entry after padding
        for (int j = 0; j < i; ++j)
            if (row[j] == t) {
                ++bad;
                break;
            }
    }
    if (bad) atomicAdd(n_bad, bad);
}

}  // namespace

#ifdef LYCHEE_TRACE
extern "C" int lychee_trace_laps(unsigned long long *host, int n_wg)
{
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(lychee::g_lap), sizeof(unsigned long long) * 4 * n_wg) == hipSuccess ? 0 : -4;
}
extern "C" int lychee_trace_read(unsigned long long *host, int n_wg)
{
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), sizeof(unsigned long long) * 8 * n_wg) == hipSuccess ? 0 : -4;
}
#endif

hipError_t launch_units(const LaunchPlan &plan, hipStream_t stream)
{
    if (plan.c.n_wg < 1 || plan.c.n_wg > kMaxWg) return hipErrorInvalidValue;
    const bool pooled = plan.r_count + plan.g_count > 0;
    const bool small = plan.t_count + plan.s_count + plan.c_count + plan.a_count > 0;
    if (pooled == small) return hipErrorInvalidValue;  // a launch carries one family of units
    const dim3 grid(plan.c.n_wg), block(kThreads);
    if (small && plan.selects && plan.c.prob_rule != 0)
        hipLaunchKernelGGL((lychee_small_kernel<2>), grid, block, 0, stream, plan);
    else if (small && plan.selects)
        hipLaunchKernelGGL((lychee_small_kernel<1>), grid, block, 0, stream, plan);
    else if (small)
        hipLaunchKernelGGL((lychee_small_kernel<0>), grid, block, 0, stream, plan);
    else if (plan.r_count == 0)
        hipLaunchKernelGGL((lychee_pool_kernel<false, true, false>), grid, block, 0, stream, plan);
    else if (plan.g_count == 0 && plan.collect)
        hipLaunchKernelGGL((lychee_pool_kernel<true, false, true>), grid, block, 0, stream, plan);
    else if (plan.g_count == 0)
        hipLaunchKernelGGL((lychee_pool_kernel<true, false, false>), grid, block, 0, stream, plan);
    else if (plan.collect)
        hipLaunchKernelGGL((lychee_pool_kernel<true, true, true>), grid, block, 0, stream, plan);
    else
        hipLaunchKernelGGL((lychee_pool_kernel<true, true, false>), grid, block, 0, stream, plan);
    return hipGetLastError();
}

hipError_t launch_validate_idx(const int32_t *idx, const int32_t *lengths, int32_t batch,
                               int32_t n_kv_heads, int32_t k, int32_t max_len, int32_t block_shift,
                               unsigned long long *n_bad, hipStream_t stream)
{
    hipLaunchKernelGGL(validate_idx_kernel, dim3(batch * n_kv_heads), dim3(256), 0, stream, idx,
                       lengths, n_kv_heads, k, max_len, block_shift, n_bad);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t stream)
{
    const size_t n_vec = bytes / 16;
    hipLaunchKernelGGL(probe_read_kernel, dim3(512), dim3(256), 0, stream,
                       static_cast<const u32x4_t *>(src), n_vec, static_cast<uint32_t *>(sink));
    return hipGetLastError();
}

hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t stream)
{
    const size_t n_vec = bytes / 16;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, stream,
                       static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), n_vec);
    return hipGetLastError();
}

}  // namespace lychee
