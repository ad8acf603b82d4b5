// R and G units (included by lychee_units.hip and lychee_layer.hip): streaming a run of cache rows - or of the
// rows an inherited set names - through the online softmax (Eq. 1, Eq. 3, o = A V), collecting
// the candidates of Eq. 2 on the way, and leaving one partial per head and piece.
#pragma once
#include "lychee_device.h"

namespace lychee {
namespace {

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
    // Launches whose thresholds are computed by units of the same launch (LATE pieces): the
    // piece keeps its rows' keys in LDS and filters them when it ends; by then the threshold
    // unit has normally published {generation, threshold} in *thr_flag.  thr_known: `thr` above
    // is valid without waiting (rows that need no sample).
    const unsigned long long *thr_flag;
    uint32_t gen;
    int32_t thr_known;
    uint32_t *timeouts;        // counts waits that gave up
};

constexpr int kSpinMax = 1 << 20;  // polls of a flag before a wait gives up (seconds; never reached in a working launch)

// Waits until the 64-bit word at `flag` carries this launch's generation in its upper half and
// returns the lower half; `fail` if that does not happen within kSpinMax polls.  The producer
// is a unit that runs on a workgroup with a lower index, started before this one, and waits for
// nothing itself.
__device__ __forceinline__ uint32_t wait_word(const unsigned long long *flag, uint32_t gen, uint32_t fail,
                                              uint32_t *timeouts)
{
    for (int spin = 0; spin < kSpinMax; ++spin) {
        const unsigned long long v = __hip_atomic_load((const LYCHEE_GLOBAL unsigned long long *)flag,
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(v >> 32) == gen) return (uint32_t)v;
        __builtin_amdgcn_s_sleep(2);
    }
    atomicAdd(timeouts, 1u);
    return fail;
}

// The threshold of a LATE piece's score row, the same in every thread (one thread polls).
__device__ __forceinline__ uint32_t late_threshold(const Emit &em, SharedAttn &sh)
{
    if (threadIdx.x == 0 && sh.late_have == 0) {
        // on a time-out nothing is collected; the select then ranks the whole row itself
        sh.late_thr = wait_word(em.thr_flag, em.gen, 0xFFFFFFFFu, em.timeouts);
        sh.late_have = 1;
    }
    __syncthreads();
    return sh.late_thr;
}

// LATE pieces, first half of a filter over the n_rows keys in sh.keys: counts this thread's
// rows that reach the threshold (`mine`), their rank among the workgroup's (`incl`, inclusive),
// and has the last thread reserve list space for all of them; the reservation's answer, which
// takes a microsecond or two, is only needed by late_write.
__device__ __forceinline__ void late_count(const Emit &em, SharedAttn &sh, int n_rows, uint32_t thr,
                                           uint32_t &mine, uint32_t &incl, int &base)
{
    mine = 0;
    for (int i = threadIdx.x; i < n_rows; i += kThreads) mine += (uint32_t)(sh.keys[i] >= thr);
    uint32_t total;
    incl = block_scan(mine, sh.scan, total);
    base = 0;
    if (threadIdx.x == kThreads - 1 && total > 0)
        base = __hip_atomic_fetch_add((LYCHEE_GLOBAL int32_t *)em.count, (int32_t)total, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
}
// Second half: sh.cand_base holds the reservation; row i of the window is position first_row + i.
__device__ __forceinline__ void late_write(const Emit &em, SharedAttn &sh, int first_row, int n_rows, uint32_t thr,
                                           uint32_t mine, uint32_t incl)
{
    int at = sh.cand_base + (int)(incl - mine);
    for (int i = threadIdx.x; i < n_rows; i += kThreads) {
        const uint32_t key = sh.keys[i];
        if (key >= thr) {
            if (at < em.cap) gstore(em.list + at, (unsigned long long)key | ((unsigned long long)(uint32_t)(first_row + i) << 32));
            ++at;
        }
    }
}

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
template <int NH, bool GATHER, bool LATE>
__device__ __forceinline__ void stream_rows(const Common &c, const uint16_t *kbase,
                                            const uint16_t *vbase, const uint4 (&qf)[NH],
                                            Acc<NH> &acc, int L, int r0, int r1,
                                            const int32_t *idx_s, const Emit &em, float sel_mul,
                                            unsigned long long *cand_buf, int &cand_left,
                                            float &pool_m, float &pool_l, SharedAttn &sh)
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
    const int n_units = units_of(c, L);  // set entries at or beyond this name nothing

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
                // (reading a tile's four entries unconditionally and ahead of the address
                // arithmetic removes the branches the compiler puts around these reads, and
                // made the gather launch 3.5 % slower)
                const int e = (r < r1) ? idx_s[(r - r0) >> bshift] : -1;
                // the entry is range-checked before it is shifted: a junk entry of 2^25 or more
                // would otherwise wrap to a negative position that passes `tpos < L`
                const bool named = (uint32_t)e < (uint32_t)n_units;
                const int tpos = named ? (e << bshift) + (r & ((1 << bshift) - 1)) : 0;
                ok = named && (tpos < L);
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
    for (int span = 0; span < n_spans; ++span) {
        float sel0[4], sel1[4];
        consume(t0, sel0);
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
            m = max_halves32(max_rows16(m));
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
            if (LATE) {
                // the threshold may not exist yet: keep the key; a full window of keys is
                // filtered here, the piece's last window when the piece ends (run_piece)
                constexpr int kWindowSpans = kKeyBuf / kSpan;
                if (ch < 8) sh.keys[(r - r0) & (kKeyBuf - 1)] = key;
                if (((span + 1) & (kWindowSpans - 1)) == 0 && span + 1 < n_spans) {  // uniform in the workgroup
                    __syncthreads();
                    const uint32_t thr = late_threshold(em, sh);
                    uint32_t mine, incl;
                    int base;
                    late_count(em, sh, kKeyBuf, thr, mine, incl, base);
                    if (threadIdx.x == kThreads - 1) sh.cand_base = base;
                    __syncthreads();
                    late_write(em, sh, r0 + (span + 1) * kSpan - kKeyBuf, kKeyBuf, thr, mine, incl);
                    __syncthreads();
                }
                continue;
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
// LATE: the piece runs in a launch that also computes its thresholds and merges its partials
// (lychee_layer_kernel): keys are filtered at the end of the piece, and the partial is written
// through to device memory, complete when run_piece returns.
template <int NH, bool GATHER, bool LATE, typename Hook>
__device__ __forceinline__ void run_piece(const Common &c, const uint16_t *q, const uint16_t *k_cache,
                                          const uint16_t *v_cache, const int32_t *idx_src,
                                          const Emit &em, float *part_o, float *part_ml,
                                          int32_t *part_count, int b, int g, uint32_t hmask, int L,
                                          int r0, int r1, int slot, bool ends_segment,
                                          SharedAttn &sh, Hook &at_rows_done)
{
    // The thread index is made opaque here: the LDS addresses below that derive from it were
    // otherwise computed once per kernel, for every variant of this function, kept across
    // everything and spilled.
    uint32_t tix = threadIdx.x;
    asm volatile("" : "+v"(tix));
    const int lane = (int)(tix & 63u);
    const int wave = (int)(tix >> 6);
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
    if (LATE && !GATHER && threadIdx.x == 0) {  // (barriers lie between this and the first use)
        sh.late_have = em.thr_known;
        sh.late_thr = em.thr;
    }

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
            stream_rows<NH, true, LATE>(c, kbase, vbase, qf, acc, L, e0, e1, sh.idx_s, em, 0.0f, nullptr, cand_left, pool_m, pool_l, sh);
        }
    } else {
        stream_rows<NH, false, LATE>(c, kbase, vbase, qf, acc, L, r0, r1, nullptr, em, sel_mul, sh.cand[wave], cand_left, pool_m, pool_l, sh);
    }
    const bool collects = !GATHER && em.list != nullptr && em.direct == 0;  // the same in every wavefront

    at_rows_done();  // what the caller wants in flight while the partial is merged and written
    if (!LATE && collects && lane == 0) sh.cand_left[wave] = cand_left;
    // Merge the 4 row slots of the wavefront (lanes l, l^16, l^32, l^48).
    const float c_log2e = c.scale_log2e;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        const float mw = max_halves32(max_rows16(acc.m[h]));
        const float a = fast_exp2((acc.m[h] - mw) * c_log2e);
        acc.m[h] = mw;
        float lw = acc.l[h] * a;
        lw = sum_halves32(sum_rows16(lw));
        acc.l[h] = lw;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float ow = acc.o[h][e] * a;
            ow = sum_halves32(sum_rows16(ow));
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
    // (the accumulators go to LDS first: nothing below needs them, and kept in registers across
    // the key filter they were spilled)
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
    int cand_base = 0;
    uint32_t late_thr = 0, late_mine = 0, late_incl = 0;
    // the piece's last window of keys: rows late_first .. r1 - 1
    const int late_first = r0 + (r1 - r0 > 0 ? (r1 - r0 - 1) / kKeyBuf * kKeyBuf : 0);
    if (LATE && collects) {
        late_thr = late_threshold(em, sh);
        late_count(em, sh, r1 - late_first, late_thr, late_mine, late_incl, cand_base);
    }
    if (!LATE && collects && threadIdx.x == kThreads - 1) {
        // room for the workgroup's last candidates, asked for by a thread that writes no
        // partial, as early as every wavefront's count is known: the answer is on its way
        // while the others merge
        int n = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) n += sh.cand_left[w];
        if (n > 0)
            cand_base = __hip_atomic_fetch_add((LYCHEE_GLOBAL int32_t *)em.count, (int32_t)n, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
    }
    if (pooled_lse && lane == 0) {
        sh.pool_ml[2 * wave] = pool_m;
        sh.pool_ml[2 * wave + 1] = pool_l;
    }
    __syncthreads();
    if (collects && threadIdx.x == kThreads - 1) sh.cand_base = cand_base;
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
            if (LATE) {
                gstore_through(part_o + prow * kHeadDim + threadIdx.x, o);
                if (threadIdx.x == 0) {
                    gstore_through(part_ml + prow * 2 + 0, M);
                    gstore_through(part_ml + prow * 2 + 1, l);
                }
            } else {
                gstore(part_o + prow * kHeadDim + threadIdx.x, o);
                if (threadIdx.x == 0) {
                    gstore(part_ml + prow * 2 + 0, M);
                    gstore(part_ml + prow * 2 + 1, l);
                }
            }
            if (threadIdx.x == 0 && ends_segment) gstore(part_count + bh, (int32_t)(slot + 1));
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
    if (LATE && collects) {
        __syncthreads();
        late_write(em, sh, late_first, r1 - late_first, late_thr, late_mine, late_incl);
    } else if (collects) {
        __syncthreads();
        int base = sh.cand_base;
        for (int w = 0; w < wave; ++w) base += sh.cand_left[w];
        const unsigned long long *buf = sh.cand[wave];
        for (int i = lane; i < cand_left; i += 64)
            if (base + i < em.cap) gstore(em.list + base + i, buf[i]);
    }
    if (LATE) wait_stores();  // the partial has reached device memory
}

template <bool GATHER, bool LATE, typename Hook>
__device__ __forceinline__ void dispatch_piece(int nh, const Common &c, const uint16_t *q,
                                               const uint16_t *k_cache, const uint16_t *v_cache,
                                               const int32_t *idx_src, const Emit &em, float *part_o,
                                               float *part_ml, int32_t *part_count, int b, int g,
                                               uint32_t hmask, int L, int r0, int r1, int slot,
                                               bool ends_segment, SharedAttn &sh, Hook &at_rows_done)
{
    switch (nh) {
    case 1: run_piece<1, GATHER, LATE>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    case 2: run_piece<2, GATHER, LATE>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    case 3: run_piece<3, GATHER, LATE>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    default: run_piece<4, GATHER, LATE>(c, q, k_cache, v_cache, idx_src, em, part_o, part_ml, part_count, b, g, hmask, L, r0, r1, slot, ends_segment, sh, at_rows_done); break;
    }
}


}  // namespace
}  // namespace lychee
