// The single launch of one layer call (Alg. 1, one pass of the layer loop's per-head loop).
//
// A model that decodes layer after layer computes the next layer's query from this layer's
// output, so the layer's work cannot be pooled with other layers', and at 128K a layer is only
// about 30 microseconds of HBM time: every dependent launch (each costs a few microseconds of gap,
// a prologue and a tail) shows.  This kernel therefore runs the whole layer in ONE launch and
// hands results from workgroup to workgroup inside it:
//
//   front units  (the first n_front workgroups, before anything else; they wait for nothing)
//       S  the select of the PREVIOUS layer call (Eq. 2), left pending by that call: its set is
//          read again only by this layer's sparse heads (Sec. 3.1), so it runs beside this
//          layer's streaming instead of after the previous layer's; copies of the sets of KV
//          heads that keep theirs
//       T  the selection thresholds of this layer (a sample of each score row)
//   R pieces     Eq. 1 / o = A V over this layer's cache rows.  The threshold of a piece's score
//                row is computed by a T unit of the same launch, so the piece keeps its rows'
//                keys in LDS and filters them when it ends (by then the T unit, about half as
//                long as a piece, has published the threshold; a piece polls for it if not)
//   G pieces     Eq. 3 over the inherited set, on the last workgroups of the grid; a piece polls
//                until the front unit that writes its KV head's set has published it
//   combine      every piece writes its partial through to device memory and counts itself in;
//                the piece that completes a segment merges the segment's partials into `out`
//
// Waiting is safe because every wait is for a front unit, front units never wait, and they run
// on the lowest workgroup indices, which are dispatched first; waits are bounded all the same.
// Partials cross from one XCD's L2 to another's without the agent-scope release fence (its
// write-back of the whole L2, executed by every workgroup, costs more than the layer): they are
// written with write-through stores, the writer waits until those have completed before it
// counts itself in, and the merging workgroup takes an acquire fence.  The sets are handed over
// the same way: written through, waited for, then flagged.
#include "lychee_internal.h"
#include "lychee_device.h"
#include "lychee_stream.h"
#include "lychee_select.h"

namespace lychee {
namespace {

struct SharedLayer {
    int32_t pre[kMaxBatch + 1];  // first block of every sequence in this workgroup's row space
    int32_t len[kMaxBatch];
    uint32_t scan[kWaves + 1];
    unsigned long long scan64[kWaves + 1];
    float fred[kWaves + 1];
    int32_t flag;
    int32_t role[2][4];            // per kind of piece: first workgroup, workgroups, segments per sequence, blocks
    uint32_t nb[2][kMaxBatch];     // per kind: blocks of one segment of every sequence
    int32_t run[3];                // the piece loop: next block of this workgroup's run, blocks per run, padded
    uint32_t gen;                  // the generation of this launch's flags
};
union SharedRole {
    SharedAttn attn;  // a piece
    SharedUnit unit;  // a front unit, or the combine that follows a piece
};

__device__ __forceinline__ uint32_t load_agent(const uint32_t *p)
{
    return __hip_atomic_load((const LYCHEE_GLOBAL uint32_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(uint32_t *p, uint32_t v)
{
    __hip_atomic_store((LYCHEE_GLOBAL uint32_t *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A front unit has written the set of (b, g), with write-through stores: once every wavefront's
// stores have completed the set is in device memory, and the flag says so.
__device__ __forceinline__ void publish_set(uint32_t *flag, uint32_t gen)
{
    wait_stores();
    __syncthreads();
    if (threadIdx.x == 0) store_agent(flag, gen);
}

// Before a gather piece reads a set that a front unit of this launch writes.
__device__ __forceinline__ void await_set(const uint32_t *flag, uint32_t gen, uint32_t *timeouts, SharedLayer &pool)
{
    if (threadIdx.x == 0) {
        int spin = 0;
        for (; spin < kSpinMax; ++spin) {
            if (load_agent(flag) == gen) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (spin == kSpinMax) atomicAdd(timeouts, 1u);  // (the piece then reads whatever the array holds; entries are range-checked)
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

template <bool COLLECT, int SELECTS>
__global__ __launch_bounds__(kThreads, 2) void lychee_layer_kernel(const LayerLaunch P)
{
    __shared__ SharedRole sh;
    __shared__ SharedLayer pool;
    // Both layer descriptors are staged in LDS, one word per thread, and read from there.  (The
    // kernel argument is never indexed with a run-time value: for `idx_src[g]` the compiler
    // emitted a scalar load whose base register held `argument + g` and whose offset register
    // held `7 g` - only their sum is a multiple of 4 -, and the scalar memory unit drops the
    // low bits of each, so that the load returned the halves of two neighbouring pointers.)
    __shared__ __align__(16) uint32_t desc_cur[kDescWords], desc_prev[kDescWords];
    const Common &c = P.c;
    const int w = blockIdx.x;
    const int W = c.n_wg;
    const int tid = threadIdx.x;

    // The generation is only ever used by thread 0 (it sets, polls and advances the flags), which
    // keeps it in a register: the load is not waited for before its first use, late in the launch.
    const uint32_t gen = tid == 0 ? load_agent(P.gen) : 0u;
    if (tid < c.batch) pool.len[tid] = clamp_len(c.lengths[tid], c.max_len);
    if (tid < kDescWords) {
        desc_cur[tid] = reinterpret_cast<const uint32_t *>(&P.cur)[tid];
        desc_prev[tid] = reinterpret_cast<const uint32_t *>(&P.prev)[tid];
    }
    __syncthreads();
    const LayerDesc &cur = *reinterpret_cast<const LayerDesc *>(desc_cur);
    const LayerDesc &prev = *reinterpret_cast<const LayerDesc *>(desc_prev);
    const uint32_t *dw = desc_cur;
    uint32_t *timeouts = c.stats + 2;

    // ------------------------------------------------------------------ front units
    if (w < P.n_front) {
        const int n_rp = P.has_prev ? prev.n_rgroups : 0;
        const int nS = SELECTS ? c.batch * n_rp : 0;
        const int nC = P.has_prev && prev.copy_keep ? c.batch * (c.n_kv_heads - n_rp) : 0;
        const int nT = COLLECT && P.has_cur && cur.emit_sel && c.block_shift == 0 ? c.batch * cur.n_rgroups * kThrSplit : 0;
        for (int j = w; j < nS + nC + nT; j += P.n_front) {
            if (j < nS) {
                const int b = j / n_rp;
                const int g = prev.rgroup[j % n_rp];
                if (SELECTS == 1) select_unit<false>(c, prev, b, g, sh.unit.sel, pool);
                if (SELECTS == 2) select_unit<true>(c, prev, b, g, sh.unit.sel, pool);
                publish_set(P.set_flags + b * c.n_kv_heads + g, gen);
            } else if (j < nS + nC) {
                const int n_keep = c.n_kv_heads - n_rp;
                const int u = j - nS;
                const int b = u / n_keep;
                int want = u % n_keep, g = 0;
                for (int gg = 0; gg < c.n_kv_heads; ++gg)
                    if (prev.rindex[gg] == 0xFF && want-- == 0) g = gg;
                copy_set_unit(c, prev, b, g);
                publish_set(P.set_flags + b * c.n_kv_heads + g, gen);
            } else {
                // a score row's sample is dealt to kThrSplit units: one round of loads each
                const int u = (j - nS - nC) / kThrSplit;
                const int n_rc = cur.n_rgroups;
                const int b = u / n_rc, rgi = u % n_rc;
                const int64_t row = (int64_t)b * n_rc + rgi;
                unsigned long long *flag = P.thr_flags + row;
                ThrSplit split;
                split.sub = (j - nS - nC) % kThrSplit;
                split.n_sub = kThrSplit;
                split.keys = reinterpret_cast<uint32_t *>(cur.sel + row * c.sel_stride);  // (free until a select ranks this row whole)
                split.arrived = P.thr_arrived + row;
                switch (__builtin_popcount(cur.rmask[cur.rgroup[rgi]] & ((1u << c.group) - 1u))) {
                case 1: threshold_unit<1>(c, cur, b, rgi, sh.unit.sel, pool, flag, gen, split); break;
                case 2: threshold_unit<2>(c, cur, b, rgi, sh.unit.sel, pool, flag, gen, split); break;
                case 3: threshold_unit<3>(c, cur, b, rgi, sh.unit.sel, pool, flag, gen, split); break;
                default: threshold_unit<4>(c, cur, b, rgi, sh.unit.sel, pool, flag, gen, split); break;
                }
            }
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ the two row spaces
    // Per sequence: blocks of 64 cache rows per retrieval KV head, blocks of gathered rows per
    // sparse KV head.  The workgroups after the front ones are split between the two kinds.
    // Everything the piece loop needs afterwards is left in LDS and read again after every
    // piece: a piece wants every vector register, and whatever the schedule kept in registers
    // across it was spilled to scratch memory by all workgroups (a launch with a scratch
    // segment also starts its wavefronts more slowly).
    // (A single sequence needs no scans over the batch: every thread evaluates it for itself.)
    const bool single = c.batch == 1;
    {
        const int n_rseg = P.has_cur ? (int)desc_u32(dw, offsetof(LayerDesc, n_rgroups)) : 0;
        const int n_gseg = P.has_cur ? (int)desc_u32(dw, offsetof(LayerDesc, n_sgroups)) : 0;
        uint32_t nb_r = 0, nb_g = 0;
        if (tid < c.batch || single) {
            const int L = pool.len[single ? 0 : tid];
            nb_r = n_rseg ? (uint32_t)((L + kBlockRows - 1) / kBlockRows) : 0u;
            nb_g = n_gseg ? (uint32_t)((gather_rows(c, L) + gather_block(c) - 1) / gather_block(c)) : 0u;
        }
        unsigned long long tot64 = (unsigned long long)nb_r | ((unsigned long long)nb_g << 32);
        if (!single) (void)block_scan64(tot64, pool.scan64, tot64);
        // (the totals are the same in every lane: scalar arithmetic from here on)
        const int64_t TR = (int64_t)uni((uint32_t)tot64) * n_rseg;
        const int64_t TG = (int64_t)uni((uint32_t)(tot64 >> 32)) * n_gseg;
        const int first = W >= 8 ? P.n_front : 0;  // tiny grids: the front workgroups also take pieces
        const int Wn = W - first;
        int W_R = 0, W_G = 0;
        if (Wn < 2) {  // a single workgroup does both kinds, one after the other
            W_R = TR > 0;
            W_G = TG > 0;
        } else if (TR > 0 && TG > 0) {
            // Gathers that wait for a select start late: by then every workgroup could have streamed
            // a = lead_blocks / Wn blocks.  Both kinds end together when a streaming workgroup takes u
            // blocks and a gathering one u - a:  TR / u + TG / (u - a) = Wn, the larger root of
            // Wn u^2 - (Wn a + TR + TG) u + TR a = 0.  Single precision is plenty (any split is a
            // valid one), and every workgroup evaluates the same operations on the same values, so
            // all agree on it.
            const float tr = (float)TR, tg = (float)TG, wn = (float)Wn;
            const float lead = P.has_prev && P.gate_mask != 0 ? (float)P.lead_blocks : 0.0f;
            const float inv_wn = __builtin_amdgcn_rcpf(wn);
            const float a = lead * inv_wn;
            const float half_b = 0.5f * (lead + tr + tg);
            float disc = half_b * half_b - tr * lead;
            disc = disc > 0.0f ? disc : 0.0f;
            const float u = (half_b + __builtin_amdgcn_sqrtf(disc)) * inv_wn;
            int wg = u - a > 0.0f ? (int)(tg * __builtin_amdgcn_rcpf(u - a) + 0.5f) : Wn;
            // a gather piece is a chain of latencies (flag, set entries, rows, merge) of about 10 us
            // whatever its size: few gather blocks get a workgroup each rather than a queue on two
            const int floor_wg = TG < Wn / 8 ? (int)TG : Wn / 8;
            wg = wg < floor_wg ? floor_wg : wg;
            // and the streaming keeps at least a third of the workgroups its share of the blocks would give it
            const int most = Wn - (int)(wn * tr * __builtin_amdgcn_rcpf(3.0f * (tr + tg)));
            wg = wg > most ? most : wg;
            W_G = wg < 1 ? 1 : (wg > Wn - 1 ? Wn - 1 : wg);
            W_R = Wn - W_G;
        } else if (TG > 0) {
            W_G = Wn;
        } else if (TR > 0) {
            W_R = Wn;
        }
        if (tid == 0) {
            pool.role[0][0] = first;
            pool.role[0][1] = W_R;
            pool.role[0][2] = n_rseg;
            pool.role[0][3] = (int32_t)TR;
            pool.role[1][0] = Wn < 2 ? first : first + W_R;
            pool.role[1][1] = W_G;
            pool.role[1][2] = n_gseg;
            pool.role[1][3] = (int32_t)TG;
            pool.gen = gen;  // (its load, issued when the kernel started, has long arrived)
        }
        if (tid < c.batch) {
            pool.nb[0][tid] = nb_r;
            pool.nb[1][tid] = nb_g;
        }
    }
    __syncthreads();

    for (int kind = 0; kind < 2; ++kind) {
        const bool gather = kind == 1;
        {
            const int role_n = uni(pool.role[kind][1]);
            const int wl = w - uni(pool.role[kind][0]);
            if (role_n <= 0 || wl < 0 || wl >= role_n) continue;  // (uniform in the workgroup)
            const int nseg = uni(pool.role[kind][2]);
            const int T_real = uni(pool.role[kind][3]);
            const uint32_t nb_mine = single ? pool.nb[kind][0] : (tid < c.batch ? pool.nb[kind][tid] : 0u);

            // Equal contiguous runs of blocks; when the segments are few, every segment is padded to
            // a whole number of runs, so that each workgroup has exactly one piece (a second piece
            // costs a second start-up and merge, which a launch this short cannot level out).
            int share = (T_real + role_n - 1) / role_n;
            int pad = 0;
            if (8ll * nseg * c.batch <= role_n) {
                const int s_last = share + (share / 8 > 1 ? share / 8 : 1);
                int s = share;
                for (; s <= s_last; ++s) {
                    uint32_t runs = nseg * ((nb_mine + s - 1) / s), all = runs;
                    if (!single) (void)block_scan(runs, pool.scan, all);
                    if ((int)all <= role_n) break;
                }
                if (s <= s_last) share = s, pad = 1;
            }
            const uint32_t mine = pad ? nseg * ((nb_mine + share - 1) / share) * share : nseg * nb_mine;
            uint32_t all;
            const uint32_t incl = single ? mine : block_scan(mine, pool.scan, all);
            if (tid < c.batch) pool.pre[tid + 1] = (int32_t)incl;
            if (tid == 0) {
                pool.pre[0] = 0;
                pool.run[0] = wl * share;  // the next block of this workgroup's run
                pool.run[1] = share;
                pool.run[2] = pad;
            }
        }
        __syncthreads();

        // One piece: where it lies, from the values in LDS alone.
        struct Piece {
            int b, g, len_b, r0, r1, slot, pieces, len;
            uint32_t hmask;
            bool ends, padding;
        };
        auto piece_at = [&](int x, int x1, int share, int pad) {
            Piece pc;
            const int brows = gather ? gather_block(c) : kBlockRows;
            pc.b = uni(find_item(pool.pre, c.batch, x));
            pc.len_b = uni(pool.len[pc.b]);
            const int seg_rows = gather ? gather_rows(c, pc.len_b) : pc.len_b;
            const int nb = (seg_rows + brows - 1) / brows;
            const int nbv = pad ? (nb + share - 1) / share * share : nb;
            const int pre_b = uni(pool.pre[pc.b]);
            const int xo = x - pre_b;
            const int gi = xo / nbv;
            const int blk = xo % nbv;
            pc.padding = blk >= nb;  // the run lies in a segment's padding
            const int seg_start = pre_b + gi * nbv;
            int len = x1 - x;
            len = len < nb - blk ? len : nb - blk;
            pc.len = len;
            pc.r0 = blk * brows;
            const int r1 = (blk + len) * brows;
            pc.r1 = r1 < seg_rows ? r1 : seg_rows;
            pc.slot = x / share - seg_start / share;
            pc.pieces = (seg_start + nb - 1) / share - seg_start / share + 1;
            pc.ends = blk + len == nb;
            const uint32_t gmask = (1u << c.group) - 1u;
            if (!gather) {
                pc.g = (int)desc_u8(dw, offsetof(LayerDesc, rgroup) + gi);
                pc.hmask = desc_u8(dw, offsetof(LayerDesc, rmask) + pc.g) & gmask;
            } else {
                pc.g = (int)desc_u8(dw, offsetof(LayerDesc, sgroup) + gi);
                pc.hmask = ~desc_u8(dw, offsetof(LayerDesc, rmask) + pc.g) & gmask;
            }
            return pc;
        };

        for (;;) {
            int x, x1, share, pad;
            auto where = [&]() {
                x = uni(pool.run[0]);
                share = uni(pool.run[1]);
                pad = uni(pool.run[2]);
                const int T = uni(pool.pre[c.batch]);
                x1 = (w - uni(pool.role[kind][0])) * share + share;
                x1 = x1 < T ? x1 : T;
            };
            where();
            if (x >= x1) break;
            {
                const Piece pc = piece_at(x, x1, share, pad);
                if (pc.padding) break;
                auto nothing = []() {};
                const uint16_t *dq = desc_ptr<const uint16_t>(dw, offsetof(LayerDesc, q));
                const uint16_t *dk = desc_ptr<const uint16_t>(dw, offsetof(LayerDesc, k_cache));
                const uint16_t *dv = desc_ptr<const uint16_t>(dw, offsetof(LayerDesc, v_cache));
                float *d_part_o = desc_ptr<float>(dw, offsetof(LayerDesc, part_o));
                float *d_part_ml = desc_ptr<float>(dw, offsetof(LayerDesc, part_ml));
                int32_t *d_part_count = desc_ptr<int32_t>(dw, offsetof(LayerDesc, part_count));
                const uint32_t my_gen = pool.gen;
                if (!gather) {
                    const int n_rseg = uni(pool.role[0][2]);
                    const int gi = (int)desc_u8(dw, offsetof(LayerDesc, rindex) + pc.g);
                    Emit em{};
                    if (COLLECT && desc_u32(dw, offsetof(LayerDesc, emit_sel))) {
                        const int64_t row = (int64_t)pc.b * n_rseg + gi;
                        em.list = desc_ptr<unsigned long long>(dw, offsetof(LayerDesc, list)) + row * c.list_row;
                        em.count = desc_ptr<int32_t>(dw, offsetof(LayerDesc, list_count)) + row;
                        em.cap = c.list_row;
                        em.direct = c.block_shift != 0;
                        if (c.prob_rule != 0)
                            em.pool_ml = desc_ptr<float>(dw, offsetof(LayerDesc, part_pool)) + row * (2 * (int64_t)c.part_stride);
                        // rows that need no sample have their threshold at once (what the T unit would say)
                        const int n = budget_of(c, pc.len_b);
                        em.thr_known = n == pc.len_b || pc.len_b <= kDirectLen || 2 * (int64_t)n >= pc.len_b;
                        em.thr = n == pc.len_b && c.prob_rule == 0 ? 0xFFFFFFFFu : 0u;
                        em.thr_flag = P.thr_flags + row;
                        em.gen = my_gen;
                        em.timeouts = timeouts;
                    }
                    dispatch_piece<false, true>(__builtin_popcount(pc.hmask), c, dq, dk, dv, nullptr, em, d_part_o, d_part_ml,
                                                d_part_count, pc.b, pc.g, pc.hmask, pc.len_b, pc.r0, pc.r1, pc.slot, pc.ends,
                                                sh.attn, nothing);
                } else {
                    if ((P.gate_mask >> pc.g) & 1ull)
                        await_set(P.set_flags + pc.b * c.n_kv_heads + pc.g, my_gen, timeouts, pool);
                    const int32_t *idx_src = desc_ptr<const int32_t>(dw, offsetof(LayerDesc, idx_src) + 8 * (size_t)pc.g) +
                                             ((int64_t)pc.b * c.n_kv_heads + pc.g) * c.k;
                    dispatch_piece<true, true>(__builtin_popcount(pc.hmask), c, dq, dk, dv, idx_src, Emit{}, d_part_o, d_part_ml,
                                               d_part_count, pc.b, pc.g, pc.hmask, pc.len_b, pc.r0, pc.r1, pc.slot, pc.ends,
                                               sh.attn, nothing);
                }
            }
            // The piece's partials are in device memory.  Count it in; whoever completes the
            // segment merges its partials (slots 0 .. pieces-1 of every head of the segment).
            __syncthreads();
            where();
            const Piece pc = piece_at(x, x1, share, pad);
            if (tid == 0) {
                int last = 1;
                if (pc.pieces > 1) {
                    uint32_t *counter = P.seg_count + (((int64_t)pc.b * c.n_kv_heads + pc.g) * 2 + kind);
                    const uint32_t old = __hip_atomic_fetch_add((LYCHEE_GLOBAL uint32_t *)counter, 1u, __ATOMIC_RELAXED,
                                                                __HIP_MEMORY_SCOPE_AGENT);
                    last = old == (uint32_t)pc.pieces - 1u;
                    if (last) store_agent(counter, 0u);  // as every launch finds it
                }
                pool.flag = last;
                pool.run[0] = x + pc.len;
            }
            __syncthreads();
            if (pool.flag) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                switch (__builtin_popcount(pc.hmask)) {
                case 1: combine_segment<1>(c, cur, pc.b, pc.g, pc.hmask, pc.pieces, sh.unit.comb); break;
                case 2: combine_segment<2>(c, cur, pc.b, pc.g, pc.hmask, pc.pieces, sh.unit.comb); break;
                case 3: combine_segment<3>(c, cur, pc.b, pc.g, pc.hmask, pc.pieces, sh.unit.comb); break;
                default: combine_segment<4>(c, cur, pc.b, pc.g, pc.hmask, pc.pieces, sh.unit.comb); break;
                }
            }
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ the generation moves on
    if (tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add((LYCHEE_GLOBAL uint32_t *)P.exit_count, 1u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
        if (old == (uint32_t)W - 1u) {
            store_agent(P.exit_count, 0u);
            store_agent(P.gen, pool.gen + 1u);
        }
    }
}

}  // namespace


hipError_t launch_layer(const LayerLaunch &plan, int build, hipStream_t stream)
{
    if (plan.c.n_wg < 1 || plan.c.n_wg > kMaxWg || plan.n_front > plan.c.n_wg) return hipErrorInvalidValue;
    const dim3 grid(plan.c.n_wg), block(kThreads);
    if (build == 0)
        hipLaunchKernelGGL((lychee_layer_kernel<false, 0>), grid, block, 0, stream, plan);
    else if (build == 1)
        hipLaunchKernelGGL((lychee_layer_kernel<true, 1>), grid, block, 0, stream, plan);
    else
        hipLaunchKernelGGL((lychee_layer_kernel<true, 2>), grid, block, 0, stream, plan);
    return hipGetLastError();
}

}  // namespace lychee
