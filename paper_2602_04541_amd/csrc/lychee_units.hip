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
// (This file holds the two kernels and their launchers; the units themselves are in
// lychee_stream.h (R, G) and lychee_select.h (C, T, S, A), on the primitives of lychee_device.h.)
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
#include "lychee_device.h"
#include "lychee_stream.h"
#include "lychee_select.h"

namespace lychee {
namespace {

// ------------------------------------------------------------------------------ the kernels
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
}

// Launches that carry pooled R and G rows.  Two workgroups per CU must fit (the static shares
// assume that every workgroup runs from the start): at most 256 registers per lane.
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
    // Tickets: workgroup w's first chunk is chunk w, without asking; every later one is W plus
    // what the counter hands out, asked for a chunk ahead.  (All workgroups asking at the start
    // of the launch were served one after the other, and the first barrier waited for it.)
    uint32_t next_ticket = (uint32_t)w;
    if (threadIdx.x == 0) {
        if (w == 0) c.tickets[(c.ticket_slot + kTicketRing / 2) % kTicketRing] = 0u;
    }

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
                Emit em{};
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
                dispatch_piece<false, false>(__builtin_popcount(hmask), c, dq, dk, dv, nullptr, em, d_part_o, d_part_ml,
                                      d_part_count, b, g, hmask, len_b, r0, r1, slot, ends, sa, at_rows_done);
            } else {
                const int g = (int)desc_u8(dw, offsetof(LayerDesc, sgroup) + gi);
                const uint32_t hmask = ~desc_u8(dw, offsetof(LayerDesc, rmask) + g) & gmask;
                const int32_t *idx_src = desc_ptr<const int32_t>(dw, offsetof(LayerDesc, idx_src) + 8 * (size_t)g) +
                                         ((int64_t)b * c.n_kv_heads + g) * c.k;
                dispatch_piece<true, false>(__builtin_popcount(hmask), c, dq, dk, dv, idx_src, Emit{},
                                     d_part_o, d_part_ml, d_part_count, b, g, hmask, len_b, r0, r1, slot, ends, sa,
                                     at_rows_done);
            }
            if (ahead_layer >= 0) {  // wave-uniform; readers of this buffer finished a piece ago
                if (threadIdx.x < kDescWords) desc_s[cur ^ 1][threadIdx.x] = ahead;
                held[cur ^ 1] = ahead_layer;
            }
            x += len;
        }
        // next chunk: every workgroup asks until it is told that none is left
        __syncthreads();
        if (threadIdx.x == 0) pool.scan[0] = next_ticket;
        __syncthreads();
        const int ticket = (int)pool.scan[0];
        __syncthreads();
        if (ticket >= n_chunks) break;
        if (threadIdx.x == 0) next_ticket = (uint32_t)W + atomicAdd(counter, 1u);
        item = n_static + ticket;
        x = T_static + ticket * chunk;
        x1 = x + chunk;
        x1 = x1 < T ? x1 : T;
    }
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
