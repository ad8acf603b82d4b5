// Host side of liblychee: argument checks, workspace carving, the table of layer
// descriptors and the stream-ordered launch sequences of a layer call and of a decode step
// (Alg. 1's layer loop restricted to its per-head loop).
#include "../../include/lychee.h"
#include "lychee_internal.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

using namespace lychee;

namespace {
// Scratch of lychee_decode_attn_static, the entry point for callers that cannot allocate: every
// GPU the library is loaded on holds this array until the process ends.  In host code the name
// is only a handle for hipGetSymbolAddress; the device address is looked up once per context
// (lychee_create, with the context's device current) and only that address is ever passed on.
static __device__ __align__(256) unsigned char scratch[LYCHEE_STATIC_SCRATCH_BYTES];

constexpr size_t kArenaBytes = 4u << 20;  // device memory for descriptor tables, per context
constexpr size_t kArenaReserved = 512;    // its first bytes hold the ring of chunk counters (256 B)
constexpr size_t kArenaStats = 256;       // and, from here, the select's fall-back counters
}

struct lychee_ctx {
    int device = 0;
    int n_cu = 256;
    int32_t wg_per_cu = 2;
    int32_t n_wg = 0;          // 0 = n_cu * wg_per_cu
    int32_t step_mode = LYCHEE_STEP_PHASED;
    int32_t g_block_rows = 48;
    int32_t tail_permille = 250;
    int32_t select_margin = 60;  // tenths of a standard deviation, see LYCHEE_OPT_SELECT_MARGIN
    int32_t select_lead = 3000;  // blocks of 64 rows streamed while a select runs, see LYCHEE_OPT_SELECT_LEAD
    uint32_t launch_seq = 0;   // pooled launches so far: picks the chunk counter
    std::vector<int32_t> used_slots;  // counters of pooled launches that no later launch has reset yet
    bool timing = false;
    struct Rec {
        int cls;
        hipEvent_t start, stop;
    };
    std::vector<Rec> recs;         // events recorded since the last read
    std::vector<hipEvent_t> pool;  // events free for reuse
    // Descriptor tables: built on the host, staged in pinned memory, copied to the arena
    // with an asynchronous copy on the caller's stream, and cached by content so that a
    // serving loop that passes the same buffers every step uploads nothing.
    void *static_scratch = nullptr;  // this device's address of the file-scope scratch array
    // What the workgroups of a layer launch hand to one another (zeroed once, then kept clean by
    // the launches themselves): the launch generation, the threshold and set flags, the
    // segments' arrival counters, and three banks of candidate counters (banks 0 and 1 alternate
    // between the layer calls that leave their select pending; calls that do not, and the layers of a
    // layer-after-layer step, use bank 2 and whichever of the others no pending select owns).
    char *sync_dev = nullptr;
    char *arena_dev = nullptr;
    char *arena_host = nullptr;  // pinned, same layout as the device arena
    size_t arena_used = 0;
    bool arena_captured = false;  // some table was uploaded or used while a stream was being captured
    struct Cached {
        uint64_t hash;
        size_t offset, bytes;
    };
    std::vector<Cached> cache;
    std::vector<LayerDesc> descs;  // a call's layer descriptors (capacity for the most layers a step takes)
    // A layer call whose select has been left for the next call (lychee_decode_attn_deferred).
    struct Pending {
        bool active = false;
        LayerDesc desc;              // the layer, its queries redirected to the workspace's copy
        lychee_shape shape;
        const int32_t *lengths = nullptr;
        void *workspace = nullptr;
        int slot = 0;                // which of the workspace's two layer slots holds its scratch
        int bank = 0;                // which bank of candidate counters it collected into
    } pending;
};

namespace {

// Layout of lychee_ctx::sync_dev
constexpr size_t kSyncGen = 0, kSyncExit = 64;
constexpr size_t kSyncRows = (size_t)kMaxBatch * kMaxKvHeads;  // (sequence, KV head) pairs a shape can have
constexpr size_t kSyncThr = 4096;                               // uint64 [kSyncRows]
constexpr size_t kSyncSet = kSyncThr + kSyncRows * 8;           // uint32 [kSyncRows]
constexpr size_t kSyncSeg = kSyncSet + kSyncRows * 4;           // uint32 [kSyncRows][2]
constexpr size_t kSyncCount = kSyncSeg + kSyncRows * 8;         // int32 [3][kSyncRows]
constexpr size_t kSyncArrived = kSyncCount + 3 * kSyncRows * 4; // uint32 [kSyncRows]
constexpr size_t kSyncBytes = kSyncArrived + kSyncRows * 4;

constexpr int kWsWg = 768;        // largest grid a launch uses
constexpr int kPartSlots = 1024;  // partial slots per head in the workspace: static runs + chunks

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Capacity of one score row's candidate list.  A threshold unit aims at n = min(k, L)
// candidates plus six standard deviations of its sample (a few thousand at the usual sizes),
// and makes every row a candidate when L <= kDirectLen or L <= 2k.  A list that still
// overflows is not an error: the select unit then ranks the whole row itself.
int32_t list_row_entries(int32_t max_len, int32_t k)
{
    int64_t cap = 4ll * k;
    if (cap < (int64_t)k + 16384) cap = (int64_t)k + 16384;
    if (cap < max_len / 64) cap = max_len / 64;
    const int64_t all = round_up(max_len, 64);
    return (int32_t)(cap < all ? cap : all);
}

// Per-layer scratch, laid out layer after layer.
struct Workspace {
    size_t sel, part_o, part_ml, part_count, part_pool, list, list_count, thr, idx_set, q_keep;  // offsets inside a layer
    size_t layer_bytes, total;
    int32_t sel_stride, list_row;
};

Workspace carve(const lychee_shape &s, int n_layers)
{
    Workspace w;
    w.sel_stride = (int32_t)round_up(s.max_len, 64);
    w.list_row = list_row_entries(s.max_len, s.k);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = (size_t)round_up((int64_t)(off + bytes), 256);
        return at;
    };
    const size_t heads = (size_t)s.batch * s.n_q_heads;
    const size_t groups = (size_t)s.batch * s.n_kv_heads;
    w.sel = take(groups * w.sel_stride * sizeof(float));
    w.part_o = take(heads * kPartSlots * kHeadDim * sizeof(float));
    w.part_ml = take(heads * kPartSlots * 2 * sizeof(float));
    w.part_count = take(heads * sizeof(int32_t));
    w.part_pool = take(groups * kPartSlots * 2 * sizeof(float));
    w.list = take(groups * (size_t)w.list_row * sizeof(unsigned long long));
    w.list_count = take(groups * sizeof(int32_t));
    w.thr = take(groups * sizeof(uint32_t));
    w.idx_set = take(groups * s.k * sizeof(int32_t));
    w.q_keep = take(heads * kHeadDim * sizeof(uint16_t));
    w.layer_bytes = off;
    w.total = off * (size_t)n_layers;
    return w;
}

int check_shape(const lychee_shape *s)
{
    if (s == nullptr) return LYCHEE_EINVAL;
    if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->max_len < 1 || s->k < 1)
        return LYCHEE_EINVAL;
    if (s->n_q_heads % s->n_kv_heads != 0) return LYCHEE_EINVAL;
    if (s->head_dim != kHeadDim) return LYCHEE_EUNSUPPORTED;
    if (s->n_kv_heads > kMaxKvHeads) return LYCHEE_EUNSUPPORTED;
    if (s->n_q_heads / s->n_kv_heads > kMaxGroup) return LYCHEE_EUNSUPPORTED;
    if (s->max_len > (1 << 24) || s->batch > kMaxBatch) return LYCHEE_EUNSUPPORTED;
    if (s->keep_ppm < 0 || s->keep_ppm > 1000000) return LYCHEE_EINVAL;
    if (s->block_size != 0 && s->block_size != 1 && s->block_size != 64) return LYCHEE_EUNSUPPORTED;
    if (s->prob_rule < 0 || s->prob_rule > 2) return LYCHEE_EINVAL;
    if (s->prob_rule != 0) {
        if (!(s->prob_param > 0.0f && s->prob_param <= 1.0f)) return LYCHEE_EINVAL;
        if (s->keep_ppm != 0 || s->block_size == 64) return LYCHEE_EUNSUPPORTED;  // one rule at a time, on tokens
    }
    if (s->kv_stride_tok < kHeadDim || s->kv_stride_batch < 0 || s->kv_stride_head < 0)
        return LYCHEE_EINVAL;
    if (s->kv_stride_tok % 8 || s->kv_stride_head % 8 || s->kv_stride_batch % 8) return LYCHEE_EINVAL;
    if (s->batch > 1 && s->kv_stride_batch == 0) return LYCHEE_EINVAL;
    if (s->n_kv_heads > 1 && s->kv_stride_head == 0) return LYCHEE_EINVAL;
    return LYCHEE_OK;
}

int check_common(lychee_ctx *ctx, const lychee_shape *shape, const void *workspace,
                 size_t workspace_bytes, int n_layers, bool continues_pending = false)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    const int rc = check_shape(shape);
    if (rc != LYCHEE_OK) return rc;
    if (workspace == nullptr || !aligned(workspace, 256)) return LYCHEE_EWORKSPACE;
    if (workspace_bytes < carve(*shape, n_layers).total) return LYCHEE_EWORKSPACE;
    // a pending select still reads this workspace: only the call that runs it may use it
    if (!continues_pending && ctx->pending.active && ctx->pending.workspace == workspace) return LYCHEE_EINVAL;
    return LYCHEE_OK;
}

int check_mask(const lychee_shape *shape, const uint8_t *mask, bool has_idx_in)
{
    if (mask == nullptr) return LYCHEE_EINVAL;
    bool any_sparse = false;
    for (int h = 0; h < shape->n_q_heads; ++h) {
        if (mask[h] > 1) return LYCHEE_EINVAL;
        any_sparse |= mask[h] == 0;
    }
    if (any_sparse && !has_idx_in) return LYCHEE_EINVAL;
    return LYCHEE_OK;
}

int make_current(lychee_ctx *ctx)
{
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return LYCHEE_EHIP;
    if (cur != ctx->device && hipSetDevice(ctx->device) != hipSuccess) return LYCHEE_EHIP;
    return LYCHEE_OK;
}

// Fills the head-type tables of a descriptor.  mask == nullptr: every head is a retrieval head.
void set_groups(LayerDesc &d, const lychee_shape &s, const uint8_t *mask)
{
    const int G = s.n_q_heads / s.n_kv_heads;
    d.n_rgroups = d.n_sgroups = 0;
    for (int g = 0; g < s.n_kv_heads; ++g) {
        uint32_t bits = 0;
        for (int i = 0; i < G; ++i)
            if (mask == nullptr || mask[g * G + i]) bits |= 1u << i;
        d.rmask[g] = (uint8_t)bits;
        d.rindex[g] = 0xFF;
        if (bits != 0) {
            d.rindex[g] = (uint8_t)d.n_rgroups;
            d.rgroup[d.n_rgroups++] = (uint8_t)g;
        }
        if (bits != (1u << G) - 1u) d.sgroup[d.n_sgroups++] = (uint8_t)g;
    }
}

void set_scratch(LayerDesc &d, const Workspace &w, char *ws, int layer_slot)
{
    char *base = ws + (size_t)layer_slot * w.layer_bytes;
    d.sel = reinterpret_cast<float *>(base + w.sel);
    d.part_o = reinterpret_cast<float *>(base + w.part_o);
    d.part_ml = reinterpret_cast<float *>(base + w.part_ml);
    d.part_count = reinterpret_cast<int32_t *>(base + w.part_count);
    d.part_pool = reinterpret_cast<float *>(base + w.part_pool);
    d.list = reinterpret_cast<unsigned long long *>(base + w.list);
    d.list_count = reinterpret_cast<int32_t *>(base + w.list_count);
    d.thr = reinterpret_cast<uint32_t *>(base + w.thr);
}

int32_t *idx_set_of(const Workspace &w, char *ws, int layer_slot)
{
    return reinterpret_cast<int32_t *>(ws + (size_t)layer_slot * w.layer_bytes + w.idx_set);
}

// FNV-1a over 64-bit words (descriptor tables are a whole number of them).
uint64_t hash_words(const void *p, size_t bytes)
{
    const unsigned char *b = static_cast<const unsigned char *>(p);
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i + 8 <= bytes; i += 8) {
        uint64_t w;
        memcpy(&w, b + i, 8);
        h = (h ^ w) * 1099511628211ull;
    }
    return h;
}
static_assert(sizeof(LayerDesc) % 8 == 0, "tables are hashed word by word");

// Returns the device address of a table with exactly these n descriptors, uploading it (one
// asynchronous copy on `stream`) unless an identical table is already resident.
const LayerDesc *resident_table(lychee_ctx *ctx, const LayerDesc *descs, size_t n, hipStream_t stream, bool *full)
{
    *full = false;
    const size_t bytes = n * sizeof(LayerDesc);
    if (bytes > kArenaBytes - kArenaReserved) return nullptr;
    const uint64_t h = hash_words(descs, bytes);
    // A graph captured from this stream replays launches (and the table's upload, from the pinned
    // mirror) that point into the arena for as long as the graph lives: once a capture has seen the
    // arena, its tables are never recycled.
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (stream != nullptr && hipStreamIsCapturing(stream, &capturing) != hipSuccess) return nullptr;
    if (capturing != hipStreamCaptureStatusNone) ctx->arena_captured = true;
    for (const auto &e : ctx->cache)
        if (e.hash == h && e.bytes == bytes && memcmp(ctx->arena_host + e.offset, descs, bytes) == 0)
            return reinterpret_cast<const LayerDesc *>(ctx->arena_dev + e.offset);
    if (ctx->arena_used + bytes > kArenaBytes) {
        if (ctx->arena_captured) {
            *full = true;  // LYCHEE_EARENA: the caller needs a fresh context (or fewer distinct buffer sets)
            return nullptr;
        }
        // Arena full: start over.  Tables still in use by enqueued launches, and staging
        // bytes of copies still in flight, must not be overwritten, so wait for the stream.
        if (hipStreamSynchronize(stream) != hipSuccess) return nullptr;
        ctx->arena_used = kArenaReserved;
        ctx->cache.clear();
    }
    const size_t off = ctx->arena_used;
    memcpy(ctx->arena_host + off, descs, bytes);
    if (hipMemcpyAsync(ctx->arena_dev + off, ctx->arena_host + off, bytes, hipMemcpyHostToDevice, stream) != hipSuccess)
        return nullptr;
    ctx->arena_used = (size_t)round_up((int64_t)(off + bytes), 256);
    ctx->cache.push_back({h, off, bytes});
    return reinterpret_cast<const LayerDesc *>(ctx->arena_dev + off);
}

struct Ranges {
    int r_first = 0, r_count = 0, g_first = 0, g_count = 0, c_first = 0, c_count = 0;
    int t_first = 0, t_count = 0, s_first = 0, s_count = 0, a_first = 0, a_count = 0;
};

hipEvent_t take_event(lychee_ctx *ctx)
{
    if (!ctx->pool.empty()) {
        hipEvent_t e = ctx->pool.back();
        ctx->pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// The part of a launch's arguments that follows from the shape and the context alone.
void fill_common(Common &c, const lychee_ctx *ctx, const lychee_shape &s, const Workspace &w,
                 const int32_t *lengths, int n_wg)
{
    c.lengths = lengths;
    c.stride_b = s.kv_stride_batch;
    c.stride_h = s.kv_stride_head;
    c.stride_t = s.kv_stride_tok;
    c.batch = s.batch;
    c.n_q_heads = s.n_q_heads;
    c.n_kv_heads = s.n_kv_heads;
    c.group = s.n_q_heads / s.n_kv_heads;
    c.k = s.k;
    c.keep_ppm = s.keep_ppm;
    c.block_shift = s.block_size == 64 ? 6 : 0;
    c.prob_rule = s.prob_rule;
    c.prob_param = s.prob_param;
    c.max_len = s.max_len;
    c.sel_stride = w.sel_stride;
    c.list_row = w.list_row;
    c.n_wg = n_wg;
    c.part_stride = kPartSlots;
    c.g_block_rows = ctx->g_block_rows;
    c.tickets = reinterpret_cast<uint32_t *>(ctx->arena_dev);
    c.stats = reinterpret_cast<uint32_t *>(ctx->arena_dev + kArenaStats);
    c.tail_permille = ctx->tail_permille;
    // chunks small enough to level the finish times, large enough that a segment
    // never has more than ~192 of them (partial slots per head are limited)
    const int64_t seg_blocks = (s.max_len + kBlockRows - 1) / kBlockRows;
    c.chunk_blocks = (int32_t)((seg_blocks + 191) / 192);
    if (c.chunk_blocks < 2) c.chunk_blocks = 2;
    c.sel_margin = 0.1f * (float)ctx->select_margin;
    c.scale = (float)(1.0 / sqrt((double)kHeadDim));
    c.scale_log2e = (float)(1.4426950408889634 / sqrt((double)kHeadDim));
}

int grid_of(const lychee_ctx *ctx)
{
    const int n_wg = ctx->n_wg > 0 ? ctx->n_wg : ctx->n_cu * ctx->wg_per_cu;
    return n_wg > kWsWg ? kWsWg : n_wg;
}

struct Launcher {
    lychee_ctx *ctx;
    const lychee_shape &s;
    const Workspace &w;
    const int32_t *lengths;
    const LayerDesc *table;       // in device memory
    const LayerDesc *host_table;  // the same descriptors on the host
    hipStream_t stream;

    int grid() const { return grid_of(ctx); }
    int go(const Ranges &r) const
    {
        if (r.r_count + r.g_count + r.c_count + r.t_count + r.s_count + r.a_count == 0) return LYCHEE_OK;
        LaunchPlan p;
        memset(&p, 0, sizeof p);
        Common &c = p.c;
        fill_common(c, ctx, s, w, lengths, grid());
        if (r.r_count || r.g_count) {
            c.ticket_slot = (int32_t)(ctx->launch_seq++ % kTicketRing);
            ctx->used_slots.push_back(c.ticket_slot);
        } else {
            // every call ends with a small-unit launch: it resets what the call's pooled
            // launches counted (a pooled launch is never followed by more than this many)
            while (c.n_clear < 4 && !ctx->used_slots.empty()) {  // (what does not fit waits for the next small launch)
                c.clear_slot[c.n_clear++] = ctx->used_slots.back();
                ctx->used_slots.pop_back();
            }
        }
        p.layers = table;
        p.r_first = r.r_first, p.r_count = r.r_count;
        p.g_first = r.g_first, p.g_count = r.g_count;
        p.c_first = r.c_first, p.c_count = r.c_count;
        p.a_first = r.a_first, p.a_count = r.a_count;
        p.t_first = r.t_first, p.t_count = r.t_count;
        p.s_first = r.s_first, p.s_count = r.s_count;
        for (int l = r.r_first; l < r.r_first + r.r_count; ++l) p.collect |= host_table[l].emit_sel;
        if (p.collect && s.block_size != 64 && ctx->n_wg == 0 && ctx->wg_per_cu == 2) {
            // A small launch that collects candidates of a few score rows (a single layer's call
            // at batch 1) is a few percent faster with one workgroup per CU: half as many pieces
            // to start, to merge and to reserve list space for.  Batches, block-granular sets
            // (no lists) and the dense baseline are faster with two.  The bound below uses
            // max_len: the lengths are on the device.
            const int64_t seg_blocks = (s.max_len + kBlockRows - 1) / kBlockRows;
            const int64_t g_rows = s.k < s.max_len ? s.k : s.max_len;
            const int64_t g_blocks = (g_rows + c.g_block_rows - 1) / c.g_block_rows;
            int64_t t_max = 0, n_segs = 0;
            for (int l = r.r_first; l < r.r_first + r.r_count; ++l) {
                n_segs += (int64_t)host_table[l].n_rgroups * s.batch;
                t_max += (int64_t)host_table[l].n_rgroups * s.batch * seg_blocks;
            }
            for (int l = r.g_first; l < r.g_first + r.g_count; ++l) {
                n_segs += (int64_t)host_table[l].n_sgroups * s.batch;
                t_max += (int64_t)host_table[l].n_sgroups * s.batch * g_blocks;
            }
            if (8 * n_segs <= ctx->n_cu && t_max < 48ll * ctx->n_cu) c.n_wg = ctx->n_cu < kWsWg ? ctx->n_cu : kWsWg;
        }
        for (int l = r.r_first; l < r.r_first + r.r_count; ++l) p.n_rseg[l] = (uint8_t)host_table[l].n_rgroups;
        for (int l = r.t_first; l < r.t_first + r.t_count; ++l) p.n_rseg[l] = (uint8_t)host_table[l].n_rgroups;
        for (int l = r.s_first; l < r.s_first + r.s_count; ++l) {
            p.n_rseg[l] = (uint8_t)host_table[l].n_rgroups;
            p.keeps[l] = (uint8_t)(host_table[l].copy_keep != 0);
        }
        for (int l = r.g_first; l < r.g_first + r.g_count; ++l) p.n_gseg[l] = (uint8_t)host_table[l].n_sgroups;
        for (int l = r.s_first; l < r.s_first + r.s_count; ++l) p.selects |= host_table[l].n_rgroups > 0;
        const int cls = r.r_count ? LYCHEE_KERNEL_STREAM : r.g_count ? LYCHEE_KERNEL_GATHER
                        : (r.t_count || r.a_count) ? LYCHEE_KERNEL_THRESHOLD : r.c_count ? LYCHEE_KERNEL_COMBINE
                        : LYCHEE_KERNEL_SELECT;
        if (!ctx->timing) return launch_units(p, stream) == hipSuccess ? LYCHEE_OK : LYCHEE_EHIP;
        lychee_ctx::Rec rec{cls, take_event(ctx), take_event(ctx)};
        if (rec.start == nullptr || rec.stop == nullptr) return LYCHEE_EHIP;
        if (hipEventRecord(rec.start, stream) != hipSuccess) return LYCHEE_EHIP;
        if (launch_units(p, stream) != hipSuccess) return LYCHEE_EHIP;
        if (hipEventRecord(rec.stop, stream) != hipSuccess) return LYCHEE_EHIP;
        ctx->recs.push_back(rec);
        return LYCHEE_OK;
    }
};

// The pooled block space of a phased step's launches (all layers' streamed rows in one launch, all
// layers' gathered rows in another) is indexed with 32-bit integers: checked before the first launch.
int check_pooled_space(const lychee_shape &s, const LayerDesc *descs, int n_layers)
{
    const int64_t seg_blocks = (s.max_len + kBlockRows - 1) / kBlockRows;
    int64_t r_segs = 0, g_segs = 0;
    for (int l = 0; l < n_layers; ++l) r_segs += descs[l].n_rgroups, g_segs += descs[l].n_sgroups;
    const int64_t segs = r_segs > g_segs ? r_segs : g_segs;
    if (segs * s.batch * (4 * seg_blocks + 8) >= (1ll << 31)) return LYCHEE_EUNSUPPORTED;  // (gathered blocks are shorter)
    return LYCHEE_OK;
}

// The row spaces of a layer launch are indexed with 32-bit integers.
int check_layer_space(const lychee_shape &s, const LayerDesc &d)
{
    const int64_t seg_blocks = (s.max_len + kBlockRows - 1) / kBlockRows;
    if ((int64_t)(d.n_rgroups + d.n_sgroups) * s.batch * (4 * seg_blocks + 8) >= (1ll << 31))
        return LYCHEE_EUNSUPPORTED;  // (gathered blocks are shorter than streamed ones)
    return LYCHEE_OK;
}

// One launch of lychee_layer_kernel: everything `cur`'s output needs (cur may be null: only the
// pending select), with the select and set copies of `prev` (may be null) among its front units.
// Every check happens before the launch; nothing else is enqueued.
int layer_launch(lychee_ctx *ctx, const lychee_shape &s, const Workspace &w, const int32_t *lengths,
                 const LayerDesc *cur, const LayerDesc *prev, hipStream_t stream)
{
    if (cur == nullptr && prev == nullptr) return LYCHEE_OK;
    LayerLaunch p;
    memset(&p, 0, sizeof p);
    const int W = grid_of(ctx);
    fill_common(p.c, ctx, s, w, lengths, W);
    const bool blocks = s.block_size == 64;
    int64_t units = 0;
    if (prev != nullptr) {
        p.prev = *prev;
        p.has_prev = 1;
        units += (int64_t)s.batch * prev->n_rgroups;
        if (prev->copy_keep) units += (int64_t)s.batch * (s.n_kv_heads - prev->n_rgroups);
    }
    if (cur != nullptr) {
        p.cur = *cur;
        p.has_cur = 1;
        if (cur->emit_sel && !blocks) units += (int64_t)s.batch * cur->n_rgroups * kThrSplit;
        if (prev != nullptr)
            for (int g = 0; g < s.n_kv_heads; ++g)
                if (cur->idx_src[g] != nullptr && cur->idx_src[g] == prev->idx_out &&
                    (prev->rindex[g] != 0xFF || prev->copy_keep))
                    p.gate_mask |= 1ull << g;
        const int rc = check_layer_space(s, *cur);
        if (rc != LYCHEE_OK) return rc;
    } else {
        // only front units: one workgroup each, up to the usual grid
        p.c.n_wg = (int32_t)(units < 1 ? 1 : (units > W ? W : units));
    }
    // The front units get up to a quarter of the grid to themselves (a handful of workgroups in a
    // batch-1 call); a grid too small to set workgroups aside lets them take pieces afterwards.
    const int wg = p.c.n_wg;
    const int front_max = cur == nullptr ? wg : (wg >= 8 ? wg / 4 : wg);
    p.n_front = (int32_t)(units < front_max ? units : front_max);
    p.lead_blocks = ctx->select_lead;
    p.gen = reinterpret_cast<uint32_t *>(ctx->sync_dev + kSyncGen);
    p.exit_count = reinterpret_cast<uint32_t *>(ctx->sync_dev + kSyncExit);
    p.thr_flags = reinterpret_cast<unsigned long long *>(ctx->sync_dev + kSyncThr);
    p.set_flags = reinterpret_cast<uint32_t *>(ctx->sync_dev + kSyncSet);
    p.seg_count = reinterpret_cast<uint32_t *>(ctx->sync_dev + kSyncSeg);
    p.thr_arrived = reinterpret_cast<uint32_t *>(ctx->sync_dev + kSyncArrived);
    const bool selects = prev != nullptr && prev->n_rgroups > 0;
    const bool collects = cur != nullptr && cur->emit_sel;
    const int build = !(selects || collects) ? 0 : (s.prob_rule != 0 ? 2 : 1);
    if (!ctx->timing) return launch_layer(p, build, stream) == hipSuccess ? LYCHEE_OK : LYCHEE_EHIP;
    lychee_ctx::Rec rec{cur != nullptr ? LYCHEE_KERNEL_STREAM : LYCHEE_KERNEL_SELECT, take_event(ctx), take_event(ctx)};
    if (rec.start == nullptr || rec.stop == nullptr) return LYCHEE_EHIP;
    if (hipEventRecord(rec.start, stream) != hipSuccess) return LYCHEE_EHIP;
    if (launch_layer(p, build, stream) != hipSuccess) return LYCHEE_EHIP;
    if (hipEventRecord(rec.stop, stream) != hipSuccess) return LYCHEE_EHIP;
    ctx->recs.push_back(rec);
    return LYCHEE_OK;
}

// The candidate counters of a layer that a layer launch streams: one of the context's two banks.
int32_t *count_bank(lychee_ctx *ctx, int bank)
{
    return reinterpret_cast<int32_t *>(ctx->sync_dev + kSyncCount) + (size_t)bank * kSyncRows;
}

int check_step_pointers(int32_t n_layers, const void *const *q, const void *const *k_cache,
                        const void *const *v_cache, void *const *out)
{
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr) return LYCHEE_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        if (q[l] == nullptr || k_cache[l] == nullptr || v_cache[l] == nullptr || out[l] == nullptr)
            return LYCHEE_EINVAL;
        if (!aligned(q[l], 16) || !aligned(k_cache[l], 16) || !aligned(v_cache[l], 16) || !aligned(out[l], 16))
            return LYCHEE_EINVAL;
    }
    return LYCHEE_OK;
}

// The hybrid decode step; k_new / v_new (both or neither) add each layer's cache append.
int decode_step(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers, const void *const *q,
                const void *const *k_new, const void *const *v_new, const void *const *k_cache,
                const void *const *v_cache, const uint8_t *head_type_masks, const int32_t *idx_in,
                void *const *out, int32_t *idx_out, const int32_t *lengths, void *workspace,
                size_t workspace_bytes, void *hip_stream)
{
    if (n_layers < 1 || n_layers >= kMaxLayers) return n_layers < 1 ? LYCHEE_EINVAL : LYCHEE_EUNSUPPORTED;
    int rc = check_common(ctx, shape, workspace, workspace_bytes, n_layers);
    if (rc != LYCHEE_OK) return rc;
    if (head_type_masks == nullptr || lengths == nullptr) return LYCHEE_EINVAL;
    if ((rc = check_step_pointers(n_layers, q, k_cache, v_cache, out)) != LYCHEE_OK) return rc;
    if ((k_new == nullptr) != (v_new == nullptr)) return LYCHEE_EINVAL;
    if (!aligned(idx_in, 4) || !aligned(idx_out, 4) || !aligned(lengths, 4)) return LYCHEE_EINVAL;
    if (idx_in != nullptr && idx_in == idx_out) return LYCHEE_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        if (k_new != nullptr && (k_new[l] == nullptr || v_new[l] == nullptr || !aligned(k_new[l], 16) ||
                                 !aligned(v_new[l], 16)))
            return LYCHEE_EINVAL;
        // only layer 0 can lack an inherited set: every later layer receives the previous one's
        rc = check_mask(shape, head_type_masks + (size_t)l * shape->n_q_heads, l > 0 || idx_in != nullptr);
        if (rc != LYCHEE_OK) return rc;
    }
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Workspace w = carve(*shape, n_layers);
    char *ws = static_cast<char *>(workspace);

    // Layer l writes the sets of its retrieval groups into its own array; a KV head whose
    // group holds no retrieval head keeps reading the array of the last layer that selected
    // for it (Sec. 3.1: the set is propagated unchanged), so nothing is copied between layers.
    // Entry n_layers of the table only assembles the caller's idx_out from those arrays.
    const bool assemble = idx_out != nullptr;
    // the last layer's selection is only needed if the caller wants the final sets
    const int n_select = assemble ? n_layers : n_layers - 1;
    std::vector<LayerDesc> &descs = ctx->descs;  // reserved at creation: no allocation here
    descs.assign((size_t)n_layers + 1, LayerDesc{});
    const int32_t *cur[kMaxKvHeads];
    for (int g = 0; g < shape->n_kv_heads; ++g) cur[g] = idx_in;
    for (int l = 0; l < n_layers; ++l) {
        LayerDesc &d = descs[l];
        memset(&d, 0, sizeof d);
        d.q = static_cast<const uint16_t *>(q[l]);
        d.k_cache = static_cast<const uint16_t *>(k_cache[l]);
        d.v_cache = static_cast<const uint16_t *>(v_cache[l]);
        if (k_new != nullptr) {
            d.k_new = static_cast<const uint16_t *>(k_new[l]);
            d.v_new = static_cast<const uint16_t *>(v_new[l]);
        }
        d.out = static_cast<uint16_t *>(out[l]);
        set_groups(d, *shape, head_type_masks + (size_t)l * shape->n_q_heads);
        set_scratch(d, w, ws, l);
        d.idx_out = idx_set_of(w, ws, l);
        for (int g = 0; g < shape->n_kv_heads; ++g) d.idx_src[g] = cur[g];
        d.emit_sel = l < n_select;
        d.copy_keep = 0;
        for (int i = 0; i < d.n_rgroups; ++i) cur[d.rgroup[i]] = d.idx_out;
    }
    LayerDesc &fin = descs[n_layers];
    memset(&fin, 0, sizeof fin);
    for (int g = 0; g < shape->n_kv_heads; ++g) {
        fin.rindex[g] = 0xFF;
        fin.idx_src[g] = cur[g];
    }
    fin.idx_out = idx_out;
    fin.copy_keep = 1;

    // (a single layer has nothing to pool across layers: its streaming and gather share a launch)
    const bool phased = ctx->step_mode == LYCHEE_STEP_PHASED && n_layers > 1 &&
                        (int64_t)n_layers * shape->batch <= kMaxItems;
    if (!phased) {
        // Layer after layer, one launch each: out[l] is complete when launch l is.  The select of
        // layer l is read again only by layer l + 1's sparse heads, so it runs among the front
        // units of launch l + 1, beside that layer's streaming; the last layer's runs alone.
        for (int l = 0; l < n_layers; ++l)
            if ((rc = check_layer_space(*shape, descs[l])) != LYCHEE_OK) return rc;
        if (k_new != nullptr) {  // every layer's append first, in one small launch (they are all inputs of the call)
            bool full;
            const LayerDesc *table = resident_table(ctx, descs.data(), descs.size(), stream, &full);
            if (table == nullptr) return full ? LYCHEE_EARENA : LYCHEE_EHIP;
            const Launcher L{ctx, *shape, w, lengths, table, descs.data(), stream};
            Ranges t;
            t.a_first = 0, t.a_count = n_layers;
            if ((rc = L.go(t)) != LYCHEE_OK) return rc;
        }
        const int other = ctx->pending.active ? 1 - ctx->pending.bank : 0;
        LayerDesc &last = descs[n_layers - 1];
        if (assemble) {  // the last layer writes the caller's array: its own sets, copies of the kept ones
            last.idx_out = idx_out;
            last.copy_keep = 1;
        }
        for (int l = 0; l < n_layers; ++l) {
            descs[l].list_count = count_bank(ctx, (l & 1) ? other : 2);
            const LayerDesc *prev = l > 0 && descs[l - 1].emit_sel ? &descs[l - 1] : nullptr;
            if ((rc = layer_launch(ctx, *shape, w, lengths, &descs[l], prev, stream)) != LYCHEE_OK) return rc;
        }
        if (assemble && (rc = layer_launch(ctx, *shape, w, lengths, nullptr, &last, stream)) != LYCHEE_OK) return rc;
    } else {
        // All layers at once, one launch per phase; each phase needs only earlier phases:
        //   A + T (appends, thresholds)  ->  R (streaming, every layer)  ->  S (select)  ->  G (gather)  ->  C (combine)
        if ((rc = check_pooled_space(*shape, descs.data(), n_layers)) != LYCHEE_OK) return rc;
        bool full;
        const LayerDesc *table = resident_table(ctx, descs.data(), descs.size(), stream, &full);
        if (table == nullptr) return full ? LYCHEE_EARENA : LYCHEE_EHIP;
        const Launcher L{ctx, *shape, w, lengths, table, descs.data(), stream};
        Ranges t;
        t.t_first = 0, t.t_count = shape->block_size == 64 ? 0 : n_select;
        if (k_new != nullptr) t.a_first = 0, t.a_count = n_layers;
        if ((rc = L.go(t)) != LYCHEE_OK) return rc;
        Ranges r;
        r.r_first = 0, r.r_count = n_layers;
        if ((rc = L.go(r)) != LYCHEE_OK) return rc;
        Ranges sl;
        sl.s_first = 0, sl.s_count = n_select;
        if ((rc = L.go(sl)) != LYCHEE_OK) return rc;
        Ranges g;
        g.g_first = 0, g.g_count = n_layers;
        if ((rc = L.go(g)) != LYCHEE_OK) return rc;
        Ranges c;
        c.c_first = 0, c.c_count = n_layers;
        if (assemble) c.s_first = n_layers, c.s_count = 1;  // the set copies ride along
        if ((rc = L.go(c)) != LYCHEE_OK) return rc;
    }
    return LYCHEE_OK;
}

// One layer call (lychee_decode_attn; lychee_decode_attn_static with the library's own scratch).
int decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q, const void *k_cache,
                const void *v_cache, const uint8_t *head_type_mask, const int32_t *idx_in, void *out,
                int32_t *idx_out, const int32_t *lengths, void *workspace, size_t workspace_bytes,
                void *hip_stream)
{
    int rc = check_common(ctx, shape, workspace, workspace_bytes, 1);
    if (rc != LYCHEE_OK) return rc;
    rc = check_mask(shape, head_type_mask, idx_in != nullptr);
    if (rc != LYCHEE_OK) return rc;
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr ||
        idx_out == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(idx_out, 4) || !aligned(idx_in, 4) || !aligned(lengths, 4))
        return LYCHEE_EINVAL;
    if (idx_in == idx_out) return LYCHEE_EINVAL;
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Workspace w = carve(*shape, 1);
    LayerDesc d;  // (on the stack: this path allocates nothing, not even host memory)
    memset(&d, 0, sizeof d);
    d.q = static_cast<const uint16_t *>(q);
    d.k_cache = static_cast<const uint16_t *>(k_cache);
    d.v_cache = static_cast<const uint16_t *>(v_cache);
    d.out = static_cast<uint16_t *>(out);
    set_groups(d, *shape, head_type_mask);
    set_scratch(d, w, static_cast<char *>(workspace), 0);
    d.idx_out = idx_out;
    for (int g = 0; g < shape->n_kv_heads; ++g) d.idx_src[g] = idx_in;
    d.emit_sel = 1;
    d.copy_keep = 1;
    d.list_count = count_bank(ctx, 2);
    if ((rc = check_layer_space(*shape, d)) != LYCHEE_OK) return rc;
    // idx_out is complete when the call's work is: the layer's launch, then its select alone
    if ((rc = layer_launch(ctx, *shape, w, lengths, &d, nullptr, stream)) != LYCHEE_OK) return rc;
    return layer_launch(ctx, *shape, w, lengths, nullptr, &d, stream);
}

}  // namespace

extern "C" {

int lychee_create(lychee_ctx **out, int device)
{
    if (out == nullptr) return LYCHEE_EINVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return LYCHEE_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return LYCHEE_EHIP;
    lychee_ctx *ctx = new (std::nothrow) lychee_ctx();
    if (ctx == nullptr) return LYCHEE_EHIP;
    ctx->cache.reserve(kArenaBytes / 1024 + 1);  // (a table is at least a descriptor: the hot calls never grow these)
    ctx->used_slots.reserve(kTicketRing);
    ctx->descs.reserve(kMaxLayers + 1);
    ctx->device = device;
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    int cur = -1;
    bool ok = hipGetDevice(&cur) == hipSuccess && hipSetDevice(device) == hipSuccess;
    ok = ok && hipMalloc(reinterpret_cast<void **>(&ctx->arena_dev), kArenaBytes) == hipSuccess;
    ok = ok && hipHostMalloc(reinterpret_cast<void **>(&ctx->arena_host), kArenaBytes, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipMemset(ctx->arena_dev, 0, kArenaReserved) == hipSuccess;
    ok = ok && hipMalloc(reinterpret_cast<void **>(&ctx->sync_dev), kSyncBytes) == hipSuccess;
    ok = ok && hipMemset(ctx->sync_dev, 0, kSyncBytes) == hipSuccess;
    const uint32_t first_gen = 1;  // (zero is what the untouched flags hold)
    ok = ok && hipMemcpy(ctx->sync_dev + kSyncGen, &first_gen, sizeof first_gen, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipGetSymbolAddress(&ctx->static_scratch, HIP_SYMBOL(scratch)) == hipSuccess &&
         ctx->static_scratch != nullptr;
    ctx->arena_used = kArenaReserved;
    if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
    if (!ok) {
        if (ctx->arena_dev) (void)hipFree(ctx->arena_dev);
        if (ctx->sync_dev) (void)hipFree(ctx->sync_dev);
        if (ctx->arena_host) (void)hipHostFree(ctx->arena_host);
        delete ctx;
        return LYCHEE_EHIP;
    }
    *out = ctx;
    return LYCHEE_OK;
}

int lychee_destroy(lychee_ctx *ctx)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    for (auto &r : ctx->recs) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    for (auto e : ctx->pool) (void)hipEventDestroy(e);
    if (ctx->arena_dev) (void)hipFree(ctx->arena_dev);
    if (ctx->sync_dev) (void)hipFree(ctx->sync_dev);
    if (ctx->arena_host) (void)hipHostFree(ctx->arena_host);
    delete ctx;
    return LYCHEE_OK;
}

int lychee_check_shape(const lychee_shape *shape, const uint8_t *head_type_mask, int has_idx_in)
{
    const int rc = check_shape(shape);
    if (rc != LYCHEE_OK || head_type_mask == nullptr) return rc;
    return check_mask(shape, head_type_mask, has_idx_in != 0);
}

size_t lychee_workspace_bytes(const lychee_shape *shape)
{
    if (check_shape(shape) != LYCHEE_OK) return 0;
    return carve(*shape, 1).total;
}

size_t lychee_step_workspace_bytes(const lychee_shape *shape, int32_t n_layers)
{
    if (check_shape(shape) != LYCHEE_OK || n_layers < 1 || n_layers > kMaxLayers) return 0;
    return carve(*shape, n_layers).total;
}

int lychee_decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                       const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                       const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return decode_attn(ctx, shape, q, k_cache, v_cache, head_type_mask, idx_in, out, idx_out, lengths, workspace,
                       workspace_bytes, hip_stream);
}

int lychee_decode_attn_static(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                              const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                              const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                              void *hip_stream)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    const int rc = check_shape(shape);
    if (rc != LYCHEE_OK) return rc;
    // the shape's scratch must fit the static array: nothing is allocated to make room
    if (carve(*shape, 1).total > (size_t)LYCHEE_STATIC_SCRATCH_BYTES) return LYCHEE_EWORKSPACE;
    if (ctx->timing) return LYCHEE_EUNSUPPORTED;  // timing creates events: not from this entry point
    return decode_attn(ctx, shape, q, k_cache, v_cache, head_type_mask, idx_in, out, idx_out, lengths,
                       ctx->static_scratch, (size_t)LYCHEE_STATIC_SCRATCH_BYTES, hip_stream);
}

int lychee_decode_attn_deferred(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                                const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                                const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_common(ctx, shape, workspace, workspace_bytes, 2, true);
    if (rc != LYCHEE_OK) return rc;
    rc = check_mask(shape, head_type_mask, idx_in != nullptr);
    if (rc != LYCHEE_OK) return rc;
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr ||
        idx_out == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(idx_out, 4) || !aligned(idx_in, 4) || !aligned(lengths, 4))
        return LYCHEE_EINVAL;
    if (idx_in == idx_out) return LYCHEE_EINVAL;
    lychee_ctx::Pending &pd = ctx->pending;
    // a pending select reads its layer's half of this workspace with this shape and these lengths
    if (pd.active && (pd.workspace != workspace || pd.lengths != lengths || memcmp(&pd.shape, shape, sizeof *shape) != 0))
        return LYCHEE_EINVAL;
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Workspace w = carve(*shape, 2);
    char *ws = static_cast<char *>(workspace);
    const int slot = pd.active ? 1 - pd.slot : 0;
    const int bank = pd.active ? 1 - pd.bank : 0;
    LayerDesc d;
    memset(&d, 0, sizeof d);
    d.q = static_cast<const uint16_t *>(q);
    d.k_cache = static_cast<const uint16_t *>(k_cache);
    d.v_cache = static_cast<const uint16_t *>(v_cache);
    d.out = static_cast<uint16_t *>(out);
    set_groups(d, *shape, head_type_mask);
    set_scratch(d, w, ws, slot);
    d.list_count = count_bank(ctx, bank);
    // a select that ranks a whole score row needs the row's queries: the threshold units leave a
    // copy (block-granular sets never take that route: their lists are always complete)
    if (shape->block_size != 64) d.q_keep = reinterpret_cast<uint16_t *>(ws + (size_t)slot * w.layer_bytes + w.q_keep);
    d.idx_out = idx_out;
    for (int g = 0; g < shape->n_kv_heads; ++g) d.idx_src[g] = idx_in;
    d.emit_sel = 1;
    d.copy_keep = 1;
    // one launch: this layer, with the pending select among its front units
    if ((rc = layer_launch(ctx, *shape, w, lengths, &d, pd.active ? &pd.desc : nullptr, stream)) != LYCHEE_OK) return rc;
    pd.active = true;
    pd.desc = d;
    if (d.q_keep != nullptr) pd.desc.q = d.q_keep;  // the caller's q may hold the next layer's queries by then
    pd.desc.q_keep = nullptr;
    pd.shape = *shape;
    pd.lengths = lengths;
    pd.workspace = workspace;
    pd.slot = slot;
    pd.bank = bank;
    return LYCHEE_OK;
}

int lychee_select_flush(lychee_ctx *ctx, void *hip_stream)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    lychee_ctx::Pending &pd = ctx->pending;
    if (!pd.active) return LYCHEE_OK;
    int rc = make_current(ctx);
    if (rc != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Workspace w = carve(pd.shape, 2);
    if ((rc = layer_launch(ctx, pd.shape, w, pd.lengths, nullptr, &pd.desc, stream)) != LYCHEE_OK) return rc;
    pd.active = false;
    return LYCHEE_OK;
}

int lychee_dense_decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                             const void *k_cache, const void *v_cache, void *out,
                             const int32_t *lengths, void *workspace, size_t workspace_bytes,
                             void *hip_stream)
{
    int rc = check_common(ctx, shape, workspace, workspace_bytes, 1);
    if (rc != LYCHEE_OK) return rc;
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(lengths, 4))
        return LYCHEE_EINVAL;
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Workspace w = carve(*shape, 1);
    LayerDesc d;
    memset(&d, 0, sizeof d);
    d.q = static_cast<const uint16_t *>(q);
    d.k_cache = static_cast<const uint16_t *>(k_cache);
    d.v_cache = static_cast<const uint16_t *>(v_cache);
    d.out = static_cast<uint16_t *>(out);
    set_groups(d, *shape, nullptr);
    set_scratch(d, w, static_cast<char *>(workspace), 0);
    if ((rc = check_layer_space(*shape, d)) != LYCHEE_OK) return rc;
    return layer_launch(ctx, *shape, w, lengths, &d, nullptr, stream);
}

int lychee_decode_step(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                       const void *const *q, const void *const *k_cache,
                       const void *const *v_cache, const uint8_t *head_type_masks,
                       const int32_t *idx_in, void *const *out, int32_t *idx_out,
                       const int32_t *lengths, void *workspace, size_t workspace_bytes,
                       void *hip_stream)
{
    return decode_step(ctx, shape, n_layers, q, nullptr, nullptr, k_cache, v_cache, head_type_masks, idx_in, out,
                       idx_out, lengths, workspace, workspace_bytes, hip_stream);
}

int lychee_decode_step_append(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                              const void *const *q, const void *const *k_new,
                              const void *const *v_new, void *const *k_cache, void *const *v_cache,
                              const uint8_t *head_type_masks, const int32_t *idx_in,
                              void *const *out, int32_t *idx_out, const int32_t *lengths,
                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (k_new == nullptr || v_new == nullptr) return LYCHEE_EINVAL;
    return decode_step(ctx, shape, n_layers, q, k_new, v_new, k_cache, v_cache, head_type_masks, idx_in, out,
                       idx_out, lengths, workspace, workspace_bytes, hip_stream);
}

int lychee_append_kv(lychee_ctx *ctx, const lychee_shape *shape, const void *k_new, const void *v_new,
                     void *k_cache, void *v_cache, const int32_t *lengths, void *hip_stream)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    int rc = check_shape(shape);
    if (rc != LYCHEE_OK) return rc;
    if (k_new == nullptr || v_new == nullptr || k_cache == nullptr || v_cache == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) ||
        !aligned(lengths, 4))
        return LYCHEE_EINVAL;
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    std::vector<LayerDesc> &descs = ctx->descs;
    descs.assign(1, LayerDesc{});
    LayerDesc &d = descs[0];
    memset(&d, 0, sizeof d);
    d.k_cache = static_cast<const uint16_t *>(k_cache);
    d.v_cache = static_cast<const uint16_t *>(v_cache);
    d.k_new = static_cast<const uint16_t *>(k_new);
    d.v_new = static_cast<const uint16_t *>(v_new);
    bool full;
    const LayerDesc *table = resident_table(ctx, descs.data(), descs.size(), stream, &full);
    if (table == nullptr) return full ? LYCHEE_EARENA : LYCHEE_EHIP;
    const Workspace w = carve(*shape, 1);
    const Launcher L{ctx, *shape, w, lengths, table, descs.data(), stream};
    Ranges a;
    a.a_first = 0, a.a_count = 1;
    return L.go(a);
}

int lychee_dense_decode_step(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                             const void *const *q, const void *const *k_cache,
                             const void *const *v_cache, void *const *out, const int32_t *lengths,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (n_layers < 1 || n_layers >= kMaxLayers) return n_layers < 1 ? LYCHEE_EINVAL : LYCHEE_EUNSUPPORTED;
    int rc = check_common(ctx, shape, workspace, workspace_bytes, n_layers);
    if (rc != LYCHEE_OK) return rc;
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(lengths, 4)) return LYCHEE_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        if (q[l] == nullptr || k_cache[l] == nullptr || v_cache[l] == nullptr || out[l] == nullptr)
            return LYCHEE_EINVAL;
        if (!aligned(q[l], 16) || !aligned(k_cache[l], 16) || !aligned(v_cache[l], 16) ||
            !aligned(out[l], 16))
            return LYCHEE_EINVAL;
    }
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Workspace w = carve(*shape, n_layers);
    std::vector<LayerDesc> &descs = ctx->descs;
    descs.assign((size_t)n_layers, LayerDesc{});
    for (int l = 0; l < n_layers; ++l) {
        LayerDesc &d = descs[l];
        memset(&d, 0, sizeof d);
        d.q = static_cast<const uint16_t *>(q[l]);
        d.k_cache = static_cast<const uint16_t *>(k_cache[l]);
        d.v_cache = static_cast<const uint16_t *>(v_cache[l]);
        d.out = static_cast<uint16_t *>(out[l]);
        set_groups(d, *shape, nullptr);
        set_scratch(d, w, static_cast<char *>(workspace), l);
    }
    if (ctx->step_mode != LYCHEE_STEP_PHASED || n_layers == 1 || (int64_t)n_layers * shape->batch > kMaxItems) {
        if ((rc = check_layer_space(*shape, descs[0])) != LYCHEE_OK) return rc;
        for (int l = 0; l < n_layers; ++l)
            if ((rc = layer_launch(ctx, *shape, w, lengths, &descs[l], nullptr, stream)) != LYCHEE_OK) return rc;
        return LYCHEE_OK;
    }
    if ((rc = check_pooled_space(*shape, descs.data(), n_layers)) != LYCHEE_OK) return rc;
    bool full;
    const LayerDesc *table = resident_table(ctx, descs.data(), descs.size(), stream, &full);
    if (table == nullptr) return full ? LYCHEE_EARENA : LYCHEE_EHIP;
    const Launcher L{ctx, *shape, w, lengths, table, descs.data(), stream};
    Ranges r;
    r.r_first = 0, r.r_count = n_layers;
    if ((rc = L.go(r)) != LYCHEE_OK) return rc;
    Ranges c;
    c.c_first = 0, c.c_count = n_layers;
    return L.go(c);
}

int lychee_validate_idx(lychee_ctx *ctx, const lychee_shape *shape, const int32_t *idx,
                        const int32_t *lengths, int64_t *n_bad, void *hip_stream)
{
    if (ctx == nullptr || idx == nullptr || lengths == nullptr || n_bad == nullptr) return LYCHEE_EINVAL;
    int rc = check_shape(shape);
    if (rc != LYCHEE_OK) return rc;
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned long long *dev = nullptr;
    if (hipMalloc(&dev, sizeof *dev) != hipSuccess) return LYCHEE_EHIP;
    unsigned long long host = 0;
    bool ok = hipMemcpyAsync(dev, &host, sizeof host, hipMemcpyHostToDevice, stream) == hipSuccess;
    ok = ok && launch_validate_idx(idx, lengths, shape->batch, shape->n_kv_heads, shape->k,
                                   shape->max_len, shape->block_size == 64 ? 6 : 0, dev, stream) == hipSuccess;
    ok = ok && hipMemcpyAsync(&host, dev, sizeof host, hipMemcpyDeviceToHost, stream) == hipSuccess;
    ok = ok && hipStreamSynchronize(stream) == hipSuccess;
    (void)hipFree(dev);
    if (!ok) return LYCHEE_EHIP;
    *n_bad = (int64_t)host;
    return LYCHEE_OK;
}

int lychee_select_stats(lychee_ctx *ctx, int64_t *too_few, int64_t *too_many, void *hip_stream)
{
    if (ctx == nullptr || too_few == nullptr || too_many == nullptr) return LYCHEE_EINVAL;
    if (make_current(ctx) != LYCHEE_OK) return LYCHEE_EHIP;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t host[2] = {0, 0};
    if (hipMemcpyAsync(host, ctx->arena_dev + kArenaStats, sizeof host, hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return LYCHEE_EHIP;
    *too_few = host[0];
    *too_many = host[1];
    return LYCHEE_OK;
}

int lychee_wait_timeouts(lychee_ctx *ctx, int64_t *timeouts, void *hip_stream)
{
    if (ctx == nullptr || timeouts == nullptr) return LYCHEE_EINVAL;
    if (make_current(ctx) != LYCHEE_OK) return LYCHEE_EHIP;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t host = 0;
    if (hipMemcpyAsync(&host, ctx->arena_dev + kArenaStats + 8, sizeof host, hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return LYCHEE_EHIP;
    *timeouts = host;
    return LYCHEE_OK;
}

int lychee_set_option(lychee_ctx *ctx, int32_t option, int32_t value)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    switch (option) {
    case LYCHEE_OPT_DEFAULTS: {
        const lychee_ctx fresh{};
        ctx->wg_per_cu = fresh.wg_per_cu;
        ctx->n_wg = fresh.n_wg;
        ctx->step_mode = fresh.step_mode;
        ctx->g_block_rows = fresh.g_block_rows;
        ctx->tail_permille = fresh.tail_permille;
        ctx->select_margin = fresh.select_margin;
        ctx->select_lead = fresh.select_lead;
        return LYCHEE_OK;
    }
    case LYCHEE_OPT_WG_PER_CU:
        if (value < 1 || value > 3) return LYCHEE_EINVAL;
        ctx->wg_per_cu = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_STEP_MODE:
        if (value != LYCHEE_STEP_PHASED && value != LYCHEE_STEP_LAYERWISE) return LYCHEE_EINVAL;
        ctx->step_mode = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_N_WG:
        if (value < 0 || value > kWsWg) return LYCHEE_EINVAL;
        ctx->n_wg = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_TAIL_PERMILLE:
        if (value < 0 || value > 1000) return LYCHEE_EINVAL;
        ctx->tail_permille = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_SELECT_MARGIN:
        if (value < -10000 || value > 100000) return LYCHEE_EINVAL;
        ctx->select_margin = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_SELECT_LEAD:
        if (value < 0 || value > (1 << 24)) return LYCHEE_EINVAL;
        ctx->select_lead = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_GATHER_BLOCK:
        if (value < 16 || value > 128 || value % 16) return LYCHEE_EINVAL;
        ctx->g_block_rows = value;
        return LYCHEE_OK;
    default:
        return LYCHEE_EINVAL;
    }
}

int lychee_timing_enable(lychee_ctx *ctx, int on)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    ctx->timing = on != 0;
    return LYCHEE_OK;
}

int lychee_timing_read(lychee_ctx *ctx, float *ms_per_class, int32_t *launches_per_class)
{
    if (ctx == nullptr || ms_per_class == nullptr || launches_per_class == nullptr) return LYCHEE_EINVAL;
    for (int i = 0; i < LYCHEE_N_KERNEL_CLASSES; ++i) {
        ms_per_class[i] = 0.0f;
        launches_per_class[i] = 0;
    }
    int rc = LYCHEE_OK;
    for (auto &r : ctx->recs) {
        float ms = 0.0f;
        if (hipEventSynchronize(r.stop) != hipSuccess ||
            hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
            rc = LYCHEE_EHIP;
        } else {
            ms_per_class[r.cls] += ms;
            launches_per_class[r.cls] += 1;
        }
        ctx->pool.push_back(r.start);
        ctx->pool.push_back(r.stop);
    }
    ctx->recs.clear();
    return rc;
}

int lychee_probe_read(lychee_ctx *ctx, const void *src, size_t bytes, void *sink, void *hip_stream)
{
    if (ctx == nullptr || src == nullptr || sink == nullptr || bytes % 16 || !aligned(src, 16))
        return LYCHEE_EINVAL;
    if (make_current(ctx) != LYCHEE_OK) return LYCHEE_EHIP;
    return launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? LYCHEE_OK : LYCHEE_EHIP;
}

int lychee_probe_copy(lychee_ctx *ctx, void *dst, const void *src, size_t bytes, void *hip_stream)
{
    if (ctx == nullptr || src == nullptr || dst == nullptr || bytes % 16 || !aligned(src, 16) ||
        !aligned(dst, 16))
        return LYCHEE_EINVAL;
    if (make_current(ctx) != LYCHEE_OK) return LYCHEE_EHIP;
    return launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? LYCHEE_OK : LYCHEE_EHIP;
}

const char *lychee_strerror(int code)
{
    switch (code) {
    case LYCHEE_OK: return "ok";
    case LYCHEE_EINVAL: return "invalid argument";
    case LYCHEE_EUNSUPPORTED: return "unsupported shape (head_dim must be 128, at most 4 query heads per KV head, at most 64 KV heads, batch at most 256, fewer than 128 layers per step)";
    case LYCHEE_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LYCHEE_EHIP: return "HIP runtime error";
    case LYCHEE_EARENA: return "the context's descriptor arena is full and a captured graph still uses it: use a new context";
    default: return "unknown error";
    }
}

}  // extern "C"
