// Host side of liblychee: argument checks, the split plan, workspace carving and the
// stream-ordered launch sequence of one layer call (attention units -> combine -> select)
// and of a whole decode step (Alg. 1's layer loop restricted to its per-head loop).
#include "../../include/lychee.h"
#include "lychee_internal.h"

#include <math.h>
#include <string.h>

#include <new>
#include <vector>

using namespace lychee;

struct lychee_ctx {
    int device = 0;
    int n_cu = 256;
    int32_t wg_per_cu = 2;
    int32_t pipeline = 1;
    int32_t cost_s2 = 3, cost_c = 1, cost_s1 = 1;
    int32_t g_block_rows = 48;
    int32_t n_wg = 0;  // 0 = n_cu * wg_per_cu
    bool timing = false;
    struct Rec {
        int cls;
        hipEvent_t start, stop;
    };
    std::vector<Rec> recs;         // events recorded since the last read
    std::vector<hipEvent_t> pool;  // events free for reuse
};

namespace {

constexpr int kWsWg = 768;      // partial slots per head the workspace provides
constexpr int kSelRing = 3;     // layers whose selection scores are alive at once (pipelined step)
constexpr int kPartRing = 4;
constexpr int kListRing = 2;

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int32_t slice_cap(int32_t max_len)
{
    const int64_t per = (max_len + kSlices - 1) / kSlices;
    return (int32_t)round_up(per, kSliceQuantum);
}

struct Workspace {
    size_t sel_off[kSelRing], part_o_off[kPartRing], part_ml_off[kPartRing], part_count_off[kPartRing];
    size_t list_off[kListRing], list_count_off[kListRing], idx_off[2], total;
    int32_t sel_stride, list_cap;
};

Workspace carve(const lychee_shape &s)
{
    Workspace w;
    w.sel_stride = (int32_t)round_up(s.max_len, 64);
    w.list_cap = slice_cap(s.max_len);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = (size_t)round_up((int64_t)(off + bytes), 256);
        return at;
    };
    const size_t heads = (size_t)s.batch * s.n_q_heads;
    const size_t groups = (size_t)s.batch * s.n_kv_heads;
    for (int i = 0; i < kSelRing; ++i) w.sel_off[i] = take(groups * w.sel_stride * sizeof(float));
    for (int i = 0; i < kPartRing; ++i) {
        w.part_o_off[i] = take(heads * kWsWg * kHeadDim * sizeof(float));
        w.part_ml_off[i] = take(heads * kWsWg * 2 * sizeof(float));
        w.part_count_off[i] = take(heads * sizeof(int32_t));
    }
    for (int i = 0; i < kListRing; ++i) {
        w.list_off[i] = take(groups * kSlices * (size_t)w.list_cap * sizeof(uint2));
        w.list_count_off[i] = take(groups * kSlices * sizeof(int32_t));
    }
    for (int i = 0; i < 2; ++i) w.idx_off[i] = take(groups * s.k * sizeof(int32_t));
    w.total = off;
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
    if (s->kv_stride_tok < kHeadDim || s->kv_stride_batch < 0 || s->kv_stride_head < 0)
        return LYCHEE_EINVAL;
    if (s->kv_stride_tok % 8 || s->kv_stride_head % 8 || s->kv_stride_batch % 8) return LYCHEE_EINVAL;
    if (s->batch > 1 && s->kv_stride_batch == 0) return LYCHEE_EINVAL;
    if (s->n_kv_heads > 1 && s->kv_stride_head == 0) return LYCHEE_EINVAL;
    return LYCHEE_OK;
}

// The head-type structure of one layer, as the kernels want it.
struct Groups {
    int n_rgroups = 0, n_sgroups = 0;
    uint8_t rgroup[kMaxKvHeads], sgroup[kMaxKvHeads], rmask[kMaxKvHeads], rindex[kMaxKvHeads];
};

Groups make_groups(const lychee_shape &s, const uint8_t *mask)  // mask == nullptr: all retrieval
{
    Groups gr;
    memset(&gr, 0, sizeof gr);
    const int G = s.n_q_heads / s.n_kv_heads;
    for (int g = 0; g < s.n_kv_heads; ++g) {
        uint32_t bits = 0;
        for (int i = 0; i < G; ++i)
            if (mask == nullptr || mask[g * G + i]) bits |= 1u << i;
        gr.rmask[g] = (uint8_t)bits;
        gr.rindex[g] = 0xFF;
        if (bits != 0) {
            gr.rindex[g] = (uint8_t)gr.n_rgroups;
            gr.rgroup[gr.n_rgroups++] = (uint8_t)g;
        }
        if (bits != (1u << G) - 1u) gr.sgroup[gr.n_sgroups++] = (uint8_t)g;
    }
    return gr;
}

// One layer's tensors and where its intermediate results live.
struct LayerIo {
    const void *q, *k_cache, *v_cache;
    void *out;
    const int32_t *idx_in;
    int32_t *idx_out;
    Groups gr;
    bool emit_sel, want_select;
    int sel_slot, part_slot, list_slot;
};

struct Planner {
    const lychee_ctx *ctx;
    const lychee_shape &s;
    const Workspace &w;
    char *ws;
    const int32_t *lengths;

    LaunchPlan blank() const
    {
        LaunchPlan p;
        memset(&p, 0, sizeof p);
        Common &c = p.c;
        c.lengths = lengths;
        c.stride_b = s.kv_stride_batch;
        c.stride_h = s.kv_stride_head;
        c.stride_t = s.kv_stride_tok;
        c.batch = s.batch;
        c.n_q_heads = s.n_q_heads;
        c.n_kv_heads = s.n_kv_heads;
        c.group = s.n_q_heads / s.n_kv_heads;
        c.k = s.k;
        c.max_len = s.max_len;
        c.sel_stride = w.sel_stride;
        c.list_cap = w.list_cap;
        int n_wg = ctx->n_wg > 0 ? ctx->n_wg : ctx->n_cu * ctx->wg_per_cu;
        c.n_wg = n_wg > kWsWg ? kWsWg : n_wg;
        c.part_stride = kWsWg;
        c.g_block_rows = ctx->g_block_rows;
        c.cost_s2 = ctx->cost_s2;
        c.cost_c = ctx->cost_c;
        c.cost_s1 = ctx->cost_s1;
        c.scale = (float)(1.0 / sqrt((double)kHeadDim));
        c.scale_log2e = (float)(1.4426950408889634 / sqrt((double)kHeadDim));
        return p;
    }
    float *part_o(int slot) const { return reinterpret_cast<float *>(ws + w.part_o_off[slot]); }
    float *part_ml(int slot) const { return reinterpret_cast<float *>(ws + w.part_ml_off[slot]); }
    int32_t *part_count(int slot) const { return reinterpret_cast<int32_t *>(ws + w.part_count_off[slot]); }
    float *sel(int slot) const { return reinterpret_cast<float *>(ws + w.sel_off[slot]); }

    void add_r(LaunchPlan &p, const LayerIo &io) const
    {
        if (io.gr.n_rgroups == 0) return;
        RPart &r = p.r;
        r.enabled = 1;
        r.q = static_cast<const uint16_t *>(io.q);
        r.k_cache = static_cast<const uint16_t *>(io.k_cache);
        r.v_cache = static_cast<const uint16_t *>(io.v_cache);
        r.sel = sel(io.sel_slot);
        r.part_o = part_o(io.part_slot);
        r.part_ml = part_ml(io.part_slot);
        r.part_count = part_count(io.part_slot);
        r.n_rgroups = io.gr.n_rgroups;
        r.emit_sel = io.emit_sel ? 1 : 0;
        memcpy(r.rgroup, io.gr.rgroup, sizeof r.rgroup);
        memcpy(r.rmask, io.gr.rmask, sizeof r.rmask);
    }
    void add_g(LaunchPlan &p, const LayerIo &io) const
    {
        if (io.gr.n_sgroups == 0) return;
        GPart &g = p.g;
        g.enabled = 1;
        g.q = static_cast<const uint16_t *>(io.q);
        g.k_cache = static_cast<const uint16_t *>(io.k_cache);
        g.v_cache = static_cast<const uint16_t *>(io.v_cache);
        g.idx = io.idx_in;
        g.part_o = part_o(io.part_slot);
        g.part_ml = part_ml(io.part_slot);
        g.part_count = part_count(io.part_slot);
        g.n_sgroups = io.gr.n_sgroups;
        memcpy(g.sgroup, io.gr.sgroup, sizeof g.sgroup);
        memcpy(g.rmask, io.gr.rmask, sizeof g.rmask);
    }
    void add_c(LaunchPlan &p, const LayerIo &io) const
    {
        CPart &c = p.comb;
        c.enabled = 1;
        c.part_o = part_o(io.part_slot);
        c.part_ml = part_ml(io.part_slot);
        c.part_count = part_count(io.part_slot);
        c.out = static_cast<uint16_t *>(io.out);
    }
    void add_s1(LaunchPlan &p, const LayerIo &io) const
    {
        if (!io.want_select || io.gr.n_rgroups == 0) return;
        S1Part &a = p.s1;
        a.enabled = 1;
        a.sel = sel(io.sel_slot);
        a.list = reinterpret_cast<uint2 *>(ws + w.list_off[io.list_slot]);
        a.list_count = reinterpret_cast<int32_t *>(ws + w.list_count_off[io.list_slot]);
        a.n_rgroups = io.gr.n_rgroups;
    }
    void add_s2(LaunchPlan &p, const LayerIo &io) const
    {
        if (!io.want_select) return;
        S2Part &a = p.s2;
        a.enabled = 1;
        a.sel = sel(io.sel_slot);
        a.list = reinterpret_cast<const uint2 *>(ws + w.list_off[io.list_slot]);
        a.list_count = reinterpret_cast<const int32_t *>(ws + w.list_count_off[io.list_slot]);
        a.idx_in = io.idx_in;
        a.idx_out = io.idx_out;
        a.n_rgroups = io.gr.n_rgroups;
        memcpy(a.rindex, io.gr.rindex, sizeof a.rindex);
    }
};

bool is_empty(const LaunchPlan &p)
{
    return !p.r.enabled && !p.g.enabled && !p.comb.enabled && !p.s1.enabled && !p.s2.enabled;
}

int launch_class(const LaunchPlan &p)
{
    if (p.r.enabled || p.g.enabled) return LYCHEE_KERNEL_ATTN;
    if (p.comb.enabled || p.s1.enabled) return LYCHEE_KERNEL_COMBINE;
    return LYCHEE_KERNEL_SELECT;
}

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

int submit(lychee_ctx *ctx, const LaunchPlan &p, hipStream_t stream)
{
    if (is_empty(p)) return LYCHEE_OK;
    if (!ctx->timing) return launch_units(p, stream) == hipSuccess ? LYCHEE_OK : LYCHEE_EHIP;
    lychee_ctx::Rec r{launch_class(p), take_event(ctx), take_event(ctx)};
    if (r.start == nullptr || r.stop == nullptr) return LYCHEE_EHIP;
    if (hipEventRecord(r.start, stream) != hipSuccess) return LYCHEE_EHIP;
    if (launch_units(p, stream) != hipSuccess) return LYCHEE_EHIP;
    if (hipEventRecord(r.stop, stream) != hipSuccess) return LYCHEE_EHIP;
    ctx->recs.push_back(r);
    return LYCHEE_OK;
}

// One layer, three dependent launches: R+G, then S1+C, then S2.
int run_layer(lychee_ctx *ctx, const Planner &pl, const LayerIo &io, hipStream_t stream)
{
    LaunchPlan a = pl.blank();
    pl.add_r(a, io);
    pl.add_g(a, io);
    int rc = submit(ctx, a, stream);
    if (rc != LYCHEE_OK) return rc;
    LaunchPlan b = pl.blank();
    pl.add_s1(b, io);
    pl.add_c(b, io);
    if ((rc = submit(ctx, b, stream)) != LYCHEE_OK) return rc;
    LaunchPlan c = pl.blank();
    pl.add_s2(c, io);
    return submit(ctx, c, stream);
}

int check_common(lychee_ctx *ctx, const lychee_shape *shape, const void *workspace,
                 size_t workspace_bytes)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    const int rc = check_shape(shape);
    if (rc != LYCHEE_OK) return rc;
    if (workspace == nullptr || !aligned(workspace, 256)) return LYCHEE_EWORKSPACE;
    if (workspace_bytes < carve(*shape).total) return LYCHEE_EWORKSPACE;
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
    ctx->device = device;
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
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
    return carve(*shape).total;
}

int lychee_decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                       const void *k_cache, const void *v_cache, const uint8_t *head_type_mask,
                       const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_common(ctx, shape, workspace, workspace_bytes);
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
    const Workspace w = carve(*shape);
    const Planner pl{ctx, *shape, w, static_cast<char *>(workspace), lengths};
    LayerIo io{q, k_cache, v_cache, out, idx_in, idx_out, make_groups(*shape, head_type_mask),
               true, true, 0, 0, 0};
    return run_layer(ctx, pl, io, static_cast<hipStream_t>(hip_stream));
}

int lychee_dense_decode_attn(lychee_ctx *ctx, const lychee_shape *shape, const void *q,
                             const void *k_cache, const void *v_cache, void *out,
                             const int32_t *lengths, void *workspace, size_t workspace_bytes,
                             void *hip_stream)
{
    int rc = check_common(ctx, shape, workspace, workspace_bytes);
    if (rc != LYCHEE_OK) return rc;
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(lengths, 4))
        return LYCHEE_EINVAL;
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const Workspace w = carve(*shape);
    const Planner pl{ctx, *shape, w, static_cast<char *>(workspace), lengths};
    LayerIo io{q, k_cache, v_cache, out, nullptr, nullptr, make_groups(*shape, nullptr),
               false, false, 0, 0, 0};
    return run_layer(ctx, pl, io, static_cast<hipStream_t>(hip_stream));
}

int lychee_decode_step(lychee_ctx *ctx, const lychee_shape *shape, int32_t n_layers,
                       const void *const *q, const void *const *k_cache,
                       const void *const *v_cache, const uint8_t *head_type_masks,
                       const int32_t *idx_in, void *const *out, int32_t *idx_out,
                       const int32_t *lengths, void *workspace, size_t workspace_bytes,
                       void *hip_stream)
{
    int rc = check_common(ctx, shape, workspace, workspace_bytes);
    if (rc != LYCHEE_OK) return rc;
    if (n_layers < 1 || q == nullptr || k_cache == nullptr || v_cache == nullptr ||
        out == nullptr || head_type_masks == nullptr || lengths == nullptr)
        return LYCHEE_EINVAL;
    if (!aligned(idx_in, 4) || !aligned(idx_out, 4) || !aligned(lengths, 4)) return LYCHEE_EINVAL;
    if (idx_in != nullptr && idx_in == idx_out) return LYCHEE_EINVAL;
    for (int l = 0; l < n_layers; ++l) {
        if (q[l] == nullptr || k_cache[l] == nullptr || v_cache[l] == nullptr || out[l] == nullptr)
            return LYCHEE_EINVAL;
        if (!aligned(q[l], 16) || !aligned(k_cache[l], 16) || !aligned(v_cache[l], 16) ||
            !aligned(out[l], 16))
            return LYCHEE_EINVAL;
        // only layer 0 can lack an inherited set: every later layer receives the previous one's
        rc = check_mask(shape, head_type_masks + (size_t)l * shape->n_q_heads, l > 0 || idx_in != nullptr);
        if (rc != LYCHEE_OK) return rc;
    }
    if ((rc = make_current(ctx)) != LYCHEE_OK) return rc;
    const Workspace w = carve(*shape);
    char *ws = static_cast<char *>(workspace);
    const Planner pl{ctx, *shape, w, ws, lengths};
    int32_t *buf[2] = {reinterpret_cast<int32_t *>(ws + w.idx_off[0]),
                       reinterpret_cast<int32_t *>(ws + w.idx_off[1])};
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    // layer l reads the sets idx(l) and writes idx(l+1); idx(0) = idx_in, idx(n) = idx_out
    auto sets_of = [&](int l) -> int32_t * {
        if (l == n_layers && idx_out != nullptr) return idx_out;
        return buf[l & 1];
    };
    auto io_of = [&](int l) {
        const bool want = l < n_layers - 1 || idx_out != nullptr;
        return LayerIo{q[l], k_cache[l], v_cache[l], out[l],
                       l == 0 ? idx_in : sets_of(l), sets_of(l + 1),
                       make_groups(*shape, head_type_masks + (size_t)l * shape->n_q_heads),
                       want, want, l % kSelRing, l % kPartRing, l % kListRing};
    };
    if (!ctx->pipeline) {
        for (int l = 0; l < n_layers; ++l)
            if ((rc = run_layer(ctx, pl, io_of(l), stream)) != LYCHEE_OK) return rc;
        return LYCHEE_OK;
    }
    // Software pipeline over launches t: the streaming of layer t shares a launch with the
    // select phases, the gather and the combine of earlier layers, whose inputs were all
    // written by earlier launches:
    //   R(t)  |  S1(t-1)  |  S2(t-2), G(t-2)  |  C(t-3)
    // G(l) needs the sets S2(l-1) wrote one launch before; C(l) needs R(l) and G(l).
    for (int t = 0; t < n_layers + 3; ++t) {
        LaunchPlan p = pl.blank();
        if (t < n_layers) pl.add_r(p, io_of(t));
        if (t - 1 >= 0 && t - 1 < n_layers) pl.add_s1(p, io_of(t - 1));
        if (t - 2 >= 0 && t - 2 < n_layers) {
            pl.add_s2(p, io_of(t - 2));
            pl.add_g(p, io_of(t - 2));
        }
        if (t - 3 >= 0 && t - 3 < n_layers) pl.add_c(p, io_of(t - 3));
        if ((rc = submit(ctx, p, stream)) != LYCHEE_OK) return rc;
    }
    return LYCHEE_OK;
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
                                   shape->max_len, dev, stream) == hipSuccess;
    ok = ok && hipMemcpyAsync(&host, dev, sizeof host, hipMemcpyDeviceToHost, stream) == hipSuccess;
    ok = ok && hipStreamSynchronize(stream) == hipSuccess;
    (void)hipFree(dev);
    if (!ok) return LYCHEE_EHIP;
    *n_bad = (int64_t)host;
    return LYCHEE_OK;
}

int lychee_set_option(lychee_ctx *ctx, int32_t option, int32_t value)
{
    if (ctx == nullptr) return LYCHEE_EINVAL;
    switch (option) {
    case LYCHEE_OPT_WG_PER_CU:
        if (value < 1 || value > 3) return LYCHEE_EINVAL;
        ctx->wg_per_cu = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_PIPELINE:
        ctx->pipeline = value != 0;
        return LYCHEE_OK;
    case LYCHEE_OPT_N_WG:
        if (value < 0 || value > kWsWg) return LYCHEE_EINVAL;
        ctx->n_wg = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_GATHER_BLOCK:
        if (value < 16 || value > 128 || value % 16) return LYCHEE_EINVAL;
        ctx->g_block_rows = value;
        return LYCHEE_OK;
    case LYCHEE_OPT_COST_S2:
    case LYCHEE_OPT_COST_C:
    case LYCHEE_OPT_COST_S1:
        if (value < 0 || value > 4096) return LYCHEE_EINVAL;
        (option == LYCHEE_OPT_COST_S2 ? ctx->cost_s2 : option == LYCHEE_OPT_COST_C ? ctx->cost_c : ctx->cost_s1) = value;
        // the kernel's balancing needs costs that do not increase from S2 to C to S1
        if (ctx->cost_c > ctx->cost_s2) ctx->cost_c = ctx->cost_s2;
        if (ctx->cost_s1 > ctx->cost_c) ctx->cost_s1 = ctx->cost_c;
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
    case LYCHEE_EUNSUPPORTED: return "unsupported shape (head_dim must be 128, at most 4 query heads per KV head, at most 64 KV heads, batch at most 256)";
    case LYCHEE_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LYCHEE_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

}  // extern "C"
