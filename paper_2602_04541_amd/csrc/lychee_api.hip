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
    int32_t unit_r = 0, unit_s = 0;  // 0 = automatic
    bool timing = false;
    struct Rec {
        int cls;
        hipEvent_t start, stop;
    };
    std::vector<Rec> recs;       // events recorded since the last read
    std::vector<hipEvent_t> pool;  // events free for reuse
};

namespace {

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

struct Workspace {
    size_t sel_off, part_o_off, part_ml_off, idx_a_off, idx_b_off, total;
    int32_t sel_stride, s_max;
};

Workspace carve(const lychee_shape &s)
{
    Workspace w;
    w.sel_stride = (int32_t)round_up(s.max_len, 64);
    w.s_max = (int32_t)((s.max_len + kMinUnitRows - 1) / kMinUnitRows);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = (size_t)round_up((int64_t)(off + bytes), 256);
        return at;
    };
    w.sel_off = take((size_t)s.batch * s.n_kv_heads * w.sel_stride * sizeof(float));
    w.part_o_off = take((size_t)s.batch * s.n_q_heads * w.s_max * kHeadDim * sizeof(float));
    w.part_ml_off = take((size_t)s.batch * s.n_q_heads * w.s_max * 2 * sizeof(float));
    w.idx_a_off = take((size_t)s.batch * s.n_kv_heads * s.k * sizeof(int32_t));
    w.idx_b_off = take((size_t)s.batch * s.n_kv_heads * s.k * sizeof(int32_t));
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
    if (s->max_len > (1 << 24) || s->batch > (1 << 16)) return LYCHEE_EUNSUPPORTED;
    if (s->kv_stride_tok < kHeadDim || s->kv_stride_batch < 0 || s->kv_stride_head < 0)
        return LYCHEE_EINVAL;
    if (s->kv_stride_tok % 8 || s->kv_stride_head % 8 || s->kv_stride_batch % 8) return LYCHEE_EINVAL;
    if (s->batch > 1 && s->kv_stride_batch == 0) return LYCHEE_EINVAL;
    if (s->n_kv_heads > 1 && s->kv_stride_head == 0) return LYCHEE_EINVAL;
    return LYCHEE_OK;
}

// The unit sizes: enough equally sized units to load every CU a few times over.
void choose_units(const lychee_ctx *ctx, const lychee_shape &s, int n_rgroups, int n_sgroups,
                  int32_t &unit_r, int32_t &unit_s)
{
    const int64_t kk = s.k < s.max_len ? s.k : s.max_len;
    const int64_t rows = (int64_t)s.batch * ((int64_t)n_rgroups * s.max_len + (int64_t)n_sgroups * kk);
    const int64_t target_units = (int64_t)ctx->n_cu * 6;
    int64_t u = round_up((rows + target_units - 1) / target_units, 64);
    if (u < 256) u = 256;
    if (u > 4096) u = 4096;
    unit_r = ctx->unit_r > 0 ? ctx->unit_r : (int32_t)u;
    unit_s = ctx->unit_s > 0 ? ctx->unit_s : (int32_t)u;
    if (unit_s > kMaxSparseUnit) unit_s = kMaxSparseUnit;
}

struct LayerPlan {
    AttnPlan attn;
    CombinePlan comb;
    SelectPlan sel;
    bool do_select;
};

// Fills the three kernel plans of one layer call.  `mask` == nullptr means dense.
void build_layer(const lychee_ctx *ctx, const lychee_shape &s, const Workspace &w, char *ws,
                 const void *q, const void *k_cache, const void *v_cache, const uint8_t *mask,
                 const int32_t *idx_in, void *out, int32_t *idx_out, const int32_t *lengths,
                 LayerPlan &lp)
{
    const int G = s.n_q_heads / s.n_kv_heads;
    AttnPlan &a = lp.attn;
    memset(&a, 0, sizeof a);
    a.q = static_cast<const uint16_t *>(q);
    a.k_cache = static_cast<const uint16_t *>(k_cache);
    a.v_cache = static_cast<const uint16_t *>(v_cache);
    a.idx_in = idx_in;
    a.lengths = lengths;
    a.sel = reinterpret_cast<float *>(ws + w.sel_off);
    a.part_o = reinterpret_cast<float *>(ws + w.part_o_off);
    a.part_ml = reinterpret_cast<float *>(ws + w.part_ml_off);
    a.stride_b = s.kv_stride_batch;
    a.stride_h = s.kv_stride_head;
    a.stride_t = s.kv_stride_tok;
    a.batch = s.batch;
    a.n_q_heads = s.n_q_heads;
    a.n_kv_heads = s.n_kv_heads;
    a.group = G;
    a.k = s.k;
    a.max_len = s.max_len;
    a.sel_stride = w.sel_stride;
    a.s_max = w.s_max;
    a.scale = (float)(1.0 / sqrt((double)kHeadDim));
    a.scale_log2e = (float)(1.4426950408889634 / sqrt((double)kHeadDim));
    a.emit_sel = mask != nullptr ? 1 : 0;
    SelectPlan &sp = lp.sel;
    memset(&sp, 0, sizeof sp);
    for (int g = 0; g < s.n_kv_heads; ++g) {
        uint32_t bits = 0;
        for (int i = 0; i < G; ++i)
            if (mask == nullptr || mask[g * G + i]) bits |= 1u << i;
        a.rmask[g] = (uint8_t)bits;
        sp.rindex[g] = 0xFF;
        if (bits != 0) {
            sp.rindex[g] = (uint8_t)a.n_rgroups;
            a.rgroup[a.n_rgroups++] = (uint8_t)g;
        }
        if (bits != (1u << G) - 1u) a.sgroup[a.n_sgroups++] = (uint8_t)g;
    }
    choose_units(ctx, s, a.n_rgroups, a.n_sgroups, a.unit_r, a.unit_s);
    a.nsplit_r = (s.max_len + a.unit_r - 1) / a.unit_r;
    const int kk = s.k < s.max_len ? s.k : s.max_len;
    a.nsplit_s = (kk + a.unit_s - 1) / a.unit_s;

    CombinePlan &c = lp.comb;
    memset(&c, 0, sizeof c);
    c.part_o = a.part_o;
    c.part_ml = a.part_ml;
    c.out = static_cast<uint16_t *>(out);
    c.batch = s.batch;
    c.n_q_heads = s.n_q_heads;
    c.group = G;
    c.s_max = w.s_max;
    c.nsplit_r = a.nsplit_r;
    c.nsplit_s = a.nsplit_s;
    c.scale_log2e = a.scale_log2e;
    memcpy(c.rmask, a.rmask, sizeof c.rmask);

    sp.sel = a.sel;
    sp.idx_in = idx_in;
    sp.lengths = lengths;
    sp.idx_out = idx_out;
    sp.batch = s.batch;
    sp.n_kv_heads = s.n_kv_heads;
    sp.k = s.k;
    sp.max_len = s.max_len;
    sp.sel_stride = w.sel_stride;
    sp.n_rgroups = a.n_rgroups;
    lp.do_select = mask != nullptr && idx_out != nullptr;
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

template <typename F>
hipError_t timed(lychee_ctx *ctx, int cls, hipStream_t stream, F &&launch)
{
    if (!ctx->timing) return launch();
    lychee_ctx::Rec r{cls, take_event(ctx), take_event(ctx)};
    if (r.start == nullptr || r.stop == nullptr) return hipErrorOutOfMemory;
    hipError_t e = hipEventRecord(r.start, stream);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    e = hipEventRecord(r.stop, stream);
    ctx->recs.push_back(r);
    return e;
}

int run_layer(lychee_ctx *ctx, const LayerPlan &lp, hipStream_t stream)
{
    if (timed(ctx, LYCHEE_KERNEL_ATTN, stream, [&] { return launch_attn_units(lp.attn, stream); }) != hipSuccess)
        return LYCHEE_EHIP;
    if (timed(ctx, LYCHEE_KERNEL_COMBINE, stream, [&] { return launch_combine(lp.comb, stream); }) != hipSuccess)
        return LYCHEE_EHIP;
    if (lp.do_select &&
        timed(ctx, LYCHEE_KERNEL_SELECT, stream, [&] { return launch_select(lp.sel, stream); }) != hipSuccess)
        return LYCHEE_EHIP;
    return LYCHEE_OK;
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
    LayerPlan lp;
    build_layer(ctx, *shape, w, static_cast<char *>(workspace), q, k_cache, v_cache,
                head_type_mask, idx_in, out, idx_out, lengths, lp);
    return run_layer(ctx, lp, static_cast<hipStream_t>(hip_stream));
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
    LayerPlan lp;
    build_layer(ctx, *shape, w, static_cast<char *>(workspace), q, k_cache, v_cache, nullptr,
                nullptr, out, nullptr, lengths, lp);
    return run_layer(ctx, lp, static_cast<hipStream_t>(hip_stream));
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
    int32_t *buf[2] = {reinterpret_cast<int32_t *>(ws + w.idx_a_off),
                       reinterpret_cast<int32_t *>(ws + w.idx_b_off)};
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int32_t *cur_in = idx_in;
    for (int l = 0; l < n_layers; ++l) {
        int32_t *cur_out = (l == n_layers - 1 && idx_out != nullptr) ? idx_out : buf[l & 1];
        LayerPlan lp;
        build_layer(ctx, *shape, w, ws, q[l], k_cache[l], v_cache[l],
                    head_type_masks + (size_t)l * shape->n_q_heads, cur_in, out[l], cur_out, lengths, lp);
        if (l == n_layers - 1 && idx_out == nullptr) lp.do_select = false;
        rc = run_layer(ctx, lp, stream);
        if (rc != LYCHEE_OK) return rc;
        cur_in = cur_out;
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

int lychee_set_unit_rows(lychee_ctx *ctx, int32_t retrieval_rows, int32_t sparse_rows)
{
    if (ctx == nullptr || retrieval_rows < 0 || sparse_rows < 0) return LYCHEE_EINVAL;
    auto fix = [](int32_t v, int32_t hi) {
        if (v == 0) return 0;
        int64_t r = round_up(v, 64);
        if (r < kMinUnitRows) r = kMinUnitRows;
        if (r > hi) r = hi;
        return (int32_t)r;
    };
    ctx->unit_r = fix(retrieval_rows, kMaxUnitRows);
    ctx->unit_s = fix(sparse_rows, kMaxSparseUnit);
    return LYCHEE_OK;
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
    case LYCHEE_EUNSUPPORTED: return "unsupported shape (head_dim must be 128, at most 4 query heads per KV head, at most 64 KV heads)";
    case LYCHEE_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LYCHEE_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

}  // extern "C"
