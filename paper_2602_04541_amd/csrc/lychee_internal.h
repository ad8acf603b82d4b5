// Internal declarations shared by the host side and the gfx950 kernels of liblychee.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lychee {

constexpr int kHeadDim = 128;
constexpr int kMaxKvHeads = 64;
constexpr int kMaxGroup = 4;
constexpr int kAttnThreads = 256;            // 4 wavefronts of 64 lanes
constexpr int kAttnWaves = kAttnThreads / 64;
constexpr int kTileRows = 16;                // rows one wavefront handles per iteration
constexpr int kMinUnitRows = 128;
constexpr int kMaxUnitRows = 65536;
constexpr int kMaxSparseUnit = 2048;         // set entries staged in LDS per sparse unit
constexpr int kSelectThreads = 1024;
constexpr float kMinusBig = -1.0e30f;        // "no score yet" sentinel of the running maximum

// Everything the attention-units kernel needs, passed by value as the kernel argument.
// A *unit* is the work of one workgroup: a run of `unit_r` cache rows of one
// (sequence, KV head) for that group's retrieval heads, or a run of `unit_s` entries of the
// inherited set for that group's sparse heads.
struct AttnPlan {
    const uint16_t *q;
    const uint16_t *k_cache;
    const uint16_t *v_cache;
    const int32_t *idx_in;
    const int32_t *lengths;
    float *sel;      // [B][n_rgroups][sel_stride] pooled selection scores (scaled logits)
    float *part_o;   // [B][H_q][s_max][128] un-normalised partial outputs
    float *part_ml;  // [B][H_q][s_max][2]   running maximum (raw dot units) and sum
    int64_t stride_b, stride_h, stride_t;
    int32_t batch, n_q_heads, n_kv_heads, group;
    int32_t k, max_len, sel_stride, s_max;
    int32_t unit_r, nsplit_r;
    int32_t unit_s, nsplit_s;
    int32_t n_rgroups, n_sgroups;
    int32_t emit_sel;
    float scale;        // 1 / sqrt(head_dim)
    float scale_log2e;  // log2(e) / sqrt(head_dim)
    uint8_t rgroup[kMaxKvHeads];  // KV heads whose group holds a retrieval head
    uint8_t sgroup[kMaxKvHeads];  // KV heads whose group holds a sparse head
    uint8_t rmask[kMaxKvHeads];   // per KV head: bit i set = query head g*G+i is a retrieval head
};

struct CombinePlan {
    const float *part_o;
    const float *part_ml;
    uint16_t *out;  // bf16 [B][H_q][128]
    int32_t batch, n_q_heads, group, s_max;
    int32_t nsplit_r, nsplit_s;
    float scale_log2e;
    uint8_t rmask[kMaxKvHeads];
};

struct SelectPlan {
    const float *sel;
    const int32_t *idx_in;
    const int32_t *lengths;
    int32_t *idx_out;
    int32_t batch, n_kv_heads, k, max_len, sel_stride, n_rgroups;
    uint8_t rindex[kMaxKvHeads];  // position of KV head g among the retrieval groups, 0xFF = none
};

hipError_t launch_attn_units(const AttnPlan &plan, hipStream_t stream);
hipError_t launch_combine(const CombinePlan &plan, hipStream_t stream);
hipError_t launch_select(const SelectPlan &plan, hipStream_t stream);
hipError_t launch_validate_idx(const int32_t *idx, const int32_t *lengths, int32_t batch,
                               int32_t n_kv_heads, int32_t k, int32_t max_len,
                               unsigned long long *n_bad, hipStream_t stream);
hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t stream);
hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t stream);

}  // namespace lychee
