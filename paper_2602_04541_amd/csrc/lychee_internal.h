// Internal declarations shared by the host side and the gfx950 kernels of liblychee.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lychee {

constexpr int kHeadDim = 128;
constexpr int kMaxKvHeads = 64;
constexpr int kMaxGroup = 4;
constexpr int kMaxBatch = 256;
#ifndef LYCHEE_THREADS
#define LYCHEE_THREADS 256
#endif
constexpr int kThreads = LYCHEE_THREADS;  // threads of every workgroup (256 or 512)
constexpr int kWaves = kThreads / 64;
constexpr int kTileRows = 16;            // rows one wavefront handles per iteration
constexpr int kBlockRows = kWaves * kTileRows;  // cache rows per block of the pooled row space
constexpr int kSliceQuantum = kThreads * 4;     // select-filter slices are multiples of this
constexpr int kMaxWg = 1024;             // upper bound of the grid of one launch
constexpr int kIdxChunk = 2048;          // set entries staged in LDS at a time
constexpr int kSlices = 32;              // slices of one score row in the select filter
constexpr int kSampleBlocks = 64;        // the threshold sample: 64 blocks of 64 scores
constexpr int kSample = 4096;
constexpr float kMinusBig = -1.0e30f;    // "no score yet" sentinel of the running maximum

// What every part of a launch shares.
struct Common {
    const int32_t *lengths;
    int64_t stride_b, stride_h, stride_t;
    int32_t batch, n_q_heads, n_kv_heads, group;
    int32_t k, max_len, sel_stride, list_cap;  // list_cap: capacity of one filter slice
    int32_t n_wg;        // grid size of this launch
    int32_t part_stride; // partial slots per head
    int32_t g_block_rows; // set entries per pooled block of gather work (fewer than kBlockRows:
                          // a gathered row costs more than a streamed one)
    int32_t cost_s2, cost_c, cost_s1;  // small-unit costs, in blocks of pooled work
    float scale;         // 1 / sqrt(head_dim)
    float scale_log2e;   // log2(e) / sqrt(head_dim)
};

// Retrieval streaming (Eq. 1, o = A V, selection scores) of one layer.
struct RPart {
    const uint16_t *q, *k_cache, *v_cache;
    float *sel;           // [B][n_rgroups][sel_stride]
    float *part_o;        // [B*H_q][part_stride][128]
    float *part_ml;       // [B*H_q][part_stride][2]
    int32_t *part_count;  // [B*H_q]
    int32_t enabled, n_rgroups, emit_sel;
    uint8_t rgroup[kMaxKvHeads];  // KV heads whose group holds a retrieval head
    uint8_t rmask[kMaxKvHeads];   // per KV head: bit i = query head g*G+i is a retrieval head
};

// Sparse gather attention (Eq. 3) of one layer.
struct GPart {
    const uint16_t *q, *k_cache, *v_cache;
    const int32_t *idx;   // [B][H_kv][k] inherited sets
    float *part_o, *part_ml;
    int32_t *part_count;
    int32_t enabled, n_sgroups;
    uint8_t sgroup[kMaxKvHeads];  // KV heads whose group holds a sparse head
    uint8_t rmask[kMaxKvHeads];
};

// Merge of the partials of one layer into its bf16 output.
struct CPart {
    const float *part_o, *part_ml;
    const int32_t *part_count;
    uint16_t *out;  // bf16 [B][H_q][128]
    int32_t enabled;
};

// Select, phase 1: threshold from a sample, ordered filter of every slice into a list.
struct S1Part {
    const float *sel;
    uint2 *list;          // [B*n_rgroups][kSlices][list_cap] (ordered key, position)
    int32_t *list_count;  // [B*n_rgroups][kSlices]
    int32_t enabled, n_rgroups;
};

// Select, phase 2: exact radix select over the filtered list, ordered write of the set.
struct S2Part {
    const float *sel;
    const uint2 *list;
    const int32_t *list_count;
    const int32_t *idx_in;
    int32_t *idx_out;
    int32_t enabled, n_rgroups;
    uint8_t rindex[kMaxKvHeads];  // position of KV head g among the retrieval groups, 0xFF = none
};

struct LaunchPlan {
    Common c;
    RPart r;
    GPart g;
    CPart comb;
    S1Part s1;
    S2Part s2;
};

hipError_t launch_units(const LaunchPlan &plan, hipStream_t stream);
hipError_t launch_validate_idx(const int32_t *idx, const int32_t *lengths, int32_t batch,
                               int32_t n_kv_heads, int32_t k, int32_t max_len,
                               unsigned long long *n_bad, hipStream_t stream);
hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t stream);
hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t stream);

}  // namespace lychee
