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
static_assert(kBlockRows == 64, "a pooled block is also the selection block of the block-granular variant");
constexpr int kMaxWg = 1024;             // upper bound of the grid of one launch
constexpr int kIdxChunk = 2048;          // set entries staged in LDS at a time
constexpr int kSampleTilesMin = 128;     // the threshold sample: 128 to 256 tiles of 16 rows
constexpr int kSampleTilesMax = 256;
constexpr int kDirectLen = 4096;         // sequences this short are ranked without a threshold
constexpr int kCandBuf = 256;            // candidates a wavefront collects in LDS between flushes
constexpr int kThrSplit = 4;             // units that share a score row's threshold sample in a layer launch
constexpr int kKeyBuf = 4096;            // rows whose keys a piece buffers in LDS when its threshold comes late
constexpr float kMinusBig = -1.0e30f;    // "no score yet" sentinel of the running maximum

constexpr int kMaxLayers = 128;          // layers one launch can cover
constexpr int kMaxItems = 2048;          // (layer, sequence) pairs of one launch's pooled rows
constexpr int kTicketRing = 64;          // chunk counters; one is cleared 32 launches before its use

// What every part of a launch shares.
struct Common {
    const int32_t *lengths;
    int64_t stride_b, stride_h, stride_t;
    int32_t batch, n_q_heads, n_kv_heads, group;
    int32_t k, max_len, sel_stride;
    int32_t keep_ppm;     // > 0: the Ratio rule's share of a sequence, in parts per million
    int32_t block_shift;  // 0: sets name positions; 6: blocks of 64 positions (App. C)
    int32_t prob_rule;    // 0: budget only; 1: Threshold, 2: Top-p (Sec. 4.4.1) with parameter
    float prob_param;     //   prob_param, on the softmax of the pooled logits
    int32_t list_row;     // capacity, in entries, of one score row's candidate list
    int32_t n_wg;         // grid size of this launch
    int32_t part_stride;  // partial slots per head
    uint32_t *tickets;    // ring of kTicketRing chunk counters, zero except the ones in use
    uint32_t *stats;      // [0] score rows ranked whole for want of candidates, [1] for a full list
    int32_t ticket_slot;  // the counter of this launch; the launch also clears the opposite one
    int32_t n_clear;      // a small-unit launch puts back to zero the counters that the pooled
    int32_t clear_slot[4];//   launches before it used: a call leaves every counter as it found it,
                          //   which is what lets a captured sequence of launches be replayed
    int32_t tail_permille;// share of the pooled blocks handed out dynamically, in chunks of
    int32_t chunk_blocks; //   chunk_blocks blocks, to whichever workgroup asks next
    int32_t g_block_rows; // set entries per pooled block of gather work (fewer than kBlockRows:
                          // a gathered row costs more than a streamed one)
    float sel_margin;     // standard deviations the threshold sample's target rank is raised by
    float scale;          // 1 / sqrt(head_dim)
    float scale_log2e;    // log2(e) / sqrt(head_dim)
};

// Everything about one layer that any unit kind needs.  A table of these lives in device
// memory; a launch names the layer ranges its unit kinds cover.
struct LayerDesc {
    const uint16_t *q, *k_cache, *v_cache;
    const uint16_t *k_new, *v_new;  // bf16 [B][H_kv][128]: the decoded token's rows, appended to the
                                    // caches by an A unit (nullptr: the caller has appended them)
    uint16_t *out;         // bf16 [B][H_q][128]
    uint16_t *q_keep;      // bf16 [B][H_q][128] or nullptr: where T units leave a copy of their group's
                           // queries, for a select that runs after the caller has reused q
    float *sel;            // [B][n_rgroups][sel_stride] pooled selection scores (scaled logits),
                           // written only for a row whose candidate list cannot be used
    float *part_o;         // [B*H_q][part_stride][128] un-normalised partial outputs
    float *part_ml;        // [B*H_q][part_stride][2]   running maximum (raw dot units) and sum
    int32_t *part_count;   // [B*H_q] partial slots in use
    float *part_pool;      // [B*n_rgroups][part_stride][2] running maximum and sum of exp of the
                           // pooled selection logits, per piece (Threshold / Top-p rules only)
    unsigned long long *list;  // [B*n_rgroups][list_row] candidates in no particular order:
                               // ordered key in the low 32 bits, position in the high 32 bits
    int32_t *list_count;   // [B*n_rgroups] candidates found (may exceed list_row: list unusable)
    uint32_t *thr;         // [B*n_rgroups] ordered key a score must reach to be a candidate
    int32_t *idx_out;      // [B][H_kv][k] where this layer's sets are written
    const int32_t *idx_src[kMaxKvHeads];  // per KV head: base of the [B][H_kv][k] array that
                                          // holds the set this layer inherits for that head
    int32_t n_rgroups, n_sgroups;
    int32_t emit_sel;      // R units collect selection candidates
    int32_t copy_keep;     // S also copies the inherited sets of heads that keep theirs
    uint8_t rgroup[kMaxKvHeads];  // KV heads whose group holds a retrieval head
    uint8_t sgroup[kMaxKvHeads];  // KV heads whose group holds a sparse head
    uint8_t rmask[kMaxKvHeads];   // per KV head: bit i = query head g*G+i is a retrieval head
    uint8_t rindex[kMaxKvHeads];  // position of KV head g among the retrieval groups, 0xFF = none
};

// Kernel argument: the layer ranges [first, first + count) of each unit kind.
struct LaunchPlan {
    Common c;
    const LayerDesc *layers;
    int32_t r_first, r_count;    // retrieval streaming
    int32_t g_first, g_count;    // sparse gather
    int32_t c_first, c_count;    // combine
    int32_t a_first, a_count;    // cache append
    int32_t t_first, t_count;    // selection thresholds
    int32_t s_first, s_count;    // select (and set copies)
    int32_t collect;             // some R layer of the launch collects selection candidates
    int32_t selects;             // some S layer of the launch has a retrieval group to select for
    // Per layer of the launch's ranges, by table index: what LayerDesc::n_rgroups / n_sgroups /
    // copy_keep say, here so that every workgroup's prologue reads them from the kernel
    // arguments instead of all of them loading the same table lines
    uint8_t n_rseg[kMaxLayers], n_gseg[kMaxLayers], keeps[kMaxLayers];
};

// Kernel argument of lychee_layer_kernel, the single launch of one layer call.  It carries, side by
// side and with hand-offs inside the launch, everything the layer's output needs and the select
// that the previous layer call left pending:
//   front units   the pending select (and set copies) of `prev`, the selection thresholds of `cur`;
//                 they run first, on the first n_front workgroups, and wait for nothing
//   R pieces      cur's retrieval streaming; a piece polls for its row's threshold when it ends
//   G pieces      cur's sparse gathers; a piece of a KV head in gate_mask polls until the front
//                 unit that writes that head's inherited set has published it
//   combine       the workgroup that writes the last partial of a (sequence, KV head, kind)
//                 segment merges the segment's partials into `out`
// Flags carry the launch's generation, a counter in device memory that the last workgroup to
// finish advances: a flag of an earlier launch, or of an earlier replay of a captured launch,
// never matches.
struct LayerLaunch {
    Common c;
    LayerDesc cur;         // the layer whose rows are streamed and gathered (has_cur)
    LayerDesc prev;        // the layer whose select is pending (has_prev)
    int32_t has_cur, has_prev;
    int32_t n_front;       // workgroups that run front units
    int32_t lead_blocks;   // blocks of 64 rows the device streams while a select runs: how much
                           // later than the streaming the gated gathers can start
    uint64_t gate_mask;    // bit g: KV head g's inherited set is written by this launch's front units
    uint32_t *gen;         // the generation (read at the start, advanced at the end)
    uint32_t *exit_count;  // workgroups that have finished
    unsigned long long *thr_flags;  // [B * n_rgroups] {generation, threshold} of cur's score rows
    uint32_t *set_flags;   // [B * H_kv] generation once the set of (sequence, KV head) is final
    uint32_t *seg_count;   // [B * H_kv * 2] partials written so far of each R / G segment (zero between launches)
    uint32_t *thr_arrived; // [B * n_rgroups] threshold units of a score row that have left their keys (likewise)
};
// 0: no selection anywhere in the launch (the dense baseline); 1: the hybrid build; 2: the one
// that also knows the probability rules
hipError_t launch_layer(const LayerLaunch &plan, int build, hipStream_t stream);

hipError_t launch_units(const LaunchPlan &plan, hipStream_t stream);
hipError_t launch_validate_idx(const int32_t *idx, const int32_t *lengths, int32_t batch,
                               int32_t n_kv_heads, int32_t k, int32_t max_len, int32_t block_shift,
                               unsigned long long *n_bad, hipStream_t stream);
hipError_t launch_probe_read(const void *src, size_t bytes, void *sink, hipStream_t stream);
hipError_t launch_probe_copy(void *dst, const void *src, size_t bytes, hipStream_t stream);

}  // namespace lychee
