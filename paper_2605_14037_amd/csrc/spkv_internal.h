// Shared between the host API (spkv_api.hip) and the kernel files (spkv_write.hip,
// spkv_decode.hip, spkv_prefill.hip, spkv_predictor.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/spkv.h"
#include "spkv_layout.h"

constexpr int kSegTokens = 256;       // bulk append: tokens per compaction segment (one per thread)
constexpr int kMaxItemTarget = 32768;

// Device-side view of one cache: plain pointers into the caller's arena.
struct SpkvView {
    int32_t B, Hq, Hkv, G, D, w;
    int32_t n_pairs;        // B * Hkv
    int32_t n_ring_pages;   // ceil(w / 64) pages per (seq, head) ring
    int32_t pt_cap;         // page-table entries per (seq, head)
    int32_t n_pages;        // pages in the long-term pool
    int32_t n_seg_cap;      // bulk-append segments per (seq, head)
    int32_t max_items;      // capacity (work-item slots) of the partial buffers
    float   theta;          // gate threshold on the logit
    int32_t n_sink;         // first positions of every sequence that are always kept (0: none)

    uint16_t* ring;         // [n_pairs][n_ring_pages] pages (K and V interleaved by half)
    float*    ring_logit;   // [n_pairs][w]
    int32_t*  t_pair;       // [n_pairs] tokens appended so far (same for all heads of a seq)
    int32_t*  kept_len;     // [n_pairs] long-term length L
    int32_t*  gate_on;      // [n_pairs] count of appended tokens with gate on
    int32_t*  pool_next;    // [1] next never-used pool page (bump allocator)
    int32_t*  free_top;     // [1] entries on the stack of recycled pages
    int32_t*  free_pages;   // [n_pages] stack of pages given back by released sequences
    int32_t*  err_flag;     // [1] set by kernels on an impossible state
    int32_t*  page_table;   // [n_pairs][pt_cap] logical page -> pool page
    uint16_t* pool;         // [n_pages] pages
    int32_t*  pos_pool;     // [n_pages][64] position of every long-term entry
    float*    logit_pool;   // [n_pages][64] utility logit of every long-term entry
    int32_t*  seg_count;    // [n_pairs][n_seg_cap] bulk scratch: kept per segment, then offsets
    int32_t*  seg_on;       // [n_pairs][n_seg_cap] bulk scratch: gate-on tokens per segment
    int32_t*  bulk_info;    // [n_pairs][8] bulk scratch, see BulkInfo in spkv_write.hip
    float*    part_acc;     // [max_items][G][D] un-normalised partial outputs
    float*    part_ml;      // [max_items][G][2] running max (log2 domain) and sum
    int32_t*  pair_items;   // [n_pairs] fused step: item count of every pair, split -> combine
    int32_t*  pair_ticket;  // [n_pairs] one-launch decode: workgroups of the pair that are done (0 between launches)
    int32_t*  pos_scratch;  // [pt_cap * 64] gather buffer for kept positions
};

// cu_seqlens travels to the append kernels by value in the kernel-argument block.
struct SpkvCu {
    int32_t v[SPKV_MAX_BATCH + 1];
};

hipError_t spkv_launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t spkv_launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// Streaming read of n_runs runs (chunks_per_run chunks of 16 KB each) of a region of
// total_runs runs by n_workgroups one-wave workgroups; sink: n_workgroups KB.
hipError_t spkv_launch_read(const void* src, long long total_runs, int chunks_per_run,
                            long long first_run, long long n_runs, long long stride,
                            int n_workgroups, void* sink, hipStream_t s);
// rows rows of src_width int32 into the first columns of rows of dst_width (>= src_width).
hipError_t spkv_launch_copy_rows(int32_t* dst, const int32_t* src, int rows, int src_width,
                                 int dst_width, hipStream_t s);
hipError_t spkv_launch_append_step(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const SpkvCu& cu, hipStream_t s);
// prefix: null, or where the prefill attention wants the per-token long-term prefix counts.
hipError_t spkv_launch_append_bulk(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const SpkvCu& cu, int n_max, int32_t* prefix,
                                   hipStream_t s);
// Split of every (seq, head) list into work items, chosen by the host per decode call:
// a pair with n half-pages (32 keys each) is cut evenly into min(ceil(n / hp_per_item),
// slots) items; item j of pair p owns partial slot p * slots + j.  In the single-token
// decode kernels mw (1, 2 or 4) items share a workgroup and a slot (see pair_split); the
// multi-token kernels always run with mw = 1.
struct SpkvSplit {
    int32_t hp_per_item;
    int32_t slots;
    int32_t mw;
};

// one_launch: the last workgroup of every pair merges (and, in the step, appends) inside the
// split launch; otherwise a second launch does.
hipError_t spkv_launch_decode(const SpkvView& v, const uint16_t* q, uint16_t* out, float* lse,
                              float sm_scale, SpkvSplit split, bool split_only, bool one_launch,
                              hipEvent_t ev0, hipEvent_t ev1, hipStream_t s);
hipError_t spkv_launch_decode_step(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const uint16_t* q, uint16_t* out, float* lse,
                                   float sm_scale, SpkvSplit split, bool one_launch, hipStream_t s);
// Utility predictor riding in the fused step (Eq. 1): inputs, the fp32 partial sums of the
// hidden layer between the two launches, and the logits it leaves for the caller.
constexpr int kPredictSplit = 4;      // ranges d_model is cut into
struct SpkvPredict {
    const uint16_t* x;      // [B][d_model] hidden states of the new tokens
    const uint16_t* w1;     // [d_hidden][d_model]
    const float* b1;        // [d_hidden] or null
    const uint16_t* w2;     // [Hkv][d_hidden]
    const float* b2;        // [Hkv] or null
    float* part;            // [kPredictSplit][B][d_hidden]
    float* logits;          // [B][Hkv]
    int32_t d_model, d_hidden;
    int32_t n_blocks;       // workgroups of the split launch that belong to the predictor
};
int spkv_predict_blocks(int n_tokens, int d_hidden);
hipError_t spkv_launch_decode_step_predict(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                           const uint16_t* q, uint16_t* out, float* lse,
                                           float sm_scale, SpkvSplit split, SpkvPredict pr,
                                           hipStream_t s);
hipError_t spkv_launch_decode_chunk(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                    const uint16_t* q, uint16_t* out, float* lse, float sm_scale,
                                    SpkvSplit split, const SpkvCu& cu, int col_groups, hipStream_t s);
hipError_t spkv_launch_soft_gated(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                  const float* f, const uint16_t* q, uint16_t* out, float* lse,
                                  float sm_scale, const SpkvCu& cu, int n_max, uint16_t* stage,
                                  float* bias, int shp, hipStream_t s);
int spkv_chunk_resident_items(int head_dim, int col_groups);
// Prefill attention of n <= n_max new tokens per sequence plus their append.  stage:
// n_pairs * shp staging half-pages (shp >= ceil((w + n_max) / 32)); prefix: one int32 per
// (new token, KV head).
// ks > 1: every span's tiles are cut into ks ranges, one workgroup each, and merged by a
// combine launch; part: spkv_prefill_partial_bytes(spans, ks, shape, head_dim) bytes.
hipError_t spkv_launch_prefill(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                               const float* f, const uint16_t* q, uint16_t* out, float* lse,
                               float sm_scale, const SpkvCu& cu, int n_max, uint16_t* stage,
                               int32_t* prefix, int shp, int ks, float* part, hipStream_t s);
// Workgroups (spans of tokens per (sequence, KV head)) of a prefill call, and the bytes of
// split-K partials for them.
struct SpkvPrefillShape {
    int nq, nw, tb;       // column groups of 16 per wave, waves per workgroup, tokens per wave
};
SpkvPrefillShape spkv_prefill_shape(int group, int n_max);   // for chunks of at most n_max tokens
int spkv_prefill_spans(int n_pairs, int group, int n_max);
size_t spkv_prefill_partial_bytes(int spans, int ks, SpkvPrefillShape sh, int head_dim);
// One-wave work items of the split-K kernel the current device holds at once (occupancy x
// compute units); 0 if the runtime cannot tell.
int spkv_split_resident_items(int head_dim);
hipError_t spkv_launch_predictor(const uint16_t* x, const uint16_t* w1, const float* b1,
                                 const uint16_t* w2, const float* b2, float* logits, float* act,
                                 int n_tokens, int d_model, int d_hidden, int n_kv_heads,
                                 hipStream_t s);
hipError_t spkv_launch_release_sequence(const SpkvView& v, int b, hipStream_t s);
// Drops every long-term entry whose stored logit fails the view's threshold (in place).
hipError_t spkv_launch_prune(const SpkvView& v, hipStream_t s);
hipError_t spkv_launch_gather_positions(const SpkvView& v, int pair, hipStream_t s);
