// Host-side declarations shared by the translation units of the library: launch plans and
// the launch functions the C ABI layer calls.
#pragma once

#include <atomic>

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "a2ats.h"
#include "common.hpp"

namespace a2ats {

// How a2ats_score_topk runs for a shape, and how it carves its workspace.
struct TopkPlan {
  bool fast;            // sampled threshold + one streaming pass (else: exact route only)
  int NG;               // head groups of 4 per KV head
  int P0;               // sampling workgroups per (sequence, KV head, head group)
  int sample_rows;      // rows each of them scores
  int chunks;           // streaming workgroups per (sequence, KV head, head group)
  int rows_per_chunk;
  int subs;             // survivor segments per wave of the streaming pass (always 1)
  int sub_rows;         // rows of a wave (rows_per_chunk / 8)
  int cap;              // survivor capacity per head in the final kernel's LDS
  int row_cap;          // row entries of one survivor segment in HBM
  size_t off_thr, off_route, off_count, off_cand, bytes;
};

struct AttnPlan {
  int n_far;            // workgroups sharing the sinks and retrieved rows of one head
  int n_win;            // workgroups sharing its window rows
  size_t bytes;
};

TopkPlan make_topk_plan(const a2ats_dims& d, int top_k, int window, int n_sink);
AttnPlan make_attn_plan(const a2ats_dims& d, int top_k, int window, int n_sink);
size_t encode_ws_bytes(const a2ats_dims& d);
hipError_t copy_topk_stats(const a2ats_dims& d, int top_k, int window, int n_sink, const void* ws,
                           uint32_t* cand_counts, hipStream_t stream);

// Raise a kernel's dynamic-LDS limit (needed above 64 KB).  The attribute is sticky, so it is set
// once per kernel and device; `slot` (16 entries, one per device) caches the largest size set.
// (Threads racing on a slot at worst set the same attribute twice.)
typedef std::atomic<size_t> LdsSlot;
template <typename K>
inline hipError_t allow_dynamic_lds(K kernel, size_t bytes, LdsSlot* slot) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) dev = 0;
  if (slot[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
  const hipError_t e =
      hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) slot[dev].store(bytes, std::memory_order_release);
  return e;
}

hipError_t launch_build_lut(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                            const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                            float* lut_scale, hipStream_t stream);
// `pg.table` null: `codes` is the contiguous matrix; else a pool of pages (see CodePages).
hipError_t launch_score_topk(const a2ats_dims& d, const uint8_t* codes, const CodePages& pg, const int32_t* lut,
                             const float* lut_scale, int top_k, int window, int n_sink,
                             const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                             float* topk_score, float* scores_out, void* ws, bool presampled, hipStream_t stream,
                             hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
// Decode prologue (append-time encode + tables) and the threshold sampling of the streaming route in
// one launch; launch_score_topk(..., presampled = true) then skips its sampling launch.  shared: one table
// and one set of thresholds per KV head (d has the real head counts; the score/top-K launches that follow
// take dims with n_q_heads = n_kv_heads).
hipError_t launch_decode_select_prologue(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                         const float* codebook, const float* weights, int mode, uint8_t* codes,
                                         const void* q, int q_dtype, const float* cos_b, const float* sin_b,
                                         float* q_rot, int32_t* lut, float* lut_scale, const int32_t* seq_lens,
                                         int32_t* thr, int P0, int sample_rows, int top_k, int window, int n_sink,
                                         bool shared, hipStream_t stream);
hipError_t launch_sparse_attn(const a2ats_dims& d, const void* q, const float* q_rot, const void* k_cache,
                              const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                              const int32_t* topk_count, int top_k, int window, int n_sink,
                              const float* cos_win, const float* sin_win, const int32_t* seq_lens,
                              void* out, void* ws, bool shared, const int32_t* page_table, int page_shift,
                              hipStream_t stream);
hipError_t launch_build_lut_shared(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                                   const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                                   float* lut_scale, hipStream_t stream);
hipError_t launch_decode_prologue(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                  const float* codebook, const float* weights, int mode, uint8_t* codes,
                                  const void* q, int q_dtype, const float* cos_b, const float* sin_b,
                                  float* q_rot, int32_t* lut, float* lut_scale, hipStream_t stream);
// The paper's geometry: one codebook of 4096 codewords over all 128 dimensions, 16-bit codes.
inline bool single_codebook(const a2ats_dims& d) {
  return d.n_sub == 1 && d.sub_dim == 128 && d.n_centroids == 4096;
}
// The few-key route of the single-codebook encoder decides a key in two steps: kEncodeSlices
// workgroups each find the best codeword of their slice ("sweep": part[key][slice] = {value, code}),
// then the smallest of the slices is picked.  `pick` hands the second step to the table-build
// kernel, which follows the sweep in the fused decode prologue.
constexpr int kEncodeSlices = 16;
constexpr int kFewSingleKeys = 8;   // at most this many keys per (sequence, KV head) take that route
struct FewKeyPick {
  const double* part;   // nullptr: nothing to pick
  uint16_t* codes;
  int n_new, pos0;
};
hipError_t launch_build_lut_single(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                                   const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                                   float* lut_scale, bool shared, FewKeyPick pick, hipStream_t stream);
// The sweep alone (n_new <= kFewSingleKeys); returns where its results are in *part.
hipError_t launch_encode_single_sweep(const a2ats_dims& d, const float* keys, int n_new, const float* codebook,
                                      const float* weights, int mode, bool prepared, void* ws,
                                      const double** part, hipStream_t stream);
hipError_t launch_score_topk_single(const a2ats_dims& d, const void* codes, const int32_t* lut, int top_k,
                                    int window, int n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                                    int32_t* topk_count, float* topk_score, float* scores_out,
                                    hipStream_t stream);
hipError_t launch_encode(const a2ats_dims& d, const float* keys, int n_new, int pos0, const float* codebook,
                         const float* weights, int mode, uint8_t* codes, void* ws, hipStream_t stream);
size_t encode_single_ws_bytes(const a2ats_dims& d);
hipError_t launch_encode_single_prepare(const a2ats_dims& d, const float* codebook, const float* weights, int mode,
                                        void* ws, hipStream_t stream);
hipError_t launch_encode_single(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                const float* codebook, const float* weights, int mode, bool prepared, void* codes,
                                void* ws, hipStream_t stream);

size_t kmeanspp_ws_bytes(const a2ats_dims& d);
hipError_t launch_kmeanspp_seed(const a2ats_dims& d, const float* keys, int n_new, const float* weights, int mode,
                                const double* u, float* codebook_out, int32_t* picks, void* ws, hipStream_t stream);
size_t fit_ws_bytes(const a2ats_dims& d);
hipError_t launch_second_moment(const a2ats_dims& d, const float* q_rot, int64_t n_samples, float* h_out, void* ws,
                                hipStream_t stream);
hipError_t launch_codebook_update(const a2ats_dims& d, const float* keys, int n_new, int pos0, const void* codes,
                                  const float* codebook, float* codebook_out, int32_t* counts_out, void* ws,
                                  hipStream_t stream);

// Copy freshly encoded code rows [B][Hkv][n_new][row_bytes] to tokens pos0 .. pos0 + n_new - 1 of a paged pool.
hipError_t launch_codes_to_pages(const a2ats_dims& d, const uint8_t* rows, int n_new, int pos0, int row_bytes,
                                 uint8_t* pool, const CodePages& pg, hipStream_t stream);

}  // namespace a2ats
