// C ABI of the library: host-side argument validation, workspace planning and launches.
// Everything is checked before the first launch, so every error path is reachable without
// a GPU.
#include <math.h>

#include "common.hpp"
#include "internal.hpp"


// Scratch memory of a2ats_sparse_attn_static: one array per GPU the library runs on, held until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address it yields (one per device) is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[8u << 20];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device), or nullptr.
void* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  g_scratch_ptr[dev].store(p, std::memory_order_release);   // (threads racing here store the same address)
  return p;
}

int check_dims(const a2ats_dims* d) {
  if (!d) return A2ATS_ERR_INVALID_ARG;
  if (d->batch < 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || d->n_sub <= 0 ||
      d->sub_dim <= 0 || d->n_centroids <= 0 || d->ctx_len < 0)
    return A2ATS_ERR_INVALID_ARG;
  if (d->n_q_heads % d->n_kv_heads != 0) return A2ATS_ERR_INVALID_ARG;
  if ((int64_t)d->n_sub * d->sub_dim != d->head_dim) return A2ATS_ERR_INVALID_ARG;
  if (d->ctx_stride < d->ctx_len) return A2ATS_ERR_INVALID_ARG;
  if (d->head_dim != 128) return A2ATS_ERR_UNSUPPORTED;
  if (!a2ats::single_codebook(*d)) {
    if (d->n_centroids != 256) return A2ATS_ERR_UNSUPPORTED;
    if (d->sub_dim != 4 && d->sub_dim != 8) return A2ATS_ERR_UNSUPPORTED;
  }
  if (d->n_q_heads / d->n_kv_heads > 8) return A2ATS_ERR_UNSUPPORTED;
  if (d->ctx_len > (1 << 20)) return A2ATS_ERR_UNSUPPORTED;
  return A2ATS_OK;
}

bool misaligned16(const void* p) { return ((uintptr_t)p & 15u) != 0; }

}  // namespace

extern "C" {

int a2ats_version(void) { return 100; }

const char* a2ats_status_string(int status) {
  switch (status) {
    case A2ATS_OK: return "ok";
    case A2ATS_ERR_INVALID_ARG: return "invalid argument";
    case A2ATS_ERR_UNSUPPORTED: return "unsupported shape";
    case A2ATS_ERR_WORKSPACE: return "workspace too small";
    case A2ATS_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

size_t a2ats_lut_elems(const a2ats_dims* d) {
  if (check_dims(d) != A2ATS_OK) return 0;
  if (a2ats::single_codebook(*d)) return (size_t)d->batch * d->n_q_heads * 4096;
  return a2ats::lut_layout(d->batch, d->n_q_heads, d->n_kv_heads, d->n_sub).total;
}

size_t a2ats_workspace_bytes(const a2ats_dims* d, int op, int32_t top_k, int32_t window) {
  if (check_dims(d) != A2ATS_OK) return (size_t)-1;
  switch (op) {
    case A2ATS_OP_ENCODE:
      return a2ats::single_codebook(*d) ? a2ats::encode_single_ws_bytes(*d) : a2ats::encode_ws_bytes(*d);
    case A2ATS_OP_LUT: return 0;
    case A2ATS_OP_SCORE_TOPK: {
      if (top_k < 0 || window < 0) return (size_t)-1;
      if (a2ats::single_codebook(*d)) return 0;
      // The plan depends on the number of sinks through the candidate count: the figure covers
      // every call with up to 64 sinks.
      size_t need = 0;
      for (int n_sink = 0; n_sink <= 64; ++n_sink) {
        const a2ats::TopkPlan p = a2ats::make_topk_plan(*d, top_k, window, n_sink);
        if (p.fast && p.bytes > need) need = p.bytes;
      }
      return need;
    }
    case A2ATS_OP_ATTN: {
      if (top_k < 0 || window < 0) return (size_t)-1;
      // The number of workgroups per head grows with the attended rows; sized for up to 64 sinks
      // (a call with more sinks than that may ask for more and is refused if `ws` is too small).
      return a2ats::make_attn_plan(*d, top_k, window, 64).bytes;
    }
    case A2ATS_OP_FIT: return a2ats::fit_ws_bytes(*d);
    case A2ATS_OP_SEED: return a2ats::single_codebook(*d) ? a2ats::kmeanspp_ws_bytes(*d) : (size_t)-1;
    default: return (size_t)-1;
  }
}

int a2ats_rope_tables(int32_t head_dim, const double* inv_freq, int32_t b, int32_t window, float* cos_b,
                      float* sin_b, float* cos_win, float* sin_win) {
  if (head_dim <= 0 || (head_dim & 1) || !inv_freq || !cos_b || !sin_b || window < 0)
    return A2ATS_ERR_INVALID_ARG;
  if (window > 0 && (!cos_win || !sin_win)) return A2ATS_ERR_INVALID_ARG;
  const int half = head_dim / 2;
  for (int t = 0; t < half; ++t) {
    const double a = (double)b * inv_freq[t];
    cos_b[t] = (float)cos(a);
    sin_b[t] = (float)sin(a);
  }
  for (int dlt = 0; dlt < window; ++dlt)
    for (int t = 0; t < half; ++t) {
      const double a = (double)dlt * inv_freq[t];
      cos_win[(size_t)dlt * half + t] = (float)cos(a);
      sin_win[(size_t)dlt * half + t] = (float)sin(a);
    }
  return A2ATS_OK;
}

int a2ats_encode_keys(const a2ats_dims* d, const float* keys, int32_t n_new, int32_t pos0,
                      const float* codebook, const float* weights, int weight_mode, uint8_t* codes,
                      void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (n_new < 0 || pos0 < 0 || (int64_t)pos0 + n_new > d->ctx_stride) return A2ATS_ERR_INVALID_ARG;
  const bool prepared = (weight_mode & A2ATS_W_PREPARED) != 0;
  weight_mode &= ~A2ATS_W_PREPARED;
  if (weight_mode != A2ATS_W_NONE && weight_mode != A2ATS_W_DIAG && weight_mode != A2ATS_W_BLOCK)
    return A2ATS_ERR_INVALID_ARG;
  if (!keys || !codebook || !codes) return A2ATS_ERR_INVALID_ARG;
  if (weight_mode != A2ATS_W_NONE && !weights) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(keys) || misaligned16(codebook)) return A2ATS_ERR_INVALID_ARG;
  if (a2ats::single_codebook(*d)) {   // every weighting goes through the transformed codewords
    if (!ws || misaligned16(ws) || ws_bytes < a2ats::encode_single_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
    if ((int64_t)d->batch * d->n_kv_heads * (int64_t)n_new >= (1LL << 31)) return A2ATS_ERR_UNSUPPORTED;
    const hipError_t e = a2ats::launch_encode_single(*d, keys, n_new, pos0, codebook, weights, weight_mode,
                                                     prepared, codes, ws, (hipStream_t)stream);
    return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
  }
  if (weight_mode != A2ATS_W_NONE) {
    if (!ws || misaligned16(ws)) return A2ATS_ERR_WORKSPACE;
    if (ws_bytes < a2ats::encode_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
  }
  if ((int64_t)n_new > 65535LL * 256) return A2ATS_ERR_UNSUPPORTED;
  const hipError_t e = a2ats::launch_encode(*d, keys, n_new, pos0, codebook, weights, weight_mode, codes,
                                            weight_mode != A2ATS_W_NONE ? ws : nullptr, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_encode_prepare(const a2ats_dims* d, const float* codebook, const float* weights, int weight_mode,
                         void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (weight_mode != A2ATS_W_NONE && weight_mode != A2ATS_W_DIAG && weight_mode != A2ATS_W_BLOCK)
    return A2ATS_ERR_INVALID_ARG;
  if (!codebook || misaligned16(codebook)) return A2ATS_ERR_INVALID_ARG;
  if (weight_mode != A2ATS_W_NONE && !weights) return A2ATS_ERR_INVALID_ARG;
  if (!a2ats::single_codebook(*d)) return A2ATS_OK;   // nothing worth keeping between calls
  if (!ws || misaligned16(ws) || ws_bytes < a2ats::encode_single_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
  const hipError_t e = a2ats::launch_encode_single_prepare(*d, codebook, weights, weight_mode, ws, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_kmeanspp_seed(const a2ats_dims* d, const float* keys, int32_t n_new, const float* weights,
                        int weight_mode, const double* u, float* codebook_out, int32_t* picks, void* ws,
                        size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (!a2ats::single_codebook(*d)) return A2ATS_ERR_UNSUPPORTED;
  if (weight_mode != A2ATS_W_NONE && weight_mode != A2ATS_W_DIAG && weight_mode != A2ATS_W_BLOCK)
    return A2ATS_ERR_INVALID_ARG;
  if (n_new < 1 || n_new > d->ctx_stride || d->batch < 1) return A2ATS_ERR_INVALID_ARG;
  if (!keys || !u || !codebook_out || misaligned16(keys)) return A2ATS_ERR_INVALID_ARG;
  if (weight_mode != A2ATS_W_NONE && !weights) return A2ATS_ERR_INVALID_ARG;
  if (!ws || misaligned16(ws) || ws_bytes < a2ats::kmeanspp_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
  const hipError_t e = a2ats::launch_kmeanspp_seed(*d, keys, n_new, weights, weight_mode, u, codebook_out, picks,
                                                   ws, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_second_moment(const a2ats_dims* d, const float* q_rot, int64_t n_samples, float* h_out, void* ws,
                        size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (n_samples < 0 || !h_out || (n_samples > 0 && !q_rot)) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(q_rot)) return A2ATS_ERR_INVALID_ARG;
  if (!ws || misaligned16(ws) || ws_bytes < a2ats::fit_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
  const hipError_t e = a2ats::launch_second_moment(*d, q_rot, n_samples, h_out, ws, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_codebook_update(const a2ats_dims* d, const float* keys, int32_t n_new, int32_t pos0, const uint8_t* codes,
                          const float* codebook, float* codebook_out, int32_t* counts, void* ws, size_t ws_bytes,
                          void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (n_new < 0 || pos0 < 0 || (int64_t)pos0 + n_new > d->ctx_stride) return A2ATS_ERR_INVALID_ARG;
  if (!codebook || !codebook_out || (n_new > 0 && (!keys || !codes))) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(keys)) return A2ATS_ERR_INVALID_ARG;
  if (!ws || misaligned16(ws) || ws_bytes < a2ats::fit_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
  const hipError_t e = a2ats::launch_codebook_update(*d, keys, n_new, pos0, codes, codebook, codebook_out, counts,
                                                     ws, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_build_lut(const a2ats_dims* d, const void* q, int q_dtype, const float* cos_b, const float* sin_b,
                    const float* codebook, float* q_rot, int32_t* lut, float* lut_scale, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (q_dtype != A2ATS_F32 && q_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (!q || !cos_b || !sin_b || !codebook || !q_rot || !lut || !lut_scale) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codebook) || misaligned16(lut)) return A2ATS_ERR_INVALID_ARG;
  const hipError_t e =
      a2ats::single_codebook(*d)
          ? a2ats::launch_build_lut_single(*d, q, q_dtype, cos_b, sin_b, codebook, q_rot, lut, lut_scale, false,
                                           a2ats::FewKeyPick{nullptr, nullptr, 0, 0},
                                           (hipStream_t)stream)
          : a2ats::launch_build_lut(*d, q, q_dtype, cos_b, sin_b, codebook, q_rot, lut, lut_scale,
                                    (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_build_lut_shared(const a2ats_dims* d, const void* q, int q_dtype, const float* cos_b,
                           const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                           float* lut_scale, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (q_dtype != A2ATS_F32 && q_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (!q || !cos_b || !sin_b || !codebook || !q_rot || !lut || !lut_scale) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codebook) || misaligned16(lut)) return A2ATS_ERR_INVALID_ARG;
  const hipError_t e =
      a2ats::single_codebook(*d)
          ? a2ats::launch_build_lut_single(*d, q, q_dtype, cos_b, sin_b, codebook, q_rot, lut, lut_scale, true,
                                           a2ats::FewKeyPick{nullptr, nullptr, 0, 0},
                                           (hipStream_t)stream)
          : a2ats::launch_build_lut_shared(*d, q, q_dtype, cos_b, sin_b, codebook, q_rot, lut, lut_scale,
                                           (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_decode_prologue(const a2ats_dims* d, const float* keys, int32_t n_new, int32_t pos0,
                          const float* codebook, const float* weights, int weight_mode, uint8_t* codes,
                          const void* q, int q_dtype, const float* cos_b, const float* sin_b, float* q_rot,
                          int32_t* lut, float* lut_scale, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (n_new < 0 || pos0 < 0 || (int64_t)pos0 + n_new > d->ctx_stride) return A2ATS_ERR_INVALID_ARG;
  const bool prepared = (weight_mode & A2ATS_W_PREPARED) != 0;
  weight_mode &= ~A2ATS_W_PREPARED;
  if (weight_mode != A2ATS_W_NONE && weight_mode != A2ATS_W_DIAG && weight_mode != A2ATS_W_BLOCK)
    return A2ATS_ERR_INVALID_ARG;
  if (q_dtype != A2ATS_F32 && q_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (!codebook || !q || !cos_b || !sin_b || !q_rot || !lut || !lut_scale) return A2ATS_ERR_INVALID_ARG;
  if (n_new > 0 && (!keys || !codes)) return A2ATS_ERR_INVALID_ARG;
  if (weight_mode != A2ATS_W_NONE && !weights) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codebook) || misaligned16(lut) || (n_new > 0 && misaligned16(keys)))
    return A2ATS_ERR_INVALID_ARG;
  if (n_new > 32) return A2ATS_ERR_UNSUPPORTED;   // prefill-sized batches go through a2ats_encode_keys
  if (a2ats::single_codebook(*d)) {
    // the float64 sweep for the appended keys, then the table build, which also picks their codes
    if (n_new > a2ats::kFewSingleKeys) return A2ATS_ERR_UNSUPPORTED;
    a2ats::FewKeyPick pick{nullptr, (uint16_t*)codes, n_new, pos0};
    if (n_new > 0 && d->batch > 0) {
      if (!ws || misaligned16(ws) || ws_bytes < a2ats::encode_single_ws_bytes(*d)) return A2ATS_ERR_WORKSPACE;
      if (a2ats::launch_encode_single_sweep(*d, keys, n_new, codebook, weights, weight_mode, prepared, ws,
                                            &pick.part, (hipStream_t)stream) != hipSuccess)
        return A2ATS_ERR_HIP;
    }
    const hipError_t e = a2ats::launch_build_lut_single(*d, q, q_dtype, cos_b, sin_b, codebook, q_rot, lut,
                                                        lut_scale, false, pick, (hipStream_t)stream);
    return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
  }
  const hipError_t e = a2ats::launch_decode_prologue(*d, keys, n_new, pos0, codebook, weights, weight_mode,
                                                     codes, q, q_dtype, cos_b, sin_b, q_rot, lut, lut_scale,
                                                     (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_decode_select(const a2ats_dims* d, const float* keys, int32_t n_new, int32_t pos0,
                        const float* codebook, const float* weights, int weight_mode, uint8_t* codes,
                        const void* q, int q_dtype, const float* cos_b, const float* sin_b, float* q_rot,
                        int32_t* lut, float* lut_scale, int32_t top_k, int32_t window, int32_t n_sink,
                        const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count, float* topk_score,
                        void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  // the selection arguments are checked before the prologue is enqueued (nothing may be launched on an error)
  if (top_k < 0 || window < 0 || n_sink < 0) return A2ATS_ERR_INVALID_ARG;
  if (top_k > 4096) return A2ATS_ERR_UNSUPPORTED;
  if (!codes || !lut || !lut_scale || !topk_count || (top_k > 0 && !topk_idx)) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codes)) return A2ATS_ERR_INVALID_ARG;
  const a2ats::TopkPlan plan = a2ats::make_topk_plan(*d, top_k, window, n_sink);
  if (!a2ats::single_codebook(*d) && plan.fast && (!ws || misaligned16(ws) || ws_bytes < plan.bytes))
    return A2ATS_ERR_WORKSPACE;
  // The fused launch has every sampling workgroup build its problem's tables: worth it while those
  // workgroups fit the 256 CUs in one round, a loss when they queue up behind each other.  Its
  // sampling workgroups read candidate rows while others write the appended rows, so it is only
  // taken when no appended row can be a candidate of any sequence (pos0 >= ctx_len - window: the
  // usual append of the current token); otherwise the two calls run one after the other.
  const long n_sample = (long)d->batch * d->n_kv_heads * plan.NG * plan.P0;
  const bool appended_rows_compete = n_new > 0 && (int64_t)pos0 < (int64_t)d->ctx_len - window;
  if (a2ats::single_codebook(*d) || !plan.fast || n_sample > 256 || appended_rows_compete) {   // the two calls, with their own checks
    rc = a2ats_decode_prologue(d, keys, n_new, pos0, codebook, weights, weight_mode, codes, q, q_dtype, cos_b,
                               sin_b, q_rot, lut, lut_scale, ws, ws_bytes, stream);
    if (rc != A2ATS_OK) return rc;
    return a2ats_score_topk(d, codes, lut, lut_scale, top_k, window, n_sink, seq_lens, topk_idx, topk_count,
                            topk_score, nullptr, ws, ws_bytes, stream);
  }
  // the checks of a2ats_decode_prologue and a2ats_score_topk for the streaming route
  if (n_new < 0 || pos0 < 0 || (int64_t)pos0 + n_new > d->ctx_stride) return A2ATS_ERR_INVALID_ARG;
  weight_mode &= ~A2ATS_W_PREPARED;
  if (weight_mode != A2ATS_W_NONE && weight_mode != A2ATS_W_DIAG && weight_mode != A2ATS_W_BLOCK)
    return A2ATS_ERR_INVALID_ARG;
  if (q_dtype != A2ATS_F32 && q_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (!codebook || !q || !cos_b || !sin_b || !q_rot || !lut || !lut_scale || !codes || !topk_idx || !topk_count)
    return A2ATS_ERR_INVALID_ARG;
  if (n_new > 0 && !keys) return A2ATS_ERR_INVALID_ARG;
  if (weight_mode != A2ATS_W_NONE && !weights) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codebook) || misaligned16(lut) || misaligned16(codes) || (n_new > 0 && misaligned16(keys)))
    return A2ATS_ERR_INVALID_ARG;
  if (n_new > 32) return A2ATS_ERR_UNSUPPORTED;
  if (!ws || misaligned16(ws) || ws_bytes < plan.bytes) return A2ATS_ERR_WORKSPACE;
  hipError_t e = a2ats::launch_decode_select_prologue(
      *d, keys, n_new, pos0, codebook, weights, weight_mode, codes, q, q_dtype, cos_b, sin_b, q_rot, lut, lut_scale,
      seq_lens, (int32_t*)((unsigned char*)ws + plan.off_thr), plan.P0, plan.sample_rows, top_k, window, n_sink,
      false, (hipStream_t)stream);
  if (e != hipSuccess) return A2ATS_ERR_HIP;
  e = a2ats::launch_score_topk(*d, codes, a2ats::CodePages{nullptr, 0, 0}, lut, lut_scale, top_k, window, n_sink,
                               seq_lens, topk_idx, topk_count, topk_score, nullptr, ws, true, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_decode_select_shared(const a2ats_dims* d, const float* keys, int32_t n_new, int32_t pos0,
                               const float* codebook, const float* weights, int weight_mode, uint8_t* codes,
                               const void* q, int q_dtype, const float* cos_b, const float* sin_b, float* q_rot,
                               int32_t* lut, float* lut_scale, int32_t top_k, int32_t window, int32_t n_sink,
                               const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                               float* topk_score, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (a2ats::single_codebook(*d)) return A2ATS_ERR_UNSUPPORTED;
  if (top_k < 0 || window < 0 || n_sink < 0) return A2ATS_ERR_INVALID_ARG;
  if (top_k > 4096) return A2ATS_ERR_UNSUPPORTED;
  if (n_new < 0 || pos0 < 0 || (int64_t)pos0 + n_new > d->ctx_stride) return A2ATS_ERR_INVALID_ARG;
  if (n_new > 32) return A2ATS_ERR_UNSUPPORTED;
  const int mode = weight_mode & ~A2ATS_W_PREPARED;
  if (mode != A2ATS_W_NONE && mode != A2ATS_W_DIAG && mode != A2ATS_W_BLOCK) return A2ATS_ERR_INVALID_ARG;
  if (q_dtype != A2ATS_F32 && q_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (!codebook || !q || !cos_b || !sin_b || !q_rot || !lut || !lut_scale || !codes || !topk_count ||
      (top_k > 0 && !topk_idx))
    return A2ATS_ERR_INVALID_ARG;
  if (n_new > 0 && !keys) return A2ATS_ERR_INVALID_ARG;
  if (mode != A2ATS_W_NONE && !weights) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codebook) || misaligned16(lut) || misaligned16(codes) || (n_new > 0 && misaligned16(keys)))
    return A2ATS_ERR_INVALID_ARG;
  a2ats_dims dk = *d;   // the score/top-K side sees one table head per KV head
  dk.n_q_heads = d->n_kv_heads;
  const a2ats::TopkPlan plan = a2ats::make_topk_plan(dk, top_k, window, n_sink);
  if (plan.fast && (!ws || misaligned16(ws) || ws_bytes < plan.bytes)) return A2ATS_ERR_WORKSPACE;
  const long n_sample = (long)d->batch * d->n_kv_heads * plan.P0;
  const bool appended_rows_compete = n_new > 0 && (int64_t)pos0 < (int64_t)d->ctx_len - window;
  hipError_t e;
  if (!plan.fast || n_sample > 256 || appended_rows_compete) {   // the three launches one after the other
    // (at most 32 keys per sequence: the append-time encoder, which needs no workspace)
    if ((e = a2ats::launch_encode(*d, keys, n_new, pos0, codebook, weights, mode, codes, nullptr,
                                  (hipStream_t)stream)) != hipSuccess)
      return A2ATS_ERR_HIP;
    if ((e = a2ats::launch_build_lut_shared(*d, q, q_dtype, cos_b, sin_b, codebook, q_rot, lut, lut_scale,
                                            (hipStream_t)stream)) != hipSuccess)
      return A2ATS_ERR_HIP;
    e = a2ats::launch_score_topk(dk, codes, a2ats::CodePages{nullptr, 0, 0}, lut, lut_scale, top_k, window, n_sink,
                                 seq_lens, topk_idx, topk_count, topk_score, nullptr, ws, false,
                                 (hipStream_t)stream);
    return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
  }
  e = a2ats::launch_decode_select_prologue(*d, keys, n_new, pos0, codebook, weights, mode, codes, q, q_dtype, cos_b,
                                           sin_b, q_rot, lut, lut_scale, seq_lens,
                                           (int32_t*)((unsigned char*)ws + plan.off_thr), plan.P0, plan.sample_rows,
                                           top_k, window, n_sink, true, (hipStream_t)stream);
  if (e != hipSuccess) return A2ATS_ERR_HIP;
  e = a2ats::launch_score_topk(dk, codes, a2ats::CodePages{nullptr, 0, 0}, lut, lut_scale, top_k, window, n_sink,
                               seq_lens, topk_idx, topk_count, topk_score, nullptr, ws, true, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

// page_table null: contiguous codes.  Otherwise a pool of pages of page_size tokens.
static int code_pages(const a2ats_dims* d, const int32_t* page_table, int32_t page_size, a2ats::CodePages* pg) {
  pg->table = nullptr;
  pg->pages_per_seq = 0;
  pg->shift = 0;
  if (!page_table) return A2ATS_OK;
  if (page_size < 16 || (page_size & (page_size - 1))) return A2ATS_ERR_INVALID_ARG;   // a power of two >= 16
  while ((1 << pg->shift) < page_size) ++pg->shift;
  pg->table = page_table;
  pg->pages_per_seq = (int32_t)((d->ctx_stride + page_size - 1) / page_size);
  return A2ATS_OK;
}

static int score_topk_impl(const a2ats_dims* d, const uint8_t* codes, const int32_t* page_table, int32_t page_size,
                           const int32_t* lut, const float* lut_scale,
                           int32_t top_k, int32_t window, int32_t n_sink, const int32_t* seq_lens,
                           int32_t* topk_idx, int32_t* topk_count, float* topk_score, float* scores_out, void* ws,
                           size_t ws_bytes, void* stream, void* ev_start, void* ev_stop) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  a2ats::CodePages pg;
  if ((rc = code_pages(d, page_table, page_size, &pg)) != A2ATS_OK) return rc;
  if (page_table && a2ats::single_codebook(*d)) return A2ATS_ERR_UNSUPPORTED;
  if (top_k < 0 || window < 0 || n_sink < 0) return A2ATS_ERR_INVALID_ARG;
  if (!codes || !lut || !lut_scale || !topk_count) return A2ATS_ERR_INVALID_ARG;
  if (top_k > 0 && !topk_idx) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(codes) || misaligned16(lut)) return A2ATS_ERR_INVALID_ARG;
  if (top_k > 4096) return A2ATS_ERR_UNSUPPORTED;
  if (a2ats::single_codebook(*d)) {
    const hipError_t e = a2ats::launch_score_topk_single(*d, codes, lut, top_k, window, n_sink, seq_lens,
                                                         topk_idx, topk_count, topk_score, scores_out,
                                                         (hipStream_t)stream);
    return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
  }
  const a2ats::TopkPlan plan = a2ats::make_topk_plan(*d, top_k, window, n_sink);
  if (plan.fast) {
    if (!ws || misaligned16(ws) || ws_bytes < plan.bytes) return A2ATS_ERR_WORKSPACE;
  }
  const hipError_t e = a2ats::launch_score_topk(*d, codes, pg, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                                topk_idx, topk_count, topk_score, scores_out, ws, false,
                                                (hipStream_t)stream, (hipEvent_t)ev_start, (hipEvent_t)ev_stop);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_score_topk(const a2ats_dims* d, const uint8_t* codes, const int32_t* lut, const float* lut_scale,
                     int32_t top_k, int32_t window, int32_t n_sink, const int32_t* seq_lens,
                     int32_t* topk_idx, int32_t* topk_count, float* topk_score, float* scores_out, void* ws,
                     size_t ws_bytes, void* stream) {
  return score_topk_impl(d, codes, nullptr, 0, lut, lut_scale, top_k, window, n_sink, seq_lens, topk_idx, topk_count,
                         topk_score, scores_out, ws, ws_bytes, stream, nullptr, nullptr);
}

int a2ats_score_topk_paged(const a2ats_dims* d, const uint8_t* code_pool, const int32_t* page_table,
                           int32_t page_size, const int32_t* lut, const float* lut_scale, int32_t top_k,
                           int32_t window, int32_t n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                           int32_t* topk_count, float* topk_score, float* scores_out, void* ws, size_t ws_bytes,
                           void* stream) {
  if (!page_table) return A2ATS_ERR_INVALID_ARG;
  return score_topk_impl(d, code_pool, page_table, page_size, lut, lut_scale, top_k, window, n_sink, seq_lens,
                         topk_idx, topk_count, topk_score, scores_out, ws, ws_bytes, stream, nullptr, nullptr);
}

int a2ats_codes_to_pages(const a2ats_dims* d, const uint8_t* new_codes, int32_t n_new, int32_t pos0,
                         uint8_t* code_pool, const int32_t* page_table, int32_t page_size, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (!page_table || !code_pool || n_new < 0 || pos0 < 0 || (int64_t)pos0 + n_new > d->ctx_stride)
    return A2ATS_ERR_INVALID_ARG;
  if (n_new > 0 && !new_codes) return A2ATS_ERR_INVALID_ARG;
  a2ats::CodePages pg;
  if ((rc = code_pages(d, page_table, page_size, &pg)) != A2ATS_OK) return rc;
  if (a2ats::single_codebook(*d)) return A2ATS_ERR_UNSUPPORTED;   // (16-bit codes are not paged)
  const int row_bytes = d->n_sub;
  if (misaligned16(new_codes) || misaligned16(code_pool)) return A2ATS_ERR_INVALID_ARG;
  const hipError_t e = a2ats::launch_codes_to_pages(*d, new_codes, n_new, pos0, row_bytes, code_pool, pg,
                                                    (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_score_topk_profiled(const a2ats_dims* d, const uint8_t* codes, const int32_t* lut,
                              const float* lut_scale, int32_t top_k, int32_t window, int32_t n_sink,
                              const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                              float* topk_score, float* scores_out, void* ws, size_t ws_bytes, void* stream,
                              void* ev_start, void* ev_stop) {
  if (!ev_start || !ev_stop) return A2ATS_ERR_INVALID_ARG;
  return score_topk_impl(d, codes, nullptr, 0, lut, lut_scale, top_k, window, n_sink, seq_lens, topk_idx, topk_count,
                         topk_score, scores_out, ws, ws_bytes, stream, ev_start, ev_stop);
}

static int sparse_attn_impl(const a2ats_dims* d, const void* q, const float* q_rot, const void* k_cache,
                            const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                            const int32_t* topk_count, int32_t top_k, int32_t window, int32_t n_sink,
                            const float* cos_win, const float* sin_win, const int32_t* seq_lens, void* out,
                            void* ws, size_t ws_bytes, bool shared, const int32_t* page_table, int page_size,
                            void* stream) {
  int rc = check_dims(d);
  int page_shift = 0;
  if (page_table) {   // a power of two of at least 16 tokens
    if (page_size < 16 || (page_size & (page_size - 1))) return A2ATS_ERR_INVALID_ARG;
    while ((1 << page_shift) < page_size) ++page_shift;
  }
  if (rc != A2ATS_OK) return rc;
  if (kv_dtype != A2ATS_F32 && kv_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (top_k < 0 || window < 0 || n_sink < 0) return A2ATS_ERR_INVALID_ARG;
  if (!q || !q_rot || !k_cache || !v_cache || !topk_count || !out) return A2ATS_ERR_INVALID_ARG;
  if (top_k > 0 && !topk_idx) return A2ATS_ERR_INVALID_ARG;
  if (window > 0 && (!cos_win || !sin_win)) return A2ATS_ERR_INVALID_ARG;
  if (misaligned16(k_cache) || misaligned16(v_cache) || misaligned16(cos_win) || misaligned16(sin_win))
    return A2ATS_ERR_INVALID_ARG;
  const a2ats::AttnPlan plan = a2ats::make_attn_plan(*d, top_k, window, n_sink);
  if (!ws || misaligned16(ws) || ws_bytes < plan.bytes) return A2ATS_ERR_WORKSPACE;
  const hipError_t e = a2ats::launch_sparse_attn(*d, q, q_rot, k_cache, v_cache, kv_dtype, topk_idx,
                                                 topk_count, top_k, window, n_sink, cos_win, sin_win,
                                                 seq_lens, out, ws, shared, page_table, page_shift,
                                                 (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_sparse_attn(const a2ats_dims* d, const void* q, const float* q_rot, const void* k_cache,
                      const void* v_cache, int kv_dtype, const int32_t* topk_idx, const int32_t* topk_count,
                      int32_t top_k, int32_t window, int32_t n_sink, const float* cos_win,
                      const float* sin_win, const int32_t* seq_lens, void* out, void* ws, size_t ws_bytes,
                      void* stream) {
  return sparse_attn_impl(d, q, q_rot, k_cache, v_cache, kv_dtype, topk_idx, topk_count, top_k, window, n_sink,
                          cos_win, sin_win, seq_lens, out, ws, ws_bytes, false, nullptr, 0, stream);
}

int a2ats_sparse_attn_static(const a2ats_dims* d, const void* q, const float* q_rot, const void* k_cache,
                             const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                             const int32_t* topk_count, int32_t top_k, int32_t window, int32_t n_sink,
                             const float* cos_win, const float* sin_win, const int32_t* seq_lens, void* out,
                             void* stream) {
  // the size check comes first, so that a shape beyond the array is refused without touching a GPU
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (top_k < 0 || window < 0 || n_sink < 0) return A2ATS_ERR_INVALID_ARG;
  if (a2ats::make_attn_plan(*d, top_k, window, n_sink).bytes > sizeof(scratch)) return A2ATS_ERR_WORKSPACE;
  void* ws = scratch_on_current_device();
  if (!ws) return A2ATS_ERR_HIP;
  return sparse_attn_impl(d, q, q_rot, k_cache, v_cache, kv_dtype, topk_idx, topk_count, top_k, window, n_sink,
                          cos_win, sin_win, seq_lens, out, ws, sizeof(scratch), false, nullptr, 0, stream);
}

int a2ats_sparse_attn_paged(const a2ats_dims* d, const void* q, const float* q_rot, const void* k_pool,
                            const void* v_pool, int kv_dtype, const int32_t* page_table, int32_t page_size,
                            const int32_t* topk_idx, const int32_t* topk_count, int32_t top_k, int32_t window,
                            int32_t n_sink, const float* cos_win, const float* sin_win, const int32_t* seq_lens,
                            void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!page_table) return A2ATS_ERR_INVALID_ARG;
  return sparse_attn_impl(d, q, q_rot, k_pool, v_pool, kv_dtype, topk_idx, topk_count, top_k, window, n_sink,
                          cos_win, sin_win, seq_lens, out, ws, ws_bytes, false, page_table, page_size, stream);
}

int a2ats_sparse_attn_shared(const a2ats_dims* d, const void* q, const float* q_rot, const void* k_cache,
                             const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                             const int32_t* topk_count, int32_t top_k, int32_t window, int32_t n_sink,
                             const float* cos_win, const float* sin_win, const int32_t* seq_lens, void* out,
                             void* ws, size_t ws_bytes, void* stream) {
  return sparse_attn_impl(d, q, q_rot, k_cache, v_cache, kv_dtype, topk_idx, topk_count, top_k, window, n_sink,
                          cos_win, sin_win, seq_lens, out, ws, ws_bytes, true, nullptr, 0, stream);
}

int a2ats_score_topk_stats(const a2ats_dims* d, int32_t top_k, int32_t window, int32_t n_sink, const void* ws,
                           uint32_t* cand_counts, void* stream) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (top_k < 0 || window < 0 || n_sink < 0 || !cand_counts) return A2ATS_ERR_INVALID_ARG;
  const a2ats::TopkPlan plan = a2ats::make_topk_plan(*d, top_k, window, n_sink);
  if (plan.fast && !ws) return A2ATS_ERR_WORKSPACE;
  const hipError_t e = a2ats::copy_topk_stats(*d, top_k, window, n_sink, ws, cand_counts, (hipStream_t)stream);
  return e == hipSuccess ? A2ATS_OK : A2ATS_ERR_HIP;
}

int a2ats_score_topk_plan(const a2ats_dims* d, int32_t top_k, int32_t window, int32_t n_sink, int32_t* out) {
  int rc = check_dims(d);
  if (rc != A2ATS_OK) return rc;
  if (top_k < 0 || window < 0 || n_sink < 0 || !out) return A2ATS_ERR_INVALID_ARG;
  const a2ats::TopkPlan p = a2ats::make_topk_plan(*d, top_k, window, n_sink);
  const int32_t v[11] = {p.fast ? 1 : 0, p.NG, p.P0, p.sample_rows, p.chunks, p.rows_per_chunk,
                         p.subs, p.sub_rows, p.row_cap, p.cap, (int32_t)(p.bytes / 256)};
  for (int i = 0; i < 11; ++i) out[i] = p.fast || i == 0 ? v[i] : 0;
  return A2ATS_OK;
}

}  // extern "C"
