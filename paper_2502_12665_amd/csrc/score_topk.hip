// Step 3 of a decode step: approximate scores by gather-summing fixed-point table entries
// through the uint8 codes (section 4.2 last equation), and exact per-head top-K (section 4).
//
// Two routes, chosen on the host from the shape:
//
//  exact route (short contexts, very large K, ragged corner cases; also the in-kernel fallback
//  of the fast route): one workgroup per query head runs an MSB-first radix select over the
//  32-bit score keys by re-streaming its sequence (3 histogram passes), then one ordered pass
//  that emits the winners in ascending position, equal scores going to the lower position.
//
//  fast route (long contexts): the code matrix is streamed from HBM once.
//    1. sample_threshold_kernel scores a strided sample of each sequence (about 1/16 of it) and
//       derives, per head, an integer threshold below the K-th score with a 5-sigma margin
//       (distribution-free: it only uses ranks of the sample).
//    2. stream_select_kernel streams all code rows, one 16-byte table read per code byte
//       serving the four heads of a group, and appends every (position, score) at or above
//       the threshold to a per-head candidate list (about 2K entries) through wave-private
//       LDS staging.
//    3. final_select_kernel (one workgroup per head) radix-selects the exact K-th key among
//       the candidates in LDS, resolves ties by position, and orders the winners by position
//       with an LDS bitmap.  If the candidate list is too short or overflowed -- possible only
//       when the sample misled (probability ~1e-6 per head) or for degenerate inputs -- the
//       workgroup runs the exact route for its head instead, so the result is always exact.
#include <math.h>

#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kExactThreads = 1024;
constexpr int kStreamThreads = 512;
constexpr int kSampleThreads = 512;
constexpr int kStageCap = 64;        // wave-private LDS staging entries per head (>= one ballot)
constexpr int kSubCap = 128;         // candidate slots a wave owns in HBM, per head
constexpr int kStreamWaves = kStreamThreads / 64;
constexpr int kSampleRows = 1024;    // rows scored by one sampling workgroup
constexpr float kSigma = 5.0f;

TopkPlan make_topk_plan(const a2ats_dims& d, int top_k, int window, int n_sink) {
  TopkPlan p{};
  const int G = d.n_q_heads / d.n_kv_heads;
  p.NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  long ncand = (long)d.ctx_len - window - n_sink;
  if (ncand < 0) ncand = 0;
  p.cap = 8192;
  p.fast = ncand >= 16384 && d.ctx_len <= (1 << 18) && top_k >= 1 && top_k <= 2048 &&
           4L * top_k <= ncand;
  if (p.fast) {
    long s_tot = ncand / 16 / kSampleRows * kSampleRows;
    if (s_tot < kSampleRows) s_tot = kSampleRows;
    if (s_tot > 8 * kSampleRows) s_tot = 8 * kSampleRows;
    p.P0 = (int)(s_tot / kSampleRows);
    const long problems = (long)d.batch * d.n_kv_heads * p.NG;
    long chunks = (512 + problems - 1) / problems;
    const long max_chunks = (ncand + 2047) / 2048;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    if (chunks > 64) chunks = 64;
    long rpc = (ncand + chunks - 1) / chunks;
    rpc = (rpc + kStreamThreads - 1) / kStreamThreads * kStreamThreads;
    p.chunks = (int)((ncand + rpc - 1) / rpc);
    p.rows_per_chunk = (int)rpc;
    const size_t heads = (size_t)d.batch * d.n_q_heads;
    p.off_thr = 0;
    // one candidate segment (count + kSubCap slots) per head, chunk and wave of the streaming pass
    const size_t segs = heads * p.chunks * kStreamWaves;
    p.off_count = p.off_thr + heads * p.P0 * sizeof(int32_t);
    p.off_cand = (p.off_count + segs * sizeof(uint32_t) + 255) / 256 * 256;
    p.bytes = p.off_cand + segs * (size_t)kSubCap * sizeof(uint2);
  }
  return p;
}

// ------------------------------------------------------------------------------------------
// Scoring primitives
// ------------------------------------------------------------------------------------------

// Score of one token for one head from an [m][c] single-head table in LDS (random c -> random
// banks; a [c][m] order would put every lane of a read on the same two banks).
template <int M>
__device__ __forceinline__ int32_t score_one_head(const uint8_t* row, const int32_t* lut1) {
  int32_t s = 0;
#pragma unroll
  for (int qd = 0; qd < M / 16; ++qd) {
    const uint4 w = *(const uint4*)(row + qd * 16);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t byte = (ww[i >> 2] >> (8 * (i & 3))) & 0xffu;
      s += lut1[(qd * 16 + i) * kCentroids + byte];
    }
  }
  return s;
}

// Scores of one token for the four heads of a group from the table in LDS, which is held as
// [M/16 halves][256 c][16 m][4 heads] (for M = 16 this is the global [c][m][4] order).
//
// LDS serves a 16-byte read 8 lanes at a time (128 B per clock); lanes whose addresses agree
// modulo 128 B collide.  With the table stored [c][m][4] (256 B per centroid row, subspace m
// at byte 16*m of the row) the bank group of a read is m mod 8, whatever the code byte is.
// Lane L therefore visits the subspaces of its row in the order m = t ^ (L & 15), t = 0..15
// (per 16-byte half row): in every read the 8 lanes served together touch 8 different bank
// groups, so random codes cause no conflicts.  The order does not matter for the result
// because scores are integer sums.
template <int M>
struct LaneSwizzle {
  uint32_t mc[M / 4];   // byte t&3 of mc[t>>2]: (m & 15) << 4 for step t of this lane
  uint32_t sel[4];      // v_perm selectors: address byte 1 <- code byte (k ^ b), byte 0 <- mc byte k
  bool swap1, swap2;    // dword index of the row is XORed with (rho >> 2)
  __device__ __forceinline__ void init(int lane) {
    const uint32_t rho = lane & 15, b = rho & 3;
#pragma unroll
    for (int d = 0; d < M / 4; ++d) {
      uint32_t v = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) v |= ((((uint32_t)(4 * d + k) ^ rho) & 15u) << 4) << (8 * k);
      mc[d] = v;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) sel[k] = 0x0c0c0000u | ((4u + ((uint32_t)k ^ b)) << 8) | (uint32_t)k;
    swap1 = (rho >> 2) & 1;
    swap2 = (rho >> 3) & 1;
  }
};

template <int M>
__device__ __forceinline__ void score_four_heads(const uint4 (&w)[M / 16], const int4* lutv,
                                                 const LaneSwizzle<M>& sw, int32_t (&acc)[4]) {
  acc[0] = acc[1] = acc[2] = acc[3] = 0;
  const unsigned char* base = (const unsigned char*)lutv;
#pragma unroll
  for (int qd = 0; qd < M / 16; ++qd) {
    // z[d] = row dword (d ^ (rho >> 2))
    const uint32_t x0 = sw.swap1 ? w[qd].y : w[qd].x, x1 = sw.swap1 ? w[qd].x : w[qd].y;
    const uint32_t x2 = sw.swap1 ? w[qd].w : w[qd].z, x3 = sw.swap1 ? w[qd].z : w[qd].w;
    const uint32_t z[4] = {sw.swap2 ? x2 : x0, sw.swap2 ? x3 : x1, sw.swap2 ? x0 : x2, sw.swap2 ? x1 : x3};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      // (code byte << 8) | (m << 4): byte offset of entry [c][m] inside this half's 64 KB table
      const uint32_t off = __builtin_amdgcn_perm(z[t >> 2], sw.mc[qd * 4 + (t >> 2)], sw.sel[t & 3]);
      const int4 e = *(const int4*)(base + qd * 65536 + off);
      acc[0] += e.x; acc[1] += e.y; acc[2] += e.z; acc[3] += e.w;
    }
  }
}

// LDS slot of global table entry e = c * M + m.
template <int M>
__device__ __forceinline__ int lds_slot(int e) {
  if (M == 16) return e;
  const int c = e / M, m = e % M;
  return (m >> 4) * (kCentroids * 16) + c * 16 + (m & 15);
}

template <int M, int NT>
__device__ __forceinline__ void load_group_lut(const int32_t* __restrict__ lut_grp, int4* lutv) {
  const int4* src = (const int4*)lut_grp;
#pragma unroll 4
  for (int e = threadIdx.x; e < kCentroids * M; e += NT) lutv[lds_slot<M>(e)] = src[e];
}

// ------------------------------------------------------------------------------------------
// Exact route (also the fallback of the fast route)
// ------------------------------------------------------------------------------------------
struct ExactLds {
  uint32_t hist[kHistBins];
  uint32_t wave_a[kExactThreads / 64];
  uint32_t wave_b[kExactThreads / 64];
  uint32_t res[2];
  int32_t sub_min[32], sub_max[32];
};

// Exact top-K for one head by the whole workgroup.  `lut1` is kCentroids*M words of LDS.
// Writes out_idx[0..kk) ascending (and out_score) ; the caller has written the count and the
// -1 padding.  Requires sr.kk >= 1.
template <int M>
__device__ void exact_select_block(const uint8_t* __restrict__ seq_codes,
                                   const int32_t* __restrict__ lut_grp, int r, float scale,
                                   const SeqRange& sr, int32_t* __restrict__ out_idx,
                                   float* __restrict__ out_score, int32_t* lut1, ExactLds& L) {
  constexpr int NT = kExactThreads;
  const int tid = threadIdx.x;
  for (int e = tid; e < kCentroids * M; e += NT)   // e = c * M + m in the global order
    lut1[(e % M) * kCentroids + e / M] = lut_grp[e * kHeadsPerGroup + r];
  __syncthreads();

  const int lo = sr.sink_end, hi = sr.win_start;
  uint32_t kth = 0, k_rem = (uint32_t)sr.kk;
  if (sr.kk < sr.ncand) {
    // Bounds of any score (sum of per-subspace minima / maxima): radix digits are taken from
    // key - key(lower bound), so that the histogram bins spread over the occupied range
    // instead of all keys sharing their leading bits.
    if (tid < 32) {
      L.sub_min[tid] = INT32_MAX;
      L.sub_max[tid] = INT32_MIN;
    }
    __syncthreads();
    for (int e = tid; e < kCentroids * M; e += NT) {   // e = m * 256 + c: a wave covers one m
      int32_t mn = lut1[e], mx = mn;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        mn = min(mn, __shfl_xor(mn, off));
        mx = max(mx, __shfl_xor(mx, off));
      }
      if ((tid & 63) == 0) {
        atomicMin(&L.sub_min[e / kCentroids], mn);
        atomicMax(&L.sub_max[e / kCentroids], mx);
      }
    }
    __syncthreads();
    int32_t s_lo = 0, s_hi = 0;
    for (int m = 0; m < M; ++m) {
      s_lo += L.sub_min[m];
      s_hi += L.sub_max[m];
    }
    const uint32_t k_lo = score_key(s_lo);
    int remaining = 32 - __clz(score_key(s_hi) - k_lo);   // significant bits of a relative key
    uint32_t prefix = 0, mask = 0;
#pragma unroll 1
    while (remaining > 0) {
      const int bits = remaining < 11 ? remaining : 11;
      const int shift = remaining - bits;
      const uint32_t dmask = (1u << bits) - 1u;
      for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
      __syncthreads();
      for (int j = lo + tid; j < hi; j += NT) {
        const uint32_t key = score_key(score_one_head<M>(seq_codes + (size_t)j * M, lut1)) - k_lo;
        if ((key & mask) == prefix) atomicAdd(&L.hist[(key >> shift) & dmask], 1u);
      }
      __syncthreads();
      block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, k_rem, L.wave_a, L.res);
      const uint32_t bin = L.res[0], above = L.res[1];
      k_rem -= above;
      prefix |= bin << shift;
      mask |= dmask << shift;
      remaining = shift;
      __syncthreads();
    }
    kth = prefix + k_lo;
  } else {
    kth = 0;  // every candidate is taken
    k_rem = (uint32_t)sr.kk;
  }

  // Ordered emission: keys above the K-th, plus the first k_rem positions that equal it.
  uint32_t eq_seen = 0, out_n = 0;
  const bool take_all = sr.kk >= sr.ncand;
#pragma unroll 1
  for (int base = lo; base < hi; base += NT) {
    const int j = base + tid;
    int32_t s = 0;
    uint32_t gt = 0, eq = 0;
    if (j < hi) {
      s = score_one_head<M>(seq_codes + (size_t)j * M, lut1);
      const uint32_t key = score_key(s);
      gt = take_all ? 1u : (key > kth ? 1u : 0u);
      eq = take_all ? 0u : (key == kth ? 1u : 0u);
    }
    uint32_t tot_eq, tot_sel;
    const uint32_t ex_eq = block_exclusive_scan<NT>(eq, L.wave_a, tot_eq);
    const uint32_t sel = gt | ((eq && (eq_seen + ex_eq < k_rem)) ? 1u : 0u);
    const uint32_t ex_sel = block_exclusive_scan<NT>(sel, L.wave_b, tot_sel);
    if (sel) {
      const uint32_t pos = out_n + ex_sel;
      out_idx[pos] = j;
      if (out_score) out_score[pos] = (float)s * scale;
    }
    eq_seen += tot_eq;
    out_n += tot_sel;
    if (out_n >= (uint32_t)sr.kk) break;
  }
}

template <int M>
__global__ __launch_bounds__(kExactThreads) void select_exact_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ topk_count,
    float* __restrict__ topk_score, int Hq, int Hkv, int NG, int ctx_len, int64_t ctx_stride,
    int top_k, int window, int n_sink) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ ExactLds L;
  const int bh = blockIdx.x, b = bh / Hq, h = bh % Hq;
  const int G = Hq / Hkv, kv = h / G, hg = h % G;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  int32_t* oi = topk_idx + (size_t)bh * top_k;
  float* os = topk_score ? topk_score + (size_t)bh * top_k : nullptr;
  if (threadIdx.x == 0) topk_count[bh] = sr.kk;
  for (int t = sr.kk + threadIdx.x; t < top_k; t += kExactThreads) {
    oi[t] = -1;
    if (os) os[t] = 0.f;
  }
  if (sr.kk == 0) return;
  const int32_t* lut_grp =
      lut + (((size_t)b * Hkv + kv) * NG + hg / kHeadsPerGroup) * (kCentroids * M * kHeadsPerGroup);
  exact_select_block<M>(codes + ((size_t)b * Hkv + kv) * ctx_stride * M, lut_grp,
                        hg % kHeadsPerGroup, lut_scale[bh], sr, oi, os, (int32_t*)dyn_lds, L);
}

// ------------------------------------------------------------------------------------------
// Debug: dense scores for every token (not on the fast path; used by parity tests)
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kStreamThreads) void score_dense_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    float* __restrict__ scores_out, int Hq, int Hkv, int NG, int ctx_len, int64_t ctx_stride) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  int4* lutv = (int4*)dyn_lds;
  const int prob = blockIdx.y;  // (b, kv, g4)
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int G = Hq / Hkv;
  load_group_lut<M, kStreamThreads>(lut + (size_t)prob * (kCentroids * M * kHeadsPerGroup), lutv);
  __syncthreads();
  int n = seq_lens ? seq_lens[b] : ctx_len;
  n = n < 0 ? 0 : (n > ctx_len ? ctx_len : n);
  const uint8_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride * M;
  LaneSwizzle<M> sw;
  sw.init(threadIdx.x & 63);
  float sc[4];
  for (int r = 0; r < 4; ++r) {
    const int hg = g4 * kHeadsPerGroup + r;
    sc[r] = hg < G ? lut_scale[(size_t)b * Hq + kv * G + hg] : 0.f;
  }
  for (int j = blockIdx.x * kStreamThreads + threadIdx.x; j < n; j += gridDim.x * kStreamThreads) {
    uint4 w[M / 16];
#pragma unroll
    for (int qd = 0; qd < M / 16; ++qd) w[qd] = *(const uint4*)(seq_codes + (size_t)j * M + qd * 16);
    int32_t acc[4];
    score_four_heads<M>(w, lutv, sw, acc);
    for (int r = 0; r < 4; ++r) {
      const int hg = g4 * kHeadsPerGroup + r;
      if (hg < G) scores_out[((size_t)b * Hq + kv * G + hg) * ctx_stride + j] = (float)acc[r] * sc[r];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Fast route, stage 1: sampled thresholds
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kSampleThreads) void sample_threshold_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ thr, int Hq, int Hkv, int NG,
    int P0, int ctx_len,
    int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kSampleThreads;
  constexpr int NW = NT / 64;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  int4* lutv = (int4*)dyn_lds;
  __shared__ uint32_t s_hist[2][kHistBins];   // two heads per word, 16-bit counts (<= 1024 each)
  __shared__ int32_t s_mm[NW][M][8];
  __shared__ int32_t s_red[M][8];
  __shared__ int32_t s_lo[kHeadsPerGroup];
  __shared__ int32_t s_shift[kHeadsPerGroup];
  __shared__ uint32_t s_wave[NW];
  __shared__ uint32_t s_res[2];

  const int p = blockIdx.x, prob = blockIdx.y;
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int G = Hq / Hkv, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);

  // sampling plan for this sequence
  const int s_p = min(kSampleRows, sr.ncand / P0);
  const long s_all = (long)s_p * P0;
  int r_p = 0;
  bool take_all = sr.ncand <= top_k || s_p == 0;
  if (!take_all) {
    const float r0 = (float)top_k * (float)s_all / (float)sr.ncand;
    const float x = 0.5f * (kSigma + sqrtf(kSigma * kSigma + 4.f * r0));
    r_p = (int)ceilf(x * x / (float)P0) + 1;
    if (r_p > s_p) take_all = true;
  }
  if (take_all) {
    if (tid < kHeadsPerGroup) {
      const int hg = g4 * kHeadsPerGroup + tid;
      if (hg < G) thr[((size_t)b * Hq + kv * G + hg) * P0 + p] = INT32_MIN;
    }
    return;
  }

  // table -> LDS, with per-(subspace, head) min / max of the entries this thread copies
  const int4* src = (const int4*)(lut + (size_t)prob * (kCentroids * M * kHeadsPerGroup));
  int32_t mn[4] = {INT32_MAX, INT32_MAX, INT32_MAX, INT32_MAX};
  int32_t mxv[4] = {INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN};
  for (int e = tid; e < kCentroids * M; e += NT) {   // e % M == tid % M for every e of a thread
    const int4 v = src[e];
    lutv[lds_slot<M>(e)] = v;
    mn[0] = min(mn[0], v.x); mn[1] = min(mn[1], v.y); mn[2] = min(mn[2], v.z); mn[3] = min(mn[3], v.w);
    mxv[0] = max(mxv[0], v.x); mxv[1] = max(mxv[1], v.y); mxv[2] = max(mxv[2], v.z); mxv[3] = max(mxv[3], v.w);
  }
  for (int i = tid; i < 2 * kHistBins; i += NT) (&s_hist[0][0])[i] = 0;
#pragma unroll
  for (int off = M; off < 64; off <<= 1) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      mn[r] = min(mn[r], __shfl_xor(mn[r], off));
      mxv[r] = max(mxv[r], __shfl_xor(mxv[r], off));
    }
  }
  if (lane < M) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      s_mm[wv][lane][r] = mn[r];
      s_mm[wv][lane][4 + r] = mxv[r];
    }
  }
  __syncthreads();
  if (tid < M * 8) {
    const int m = tid / 8, c = tid % 8;
    int32_t v = s_mm[0][m][c];
    for (int w = 1; w < NW; ++w) v = c < 4 ? min(v, s_mm[w][m][c]) : max(v, s_mm[w][m][c]);
    s_red[m][c] = v;
  }
  __syncthreads();
  if (tid < kHeadsPerGroup) {
    int32_t lo = 0, hi = 0;
    for (int m = 0; m < M; ++m) {
      lo += s_red[m][tid];
      hi += s_red[m][4 + tid];
    }
    const uint32_t range = (uint32_t)(hi - lo);
    int sh = 32 - __clz(range) - 11;   // smallest shift with (range >> shift) < 2048
    s_lo[tid] = lo;
    s_shift[tid] = sh < 0 ? 0 : sh;
  }
  __syncthreads();

  // score this workgroup's share of the strided sample
  LaneSwizzle<M> sw;
  sw.init(lane);
  const uint8_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride * M;
  const int lo0 = s_lo[0], lo1 = s_lo[1], lo2 = s_lo[2], lo3 = s_lo[3];
  const int sh0 = s_shift[0], sh1 = s_shift[1], sh2 = s_shift[2], sh3 = s_shift[3];
  for (int i = tid; i < s_p; i += NT) {
    const long g = (long)p * s_p + i;
    const int j = sr.sink_end + (int)((g * sr.ncand) / s_all);
    uint4 w[M / 16];
#pragma unroll
    for (int qd = 0; qd < M / 16; ++qd) w[qd] = *(const uint4*)(seq_codes + (size_t)j * M + qd * 16);
    int32_t acc[4];
    score_four_heads<M>(w, lutv, sw, acc);
    atomicAdd(&s_hist[0][(uint32_t)(acc[0] - lo0) >> sh0], 1u);
    atomicAdd(&s_hist[0][(uint32_t)(acc[1] - lo1) >> sh1], 1u << 16);
    atomicAdd(&s_hist[1][(uint32_t)(acc[2] - lo2) >> sh2], 1u);
    atomicAdd(&s_hist[1][(uint32_t)(acc[3] - lo3) >> sh3], 1u << 16);
  }
  __syncthreads();
#pragma unroll 1
  for (int r = 0; r < kHeadsPerGroup; ++r) {
    block_find_rank_desc<NT, kHistBins>(
        [&](int i) { return (s_hist[r >> 1][i] >> (16 * (r & 1))) & 0xffffu; }, (uint32_t)r_p, s_wave, s_res);
    if (tid == 0) {
      const int hg = g4 * kHeadsPerGroup + r;
      // lower edge of the bin holding the r_p-th largest sample: at least r_p samples are >= it
      if (hg < G)
        thr[((size_t)b * Hq + kv * G + hg) * P0 + p] = s_lo[r] + (int32_t)(s_res[0] << s_shift[r]);
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// Fast route, stage 2: one pass over the code matrix
// ------------------------------------------------------------------------------------------
template <int M>
__device__ __forceinline__ void stream_select_body(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ thr,
    uint32_t* __restrict__ seg_count, uint2* __restrict__ cand, int Hq, int Hkv, int NG, int P0,
    int rows_per_chunk, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kStreamThreads;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  int4* lutv = (int4*)dyn_lds;
  uint2* stage_all = (uint2*)(dyn_lds + (size_t)kCentroids * M * sizeof(int4));

  const int chunk = blockIdx.x, n_chunks = gridDim.x, prob = blockIdx.y;
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int G = Hq / Hkv, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  const long begin = (long)sr.sink_end + (long)chunk * rows_per_chunk;
  const int end = (int)min((long)sr.win_start, begin + rows_per_chunk);

  // Every (head, chunk, wave) owns one candidate segment in HBM: no atomics, no contention.
  size_t seg[4];
  bool live[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int hg = g4 * kHeadsPerGroup + r;
    live[r] = hg < G;
    const size_t head = (size_t)b * Hq + kv * G + (live[r] ? hg : 0);
    seg[r] = (head * n_chunks + chunk) * kStreamWaves + wv;
  }
  if (begin >= sr.win_start) {   // nothing to score: publish empty segments
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (live[r] && lane == 0) seg_count[seg[r]] = 0;
    return;
  }

  load_group_lut<M, NT>(lut + (size_t)prob * (kCentroids * M * kHeadsPerGroup), lutv);

  int32_t T[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int32_t t = INT32_MAX;   // padded heads never produce candidates
    if (live[r]) {
      const size_t head = seg[r] / ((size_t)n_chunks * kStreamWaves);
      t = thr[head * P0];
      for (int pp = 1; pp < P0; ++pp) t = min(t, thr[head * P0 + pp]);
    }
    T[r] = t;
  }
  __syncthreads();

  uint2* stage = stage_all + (size_t)wv * kHeadsPerGroup * kStageCap;
  LaneSwizzle<M> sw;
  sw.init(lane);
  int cnt[4] = {0, 0, 0, 0};   // staged in LDS, per head (wave-uniform)
  int done[4] = {0, 0, 0, 0};  // already copied to this wave's HBM segment

  // Copy the staged entries of head r to the wave's segment.  Entries past the segment capacity
  // are dropped but still counted, which the final kernel recognises as an overflow.
  auto flush = [&](int r) {
    const int n = cnt[r];
    if (n == 0) return;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    for (int i = lane; i < n; i += 64)
      if (done[r] + i < kSubCap) cand[seg[r] * kSubCap + done[r] + i] = stage[r * kStageCap + i];
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    done[r] += n;
    cnt[r] = 0;
  };

  const uint8_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride * M;
  // Rows are read U at a time per thread, one full step ahead of their use (two register sets
  // used alternately), so every wave keeps up to 2*U 16-byte loads in flight while it gathers.
  constexpr int U = 4;
  constexpr int STEP = NT * U;
  uint4 rows_a[U][M / 16], rows_b[U][M / 16];
  // Loads are unconditional (row index clamped into the chunk) so that the wait before the
  // gathers only covers the older of the two row sets in flight.
  auto load_rows = [&](int base, uint4 (&dst)[U][M / 16]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = base + u * NT + tid;
      const int jl = j < end ? j : end - 1;
#pragma unroll
      for (int qd = 0; qd < M / 16; ++qd)
        dst[u][qd] = load_stream_u4(seq_codes + (size_t)jl * M + qd * 16);
    }
  };
  auto process = [&](int base, const uint4 (&rows)[U][M / 16]) {
    // Scores and the per-head "at or above threshold" wave masks are formed together, so the
    // gathered table entries die inside this straight-line block.
    int32_t acc[U][4];
    uint64_t hit[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      score_four_heads<M>(rows[u], lutv, sw, acc[u]);
      const bool valid = base + u * NT + tid < end;
#pragma unroll
      for (int r = 0; r < 4; ++r) hit[u][r] = __ballot(valid && acc[u][r] >= T[r]);
      __builtin_amdgcn_sched_barrier(0);   // one row's gathers at a time: bounds live registers
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = base + u * NT + tid;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint64_t mask = hit[u][r];
        if (mask) {
          const int n = __popcll(mask);
          if (cnt[r] + n > kStageCap) flush(r);
          if ((mask >> lane) & 1)
            stage[r * kStageCap + cnt[r] + lanes_below(mask)] = make_uint2((uint32_t)j, (uint32_t)acc[u][r]);
          cnt[r] += n;
        }
      }
    }
  };
  load_rows((int)begin, rows_a);
#pragma unroll 1
  for (int base = (int)begin; base < end; base += 2 * STEP) {
    load_rows(base + STEP, rows_b);
    process(base, rows_a);
    load_rows(base + 2 * STEP, rows_a);
    process(base + STEP, rows_b);
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    flush(r);
    if (live[r] && lane == 0) seg_count[seg[r]] = (uint32_t)done[r];
  }
}

#define A2ATS_STREAM_ARGS                                                                          \
  const uint8_t *__restrict__ codes, const int32_t *__restrict__ lut,                             \
      const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ thr,                      \
      uint32_t *__restrict__ seg_count, uint2 *__restrict__ cand, int Hq, int Hkv, int NG, int P0, \
      int rows_per_chunk, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink
#define A2ATS_STREAM_PASS                                                                          \
  codes, lut, seq_lens, thr, seg_count, cand, Hq, Hkv, NG, P0, rows_per_chunk, ctx_len,            \
      ctx_stride, top_k, window, n_sink

// M = 16: 80 KB of LDS per workgroup, two workgroups per CU -> 4 waves per SIMD, 128 VGPRs.
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_select_kernel16(A2ATS_STREAM_ARGS) { stream_select_body<16>(A2ATS_STREAM_PASS); }
// M = 32: 144 KB of LDS, one workgroup per CU -> 2 waves per SIMD.
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void stream_select_kernel32(A2ATS_STREAM_ARGS) { stream_select_body<32>(A2ATS_STREAM_PASS); }


// ------------------------------------------------------------------------------------------
// Fast route, stage 3: exact selection among the candidates, ordered output
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kExactThreads) void final_select_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    const uint32_t* __restrict__ seg_count, const uint2* __restrict__ cand,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ topk_count,
    float* __restrict__ topk_score, int Hq, int Hkv, int NG, int n_seg, int cap, int ctx_len,
    int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kExactThreads;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ ExactLds L;
  const int bh = blockIdx.x, b = bh / Hq, h = bh % Hq;
  const int G = Hq / Hkv, kv = h / G, hg = h % G, tid = threadIdx.x;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  int32_t* oi = topk_idx + (size_t)bh * top_k;
  float* os = topk_score ? topk_score + (size_t)bh * top_k : nullptr;
  if (tid == 0) topk_count[bh] = sr.kk;
  for (int t = sr.kk + tid; t < top_k; t += NT) {
    oi[t] = -1;
    if (os) os[t] = 0.f;
  }
  if (sr.kk == 0) return;
  const float scale = lut_scale[bh];
  // Candidate segments of this head (one per chunk and wave of the streaming pass): exclusive
  // prefix of their sizes.  n_seg <= 512 <= NT.
  __shared__ uint32_t s_seg_off[513];
  __shared__ uint32_t s_overflow;
  if (tid == 0) s_overflow = 0;
  __syncthreads();
  uint32_t my_cnt = 0;
  if (tid < n_seg) {
    my_cnt = seg_count[(size_t)bh * n_seg + tid];
    if (my_cnt > (uint32_t)kSubCap) s_overflow = 1;
  }
  uint32_t n_c;
  const uint32_t my_off = block_exclusive_scan<NT>(my_cnt, L.wave_a, n_c);
  if (tid < n_seg) s_seg_off[tid] = my_off;
  if (tid == 0) s_seg_off[n_seg] = n_c;
  __syncthreads();
  if (s_overflow || n_c > (uint32_t)cap || n_c < (uint32_t)sr.kk) {
    const int32_t* lut_grp = lut + (((size_t)b * Hkv + kv) * NG + hg / kHeadsPerGroup) *
                                       (kCentroids * M * kHeadsPerGroup);
    exact_select_block<M>(codes + ((size_t)b * Hkv + kv) * ctx_stride * M, lut_grp,
                          hg % kHeadsPerGroup, scale, sr, oi, os, (int32_t*)dyn_lds, L);
    return;
  }

  // LDS carve-up: candidate positions and keys, position bitmap, per-word prefix counts
  const int n_words = (ctx_len + 31) / 32;
  uint32_t* c_idx = (uint32_t*)dyn_lds;
  uint32_t* c_key = c_idx + cap;
  uint32_t* bitmap = c_key + cap;
  uint16_t* wpre = (uint16_t*)(bitmap + n_words);
  constexpr uint32_t kDropped = 0x80000000u;

  // Candidate keys are stored relative to the smallest one, so that the radix digits spread
  // over the occupied range (all candidates share the leading bits of their absolute keys).
  uint32_t kmin = 0xffffffffu, kmax = 0;
  for (uint32_t i = tid; i < n_c; i += NT) {
    int lo_s = 0, hi_s = n_seg;   // segment holding flat candidate i: last s with off[s] <= i
    while (hi_s - lo_s > 1) {
      const int mid = (lo_s + hi_s) >> 1;
      if (s_seg_off[mid] <= i) lo_s = mid; else hi_s = mid;
    }
    const uint2 e = cand[((size_t)bh * n_seg + lo_s) * kSubCap + (i - s_seg_off[lo_s])];
    const uint32_t key = score_key((int32_t)e.y);
    c_idx[i] = e.x;
    c_key[i] = key;
    kmin = min(kmin, key);
    kmax = max(kmax, key);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    kmin = min(kmin, __shfl_xor(kmin, off));
    kmax = max(kmax, __shfl_xor(kmax, off));
  }
  if ((tid & 63) == 0) {
    L.wave_a[tid >> 6] = kmin;
    L.wave_b[tid >> 6] = kmax;
  }
  __syncthreads();
  kmin = L.wave_a[0];
  kmax = L.wave_b[0];
  for (int w = 1; w < NT / 64; ++w) {
    kmin = min(kmin, L.wave_a[w]);
    kmax = max(kmax, L.wave_b[w]);
  }
  __syncthreads();
  for (uint32_t i = tid; i < n_c; i += NT) c_key[i] -= kmin;
  // K-th largest key among the candidates: MSB-first radix select over the significant bits
  uint32_t prefix = 0, mask = 0, k_rem = (uint32_t)sr.kk, n_eq = n_c;
  int remaining = 32 - __clz(kmax - kmin);
#pragma unroll 1
  while (remaining > 0) {
    const int bits = remaining < 11 ? remaining : 11;
    const int shift = remaining - bits;
    const uint32_t dmask = (1u << bits) - 1u;
    for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n_c; i += NT) {
      const uint32_t key = c_key[i];
      if ((key & mask) == prefix) atomicAdd(&L.hist[(key >> shift) & dmask], 1u);
    }
    __syncthreads();
    block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, k_rem, L.wave_a, L.res);
    const uint32_t bin = L.res[0], above = L.res[1];
    n_eq = L.hist[bin];
    k_rem -= above;
    prefix |= bin << shift;
    mask |= dmask << shift;
    remaining = shift;
    __syncthreads();
  }
  const uint32_t kth = prefix;   // relative to kmin, like c_key[]

  // Rank of a position among the set bits of the bitmap: prefix popcounts per 32-bit word.
  const int wpt = (n_words + NT - 1) / NT;
  auto build_word_prefix = [&](uint32_t* s_wave) {
    uint32_t loc = 0;
    for (int i = 0; i < wpt; ++i) {
      const int w = tid * wpt + i;
      if (w < n_words) loc += __popc(bitmap[w]);
    }
    uint32_t tot;
    uint32_t run = block_exclusive_scan<NT>(loc, s_wave, tot);
    for (int i = 0; i < wpt; ++i) {
      const int w = tid * wpt + i;
      if (w < n_words) {
        wpre[w] = (uint16_t)run;
        run += __popc(bitmap[w]);
      }
    }
    __syncthreads();
  };
  auto rank_of = [&](uint32_t pos) -> uint32_t {
    return (uint32_t)wpre[pos >> 5] + __popc(bitmap[pos >> 5] & ((1u << (pos & 31)) - 1u));
  };

  if (n_eq > k_rem) {   // more candidates tie with the K-th key than fit: lowest positions win
    for (int w = tid; w < n_words; w += NT) bitmap[w] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n_c; i += NT)
      if (c_key[i] == kth) atomicOr(&bitmap[c_idx[i] >> 5], 1u << (c_idx[i] & 31));
    __syncthreads();
    build_word_prefix(L.wave_a);
    for (uint32_t i = tid; i < n_c; i += NT)
      if (c_key[i] == kth && rank_of(c_idx[i]) >= k_rem) c_idx[i] |= kDropped;
    __syncthreads();
  }
  for (int w = tid; w < n_words; w += NT) bitmap[w] = 0;
  __syncthreads();
  for (uint32_t i = tid; i < n_c; i += NT)
    if (c_key[i] >= kth && !(c_idx[i] & kDropped)) atomicOr(&bitmap[c_idx[i] >> 5], 1u << (c_idx[i] & 31));
  __syncthreads();
  build_word_prefix(L.wave_b);
  for (uint32_t i = tid; i < n_c; i += NT) {
    if (c_key[i] >= kth && !(c_idx[i] & kDropped)) {
      const uint32_t pos = rank_of(c_idx[i]);
      oi[pos] = (int32_t)c_idx[i];
      if (os) os[pos] = (float)key_score(c_key[i] + kmin) * scale;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
static hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

void set_profile_events(void* a, void* b) {
  g_ev_start = (hipEvent_t)a;
  g_ev_stop = (hipEvent_t)b;
}

__global__ void sum_segments_kernel(const uint32_t* __restrict__ seg_count, uint32_t* __restrict__ out,
                                    int heads, int n_seg) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= heads) return;
  uint32_t tot = 0;
  for (int s = 0; s < n_seg; ++s) tot += seg_count[(size_t)h * n_seg + s];
  out[h] = tot;
}

hipError_t copy_topk_stats(const a2ats_dims& d, int top_k, int window, int n_sink, const void* ws,
                           uint32_t* cand_counts, hipStream_t stream) {
  const TopkPlan plan = make_topk_plan(d, top_k, window, n_sink);
  const int heads = d.batch * d.n_q_heads;
  if (heads == 0) return hipSuccess;
  if (!plan.fast) return hipMemsetAsync(cand_counts, 0xff, (size_t)heads * sizeof(uint32_t), stream);
  hipLaunchKernelGGL(sum_segments_kernel, dim3((heads + 255) / 256), dim3(256), 0, stream,
                     (const uint32_t*)((const unsigned char*)ws + plan.off_count), cand_counts, heads,
                     plan.chunks * kStreamWaves);
  return hipGetLastError();
}

// Raise a kernel's dynamic-LDS limit (needed above 64 KB).  The attribute is sticky, so it is set
// once per kernel and device; `slot` is a per-call-site cache of the largest size set so far.
template <typename K>
static hipError_t allow_lds(K kernel, size_t bytes, size_t* slot) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) dev = 0;
  if (slot[dev] >= bytes) return hipSuccess;
  const hipError_t e =
      hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) slot[dev] = bytes;
  return e;
}

template <int M>
static hipError_t launch_score_topk_m(const a2ats_dims& d, const TopkPlan& plan, const uint8_t* codes,
                                      const int32_t* lut, const float* lut_scale, int top_k, int window,
                                      int n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                                      int32_t* topk_count, float* topk_score, float* scores_out,
                                      void* ws, hipStream_t stream) {
  const int Hq = d.n_q_heads, Hkv = d.n_kv_heads, NG = plan.NG;
  const int heads = d.batch * Hq, problems = d.batch * Hkv * NG;
  const size_t lut4_bytes = (size_t)kCentroids * M * sizeof(int4);
  const size_t lut1_bytes = (size_t)kCentroids * M * sizeof(int32_t);
  hipError_t err;
  static size_t s_dense[16], s_exact[16], s_sample[16], s_stream[16], s_final[16];
  if (heads == 0) return hipSuccess;

  if (scores_out) {
    if ((err = allow_lds(score_dense_kernel<M>, lut4_bytes, s_dense)) != hipSuccess) return err;
    int gx = (d.ctx_len + kStreamThreads * 8 - 1) / (kStreamThreads * 8);
    gx = gx < 1 ? 1 : gx;
    hipLaunchKernelGGL((score_dense_kernel<M>), dim3(gx, problems), dim3(kStreamThreads), lut4_bytes,
                       stream, codes, lut, lut_scale, seq_lens, scores_out, Hq, Hkv, NG, d.ctx_len,
                       d.ctx_stride);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }

  if (!plan.fast) {
    if ((err = allow_lds(select_exact_kernel<M>, lut1_bytes, s_exact)) != hipSuccess) return err;
    hipLaunchKernelGGL((select_exact_kernel<M>), dim3(heads), dim3(kExactThreads), lut1_bytes, stream,
                       codes, lut, lut_scale, seq_lens, topk_idx, topk_count, topk_score, Hq, Hkv, NG,
                       d.ctx_len, d.ctx_stride, top_k, window, n_sink);
    return hipGetLastError();
  }

  unsigned char* wsb = (unsigned char*)ws;
  int32_t* thr = (int32_t*)(wsb + plan.off_thr);
  uint32_t* seg_count = (uint32_t*)(wsb + plan.off_count);
  uint2* cand = (uint2*)(wsb + plan.off_cand);

  if ((err = allow_lds(sample_threshold_kernel<M>, lut4_bytes, s_sample)) != hipSuccess) return err;
  hipLaunchKernelGGL((sample_threshold_kernel<M>), dim3(plan.P0, problems), dim3(kSampleThreads),
                     lut4_bytes, stream, codes, lut, seq_lens, thr, Hq, Hkv, NG, plan.P0,
                     d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  if ((err = hipGetLastError()) != hipSuccess) return err;

  const size_t stream_lds =
      lut4_bytes + (size_t)(kStreamThreads / 64) * kHeadsPerGroup * kStageCap * sizeof(uint2);
  auto stream_kernel = M == 16 ? stream_select_kernel16 : stream_select_kernel32;
  if ((err = allow_lds(stream_kernel, stream_lds, s_stream)) != hipSuccess) return err;
  if (g_ev_start && g_ev_stop) (void)hipEventRecord(g_ev_start, stream);
  hipLaunchKernelGGL(stream_kernel, dim3(plan.chunks, problems), dim3(kStreamThreads),
                     stream_lds, stream, codes, lut, seq_lens, thr, seg_count, cand, Hq, Hkv, NG,
                     plan.P0, plan.rows_per_chunk, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  if (g_ev_start && g_ev_stop) (void)hipEventRecord(g_ev_stop, stream);
  if ((err = hipGetLastError()) != hipSuccess) return err;

  const int n_words = (d.ctx_len + 31) / 32;
  size_t final_lds = (size_t)plan.cap * 8 + (size_t)n_words * 4 + (size_t)n_words * 2;
  if (final_lds < lut1_bytes) final_lds = lut1_bytes;
  final_lds = (final_lds + 15) / 16 * 16;
  if ((err = allow_lds(final_select_kernel<M>, final_lds, s_final)) != hipSuccess) return err;
  hipLaunchKernelGGL((final_select_kernel<M>), dim3(heads), dim3(kExactThreads), final_lds, stream,
                     codes, lut, lut_scale, seq_lens, seg_count, cand, topk_idx, topk_count,
                     topk_score, Hq, Hkv, NG, plan.chunks * kStreamWaves, plan.cap, d.ctx_len,
                     d.ctx_stride, top_k, window, n_sink);
  return hipGetLastError();
}

hipError_t launch_score_topk(const a2ats_dims& d, const uint8_t* codes, const int32_t* lut,
                             const float* lut_scale, int top_k, int window, int n_sink,
                             const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                             float* topk_score, float* scores_out, void* ws, hipStream_t stream) {
  const TopkPlan plan = make_topk_plan(d, top_k, window, n_sink);
  if (d.n_sub == 16)
    return launch_score_topk_m<16>(d, plan, codes, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                   topk_idx, topk_count, topk_score, scores_out, ws, stream);
  return launch_score_topk_m<32>(d, plan, codes, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                 topk_idx, topk_count, topk_score, scores_out, ws, stream);
}

}  // namespace a2ats
