// The paper's own vector-quantisation geometry (section 5.1): ONE codebook of 4096 codewords per
// head over all D = 128 dimensions (M = 1), a 16-bit code per token.  The approximate score of a
// token is then a single table entry, u^_j = q~ . C[s_j] (section 2.2 eq. "attention weights
// approximation", section 4.2 last equation), so the code stream is 2 bytes per token and there
// are at most 4096 distinct scores per head: selection is dominated by exact ties.
//
//   build_lut_single_kernel    q~ = q R_b and the 4096 scores q~ . c per head, float64 inner
//                              products rounded once to float32 and stored as order-preserving
//                              32-bit keys (no fixed-point scale is needed: a score is one entry)
//   select_single_kernel       exact top-K per head: candidates counted per codeword, a weighted
//                              selection over the 4096 codewords, then one ordered pass that emits
//                              the winners in ascending position, equal scores to the lower position
// (the key encoder of this geometry lives in encode_single.hip)
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kCodewords = 4096;
constexpr int kSD = 128;   // head dimension = subspace dimension

// float32 score <-> signed 32-bit key with the same order (so that the integer selection
// machinery of the product-quantised path applies unchanged).
__device__ __forceinline__ int32_t float_to_key(float f) {
  const int32_t b = __float_as_int(f);
  return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_to_float(int32_t k) {
  return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}

// ------------------------------------------------------------------------------------------
// Tables
// ------------------------------------------------------------------------------------------
// float64 sum over aligned groups of 8 lanes, the same value in every lane of the group.
template <int CTRL>
__device__ __forceinline__ double add_dpp_f64(double x) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, 0xf, 0xf, false);
  return x + __hiloint2double(hi, lo);
}
__device__ __forceinline__ double group8_sum_f64(double v) {
  v = add_dpp_f64<0xB1>(v);      // quad_perm [1,0,3,2]
  v = add_dpp_f64<0x4E>(v);      // quad_perm [2,3,0,1]
  return add_dpp_f64<0x141>(v);  // row_half_mirror
}

constexpr int kLutChunk = 256;   // codewords per workgroup

// `shared`: one table per KV head, from the float32 sum of its heads' rotated queries (selection
// shared by the query heads of a KV head); the table array is then laid out for Hq = Hkv.
template <bool QBF16>
__global__ __launch_bounds__(kLutChunk) void build_lut_single_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int Hq, int Hkv, int shared, FewKeyPick pick, int64_t ctx_stride) {
  constexpr int HALF = kSD / 2;
  __shared__ __align__(16) float s_q[8][kSD];   // q~ of the (up to) 8 query heads of this KV head
  __shared__ int32_t s_out[8][kLutChunk];       // the chunk's table entries, written out in one coalesced pass
  const int chunk = blockIdx.x, bkv = blockIdx.y, b = bkv / Hkv, kv = bkv % Hkv;
  const int G = Hq / Hkv, tid = threadIdx.x;
  for (int i = tid; i < G * HALF; i += kLutChunk) {
    const int g = i / HALF, t = i % HALF;
    const size_t base = ((size_t)b * Hq + kv * G + g) * kSD;
    double x1, x2;
    if (QBF16) {
      const uint16_t* qp = (const uint16_t*)q_in;
      x1 = (double)bf16_to_f32(qp[base + t]);
      x2 = (double)bf16_to_f32(qp[base + t + HALF]);
    } else {
      const float* qp = (const float*)q_in;
      x1 = (double)qp[base + t];
      x2 = (double)qp[base + t + HALF];
    }
    const double c = (double)cos_b[t], s = (double)sin_b[t];
    const float o1 = (float)(x1 * c - x2 * s), o2 = (float)(x2 * c + x1 * s);
    s_q[g][t] = o1;
    s_q[g][t + HALF] = o2;
    if (chunk == 0) {
      q_rot[base + t] = o1;
      q_rot[base + t + HALF] = o2;
      if (t == 0 && !shared) lut_scale[(size_t)b * Hq + kv * G + g] = 1.f;
    }
  }
  __syncthreads();
  if (shared) {
    double sum = 0.0;
    if (tid < kSD)
      for (int g = 0; g < G; ++g) sum += (double)s_q[g][tid];
    __syncthreads();
    if (tid < kSD) s_q[0][tid] = (float)sum;
    if (chunk == 0 && tid == 0) lut_scale[(size_t)b * Hkv + kv] = 1.f;
    __syncthreads();
  }
  const int Gt = shared ? 1 : G, Ht = shared ? Hkv : Hq;   // table heads
  // Eight lanes share a codeword: lane part p holds dimensions {32 i + 4 p .. + 3}, i < 4, so that one
  // load instruction of a wave reads eight whole 128-byte lines (a lane reading its own 512-byte row
  // touches 64 lines per instruction and the rows of the waves of a CU evict each other from the
  // vector cache).  A lane row handles 8 consecutive codewords, one per pass; the query (as float64,
  // four heads at a time) stays in registers across the passes.
  const int lane = tid & 63, wave = tid >> 6, p = lane & 7, r = lane >> 3;
  const int cl0 = wave * 64 + r * 8;   // first of this lane row's codewords, within the chunk
  const float* cw0 = codebook + ((size_t)kv * kCodewords + chunk * kLutChunk + cl0) * kSD + 4 * p;
#pragma unroll 1
  for (int g0 = 0; g0 < Gt; g0 += 4) {
    double qd[4][16];
#pragma unroll
    for (int gg = 0; gg < 4; ++gg) {
      const int g = g0 + gg < Gt ? g0 + gg : g0;   // a head past the end repeats the first; its result is dropped
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 f = *(const float4*)&s_q[g][32 * i + 4 * p];
        qd[gg][4 * i] = (double)f.x;
        qd[gg][4 * i + 1] = (double)f.y;
        qd[gg][4 * i + 2] = (double)f.z;
        qd[gg][4 * i + 3] = (double)f.w;
      }
    }
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
      float4 row[4][4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int i = 0; i < 4; ++i) row[jj][i] = *(const float4*)(cw0 + (size_t)(4 * half + jj) * kSD + 32 * i);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const double c0 = (double)row[jj][i].x, c1 = (double)row[jj][i].y, c2 = (double)row[jj][i].z,
                       c3 = (double)row[jj][i].w;
#pragma unroll
          for (int gg = 0; gg < 4; ++gg)
            acc[gg] += qd[gg][4 * i] * c0 + qd[gg][4 * i + 1] * c1 + qd[gg][4 * i + 2] * c2 + qd[gg][4 * i + 3] * c3;
        }
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
          const double tot = group8_sum_f64(acc[gg]);
          if (p == gg && g0 + gg < Gt) s_out[g0 + gg][cl0 + 4 * half + jj] = float_to_key((float)tot);
        }
      }
    }
  }
  __syncthreads();
  for (int g = 0; g < Gt; ++g)
    lut[((size_t)b * Ht + kv * Gt + g) * kCodewords + chunk * kLutChunk + tid] = s_out[g][tid];
  // Fused decode prologue: the launch before this one swept the codewords for the keys appended in
  // this step; the first workgroup of a (sequence, KV head) picks the smallest of the slices for each
  // of its keys (slices hold ascending codes: strict < keeps the lower code on equal values).
  if (pick.part && chunk == 0 && tid < pick.n_new) {
    const double* mine = pick.part + ((size_t)bkv * pick.n_new + tid) * kEncodeSlices * 2;
    double best = mine[0];
    int arg = (int)mine[1];
    for (int sl = 1; sl < kEncodeSlices; ++sl) {
      const double dv = mine[2 * sl];
      if (dv < best) {
        best = dv;
        arg = (int)mine[2 * sl + 1];
      }
    }
    pick.codes[(size_t)bkv * ctx_stride + pick.pos0 + tid] = (uint16_t)arg;
  }
}

hipError_t launch_build_lut_single(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                                   const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                                   float* lut_scale, bool shared, FewKeyPick pick, hipStream_t stream) {
  const dim3 grid(kCodewords / kLutChunk, d.batch * d.n_kv_heads), block(kLutChunk);
  if (grid.y == 0) return hipSuccess;
  if (q_dtype == A2ATS_BF16)
    hipLaunchKernelGGL((build_lut_single_kernel<true>), grid, block, 0, stream, q, cos_b, sin_b, codebook,
                       q_rot, lut, lut_scale, d.n_q_heads, d.n_kv_heads, shared ? 1 : 0, pick, d.ctx_stride);
  else
    hipLaunchKernelGGL((build_lut_single_kernel<false>), grid, block, 0, stream, q, cos_b, sin_b, codebook,
                       q_rot, lut, lut_scale, d.n_q_heads, d.n_kv_heads, shared ? 1 : 0, pick, d.ctx_stride);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Selection
// ------------------------------------------------------------------------------------------
constexpr int kSelThreads = 512;
constexpr int kPerThread = 8;                       // consecutive tokens per thread and round
constexpr int kRound = kSelThreads * kPerThread;    // tokens per round

constexpr int kSpan = 32;                           // rounds a thread keeps in registers
constexpr int kSpanTokens = kSpan * kRound;         // 131072
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSmallSel = 128;                      // a K-th-key bin of at most this many codewords is finished by counting

struct SelLds {
  int32_t table[kCodewords];    // the head's scores as order-preserving keys
  uint32_t count[kCodewords + 1];   // candidate tokens per codeword (+ a spare bin)
  uint32_t hist[kHistBins];
  uint32_t wave_tot[kSpan][kSelWaves];   // packed (above, equal) counts per round and wave
  uint32_t wave_pre[kSpan][kSelWaves];   // ... exclusive over the waves of a round
  uint32_t round_tot[kSpan];
  uint32_t wave_a[kSelWaves];
  uint32_t res[2];
  uint32_t kmin, kmax;
  uint32_t small_n;                 // codewords in the bin of the K-th key after a radix level
  uint32_t small_key[kSmallSel], small_w[kSmallSel];
  uint8_t cls[kCodewords];          // per codeword: 1 = above the K-th key, 2 = equal to it, 0 = below
};

// The codes of tokens [j0, j0 + 8) of a sequence.  Branch-free: a start beyond the row is moved
// back into it (the caller masks such tokens by position), so every load is unconditional and a
// thread's loads are all in flight together.  ALIGNED rows (16-byte aligned, a multiple of 8
// codes long) take one 16-byte load, others eight 2-byte loads.
template <bool ALIGNED>
__device__ __forceinline__ uint4 load_codes8(const uint16_t* __restrict__ seq_codes, int j0, int row_len) {
  if (ALIGNED) return *(const uint4*)(seq_codes + min(j0, row_len - kPerThread));
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) w[i >> 1] |= (uint32_t)seq_codes[min(j0 + i, row_len - 1)] << (16 * (i & 1));
  return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ uint32_t code_of(const uint4& v, int i) {
  const uint32_t w = i < 2 ? v.x : (i < 4 ? v.y : (i < 6 ? v.z : v.w));
  return (w >> (16 * (i & 1))) & (kCodewords - 1);   // the mask keeps a bad code inside the table
}
// Bit i set when token j0 + i is a candidate, i.e. lies in [lo, hi).
__device__ __forceinline__ uint32_t valid_mask8(int j0, int lo, int hi) {
  const int a = min(max(lo - j0, 0), kPerThread), e = min(max(hi - j0, 0), kPerThread);
  return ((1u << e) - 1u) & ~((1u << a) - 1u);
}

// Bit 2i set when bit i of an 8-bit mask is.
__device__ __forceinline__ uint32_t spread8(uint32_t m) {
  m = (m | (m << 4)) & 0x0f0fu;
  m = (m | (m << 2)) & 0x3333u;
  return (m | (m << 1)) & 0x5555u;
}

// One workgroup per head.  A score is one table entry, so the K-th largest score over the
// candidate tokens is a weighted selection over the 4096 codewords: (1) count the candidates per
// codeword (one pass over the 2-byte codes), (2) find the K-th key over the 4096 keys weighted by
// those counts, (3) a pass that emits the winners in ascending position, equal scores going to
// the lower position.  A thread keeps the codes of kSpan rounds of 8 consecutive tokens in
// registers (one span = 131072 tokens per workgroup): all its loads are in flight together, a
// context of one span is read once and serves both passes, and the rounds share one scan of their
// packed (above, equal) counts over the waves instead of one scan and two barriers per round.
template <bool ALIGNED>
__global__ __launch_bounds__(kSelThreads) void select_single_kernel(
    const uint16_t* __restrict__ codes, const int32_t* __restrict__ lut, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ topk_count, float* __restrict__ topk_score,
    int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kSelThreads;
  __shared__ SelLds L;
  const int bh = blockIdx.x, b = bh / Hq, h = bh % Hq, G = Hq / Hkv, kv = h / G, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, wave_u = __builtin_amdgcn_readfirstlane(wave);
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  int32_t* oi = topk_idx + (size_t)bh * top_k;
  float* os = topk_score ? topk_score + (size_t)bh * top_k : nullptr;
  if (tid == 0) topk_count[bh] = sr.kk;
  for (int t = sr.kk + tid; t < top_k; t += NT) {
    oi[t] = -1;
    if (os) os[t] = 0.f;
  }
  if (sr.kk == 0) return;

  const uint16_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride;
  const int row_len = (int)ctx_stride;
  const int lo = sr.sink_end, hi = sr.win_start;
  const int first = lo & ~(kPerThread - 1);   // rounds start on a multiple of 8 tokens
  const int n_span = (hi - first + kSpanTokens - 1) / kSpanTokens;
  const bool take_all = sr.kk >= sr.ncand;

  // Requests in the order their data is needed last-to-first is wrong for in-order returns: the
  // table is asked for first (it is small), the codes after it, so the count pass can start on the
  // first round's codes while the later rounds are still arriving.
  constexpr int kTablePer = kCodewords / NT;
  const int32_t* head_table = lut + (size_t)bh * kCodewords;
  int32_t tv[kTablePer];
#pragma unroll
  for (int i = 0; i < kTablePer; ++i) tv[i] = head_table[i * NT + tid];
  uint4 cv[kSpan];
  if (!take_all || n_span == 1) {
#pragma unroll
    for (int r = 0; r < kSpan; ++r) cv[r] = load_codes8<ALIGNED>(seq_codes, first + r * kRound + tid * kPerThread, row_len);
  }
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int i = 0; i < kTablePer; ++i) {
    L.table[i * NT + tid] = tv[i];
    L.count[i * NT + tid] = 0;
    kmin = min(kmin, score_key(tv[i]));
    kmax = max(kmax, score_key(tv[i]));
  }
  if (tid == 0) {
    L.kmin = 0xffffffffu;
    L.kmax = 0u;
  }
  __syncthreads();

  uint32_t kth = 0, k_rem = (uint32_t)sr.kk;
  if (!take_all) {
    // (1) candidates per codeword
#pragma unroll 1
    for (int sp = 0; sp < n_span; ++sp) {
      const int s0 = first + sp * kSpanTokens;
      if (sp > 0) {
#pragma unroll
        for (int r = 0; r < kSpan; ++r) cv[r] = load_codes8<ALIGNED>(seq_codes, s0 + r * kRound + tid * kPerThread, row_len);
      }
#pragma unroll
      for (int r = 0; r < kSpan; ++r) {
        const int jw = s0 + r * kRound + wave_u * (64 * kPerThread);   // first token of this wave's share
        if (jw >= lo && jw + 64 * kPerThread <= hi) {   // (wave-uniform) every token is a candidate
#pragma unroll
          for (int i = 0; i < kPerThread; ++i) atomicAdd(&L.count[code_of(cv[r], i)], 1u);
        } else {
          const uint32_t vm = valid_mask8(s0 + r * kRound + tid * kPerThread, lo, hi);
#pragma unroll
          for (int i = 0; i < kPerThread; ++i)   // tokens outside the candidate range count in a spare bin
            atomicAdd(&L.count[(vm >> i) & 1u ? code_of(cv[r], i) : (uint32_t)kCodewords], 1u);
        }
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      kmin = min(kmin, __shfl_xor(kmin, off));
      kmax = max(kmax, __shfl_xor(kmax, off));
    }
    if (lane == 0) {
      atomicMin(&L.kmin, kmin);
      atomicMax(&L.kmax, kmax);
    }
    __syncthreads();
    // (2) the K-th largest key over the codewords weighted by those counts.  First a level of
    // 2048 bins LINEAR in the score between the smallest and the largest table entry (the bit
    // pattern of a float spends its leading digits on the exponent: a level on those would put
    // every score of one binade into one bin); the mapping is monotone, so the bin of the K-th
    // key is exact.  That bin usually holds a handful of codewords: they are listed, and every
    // member adds up the candidates above and at its own key -- the member whose range contains
    // k_rem is the K-th key.  A crowded bin (many equal or nearly equal scores), or a table whose
    // range is empty or not finite, is finished by an MSB-first radix select on the keys.
    const uint32_t k_lo = L.kmin;
    const float s_lo = key_to_float(key_score(k_lo)), span = key_to_float(key_score(L.kmax)) - s_lo;
    const bool use_lin = span >= 1e-30f && span < INFINITY;
    const float lin_scale = use_lin ? (float)kHistBins / span : 0.f;
    auto lin_bin = [&](int32_t entry) {
      return (uint32_t)min((int)((key_to_float(entry) - s_lo) * lin_scale), kHistBins - 1);
    };
    uint32_t bin1 = 0;
    bool found = false;
    if (use_lin) {
      // this thread's 8 codewords, read once (the loops below would otherwise wait for LDS per codeword)
      uint32_t w8[kTablePer], b8[kTablePer];
#pragma unroll
      for (int i = 0; i < kTablePer; ++i) {
        w8[i] = L.count[i * NT + tid];
        b8[i] = lin_bin(tv[i]);
      }
      for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
      if (tid == 0) L.small_n = 0;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kTablePer; ++i)
        if (w8[i]) atomicAdd(&L.hist[b8[i]], w8[i]);
      __syncthreads();
      block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, k_rem, L.wave_a, L.res);
      bin1 = L.res[0];
      k_rem -= L.res[1];
#pragma unroll
      for (int i = 0; i < kTablePer; ++i) {
        if (w8[i] && b8[i] == bin1) {
          const uint32_t at = atomicAdd(&L.small_n, 1u);
          if (at < (uint32_t)kSmallSel) {
            L.small_key[at] = score_key(tv[i]);
            L.small_w[at] = w8[i];
          }
        }
      }
      __syncthreads();
      const uint32_t n_small = L.small_n;
      if (n_small <= (uint32_t)kSmallSel) {
        if ((uint32_t)tid < n_small) {
          const uint32_t key = L.small_key[tid];
          uint32_t gt = 0, eq = 0;
          for (uint32_t u = 0; u < n_small; ++u) {
            const uint32_t ku = L.small_key[u], wu = L.small_w[u];
            gt += ku > key ? wu : 0u;
            eq += ku == key ? wu : 0u;
          }
          if (gt < k_rem && k_rem <= gt + eq) {   // every member at the K-th key writes the same two words
            L.res[0] = key;
            L.res[1] = k_rem - gt;
          }
        }
        __syncthreads();
        kth = L.res[0];
        k_rem = L.res[1];
        found = true;
      }
    }
    if (!found) {
      int remaining = 32 - __clz(L.kmax - k_lo);
      uint32_t prefix = 0, mask = 0;
#pragma unroll 1
      while (remaining > 0) {
        const int bits = remaining < 11 ? remaining : 11;
        const int shift = remaining - bits;
        const uint32_t dmask = (1u << bits) - 1u;
        __syncthreads();   // the histogram may still be read
        for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
        __syncthreads();
        for (int e = tid; e < kCodewords; e += NT) {
          const int32_t entry = L.table[e];
          const uint32_t rel = score_key(entry) - k_lo, w = L.count[e];
          if (w && (!use_lin || lin_bin(entry) == bin1) && (rel & mask) == prefix)
            atomicAdd(&L.hist[(rel >> shift) & dmask], w);
        }
        __syncthreads();
        block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, k_rem, L.wave_a, L.res);
        const uint32_t bin = L.res[0], above = L.res[1];
        k_rem -= above;
        prefix |= bin << shift;
        mask |= dmask << shift;
        remaining = shift;
      }
      kth = prefix + k_lo;
    }
  }
  // class of every codeword, one byte each: the emission pass then costs one byte read per token
#pragma unroll
  for (int i = 0; i < kTablePer; ++i) {
    const uint32_t key = score_key(tv[i]);
    L.cls[i * NT + tid] = take_all ? 1 : (key > kth ? 1 : (key == kth ? 2 : 0));
  }
  __syncthreads();

  // (3) ordered emission: keys above the K-th, plus the first k_rem positions that equal it
  uint32_t out_n = 0, eq_seen = 0;
#pragma unroll 1
  for (int sp = 0; sp < n_span; ++sp) {
    const int s0 = first + sp * kSpanTokens;
    if (n_span > 1) {
      __syncthreads();   // the scan arrays of the span before are still being read
#pragma unroll
      for (int r = 0; r < kSpan; ++r) cv[r] = load_codes8<ALIGNED>(seq_codes, s0 + r * kRound + tid * kPerThread, row_len);
    }
    // two bits per token (bit 2i: above the K-th key, bit 2i + 1: equal to it), two rounds per word
    uint32_t cbits[kSpan / 2];
    uint32_t pre[kSpan];   // packed (above, equal) counts of the lanes before this one, per round
#pragma unroll
    for (int i = 0; i < kSpan / 2; ++i) cbits[i] = 0;
#pragma unroll
    for (int r = 0; r < kSpan; ++r) {
      uint32_t c2 = 0;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) c2 |= (uint32_t)L.cls[code_of(cv[r], i)] << (2 * i);
      const int jw = s0 + r * kRound + wave_u * (64 * kPerThread);
      if (!(jw >= lo && jw + 64 * kPerThread <= hi)) {   // (wave-uniform) some tokens are not candidates
        const uint32_t vm = spread8(valid_mask8(s0 + r * kRound + tid * kPerThread, lo, hi));
        c2 &= vm | (vm << 1);
      }
      cbits[r / 2] |= c2 << (16 * (r % 2));
      const uint32_t own = (uint32_t)__popc(c2 & 0x5555u) | ((uint32_t)__popc(c2 & 0xaaaau) << 16);
      const uint32_t v = wave_inclusive_scan(own);
      pre[r] = v - own;
      if (lane == 63) L.wave_tot[r][wave] = v;
    }
    __syncthreads();
    if (tid < kSpan * kSelWaves) {   // exclusive scan over the 16 waves of each round (16-lane groups)
      const int r = tid / kSelWaves, w = tid % kSelWaves;
      const uint32_t own = L.wave_tot[r][w];
      uint32_t v = own;
#pragma unroll
      for (int off = 1; off < kSelWaves; off <<= 1) {
        const uint32_t n = __shfl_up(v, off, kSelWaves);
        if (w >= off) v += n;
      }
      L.wave_pre[r][w] = v - own;
      if (w == kSelWaves - 1) L.round_tot[r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSpan; ++r) {
      const uint32_t c2 = (cbits[r / 2] >> (16 * (r % 2))) & 0xffffu;
      const uint32_t g = c2 & 0x5555u, e = (c2 >> 1) & 0x5555u;   // token i at bit 2i
      const uint32_t tot = L.round_tot[r];
      const uint32_t own_pre = pre[r];
      if (g | e) {
        const int j0 = s0 + r * kRound + tid * kPerThread;
        const uint32_t p = own_pre + L.wave_pre[r][wave];
        // winners of this thread: everything above the K-th, and the equal ones whose rank among
        // the equal ones is below k_rem
        const uint32_t gt_before = p & 0xffffu, eq_before = eq_seen + (p >> 16);
        uint32_t e_take = 0;
        if (e && eq_before < k_rem) {
          const uint32_t room = k_rem - eq_before;   // >= 1
          e_take = e;
          if ((uint32_t)__popc(e) > room) {          // keep the lowest `room` set bits
#pragma unroll 1
            for (uint32_t drop = (uint32_t)__popc(e) - room; drop; --drop) e_take &= ~(0x80000000u >> __clz(e_take));
          }
        }
        uint32_t m = g | e_take;
#pragma unroll 1
        while (m) {
          const int bit = __ffs(m) - 1, i = bit >> 1;
          const uint32_t below = (1u << bit) - 1u;
          const uint32_t slot = out_n + gt_before + (uint32_t)__popc(g & below) + min(eq_before, k_rem) + (uint32_t)__popc(e_take & below);
          oi[slot] = j0 + i;
          if (os) os[slot] = key_to_float(L.table[seq_codes[j0 + i] & (kCodewords - 1)]);
          m &= m - 1;
        }
      }
      out_n += tot & 0xffffu;
      eq_seen += tot >> 16;
    }
    if (out_n + min(eq_seen, k_rem) >= (uint32_t)sr.kk) break;   // uniform over the workgroup
  }
}

// Debug / parity: every token's score as float.
__global__ __launch_bounds__(256) void score_dense_single_kernel(
    const uint16_t* __restrict__ codes, const int32_t* __restrict__ lut, const int32_t* __restrict__ seq_lens,
    float* __restrict__ scores_out, int Hq, int Hkv, int ctx_len, int64_t ctx_stride) {
  const int bh = blockIdx.y, b = bh / Hq, h = bh % Hq, G = Hq / Hkv, kv = h / G;
  int n = seq_lens ? seq_lens[b] : ctx_len;
  n = n < 0 ? 0 : (n > ctx_len ? ctx_len : n);
  const uint16_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride;
  const int32_t* table = lut + (size_t)bh * kCodewords;
  for (int j = blockIdx.x * 256 + threadIdx.x; j < n; j += gridDim.x * 256)
    scores_out[(size_t)bh * ctx_stride + j] = key_to_float(table[seq_codes[j] & (kCodewords - 1)]);
}

hipError_t launch_score_topk_single(const a2ats_dims& d, const void* codes, const int32_t* lut, int top_k,
                                    int window, int n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                                    int32_t* topk_count, float* topk_score, float* scores_out,
                                    hipStream_t stream) {
  const int heads = d.batch * d.n_q_heads;
  if (heads == 0) return hipSuccess;
  if (scores_out) {
    int gx = (d.ctx_len + 256 * 8 - 1) / (256 * 8);
    if (gx < 1) gx = 1;
    hipLaunchKernelGGL(score_dense_single_kernel, dim3(gx, heads), dim3(256), 0, stream,
                       (const uint16_t*)codes, lut, seq_lens, scores_out, d.n_q_heads, d.n_kv_heads,
                       d.ctx_len, d.ctx_stride);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  const bool aligned = (((uintptr_t)codes) & 15u) == 0 && d.ctx_stride % kPerThread == 0 && d.ctx_stride >= kPerThread;
  if (aligned)
    hipLaunchKernelGGL(select_single_kernel<true>, dim3(heads), dim3(kSelThreads), 0, stream,
                       (const uint16_t*)codes, lut, seq_lens, topk_idx, topk_count, topk_score, d.n_q_heads,
                       d.n_kv_heads, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  else
    hipLaunchKernelGGL(select_single_kernel<false>, dim3(heads), dim3(kSelThreads), 0, stream,
                       (const uint16_t*)codes, lut, seq_lens, topk_idx, topk_count, topk_score, d.n_q_heads,
                       d.n_kv_heads, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  return hipGetLastError();
}

}  // namespace a2ats
