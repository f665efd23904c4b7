// Coarse scoring of code rows against a group's 16-bit table in LDS, and the sampled thresholds of
// the streaming route of a2ats_score_topk (shared by the sampling kernel of score_topk.hip and the
// fused decode launch of build_lut.hip).
#pragma once
#include "common.hpp"

namespace a2ats {

constexpr float kSigma = 5.0f;   // margin of the sampled rank, in standard deviations

// Coarse scores of one token for the four heads of a group.  The coarse table sits in LDS with
// one 256-byte row per centroid id c: the 8-byte entry (two 32-bit words, each holding two heads'
// 16-bit values) of subspace m is at byte (c << 8) | ((m >> 4) << 7) | ((m & 15) << 3); for
// M = 16 the upper half of each row holds a second copy of the lower half.
//
// The LDS of this part has 64 four-byte banks (a 256-byte row spans all of them once) and serves
// an 8-byte read 32 lanes at a time; lanes collide when they touch the same banks.  With this
// layout the banks of a read depend only on the column, not on the (random) code byte.  Lane L
// visits the subspaces of a 16-byte half row in the order m = t ^ (L & 15), t = 0..15, and lanes
// 16..31 of each half-wave are on the other half of the row from lanes 0..15 (the second copy for
// M = 16; the two half rows in the other order for M = 32): the 32 lanes served together always
// touch 32 different entries, so random codes cause no conflicts.  (Measured per 64-lane read,
// two 8-wave workgroups per CU: 3.2 clocks; 4.8 with the columns of one half only; 62 with every
// lane on the same column.)  The visiting order does not change the result because the scores are
// integer sums.  One v_perm_b32 assembles the whole LDS address of a read from the code byte and a
// per-lane constant.
constexpr int kCoarseLdsBytes = kCentroids * 256;

// Byte offset of the coarse entry of (centroid c, subspace m) in the LDS table.
__device__ __forceinline__ uint32_t coarse_lds_offset(int c, int m) {
  return ((uint32_t)c << 8) | (((uint32_t)m >> 4) << 7) | (((uint32_t)m & 15u) << 3);
}
// Put one entry (or two neighbouring ones, V = int4) there, with its second copy when M = 16.
template <int M, typename V>
__device__ __forceinline__ void store_coarse_lds(unsigned char* tbl, int c, int m, const V& entry) {
  *(V*)(tbl + coarse_lds_offset(c, m)) = entry;
  if (M == 16) *(V*)(tbl + coarse_lds_offset(c, m) + 128) = entry;
}

template <int M>
struct LaneSwizzle {
  uint32_t mc[M / 4];   // byte t&3 of mc[t>>2]: low address byte for step t of this lane
  uint32_t sel[4];      // v_perm selectors: address byte 1 <- code byte (k ^ b), byte 0 <- mc byte k
  bool swap1, swap2;    // dword index of the row is XORed with (rho >> 2)
  // M = 32: lanes 16..31 of a half-wave take the two 16-byte halves of a code row in the other
  // order.  A caller loads  w[qd] = 16 bytes at row + ((16 * qd) ^ row_swz)  (0 or 16).
  uint32_t row_swz;
  __device__ __forceinline__ void init(int lane) {
    const uint32_t rho = lane & 15, b = rho & 3, hi = (lane >> 4) & 1;
#pragma unroll
    for (int d = 0; d < M / 4; ++d) {
      uint32_t v = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t t = 4 * d + k;                       // step within the whole row
        const uint32_t m_low = (t ^ rho) & 15u, half = M == 16 ? hi : ((t >> 4) ^ hi);
        v |= ((half << 7) | (m_low << 3)) << (8 * k);
      }
      mc[d] = v;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) sel[k] = 0x0c0c0000u | ((4u + ((uint32_t)k ^ b)) << 8) | (uint32_t)k;
    swap1 = (rho >> 2) & 1;
    swap2 = (rho >> 3) & 1;
    row_swz = (M == 32 && hi) ? 16u : 0u;
  }
};

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const u32x2_t* lds_u2_ptr;

// kBaseZero: the table starts at LDS address 0 (kernel without static LDS), so the v_perm result
// is the address itself; otherwise it is an offset from `tbl`.  `w` holds the lane's code row as
// loaded under LaneSwizzle::row_swz.
template <int M, bool kBaseZero>
__device__ __forceinline__ void score_coarse(const uint4 (&w)[M / 16], const unsigned char* tbl,
                                             const LaneSwizzle<M>& sw, uint32_t& a01, uint32_t& a23) {
  a01 = 0;
  a23 = 0;
#pragma unroll
  for (int qd = 0; qd < M / 16; ++qd) {
    // z[d] = row dword (d ^ (rho >> 2))
    const uint4 wq = w[qd];
    const uint32_t x0 = sw.swap1 ? wq.y : wq.x, x1 = sw.swap1 ? wq.x : wq.y;
    const uint32_t x2 = sw.swap1 ? wq.w : wq.z, x3 = sw.swap1 ? wq.z : wq.w;
    const uint32_t z[4] = {sw.swap2 ? x2 : x0, sw.swap2 ? x3 : x1, sw.swap2 ? x0 : x2, sw.swap2 ? x1 : x3};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const uint32_t off = __builtin_amdgcn_perm(z[t >> 2], sw.mc[qd * 4 + (t >> 2)], sw.sel[t & 3]);
      u32x2_t e;
      if (kBaseZero) e = *(lds_u2_ptr)(uintptr_t)off;
      else e = *(const u32x2_t*)(tbl + off);
      a01 += e.x;
      a23 += e.y;
    }
  }
}

// Copy a problem's coarse table from its global order [half][c][16 m] to the LDS layout above.
template <int M, int NT>
__device__ __forceinline__ void load_coarse_table(const int32_t* __restrict__ lut, const LutLayout& lay,
                                                  int prob, unsigned char* tbl) {
  const int4* src = (const int4*)(lut + lay.off_coarse + (size_t)prob * (kCentroids * M * 2));
#pragma unroll 4
  for (int e = threadIdx.x; e < kCentroids * M / 2; e += NT) {   // e: pair of entries (2 * e, 2 * e + 1)
    const int half = e / (kCentroids * 8), c = (e / 8) % kCentroids, mp = e % 8;
    store_coarse_lds<M>(tbl, c, 16 * half + 2 * mp, src[e]);
  }
}

// One sampling workgroup: part p of the P0 parts of problem `prob` (a sequence, KV head and group
// of four query heads).  `tbl`: kCoarseLdsBytes of LDS for the group's coarse table; TABLE_IN_LDS:
// the caller has put the table there already (and synchronised), otherwise it is copied from `lut`.
template <int M, int NT, bool TABLE_IN_LDS>
__device__ __forceinline__ void sample_threshold_body(
    int prob, int p, const uint8_t* __restrict__ codes, const CodePages& pg, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ thr, int B, int Hq, int Hkv, int NG,
    int P0, int sample_rows, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink,
    unsigned char* tbl) {
  __shared__ uint32_t s_hist[2][kHistBins];   // two heads per word, 16-bit counts (a workgroup scores at most 8192 rows)

  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int G = Hq / Hkv, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);

  // sampling plan for this sequence
  const int s_p = min(sample_rows, sr.ncand / P0);
  const long s_all = (long)s_p * P0;
  int r_p = 0;
  bool take_all = sr.ncand <= top_k || s_p == 0;
  if (!take_all) {
    // rank r in the merged sample with r - sigma * sqrt(r) >= K * S / N, shared out over the P0 parts
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

  const int n_real = min(kHeadsPerGroup, G - g4 * kHeadsPerGroup);   // heads of this group that exist
  const LutLayout lay = lut_layout(B, Hq, Hkv, M);
  if (!TABLE_IN_LDS) load_coarse_table<M, NT>(lut, lay, prob, tbl);
  for (int i = tid; i < 2 * kHistBins; i += NT) (&s_hist[0][0])[i] = 0;
  __syncthreads();

  // Score this workgroup's share of the strided sample.  A coarse score is below 2^16, so
  // score >> 5 indexes a 2048-bin histogram directly.
  LaneSwizzle<M> sw;
  sw.init(lane);
  const SeqCodes seq_codes = seq_codes_of<M>(codes, pg, b, kv, Hkv, ctx_stride);
  // The sample is taken in runs of kRun consecutive rows (one 128-byte line of the code matrix),
  // the runs evenly spread over the candidates: HBM delivers whole lines, so a row-strided sample
  // would fetch eight times the bytes it uses.  (For rows drawn independently, as in the synthetic
  // workloads, this changes nothing statistically; if neighbouring tokens' scores are correlated
  // the estimate is noisier, which costs at most a detour over the exact route.)
  // (run * ncand / n_runs in 32-bit pieces: with ncand = qn * n_runs + rn it is run * qn + run * rn /
  // n_runs, and run * rn < n_runs^2 <= 2^29; a 64-bit division is ~150 instructions per row)
  constexpr int kRun = 128 / M;
  const uint32_t n_runs = (uint32_t)((s_all + kRun - 1) / kRun);
  const uint32_t qn = (uint32_t)sr.ncand / n_runs, rn = (uint32_t)sr.ncand - qn * n_runs;
  // Two rows per thread and round, both requested before either is scored (the rows are cold; four at a
  // time measured the same).
  constexpr int kPair = 2;
#pragma unroll 1
  for (int i0 = tid; i0 < s_p; i0 += kPair * NT) {
    uint4 w[kPair][M / 16];
#pragma unroll
    for (int u = 0; u < kPair; ++u) {
      const int i = min(i0 + u * NT, s_p - 1);   // (a slot past the end repeats the last row and is not counted)
      const uint32_t g = (uint32_t)p * (uint32_t)s_p + (uint32_t)i;
      const uint32_t run = g / kRun;
      int j = sr.sink_end + (int)(run * qn + (run * rn) / n_runs);
      j = max(sr.sink_end, j & ~(kRun - 1)) + (int)(g % kRun);
      j = min(j, sr.win_start - 1);
      const uint8_t* row = row_ptr<M>(seq_codes, j);
#pragma unroll
      for (int qd = 0; qd < M / 16; ++qd) w[u][qd] = *(const uint4*)(row + ((uint32_t)(qd * 16) ^ sw.row_swz));
    }
#pragma unroll
    for (int u = 0; u < kPair; ++u) {
      if (i0 + u * NT >= s_p) continue;
      uint32_t a01, a23;
      score_coarse<M, false>(w[u], tbl, sw, a01, a23);
      // (a head slot past the group's last head has an all-zero table: every row would land in the same
      // bin, a thousand atomics on one address for a histogram nobody reads)
      atomicAdd(&s_hist[0][(a01 & 0xffffu) >> 5], 1u);
      if (n_real > 1) atomicAdd(&s_hist[0][a01 >> 21], 1u << 16);
      if (n_real > 2) atomicAdd(&s_hist[1][(a23 & 0xffffu) >> 5], 1u);
      if (n_real > 3) atomicAdd(&s_hist[1][a23 >> 21], 1u << 16);
    }
  }
  __syncthreads();
  // Rank search, one wave per head: lane l owns bins [32 l, 32 l + 32); a suffix scan over the
  // lanes finds the one whose range holds the r_p-th largest sample; the wave then searches that range.
  if (wv < kHeadsPerGroup) {
    const int r = wv;
    const int hg = g4 * kHeadsPerGroup + r;
    const uint32_t* hrow = s_hist[r >> 1];
    const int fsh = 16 * (r & 1);
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const int ii = (i + lane) & 31;   // rotate the walk so the lanes of a read hit different banks
      sum += (hrow[32 * lane + ii] >> fsh) & 0xffffu;
    }
    // inclusive suffix sum over lanes (higher lanes hold higher bins) = total - exclusive prefix
    const uint32_t pre = wave_inclusive_scan(sum);
    const uint32_t inc = (uint32_t)__builtin_amdgcn_readlane((int)pre, 63) - pre + sum;
    const uint32_t k = (uint32_t)r_p, above_lane = inc - sum;
    const uint64_t owner = __ballot(above_lane < k && k <= inc);   // the lane whose 32 bins hold the rank
    if (owner != 0 && hg < G) {
      // Second level, by the whole wave: lane i < 32 takes bin 31 - i of the owner's range (so
      // bins descend with the lane index) and a prefix sum finds the first lane that reaches k.
      const int src = __ffsll((unsigned long long)owner) - 1;
      const uint32_t above = (uint32_t)__builtin_amdgcn_readlane((int)above_lane, src);
      const uint32_t c = lane < 32 ? (hrow[32 * src + 31 - lane] >> fsh) & 0xffffu : 0u;
      const uint32_t incl = wave_inclusive_scan(c);   // lanes >= 32 hold zeros
      const uint64_t reach = __ballot(lane < 32 && above + incl >= k);
      const int bin = 32 * src + 31 - (__ffsll((unsigned long long)reach) - 1);
      // Lower edge of the bin holding the r_p-th largest sample (at least r_p samples reach it),
      // lowered by M: a row's coarse score is below its exact score by less than M coarse units,
      // and the final kernel needs that much slack to prove its result complete.
      if (lane == 0) thr[((size_t)b * Hq + kv * G + hg) * P0 + p] = max(0, (bin << 5) - M);
    }
  }
}


}  // namespace a2ats
