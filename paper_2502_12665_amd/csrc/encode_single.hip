// Key encoder for the paper's own geometry (section 5.1: one codebook of 4096 codewords over all
// D = 128 dimensions; section 4.2: query-aware assignment with the full D x D matrix H):
//     code = argmin_c (k - c) H (k - c)^T ,  lowest c on exact ties.
//
// With the Cholesky factor of section 4.2 (H = L L^T, z = k L, c^z = c L) the distortion is the
// plain squared distance ||z - c^z||^2, and minimising it over c is minimising
//     s_c = 1/2 ||c^z||^2 - z . c^z ,
// a dense [keys x 128] . [128 x 4096] contraction: 1 Mflop per key, the one matrix-core shape of
// this library.  The kernels:
//
//   encode_single_factor_kernel    per KV head: L in float64 (Cholesky in LDS, or the identity /
//                                  a diagonal for the unweighted / per-dimension modes)
//   encode_single_codewords_kernel c^z = c L in float64; kept transposed in float64 for the exact
//                                  re-check, and split into two bf16 terms (hi + lo, 16 significant
//                                  bits) laid out in matrix-core operand order, with 1/2 ||c^z||^2
//   encode_single_kernel           512 keys per workgroup: z = k L on the matrix cores, split the
//                                  same way, kept in registers as the B operands; the codewords
//                                  stream through LDS 32 at a time as the A operand; three bf16
//                                  products per term (hi.hi + hi.lo + lo.hi, float32 accumulate)
//                                  give the scores to about 2^-18 relative.  Every lane owns one
//                                  key column of the 32 x 32 result tile, so the running smallest
//                                  three scores (and the codes of the first two) are per-lane
//                                  registers; nothing crosses lanes until the end.
//   encode_single_recheck_kernel   keys whose two smallest scores are closer than the rounding reach
//                                  of the bf16 products are decided in float64 between those two
//                                  codewords; keys with three that close (and the few-key append
//                                  path) by a float64 sweep over all 4096.  So the emitted code is
//                                  the float64 argmin.
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {
namespace {

constexpr int kCW = 4096;               // codewords per KV head
constexpr int kD = 128;                 // head dimension
constexpr int kEncWaves = 8;
constexpr int kEncThreads = 64 * kEncWaves;
constexpr int kKeysPerWave = 64;        // two 32-key column tiles
constexpr int kKeysPerWG = kKeysPerWave * kEncWaves;
constexpr int kFragBytes = 2 * 8 * 64 * 16;   // (hi, lo) x 8 k-steps x 64 lanes x 16 bytes: 32 rows of 128 dims
constexpr int kBlocks = kCW / 32;       // streamed 32-codeword blocks
constexpr int kFewSingle = 8;           // at most this many keys per (sequence, KV head): float64 sweep only
constexpr float kReach = 1.5e-5f;       // rounding reach of a score, relative to (|z| + |k| |L|_F) max|c^z|

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct EncWs {
  size_t off_L, off_sd, off_czT, off_cfrag, off_cbias, off_cstat, off_Lfrag, off_count, off_list, bytes;
};

EncWs enc_single_ws(const a2ats_dims& d) {
  const size_t Hkv = (size_t)d.n_kv_heads;
  const size_t keys_max = (size_t)d.batch * Hkv * (size_t)d.ctx_stride;
  EncWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    const size_t at = o;
    o += (bytes + 255) & ~(size_t)255;
    return at;
  };
  w.off_L = take(Hkv * kD * kD * sizeof(double));
  w.off_sd = take(Hkv * kD * sizeof(double));
  w.off_czT = take(Hkv * kD * kCW * sizeof(double));
  w.off_cfrag = take(Hkv * kBlocks * (size_t)kFragBytes);
  w.off_cbias = take(Hkv * kCW * sizeof(float));
  w.off_cstat = take(Hkv * 4 * sizeof(float));
  w.off_Lfrag = take(Hkv * 4 * (size_t)kFragBytes);
  w.off_count = take(sizeof(uint32_t));
  w.off_list = take(keys_max * 2 * sizeof(uint32_t));
  w.bytes = o;
  return w;
}

// Position of dimension t inside a 16-dimension k-step of an operand fragment: lane half g holds
// dims {4g .. 4g+3} and {8+4g .. 8+4g+3}.  This is the order in which the transform's result tile
// leaves the matrix core (row 8(v/4) + 4g + v%4 in register v), so z needs no shuffling to become
// an operand; the codewords are stored in the same order.
__device__ __forceinline__ void frag_slot(int t, int& kt, int& g, int& i) {
  kt = t >> 4;
  const int u = t & 15;
  g = (u >> 2) & 1;
  i = ((u >> 3) << 2) | (u & 3);
}

// ------------------------------------------------------------------------------------------
// Per KV head: the factor L (H = L L^T), its Frobenius norm, and L^T as bf16 hi/lo A operands.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_single_factor_kernel(
    const float* __restrict__ weights, int mode, double* __restrict__ Lmat, double* __restrict__ sd,
    uint16_t* __restrict__ Lfrag, float* __restrict__ cstat, uint32_t* __restrict__ counter) {
  extern __shared__ double s_A[];   // 128 x 128, lower triangle in use
  __shared__ double s_red[256];
  const int kv = blockIdx.x, tid = threadIdx.x;
  if (kv == 0 && tid == 0) *counter = 0;
  double* L = Lmat + (size_t)kv * kD * kD;
  if (mode != A2ATS_W_BLOCK) {
    if (tid < kD) sd[(size_t)kv * kD + tid] = mode == A2ATS_W_DIAG ? sqrt((double)weights[(size_t)kv * kD + tid]) : 1.0;
    if (tid == 0) {
      cstat[kv * 4 + 0] = 0.f;
      cstat[kv * 4 + 1] = 0.f;
    }
    return;
  }
  const float* H = weights + (size_t)kv * kD * kD;
  for (int e = tid; e < kD * kD; e += 256) s_A[e] = (e % kD) <= (e / kD) ? (double)H[e] : 0.0;
  __syncthreads();
  const int ty = tid >> 4, tx = tid & 15;
  for (int j = 0; j < kD; ++j) {   // right-looking: scale column j, then update the trailing triangle
    if (tid == 0) {
      const double s = s_A[j * kD + j];
      s_A[j * kD + j] = sqrt(s > 0.0 ? s : 0.0);
    }
    __syncthreads();
    const double dj = s_A[j * kD + j];
    for (int i = j + 1 + tid; i < kD; i += 256) s_A[i * kD + j] = dj > 0.0 ? s_A[i * kD + j] / dj : 0.0;
    __syncthreads();
    for (int i = j + 1 + ty; i < kD; i += 16) {
      const double lij = s_A[i * kD + j];
      for (int k = j + 1 + tx; k <= i; k += 16) s_A[i * kD + k] -= lij * s_A[k * kD + j];
    }
    __syncthreads();
  }
  double f2 = 0.0;
  for (int e = tid; e < kD * kD; e += 256) {
    const double v = s_A[e];
    L[e] = v;
    f2 += v * v;
  }
  s_red[tid] = f2;
  __syncthreads();
  for (int s = 128; s >= 1; s >>= 1) {
    if (tid < s) s_red[tid] += s_red[tid + s];
    __syncthreads();
  }
  if (tid == 0) {
    cstat[kv * 4 + 0] = 0.f;
    cstat[kv * 4 + 1] = __double2float_ru(sqrt(s_red[0]));
  }
  // A operand of the transform D[t'][key] = sum_r L[r][t'] k[r]: row t' = 32 rt + lane % 32,
  // k-step kt, lane half g, element i <-> r = 16 kt + 8 g + i (the keys are loaded in that order).
  uint16_t* frag = Lfrag + (size_t)kv * 4 * (kFragBytes / 2);
  for (int e = tid; e < 4 * 8 * 64 * 8; e += 256) {
    const int i = e & 7, l = (e >> 3) & 63, kt = (e >> 9) & 7, rt = e >> 12;
    const int tp = 32 * rt + (l & 31), r = 16 * kt + 8 * (l >> 5) + i;
    const double v = s_A[r * kD + tp];   // zero above the diagonal (r < t')
    const uint16_t hi = f32_to_bf16((float)v);
    const uint16_t lo = f32_to_bf16((float)(v - (double)bf16_to_f32(hi)));
    frag[(size_t)rt * (kFragBytes / 2) + ((0 * 8 + kt) * 64 + l) * 8 + i] = hi;
    frag[(size_t)rt * (kFragBytes / 2) + ((1 * 8 + kt) * 64 + l) * 8 + i] = lo;
  }
}

// ------------------------------------------------------------------------------------------
// c^z = c L for 64 codewords per workgroup (float64), in the three forms the other kernels read.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_single_codewords_kernel(
    const float* __restrict__ codebook, int mode, const double* __restrict__ Lmat, const double* __restrict__ sd,
    double* __restrict__ czT, uint16_t* __restrict__ cfrag, float* __restrict__ cbias, float* __restrict__ cstat) {
  __shared__ float s_c[64][kD + 1];
  __shared__ double s_n[4][64];
  const int kv = blockIdx.y, c0 = blockIdx.x * 64, tid = threadIdx.x;
  const int c = tid & 63, tq = __builtin_amdgcn_readfirstlane(tid >> 6);
  const float* cw = codebook + ((size_t)kv * kCW + c0) * kD;
  for (int e = tid; e < 64 * kD; e += 256) s_c[e / kD][e % kD] = cw[e];
  __syncthreads();
  double acc[32];
  if (mode == A2ATS_W_BLOCK) {
#pragma unroll
    for (int u = 0; u < 32; ++u) acc[u] = 0.0;
    const double* L = Lmat + (size_t)kv * kD * kD + 32 * tq;
    for (int r = 32 * tq; r < kD; ++r) {   // L[r][t] = 0 for r < t
      const double cv = (double)s_c[c][r];
#pragma unroll
      for (int u = 0; u < 32; ++u) acc[u] += cv * L[(size_t)r * kD + u];
    }
  } else {
#pragma unroll
    for (int u = 0; u < 32; ++u) acc[u] = (double)s_c[c][32 * tq + u] * sd[(size_t)kv * kD + 32 * tq + u];
  }
  double n2 = 0.0;
#pragma unroll
  for (int u = 0; u < 32; ++u) n2 += acc[u] * acc[u];
  s_n[tq][c] = n2;
  const int cg = c0 + c, cb = cg >> 5, row = cg & 31;
  uint16_t* blk = cfrag + ((size_t)kv * kBlocks + cb) * (kFragBytes / 2);
#pragma unroll
  for (int u = 0; u < 32; ++u) {
    const int t = 32 * tq + u;
    czT[((size_t)kv * kD + t) * kCW + cg] = acc[u];
    int kt, g, i;
    frag_slot(t, kt, g, i);
    const uint16_t hi = f32_to_bf16((float)acc[u]);
    const uint16_t lo = f32_to_bf16((float)(acc[u] - (double)bf16_to_f32(hi)));
    blk[((0 * 8 + kt) * 64 + row + 32 * g) * 8 + i] = hi;
    blk[((1 * 8 + kt) * 64 + row + 32 * g) * 8 + i] = lo;
  }
  __syncthreads();
  if (tq == 0) {
    const double n = s_n[0][c] + s_n[1][c] + s_n[2][c] + s_n[3][c];
    cbias[(size_t)kv * kCW + cg] = (float)(0.5 * n);
    // max over the codewords of |c^z|, rounded up (a non-negative float orders like its bits)
    atomicMax((uint32_t*)&cstat[kv * 4 + 0], __float_as_uint(__double2float_ru(sqrt(n))));
  }
}

// ------------------------------------------------------------------------------------------
// Main pass
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void split8(const float (&z)[8], bf16x8& hi, bf16x8& lo, float& n2) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16 h = (__bf16)z[i];
    const float rest = z[i] - (float)h;
    const __bf16 l = (__bf16)rest;
    hi[i] = h;
    lo[i] = l;
    const float kept = (float)h + (float)l;
    n2 += kept * kept;
  }
}

// Insert score s (code `c`, wave-uniform) into the running smallest three s1 <= s2 <= s3 of a lane.
__device__ __forceinline__ void top3_insert(float s, int c, float& s1, float& s2, float& s3, int& c1, int& c2) {
  s3 = __builtin_amdgcn_fmed3f(s2, s3, s);
  c2 = s < s2 ? c : c2;
  c2 = s < s1 ? c1 : c2;
  s2 = __builtin_amdgcn_fmed3f(s1, s2, s);
  c1 = s < s1 ? c : c1;
  s1 = fminf(s1, s);
}

template <int MODE>
__global__ __launch_bounds__(kEncThreads) void encode_single_kernel(
    const float* __restrict__ keys, const double* __restrict__ sd, const uint8_t* __restrict__ cfrag,
    const float* __restrict__ cbias, const float* __restrict__ cstat, const uint8_t* __restrict__ Lfrag,
    uint16_t* __restrict__ codes, uint32_t* __restrict__ counter, uint32_t* __restrict__ list, int Hkv,
    int n_new, int pos0, int64_t ctx_stride) {
  __shared__ __align__(16) uint8_t s_mem[4 * kFragBytes];   // transform: all of L^T; main loop: two blocks
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, g = lane >> 5;
  const int bkv = blockIdx.y, kv = bkv % Hkv;
  const long key_first = (long)blockIdx.x * kKeysPerWG + wave * kKeysPerWave;
  const float* seq_keys = keys + (size_t)bkv * n_new * kD;

  bf16x8 zh[2][8], zl[2][8];
  float zn2[2] = {0.f, 0.f}, kn2[2] = {0.f, 0.f};
  if (MODE == A2ATS_W_BLOCK) {
    const uint8_t* gl = Lfrag + (size_t)kv * 4 * kFragBytes;
    for (int o = tid * 16; o < 4 * kFragBytes; o += kEncThreads * 16) *(uint4*)(s_mem + o) = *(const uint4*)(gl + o);
    __syncthreads();
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const long jr = min(key_first + 32 * tile + col, (long)n_new - 1);
      const float* kp = seq_keys + (size_t)jr * kD;
      bf16x8 kh[8], kl[8];
#pragma unroll
      for (int kt = 0; kt < 8; ++kt) {   // operand element i <-> dimension 16 kt + 8 g + i
        const float4 a = *(const float4*)(kp + 16 * kt + 8 * g), b = *(const float4*)(kp + 16 * kt + 8 * g + 4);
        const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        split8(x, kh[kt], kl[kt], kn2[tile]);
      }
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) {
        f32x16 acc = {0};
        const uint8_t* blk = s_mem + rt * kFragBytes;
#pragma unroll
        for (int kt = 2 * rt; kt < 8; ++kt) {   // L^T is upper triangular: rows 32 rt.. need r >= 32 rt only
          const bf16x8 a_hi = *(const bf16x8*)(blk + ((0 * 8 + kt) * 64 + lane) * 16);
          const bf16x8 a_lo = *(const bf16x8*)(blk + ((1 * 8 + kt) * 64 + lane) * 16);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, kh[kt], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, kl[kt], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, kh[kt], acc, 0, 0, 0);
        }
        // register v holds z[32 rt + 8 (v/4) + 4 g + v%4]: elements 0..7 of k-steps 2 rt and 2 rt + 1
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          float x[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = acc[8 * half + i];
          split8(x, zh[tile][2 * rt + half], zl[tile][2 * rt + half], zn2[tile]);
        }
      }
    }
    __syncthreads();   // L^T is done with; the main loop reuses the memory
  } else {
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const long jr = min(key_first + 32 * tile + col, (long)n_new - 1);
      const float* kp = seq_keys + (size_t)jr * kD;
#pragma unroll
      for (int kt = 0; kt < 8; ++kt) {   // operand element i <-> dimension 16 kt + 8 (i/4) + 4 g + i%4
        const int t0 = 16 * kt + 4 * g;
        const float4 a = *(const float4*)(kp + t0), b = *(const float4*)(kp + t0 + 8);
        float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        if (MODE == A2ATS_W_DIAG) {
          const double* s = sd + (size_t)kv * kD;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            x[i] *= (float)s[t0 + i];
            x[4 + i] *= (float)s[t0 + 8 + i];
          }
        }
        split8(x, zh[tile][kt], zl[tile][kt], zn2[tile]);
      }
    }
  }

  // main loop: blocks of 32 codewords through a double buffer in LDS
  const uint8_t* gblk = cfrag + (size_t)kv * kBlocks * kFragBytes;
  const float* gbias = cbias + (size_t)kv * kCW;
  constexpr int kBuf = kFragBytes + 128;
  {
    *(uint4*)(s_mem + tid * 32) = *(const uint4*)(gblk + tid * 32);
    *(uint4*)(s_mem + tid * 32 + 16) = *(const uint4*)(gblk + tid * 32 + 16);
    if (tid < 8) *(uint4*)(s_mem + kFragBytes + tid * 16) = *(const uint4*)(gbias + tid * 4);
  }
  __syncthreads();
  float s1[2], s2[2], s3[2];
  int c1[2] = {0, 0}, c2[2] = {0, 0};
#pragma unroll
  for (int tile = 0; tile < 2; ++tile) s1[tile] = s2[tile] = s3[tile] = INFINITY;
#pragma unroll 1
  for (int cb = 0; cb < kBlocks; ++cb) {
    const uint8_t* blk = s_mem + (cb & 1) * kBuf;
    uint8_t* nxt = s_mem + ((cb + 1) & 1) * kBuf;
    uint4 p0, p1, pb;
    const bool more = cb + 1 < kBlocks;
    if (more) {
      const uint8_t* src = gblk + (size_t)(cb + 1) * kFragBytes + tid * 32;
      p0 = *(const uint4*)src;
      p1 = *(const uint4*)(src + 16);
      if (tid < 8) pb = *(const uint4*)(gbias + (cb + 1) * 32 + tid * 4);
    }
    f32x16 acc0 = {0}, acc1 = {0};
#pragma unroll
    for (int kt = 0; kt < 8; ++kt) {
      const bf16x8 a_hi = *(const bf16x8*)(blk + ((0 * 8 + kt) * 64 + lane) * 16);
      const bf16x8 a_lo = *(const bf16x8*)(blk + ((1 * 8 + kt) * 64 + lane) * 16);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zh[0][kt], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zh[1][kt], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zl[0][kt], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zl[1][kt], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, zh[0][kt], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, zh[1][kt], acc1, 0, 0, 0);
    }
    // register v of a tile: codeword 32 cb + 8 (v/4) + 4 g + v%4 (the 4 g is added at the end)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 bias = *(const float4*)(blk + kFragBytes + (8 * q + 4 * g) * 4);
      const float bq[4] = {bias.x, bias.y, bias.z, bias.w};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = cb * 32 + 8 * q + r;
        top3_insert(bq[r] - acc0[4 * q + r], c, s1[0], s2[0], s3[0], c1[0], c2[0]);
        top3_insert(bq[r] - acc1[4 * q + r], c, s1[1], s2[1], s3[1], c1[1], c2[1]);
      }
    }
    if (more) {
      *(uint4*)(nxt + tid * 32) = p0;
      *(uint4*)(nxt + tid * 32 + 16) = p1;
      if (tid < 8) *(uint4*)(nxt + kFragBytes + tid * 16) = pb;
    }
    __syncthreads();
  }

  // The two lane halves of a key column hold disjoint codewords: merge them, decide, flag.
  const float cmax = cstat[kv * 4 + 0], lf = cstat[kv * 4 + 1];
#pragma unroll
  for (int tile = 0; tile < 2; ++tile) {
    const int a1 = c1[tile] + 4 * g, a2 = c2[tile] + 4 * g;
    const float o1 = __shfl_xor(s1[tile], 32), o2 = __shfl_xor(s2[tile], 32), o3 = __shfl_xor(s3[tile], 32);
    const int b1 = __shfl_xor(a1, 32), b2 = __shfl_xor(a2, 32);
    const float zn = zn2[tile] + __shfl_xor(zn2[tile], 32), kn = kn2[tile] + __shfl_xor(kn2[tile], 32);
    // smallest three of the six, with the codes of the first two (equal scores: lower code first)
    float m1 = s1[tile], m2 = s2[tile], m3 = s3[tile];
    int d1 = a1, d2 = a2;
    const float os[3] = {o1, o2, o3};
    const int oc[3] = {b1, b2, 0x7fffffff};   // the third one's code is not tracked and never wins a tie
#pragma unroll
    for (int e = 0; e < 3; ++e) {
      const float s = os[e];
      const int c = oc[e];
      const bool lt1 = s < m1 || (s == m1 && c < d1), lt2 = s < m2 || (s == m2 && c < d2);
      m3 = lt2 ? m2 : fminf(m3, s);
      d2 = lt1 ? d1 : (lt2 ? c : d2);
      m2 = lt1 ? m1 : (lt2 ? s : m2);
      d1 = lt1 ? c : d1;
      m1 = lt1 ? s : m1;
    }
    const long j = key_first + 32 * tile + col;
    if (g == 0 && j < n_new) {
      const float reach = kReach * (sqrtf(zn) + (MODE == A2ATS_W_BLOCK ? sqrtf(kn) * lf : 0.f)) * cmax;
      codes[(size_t)bkv * ctx_stride + pos0 + j] = (uint16_t)d1;
      if (!(m2 - m1 > reach)) {
        const uint32_t at = atomicAdd(counter, 1u);
        const uint32_t full = !(m3 - m1 > reach) ? 0x80000000u : 0u;
        list[2 * (size_t)at] = (uint32_t)((size_t)bkv * n_new + j) | full;
        list[2 * (size_t)at + 1] = (uint32_t)d1 | ((uint32_t)d2 << 16);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Exact decisions in float64
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_single_recheck_kernel(
    const float* __restrict__ keys, int mode, const double* __restrict__ Lmat, const double* __restrict__ sd,
    const double* __restrict__ czT, uint16_t* __restrict__ codes, const uint32_t* __restrict__ counter,
    const uint32_t* __restrict__ list, uint32_t n_all, int Hkv, int n_new, int pos0, int64_t ctx_stride) {
  __shared__ double s_k[kD], s_z[kD], s_d[256];
  __shared__ int s_i[256];
  const int tid = threadIdx.x;
  const uint32_t count = list ? *counter : n_all;   // no list: every key, by a full sweep
  for (uint32_t it = blockIdx.x; it < count; it += gridDim.x) {
    uint32_t key = it, pair = 0;
    bool full = true;
    if (list) {
      key = list[2 * (size_t)it] & 0x7fffffffu;
      full = (list[2 * (size_t)it] >> 31) != 0;
      pair = list[2 * (size_t)it + 1];
    }
    const int bkv = (int)(key / (uint32_t)n_new), j = (int)(key % (uint32_t)n_new), kv = bkv % Hkv;
    __syncthreads();   // the arrays of the key before are still being read
    if (tid < kD) s_k[tid] = (double)keys[((size_t)bkv * n_new + j) * kD + tid];
    __syncthreads();
    if (tid < kD) {
      double z;
      if (mode == A2ATS_W_BLOCK) {
        const double* L = Lmat + (size_t)kv * kD * kD;
        z = 0.0;
        for (int r = tid; r < kD; ++r) z += s_k[r] * L[(size_t)r * kD + tid];
      } else {
        z = s_k[tid] * sd[(size_t)kv * kD + tid];
      }
      s_z[tid] = z;
    }
    __syncthreads();
    const double* cz = czT + (size_t)kv * kD * kCW;
    double best;
    int arg;
    if (!full) {   // between the two candidates: dimensions over threads, two sums
      const int ca = (int)(pair & 0xffffu), cb = (int)(pair >> 16);
      double da = 0.0, db = 0.0;
      if (tid < kD) {
        const double ea = s_z[tid] - cz[(size_t)tid * kCW + ca], eb = s_z[tid] - cz[(size_t)tid * kCW + cb];
        da = ea * ea;
        db = eb * eb;
      }
      s_d[tid] = da;
      __syncthreads();
      for (int s = 64; s >= 1; s >>= 1) {
        if (tid < s) s_d[tid] += s_d[tid + s];
        __syncthreads();
      }
      const double ta = s_d[0];
      __syncthreads();
      s_d[tid] = db;
      __syncthreads();
      for (int s = 64; s >= 1; s >>= 1) {
        if (tid < s) s_d[tid] += s_d[tid + s];
        __syncthreads();
      }
      const double tb = s_d[0];
      arg = (tb < ta || (tb == ta && cb < ca)) ? cb : ca;
      if (tid == 0) codes[(size_t)bkv * ctx_stride + pos0 + j] = (uint16_t)arg;
      continue;
    }
    double d[kCW / 256];
#pragma unroll
    for (int q = 0; q < kCW / 256; ++q) d[q] = 0.0;
    for (int t = 0; t < kD; ++t) {
      const double zt = s_z[t];
#pragma unroll
      for (int q = 0; q < kCW / 256; ++q) {
        const double e = zt - cz[(size_t)t * kCW + tid + 256 * q];
        d[q] += e * e;
      }
    }
    best = d[0];
    arg = tid;
#pragma unroll
    for (int q = 1; q < kCW / 256; ++q)
      if (d[q] < best) {
        best = d[q];
        arg = tid + 256 * q;
      }
    s_d[tid] = best;
    s_i[tid] = arg;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
      if (tid < s) {
        const double o = s_d[tid + s];
        const int oi = s_i[tid + s];
        if (o < s_d[tid] || (o == s_d[tid] && oi < s_i[tid])) {
          s_d[tid] = o;
          s_i[tid] = oi;
        }
      }
      __syncthreads();
    }
    if (tid == 0) codes[(size_t)bkv * ctx_stride + pos0 + j] = (uint16_t)s_i[0];
  }
}

LdsSlot g_factor_lds[16];

}  // namespace

size_t encode_single_ws_bytes(const a2ats_dims& d) { return enc_single_ws(d).bytes; }

hipError_t launch_encode_single(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                const float* codebook, const float* weights, int mode, void* codes, void* ws,
                                hipStream_t stream) {
  if (n_new == 0 || d.batch == 0) return hipSuccess;
  const EncWs w = enc_single_ws(d);
  uint8_t* base = (uint8_t*)ws;
  double* Lmat = (double*)(base + w.off_L);
  double* sd = (double*)(base + w.off_sd);
  double* czT = (double*)(base + w.off_czT);
  uint8_t* cfrag = base + w.off_cfrag;
  float* cbias = (float*)(base + w.off_cbias);
  float* cstat = (float*)(base + w.off_cstat);
  uint8_t* Lfrag = base + w.off_Lfrag;
  uint32_t* counter = (uint32_t*)(base + w.off_count);
  uint32_t* list = (uint32_t*)(base + w.off_list);
  const int Hkv = d.n_kv_heads, bkv = d.batch * Hkv;

  const size_t factor_lds = (size_t)kD * kD * sizeof(double);
  hipError_t err = allow_dynamic_lds(encode_single_factor_kernel, factor_lds, g_factor_lds);
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(encode_single_factor_kernel, dim3(Hkv), dim3(256), factor_lds, stream, weights, mode, Lmat,
                     sd, (uint16_t*)Lfrag, cstat, counter);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  hipLaunchKernelGGL(encode_single_codewords_kernel, dim3(kCW / 64, Hkv), dim3(256), 0, stream, codebook, mode,
                     Lmat, sd, czT, (uint16_t*)cfrag, cbias, cstat);
  if ((err = hipGetLastError()) != hipSuccess) return err;

  const uint32_t n_all = (uint32_t)((size_t)bkv * n_new);
  if (n_new <= kFewSingle) {
    hipLaunchKernelGGL(encode_single_recheck_kernel, dim3(n_all), dim3(256), 0, stream, keys, mode, Lmat, sd, czT,
                       (uint16_t*)codes, counter, (const uint32_t*)nullptr, n_all, Hkv, n_new, pos0, d.ctx_stride);
    return hipGetLastError();
  }
  const dim3 grid((n_new + kKeysPerWG - 1) / kKeysPerWG, bkv), block(kEncThreads);
#define A2ATS_LAUNCH_ENC1(MODE)                                                                        \
  hipLaunchKernelGGL((encode_single_kernel<MODE>), grid, block, 0, stream, keys, sd, cfrag, cbias, cstat, \
                     Lfrag, (uint16_t*)codes, counter, list, Hkv, n_new, pos0, d.ctx_stride)
  if (mode == A2ATS_W_NONE) A2ATS_LAUNCH_ENC1(A2ATS_W_NONE);
  else if (mode == A2ATS_W_DIAG) A2ATS_LAUNCH_ENC1(A2ATS_W_DIAG);
  else A2ATS_LAUNCH_ENC1(A2ATS_W_BLOCK);
#undef A2ATS_LAUNCH_ENC1
  if ((err = hipGetLastError()) != hipSuccess) return err;
  const uint32_t re_grid = n_all < 2048u ? n_all : 2048u;
  hipLaunchKernelGGL(encode_single_recheck_kernel, dim3(re_grid), dim3(256), 0, stream, keys, mode, Lmat, sd, czT,
                     (uint16_t*)codes, counter, (const uint32_t*)list, n_all, Hkv, n_new, pos0, d.ctx_stride);
  return hipGetLastError();
}

}  // namespace a2ats
