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
//   encode_single_transform_kernel z = k L in float64, rounded once to float32 (full-matrix mode only;
//                                  a few k keys at a time, into a buffer the main pass reads as keys)
//   encode_single_kernel           256 keys per workgroup: z is split the same way and kept in
//                                  registers as the B operands; the codewords stream through LDS
//                                  32 at a time as the A operand; three bf16 products per term
//                                  (hi.hi + hi.lo + lo.hi, float32 accumulate) give the scores to
//                                  about 2^-18 relative.  Every lane owns one key column of the
//                                  32 x 32 result tile, so the running smallest three scores (and
//                                  the codes of the first two) are per-lane registers; nothing
//                                  crosses lanes until the end.
//   encode_single_recheck_kernel   keys whose two smallest scores are closer than the rounding reach
//                                  of the bf16 products are decided in float64 between those two
//                                  codewords; keys with three that close by a float64 sweep over all
//                                  4096.  So the emitted code is the float64 argmin.
//   encode_single_heff_kernel      L L^T (full-matrix mode), for w = c (L L^T) kept beside c^z
//   encode_single_sweep_kernel     the few-key (decode-time append) route: the distortion expanded as
//                                  |z|^2 - 2 k . w_c + |c^z|^2, so one float64 pass of dot products
//                                  over w decides the key; 16 workgroups per key, then
//                                  encode_single_sweep_pick_kernel
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {
namespace {

constexpr int kCW = 4096;               // codewords per KV head
constexpr int kD = 128;                 // head dimension
constexpr int kEncWaves = 4;           // two workgroups per CU: one wave of each per SIMD
constexpr int kEncThreads = 64 * kEncWaves;
constexpr int kKeysPerWave = 64;        // two 32-key column tiles
constexpr int kKeysPerWG = kKeysPerWave * kEncWaves;
constexpr int kFragBytes = 2 * 8 * 64 * 16;   // (hi, lo) x 8 k-steps x 64 lanes x 16 bytes: 32 rows of 128 dims
constexpr int kBlocks = kCW / 32;       // streamed 32-codeword blocks
static_assert(kFragBytes / 16 / kEncThreads == 4, "a thread stages four 16-byte pieces of a block");
constexpr int kFewSingle = kFewSingleKeys;   // at most this many keys per (sequence, KV head): float64 sweep only
constexpr int kSlices = kEncodeSlices;  // workgroups sharing the codewords of one such key
constexpr float kReach = 1.5e-5f;       // rounding reach of a score, relative to |z| max|c^z|
constexpr int kChunk = 16384;           // keys per (sequence, KV head) transformed at a time

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct EncWs {
  size_t off_L, off_sd, off_heff, off_czT, off_wT, off_chalf, off_cfrag, off_cbias, off_cstat, off_z, off_count, off_list,
      off_part, bytes;
  int chunk;   // keys per (sequence, KV head) the transform buffer holds
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
  w.off_heff = take(Hkv * kD * kD * sizeof(double));
  w.off_czT = take(Hkv * kD * kCW * sizeof(double));
  w.off_wT = take(Hkv * kD * kCW * sizeof(double));
  w.off_chalf = take(Hkv * kCW * sizeof(double));
  w.off_cfrag = take(Hkv * kBlocks * (size_t)kFragBytes);
  w.off_cbias = take(Hkv * kCW * sizeof(float));
  w.off_cstat = take(Hkv * 4 * sizeof(float));
  w.chunk = (int)(d.ctx_stride < kChunk ? d.ctx_stride : kChunk);
  w.off_z = take((size_t)d.batch * Hkv * w.chunk * kD * sizeof(float));
  w.off_count = take(sizeof(uint32_t));
  w.off_list = take(keys_max * 2 * sizeof(uint32_t));
  w.off_part = take((size_t)d.batch * Hkv * kFewSingle * kSlices * 2 * sizeof(double));
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
// Per KV head: the factor L (H = L L^T) and its Frobenius norm.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_single_factor_kernel(
    const float* __restrict__ weights, int mode, double* __restrict__ Lmat, double* __restrict__ sd,
    float* __restrict__ cstat) {
  extern __shared__ double s_A[];   // 128 x 128, lower triangle in use
  __shared__ double s_red[256];
  const int kv = blockIdx.x, tid = threadIdx.x;
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
}

// ------------------------------------------------------------------------------------------
// L L^T, the matrix the factor stands for (equal to H up to rounding when H is positive definite;
// the few-key route weighs with it so that both routes minimise the same distortion).
// One workgroup per row i: thread j sums L[i][m] L[j][m] over m.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kD) void encode_single_heff_kernel(const double* __restrict__ Lmat,
                                                                double* __restrict__ heff) {
  const int kv = blockIdx.y, i = blockIdx.x, j = threadIdx.x;
  const double* L = Lmat + (size_t)kv * kD * kD;
  double s0 = 0.0, s1 = 0.0;
  const int m_end = (i < j ? i : j) + 1;   // L[r][m] = 0 for m > r
  int m = 0;
  for (; m + 1 < m_end; m += 2) {
    s0 += L[(size_t)i * kD + m] * L[(size_t)j * kD + m];
    s1 += L[(size_t)i * kD + m + 1] * L[(size_t)j * kD + m + 1];
  }
  if (m < m_end) s0 += L[(size_t)i * kD + m] * L[(size_t)j * kD + m];
  heff[((size_t)kv * kD + i) * kD + j] = s0 + s1;
}

// ------------------------------------------------------------------------------------------
// c^z = c L for 64 codewords per workgroup (float64), in the three forms the other kernels read,
// and w = c (L L^T) with 1/2 |c^z|^2 in float64 for the few-key route.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_single_codewords_kernel(
    const float* __restrict__ codebook, int mode, const double* __restrict__ Lmat, const double* __restrict__ sd,
    const double* __restrict__ heff, double* __restrict__ czT, double* __restrict__ wT, double* __restrict__ chalf,
    uint16_t* __restrict__ cfrag, float* __restrict__ cbias, float* __restrict__ cstat) {
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
    const double neg = -acc[u];   // the operand is -c^z: the matrix core then leaves 1/2 |c^z|^2 - z . c^z
    const uint16_t hi = f32_to_bf16((float)neg);
    const uint16_t lo = f32_to_bf16((float)(neg - (double)bf16_to_f32(hi)));
    blk[((0 * 8 + kt) * 64 + row + 32 * g) * 8 + i] = hi;
    blk[((1 * 8 + kt) * 64 + row + 32 * g) * 8 + i] = lo;
  }
  __syncthreads();
  if (tq == 0) {
    const double n = s_n[0][c] + s_n[1][c] + s_n[2][c] + s_n[3][c];
    cbias[(size_t)kv * kCW + cg] = (float)(0.5 * n);
    chalf[(size_t)kv * kCW + cg] = 0.5 * n;
    // max over the codewords of |c^z|, rounded up (a non-negative float orders like its bits)
    atomicMax((uint32_t*)&cstat[kv * 4 + 0], __float_as_uint(__double2float_ru(sqrt(n))));
  }
  // w = c (L L^T): the distortion is |z|^2 - 2 k . w + |c^z|^2, so the few-key route needs no z
  if (mode == A2ATS_W_BLOCK) {
#pragma unroll
    for (int u = 0; u < 32; ++u) acc[u] = 0.0;
    const double* Hm = heff + (size_t)kv * kD * kD + 32 * tq;
    for (int r = 0; r < kD; ++r) {
      const double cv = (double)s_c[c][r];
#pragma unroll
      for (int u = 0; u < 32; ++u) acc[u] += cv * Hm[(size_t)r * kD + u];
    }
  } else {
#pragma unroll
    for (int u = 0; u < 32; ++u) {
      const double sdu = sd[(size_t)kv * kD + 32 * tq + u];
      acc[u] = (double)s_c[c][32 * tq + u] * sdu * sdu;
    }
  }
#pragma unroll
  for (int u = 0; u < 32; ++u) wT[((size_t)kv * kD + 32 * tq + u) * kCW + cg] = acc[u];
}

// ------------------------------------------------------------------------------------------
// z = k L for rows j0 .. j0 + n_part - 1 of every sequence, float64 accumulation, one rounding.
// A thread owns one key and 32 consecutive output dimensions; the rows of L it needs are the same
// for the whole wave.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_single_transform_kernel(
    const float* __restrict__ keys, const double* __restrict__ Lmat, float* __restrict__ z, int Hkv, int n_new,
    int j0, int n_part, int chunk) {
  __shared__ float s_k[64][kD + 1];
  const int bkv = blockIdx.y, kv = bkv % Hkv, tid = threadIdx.x;
  const int key = tid & 63, og = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int first = blockIdx.x * 64;
  const float* src = keys + ((size_t)bkv * n_new + j0) * kD;
  for (int e = tid; e < 64 * (kD / 4); e += 256) {
    const int row = e / (kD / 4), c4 = e % (kD / 4);
    const float4 f = *(const float4*)(src + (size_t)min(first + row, n_part - 1) * kD + 4 * c4);
    s_k[row][4 * c4] = f.x, s_k[row][4 * c4 + 1] = f.y, s_k[row][4 * c4 + 2] = f.z, s_k[row][4 * c4 + 3] = f.w;
  }
  __syncthreads();
  double acc[32];
#pragma unroll
  for (int u = 0; u < 32; ++u) acc[u] = 0.0;
  const double* L = Lmat + (size_t)kv * kD * kD + 32 * og;
  for (int r = 32 * og; r < kD; ++r) {   // L[r][t] = 0 for r < t
    const double kr = (double)s_k[key][r];
#pragma unroll
    for (int u = 0; u < 32; ++u) acc[u] += kr * L[(size_t)r * kD + u];
  }
  if (first + key < n_part) {
    float* dst = z + ((size_t)bkv * chunk + first + key) * kD + 32 * og;
#pragma unroll
    for (int u = 0; u < 32; u += 4)
      *(float4*)(dst + u) = make_float4((float)acc[u], (float)acc[u + 1], (float)acc[u + 2], (float)acc[u + 3]);
  }
}

// ------------------------------------------------------------------------------------------
// Main pass
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void split8(const float (&z)[8], bf16x8& hi, bf16x8& lo, float& n2) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int i = 0; i < 8; i += 2) {   // two at a time: one packed conversion each for hi and lo
    const f32x2 v = {z[i], z[i + 1]};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    const f32x2 back = __builtin_convertvector(h, f32x2);
    const bf16x2 l = __builtin_convertvector(v - back, bf16x2);
    hi[i] = h.x, hi[i + 1] = h.y;
    lo[i] = l.x, lo[i + 1] = l.y;
    n2 += z[i] * z[i] + z[i + 1] * z[i + 1];   // (the norm only scales the rounding reach)
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
__global__ __launch_bounds__(kEncThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void encode_single_kernel(
    const float* __restrict__ keys, const double* __restrict__ sd, const uint8_t* __restrict__ cfrag,
    const float* __restrict__ cbias, const float* __restrict__ cstat, uint16_t* __restrict__ codes,
    uint32_t* __restrict__ counter, uint32_t* __restrict__ list, int Hkv, int n_new, int pos0,
    int64_t ctx_stride, int j0, int n_part, int64_t seq_stride) {
  // `keys` holds rows j0 .. j0 + n_part - 1 of every sequence, seq_stride floats apart (the
  // caller's keys themselves, or the transformed copy of one part of them).
  __shared__ __align__(16) uint8_t s_mem[2 * (kFragBytes + 128)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, g = lane >> 5;
  const int bkv = blockIdx.y, kv = bkv % Hkv;
  const long key_first = (long)blockIdx.x * kKeysPerWG + wave * kKeysPerWave;
  const float* seq_keys = keys + (size_t)bkv * seq_stride;

  bf16x8 zh[2][8], zl[2][8];
  float zn2[2] = {0.f, 0.f};
  {
    // (four k-steps of loads in flight at a time: with all sixteen the registers they land in
    // and the 128 the operands need do not fit, and the spills cost far more than the latency)
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const long jr = min(key_first + 32 * tile + col, (long)n_part - 1);
      const float* kp = seq_keys + (size_t)jr * kD;
#pragma unroll
      for (int k4 = 0; k4 < 8; k4 += 4) {
        float4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {   // operand element i <-> dimension 16 kt + 8 (i/4) + 4 g + i%4
          a[u] = *(const float4*)(kp + 16 * (k4 + u) + 4 * g);
          b[u] = *(const float4*)(kp + 16 * (k4 + u) + 4 * g + 8);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int kt = k4 + u, t0 = 16 * kt + 4 * g;
          float x[8] = {a[u].x, a[u].y, a[u].z, a[u].w, b[u].x, b[u].y, b[u].z, b[u].w};
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
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // Main loop: blocks of 32 codewords (operands + their 1/2 |c^z|^2) through a double buffer in
  // LDS.  The accumulators start at 1/2 |c^z|^2 and the stored operands are -c^z, so the matrix
  // core leaves the score itself.  Ranking: a score only matters if it is below the lane's third
  // smallest so far, which after the first blocks is rare, so four scores at a time are tested by
  // their minimum and the insertion is skipped by the whole wave when no lane needs it.  (The
  // vector ALU issues one instruction per four cycles per SIMD and a product takes 32: ten
  // instructions per score would cost more than the products.)  Two workgroups share a CU, one wave
  // of each per SIMD, so one computes while the other waits at its barrier.
  const uint8_t* gblk = cfrag + (size_t)kv * kBlocks * kFragBytes;
  const float* gbias = cbias + (size_t)kv * kCW;
  constexpr int kBuf = kFragBytes + 128;
  float s1[2], s2[2], s3[2];
  int c1[2] = {0, 0}, c2[2] = {0, 0};
#pragma unroll
  for (int tile = 0; tile < 2; ++tile) s1[tile] = s2[tile] = s3[tile] = INFINITY;

  // The loads of the next block are written as asm statements: as ordinary loads the compiler
  // sinks them past the ranking branches down to their only use, the LDS store before the barrier,
  // and every step then waits for global memory in the open.  The matching wait is explicit
  // (loads the compiler does not know of only make its own, counted waits stricter).
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto prefetch = [&](int bi, u32x4 (&p)[kFragBytes / 16 / kEncThreads], float& pb) {
    bi = min(bi, kBlocks - 1);   // the step of the last block loads it once more, unused
    const uint8_t* src = gblk + (size_t)bi * kFragBytes + tid * 16;
#pragma unroll
    for (int i = 0; i < kFragBytes / 16 / kEncThreads; ++i)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(p[i]) : "v"(src + i * kEncThreads * 16) : "memory");
    const float* bsrc = gbias + bi * 32 + (tid & 31);
    asm volatile("global_load_dword %0, %1, off" : "=&v"(pb) : "v"(bsrc) : "memory");
  };
  auto stage = [&](int bi, u32x4 (&p)[kFragBytes / 16 / kEncThreads], float& pb) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(p[0]), "+v"(p[1]), "+v"(p[2]), "+v"(p[3]), "+v"(pb)::"memory");
    uint8_t* dst = s_mem + (bi & 1) * kBuf;
#pragma unroll
    for (int i = 0; i < kFragBytes / 16 / kEncThreads; ++i) *(u32x4*)(dst + tid * 16 + i * kEncThreads * 16) = p[i];
    *(float*)(dst + kFragBytes + (tid & 31) * 4) = pb;   // several threads write each word, all the same
  };
  {
    u32x4 p[kFragBytes / 16 / kEncThreads];
    float pb;
    prefetch(0, p, pb);
    stage(0, p, pb);
  }
  __syncthreads();
#pragma unroll 1
  for (int cb = 0; cb < kBlocks; ++cb) {
    // The order of the memory operations is pinned (nothing crosses a fence): the next block is
    // requested from global memory first, and the operands of k-step kt + 1 are requested from
    // LDS before the six products of k-step kt, so neither latency is waited for in the open.
    u32x4 p[kFragBytes / 16 / kEncThreads];
    float pb;
    prefetch(cb + 1, p, pb);
    __builtin_amdgcn_sched_barrier(0);
    const uint8_t* blk = s_mem + (cb & 1) * kBuf;
    const uint8_t* fr = blk + lane * 16;
    bf16x8 a_hi = *(const bf16x8*)fr, a_lo = *(const bf16x8*)(fr + 8 * 1024);
    // register v of a tile: codeword 32 cb + 8 (v/4) + 4 g + v%4 (the 4 g is added at the end)
    f32x16 acc0, acc1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 f = *(const float4*)(blk + kFragBytes + (8 * q + 4 * g) * 4);
      acc0[4 * q] = acc1[4 * q] = f.x;
      acc0[4 * q + 1] = acc1[4 * q + 1] = f.y;
      acc0[4 * q + 2] = acc1[4 * q + 2] = f.z;
      acc0[4 * q + 3] = acc1[4 * q + 3] = f.w;
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kt = 0; kt < 8; ++kt) {
      bf16x8 n_hi = a_hi, n_lo = a_lo;
      if (kt < 7) {
        n_hi = *(const bf16x8*)(fr + (kt + 1) * 1024);
        n_lo = *(const bf16x8*)(fr + (8 + kt + 1) * 1024);
      }
      __builtin_amdgcn_sched_barrier(0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zh[0][kt], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zh[1][kt], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zl[0][kt], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, zl[1][kt], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, zh[0][kt], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, zh[1][kt], acc1, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      a_hi = n_hi;
      a_lo = n_lo;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float m0 = fminf(fminf(acc0[4 * q], acc0[4 * q + 1]), fminf(acc0[4 * q + 2], acc0[4 * q + 3]));
      if (m0 < s3[0]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) top3_insert(acc0[4 * q + r], cb * 32 + 8 * q + r, s1[0], s2[0], s3[0], c1[0], c2[0]);
      }
      const float m1 = fminf(fminf(acc1[4 * q], acc1[4 * q + 1]), fminf(acc1[4 * q + 2], acc1[4 * q + 3]));
      if (m1 < s3[1]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) top3_insert(acc1[4 * q + r], cb * 32 + 8 * q + r, s1[1], s2[1], s3[1], c1[1], c2[1]);
      }
    }
    stage(cb + 1, p, pb);
    __syncthreads();
  }

  // The two lane halves of a key column hold disjoint codewords: merge them, decide, flag.
  const float cmax = cstat[kv * 4 + 0];
#pragma unroll
  for (int tile = 0; tile < 2; ++tile) {
    const int a1 = c1[tile] + 4 * g, a2 = c2[tile] + 4 * g;
    const float o1 = __shfl_xor(s1[tile], 32), o2 = __shfl_xor(s2[tile], 32), o3 = __shfl_xor(s3[tile], 32);
    const int b1 = __shfl_xor(a1, 32), b2 = __shfl_xor(a2, 32);
    const float zn = zn2[tile] + __shfl_xor(zn2[tile], 32);
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
    if (g == 0 && j < n_part) {
      const float reach = kReach * sqrtf(zn) * cmax;
      codes[(size_t)bkv * ctx_stride + pos0 + j0 + j] = (uint16_t)d1;
      if (!(m2 - m1 > reach)) {
        const uint32_t at = atomicAdd(counter, 1u);
        const uint32_t full = !(m3 - m1 > reach) ? 0x80000000u : 0u;
        list[2 * (size_t)at] = (uint32_t)((size_t)bkv * n_new + j0 + j) | full;
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
    const uint32_t* __restrict__ list, int Hkv, int n_new, int pos0, int64_t ctx_stride) {
  __shared__ double s_k[kD], s_z[kD], s_d[256];
  __shared__ int s_i[256];
  const int tid = threadIdx.x;
  const uint32_t count = *counter;
  for (uint32_t it = blockIdx.x; it < count; it += gridDim.x) {
    const uint32_t key = list[2 * (size_t)it] & 0x7fffffffu, pair = list[2 * (size_t)it + 1];
    const bool full = (list[2 * (size_t)it] >> 31) != 0;
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

__global__ void encode_single_clear_kernel(uint32_t* counter) { *counter = 0; }

// The few-key (append) route: every key is decided by a float64 sweep, its 4096 codewords split
// over kSlices workgroups (one workgroup would read 4 MB by itself).  With w_c = c (L L^T) the
// distortion of codeword c is |z|^2 - 2 k . w_c + |c^z|^2, so the sweep minimises
// 1/2 |c^z|^2 - k . w_c and needs neither z nor L: one pass of dot products over wT.
// part[key][slice] = {smallest value of the slice, its code as a double}.
// 512 threads and at most 128 registers each, so that the two workgroups per CU of the usual
// decode batch (32 keys x 16 slices on 256 CUs) are resident together.
constexpr int kSweepThreads = 512;
__global__ __launch_bounds__(kSweepThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void encode_single_sweep_kernel(
    const float* __restrict__ keys, const double* __restrict__ wT, const double* __restrict__ chalf,
    double* __restrict__ part, int Hkv, int n_new) {
  constexpr int PER = kCW / kSlices;   // codewords per slice
  static_assert(PER == 256 && kSweepThreads == 2 * PER, "a thread owns one codeword and half of the dimensions");
  __shared__ double s_k[kD], s_p[2][PER];
  __shared__ int s_i[PER];
  const int tid = threadIdx.x, slice = blockIdx.y, key = blockIdx.x;
  const int bkv = key / n_new, kv = bkv % Hkv;
  // thread = (codeword, half of the dimensions): the first 32 of its 64 entries are requested before
  // the key is looked at; each is replaced by its successor as it is used.  (The fences keep the
  // compiler from requesting the second half up front as well, which would not fit the registers.)
  const int cl = tid & (PER - 1), th = tid >> 8, c = slice * PER + cl;
  const double* w = wT + ((size_t)kv * kD + 64 * th) * kCW + c;
  double wv[32];
#pragma unroll
  for (int t = 0; t < 32; ++t) wv[t] = w[(size_t)t * kCW];
  const double half = chalf[(size_t)kv * kCW + c];
  if (tid < kD) s_k[tid] = (double)keys[(size_t)key * kD + tid];
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  double d0 = 0.0, d1 = 0.0;
#pragma unroll
  for (int t = 0; t < 32; t += 2) {
    d0 += s_k[64 * th + t] * wv[t];
    d1 += s_k[64 * th + t + 1] * wv[t + 1];
    wv[t] = w[(size_t)(32 + t) * kCW];
    wv[t + 1] = w[(size_t)(32 + t + 1) * kCW];
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int t = 0; t < 32; t += 2) {
    d0 += s_k[64 * th + 32 + t] * wv[t];
    d1 += s_k[64 * th + 32 + t + 1] * wv[t + 1];
  }
  s_p[th][cl] = d0 + d1;
  __syncthreads();
  if (tid < PER) {
    s_p[0][tid] = half - (s_p[0][tid] + s_p[1][tid]);
    s_i[tid] = c;
  }
  __syncthreads();
  for (int s = PER / 2; s >= 1; s >>= 1) {
    if (tid < s) {
      const double o = s_p[0][tid + s];
      const int oi = s_i[tid + s];
      if (o < s_p[0][tid] || (o == s_p[0][tid] && oi < s_i[tid])) {
        s_p[0][tid] = o;
        s_i[tid] = oi;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    part[((size_t)key * kSlices + slice) * 2] = s_p[0][0];
    part[((size_t)key * kSlices + slice) * 2 + 1] = (double)s_i[0];
  }
}

__global__ void encode_single_sweep_pick_kernel(const double* __restrict__ part, uint16_t* __restrict__ codes,
                                                uint32_t n_all, int n_new, int pos0, int64_t ctx_stride) {
  const uint32_t key = blockIdx.x * blockDim.x + threadIdx.x;
  if (key >= n_all) return;
  double best = part[(size_t)key * kSlices * 2];
  int arg = (int)part[(size_t)key * kSlices * 2 + 1];
  for (int s = 1; s < kSlices; ++s) {   // slices hold ascending codes: strict < keeps the lower code
    const double d = part[((size_t)key * kSlices + s) * 2];
    if (d < best) {
      best = d;
      arg = (int)part[((size_t)key * kSlices + s) * 2 + 1];
    }
  }
  const int bkv = (int)(key / (uint32_t)n_new), j = (int)(key % (uint32_t)n_new);
  codes[(size_t)bkv * ctx_stride + pos0 + j] = (uint16_t)arg;
}

// ------------------------------------------------------------------------------------------
// k-means++ seeding under the query-aware distortion (section 4.2 initialises its k-means that
// way): the first codeword is key floor(u_0 n), every further one is drawn with probability
// proportional to the distortion to the nearest codeword chosen so far.  The draws are sequential,
// so one workgroup per KV head runs all of them; the caller supplies the uniform numbers u.
// Distortions are ||z_i - z_c||^2 in float64 over the float32 transformed keys z = k L.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void scale_keys_kernel(const float* __restrict__ keys, const double* __restrict__ sd,
                                                         float* __restrict__ z, int Hkv, size_t n_rows_per_seq) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;   // element of [B*Hkv][n][128]
  const int bkv = blockIdx.y, kv = bkv % Hkv;
  if (e >= n_rows_per_seq * kD) return;
  const size_t at = (size_t)bkv * n_rows_per_seq * kD + e;
  z[at] = (float)((double)keys[at] * sd[(size_t)kv * kD + e % kD]);
}

constexpr int kSeedThreads = 1024;
constexpr int kSeedChunk = 4;   // consecutive rows per thread of the update kernel = rows per partial sum

// State of the draws of one KV head between the kernels of a round.
struct SeedState {
  long pick;          // row of the codeword drawn last
  float zc[kD];       // its transformed key
};

__device__ __forceinline__ const float* seed_row(const float* base, long i, int kv, int Hkv, int n_new) {
  return base + (((size_t)(i / n_new) * Hkv + kv) * n_new + i % n_new) * kD;
}

// Records draw r (st->pick): the codeword is the key itself; keeps its transformed key for the update.
__device__ __forceinline__ void seed_record(SeedState* st, const float* keys, const float* z, float* codebook_out,
                                            int32_t* picks, long pick, int r, int kv, int Hkv, int n_new, int tid) {
  if (tid < kD) {
    codebook_out[((size_t)kv * kCW + r) * kD + tid] = seed_row(keys, pick, kv, Hkv, n_new)[tid];
    st->zc[tid] = seed_row(z, pick, kv, Hkv, n_new)[tid];
  }
  if (tid == 0) {
    st->pick = pick;
    if (picks) picks[(size_t)kv * kCW + r] = (int32_t)pick;
  }
}

__global__ __launch_bounds__(128) void seed_first_kernel(const float* __restrict__ keys, const float* __restrict__ z,
                                                         const double* __restrict__ u, SeedState* __restrict__ state,
                                                         float* __restrict__ codebook_out, int32_t* __restrict__ picks,
                                                         int B, int Hkv, int n_new) {
  const int kv = blockIdx.x;
  const long rows = (long)B * n_new;
  const long pick = min(rows - 1, (long)(u[(size_t)kv * kCW] * (double)rows));
  seed_record(state + kv, keys, z, codebook_out, picks, pick, 0, kv, Hkv, n_new, threadIdx.x);
}

// Distortions of every row to the codeword drawn last, running minimum, and one partial sum per
// kSeedChunk consecutive rows (summed in row order).
__global__ __launch_bounds__(256) void seed_update_kernel(const float* __restrict__ z, const SeedState* __restrict__ state,
                                                          double* __restrict__ dmin, double* __restrict__ partial,
                                                          int B, int Hkv, int n_new, int first_round) {
  __shared__ double s_zc[kD];
  const int kv = blockIdx.y, tid = threadIdx.x;
  const long rows = (long)B * n_new, n_part = (rows + kSeedChunk - 1) / kSeedChunk;
  if (tid < kD) s_zc[tid] = (double)state[kv].zc[tid];
  __syncthreads();
  const long p = (long)blockIdx.x * 256 + tid;
  if (p >= n_part) return;
  double* d = dmin + (size_t)kv * rows;
  double own = 0.0;
  for (long i = p * kSeedChunk; i < min(rows, (p + 1) * kSeedChunk); ++i) {
    const float4* zi = (const float4*)seed_row(z, i, kv, Hkv, n_new);
    double acc = 0.0;
#pragma unroll 8
    for (int t4 = 0; t4 < kD / 4; ++t4) {
      const float4 f = zi[t4];
      const double e0 = (double)f.x - s_zc[4 * t4], e1 = (double)f.y - s_zc[4 * t4 + 1];
      const double e2 = (double)f.z - s_zc[4 * t4 + 2], e3 = (double)f.w - s_zc[4 * t4 + 3];
      acc += e0 * e0;
      acc += e1 * e1;
      acc += e2 * e2;
      acc += e3 * e3;
    }
    const double dm = first_round ? acc : fmin(d[i], acc);
    d[i] = dm;
    own += dm;
  }
  partial[(size_t)kv * n_part + p] = own;
}

// Draw r: the first row whose inclusive prefix sum of the distortions exceeds u_r times their total.
__global__ __launch_bounds__(kSeedThreads) void seed_pick_kernel(
    const float* __restrict__ keys, const float* __restrict__ z, const double* __restrict__ u,
    const double* __restrict__ dmin, const double* __restrict__ partial, SeedState* __restrict__ state,
    float* __restrict__ codebook_out, int32_t* __restrict__ picks, int B, int Hkv, int n_new, int r) {
  __shared__ double s_wave[kSeedThreads / 64];
  __shared__ long s_pick;
  __shared__ int s_owner;
  const int kv = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long rows = (long)B * n_new, n_part = (rows + kSeedChunk - 1) / kSeedChunk;
  const long per = (n_part + kSeedThreads - 1) / kSeedThreads;
  const long p_lo = min(n_part, tid * per), p_hi = min(n_part, p_lo + per);   // this thread's contiguous partials
  const double* pk = partial + (size_t)kv * n_part;
  double own = 0.0;
  for (long p = p_lo; p < p_hi; ++p) own += pk[p];
  double inc = own;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const double o = __shfl_up(inc, off);
    if (lane >= off) inc += o;
  }
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  double base = 0.0, total = 0.0;
  for (int w = 0; w < kSeedThreads / 64; ++w) {
    if (w < wave) base += s_wave[w];
    total += s_wave[w];
  }
  base += inc - own;
  const double ur = u[(size_t)kv * kCW + r], target = ur * total;
  // all distortions zero (every key equals a chosen codeword): a uniform draw instead
  if (tid == 0) {
    s_pick = total > 0.0 ? 0 : min(rows - 1, (long)(ur * (double)rows));
    s_owner = -1;
  }
  __syncthreads();
  // the row belongs to the last thread whose exclusive prefix does not exceed the target
  // (prefixes do not decrease with the thread index)
  const uint64_t below = __ballot(total > 0.0 && p_lo < p_hi && base <= target);
  if (lane == 0 && below) atomicMax(&s_owner, wave * 64 + 63 - (int)__clzll((unsigned long long)below));
  __syncthreads();
  if (tid == s_owner) {
    const double* d = dmin + (size_t)kv * rows;
    double run = base;
    long found = min(rows, p_hi * kSeedChunk) - 1;   // (rounding: if the walk falls short, the thread's last row)
    bool done = false;
    for (long p = p_lo; p < p_hi && !done; ++p) {
      if (run + pk[p] > target || p == p_hi - 1) {   // the row is in this partial (or the walk ends here)
        for (long i = p * kSeedChunk; i < min(rows, (p + 1) * kSeedChunk); ++i) {
          run += d[i];
          if (run > target) {
            found = i;
            done = true;
            break;
          }
        }
        if (!done && p < p_hi - 1) continue;   // rounding: the partial fell just short; go on
        done = true;
      } else {
        run += pk[p];
      }
    }
    s_pick = found;
  }
  __syncthreads();
  seed_record(state + kv, keys, z, codebook_out, picks, s_pick, r, kv, Hkv, n_new, tid);
}

LdsSlot g_factor_lds[16];

}  // namespace

size_t encode_single_ws_bytes(const a2ats_dims& d) { return enc_single_ws(d).bytes; }

hipError_t launch_encode_single_prepare(const a2ats_dims& d, const float* codebook, const float* weights, int mode,
                                        void* ws, hipStream_t stream) {
  const EncWs w = enc_single_ws(d);
  uint8_t* base = (uint8_t*)ws;
  double* Lmat = (double*)(base + w.off_L);
  double* sd = (double*)(base + w.off_sd);
  float* cstat = (float*)(base + w.off_cstat);
  const size_t factor_lds = (size_t)kD * kD * sizeof(double);
  hipError_t err = allow_dynamic_lds(encode_single_factor_kernel, factor_lds, g_factor_lds);
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(encode_single_factor_kernel, dim3(d.n_kv_heads), dim3(256), factor_lds, stream, weights, mode,
                     Lmat, sd, cstat);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  double* heff = (double*)(base + w.off_heff);
  if (mode == A2ATS_W_BLOCK) {
    hipLaunchKernelGGL(encode_single_heff_kernel, dim3(kD, d.n_kv_heads), dim3(kD), 0, stream, Lmat, heff);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  hipLaunchKernelGGL(encode_single_codewords_kernel, dim3(kCW / 64, d.n_kv_heads), dim3(256), 0, stream, codebook,
                     mode, Lmat, sd, heff, (double*)(base + w.off_czT), (double*)(base + w.off_wT),
                     (double*)(base + w.off_chalf), (uint16_t*)(base + w.off_cfrag), (float*)(base + w.off_cbias),
                     cstat);
  return hipGetLastError();
}

hipError_t launch_encode_single_sweep(const a2ats_dims& d, const float* keys, int n_new, const float* codebook,
                                      const float* weights, int mode, bool prepared, void* ws,
                                      const double** part_out, hipStream_t stream) {
  const EncWs w = enc_single_ws(d);
  uint8_t* base = (uint8_t*)ws;
  double* part = (double*)(base + w.off_part);
  *part_out = part;
  hipError_t err;
  if (!prepared && (err = launch_encode_single_prepare(d, codebook, weights, mode, ws, stream)) != hipSuccess)
    return err;
  const uint32_t n_all = (uint32_t)((size_t)d.batch * d.n_kv_heads * n_new);
  hipLaunchKernelGGL(encode_single_sweep_kernel, dim3(n_all, kSlices), dim3(kSweepThreads), 0, stream, keys,
                     (const double*)(base + w.off_wT), (const double*)(base + w.off_chalf), part, d.n_kv_heads,
                     n_new);
  return hipGetLastError();
}

hipError_t launch_encode_single(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                const float* codebook, const float* weights, int mode, bool prepared, void* codes,
                                void* ws, hipStream_t stream) {
  if (n_new == 0 || d.batch == 0) return hipSuccess;
  const EncWs w = enc_single_ws(d);
  uint8_t* base = (uint8_t*)ws;
  double* Lmat = (double*)(base + w.off_L);
  double* sd = (double*)(base + w.off_sd);
  double* czT = (double*)(base + w.off_czT);
  uint8_t* cfrag = base + w.off_cfrag;
  float* cbias = (float*)(base + w.off_cbias);
  float* cstat = (float*)(base + w.off_cstat);
  float* zbuf = (float*)(base + w.off_z);
  uint32_t* counter = (uint32_t*)(base + w.off_count);
  uint32_t* list = (uint32_t*)(base + w.off_list);
  double* part = (double*)(base + w.off_part);
  const int Hkv = d.n_kv_heads, bkv = d.batch * Hkv;
  hipError_t err;
  if (!prepared && (err = launch_encode_single_prepare(d, codebook, weights, mode, ws, stream)) != hipSuccess)
    return err;

  const uint32_t n_all = (uint32_t)((size_t)bkv * n_new);
  if (n_new <= kFewSingle) {
    hipLaunchKernelGGL(encode_single_sweep_kernel, dim3(n_all, kSlices), dim3(kSweepThreads), 0, stream, keys,
                       (const double*)(base + w.off_wT), (const double*)(base + w.off_chalf), part, Hkv, n_new);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    hipLaunchKernelGGL(encode_single_sweep_pick_kernel, dim3((n_all + 63) / 64), dim3(64), 0, stream, part,
                       (uint16_t*)codes, n_all, n_new, pos0, d.ctx_stride);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(encode_single_clear_kernel, dim3(1), dim3(1), 0, stream, counter);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (mode == A2ATS_W_BLOCK) {   // part by part: transform into the buffer, then the plain pass over it
    for (int j0 = 0; j0 < n_new; j0 += w.chunk) {
      const int n_part = n_new - j0 < w.chunk ? n_new - j0 : w.chunk;
      hipLaunchKernelGGL(encode_single_transform_kernel, dim3((n_part + 63) / 64, bkv), dim3(256), 0, stream, keys,
                         Lmat, zbuf, Hkv, n_new, j0, n_part, w.chunk);
      if ((err = hipGetLastError()) != hipSuccess) return err;
      hipLaunchKernelGGL((encode_single_kernel<A2ATS_W_NONE>), dim3((n_part + kKeysPerWG - 1) / kKeysPerWG, bkv),
                         dim3(kEncThreads), 0, stream, zbuf, sd, cfrag, cbias, cstat, (uint16_t*)codes, counter, list,
                         Hkv, n_new, pos0, d.ctx_stride, j0, n_part, (int64_t)w.chunk * kD);
      if ((err = hipGetLastError()) != hipSuccess) return err;
    }
  } else {
    const dim3 grid((n_new + kKeysPerWG - 1) / kKeysPerWG, bkv), block(kEncThreads);
    if (mode == A2ATS_W_NONE)
      hipLaunchKernelGGL((encode_single_kernel<A2ATS_W_NONE>), grid, block, 0, stream, keys, sd, cfrag, cbias, cstat,
                         (uint16_t*)codes, counter, list, Hkv, n_new, pos0, d.ctx_stride, 0, n_new, (int64_t)n_new * kD);
    else
      hipLaunchKernelGGL((encode_single_kernel<A2ATS_W_DIAG>), grid, block, 0, stream, keys, sd, cfrag, cbias, cstat,
                         (uint16_t*)codes, counter, list, Hkv, n_new, pos0, d.ctx_stride, 0, n_new, (int64_t)n_new * kD);
  }
  if ((err = hipGetLastError()) != hipSuccess) return err;
  const uint32_t re_grid = n_all < 2048u ? n_all : 2048u;
  hipLaunchKernelGGL(encode_single_recheck_kernel, dim3(re_grid), dim3(256), 0, stream, keys, mode, Lmat, sd, czT,
                     (uint16_t*)codes, counter, (const uint32_t*)list, Hkv, n_new, pos0, d.ctx_stride);
  return hipGetLastError();
}

struct SeedWs {
  size_t off_z, off_d, off_partial, off_state, bytes;
};
static SeedWs seed_ws(const a2ats_dims& d) {
  const size_t rows = (size_t)d.batch * d.n_kv_heads * (size_t)d.ctx_stride;
  SeedWs w;
  size_t o = enc_single_ws(d).bytes;
  auto take = [&](size_t bytes) {
    const size_t at = o;
    o += (bytes + 255) & ~(size_t)255;
    return at;
  };
  w.off_z = take(rows * kD * sizeof(float));
  w.off_d = take(rows * sizeof(double));
  w.off_partial = take((rows / kSeedChunk + d.n_kv_heads) * sizeof(double));
  w.off_state = take((size_t)d.n_kv_heads * sizeof(SeedState));
  w.bytes = o;
  return w;
}

size_t kmeanspp_ws_bytes(const a2ats_dims& d) { return seed_ws(d).bytes; }

hipError_t launch_kmeanspp_seed(const a2ats_dims& d, const float* keys, int n_new, const float* weights, int mode,
                                const double* u, float* codebook_out, int32_t* picks, void* ws, hipStream_t stream) {
  if (d.n_kv_heads == 0) return hipSuccess;
  const EncWs w = enc_single_ws(d);
  const SeedWs sw = seed_ws(d);
  uint8_t* base = (uint8_t*)ws;
  double* Lmat = (double*)(base + w.off_L);
  double* sd = (double*)(base + w.off_sd);
  float* cstat = (float*)(base + w.off_cstat);
  float* z = (float*)(base + sw.off_z);
  double* dmin = (double*)(base + sw.off_d);
  double* partial = (double*)(base + sw.off_partial);
  SeedState* state = (SeedState*)(base + sw.off_state);
  const int Hkv = d.n_kv_heads, bkv = d.batch * Hkv;
  const size_t factor_lds = (size_t)kD * kD * sizeof(double);
  hipError_t err = allow_dynamic_lds(encode_single_factor_kernel, factor_lds, g_factor_lds);
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(encode_single_factor_kernel, dim3(Hkv), dim3(256), factor_lds, stream, weights, mode, Lmat, sd,
                     cstat);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  if (mode == A2ATS_W_BLOCK)
    hipLaunchKernelGGL(encode_single_transform_kernel, dim3((n_new + 63) / 64, bkv), dim3(256), 0, stream, keys, Lmat,
                       z, Hkv, n_new, 0, n_new, n_new);
  else
    hipLaunchKernelGGL(scale_keys_kernel, dim3((unsigned)(((size_t)n_new * kD + 255) / 256), bkv), dim3(256), 0,
                       stream, keys, sd, z, Hkv, (size_t)n_new);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  // 4096 sequential draws: per draw one kernel over all rows (distortions to the codeword drawn
  // last) and one workgroup per KV head that turns the partial sums into the next draw
  const long rows = (long)d.batch * n_new, n_part = (rows + kSeedChunk - 1) / kSeedChunk;
  hipLaunchKernelGGL(seed_first_kernel, dim3(Hkv), dim3(128), 0, stream, keys, z, u, state, codebook_out, picks,
                     d.batch, Hkv, n_new);
  if ((err = hipGetLastError()) != hipSuccess) return err;
  for (int r = 1; r < kCW; ++r) {
    hipLaunchKernelGGL(seed_update_kernel, dim3((unsigned)((n_part + 255) / 256), Hkv), dim3(256), 0, stream, z, state,
                       dmin, partial, d.batch, Hkv, n_new, r == 1 ? 1 : 0);
    hipLaunchKernelGGL(seed_pick_kernel, dim3(Hkv), dim3(kSeedThreads), 0, stream, keys, z, u, dmin, partial, state,
                       codebook_out, picks, d.batch, Hkv, n_new, r);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  return hipSuccess;
}

}  // namespace a2ats
