// Shared device helpers for the gfx950 kernels: wave64 lane utilities, block scans and the
// rank search over an LDS histogram used by every selection stage.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "a2ats.h"

namespace a2ats {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kCentroids = 256;    // one uint8 code per subspace
constexpr int kHeadsPerGroup = 4;  // query heads served by one 16-byte table entry
constexpr int kHistBins = 2048;

__device__ __forceinline__ int lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Number of set bits of `mask` below the calling lane.
__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Word offsets (int32 units) of the three parts of the lookup-table blob, see a2ats.h.
struct LutLayout {
  size_t off_exact;   // [B*Hq][256][M] int32
  size_t off_coarse;  // [B*Hkv*NG][M/16][256][16] x 4 uint16
  size_t off_meta;    // [B*Hq][4] int32: {sum of subspace minima, shift, sum of subspace maxima, 0}
  size_t total;
};
__host__ __device__ inline LutLayout lut_layout(int B, int Hq, int Hkv, int M) {
  const int G = Hq / Hkv, NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  const size_t heads = (size_t)B * Hq, probs = (size_t)B * Hkv * NG;
  LutLayout l;
  l.off_exact = 0;
  l.off_coarse = heads * M * kCentroids;
  l.off_meta = l.off_coarse + probs * kCentroids * M * 2;
  l.total = l.off_meta + heads * 4;
  return l;
}

// Integer score -> unsigned key with the same order.
__device__ __forceinline__ uint32_t score_key(int32_t s) { return (uint32_t)s ^ 0x80000000u; }
__device__ __forceinline__ int32_t key_score(uint32_t k) { return (int32_t)(k ^ 0x80000000u); }

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (a shuffle
// goes through the LDS crossbar, one round trip per step, and these scans sit on critical paths):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of rows 0 and 2 is added
// to rows 1 and 3, then lane 31 to the upper half.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);   // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);   // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);   // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31
  return v;
}

// Maximum over the 64 lanes of a wave, valid in lane 63 (same moves as wave_inclusive_scan).
__device__ __forceinline__ uint32_t wave_max_to_last_lane(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false));
  return v;
}

// Sum / bitwise OR over aligned groups of 8 lanes, result in every lane of the group (swaps inside
// quads, then the mirror image within 8 lanes).
__device__ __forceinline__ int32_t group8_sum(int32_t v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);   // row_half_mirror
  return v;
}
__device__ __forceinline__ int32_t group8_or(int32_t v) {
  v |= __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);
  v |= __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);
  v |= __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);
  return v;
}

// Exclusive prefix sum of `v` over the block (NT threads, NT a multiple of 64).  `s_wave` is an
// LDS array of NT/64 words owned by this call site.  Returns the exclusive prefix and the
// block total.  One barrier; callers alternate between two `s_wave` arrays when they scan
// repeatedly so that a second barrier is not needed.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* s_wave,
                                                         uint32_t& total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint32_t inc = wave_inclusive_scan(v);
  if (lane == 63) s_wave[wv] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) {
    uint32_t w = s_wave[i];
    if (i < wv) base += w;
    tot += w;
  }
  total = tot;
  return base + inc - v;
}

// Rank search over a histogram of NB bins, scanning from the highest bin down: finds the bin
// T with  sum_{bin > T} count < k <= sum_{bin >= T} count  (1 <= k <= sum of all bins).
// `count(bin)` reads one bin (normally from LDS).  s_res[0] = T, s_res[1] = sum_{bin > T}.
// Two barriers; every thread of the block must call it.  s_wave: NT/64 words of LDS,
// s_res: 2 words of LDS.
template <int NT, int NB, typename Count>
__device__ __forceinline__ void block_find_rank_desc(Count count, uint32_t k, uint32_t* s_wave,
                                                     uint32_t* s_res) {
  static_assert(NB % NT == 0, "bins must divide evenly over the block");
  constexpr int PER = NB / NT;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int top = NB - 1 - (int)threadIdx.x * PER;
  uint32_t loc[PER];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    loc[i] = count(top - i);
    sum += loc[i];
  }
  uint32_t inc = wave_inclusive_scan(sum);
  if (lane == 63) s_wave[wv] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int i = 0; i < wv; ++i) base += s_wave[i];
  inc += base;
  uint32_t run = inc - sum;
  if (run < k && k <= inc) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      if (run + loc[i] >= k) {
        s_res[0] = (uint32_t)(top - i);
        s_res[1] = run;
        break;
      }
      run += loc[i];
    }
  }
  __syncthreads();
}

// Workgroups are dealt to the 8 XCDs (each with its own L2) round-robin by linear workgroup id.
// Map a linear id to (problem, part) so that every part of a problem runs on XCD (problem % 8):
// the table that kernel k wrote or read for a problem is then in the L2 that kernel k+1's
// workgroups for the same problem use.  Falls back to the plain order when the number of
// problems is not a multiple of 8.
__device__ __forceinline__ void xcd_map(int linear, int parts, int problems, int& problem, int& part) {
  if ((problems & 7) == 0) {
    const int xcd = linear & 7, slot = linear >> 3;
    problem = (slot / parts) * 8 + xcd;
    part = slot % parts;
  } else {
    problem = linear / parts;
    part = linear % parts;
  }
}

// The same for problems that come in sets of `ng` reading the same rows (the head groups of one KV
// head, problem = kv_problem * ng + g): all parts of all ng problems of a set run on XCD
// (kv_problem % 8), and the ng workgroups that stream the same part are neighbours in the launch
// order, so the rows come from HBM once and from that XCD's L2 for the others.
__device__ __forceinline__ void xcd_map_sets(int linear, int parts, int problems, int ng, int& problem, int& part) {
  if (ng > 1 && problems % (8 * ng) == 0) {
    const int xcd = linear & 7, slot = linear >> 3;
    const int unit = slot / (parts * ng), inner = slot % (parts * ng);
    problem = (unit * 8 + xcd) * ng + inner % ng;
    part = inner / ng;
  } else {
    xcd_map(linear, parts, problems, problem, part);
  }
}

// Division of small block-index-sized numbers by a launch constant without the ~35-instruction
// software division (which every wave of a workgroup would run before its first load):
// n / d = umulhi(n, 2^32 / d + 1), exact while n * d < 2^32.
struct FastDiv {
  uint32_t d, m;
};
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d < 1u ? 1u : d;
  f.m = f.d == 1u ? 0u : (uint32_t)((1ull << 32) / f.d + 1ull);
  return f;
}
__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f) { return f.d == 1u ? n : __umulhi(n, f.m); }

// xcd_map / xcd_map_sets with the divisions prepared on the host, plus the split of a problem
// index ((b * Hkv + kv) * NG + g4) into its parts.  All indices stay far below the 2^32 / d limit
// (workgroups per launch <= 2^20, divisors <= 2^11).
struct GridMap {
  FastDiv parts, ng, parts_ng, hkv;
  int mode;   // 0: linear = problem * parts + part; 1: xcd_map; 2: xcd_map_sets
};
inline GridMap make_grid_map(int parts, int problems, int ng, int hkv) {
  GridMap g;
  g.parts = make_fastdiv((uint32_t)parts);
  g.ng = make_fastdiv((uint32_t)ng);
  g.parts_ng = make_fastdiv((uint32_t)(parts * ng));
  g.hkv = make_fastdiv((uint32_t)hkv);
  g.mode = (ng > 1 && problems % (8 * ng) == 0) ? 2 : ((problems & 7) == 0 ? 1 : 0);
  return g;
}
__device__ __forceinline__ void map_block(uint32_t linear, const GridMap& gm, int& problem, int& part) {
  if (gm.mode == 2) {
    const uint32_t xcd = linear & 7u, slot = linear >> 3;
    const uint32_t unit = fast_div(slot, gm.parts_ng), inner = slot - unit * gm.parts_ng.d;
    const uint32_t pt = fast_div(inner, gm.ng);
    problem = (int)((unit * 8u + xcd) * gm.ng.d + (inner - pt * gm.ng.d));
    part = (int)pt;
  } else if (gm.mode == 1) {
    const uint32_t xcd = linear & 7u, slot = linear >> 3;
    const uint32_t q = fast_div(slot, gm.parts);
    problem = (int)(q * 8u + xcd);
    part = (int)(slot - q * gm.parts.d);
  } else {
    const uint32_t q = fast_div(linear, gm.parts);
    problem = (int)q;
    part = (int)(linear - q * gm.parts.d);
  }
}
__device__ __forceinline__ void split_problem(int prob, const GridMap& gm, int& b, int& kv, int& g4) {
  const uint32_t bkv = fast_div((uint32_t)prob, gm.ng);
  g4 = (int)((uint32_t)prob - bkv * gm.ng.d);
  const uint32_t bb = fast_div(bkv, gm.hkv);
  b = (int)bb;
  kv = (int)(bkv - bb * gm.hkv.d);
}

// Per-sequence geometry of the candidate range (sinks and window never compete).
struct SeqRange {
  int n;          // tokens in the sequence
  int win_start;  // first window position
  int sink_end;   // one past the last sink
  int ncand;      // win_start - sink_end
  int kk;         // min(top_k, ncand)
};

__device__ __forceinline__ SeqRange seq_range(int ctx_len, const int32_t* seq_lens, int b,
                                              int window, int n_sink, int top_k) {
  SeqRange r;
  r.n = seq_lens ? seq_lens[b] : ctx_len;
  r.n = r.n < 0 ? 0 : (r.n > ctx_len ? ctx_len : r.n);
  r.win_start = r.n - window > 0 ? r.n - window : 0;
  r.sink_end = n_sink < r.win_start ? n_sink : r.win_start;
  r.ncand = r.win_start - r.sink_end;
  r.kk = top_k < r.ncand ? top_k : r.ncand;
  return r;
}

// Optional paging of the code matrix.  With `table` set, `codes` is a pool of pages
// [page][Hkv][page_size][M] (page_size = 1 << shift tokens of one sequence, all KV heads) and
// table[b * pages_per_seq + (j >> shift)] names the page that holds token j of sequence b;
// with `table` null the matrix is contiguous, [B][Hkv][ctx_stride][M].
struct CodePages {
  const int32_t* table;
  int32_t pages_per_seq;
  int32_t shift;
};
// The code rows of one (sequence, KV head).
struct SeqCodes {
  const uint8_t* base;    // contiguous: row 0; paged: the KV head's rows inside page 0 of the pool
  const int32_t* pages;   // paged: the sequence's page numbers (else null)
  uint32_t shift, mask;   // token -> (page slot j >> shift, row j & mask)
  size_t page_bytes;      // bytes from a page to the next
};
template <int M>
__device__ __forceinline__ SeqCodes seq_codes_of(const uint8_t* codes, const CodePages& pg, int b, int kv, int Hkv,
                                                 int64_t ctx_stride) {
  SeqCodes s;
  if (pg.table == nullptr) {
    s.base = codes + ((size_t)b * Hkv + kv) * (size_t)ctx_stride * M;
    s.pages = nullptr;
    s.shift = 0;
    s.mask = 0;
    s.page_bytes = 0;
  } else {
    s.base = codes + ((size_t)kv << pg.shift) * M;
    s.pages = pg.table + (size_t)b * pg.pages_per_seq;
    s.shift = (uint32_t)pg.shift;
    s.mask = (1u << pg.shift) - 1u;
    s.page_bytes = ((size_t)Hkv << pg.shift) * M;
  }
  return s;
}
// Row j given the number of its page (paged layout only).
template <int M>
__device__ __forceinline__ const uint8_t* row_in_page(const SeqCodes& s, int page, int j) {
  return s.base + (size_t)page * s.page_bytes + (size_t)((uint32_t)j & s.mask) * M;
}
template <int M>
__device__ __forceinline__ const uint8_t* row_ptr(const SeqCodes& s, int j) {
  if (s.pages == nullptr) return s.base + (size_t)j * M;
  return row_in_page<M>(s, s.pages[(uint32_t)j >> s.shift], j);
}

// 16-byte load that tells the caches the line will not be reused (streamed data).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream_u4(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Round-to-nearest-even float -> bf16 (finite inputs; NaN is kept a NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace a2ats
