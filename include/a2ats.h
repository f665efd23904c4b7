/*
 * a2ats.h -- C ABI of the MI355X (gfx950) implementation of the A2ATS decode-time
 * retrieval path (arXiv 2502.12665): windowed-RoPE query, per-subspace lookup tables,
 * code gather-sum scoring with exact top-K, selective attention over the retrieved
 * tokens plus the recent window, and the prefill-side key encoder.
 *
 * General contract
 *   - Every pointer marked [dev] is a device pointer owned by the caller; [host] is a
 *     host pointer.  The library never allocates, frees or retains memory and never
 *     synchronises: all work is enqueued on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream).  Scratch memory comes from the caller (`ws`), sized by
 *     a2ats_workspace_bytes(); its contents are undefined on entry and on return.
 *   - All arguments are validated on the host before anything is launched; on error
 *     nothing has been enqueued.  Return value: A2ATS_OK (0) or a negative a2ats_status.
 *   - Row-major layouts, last index fastest.  Query head h reads KV head h / G,
 *     G = n_q_heads / n_kv_heads.  Positions are 0-based; a sequence of n tokens has its
 *     current (query) token at position n - 1 with its key/value/code already cached.
 *   - seq_lens ([dev], nullable, int32 [B]): tokens per sequence, 0 <= seq_lens[b] <=
 *     ctx_len; NULL means every sequence has ctx_len tokens.
 *   - Supported shapes: head_dim == 128, G <= 8, ctx_len <= 2^20, top_k <= 4096, and one of
 *     two quantiser geometries:
 *       product quantisation   n_centroids == 256, sub_dim in {4, 8} (n_sub * sub_dim ==
 *                              head_dim), one uint8 code per subspace;
 *       single codebook        n_sub == 1, sub_dim == 128, n_centroids == 4096 (the paper's
 *                              own setting, section 5.1): one uint16 code per token, so every
 *                              `codes` argument is read as uint16 [B*Hkv*ctx_stride] (2-byte
 *                              aligned; its pointer type in the signatures stays uint8_t*).
 *     Anything else returns A2ATS_ERR_UNSUPPORTED.  Differences of the single-codebook
 *     geometry are stated with each call ("Single codebook:").
 *
 * Lookup-table format (shared by a2ats_build_lut and a2ats_score_topk)
 *   `lut` is one int32 array of a2ats_lut_elems() words produced by a2ats_build_lut and consumed
 *   by a2ats_score_topk.  With NG = ceil(G/4) groups of four query heads per KV head it holds
 *     exact  [B*Hq][256][M] int32            exact[b,h,c,m] = round(2^e * <q_rot[b,h,m*ds:(m+1)*ds],
 *                                            codebook[kv,m,c,:]>), inner product in float64; the
 *                                            power of two 2^e is chosen per head so that a sum of
 *                                            M entries stays below 2^30; lut_scale[b,h] = 2^-e
 *     coarse [B*Hkv*NG][M/16][256][16][4] uint16   coarse[.., c, m, r] = (exact[b,h,c,m] - min_c'
 *                                            exact[b,h,c',m]) >> s for head h = kv*G + 4*g4 + r
 *                                            (0 for heads past G); s is the smallest shift for
 *                                            which every coarse entry is <= floor(65535 / M)
 *     meta   [B*Hq][4] int32                 {sum_m min_c exact[b,h,c,m], s, sum_m max_c exact[b,h,c,m], 0}
 *   in this order.  A token's approximate score is lut_scale * sum_m exact[.., codes[j,m], m]:
 *   integer accumulation makes it independent of summation order, so equal code rows score
 *   exactly equal and ties resolve by token index.  Its coarse score sum_m coarse[.., codes[j,m],
 *   m, r] fits 16 bits and satisfies  exact = meta[0] + (coarse << s) + rem, 0 <= rem < M * 2^s,
 *   which is what lets the streaming pass filter with 16-bit arithmetic and still be exact.
 *   Single codebook: a score is one table entry, so `lut` is just [B*Hq][4096] int32 with
 *   lut[b,h,c] = the float32 value of <q_rot[b,h,:], codebook[kv,0,c,:]> (inner product in
 *   float64, rounded once) mapped to a signed integer with the same order (bits b of a float
 *   >= 0 map to b, of a float < 0 to b ^ 0x7fffffff), and lut_scale[b,h] = 1.
 */
#ifndef A2ATS_H_
#define A2ATS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct a2ats_dims {
  int32_t batch;        /* B                                        */
  int32_t n_q_heads;    /* Hq                                       */
  int32_t n_kv_heads;   /* Hkv, divides Hq                          */
  int32_t head_dim;     /* D                                        */
  int32_t n_sub;        /* M   subspaces                            */
  int32_t sub_dim;      /* ds  (M * ds == D)                        */
  int32_t n_centroids;  /* L   (256: one uint8 code per subspace)   */
  int32_t ctx_len;      /* N   tokens in the cache incl. the current one */
  int64_t ctx_stride;   /* token-axis capacity of codes / k / v, >= N    */
} a2ats_dims;

typedef enum a2ats_status {
  A2ATS_OK = 0,
  A2ATS_ERR_INVALID_ARG = -1, /* NULL required pointer, inconsistent dims, negative sizes */
  A2ATS_ERR_UNSUPPORTED = -2, /* shape outside the compiled kernel set                    */
  A2ATS_ERR_WORKSPACE = -3,   /* ws_bytes smaller than a2ats_workspace_bytes()            */
  A2ATS_ERR_HIP = -4          /* a launch failed (hipGetLastError after the launch)       */
} a2ats_status;

enum { A2ATS_F32 = 0, A2ATS_BF16 = 1 };                       /* element types of q / k / v / out */
enum { A2ATS_W_NONE = 0, A2ATS_W_DIAG = 1, A2ATS_W_BLOCK = 2 }; /* encoder distortion              */
enum { A2ATS_W_PREPARED = 0x100 };   /* flag for weight_mode, see a2ats_encode_prepare */
enum { A2ATS_OP_ENCODE = 0, A2ATS_OP_LUT = 1, A2ATS_OP_SCORE_TOPK = 2, A2ATS_OP_ATTN = 3, A2ATS_OP_FIT = 4,
       A2ATS_OP_SEED = 5 };

int a2ats_version(void);
const char* a2ats_status_string(int status);

/* Number of int32 elements of the lookup-table array for these dims (see the format above). */
size_t a2ats_lut_elems(const a2ats_dims* dims);

/* Scratch bytes `op` needs for these dims (0 if it needs none; (size_t)-1 on bad dims).  For
 * A2ATS_OP_ATTN and A2ATS_OP_SCORE_TOPK the figure covers every call with up to 64 sink tokens; a
 * call with more may need more and is refused with A2ATS_ERR_WORKSPACE if `ws` is too small. */
size_t a2ats_workspace_bytes(const a2ats_dims* dims, int op, int32_t top_k, int32_t window);

/*
 * Host helper: rotation tables for WRoPE (paper section 4.1, eq. "WRoPE"; section 2.1).
 * Dimension t is paired with t + D/2; the pair turns by position * inv_freq[t].
 *   cos_b, sin_b     [host, out, float32 D/2]          angle b * inv_freq[t]   (fixed offset b)
 *   cos_win, sin_win [host, out, float32 window * D/2] angle delta * inv_freq[t], delta = 0..window-1
 * Angles are formed and evaluated in float64 and rounded once to float32.  cos_win/sin_win
 * may be NULL when window == 0.  The caller copies the tables to the device.
 */
int a2ats_rope_tables(int32_t head_dim, const double* inv_freq, int32_t b, int32_t window,
                      float* cos_b, float* sin_b, float* cos_win, float* sin_win);

/*
 * Prefill / append-side key encoder (paper section 4.2, query-aware quantisation function
 * f'; section 2.2, f).  For every new key row and subspace m:
 *     codes[b, kv, pos0 + j, m] = argmin_c (k_m - C[kv,m,c]) H_m (k_m - C[kv,m,c])^T ,
 * lowest c on exact ties.  weight_mode selects H_m:
 *     A2ATS_W_NONE   H_m = I (plain nearest centroid), weights ignored (may be NULL)
 *     A2ATS_W_DIAG   H_m = diag(weights[kv, m*ds .. m*ds+ds-1]),  weights [dev, f32 Hkv*D], > 0
 *     A2ATS_W_BLOCK  H_m = weights[kv, m, :, :],  weights [dev, f32 Hkv*M*ds*ds], symmetric
 *                    positive definite (the ds x ds diagonal blocks of E[q^T q])
 *   keys     [dev, f32  B*Hkv*n_new*D]     pre-RoPE keys, dense (no stride)
 *   codebook [dev, f32  Hkv*M*256*ds]
 *   codes    [dev, u8   B*Hkv*ctx_stride*M] rows pos0 .. pos0+n_new-1 are written
 * Distances are evaluated in float32 and re-evaluated in float64 from the definition
 * whenever the two smallest are closer than 1e-4 relative, so codes equal the float64
 * argmin.  The weighted modes need a2ats_workspace_bytes(dims, A2ATS_OP_ENCODE, 0, 0) bytes
 * of workspace (transformed centroids); A2ATS_W_NONE needs none.  n_new == 0 is a no-op.
 * Single codebook: H is the full D x D matrix (A2ATS_W_BLOCK: weights [dev, f32 Hkv*D*D], the
 * lower triangle is read) and the argmin is over 4096 codewords of all 128 dimensions:
 * codes [dev, u16 B*Hkv*ctx_stride].  With the Cholesky factor of section 4.2 (H = L L^T,
 * z = k L, c^z = c L) the distortion is ||z - c^z||^2; the scores 1/2||c^z||^2 - z.c^z are
 * formed on the matrix cores from bf16 hi/lo splits of both operands (about 2^-18 relative),
 * and every key whose two best scores are closer than that arithmetic can tell apart is decided
 * again in float64, so codes equal the float64 argmin.  Every weight mode needs the workspace
 * (L, c^z in three forms and w = c (L L^T), 10.8 MB per KV head; a buffer of transformed keys for
 * up to 16384 rows per sequence and KV head; 8 bytes per key that ctx_stride allows); each call
 * derives them again unless weight_mode carries A2ATS_W_PREPARED (see a2ats_encode_prepare).  Up
 * to 8 keys per sequence and KV head (the decode-time append) are decided by one float64 sweep
 * each, over the expanded form 1/2||c^z||^2 - k.w of the same distortion.
 * B*Hkv*n_new must stay below 2^31.
 */
int a2ats_encode_keys(const a2ats_dims* dims, const float* keys, int32_t n_new, int32_t pos0,
                      const float* codebook, const float* weights, int weight_mode,
                      uint8_t* codes, void* ws, size_t ws_bytes, void* stream);

/*
 * The part of a2ats_encode_keys that depends on the codebook and the weights only (paper section
 * 4.2: the Cholesky factor L of H and the transformed codewords c^z = c L), for callers that
 * encode against the same codebook and weights many times (one key per decode step).  Fills the
 * codeword part of `ws`; a later a2ats_encode_keys with the same dims, codebook, weights, mode
 * and workspace may then pass weight_mode | A2ATS_W_PREPARED to skip that part (it must not have
 * used `ws` for anything else in between; a2ats_encode_keys itself leaves that part intact).
 * Product quantisation: returns A2ATS_OK without doing anything, and A2ATS_W_PREPARED is ignored
 * (the preparation there is a few microseconds).  Arguments as in a2ats_encode_keys.
 */
int a2ats_encode_prepare(const a2ats_dims* dims, const float* codebook, const float* weights,
                         int weight_mode, void* ws, size_t ws_bytes, void* stream);

/*
 * Steps 1-2 of a decode step (paper section 4.1: q~ = q R_b; section 4.2 last equation /
 * section 2.2 eq. "attention weights approximation": u^_j = q~ . c_{s_j}, tabulated per
 * subspace).
 *   q         [dev, q_dtype B*Hq*D]   pre-RoPE query of the current token
 *   cos_b/sin_b [dev, f32 D/2]        from a2ats_rope_tables
 *   codebook  [dev, f32 Hkv*M*256*ds]
 *   q_rot     [dev, out, f32 B*Hq*D]  q R_b, rotated in float64, rounded once
 *   lut       [dev, out, int32 a2ats_lut_elems()]   see "Lookup-table format" (16-byte aligned)
 *   lut_scale [dev, out, f32 B*Hq]
 * Inner products are accumulated in float64.  Needs no workspace.
 * Single codebook: codebook [dev, f32 Hkv*4096*D]; see "Lookup-table format".
 */
int a2ats_build_lut(const a2ats_dims* dims, const void* q, int q_dtype, const float* cos_b,
                    const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                    float* lut_scale, void* stream);

/*
 * a2ats_encode_keys (for n_new <= 32 keys per sequence and KV head, the decode-time append of the
 * current token's key: paper section 4.3, the GPU "assigns codewords to key states" each step) and
 * a2ats_build_lut in one launch.  The two do not depend on each other: the appended code rows are
 * at positions pos0 .. pos0 + n_new - 1.  Arguments, layouts and results are exactly those of the
 * two calls; n_new > 32 returns A2ATS_ERR_UNSUPPORTED, n_new == 0 builds the tables only (keys /
 * codes may then be NULL).  Product quantisation needs no workspace (ws may be NULL).
 * Single codebook: at most 8 keys per sequence and KV head; two launches (the float64 sweep of
 * a2ats_encode_keys' few-key route, then the table build, which also picks the codes); `ws` as for
 * a2ats_encode_keys, and weight_mode may carry A2ATS_W_PREPARED in the same way.
 */
int a2ats_decode_prologue(const a2ats_dims* dims, const float* keys, int32_t n_new, int32_t pos0,
                          const float* codebook, const float* weights, int weight_mode,
                          uint8_t* codes, const void* q, int q_dtype, const float* cos_b,
                          const float* sin_b, float* q_rot, int32_t* lut, float* lut_scale,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * a2ats_decode_prologue followed by a2ats_score_topk (without its debug output) as one call: steps
 * 1-3 of a decode step plus the append of the current token's key (paper sections 4.1-4.3).  Where
 * a2ats_score_topk takes its streaming route (product quantisation, at least 16384 candidates,
 * 1 <= top_k <= 2048, 4 top_k <= candidates) the call needs one launch less than the two: the
 * workgroups that sample the thresholds build their problem's tables themselves and keep the coarse
 * copy in LDS.  That is done while (a) those workgroups, batch * n_kv_heads * head groups * sampling
 * parts, number at most 256, one per CU, and (b) no appended row can be a candidate of any sequence,
 * pos0 >= ctx_len - window (the usual append of the current token; the sampling workgroups read
 * candidate rows while others write the appended ones).  Elsewhere it simply makes the two calls.
 * Arguments are the union of theirs and are all checked before anything is enqueued; every output
 * (codes, q_rot, lut, lut_scale, topk_*) is bit for bit what the two calls write.
 * `ws`: a2ats_workspace_bytes(dims, A2ATS_OP_SCORE_TOPK, top_k, window) bytes for product
 * quantisation (the prologue needs none there), a2ats_workspace_bytes(dims, A2ATS_OP_ENCODE, 0, 0)
 * for the single codebook (its selection needs none).
 */
int a2ats_decode_select(const a2ats_dims* dims, const float* keys, int32_t n_new, int32_t pos0,
                        const float* codebook, const float* weights, int weight_mode, uint8_t* codes,
                        const void* q, int q_dtype, const float* cos_b, const float* sin_b,
                        float* q_rot, int32_t* lut, float* lut_scale, int32_t top_k, int32_t window,
                        int32_t n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                        int32_t* topk_count, float* topk_score, void* ws, size_t ws_bytes,
                        void* stream);

/*
 * Step 3 of a decode step: approximate scores for every cached token by gather-summing
 * table entries through its codes, then exact top-K (paper section 4: "retrieves the
 * top-K tokens with the highest attention scores").  For sequence b with n tokens the
 * candidates are positions [sink_end, n - window), sink_end = min(n_sink, max(0, n - window)):
 * sinks and the recent window are always attended and never compete.  Selection is per
 * query head; equal scores go to the lower position.
 *   codes      [dev, u8 B*Hkv*ctx_stride*M]
 *   lut, lut_scale   from a2ats_build_lut
 *   topk_idx   [dev, out, int32 B*Hq*top_k]  selected positions in ascending order;
 *                                            slots past topk_count are -1
 *   topk_count [dev, out, int32 B*Hq]        K' = min(top_k, #candidates)
 *   topk_score [dev, out, nullable, f32 B*Hq*top_k] score of each selected position
 *   scores_out [dev, out, nullable, f32 B*Hq*ctx_stride] debug: every token's score
 *              (positions >= n are not written)
 * top_k == 0 is allowed.  window >= 0, n_sink >= 0.
 * Single codebook: codes [dev, u16 B*Hkv*ctx_stride]; a score is the table entry of the token's
 * code, there are at most 4096 distinct scores per head and ties (by position) decide most
 * selections; needs no workspace (a2ats_workspace_bytes returns 0) and lut_scale is not read.
 */
int a2ats_score_topk(const a2ats_dims* dims, const uint8_t* codes, const int32_t* lut,
                     const float* lut_scale, int32_t top_k, int32_t window, int32_t n_sink,
                     const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                     float* topk_score, float* scores_out, void* ws, size_t ws_bytes,
                     void* stream);

/*
 * Step 4: exact attention over S = sinks U top-K U window (paper section 2.1 eq. "output
 * state" restricted to S; section 4.1 eq. "WRoPE").  With i = n - 1:
 *     logit_j = q R_{i-j} k_j^T / sqrt(D)   for i - j <  window
 *     logit_j = q R_b     k_j^T / sqrt(D)   otherwise (q R_b = q_rot)
 *     out     = sum_{j in S} softmax(logit)_j v_j
 * Keys are the exact pre-RoPE keys.  float32 accumulation; out is rounded once to kv_dtype.
 *   q        [dev, kv_dtype B*Hq*D]      q_rot [dev, f32 B*Hq*D]
 *   k_cache, v_cache [dev, kv_dtype B*Hkv*ctx_stride*D]
 *   topk_idx [dev, int32 B*Hq*top_k], topk_count [dev, int32 B*Hq]  (every index must be a
 *            candidate position of its sequence; the kernels do not re-check)
 *   cos_win/sin_win [dev, f32 window*D/2] from a2ats_rope_tables (may be NULL if window == 0)
 *   out      [dev, out, kv_dtype B*Hq*D]  (zeros for an empty sequence)
 */
int a2ats_sparse_attn(const a2ats_dims* dims, const void* q, const float* q_rot,
                      const void* k_cache, const void* v_cache, int kv_dtype,
                      const int32_t* topk_idx, const int32_t* topk_count, int32_t top_k,
                      int32_t window, int32_t n_sink, const float* cos_win, const float* sin_win,
                      const int32_t* seq_lens, void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * a2ats_sparse_attn for callers that cannot allocate or pass scratch memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the partial attention states that
 * a2ats_sparse_attn keeps in `ws` live in an 8 MiB array inside the library instead (one per GPU the
 * library runs on, held until the process ends).  The call allocates nothing.  Arguments and results
 * are those of a2ats_sparse_attn without `ws` / `ws_bytes`.  A shape whose
 * a2ats_workspace_bytes(dims, A2ATS_OP_ATTN, ...) figure for this n_sink exceeds 8 MiB is refused with
 * A2ATS_ERR_WORKSPACE before anything is enqueued (at 520 bytes per query head and workgroup, that is
 * beyond every shape of section 5: 0.7 MB at batch 4 x 32 heads, 1.4 MB at batch 32 x 28 heads).
 * Every call on a GPU uses that GPU's array: calls that overlap in time on one GPU (different
 * streams, different threads) race and must be serialised by the caller.  Nothing in the array has
 * to start at zero: every state a call reads has been written by the same call.
 */
int a2ats_sparse_attn_static(const a2ats_dims* dims, const void* q, const float* q_rot,
                             const void* k_cache, const void* v_cache, int kv_dtype,
                             const int32_t* topk_idx, const int32_t* topk_count, int32_t top_k,
                             int32_t window, int32_t n_sink, const float* cos_win, const float* sin_win,
                             const int32_t* seq_lens, void* out, void* stream);

/*
 * a2ats_sparse_attn over a PAGED key/value cache: k_pool / v_pool are pools of pages,
 *   [dev, kv_dtype n_pages * Hkv * page_size * D], page p holding page_size consecutive tokens of one
 *   sequence for all KV heads ([Hkv][page_size][D]), and
 *   page_table [dev, int32 B * ceil(ctx_stride / page_size)] maps (sequence b, token j) to page
 *   page_table[b][j / page_size] (row j % page_size of it).  page_size: a power of two >= 16.
 * Every page number reachable through seq_lens / ctx_len must be a valid page of the pools (not
 * checked on the device).  (a2ats_score_topk_paged reads a code matrix paged the same way.)
 * Everything else as a2ats_sparse_attn; results are identical to the
 * contiguous layout.
 */
int a2ats_sparse_attn_paged(const a2ats_dims* dims, const void* q, const float* q_rot, const void* k_pool,
                            const void* v_pool, int kv_dtype, const int32_t* page_table,
                            int32_t page_size, const int32_t* topk_idx, const int32_t* topk_count,
                            int32_t top_k, int32_t window, int32_t n_sink, const float* cos_win,
                            const float* sin_win, const int32_t* seq_lens, void* out, void* ws,
                            size_t ws_bytes, void* stream);

/*
 * a2ats_score_topk over a PAGED code matrix (section 4.3 keeps the codes beside the key/value cache;
 * serving stacks keep that cache in pages): code_pool [dev, uint8 n_pages * Hkv * page_size * M] holds
 * pages of page_size consecutive tokens of one sequence for all KV heads ([Hkv][page_size][M]), and
 * page_table [dev, int32 B * ceil(ctx_stride / page_size)] maps (sequence b, token j) to page
 * page_table[b][j / page_size] (row j % page_size of it) -- the table and page size of
 * a2ats_sparse_attn_paged.  page_size: a power of two >= 16.  Every page number reachable through
 * seq_lens / ctx_len must be a valid page of the pool (not checked on the device).  Product-quantised
 * codes only (n_sub 16 or 32; the single-codebook geometry returns A2ATS_ERR_UNSUPPORTED).  Everything
 * else as a2ats_score_topk (same workspace size, same outputs, scores_out stays [B*Hq][ctx_stride]);
 * results are identical to the contiguous layout.
 */
int a2ats_score_topk_paged(const a2ats_dims* dims, const uint8_t* code_pool, const int32_t* page_table,
                           int32_t page_size, const int32_t* lut, const float* lut_scale, int32_t top_k,
                           int32_t window, int32_t n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                           int32_t* topk_count, float* topk_score, float* scores_out, void* ws, size_t ws_bytes,
                           void* stream);

/*
 * Append path of the paged code matrix: copy the code rows of n_new freshly encoded tokens,
 * new_codes [dev, uint8 B * Hkv * n_new * M] (what a2ats_encode_keys writes for dims with
 * ctx_stride = n_new and pos0 = 0), to tokens pos0 .. pos0 + n_new - 1 of every sequence in code_pool
 * through page_table (layouts as in a2ats_score_topk_paged).  pos0 + n_new <= ctx_stride.
 */
int a2ats_codes_to_pages(const a2ats_dims* dims, const uint8_t* new_codes, int32_t n_new, int32_t pos0,
                         uint8_t* code_pool, const int32_t* page_table, int32_t page_size, void* stream);

/*
 * a2ats_sparse_attn on the HOST CPU, for a key/value cache kept in host memory (the placement of
 * section 4.3: the GPU scores and selects, the CPU attends over the retrieved tokens next to the
 * cache, and only indices, queries and outputs cross the bus).  Same function and arguments as
 * a2ats_sparse_attn, except that EVERY pointer is a host pointer (q, q_rot, k_cache, v_cache,
 * topk_idx, topk_count, cos_win, sin_win, seq_lens, out), there is no workspace and no stream: the
 * call runs on n_threads OpenMP threads (0 = the runtime's default) and returns when `out` is
 * written.  It never touches a GPU and is not a fallback of anything: no other entry point calls it.
 * float32 accumulation; AVX2 + FMA inner loops when the CPU has them, scalar otherwise.  head_dim 128.
 */
int a2ats_sparse_attn_host(const a2ats_dims* dims, const void* q, const float* q_rot, const void* k_cache,
                           const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                           const int32_t* topk_count, int32_t top_k, int32_t window, int32_t n_sink,
                           const float* cos_win, const float* sin_win, const int32_t* seq_lens, void* out,
                           int32_t n_threads);

/*
 * Selection shared by the query heads of a KV head (grouped-query attention; the paper selects
 * "for each attention head" and does not say which kind, so per query head is the reading of the
 * calls above and this is the alternative): the group's score of a token is the SUM over the G
 * query heads of the approximate scores of section 4.2, sum_g q~_g . c_{s_j} = (sum_g q~_g) . c_{s_j};
 * one top-K per KV head; all G heads attend the same retrieved rows, which are then fetched from
 * HBM once per KV head instead of once per query head.
 *   a2ats_build_lut_shared   as a2ats_build_lut, but `lut` / `lut_scale` describe ONE table head per
 *                            KV head, built from the float32 sum of the G rotated queries: they have
 *                            the format and size of a2ats_build_lut for dims with n_q_heads set to
 *                            n_kv_heads (lut_scale [B*Hkv]).  q_rot is still [B*Hq*D], per head.
 *   a2ats_score_topk         is then called with those dims (n_q_heads = n_kv_heads):
 *                            topk_idx [B*Hkv*top_k], topk_count [B*Hkv].
 *   a2ats_sparse_attn_shared as a2ats_sparse_attn with the real dims, topk_idx / topk_count per KV
 *                            head as above; workspace as A2ATS_OP_ATTN.
 *   a2ats_decode_select_shared  a2ats_encode_keys (the append of up to 32 keys per sequence and KV head)
 *                            + a2ats_build_lut_shared + a2ats_score_topk with those dims, as one call
 *                            (what a2ats_decode_select is for the per-head selection: on the streaming
 *                            route, with at most 256 sampling workgroups = batch * n_kv_heads * sampling
 *                            parts and pos0 >= ctx_len - window, one launch does the append, the
 *                            tables and the threshold sampling; elsewhere the three launches follow
 *                            each other).  `dims` are the real ones; lut, lut_scale, topk_* and `ws`
 *                            (a2ats_workspace_bytes(.., A2ATS_OP_SCORE_TOPK, ..)) are those of dims with
 *                            n_q_heads = n_kv_heads.  Every output is bit for bit what the three calls
 *                            write.  Product quantisation only (A2ATS_ERR_UNSUPPORTED otherwise).
 * The other three serve both quantiser geometries.
 */
int a2ats_build_lut_shared(const a2ats_dims* dims, const void* q, int q_dtype, const float* cos_b,
                           const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                           float* lut_scale, void* stream);
int a2ats_sparse_attn_shared(const a2ats_dims* dims, const void* q, const float* q_rot,
                             const void* k_cache, const void* v_cache, int kv_dtype,
                             const int32_t* topk_idx, const int32_t* topk_count, int32_t top_k,
                             int32_t window, int32_t n_sink, const float* cos_win,
                             const float* sin_win, const int32_t* seq_lens, void* out, void* ws,
                             size_t ws_bytes, void* stream);
int a2ats_decode_select_shared(const a2ats_dims* dims, const float* keys, int32_t n_new, int32_t pos0,
                               const float* codebook, const float* weights, int weight_mode,
                               uint8_t* codes, const void* q, int q_dtype, const float* cos_b,
                               const float* sin_b, float* q_rot, int32_t* lut, float* lut_scale,
                               int32_t top_k, int32_t window, int32_t n_sink, const int32_t* seq_lens,
                               int32_t* topk_idx, int32_t* topk_count, float* topk_score, void* ws,
                               size_t ws_bytes, void* stream);

/*
 * Offline codebook construction (paper section 4.2).
 *
 * a2ats_second_moment: H = E[q~^T q~], one D x D matrix per KV head, from n_samples rotated query
 * rows; the G query heads of a KV head are pooled.
 *   q_rot  [dev, f32 n_samples*Hq*D]   rotated queries (e.g. the q_rot output of a2ats_build_lut)
 *   h_out  [dev, out, f32 Hkv*D*D]     accumulated in float64, rounded once; zeros if n_samples == 0
 * H (or its diagonal / diagonal blocks) is the `weights` argument of a2ats_encode_keys.
 *
 * a2ats_codebook_update: the centroid step of k-means under the query-aware distortion.  The paper
 * runs k-means on z = k L and maps the centroids back with L^-1; the mean is linear, so the new
 * codeword is the mean of the keys assigned to it.  One Lloyd iteration is a2ats_encode_keys (the
 * assignment under (k - c) H (k - c)^T) followed by this call on the same keys and codes.
 *   keys, n_new, pos0, codes   as written by a2ats_encode_keys (all B sequences are pooled per KV head)
 *   codebook      [dev, f32 Hkv*M*L*ds]       the codebook the codes refer to
 *   codebook_out  [dev, out, f32 Hkv*M*L*ds]  means in float64, rounded once; a codeword without keys
 *                                             keeps its value (may alias `codebook`)
 *   counts        [dev, out, nullable, int32 Hkv*M*L]  keys per codeword
 * The sums are float64 hardware atomics: the last bits of a mean can differ from run to run.
 * Both calls need a2ats_workspace_bytes(dims, A2ATS_OP_FIT, 0, 0) bytes of workspace.
 */
/*
 * k-means++ seeding of a single codebook under the query-aware distortion (section 4.2 initialises
 * its k-means with k-means++).  The keys of all B sequences are pooled per KV head (row i = b*n_new
 * + j); codeword 0 is row min(rows - 1, floor(u[kv,0] * rows)); codeword r > 0 is the first row whose
 * inclusive prefix sum of d exceeds u[kv,r] * sum(d) (so row i is drawn with probability d_i / sum(d)), d_i being the distortion of row i to the nearest
 * codeword chosen so far, (k - c) H (k - c)^T evaluated as ||z_i - z_c||^2 in float64 over z = k L
 * rounded once to float32 (if every d is zero: row floor(u * rows)).
 *   keys, weights, weight_mode   as in a2ats_encode_keys, 1 <= n_new <= ctx_stride
 *   u             [dev, f64 Hkv*4096]      uniform numbers in [0, 1) supplied by the caller
 *   codebook_out  [dev, out, f32 Hkv*4096*D] the chosen keys
 *   picks         [dev, out, nullable, int32 Hkv*4096] their row numbers
 * Workspace a2ats_workspace_bytes(dims, A2ATS_OP_SEED, 0, 0).  One workgroup per KV head runs the 4096
 * sequential draws (one update and one pick launch per draw): meant for calibration sets of up to ~10^5 keys per KV head.  Single codebook only.
 */
int a2ats_kmeanspp_seed(const a2ats_dims* dims, const float* keys, int32_t n_new, const float* weights,
                        int weight_mode, const double* u, float* codebook_out, int32_t* picks, void* ws,
                        size_t ws_bytes, void* stream);
int a2ats_second_moment(const a2ats_dims* dims, const float* q_rot, int64_t n_samples, float* h_out,
                        void* ws, size_t ws_bytes, void* stream);
int a2ats_codebook_update(const a2ats_dims* dims, const float* keys, int32_t n_new, int32_t pos0,
                          const uint8_t* codes, const float* codebook, float* codebook_out,
                          int32_t* counts, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Diagnostics and profiling aids.  None of these is part of the method; nothing above needs them.
 * ------------------------------------------------------------------------------------------------ */

/*
 * After an a2ats_score_topk call with the same dims / top_k / window / n_sink and the same `ws`,
 * write per head into cand_counts [dev, out, uint32 B*Hq] (asynchronously, on `stream`): bits 0-27
 * the number of rows the streaming pass kept for that head, bits 28-31 the route the final kernel
 * took (0 = fast; 1 = too few survivors, 2 = too many, 3 = a segment overflowed, 4 = completeness
 * proof failed: 1-4 end in the exact fallback).  For shapes served by the exact route alone every
 * entry is 0xFFFFFFFF.
 */
int a2ats_score_topk_stats(const a2ats_dims* dims, int32_t top_k, int32_t window, int32_t n_sink,
                           const void* ws, uint32_t* cand_counts, void* stream);

/*
 * Host only, no GPU needed: how a2ats_score_topk would lay out its work for these dims / top_k /
 * window / n_sink.  Writes 11 numbers to plan [host, out, int32 11]:
 * [0] 1 if the sampled-threshold + streaming route is used (0: the exact route alone, the rest is 0),
 * [1] groups of four query heads per KV head, [2] sampling workgroups per (sequence, KV head, group),
 * [3] rows each of them scores, [4] streaming workgroups (chunks) per problem, [5] rows per chunk,
 * [6] survivor segments per wave of a chunk (always 1), [7] rows per segment, [8] entries a segment can hold,
 * [9] survivors per head the final kernel can hold, [10] workspace bytes the call needs, divided by 256.
 */
int a2ats_score_topk_plan(const a2ats_dims* dims, int32_t top_k, int32_t window, int32_t n_sink, int32_t* plan);

/*
 * a2ats_score_topk with a pair of events (hipEvent_t passed as void*, both non-NULL, created by the
 * caller) attached to the dispatch of the code-streaming kernel on `stream`, so that the elapsed
 * time between them is that kernel's own duration.  Everything else as a2ats_score_topk; the events
 * are only used where the streaming route runs.  No state is kept between calls.
 */
int a2ats_score_topk_profiled(const a2ats_dims* dims, const uint8_t* codes, const int32_t* lut,
                              const float* lut_scale, int32_t top_k, int32_t window, int32_t n_sink,
                              const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                              float* topk_score, float* scores_out, void* ws, size_t ws_bytes,
                              void* stream, void* ev_start, void* ev_stop);

#ifdef __cplusplus
}
#endif
#endif /* A2ATS_H_ */
