"""ctypes wrapper around the plain-C CPU oracle (oracle/a2ats_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing under the product package imports it,
and it imports nothing from the product package.

All wrappers take torch CPU tensors (or anything np.asarray accepts), widen
float inputs to float32 exactly (bf16 -> f32 is exact) and return numpy arrays
in float64 / int32 / uint8.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "a2ats_oracle.c")
_LIB = os.path.join(_HERE, "liba2ats_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math) into oracle/liba2ats_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def threads() -> int:
    return int(_load().a2ats_oracle_threads())


def _f32(x) -> np.ndarray:
    if hasattr(x, "detach"):
        import torch
        x = x.detach().to("cpu").to(torch.float32).numpy()
    return np.ascontiguousarray(x, dtype=np.float32)


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):
        import torch
        x = x.detach().to("cpu").to(torch.float64).numpy()
    return np.ascontiguousarray(x, dtype=np.float64)


def _codes(x) -> np.ndarray:
    """Codes as a contiguous uint8 or uint16 array (uint16 for codebooks of more than 256 codewords)."""
    if hasattr(x, "detach"):
        import torch
        x = x.detach().to("cpu")
        x = x.view(torch.int16).numpy().view(np.uint16) if x.dtype in (torch.int16, torch.uint16) else x.numpy()
    x = np.asarray(x)
    assert x.dtype in (np.uint8, np.uint16), x.dtype
    return np.ascontiguousarray(x)


def _u8(x) -> np.ndarray:
    if hasattr(x, "detach"):
        x = x.detach().to("cpu").numpy()
    return np.ascontiguousarray(x, dtype=np.uint8)


def _i32(x) -> Optional[np.ndarray]:
    if x is None:
        return None
    if hasattr(x, "detach"):
        x = x.detach().to("cpu").numpy()
    return np.ascontiguousarray(x, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


_I = ctypes.c_int
_L = ctypes.c_int64
_D = ctypes.c_double


def rope(x, inv_freq, pos: float) -> np.ndarray:
    """x R_pos for every row of x [..., D] (section 2.1)."""
    x = _f32(x)
    D = x.shape[-1]
    out = np.empty(x.shape, dtype=np.float64)
    inv = _f64(inv_freq)
    _load().a2ats_oracle_rope(_p(x), _L(x.size // D), _I(D), _p(inv), _D(float(pos)), _p(out))
    return out


def lut(q_rot, codebook, n_q_heads: int) -> np.ndarray:
    """[B,Hq,M,L] float64 table of q~ . centroid per subspace."""
    q_rot = _f64(q_rot)
    cb = _f32(codebook)
    B, Hq, D = q_rot.shape
    Hkv, M, L, ds = cb.shape
    assert Hq == n_q_heads and M * ds == D
    out = np.empty((B, Hq, M, L), dtype=np.float64)
    _load().a2ats_oracle_lut(_p(q_rot), _p(cb), _I(B), _I(Hq), _I(Hkv), _I(M), _I(L), _I(ds), _p(out))
    return out


def scores_explicit(q_rot, codebook, codes, n_ctx: int) -> np.ndarray:
    """[B,Hq,N] approximate scores q~ . k^_j by explicit reconstruction."""
    q_rot = _f64(q_rot)
    cb = _f32(codebook)
    codes = _codes(codes)
    B, Hq, D = q_rot.shape
    Hkv, M, L, ds = cb.shape
    S = codes.shape[2]
    assert codes.shape == (B, Hkv, S, M) and n_ctx <= S
    out = np.empty((B, Hq, n_ctx), dtype=np.float64)
    _load().a2ats_oracle_scores_explicit(_p(q_rot), _p(cb), _p(codes), _I(codes.itemsize), _I(B), _I(Hq), _I(Hkv), _I(M),
                                         _I(L), _I(ds), _L(n_ctx), _L(S), _p(out))
    return out


def scores_lut(lut_, codes, n_kv_heads: int, n_ctx: int) -> np.ndarray:
    lut_ = _f64(lut_)
    codes = _codes(codes)
    B, Hq, M, L = lut_.shape
    S = codes.shape[2]
    out = np.empty((B, Hq, n_ctx), dtype=np.float64)
    _load().a2ats_oracle_scores_lut(_p(lut_), _p(codes), _I(codes.itemsize), _I(B), _I(Hq), _I(n_kv_heads), _I(M), _I(L),
                                    _L(n_ctx), _L(S), _p(out))
    return out


def group_scores(scores, n_kv_heads: int) -> np.ndarray:
    """[B,Hkv,N]: the scores of the G query heads of each KV head added up (grouped-query
    attention with one selection per KV head; section 4 selects per attention head and leaves
    the grouped case open -- the sum is this build's reading, stated in the design notes).
    Query head h belongs to KV head h // G."""
    s = _f64(scores)
    B, Hq, N = s.shape
    G = Hq // n_kv_heads
    out = np.zeros((B, n_kv_heads, N), dtype=np.float64)
    for g in range(G):                       # plain left-to-right sum over the group
        out += s[:, [kv * G + g for kv in range(n_kv_heads)], :]
    return out


def topk(scores, top_k: int, window: int, n_sink: int = 0, seq_lens=None
         ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Full-sort top-K: (idx [B,Hq,K] ascending / -1 padded, count [B,Hq], kth score [B,Hq])."""
    scores = _f64(scores)
    B, Hq, N = scores.shape
    sl = _i32(seq_lens)
    idx = np.empty((B, Hq, max(top_k, 0)), dtype=np.int32)
    cnt = np.empty((B, Hq), dtype=np.int32)
    kth = np.empty((B, Hq), dtype=np.float64)
    _load().a2ats_oracle_topk(_p(scores), _I(B), _I(Hq), _L(N), _I(top_k), _I(window), _I(n_sink),
                              _p(sl), _p(idx), _p(cnt), _p(kth))
    return idx, cnt, kth


def sparse_attn(q, k, v, topk_idx, topk_count, n_ctx: int, window: int, n_sink: int, inv_freq,
                b_off: float, seq_lens=None) -> np.ndarray:
    """[B,Hq,D] float64 selective attention over sinks U top-K U window under WRoPE."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    idx, cnt = _i32(topk_idx), _i32(topk_count)
    B, Hq, D = q.shape
    _, Hkv, S, _ = k.shape
    K = idx.shape[2]
    out = np.empty((B, Hq, D), dtype=np.float64)
    rc = _load().a2ats_oracle_sparse_attn(_p(q), _p(k), _p(v), _p(idx), _p(cnt), _I(B), _I(Hq), _I(Hkv),
                                          _I(D), _L(n_ctx), _L(S), _I(K), _I(window), _I(n_sink),
                                          _p(_f64(inv_freq)), _D(float(b_off)), _p(_i32(seq_lens)), _p(out))
    if rc != 0:
        raise ValueError("top-K index outside the candidate range")
    return out


def dense_wrope_attn(q, k, v, n_ctx: int, window: int, inv_freq, b_off: float, seq_lens=None
                     ) -> np.ndarray:
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, Hq, D = q.shape
    _, Hkv, S, _ = k.shape
    out = np.empty((B, Hq, D), dtype=np.float64)
    _load().a2ats_oracle_dense_wrope_attn(_p(q), _p(k), _p(v), _I(B), _I(Hq), _I(Hkv), _I(D), _L(n_ctx),
                                          _L(S), _I(window), _p(_f64(inv_freq)), _D(float(b_off)),
                                          _p(_i32(seq_lens)), _p(out))
    return out


W_NONE, W_DIAG, W_BLOCK = 0, 1, 2


def encode(keys, codebook, weights=None, mode: int = W_NONE, want_margins: bool = False):
    """codes [B,Hkv,n,M] uint8 (and, if asked, the best / second-best distortions)."""
    keys, cb = _f32(keys), _f32(codebook)
    B, Hkv, n, D = keys.shape
    _, M, L, ds = cb.shape
    w = None if weights is None else _f32(weights)
    assert mode == W_NONE or w is not None
    codes = np.empty((B, Hkv, n, M), dtype=np.uint8 if L <= 256 else np.uint16)
    best = np.empty((B, Hkv, n, M), dtype=np.float64) if want_margins else None
    second = np.empty((B, Hkv, n, M), dtype=np.float64) if want_margins else None
    rc = _load().a2ats_oracle_encode(_p(keys), _p(cb), _p(w), _I(mode), _I(B), _I(Hkv), _L(n), _I(M), _I(L),
                                     _I(ds), _p(codes), _I(codes.itemsize), _p(best), _p(second))
    assert rc == 0, rc
    if want_margins:
        return codes, best, second
    return codes


def encode_cholesky(keys, codebook, h_block, want_margins: bool = False):
    keys, cb, w = _f32(keys), _f32(codebook), _f32(h_block)
    B, Hkv, n, D = keys.shape
    _, M, L, ds = cb.shape
    codes = np.empty((B, Hkv, n, M), dtype=np.uint8 if L <= 256 else np.uint16)
    best = np.empty((B, Hkv, n, M), dtype=np.float64) if want_margins else None
    second = np.empty((B, Hkv, n, M), dtype=np.float64) if want_margins else None
    rc = _load().a2ats_oracle_encode_cholesky(_p(keys), _p(cb), _p(w), _I(B), _I(Hkv), _L(n), _I(M),
                                              _I(L), _I(ds), _p(codes), _I(codes.itemsize), _p(best), _p(second))
    if rc != 0:
        raise ValueError("weight block is not positive definite")
    if want_margins:
        return codes, best, second
    return codes


# ---------------------------------------------------------------------------------------------
# Offline codebook construction (section 4.2: second moment of the queries, k-means under the
# query-aware distortion).  Plain numpy, float64.
# ---------------------------------------------------------------------------------------------
def second_moment(q_rot, n_kv_heads: int) -> np.ndarray:
    """H [Hkv,D,D] = E[q~^T q~] (section 4.2), the mean of the outer products of the rotated
    queries q_rot [n,Hq,D]; the G query heads of a KV head share its codebook, so their samples
    are pooled (query head h belongs to KV head h // G)."""
    q = _f64(q_rot)
    n, Hq, D = q.shape
    G = Hq // n_kv_heads
    H = np.zeros((n_kv_heads, D, D), dtype=np.float64)
    for kv in range(n_kv_heads):
        for g in range(G):
            x = q[:, kv * G + g, :]
            for i in range(n):
                H[kv] += np.outer(x[i], x[i])
        H[kv] /= n * G
    return H


def distortion(keys, codebook, codes, h_full) -> np.ndarray:
    """J' [Hkv] = sum over the keys of (k - c) H (k - c)^T (section 4.2, the query-aware objective),
    keys [B,Hkv,n,D], one codebook [Hkv,1,L,D], codes [B,Hkv,n,1], H [Hkv,D,D]."""
    k, cb, H = _f64(keys), _f64(codebook), _f64(h_full)
    c = np.asarray(codes).astype(np.int64).reshape(k.shape[0], k.shape[1], k.shape[2])
    out = np.zeros(k.shape[1], dtype=np.float64)
    for kv in range(k.shape[1]):
        for b in range(k.shape[0]):
            e = k[b, kv] - cb[kv, 0][c[b, kv]]
            out[kv] += np.einsum("nd,de,ne->", e, H[kv], e)
    return out


def lloyd_update(keys, codes, codebook):
    """The centroid step of k-means (section 4.2 runs k-means on z = k L and maps the centroids
    back with L^-1; the mean is linear, so that is the mean of the assigned keys themselves):
    new codebook [Hkv,1,L,D] float64 and counts [Hkv,L]; a codeword that no key was assigned to
    keeps its old value.  The keys of all B sequences are pooled per KV head."""
    k, cb = _f64(keys), _f64(codebook)
    B, Hkv, n, D = k.shape
    L = cb.shape[2]
    c = np.asarray(codes).astype(np.int64).reshape(B, Hkv, n)
    new = cb.copy()
    counts = np.zeros((Hkv, L), dtype=np.int64)
    for kv in range(Hkv):
        sums = np.zeros((L, D), dtype=np.float64)
        for b in range(B):
            for j in range(n):
                sums[c[b, kv, j]] += k[b, kv, j]
                counts[kv, c[b, kv, j]] += 1
        used = counts[kv] > 0
        new[kv, 0][used] = sums[used] / counts[kv][used, None]
    return new, counts


def _seed_distortions(z, pick):
    """||z_i - z_pick||^2 for every row i (float64)."""
    e = z - z[pick]
    return np.einsum("nd,nd->n", e, e)


def _seed_draw(d, u_r, n_rows):
    """One k-means++ draw: the first row whose inclusive prefix sum of d exceeds u_r * sum(d) (inverse
    of the cumulative distribution: row i is drawn with probability d_i / sum(d)); uniform over the
    rows if every distortion is zero.  Returns (row, prefix sums, target)."""
    cum = np.cumsum(d)
    if cum[-1] > 0.0:
        target = u_r * cum[-1]
        return min(n_rows - 1, int(np.searchsorted(cum, target, side="right"))), cum, target
    return min(n_rows - 1, int(u_r * n_rows)), cum, 0.0


def _seed_rows(keys, h_full, kv):
    k = _f64(keys)
    B, Hkv, n, D = k.shape
    rows = k[:, kv].reshape(B * n, D)
    Lc = np.eye(D) if h_full is None else np.linalg.cholesky(_f64(h_full)[kv])
    return rows @ Lc


def kmeanspp_seed(keys, h_full, u, n_codewords: int):
    """k-means++ seeding (Arthur & Vassilvitskii; section 4.2 initialises its k-means with it) under
    the query-aware distortion (k - c) H (k - c)^T = ||z_k - z_c||^2, z = k L, H = L L^T (section 4.2,
    Cholesky reformulation).  keys [B,Hkv,n,D] (pooled per KV head, row i = b*n + j), H [Hkv,D,D]
    (None: identity), u [Hkv,n_codewords] uniform numbers in [0,1) standing in for the random draws.
    Codeword 0 is row floor(u_0 rows); codeword r is drawn with probability d_i / sum(d), d_i the
    distortion of row i to the nearest codeword chosen so far.  Float64 throughout.
    Returns picks [Hkv,n_codewords]."""
    B, Hkv, n, D = np.asarray(keys).shape
    uu = _f64(u)
    picks = np.zeros((Hkv, n_codewords), dtype=np.int64)
    for kv in range(Hkv):
        z = _seed_rows(keys, h_full, kv)
        pick = min(B * n - 1, int(uu[kv, 0] * (B * n)))
        d = None
        for r in range(n_codewords):
            picks[kv, r] = pick
            if r == n_codewords - 1:
                break
            dist = _seed_distortions(z, pick)
            d = dist if d is None else np.minimum(d, dist)
            pick, _, _ = _seed_draw(d, uu[kv, r + 1], B * n)
    return picks


def kmeanspp_check(keys, h_full, u, picks, rel_tol: float):
    """Checks a sequence of k-means++ draws made elsewhere against the definition, draw by draw.
    The draws are sequential (each depends on the codewords chosen before it), so one draw decided
    differently changes all later ones; here draw r is therefore evaluated GIVEN picks[:, :r] as the
    history.  For every draw the definition's row (kmeanspp_seed's rule, float64) is compared with
    picks[kv, r]:
      equal                                  -> counted in n_equal;
      different, but picks[kv, r] is the row the rule gives for a target moved by at most
      rel_tol * sum(d) (its prefix interval [cum[g-1], cum[g]) comes that close to the target, and
      d_g > 0)                               -> counted in n_near (a draw on a prefix boundary);
      anything else                          -> recorded in wrong [(kv, r, definition's row, given row)].
    Returns (n_equal, n_near, wrong)."""
    B, Hkv, n, D = np.asarray(keys).shape
    uu = _f64(u)
    pk = np.asarray(picks).astype(np.int64)
    n_codewords = pk.shape[1]
    n_equal = n_near = 0
    wrong = []
    for kv in range(Hkv):
        z = _seed_rows(keys, h_full, kv)
        want0 = min(B * n - 1, int(uu[kv, 0] * (B * n)))
        if pk[kv, 0] == want0:
            n_equal += 1
        else:
            wrong.append((kv, 0, want0, int(pk[kv, 0])))
        d = None
        for r in range(1, n_codewords):
            prev = int(pk[kv, r - 1])
            if not 0 <= prev < B * n:
                wrong.append((kv, r - 1, -1, prev))
                break
            dist = _seed_distortions(z, prev)
            d = dist if d is None else np.minimum(d, dist)
            want, cum, target = _seed_draw(d, uu[kv, r], B * n)
            g = int(pk[kv, r])
            if g == want:
                n_equal += 1
                continue
            tol = rel_tol * cum[-1]
            ok = 0 <= g < B * n and cum[-1] > 0.0 and d[g] > 0.0
            if ok:
                lo = cum[g - 1] if g > 0 else 0.0
                ok = lo - tol <= target <= cum[g] + tol
            if ok:
                n_near += 1
            else:
                wrong.append((kv, r, want, g))
    return n_equal, n_near, wrong
