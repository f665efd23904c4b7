"""Thin ctypes binding over liba2ats.so (the C ABI in include/a2ats.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch is
used for device memory and for the current HIP stream.  There is no CPU fallback: if
the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liba2ats.so")

F32, BF16 = 0, 1
W_NONE, W_DIAG, W_BLOCK = 0, 1, 2
W_PREPARED = 0x100
OP_ENCODE, OP_LUT, OP_SCORE_TOPK, OP_ATTN, OP_FIT, OP_SEED = 0, 1, 2, 3, 4, 5
EXPORTS = ["a2ats_version", "a2ats_status_string", "a2ats_lut_elems", "a2ats_workspace_bytes", "a2ats_encode_prepare",
           "a2ats_rope_tables", "a2ats_encode_keys", "a2ats_build_lut", "a2ats_score_topk",
           "a2ats_sparse_attn", "a2ats_score_topk_stats", "a2ats_score_topk_plan", "a2ats_score_topk_profiled",
           "a2ats_decode_prologue", "a2ats_decode_select", "a2ats_build_lut_shared", "a2ats_sparse_attn_shared",
           "a2ats_decode_select_shared",
           "a2ats_second_moment", "a2ats_codebook_update", "a2ats_kmeanspp_seed", "a2ats_sparse_attn_paged",
           "a2ats_sparse_attn_static", "a2ats_score_topk_paged", "a2ats_codes_to_pages",
           "a2ats_sparse_attn_host"]


class A2atsError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


class Dims(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("n_sub", ctypes.c_int32), ("sub_dim", ctypes.c_int32),
                ("n_centroids", ctypes.c_int32), ("ctx_len", ctypes.c_int32), ("ctx_stride", ctypes.c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library (build it with paper_2502_12665_amd.build.build() first)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run __graft_entry__.build() "
                                    "or `python -m paper_2502_12665_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp = ctypes.POINTER(Dims)
        L.a2ats_version.restype = ctypes.c_int
        L.a2ats_status_string.restype = ctypes.c_char_p
        L.a2ats_status_string.argtypes = [ctypes.c_int]
        L.a2ats_lut_elems.restype = sz
        L.a2ats_lut_elems.argtypes = [dp]
        L.a2ats_workspace_bytes.restype = sz
        L.a2ats_workspace_bytes.argtypes = [dp, ctypes.c_int, i32, i32]
        L.a2ats_rope_tables.restype = ctypes.c_int
        L.a2ats_rope_tables.argtypes = [i32, vp, i32, i32, vp, vp, vp, vp]
        L.a2ats_encode_keys.restype = ctypes.c_int
        L.a2ats_encode_keys.argtypes = [dp, vp, i32, i32, vp, vp, ctypes.c_int, vp, vp, sz, vp]
        L.a2ats_build_lut.restype = ctypes.c_int
        L.a2ats_encode_prepare.argtypes = [dp, vp, vp, ctypes.c_int, vp, sz, vp]
        L.a2ats_encode_prepare.restype = ctypes.c_int
        L.a2ats_build_lut.argtypes = [dp, vp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp]
        L.a2ats_decode_prologue.restype = ctypes.c_int
        L.a2ats_decode_prologue.argtypes = [dp, vp, i32, i32, vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, vp,
                                            vp, vp, vp, vp, vp, sz, vp]
        L.a2ats_decode_select.restype = ctypes.c_int
        L.a2ats_decode_select.argtypes = [dp, vp, i32, i32, vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, vp, vp, vp,
                                          vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.a2ats_decode_select_shared.restype = ctypes.c_int
        L.a2ats_decode_select_shared.argtypes = L.a2ats_decode_select.argtypes
        L.a2ats_score_topk.restype = ctypes.c_int
        L.a2ats_score_topk.argtypes = [dp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.a2ats_sparse_attn.restype = ctypes.c_int
        L.a2ats_sparse_attn.argtypes = [dp, vp, vp, vp, vp, ctypes.c_int, vp, vp, i32, i32, i32, vp, vp,
                                        vp, vp, vp, sz, vp]
        L.a2ats_sparse_attn_static.restype = ctypes.c_int
        L.a2ats_sparse_attn_static.argtypes = [dp, vp, vp, vp, vp, ctypes.c_int, vp, vp, i32, i32, i32, vp, vp,
                                               vp, vp, vp]
        L.a2ats_sparse_attn_shared.restype = ctypes.c_int
        L.a2ats_sparse_attn_shared.argtypes = L.a2ats_sparse_attn.argtypes
        L.a2ats_sparse_attn_paged.restype = ctypes.c_int
        L.a2ats_sparse_attn_paged.argtypes = [dp, vp, vp, vp, vp, ctypes.c_int, vp, i32, vp, vp, i32, i32, i32, vp, vp,
                                              vp, vp, vp, sz, vp]
        L.a2ats_build_lut_shared.restype = ctypes.c_int
        L.a2ats_build_lut_shared.argtypes = L.a2ats_build_lut.argtypes
        L.a2ats_kmeanspp_seed.restype = ctypes.c_int
        L.a2ats_kmeanspp_seed.argtypes = [dp, vp, i32, vp, ctypes.c_int, vp, vp, vp, vp, sz, vp]
        L.a2ats_second_moment.restype = ctypes.c_int
        L.a2ats_second_moment.argtypes = [dp, vp, ctypes.c_int64, vp, vp, sz, vp]
        L.a2ats_codebook_update.restype = ctypes.c_int
        L.a2ats_codebook_update.argtypes = [dp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.a2ats_score_topk_plan.restype = ctypes.c_int
        L.a2ats_score_topk_plan.argtypes = [dp, i32, i32, i32, ctypes.POINTER(ctypes.c_int32)]
        L.a2ats_score_topk_stats.restype = ctypes.c_int
        L.a2ats_score_topk_stats.argtypes = [dp, i32, i32, i32, vp, vp, vp]
        L.a2ats_score_topk_profiled.restype = ctypes.c_int
        L.a2ats_score_topk_profiled.argtypes = L.a2ats_score_topk.argtypes + [vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().a2ats_status_string(int(status)).decode()


def version() -> int:
    return int(lib().a2ats_version())


def make_dims(batch, n_q_heads, n_kv_heads, head_dim, n_sub, ctx_len, ctx_stride=None,
              n_centroids=256, sub_dim=None) -> Dims:
    return Dims(batch, n_q_heads, n_kv_heads, head_dim, n_sub,
                head_dim // n_sub if sub_dim is None else sub_dim, n_centroids, ctx_len,
                ctx_len if ctx_stride is None else ctx_stride)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors crossing the C ABI must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def host_device_pointer(t: torch.Tensor) -> int:
    """Device-side address of a pinned host tensor (hipHostGetDevicePointer); raises if the memory is
    not mapped into the device's address space.  For caches kept in host memory and read by the GPU
    over PCIe."""
    assert t.device.type == "cpu" and t.is_pinned() and t.is_contiguous()
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipHostGetDevicePointer.restype = ctypes.c_int
    hip.hipHostGetDevicePointer.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_uint]
    dev = ctypes.c_void_p()
    rc = hip.hipHostGetDevicePointer(ctypes.byref(dev), ctypes.c_void_p(t.data_ptr()), 0)
    if rc != 0 or not dev.value:
        raise RuntimeError(f"hipHostGetDevicePointer failed ({rc}): the tensor is not mapped for the device")
    return int(dev.value)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _check(rc: int, what: str):
    if rc != 0:
        raise A2atsError(rc, what)


def lut_elems(dims: Dims) -> int:
    return int(lib().a2ats_lut_elems(ctypes.byref(dims)))


def workspace_bytes(dims: Dims, op: int, top_k: int = 0, window: int = 0) -> int:
    n = int(lib().a2ats_workspace_bytes(ctypes.byref(dims), op, top_k, window))
    if n == ctypes.c_size_t(-1).value:
        raise A2atsError(-1, "a2ats_workspace_bytes")
    return n


def rope_tables(head_dim: int, inv_freq: torch.Tensor, b: int, window: int, device=None):
    """Host helper -> (cos_b, sin_b [D/2], cos_win, sin_win [window, D/2]) float32, moved to `device`."""
    inv = inv_freq.detach().to("cpu", torch.float64).contiguous()
    half = head_dim // 2
    cb, sb = torch.empty(half, dtype=torch.float32), torch.empty(half, dtype=torch.float32)
    cw = torch.empty(max(window, 1), half, dtype=torch.float32)
    sw = torch.empty(max(window, 1), half, dtype=torch.float32)
    rc = lib().a2ats_rope_tables(head_dim, _ptr(inv), int(b), int(window), _ptr(cb), _ptr(sb), _ptr(cw), _ptr(sw))
    _check(rc, "a2ats_rope_tables")
    outs = (cb, sb, cw, sw)
    return tuple(t.to(device) for t in outs) if device is not None else outs


def encode_keys(dims: Dims, keys, n_new: int, pos0: int, codebook, weights, weight_mode: int, codes,
                ws: Optional[torch.Tensor] = None):
    rc = lib().a2ats_encode_keys(ctypes.byref(dims), _ptr(keys), n_new, pos0, _ptr(codebook), _ptr(weights),
                                 weight_mode, _ptr(codes), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                 _stream())
    _check(rc, "a2ats_encode_keys")


def encode_prepare(dims: Dims, codebook, weights, weight_mode: int, ws: torch.Tensor):
    rc = lib().a2ats_encode_prepare(ctypes.byref(dims), _ptr(codebook), _ptr(weights), weight_mode, _ptr(ws),
                                    ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_encode_prepare")


def build_lut(dims: Dims, q, cos_b, sin_b, codebook, q_rot, lut, lut_scale):
    rc = lib().a2ats_build_lut(ctypes.byref(dims), _ptr(q), _dtype_code(q), _ptr(cos_b), _ptr(sin_b),
                               _ptr(codebook), _ptr(q_rot), _ptr(lut), _ptr(lut_scale), _stream())
    _check(rc, "a2ats_build_lut")


def decode_prologue(dims: Dims, keys, n_new: int, pos0: int, codebook, weights, weight_mode: int, codes,
                    q, cos_b, sin_b, q_rot, lut, lut_scale, ws: Optional[torch.Tensor] = None):
    """encode_keys (the decode-time append of a few keys) and build_lut fused; `ws` for the single codebook."""
    rc = lib().a2ats_decode_prologue(ctypes.byref(dims), _ptr(keys), n_new, pos0, _ptr(codebook),
                                     _ptr(weights), weight_mode, _ptr(codes), _ptr(q), _dtype_code(q),
                                     _ptr(cos_b), _ptr(sin_b), _ptr(q_rot), _ptr(lut), _ptr(lut_scale),
                                     _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_decode_prologue")


def decode_select(dims: Dims, keys, n_new: int, pos0: int, codebook, weights, weight_mode: int, codes,
                  q, cos_b, sin_b, q_rot, lut, lut_scale, top_k: int, window: int, n_sink: int, seq_lens,
                  topk_idx, topk_count, topk_score=None, ws: Optional[torch.Tensor] = None):
    """decode_prologue + score_topk as one call (one launch less on the streaming route)."""
    rc = lib().a2ats_decode_select(ctypes.byref(dims), _ptr(keys), n_new, pos0, _ptr(codebook), _ptr(weights),
                                   weight_mode, _ptr(codes), _ptr(q), _dtype_code(q), _ptr(cos_b), _ptr(sin_b),
                                   _ptr(q_rot), _ptr(lut), _ptr(lut_scale), top_k, window, n_sink, _ptr(seq_lens),
                                   _ptr(topk_idx), _ptr(topk_count), _ptr(topk_score), _ptr(ws),
                                   0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_decode_select")


def decode_select_shared(dims: Dims, keys, n_new: int, pos0: int, codebook, weights, weight_mode: int, codes,
                         q, cos_b, sin_b, q_rot, lut, lut_scale, top_k: int, window: int, n_sink: int, seq_lens,
                         topk_idx, topk_count, topk_score=None, ws: Optional[torch.Tensor] = None):
    """encode_keys + build_lut_shared + score_topk (one selection per KV head) as one call; `dims` are the
    real ones, lut / lut_scale / topk_* / ws those of dims with n_q_heads = n_kv_heads."""
    rc = lib().a2ats_decode_select_shared(ctypes.byref(dims), _ptr(keys), n_new, pos0, _ptr(codebook),
                                          _ptr(weights), weight_mode, _ptr(codes), _ptr(q), _dtype_code(q),
                                          _ptr(cos_b), _ptr(sin_b), _ptr(q_rot), _ptr(lut), _ptr(lut_scale), top_k,
                                          window, n_sink, _ptr(seq_lens), _ptr(topk_idx), _ptr(topk_count),
                                          _ptr(topk_score), _ptr(ws),
                                          0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_decode_select_shared")


def score_topk(dims: Dims, codes, lut, lut_scale, top_k: int, window: int, n_sink: int, seq_lens,
               topk_idx, topk_count, topk_score=None, scores_out=None, ws: Optional[torch.Tensor] = None):
    rc = lib().a2ats_score_topk(ctypes.byref(dims), _ptr(codes), _ptr(lut), _ptr(lut_scale), top_k, window,
                                n_sink, _ptr(seq_lens), _ptr(topk_idx), _ptr(topk_count), _ptr(topk_score),
                                _ptr(scores_out), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                _stream())
    _check(rc, "a2ats_score_topk")


def sparse_attn(dims: Dims, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k: int, window: int,
                n_sink: int, cos_win, sin_win, seq_lens, out, ws: Optional[torch.Tensor] = None):
    rc = lib().a2ats_sparse_attn(ctypes.byref(dims), _ptr(q), _ptr(q_rot), _ptr(k_cache), _ptr(v_cache),
                                 _dtype_code(k_cache), _ptr(topk_idx), _ptr(topk_count), top_k, window, n_sink,
                                 _ptr(cos_win), _ptr(sin_win), _ptr(seq_lens), _ptr(out), _ptr(ws),
                                 0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_sparse_attn")


def sparse_attn_static(dims: Dims, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k: int, window: int,
                       n_sink: int, cos_win, sin_win, seq_lens, out):
    """sparse_attn with its scratch memory inside the library (allocates nothing; at most 8 MiB of it)."""
    rc = lib().a2ats_sparse_attn_static(ctypes.byref(dims), _ptr(q), _ptr(q_rot), _ptr(k_cache), _ptr(v_cache),
                                        _dtype_code(k_cache), _ptr(topk_idx), _ptr(topk_count), top_k, window,
                                        n_sink, _ptr(cos_win), _ptr(sin_win), _ptr(seq_lens), _ptr(out), _stream())
    _check(rc, "a2ats_sparse_attn_static")


def sparse_attn_host(dims: Dims, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k: int, window: int,
                     n_sink: int, cos_win, sin_win, seq_lens, out, n_threads: int = 0):
    """sparse_attn on the host CPU over a cache in host memory: every tensor is a CPU tensor."""
    for t in (q, q_rot, k_cache, v_cache, topk_idx, topk_count, cos_win, sin_win, seq_lens, out):
        assert t is None or t.device.type == "cpu", "a2ats_sparse_attn_host takes host pointers"
    rc = lib().a2ats_sparse_attn_host(ctypes.byref(dims), _ptr(q), _ptr(q_rot), _ptr(k_cache), _ptr(v_cache),
                                      _dtype_code(k_cache), _ptr(topk_idx), _ptr(topk_count), top_k, window, n_sink,
                                      _ptr(cos_win), _ptr(sin_win), _ptr(seq_lens), _ptr(out), n_threads)
    _check(rc, "a2ats_sparse_attn_host")


def build_lut_shared(dims: Dims, q, cos_b, sin_b, codebook, q_rot, lut, lut_scale):
    """Tables of one head per KV head from the summed rotated queries of its group (lut / lut_scale
    sized for dims with n_q_heads = n_kv_heads); q_rot per query head."""
    rc = lib().a2ats_build_lut_shared(ctypes.byref(dims), _ptr(q), _dtype_code(q), _ptr(cos_b), _ptr(sin_b),
                                      _ptr(codebook), _ptr(q_rot), _ptr(lut), _ptr(lut_scale), _stream())
    _check(rc, "a2ats_build_lut_shared")


def sparse_attn_shared(dims: Dims, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k: int, window: int,
                       n_sink: int, cos_win, sin_win, seq_lens, out, ws: Optional[torch.Tensor] = None):
    """sparse_attn with one selection per KV head (topk_idx [B,Hkv,K], topk_count [B,Hkv])."""
    rc = lib().a2ats_sparse_attn_shared(ctypes.byref(dims), _ptr(q), _ptr(q_rot), _ptr(k_cache), _ptr(v_cache),
                                        _dtype_code(k_cache), _ptr(topk_idx), _ptr(topk_count), top_k, window,
                                        n_sink, _ptr(cos_win), _ptr(sin_win), _ptr(seq_lens), _ptr(out), _ptr(ws),
                                        0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_sparse_attn_shared")


def kmeanspp_seed(dims: Dims, keys, n_new: int, weights, weight_mode: int, u, codebook_out, picks, ws: torch.Tensor):
    rc = lib().a2ats_kmeanspp_seed(ctypes.byref(dims), _ptr(keys), n_new, _ptr(weights), weight_mode, _ptr(u),
                                   _ptr(codebook_out), _ptr(picks), _ptr(ws), ws.numel() * ws.element_size(),
                                   _stream())
    _check(rc, "a2ats_kmeanspp_seed")


def second_moment(dims: Dims, q_rot, n_samples: int, h_out, ws: torch.Tensor):
    rc = lib().a2ats_second_moment(ctypes.byref(dims), _ptr(q_rot), n_samples, _ptr(h_out), _ptr(ws),
                                   ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_second_moment")


def codebook_update(dims: Dims, keys, n_new: int, pos0: int, codes, codebook, codebook_out, counts, ws: torch.Tensor):
    rc = lib().a2ats_codebook_update(ctypes.byref(dims), _ptr(keys), n_new, pos0, _ptr(codes), _ptr(codebook),
                                     _ptr(codebook_out), _ptr(counts), _ptr(ws), ws.numel() * ws.element_size(),
                                     _stream())
    _check(rc, "a2ats_codebook_update")


def sparse_attn_paged(dims: Dims, q, q_rot, k_pool, v_pool, page_table, page_size: int, topk_idx, topk_count,
                      top_k: int, window: int, n_sink: int, cos_win, sin_win, seq_lens, out, ws: torch.Tensor):
    """sparse_attn over pools of pages [page][Hkv][page_size][D] addressed through page_table [B, pages]."""
    rc = lib().a2ats_sparse_attn_paged(ctypes.byref(dims), _ptr(q), _ptr(q_rot), _ptr(k_pool), _ptr(v_pool),
                                       _dtype_code(k_pool), _ptr(page_table), page_size, _ptr(topk_idx),
                                       _ptr(topk_count), top_k, window, n_sink, _ptr(cos_win), _ptr(sin_win),
                                       _ptr(seq_lens), _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_sparse_attn_paged")


def score_topk_paged(dims: Dims, code_pool, page_table, page_size: int, lut, lut_scale, top_k: int, window: int,
                     n_sink: int, seq_lens, topk_idx, topk_count, topk_score=None, scores_out=None,
                     ws: Optional[torch.Tensor] = None):
    """score_topk over a pool of code pages [page][Hkv][page_size][M] addressed through page_table [B, pages]."""
    rc = lib().a2ats_score_topk_paged(ctypes.byref(dims), _ptr(code_pool), _ptr(page_table), page_size, _ptr(lut),
                                      _ptr(lut_scale), top_k, window, n_sink, _ptr(seq_lens), _ptr(topk_idx),
                                      _ptr(topk_count), _ptr(topk_score), _ptr(scores_out), _ptr(ws),
                                      0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "a2ats_score_topk_paged")


def codes_to_pages(dims: Dims, new_codes, n_new: int, pos0: int, code_pool, page_table, page_size: int):
    """Copy the code rows [B, Hkv, n_new, M] of freshly encoded tokens to tokens pos0.. of the paged pool."""
    rc = lib().a2ats_codes_to_pages(ctypes.byref(dims), _ptr(new_codes), n_new, pos0, _ptr(code_pool),
                                    _ptr(page_table), page_size, _stream())
    _check(rc, "a2ats_codes_to_pages")


PLAN_FIELDS = ("fast", "head_groups", "sample_parts", "sample_rows", "chunks", "rows_per_chunk",
               "segments_per_wave", "rows_per_segment", "segment_capacity", "survivor_capacity",
               "workspace_bytes_div_256")


def score_topk_plan(dims: Dims, top_k: int, window: int, n_sink: int) -> dict:
    """How a2ats_score_topk lays out its work for this shape (host only; no GPU needed)."""
    out = (ctypes.c_int32 * len(PLAN_FIELDS))()
    _check(lib().a2ats_score_topk_plan(ctypes.byref(dims), top_k, window, n_sink, out), "a2ats_score_topk_plan")
    return dict(zip(PLAN_FIELDS, (int(v) for v in out)))


def score_topk_stats(dims: Dims, top_k: int, window: int, n_sink: int, ws, cand_counts):
    rc = lib().a2ats_score_topk_stats(ctypes.byref(dims), top_k, window, n_sink, _ptr(ws), _ptr(cand_counts),
                                      _stream())
    _check(rc, "a2ats_score_topk_stats")


def score_topk_profiled(dims: Dims, codes, lut, lut_scale, top_k: int, window: int, n_sink: int, seq_lens,
                        topk_idx, topk_count, topk_score, scores_out, ws: Optional[torch.Tensor],
                        ev_start: int, ev_stop: int):
    """score_topk with a pair of HIP events (handles) attached to the dispatch of the code-streaming kernel."""
    rc = lib().a2ats_score_topk_profiled(ctypes.byref(dims), _ptr(codes), _ptr(lut), _ptr(lut_scale), top_k, window,
                                         n_sink, _ptr(seq_lens), _ptr(topk_idx), _ptr(topk_count), _ptr(topk_score),
                                         _ptr(scores_out), _ptr(ws),
                                         0 if ws is None else ws.numel() * ws.element_size(), _stream(),
                                         ctypes.c_void_p(ev_start), ctypes.c_void_p(ev_stop))
    _check(rc, "a2ats_score_topk_profiled")


class DecodeState:
    """Device buffers for one decode step of a fixed shape (allocation only; no arithmetic)."""

    def __init__(self, dims: Dims, top_k: int, window: int, n_sink: int, kv_dtype: torch.dtype,
                 inv_freq: torch.Tensor, wrope_b: int, device="cuda", want_scores=False):
        self.dims, self.top_k, self.window, self.n_sink = dims, top_k, window, n_sink
        B, Hq, D = dims.batch, dims.n_q_heads, dims.head_dim
        dev = torch.device(device)
        self.cos_b, self.sin_b, self.cos_win, self.sin_win = rope_tables(D, inv_freq, wrope_b, window, dev)
        self.q_rot = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
        self.lut = torch.empty(max(lut_elems(dims), 4), dtype=torch.int32, device=dev)
        self.lut_scale = torch.empty(B, Hq, dtype=torch.float32, device=dev)
        self.topk_idx = torch.empty(B, Hq, top_k, dtype=torch.int32, device=dev)
        self.topk_count = torch.empty(B, Hq, dtype=torch.int32, device=dev)
        self.topk_score = torch.empty(B, Hq, max(top_k, 1), dtype=torch.float32, device=dev)
        self.scores = torch.empty(B, Hq, dims.ctx_stride, dtype=torch.float32, device=dev) if want_scores else None
        self.out = torch.empty(B, Hq, D, dtype=kv_dtype, device=dev)
        n_ws = max(workspace_bytes(dims, OP_SCORE_TOPK, top_k, window),
                   workspace_bytes(dims, OP_ATTN, top_k, window),
                   workspace_bytes(dims, OP_ENCODE), 256)
        self.ws = torch.empty(n_ws, dtype=torch.uint8, device=dev)

    def step(self, q, codes, k_cache, v_cache, codebook, seq_lens=None, with_scores=False):
        """build_lut -> score_topk -> sparse_attn on the current stream; returns self.out."""
        build_lut(self.dims, q, self.cos_b, self.sin_b, codebook, self.q_rot, self.lut, self.lut_scale)
        score_topk(self.dims, codes, self.lut, self.lut_scale, self.top_k, self.window, self.n_sink, seq_lens,
                   self.topk_idx, self.topk_count, self.topk_score,
                   self.scores if with_scores else None, self.ws)
        sparse_attn(self.dims, q, self.q_rot, k_cache, v_cache, self.topk_idx, self.topk_count, self.top_k,
                    self.window, self.n_sink, self.cos_win, self.sin_win, seq_lens, self.out, self.ws)
        return self.out
