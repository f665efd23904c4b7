"""a2ats_sparse_attn_host (selective attention on the CPU over a cache in host memory) against the
oracle.  Runs without a GPU: every pointer of this entry point is a host pointer."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2502_12665_amd import synth


@pytest.fixture(scope="module")
def binding():
    from paper_2502_12665_amd import binding as B
    B.lib()
    return B


@pytest.mark.parametrize("dtype, lens, n_sink, window, n_threads", [
    ("bf16", None, 0, 64, 0),
    ("bf16", [3000, 1234, 40], 4, 100, 3),
    ("f32", [3000, 17, 0], 2, 64, 1),
    ("f32", None, 0, 0, 2),
])
def test_host_attention_matches_the_oracle(oracle, binding, dtype, lens, n_sink, window, n_threads):
    """Selection by the oracle, attention by the library's host kernel: the output equals the oracle's
    selective attention within the tolerance of the GPU kernel (2e-2 absolute for bf16 rows, 2e-4 for
    float32), with sinks, ragged lengths (also an empty and a shorter-than-window sequence), several
    thread counts and an empty window."""
    B = binding
    wl = synth.Workload("host", 3, 8, 2, 128, 16, 3000, 200, window, n_sink=n_sink, kv_dtype=dtype, seed=71)
    x = synth.make_decode_inputs(wl)
    N, K = wl.ctx_len, wl.top_k
    sl = None if lens is None else np.asarray(lens, dtype=np.int32)
    q_rot = oracle.rope(x["q"], x["inv_freq"], wl.wrope_b)
    scores = oracle.scores_explicit(q_rot, x["codebook"], x["codes"], N)
    idx, cnt, _ = oracle.topk(scores, K, window, n_sink, sl)
    want = oracle.sparse_attn(x["q"], x["k"], x["v"], idx, cnt, N, window, n_sink, x["inv_freq"], float(wl.wrope_b), sl)
    dims = B.make_dims(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sub, N)
    _, _, cos_win, sin_win = B.rope_tables(wl.head_dim, x["inv_freq"], wl.wrope_b, window)
    out = torch.full((wl.batch, wl.n_q_heads, 128), 7.0).to(x["k"].dtype)
    B.sparse_attn_host(dims, x["q"].contiguous(), torch.from_numpy(q_rot.astype(np.float32)), x["k"], x["v"],
                       torch.from_numpy(idx), torch.from_numpy(cnt), K, window, n_sink, cos_win, sin_win,
                       None if sl is None else torch.from_numpy(sl), out, n_threads)
    err = np.abs(out.float().numpy().astype(np.float64) - want).max()
    assert err <= (2e-2 if dtype == "bf16" else 2e-4), err
    if lens is not None and 0 in lens:
        assert float(out[lens.index(0)].float().abs().max()) == 0.0


def test_host_attention_checks_its_arguments(binding):
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)
    d = binding.make_dims(1, 8, 2, 128, 16, 64)

    def call(d, q=one, top_k=4, window=8, n_sink=0, kv_dtype=1, idx=one, cw=one, threads=1):
        return L.a2ats_sparse_attn_host(ctypes.byref(d), q, one, one, one, kv_dtype, idx, one, top_k, window, n_sink,
                                        cw, one, null, one, threads)
    assert call(d, q=null) == -1
    assert call(d, top_k=-1) == -1 and call(d, window=-1) == -1 and call(d, n_sink=-1) == -1
    assert call(d, kv_dtype=5) == -1
    assert call(d, idx=null) == -1
    assert call(d, cw=null) == -1
    assert call(d, threads=-2) == -1
    assert call(binding.make_dims(1, 8, 3, 128, 16, 64)) == -1      # heads not a multiple of KV heads
    assert call(binding.make_dims(1, 8, 2, 64, 16, 64)) == -2       # head_dim 64
