"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI binding, run the
CPU oracle on the same seeded inputs, and compare under the stated tolerances.

Tolerances (element by element):
  q_rot        |d| <= 2e-6 * max(1, |x|)          (float64 rotation rounded once to float32; the
                                                   library's tables are float32-rounded angles)
  table / score|d| <= 1e-4 * max(1, |s|)          (1e-4 relative, floored at 1e-4 absolute)
  top-K        index sets bit-exact, except positions whose oracle score lies within
               1e-6 * max(1, |tau|) of the oracle's K-th score tau without being equal to it
               (near-ties; counted, and the count must stay below 0.1 % of the selected slots)
  attention    |d| <= 2e-2 absolute (bf16 I/O), 2e-4 absolute for float32 I/O
  codes        bit-exact, except subvectors whose two smallest oracle distortions differ by less
               than 1e-6 * max(1, d2) (counted; same 0.1 % bound)
"""
from __future__ import annotations

import sys

import numpy as np
import torch

from paper_2502_12665_amd import binding as B
from paper_2502_12665_amd import synth


def log(msg: str):
    print(f"[parity] {msg}", flush=True)
    sys.stdout.flush()


def dims_of(wl: synth.Workload, ctx_stride=None):
    return B.make_dims(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sub, wl.ctx_len, ctx_stride,
                       n_centroids=wl.n_centroids)


def to_dev(x: dict, device="cuda") -> dict:
    return {k: (v.to(device) if (isinstance(v, torch.Tensor) and k != "inv_freq") else v) for k, v in x.items()}


def gpu_decode(wl: synth.Workload, xd: dict, seq_lens=None, n_sink=None, want_scores=True, ctx_stride=None):
    """One decode step on the GPU.  xd: device tensors from synth.make_decode_inputs."""
    n_sink = wl.n_sink if n_sink is None else n_sink
    stride = xd["codes"].shape[2]
    dims = dims_of(wl, stride)
    st = B.DecodeState(dims, wl.top_k, wl.window, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b,
                       want_scores=want_scores)
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32, device="cuda")
    st.topk_idx.fill_(-7)
    st.topk_count.fill_(-7)
    if st.scores is not None:
        st.scores.fill_(float("nan"))
    st.step(xd["q"], xd["codes"], xd["k"], xd["v"], xd["codebook"], seq_lens=sl, with_scores=want_scores)
    torch.cuda.synchronize()
    return st


def lut_as_float(st, wl: synth.Workload) -> np.ndarray:
    """Exact part of the library table -> [B,Hq,M,L] float64 (dequantised), for comparison with the
    oracle's table."""
    n = wl.batch * wl.n_q_heads * wl.n_sub * 256
    t = st.lut[:n].cpu().numpy().reshape(wl.batch, wl.n_q_heads, 256, wl.n_sub).astype(np.float64)
    t = np.ascontiguousarray(t.transpose(0, 1, 3, 2))   # library order is [c][m]
    return t * st.lut_scale.cpu().numpy().astype(np.float64)[:, :, None, None]


def coarse_table_consistent(st, wl: synth.Workload) -> bool:
    """The 16-bit coarse copy of the table must obey exact = base + (coarse << s) + rem with
    0 <= rem < 2^s per entry (summed over subspaces: rem < M * 2^s), for every head."""
    Bn, Hq, Hkv, M, G = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.n_sub, wl.group
    NG = (G + 3) // 4
    lut = st.lut.cpu().numpy()
    n_exact = Bn * Hq * M * 256
    n_coarse = Bn * Hkv * NG * 256 * M * 2
    exact = lut[:n_exact].reshape(Bn, Hq, 256, M).astype(np.int64).transpose(0, 1, 3, 2)   # -> [B,Hq,m,c]
    coarse = lut[n_exact:n_exact + n_coarse].view(np.uint16).reshape(Bn, Hkv, NG, M // 16, 256, 16, 4).astype(np.int64)
    meta = lut[n_exact + n_coarse:n_exact + n_coarse + Bn * Hq * 4].reshape(Bn, Hq, 4).astype(np.int64)
    for h in range(Hq):
        kv, hg = divmod(h, G)
        c = coarse[:, kv, hg // 4, :, :, :, hg % 4]                      # [B, half, 256 c, 16 m]
        c = np.transpose(c, (0, 1, 3, 2)).reshape(Bn, M, 256)            # [B, m, c]
        mins = exact[:, h].min(axis=2)                                   # [B, M]
        s = meta[:, h, 1]
        if not np.array_equal(meta[:, h, 0], mins.sum(axis=1)):
            return False
        if not np.array_equal(meta[:, h, 2], exact[:, h].max(axis=2).sum(axis=1)):
            return False
        rem = exact[:, h] - mins[:, :, None] - (c << s[:, None, None])
        if (rem < 0).any() or (rem >= (1 << s)[:, None, None]).any() or c.max() > 65535 // M:
            return False
    return True


def check_scores(got: np.ndarray, want: np.ndarray, what="scores"):
    if want.size == 0:
        return 0.0
    tol = 1e-4 * np.maximum(1.0, np.abs(want))
    err = np.abs(got - want)
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond 1e-4 rel; worst {err.max():.3e}"
    return float(err.max())


def compare_topk(g_idx, g_cnt, o_idx, o_cnt, o_scores, o_kth):
    """Index-set comparison per (b, h) with the near-tie rule.  Returns (#excluded, #slots)."""
    Bq, Hq = g_cnt.shape
    excluded = 0
    slots = 0
    for b in range(Bq):
        for h in range(Hq):
            assert g_cnt[b, h] == o_cnt[b, h], (b, h, g_cnt[b, h], o_cnt[b, h])
            c = int(o_cnt[b, h])
            slots += c
            gi, oi = g_idx[b, h, :c], o_idx[b, h, :c]
            assert np.all(g_idx[b, h, c:] == -1), (b, h)
            if c == 0:
                continue
            assert np.all(np.diff(gi) > 0), f"({b},{h}) indices not strictly ascending"
            if np.array_equal(gi, oi):
                continue
            diff = np.setxor1d(gi, oi)
            tau = o_kth[b, h]
            s = o_scores[b, h][diff]
            near = (np.abs(s - tau) <= 1e-6 * max(1.0, abs(tau))) & (s != tau)
            assert near.all(), (f"({b},{h}) top-K sets differ outside near-ties: positions {diff[~near][:8]}, "
                                f"scores {s[~near][:8]}, tau {tau}")
            excluded += len(diff)
    assert excluded <= max(2, 1e-3 * slots), f"{excluded} near-tie exclusions in {slots} slots"
    return excluded, slots


def compare_codes(g_codes, o_codes, best, second):
    diff = g_codes != o_codes
    if not diff.any():
        return 0
    near = (second - best) <= 1e-6 * np.maximum(1.0, second)
    assert not (diff & ~near).any(), f"{(diff & ~near).sum()} codes differ outside near-ties"
    n = int(diff.sum())
    assert n <= max(2, 1e-3 * diff.size)
    return n


def oracle_decode(orc, wl: synth.Workload, x: dict, seq_lens=None, n_sink=None):
    """Oracle results for CPU inputs x (full tensors of a small problem, or a one-KV-head slice)."""
    n_sink = wl.n_sink if n_sink is None else n_sink
    N = wl.ctx_len
    qrot = orc.rope(x["q"], x["inv_freq"], wl.wrope_b)
    scores = orc.scores_explicit(qrot, x["codebook"], x["codes"], N)
    idx, cnt, kth = orc.topk(scores, wl.top_k, wl.window, n_sink, seq_lens)
    out = orc.sparse_attn(x["q"], x["k"], x["v"], idx, cnt, N, wl.window, n_sink, x["inv_freq"],
                          float(wl.wrope_b), seq_lens)
    return {"q_rot": qrot, "scores": scores, "idx": idx, "cnt": cnt, "kth": kth, "out": out}


def slice_problem(wl: synth.Workload, xd: dict, b: int, kv: int):
    """CPU copy of the (b, kv) sub-problem of device inputs, as a batch-1 / one-KV-head workload."""
    G = wl.group
    sub = wl.replace(batch=1, n_q_heads=G, n_kv_heads=1)
    x = {
        "q": xd["q"][b:b + 1, kv * G:(kv + 1) * G].cpu(),
        "codebook": xd["codebook"][kv:kv + 1].cpu(),
        "codes": xd["codes"][b:b + 1, kv:kv + 1].cpu(),
        "k": xd["k"][b:b + 1, kv:kv + 1].cpu(),
        "v": xd["v"][b:b + 1, kv:kv + 1].cpu(),
        "inv_freq": xd["inv_freq"],
    }
    return sub, x


def check_step_against_oracle(orc, wl, st, x_cpu, b_sel=None, kv_sel=None, seq_lens=None, n_sink=None,
                              attn_tol=None):
    """Compare a finished GPU step `st` with the oracle, for the whole problem (x_cpu = all inputs on
    the CPU, b_sel None) or for one (b, kv) slice (x_cpu from slice_problem)."""
    n_sink = wl.n_sink if n_sink is None else n_sink
    G = wl.group
    if b_sel is None:
        sub, bs, hs = wl, slice(None), slice(None)
        sl = seq_lens
    else:
        sub = wl.replace(batch=1, n_q_heads=G, n_kv_heads=1)
        bs, hs = slice(b_sel, b_sel + 1), slice(kv_sel * G, (kv_sel + 1) * G)
        sl = None if seq_lens is None else np.asarray(seq_lens, dtype=np.int32)[b_sel:b_sel + 1]
    ref = oracle_decode(orc, sub, x_cpu, sl, n_sink)
    N = wl.ctx_len
    # rotation
    g_qrot = st.q_rot.cpu().numpy()[bs, hs].astype(np.float64)
    err = np.abs(g_qrot - ref["q_rot"])
    assert (err <= 2e-6 * np.maximum(1.0, np.abs(ref["q_rot"]))).all(), f"q_rot err {err.max():.3e}"
    # scores (only positions < n are written)
    if st.scores is not None:
        g_sc = st.scores.cpu().numpy()[bs, hs, :N].astype(np.float64)
        for bi in range(g_sc.shape[0]):
            n = N if sl is None else int(sl[bi])
            check_scores(g_sc[bi, :, :n], ref["scores"][bi, :, :n])
            assert np.isnan(g_sc[bi, :, n:]).all(), "scores written past the sequence end"
    # top-K
    g_idx = st.topk_idx.cpu().numpy()[bs, hs]
    g_cnt = st.topk_count.cpu().numpy()[bs, hs]
    exc, slots = compare_topk(g_idx, g_cnt, ref["idx"], ref["cnt"], ref["scores"], ref["kth"])
    if st.scores is not None and wl.top_k > 0:
        g_ts = st.topk_score.cpu().numpy()[bs, hs]
        g_sc32 = st.scores.cpu().numpy()[bs, hs]
        for bi in range(g_idx.shape[0]):
            for hi in range(g_idx.shape[1]):
                c = g_cnt[bi, hi]
                np.testing.assert_array_equal(g_ts[bi, hi, :c], g_sc32[bi, hi][g_idx[bi, hi, :c]])
    # attention
    tol = attn_tol if attn_tol is not None else (2e-2 if wl.kv_dtype == "bf16" else 2e-4)
    g_out = st.out.float().cpu().numpy()[bs, hs].astype(np.float64)
    aerr = np.abs(g_out - ref["out"]).max()
    assert aerr <= tol, f"attention err {aerr:.3e} > {tol}"
    return {"excluded": exc, "slots": slots, "attn_err": float(aerr)}
