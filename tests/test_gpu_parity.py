"""GPU parity: the HIP path, called through the C ABI binding, against the CPU oracle on the
same seeded inputs.  Tolerances are stated in tests/helpers.py."""
import itertools

import numpy as np
import pytest
import torch

from paper_2502_12665_amd import binding as B
from paper_2502_12665_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    B.lib()   # fails loudly if the library is not built


def _run_and_check(oracle, wl, seq_lens=None, n_sink=None, ctx_stride=None, x=None, mutate=None):
    x = synth.make_decode_inputs(wl, ctx_stride=ctx_stride) if x is None else x
    if mutate is not None:
        mutate(x)
    xd = H.to_dev(x)
    st = H.gpu_decode(wl, xd, seq_lens=seq_lens, n_sink=n_sink)
    return st, H.check_step_against_oracle(oracle, wl, st, x, seq_lens=seq_lens, n_sink=n_sink)


def test_tiny_shape_sweep_exact_route(oracle):
    w = 16
    n_cases = 0
    for G, (N, K), n_sink in itertools.product((1, 4, 7), [(1, 1), (w, 7), (w + 1, 1), (w + 7, 7), (257, 0),
                                                           (257, 7), (257, 257), (1000, 1), (1000, 7),
                                                           (1000, 1000)], (0, 4)):
        M = 32 if G == 7 else 16
        wl = synth.Workload(f"sweep_G{G}_N{N}_K{K}_s{n_sink}", 2, 2 * G, 2, 128, M, N, K, w, n_sink=n_sink,
                            kv_dtype="f32" if G == 1 else "bf16", rope_base=10000.0, seed=N + K + G)
        H.log(wl.name)
        _run_and_check(oracle, wl, ctx_stride=N + 5)
        n_cases += 1
    # ragged lengths, including an empty sequence and one shorter than the window
    wl = synth.Workload("sweep_ragged", 4, 8, 2, 128, 16, 600, 9, w, n_sink=4, seed=3)
    H.log(wl.name)
    _run_and_check(oracle, wl, seq_lens=[600, 0, 11, 333], ctx_stride=640)
    assert n_cases == 60


def test_config1_tiny(oracle):
    wl = synth.WORKLOADS["c1_tiny"]
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl)
    H.log(f"{wl.name}: {res}")
    # table parity (1e-4 relative) against the oracle's float64 table
    x = synth.make_decode_inputs(wl)
    lut = oracle.lut(oracle.rope(x["q"], x["inv_freq"], wl.wrope_b), x["codebook"], wl.n_q_heads)
    H.check_scores(H.lut_as_float(st, wl), lut, "table")
    assert H.coarse_table_consistent(st, wl)


@pytest.mark.parametrize("name,G,M,N,K,w,n_sink,seq_lens,stride", [
    ("fast_m16_g4", 4, 16, 20000, 600, 128, 0, None, None),
    ("fast_m16_g4_ragged", 4, 16, 24000, 512, 64, 4, [24000, 17001, 300, 0], 24064),
    ("fast_m32_g7", 7, 32, 18000, 500, 100, 4, [18000, 16500], 18016),
    ("fast_m16_g1_k1", 1, 16, 40000, 1, 64, 0, None, None),
    ("fast_m16_g8", 8, 16, 17000, 2048, 256, 0, None, None),
])
def test_fast_route_medium(oracle, name, G, M, N, K, w, n_sink, seq_lens, stride):
    Bn = len(seq_lens) if seq_lens else 2
    wl = synth.Workload(name, Bn, 2 * G, 2, 128, M, N, K, w, n_sink=n_sink, seed=11)
    H.log(wl.name)
    dims = H.dims_of(wl, stride)
    assert B.workspace_bytes(dims, B.OP_SCORE_TOPK, K, w) > 0, "expected the fast route"
    st, res = _run_and_check(oracle, wl, seq_lens=seq_lens, ctx_stride=stride)
    assert H.coarse_table_consistent(st, wl)
    H.log(f"{name}: {res}")


def test_random_shapes_whole_step(oracle):
    """Twenty seeded random shapes of the whole decode step against the oracle: 1 to 8 query heads per KV
    head, both subspace counts, contexts on either side of the exact / streaming boundary, any K up to a
    quarter of the candidates, windows from 0 to 300, sinks, ragged lengths (empty and nearly full
    sequences), padded strides, both cache types."""
    import random
    rng = random.Random(20260)
    for it in range(20):
        G = rng.choice([1, 2, 3, 4, 5, 7, 8])
        M = rng.choice([16, 32])
        Bn = rng.choice([1, 2, 3])
        short = rng.random() < 0.35
        N = rng.randint(300, 16000) if short else rng.randint(16500, 50000)
        w = rng.choice([0, 1, 16, 64, 128, 300])
        n_sink = rng.choice([0, 4, 17])
        kmax = max(1, min(2048, N if short else (N - w - n_sink) // 4))
        K = rng.choice([1, 7, 64, rng.randint(1, kmax), kmax])
        lens = None
        if rng.random() < 0.5:
            lens = [N] + [rng.choice([0, rng.randint(1, N), N - 1]) for _ in range(Bn - 1)]
        stride = N + rng.choice([0, 5, 64])
        wl = synth.Workload(f"rnd{it}", Bn, 2 * G, 2, 128, M, N, K, w, n_sink=n_sink, seed=2000 + it,
                            kv_dtype=rng.choice(["bf16", "f32"]))
        H.log(f"case {it}: B{Bn} G{G} M{M} N{N} K{K} w{w} sinks {n_sink} lens {lens} stride {stride} {wl.kv_dtype}")
        _, res = _run_and_check(oracle, wl, seq_lens=lens, ctx_stride=stride)
        H.log(f"   {res}")


def test_config2_llama8b_32k(oracle):
    wl = synth.WORKLOADS["c2_llama8b_32k"]
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl)
    H.log(f"{wl.name}: {res}")
    x = synth.make_decode_inputs(wl, with_kv=False)
    lut = oracle.lut(oracle.rope(x["q"], x["inv_freq"], wl.wrope_b), x["codebook"], wl.n_q_heads)
    H.check_scores(H.lut_as_float(st, wl), lut, "table")


def test_exact_ties_go_to_the_lowest_position(oracle):
    # (a) every code row identical: all scores equal, the fast route's candidate list overflows
    #     and the in-kernel exact fallback must return the first K candidates
    wl = synth.Workload("ties_all_equal", 1, 4, 1, 128, 16, 20000, 300, 64, n_sink=4, seed=5)

    def all_same(x):
        x["codes"][:] = x["codes"][:, :, :1]
    H.log(wl.name)
    st, _ = _run_and_check(oracle, wl, mutate=all_same)
    want = np.arange(4, 304, dtype=np.int32)
    for h in range(4):
        np.testing.assert_array_equal(st.topk_idx.cpu().numpy()[0, h], want)
    # (b) rows drawn from 40 distinct patterns: ~500 exact copies of each score, so the K-th key is
    #     shared by many candidates and the position tie-break inside the candidate list decides
    wl = synth.Workload("ties_few_patterns", 2, 8, 2, 128, 16, 20000, 700, 64, seed=6)

    def few_patterns(x):
        g = torch.Generator().manual_seed(1)
        pick = torch.randint(0, 40, (wl.batch, wl.n_kv_heads, wl.ctx_len), generator=g)
        pat = x["codes"][:, :, :40].clone()
        x["codes"][:, :, :wl.ctx_len] = torch.gather(pat, 2, pick[..., None].expand(-1, -1, -1, wl.n_sub))
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl, mutate=few_patterns)
    assert res["excluded"] == 0
    # (c) same on the exact route
    wl = synth.Workload("ties_few_patterns_exact", 1, 4, 1, 128, 16, 3000, 100, 64, seed=7)

    def few_patterns_small(x):
        g = torch.Generator().manual_seed(2)
        pick = torch.randint(0, 7, (1, 1, wl.ctx_len), generator=g)
        pat = x["codes"][:, :, :7].clone()
        x["codes"][:, :, :wl.ctx_len] = torch.gather(pat, 2, pick[..., None].expand(-1, -1, -1, wl.n_sub))
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl, mutate=few_patterns_small)
    assert res["excluded"] == 0


def test_attention_with_oracle_indices_and_full_retrieval(oracle):
    """a5 alone: feed the oracle's own top-K to the GPU attention; and K >= n - w gives dense WRoPE."""
    wl = synth.Workload("attn_only", 2, 8, 2, 128, 16, 3000, 200, 64, n_sink=4, seed=9)
    x = synth.make_decode_inputs(wl)
    ref = H.oracle_decode(oracle, wl, x)
    xd = H.to_dev(x)
    st = H.gpu_decode(wl, xd)
    st.topk_idx.copy_(torch.from_numpy(ref["idx"]))
    st.topk_count.copy_(torch.from_numpy(ref["cnt"]))
    B.sparse_attn(st.dims, xd["q"], st.q_rot, xd["k"], xd["v"], st.topk_idx, st.topk_count, wl.top_k,
                  wl.window, wl.n_sink, st.cos_win, st.sin_win, None, st.out, st.ws)
    torch.cuda.synchronize()
    err = np.abs(st.out.float().cpu().numpy() - ref["out"]).max()
    H.log(f"attention with oracle indices: err {err:.3e}")
    assert err <= 2e-2
    for dt, tol in (("f32", 2e-4), ("bf16", 2e-2)):
        wl2 = synth.Workload("attn_dense", 2, 8, 2, 128, 16, 700, 700, 64, n_sink=0, kv_dtype=dt, seed=10)
        x2 = synth.make_decode_inputs(wl2)
        st2 = H.gpu_decode(wl2, H.to_dev(x2))
        dense = oracle.dense_wrope_attn(x2["q"], x2["k"], x2["v"], wl2.ctx_len, wl2.window, x2["inv_freq"],
                                        float(wl2.wrope_b))
        err = np.abs(st2.out.float().cpu().numpy() - dense).max()
        H.log(f"K = n - w, {dt}: err vs dense WRoPE {err:.3e}")
        assert err <= tol


@pytest.mark.parametrize("M,mode", [(16, "none"), (16, "diag"), (16, "block"), (32, "none"), (32, "diag"),
                                    (32, "block")])
def test_encode_keys(oracle, M, mode):
    wl = synth.Workload(f"enc_m{M}_{mode}", 2, 8, 2, 128, M, 2048, 16, 16, seed=21)
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl)
    code = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = {"none": None, "diag": hm["h_diag"], "block": hm["h_block"]}[mode]
    dims = H.dims_of(wl, 2100)
    ws = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
    for n_new, pos0, stress in ((1000, 37, False), (777, 0, True), (1, 2099, False), (17, 5, True)):
        H.log(f"{wl.name} n_new={n_new} stress={stress}")
        keys = synth.make_encode_keys(wl, n_new, stress=stress)
        codes = torch.full((wl.batch, wl.n_kv_heads, 2100, M), 0xEE, dtype=torch.uint8, device="cuda")
        B.encode_keys(dims, keys.cuda(), n_new, pos0, cb.cuda(), None if weights is None else weights.cuda(),
                      code, codes, ws)
        torch.cuda.synchronize()
        got = codes.cpu().numpy()
        want, b1, b2 = oracle.encode(keys, cb, weights, code, want_margins=True)
        n_near = H.compare_codes(got[:, :, pos0:pos0 + n_new], want, b1, b2)
        assert (got[:, :, :pos0] == 0xEE).all() and (got[:, :, pos0 + n_new:] == 0xEE).all()
        if mode != "none" and stress:
            plain = oracle.encode(keys, cb)
            assert (want != plain).mean() > 0.02, "weighting should matter on the stress keys"
        H.log(f"  near-tie exclusions: {n_near}")


def test_run_to_run_determinism():
    wl = synth.Workload("determinism", 2, 8, 2, 128, 16, 30000, 900, 128, seed=4)
    xd = H.to_dev(synth.make_decode_inputs(wl))
    outs = []
    for _ in range(3):
        st = H.gpu_decode(wl, xd, want_scores=False)
        outs.append((st.topk_idx.cpu().clone(), st.topk_score.cpu().clone(), st.out.cpu().clone()))
    for o in outs[1:]:
        assert torch.equal(o[0], outs[0][0]) and torch.equal(o[1], outs[0][1])
        assert torch.equal(o[2].view(torch.int16), outs[0][2].view(torch.int16))


# ------------------------------------------------------------------ full-size configurations
def _full_size_check(oracle, wl, sample, plant=False, n_sink=0):
    """Run one decode step at a benchmark configuration's full size (inputs generated on the GPU with
    the seeded torch generator), then (a) compare sampled (sequence, KV head) problems element by
    element with the oracle and (b) check properties that hold for every head at any size."""
    H.log(f"{wl.name}: generating inputs on the GPU")
    xd = synth.make_decode_inputs(wl, device="cuda")
    if plant:
        _plant_similar_keys(oracle, wl, xd)
    H.log(f"{wl.name}: GPU step")
    st = H.gpu_decode(wl, xd, want_scores=True, n_sink=n_sink)
    # (b) properties over all heads, computed with torch library routines on the library's own scores
    N, K, w = wl.ctx_len, wl.top_k, wl.window
    cnt = st.topk_count
    assert int(cnt.min()) == int(cnt.max()) == min(K, N - w - n_sink)
    idx = st.topk_idx.long()
    assert int(idx.min()) >= n_sink and int(idx.max()) < N - w
    assert bool((idx[:, :, 1:] > idx[:, :, :-1]).all()), "indices not strictly ascending"
    sc = st.scores[:, :, :N]
    sel = torch.zeros_like(sc, dtype=torch.bool).scatter_(2, idx, True)
    cand = torch.zeros(N, dtype=torch.bool, device="cuda")
    cand[n_sink:N - w] = True
    neg = torch.full_like(sc, float("-inf"))
    min_sel = torch.where(sel, sc, -neg).amin(dim=2)
    max_unsel = torch.where(~sel & cand, sc, neg).amax(dim=2)
    assert bool((min_sel >= max_unsel).all()), "a rejected candidate outscores a selected one"
    # ties at the threshold: among positions scoring exactly the K-th score, the selected ones come first
    eq = (sc == min_sel[:, :, None]) & cand
    pos = torch.arange(N, device="cuda")
    last_sel_eq = torch.where(eq & sel, pos, torch.full_like(pos, -1)).amax(dim=2)
    first_unsel_eq = torch.where(eq & ~sel, pos, torch.full_like(pos, N)).amin(dim=2)
    assert bool((last_sel_eq < first_unsel_eq).all()), "a tie at the K-th score did not go to the lower position"
    np.testing.assert_array_equal(st.topk_score.cpu().numpy(), torch.gather(sc, 2, idx).cpu().numpy())
    cc = torch.empty(wl.batch, wl.n_q_heads, dtype=torch.int32, device="cuda")
    # (a) sampled problems against the oracle
    tot_exc = 0
    for (b, kv) in sample:
        H.log(f"{wl.name}: oracle on problem (b={b}, kv={kv})")
        sub, x = H.slice_problem(wl, xd, b, kv)
        res = H.check_step_against_oracle(oracle, wl, st, x, b_sel=b, kv_sel=kv, n_sink=n_sink)
        tot_exc += res["excluded"]
        H.log(f"  {res}")
    return st, tot_exc


def test_ragged_batch_with_several_segments_per_wave(oracle):
    """A batch large enough that a wave of the streaming pass owns several survivor segments (the
    configuration-3 shape: two runs per wave), with sequences that end inside a run, inside the first
    run, below the streaming route's minimum, and at zero length."""
    wl = synth.Workload("ragged_runs", 16, 32, 8, 128, 16, 32768, 1024, 128, n_sink=4, seed=29)
    lens = [32768, 0, 100, 16384 + 77, 20000, 32768, 5000, 24577, 32767, 17000, 31000, 28673, 19999, 32768, 16600, 300]
    H.log(f"{wl.name}: generating inputs on the GPU")
    xd = synth.make_decode_inputs(wl, device="cuda")
    st = H.gpu_decode(wl, xd, seq_lens=lens, want_scores=True)
    cnt = st.topk_count.cpu().numpy()
    for b, n in enumerate(lens):
        assert (cnt[b] == min(wl.top_k, max(0, n - wl.window - min(4, max(0, n - wl.window))))).all(), (b, n)
    for (b, kv) in [(0, 0), (3, 5), (4, 2), (7, 7), (8, 1), (2, 3), (6, 4)]:
        H.log(f"{wl.name}: oracle on problem (b={b}, kv={kv}, n={lens[b]})")
        sub, x = H.slice_problem(wl, xd, b, kv)
        res = H.check_step_against_oracle(oracle, wl, st, x, b_sel=b, kv_sel=kv, seq_lens=lens)
        H.log(f"  {res}")


def _plant_similar_keys(oracle, wl, xd):
    """Give 1 % of the candidate tokens of every (sequence, KV head) a key pulled towards the rotated
    query of the group's first head, and re-encode those keys (nearest centroid), so that the top-K
    has structure.  Built with the oracle's own rotation and encoder; tests only."""
    G, N, w = wl.group, wl.ctx_len, wl.window
    g = torch.Generator().manual_seed(1234)
    qrot = oracle.rope(xd["q"].cpu(), xd["inv_freq"], wl.wrope_b)           # [B,Hq,D]
    cb = xd["codebook"].cpu()
    n_pl = (N - w) // 100
    for b in range(wl.batch):
        for kv in range(wl.n_kv_heads):
            d = torch.from_numpy(qrot[b, kv * G]).float()
            d = d / d.norm()
            pos = torch.randperm(N - w, generator=g)[:n_pl]
            keys = xd["k"][b, kv, pos.cuda()].float().cpu() + 4.0 * d
            codes = oracle.encode(keys[None, None], cb[kv:kv + 1])[0, 0]
            xd["k"][b, kv, pos.cuda()] = keys.to(xd["k"].dtype).cuda()
            xd["codes"][b, kv, pos.cuda()] = torch.from_numpy(codes).cuda()


def _timed_path_against_oracle_everywhere(oracle, wl, plant=False, n_sink=0, seq_lens=None):
    """The step bench.py times -- a2ats_decode_select (append of the current token's key under the
    per-dimension query-aware distortion, rotation, tables, threshold sampling, streaming and final
    kernels) followed by a2ats_sparse_attn -- at a benchmark configuration's full size, compared with
    the oracle for EVERY (sequence, KV head) problem: the appended code row, the rotated queries, the
    top-K index sets (near-tie rule of tests/helpers.py, exclusions counted) and the attention output.
    The oracle runs one sequence (all its KV heads) at a time."""
    N, K, w, G = wl.ctx_len, wl.top_k, wl.window, wl.group
    H.log(f"{wl.name}: generating inputs on the GPU")
    xd = synth.make_decode_inputs(wl, device="cuda")
    if plant:
        _plant_similar_keys(oracle, wl, xd)
    hm = synth.make_query_second_moment(wl)
    h_diag = hm["h_diag"].cuda()
    new_key = xd["k"][:, :, N - 1:N, :].float().contiguous()
    dims = H.dims_of(wl)
    st = B.DecodeState(dims, K, w, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32, device="cuda")
    st.topk_idx.fill_(-7)
    st.topk_count.fill_(-7)
    xd["codes"][:, :, N - 1].fill_(0xEE)   # the row the call has to write
    H.log(f"{wl.name}: decode_select + sparse_attn")
    B.decode_select(dims, new_key, 1, N - 1, xd["codebook"], h_diag, B.W_DIAG, xd["codes"], xd["q"], st.cos_b,
                    st.sin_b, st.q_rot, st.lut, st.lut_scale, K, w, n_sink, sl, st.topk_idx, st.topk_count, None,
                    st.ws)
    stats = torch.empty(wl.batch, wl.n_q_heads, dtype=torch.int32, device="cuda")
    B.score_topk_stats(dims, K, w, n_sink, st.ws, stats)
    B.sparse_attn(dims, xd["q"], st.q_rot, xd["k"], xd["v"], st.topk_idx, st.topk_count, K, w, n_sink, st.cos_win,
                  st.sin_win, sl, st.out, st.ws)
    torch.cuda.synchronize()
    raw = stats.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
    fallback_heads = int(((raw >> 28) != 0).sum()) if (raw != 0xFFFFFFFF).all() else -1
    want_code, b1, b2 = oracle.encode(new_key.cpu(), xd["codebook"].cpu(), hm["h_diag"], oracle.W_DIAG,
                                      want_margins=True)
    n_code = H.compare_codes(xd["codes"][:, :, N - 1:N].cpu().numpy(), want_code, b1, b2)
    g_qrot = st.q_rot.cpu().numpy().astype(np.float64)
    g_idx, g_cnt = st.topk_idx.cpu().numpy(), st.topk_count.cpu().numpy()
    g_out = st.out.float().cpu().numpy().astype(np.float64)
    tol = 2e-2 if wl.kv_dtype == "bf16" else 2e-4
    exc = slots = 0
    worst = 0.0
    for b in range(wl.batch):
        x = {k: xd[k][b:b + 1].cpu() for k in ("q", "codes", "k", "v")}
        lens_b = None if seq_lens is None else np.asarray(seq_lens[b:b + 1], dtype=np.int32)
        sub = wl.replace(batch=1)
        qrot = oracle.rope(x["q"], xd["inv_freq"], wl.wrope_b)
        err = np.abs(g_qrot[b:b + 1] - qrot)
        assert (err <= 2e-6 * np.maximum(1.0, np.abs(qrot))).all(), f"q_rot err {err.max():.3e} (b={b})"
        scores = oracle.scores_explicit(qrot, xd["codebook"].cpu(), x["codes"], N)
        idx, cnt, kth = oracle.topk(scores, K, w, n_sink, lens_b)
        e, s_ = H.compare_topk(g_idx[b:b + 1], g_cnt[b:b + 1], idx, cnt, scores, kth)
        exc += e
        slots += s_
        # the library's own selection goes into the oracle's attention (a near-tie swap would otherwise
        # show up twice); identical to the oracle's whenever nothing was excluded
        out = oracle.sparse_attn(x["q"], x["k"], x["v"], g_idx[b:b + 1], g_cnt[b:b + 1], N, w, n_sink,
                                 xd["inv_freq"], float(wl.wrope_b), lens_b)
        aerr = float(np.abs(g_out[b:b + 1] - out).max())
        assert aerr <= tol, f"attention err {aerr:.3e} > {tol} (b={b})"
        worst = max(worst, aerr)
        if b % 4 == 0 or b == wl.batch - 1:
            H.log(f"{wl.name}: sequences 0..{b} compared")
    n_prob = wl.batch * wl.n_kv_heads
    H.log(f"{wl.name}: problems compared {n_prob}/{n_prob} (query heads {wl.batch * wl.n_q_heads}), top-K exclusions "
          f"{exc} of {slots} slots, code exclusions {n_code}, attention max err {worst:.2e}, heads on the exact "
          f"fallback {fallback_heads}")
    assert exc <= 1e-3 * max(slots, 1)
    return exc


def test_config3_batched_32k_planted(oracle):
    wl = synth.WORKLOADS["c3_batched_32k"]
    _full_size_check(oracle, wl, sample=[(0, 0), (7, 3), (15, 7)], plant=True)
    _timed_path_against_oracle_everywhere(oracle, wl, plant=True)


def test_config4_long_128k(oracle):
    wl = synth.WORKLOADS["c4_long_128k"]
    _full_size_check(oracle, wl, sample=[(0, 0), (1, 5), (3, 7)])
    _timed_path_against_oracle_everywhere(oracle, wl)


def test_config4_size_with_sinks_and_ragged_lengths(oracle):
    """The 131072-token shape with 4 sink tokens and per-sequence lengths: a full one, one that ends
    inside a streaming chunk, one just above the streaming route's minimum and a short one."""
    wl = synth.WORKLOADS["c4_long_128k"].replace(name="c4_sinks_ragged", n_sink=4, seed=77)
    _timed_path_against_oracle_everywhere(oracle, wl, n_sink=4, seq_lens=[131072, 100003, 16700, 3000])


def test_config5_qwen7b_64k_decode(oracle):
    wl = synth.WORKLOADS["c5_qwen7b_64k"]
    _full_size_check(oracle, wl, sample=[(0, 0), (13, 2), (31, 3)])
    _timed_path_against_oracle_everywhere(oracle, wl)


def test_single_codebook_full_size_every_problem(oracle):
    """The paper's own geometry (one codebook of 4096, 16-bit codes) at the 131072-token shape: one
    decode step (tables, selection, attention), every problem against the oracle."""
    wl = synth.WORKLOADS["p4_single_codebook_128k"]
    N, K, w = wl.ctx_len, wl.top_k, wl.window
    H.log(f"{wl.name}: generating inputs on the GPU")
    xd = synth.make_decode_inputs(wl, device="cuda")
    st = H.gpu_decode(wl, xd, want_scores=False)
    g_idx, g_cnt = st.topk_idx.cpu().numpy(), st.topk_count.cpu().numpy()
    g_out = st.out.float().cpu().numpy().astype(np.float64)
    exc = slots = 0
    worst = 0.0
    for b in range(wl.batch):
        x = {k: xd[k][b:b + 1].cpu() for k in ("q", "codes", "k", "v")}
        qrot = oracle.rope(x["q"], xd["inv_freq"], wl.wrope_b)
        # a score of this geometry is one float32 table entry: the oracle's float64 score rounded once
        scores = oracle.scores_explicit(qrot, xd["codebook"].cpu(), x["codes"], N).astype(np.float32).astype(np.float64)
        idx, cnt, kth = oracle.topk(scores, K, w, 0, None)
        e, s_ = H.compare_topk(g_idx[b:b + 1], g_cnt[b:b + 1], idx, cnt, scores, kth)
        exc += e
        slots += s_
        out = oracle.sparse_attn(x["q"], x["k"], x["v"], g_idx[b:b + 1], g_cnt[b:b + 1], N, w, 0, xd["inv_freq"],
                                 float(wl.wrope_b), None)
        worst = max(worst, float(np.abs(g_out[b:b + 1] - out).max()))
    n_prob = wl.batch * wl.n_kv_heads
    H.log(f"{wl.name}: problems compared {n_prob}/{n_prob}, top-K exclusions {exc} of {slots} slots, attention "
          f"max err {worst:.2e}")
    assert worst <= 2e-2 and exc <= 1e-3 * slots


def test_config5_encode_then_decode(oracle):
    """Configuration 5's prefill side: encode 65536 float32 pre-RoPE keys per KV head under the
    per-dimension query-aware distortion (weights = diagonal of a seeded PSD query second moment),
    here for 4 of the 32 sequences at full length, compare one whole sequence plus a 1 % sample of
    the other three with the oracle, and check that a decode step over the produced codes agrees with
    the oracle run on the same codes."""
    wl = synth.WORKLOADS["c5_qwen7b_64k"].replace(batch=4)
    N, M = wl.ctx_len, wl.n_sub
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl, "cuda")
    H.log("c5 encode: generating keys")
    keys = synth.make_encode_keys(wl, N, device="cuda")
    dims = H.dims_of(wl)
    ws = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
    codes = torch.empty(wl.batch, wl.n_kv_heads, N, M, dtype=torch.uint8, device="cuda")
    H.log("c5 encode: GPU")
    B.encode_keys(dims, keys, N, 0, cb, hm["h_diag"].cuda(), B.W_DIAG, codes, ws)
    torch.cuda.synchronize()
    H.log("c5 encode: oracle on sequence 0 (all KV heads)")
    want, b1, b2 = oracle.encode(keys[:1].cpu(), cb.cpu(), hm["h_diag"], oracle.W_DIAG, want_margins=True)
    n0 = H.compare_codes(codes[:1].cpu().numpy(), want, b1, b2)
    g = torch.Generator().manual_seed(5)
    pick = torch.randperm(N, generator=g)[:N // 100]
    sub_keys = keys[1:, :, pick.cuda()].cpu().contiguous()
    want, b1, b2 = oracle.encode(sub_keys, cb.cpu(), hm["h_diag"], oracle.W_DIAG, want_margins=True)
    n1 = H.compare_codes(codes[1:, :, pick.cuda()].cpu().numpy(), want, b1, b2)
    H.log(f"c5 encode: near-tie exclusions {n0} + {n1}")
    # decode over the encoder's codes
    xd = synth.make_decode_inputs(wl, device="cuda")
    xd["codes"] = codes
    xd["k"] = keys.to(torch.bfloat16)
    st = H.gpu_decode(wl, xd)
    for (b, kv) in [(0, 0), (3, 2)]:
        sub, x = H.slice_problem(wl, xd, b, kv)
        res = H.check_step_against_oracle(oracle, wl, st, x, b_sel=b, kv_sel=kv)
        H.log(f"  decode on encoded keys (b={b}, kv={kv}): {res}")


@pytest.mark.parametrize("name,n_new,mode", [("c1_tiny", 1, "none"), ("c2_llama8b_32k", 1, "diag"),
                                             ("c5_qwen7b_64k", 3, "block")])
def test_decode_prologue_equals_the_two_calls(name, n_new, mode):
    """The fused prologue (append-time encode + table build in one launch) must write bit for bit
    what a2ats_encode_keys and a2ats_build_lut write."""
    wl = synth.WORKLOADS[name].replace(batch=min(synth.WORKLOADS[name].batch, 4), ctx_len=4096)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    hm = synth.make_query_second_moment(wl)
    wmode = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = None if mode == "none" else hm["h_diag" if mode == "diag" else "h_block"].cuda()
    keys = synth.make_encode_keys(wl, n_new, device="cuda", stress=True)
    dims = H.dims_of(wl)
    pos0 = wl.ctx_len - n_new
    res = []
    for fused in (False, True):
        st = B.DecodeState(dims, wl.top_k, wl.window, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        st.lut.fill_(-1)
        codes = xd["codes"].clone()
        if fused:
            B.decode_prologue(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, xd["q"],
                              st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale)
        else:
            ws = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
            B.encode_keys(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, ws)
            B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
        torch.cuda.synchronize()
        res.append((codes.cpu(), st.lut.cpu(), st.lut_scale.cpu(), st.q_rot.cpu()))
    for a, b in zip(*res):
        assert torch.equal(a, b)
    assert not torch.equal(res[0][0][:, :, pos0:], xd["codes"][:, :, pos0:].cpu())   # the rows were rewritten


@pytest.mark.parametrize("name,Bn,Hkv,M,n_new,mode", [
    ("many_pairs_several_sweeps", 8, 8, 16, 32, "diag"),     # 32768 pairs: 128 encoding workgroups of 16 sweeps
    ("folded_two_sweeps", 40, 8, 16, 2, "block"),            # 320 table workgroups: they encode as well, 2 pairs a wave
    ("folded_m32_ragged_share", 33, 8, 32, 3, "none"),       # 264 table workgroups, 25344 pairs: the last ones idle
])
def test_decode_prologue_launch_shapes(name, Bn, Hkv, M, n_new, mode):
    """The prologue's ways of sharing out the append-time encoding (one pair per wave and sweep in
    workgroups of their own, or, when those would not fit beside the table workgroups, in the table
    workgroups themselves) write bit for bit what a2ats_encode_keys and a2ats_build_lut write."""
    wl = synth.Workload(name, Bn, Hkv, Hkv, 128, M, 2048, 64, 32, seed=83)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    hm = synth.make_query_second_moment(wl)
    wmode = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = None if mode == "none" else hm["h_diag" if mode == "diag" else "h_block"].cuda()
    keys = synth.make_encode_keys(wl, n_new, device="cuda", stress=True)
    dims = H.dims_of(wl)
    pos0 = wl.ctx_len - n_new
    res = []
    for fused in (False, True):
        st = B.DecodeState(dims, wl.top_k, wl.window, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        st.lut.fill_(-1)
        codes = xd["codes"].clone()
        if fused:
            B.decode_prologue(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, xd["q"],
                              st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale)
        else:
            ws = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
            B.encode_keys(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, ws)
            B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
        torch.cuda.synchronize()
        res.append((codes.cpu(), st.lut.cpu(), st.lut_scale.cpu(), st.q_rot.cpu()))
    for a, b in zip(*res):
        assert torch.equal(a, b)
    assert not torch.equal(res[0][0][:, :, pos0:], xd["codes"][:, :, pos0:].cpu())   # the rows were rewritten


@pytest.mark.parametrize("name,Bn,G,M,N,K,w,n_sink,n_new,mode,seq_lens", [
    ("sel_m16_g4", 2, 4, 16, 40000, 600, 128, 0, 1, "diag", None),
    ("sel_m16_g4_ragged", 4, 4, 16, 24000, 512, 64, 4, 2, "block", [24000, 17001, 300, 0]),
    ("sel_m32_g7", 2, 7, 32, 20000, 500, 100, 4, 1, "diag", [20000, 16500]),
    ("sel_m16_g8", 8, 8, 16, 33000, 2048, 256, 0, 1, "none", None),
    ("sel_exact_route", 2, 4, 16, 3000, 64, 32, 0, 1, "diag", None),
    ("sel_window_0", 2, 4, 16, 20000, 256, 0, 0, 1, "diag", None),          # the appended row is a candidate
    ("sel_window_below_n_new", 2, 4, 16, 20000, 256, 1, 0, 3, "diag", None),   # two of the three appended rows are
])
def test_decode_select_equals_the_two_calls(name, Bn, G, M, N, K, w, n_sink, n_new, mode, seq_lens):
    """a2ats_decode_select (append-time encode, tables and threshold sampling in one launch, then the
    streaming and final kernels) writes bit for bit what a2ats_decode_prologue + a2ats_score_topk write:
    codes, rotated queries, the whole table blob, scales, indices, counts and scores; and the same
    survivor statistics, i.e. the same thresholds.  Also on a shape of the exact route (plain two calls) and
    with a window shorter than the append (appended rows are candidates: the call must not sample the code
    matrix while they are being written, so it makes the two calls)."""
    wl = synth.Workload(name, Bn, 2 * G, 2, 128, M, N, K, w, n_sink=n_sink, seed=61)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    hm = synth.make_query_second_moment(wl)
    wmode = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = None if mode == "none" else hm["h_diag" if mode == "diag" else "h_block"].cuda()
    keys = synth.make_encode_keys(wl, n_new, device="cuda", stress=True)
    dims = H.dims_of(wl)
    pos0 = N - n_new
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32, device="cuda")
    res = []
    for fused in (False, True):
        st = B.DecodeState(dims, K, w, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        st.lut.fill_(-1)
        st.ws.fill_(0x5a)
        st.topk_idx.fill_(-7)
        codes = xd["codes"].clone()
        if fused:
            B.decode_select(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, xd["q"], st.cos_b,
                            st.sin_b, st.q_rot, st.lut, st.lut_scale, K, w, n_sink, sl, st.topk_idx, st.topk_count,
                            st.topk_score, st.ws)
        else:
            B.decode_prologue(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, xd["q"], st.cos_b,
                              st.sin_b, st.q_rot, st.lut, st.lut_scale)
            B.score_topk(dims, codes, st.lut, st.lut_scale, K, w, n_sink, sl, st.topk_idx, st.topk_count,
                         st.topk_score, None, st.ws)
        stats = torch.empty(Bn, 2 * G, dtype=torch.int32, device="cuda")
        B.score_topk_stats(dims, K, w, n_sink, st.ws, stats)
        torch.cuda.synchronize()
        res.append((codes.cpu(), st.lut.cpu(), st.lut_scale.cpu(), st.q_rot.cpu(), st.topk_idx.cpu(),
                    st.topk_count.cpu(), st.topk_score.cpu(), stats.cpu()))
    for i, (a, b) in enumerate(zip(*res)):
        assert torch.equal(a, b), f"output {i} differs"
    fast = B.score_topk_plan(dims, K, w, n_sink)["fast"]
    assert fast == (name != "sel_exact_route")
    assert int(res[1][5].max()) > 0


@pytest.mark.parametrize("name,Bn,Hkv,G,M,N,K,w,n_sink,n_new,mode,seq_lens", [
    ("shsel_m16_g4", 2, 2, 4, 16, 40000, 600, 128, 0, 1, "diag", None),
    ("shsel_m32_g7_ragged", 2, 2, 7, 32, 20000, 500, 100, 4, 2, "block", [20000, 16500]),
    ("shsel_m16_g8_batch", 4, 8, 8, 16, 33000, 2048, 256, 0, 1, "none", None),
    ("shsel_many_problems", 40, 8, 2, 16, 20000, 256, 64, 0, 1, "diag", None),   # 320 sampling workgroups: three launches
    ("shsel_exact_route", 2, 2, 4, 16, 3000, 64, 32, 0, 1, "diag", None),
    ("shsel_window_0", 2, 2, 4, 16, 20000, 256, 0, 0, 1, "diag", None),          # the appended row is a candidate
])
def test_decode_select_shared_equals_the_three_calls(name, Bn, Hkv, G, M, N, K, w, n_sink, n_new, mode, seq_lens):
    """a2ats_decode_select_shared (one selection per KV head: append-time encode, shared tables and threshold
    sampling in one launch, then the streaming and final kernels) writes bit for bit what a2ats_encode_keys +
    a2ats_build_lut_shared + a2ats_score_topk (dims with n_q_heads = n_kv_heads) write, and leaves the same
    survivor statistics; also where it has to make the three launches one after the other."""
    wl = synth.Workload(name, Bn, Hkv * G, Hkv, 128, M, N, K, w, n_sink=n_sink, seed=67)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    hm = synth.make_query_second_moment(wl)
    wmode = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = None if mode == "none" else hm["h_diag" if mode == "diag" else "h_block"].cuda()
    keys = synth.make_encode_keys(wl, n_new, device="cuda", stress=True)
    dims = H.dims_of(wl)
    dims_kv = B.make_dims(Bn, Hkv, Hkv, 128, M, N)
    pos0 = N - n_new
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32, device="cuda")
    res = []
    for fused in (False, True):
        st = B.DecodeState(dims, K, w, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        sk = B.DecodeState(dims_kv, K, w, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        sk.lut.fill_(-1)
        sk.ws.fill_(0x5a)
        sk.topk_idx.fill_(-7)
        st.q_rot.fill_(-3.0)
        codes = xd["codes"].clone()
        if fused:
            B.decode_select_shared(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, xd["q"], st.cos_b,
                                   st.sin_b, st.q_rot, sk.lut, sk.lut_scale, K, w, n_sink, sl, sk.topk_idx,
                                   sk.topk_count, sk.topk_score, sk.ws)
        else:
            ws = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
            B.encode_keys(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, ws)
            B.build_lut_shared(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, sk.lut, sk.lut_scale)
            B.score_topk(dims_kv, codes, sk.lut, sk.lut_scale, K, w, n_sink, sl, sk.topk_idx, sk.topk_count,
                         sk.topk_score, None, sk.ws)
        stats = torch.empty(Bn, Hkv, dtype=torch.int32, device="cuda")
        B.score_topk_stats(dims_kv, K, w, n_sink, sk.ws, stats)
        torch.cuda.synchronize()
        res.append((codes.cpu(), sk.lut.cpu(), sk.lut_scale.cpu(), st.q_rot.cpu(), sk.topk_idx.cpu(),
                    sk.topk_count.cpu(), sk.topk_score.cpu(), stats.cpu()))
    for i, (a, b) in enumerate(zip(*res)):
        assert torch.equal(a, b), f"output {i} differs"
    assert B.score_topk_plan(dims_kv, K, w, n_sink)["fast"] == (name != "shsel_exact_route")
    assert int(res[1][5].max()) > 0
    assert not torch.equal(res[1][0][:, :, pos0:], xd["codes"][:, :, pos0:].cpu())   # the appended rows were encoded


@pytest.mark.parametrize("shared", [False, True])
def test_decode_select_without_an_append(shared):
    """n_new = 0 (no key to append: keys may be NULL): the fused calls build the tables and select as the
    separate calls do, and leave the code matrix alone."""
    wl = synth.Workload("n0", 2, 8, 2, 128, 16, 30000, 500, 64, seed=3)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    dims = H.dims_of(wl)
    dsel = B.make_dims(2, 2, 2, 128, 16, 30000) if shared else dims
    st = B.DecodeState(dims, 500, 64, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    got = B.DecodeState(dsel, 500, 64, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    ref = B.DecodeState(dsel, 500, 64, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    codes = xd["codes"].clone()
    fused = B.decode_select_shared if shared else B.decode_select
    fused(dims, None, 0, 0, xd["codebook"], None, B.W_NONE, codes, xd["q"], st.cos_b, st.sin_b, st.q_rot, got.lut,
          got.lut_scale, 500, 64, 0, None, got.topk_idx, got.topk_count, None, got.ws)
    (B.build_lut_shared if shared else B.build_lut)(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, ref.lut,
                                                    ref.lut_scale)
    B.score_topk(dsel, codes, ref.lut, ref.lut_scale, 500, 64, 0, None, ref.topk_idx, ref.topk_count, None, None, ref.ws)
    torch.cuda.synchronize()
    assert torch.equal(got.topk_idx, ref.topk_idx) and torch.equal(got.topk_count, ref.topk_count)
    assert torch.equal(got.lut, ref.lut) and torch.equal(got.lut_scale, ref.lut_scale)
    assert torch.equal(codes, xd["codes"])
    assert int(got.topk_count.min()) == 500


@pytest.mark.parametrize("mode,n_new", [("none", 1), ("diag", 3), ("block", 8)])
def test_single_codebook_decode_prologue_equals_the_two_calls(mode, n_new):
    """The fused prologue in the single-codebook geometry (the sweep of the few-key encoder, then the
    table build that also picks the codes) writes bit for bit what the two calls write, with and
    without a prepared workspace."""
    wl = _single(f"single_prologue_{mode}", 3, 8, 2, 3000, 16, 16, seed=41)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    hm = synth.make_query_second_moment(wl)
    wmode = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = None if mode == "none" else hm["h_diag" if mode == "diag" else "h_block"].cuda()
    keys = synth.make_encode_keys(wl, n_new, device="cuda", stress=True)
    dims = H.dims_of(wl)
    pos0 = wl.ctx_len - n_new
    res = []
    for how in ("two calls", "fused", "fused, prepared"):
        st = B.DecodeState(dims, wl.top_k, wl.window, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        st.lut.fill_(-1)
        codes = xd["codes"].clone()
        ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
        if how == "two calls":
            B.encode_keys(dims, keys, n_new, pos0, xd["codebook"], weights, wmode, codes, ws)
            B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
        else:
            flag = 0
            if how == "fused, prepared":
                B.encode_prepare(dims, xd["codebook"], weights, wmode, ws)
                flag = B.W_PREPARED
            B.decode_prologue(dims, keys, n_new, pos0, xd["codebook"], weights, wmode | flag, codes, xd["q"],
                              st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale, ws)
        torch.cuda.synchronize()
        res.append((codes.cpu(), st.lut.cpu(), st.lut_scale.cpu(), st.q_rot.cpu()))
    for other in res[1:]:
        for a, b in zip(res[0], other):
            assert torch.equal(a, b)
    assert not torch.equal(res[0][0][:, :, pos0:], xd["codes"][:, :, pos0:].cpu())   # the rows were rewritten


@pytest.mark.parametrize("top_k,expect_fast", [(2048, True), (4096, False)])
def test_maximum_context_length_and_top_k(oracle, top_k, expect_fast):
    """The largest context the library accepts (2^20 tokens) with the largest K of the streaming
    route (2048) and the largest K of all (4096, exact route), whole step against the oracle."""
    wl = synth.Workload(f"max_ctx_K{top_k}", 1, 4, 1, 128, 16, 1 << 20, top_k, 256, n_sink=4, seed=9)
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl)
    H.log(f"  {res}")
    assert res["excluded"] <= res["slots"] // 1000
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    surv, route = _routes(wl, xd, n_sink=4)
    if expect_fast:
        assert (route == 0).all() and surv.max() <= 4 * top_k
    else:
        assert (surv == 0x0FFFFFFF).all()   # the exact-only route reports no survivor lists


# ---------------------------------------------------------------------------
# The paper's own geometry: one codebook of 4096 codewords per head (M = 1), 16-bit codes.
# ---------------------------------------------------------------------------
def _single(name, Bn, Hq, Hkv, N, K, w, **kw):
    return synth.Workload(name, Bn, Hq, Hkv, 128, 1, N, K, w, n_centroids=4096, **kw)


def test_single_codebook_small_shapes(oracle):
    """Whole steps against the oracle over small shapes: tiny and ragged contexts, K from 0 to all
    candidates, sinks, unaligned token-axis capacity, float32 and bf16 caches."""
    w = 16
    for G, (N, K), n_sink in itertools.product((1, 4, 7), [(1, 1), (w + 1, 1), (w + 7, 7), (257, 0), (257, 257),
                                                           (1000, 7), (9000, 300)], (0, 4)):
        wl = _single(f"single_G{G}_N{N}_K{K}_s{n_sink}", 2, 2 * G, 2, N, K, w, n_sink=n_sink,
                     kv_dtype="f32" if G == 1 else "bf16", rope_base=10000.0, seed=N + K + G)
        H.log(wl.name)
        _run_and_check(oracle, wl, ctx_stride=N + (5 if G == 4 else 0))
    wl = _single("single_ragged", 4, 8, 2, 600, 9, w, n_sink=4, seed=3)
    H.log(wl.name)
    _run_and_check(oracle, wl, seq_lens=[600, 0, 7, 333])


def test_single_codebook_heavy_ties(oracle):
    """With 4096 codewords there are at most 4096 distinct scores per head, so at 60000 tokens every
    score is shared by ~15 tokens and the K-th score almost always is: the position tie-break decides."""
    wl = _single("single_ties", 2, 8, 2, 60000, 1000, 64, seed=21)
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl)
    H.log(f"  {res}")
    assert res["excluded"] <= res["slots"] // 1000


def test_single_codebook_crowded_and_degenerate_tables(oracle):
    """The selection finds the K-th score with one level of bins linear in the score and finishes a bin
    of few codewords by counting.  Tables it cannot finish that way: thousands of nearly equal and
    hundreds of exactly equal scores around the K-th (the bin is crowded: radix levels inside it),
    and a table of identical scores (empty range: the lowest positions win)."""
    wl = _single("single_crowded", 2, 8, 2, 8000, 3900, 64, n_sink=4, seed=17)

    def crowd(x):
        g = torch.Generator().manual_seed(3)
        cb = x["codebook"]
        cb[:, 0, :3000] = 1e-3 * torch.randn(cb.shape[0], 3000, cb.shape[-1], generator=g)
        cb[:, 0, 3000:3200] = cb[:, 0, 2999:3000]
        x["codes"][...] = torch.randint(0, 4096, x["codes"].shape, generator=g).to(x["codes"].dtype)

    H.log(wl.name)
    st, res = _run_and_check(oracle, wl, mutate=crowd)
    H.log(f"  {res}")
    assert res["excluded"] <= res["slots"] // 100

    def flat(x):
        x["q"].zero_()

    wl = _single("single_flat", 1, 4, 2, 5000, 700, 64, n_sink=4, seed=18)
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl, mutate=flat)
    torch.cuda.synchronize()
    idx = st.topk_idx.cpu().numpy()
    assert (idx[:, :, :700] == np.arange(4, 704)[None, None]).all()   # after the 4 sinks


@pytest.mark.parametrize("mode", ["none", "diag", "block"])
def test_single_codebook_encode(oracle, mode):
    """Key encoder of the single-codebook geometry (full D x D matrix H in "block" mode) against the
    oracle: the matrix-core route with ragged tiles, the few-key route, keys far from every codeword,
    and keys planted so that two or three codewords are almost or exactly equally near (those go
    through the float64 re-check)."""
    wl = _single(f"single_enc_{mode}", 2, 4, 2, 3000, 16, 16, seed=33)
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl)
    cb[:, :, 77] = cb[:, :, 5]   # a duplicated codeword: exact ties, the lower code must win
    code = {"none": B.W_NONE, "diag": B.W_DIAG, "block": B.W_BLOCK}[mode]
    weights = {"none": None, "diag": hm["h_diag"], "block": hm["h_block"]}[mode]
    stride = 3100
    dims = H.dims_of(wl, stride)
    ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    for n_new, pos0, kind in ((1300, 37, "near"), (777, 0, "far"), (3, 3096, "near"), (8, 5, "far"),
                              (9, 0, "near"), (1100, 1000, "planted")):
        H.log(f"{wl.name} n_new={n_new} {kind}")
        keys = synth.make_encode_keys(wl, n_new, stress=(kind == "far"))
        if kind == "planted":
            g = torch.Generator().manual_seed(5)
            a, b, c = (torch.randint(0, 4096, (n_new,), generator=g) for _ in range(3))
            a[:50] = 5   # near the duplicated codeword
            for kv in range(wl.n_kv_heads):
                two = 0.5 * (cb[kv, 0, a] + cb[kv, 0, b])
                three = (cb[kv, 0, a] + cb[kv, 0, b] + cb[kv, 0, c]) / 3.0
                mid = torch.where((torch.arange(n_new) % 3 == 0)[:, None], three, two)
                mid[:50] = cb[kv, 0, 5]
                noise = torch.randn(wl.batch, n_new, 128, generator=g) * (10.0 ** -torch.randint(3, 7, (n_new, 1), generator=g))
                keys[:, kv] = mid[None] + noise.to(torch.float32)
        codes = torch.full((wl.batch, wl.n_kv_heads, stride, 1), 0x7EEE, dtype=torch.int16, device="cuda")
        B.encode_keys(dims, keys.cuda(), n_new, pos0, cb.cuda(), None if weights is None else weights.cuda(),
                      code, codes, ws)
        torch.cuda.synchronize()
        got = codes.cpu().numpy().view(np.uint16)
        if mode == "block":
            want, b1, b2 = oracle.encode_cholesky(keys, cb, weights, want_margins=True)
        else:
            want, b1, b2 = oracle.encode(keys, cb, weights, code, want_margins=True)
        n_near = H.compare_codes(got[:, :, pos0:pos0 + n_new], want, b1, b2)
        assert (got[:, :, :pos0] == 0x7EEE).all() and (got[:, :, pos0 + n_new:] == 0x7EEE).all()
        # the same call on a prepared workspace (factor and transformed codewords kept) gives the same codes
        again = torch.full_like(codes, 0x7EEE)
        B.encode_prepare(dims, cb.cuda(), None if weights is None else weights.cuda(), code, ws)
        B.encode_keys(dims, keys.cuda(), n_new, pos0, cb.cuda(), None if weights is None else weights.cuda(),
                      code | B.W_PREPARED, again, ws)
        torch.cuda.synchronize()
        assert torch.equal(again, codes)
        if kind == "planted":
            assert ((got[:, :, pos0:pos0 + 50] == 5) | (want[:, :, :50] != 5)).all()
            close = ((b2 - b1) <= 1e-3 * np.maximum(1.0, b2)).mean()
            assert close > 0.3, close
        H.log(f"  near-tie exclusions: {n_near}")


def test_single_codebook_encode_many_keys(oracle):
    """More keys per sequence than the transform buffer holds at once (16384): the full-matrix mode then
    works part by part; every part must land at its own positions."""
    wl = _single("single_enc_parts", 1, 1, 1, 40000, 16, 16, seed=5)
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl)
    n = 40000
    keys = synth.make_encode_keys(wl, n, stress=True)
    dims = H.dims_of(wl, n + 7)
    ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    codes = torch.full((1, 1, n + 7, 1), 0x7EEE, dtype=torch.int16, device="cuda")
    B.encode_keys(dims, keys.cuda(), n, 3, cb.cuda(), hm["h_block"].cuda(), B.W_BLOCK, codes, ws)
    torch.cuda.synchronize()
    got = codes.cpu().numpy().view(np.uint16)
    want, b1, b2 = oracle.encode_cholesky(keys, cb, hm["h_block"], want_margins=True)
    n_near = H.compare_codes(got[:, :, 3:3 + n], want, b1, b2)
    assert (got[:, :, :3] == 0x7EEE).all() and (got[:, :, 3 + n:] == 0x7EEE).all()
    H.log(f"{wl.name}: near-tie exclusions {n_near}")


def test_single_codebook_long_context(oracle):
    """More tokens than a workgroup keeps in registers at once (131072): the selection kernel then
    walks the codes span by span, in both of its passes; and the largest context and K the library
    accepts (2^20 tokens, K = 4096)."""
    wl = _single("single_long", 1, 4, 2, 300000, 2048, 64, n_sink=4, seed=8)
    H.log(wl.name)
    _run_and_check(oracle, wl)
    _run_and_check(oracle, wl, ctx_stride=300003)
    wl = _single("single_max", 1, 2, 1, 1 << 20, 4096, 256, n_sink=4, seed=10)
    H.log(wl.name)
    st, res = _run_and_check(oracle, wl)
    H.log(f"  {res}")


def test_single_codebook_full_size(oracle):
    wl = synth.WORKLOADS["p4_single_codebook_128k"]
    _full_size_check(oracle, wl, sample=[(0, 0), (3, 7)])


def _routes(wl, xd, n_sink=0):
    """Run tables + score/top-K alone and return (survivors per head, route per head)."""
    dims = H.dims_of(wl, xd["codes"].shape[2])
    st = B.DecodeState(dims, wl.top_k, wl.window, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
    B.score_topk(dims, xd["codes"], st.lut, st.lut_scale, wl.top_k, wl.window, n_sink, None, st.topk_idx,
                 st.topk_count, None, None, st.ws)
    out = torch.empty(wl.batch, wl.n_q_heads, dtype=torch.int32, device="cuda")
    B.score_topk_stats(dims, wl.top_k, wl.window, n_sink, st.ws, out)
    torch.cuda.synchronize()
    raw = out.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
    return raw & 0x0FFFFFFF, raw >> 28


def test_fast_route_is_taken_and_fallback_triggers():
    """Ordinary inputs must be served by the streaming route for every head (no silent exact
    fallback), with a survivor list of modest size; degenerate inputs must fall back."""
    for name in ("c2_llama8b_32k", "c3_batched_32k", "c4_long_128k", "c5_qwen7b_64k"):
        wl = synth.WORKLOADS[name]
        xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
        surv, route = _routes(wl, xd)
        H.log(f"{name}: survivors per head mean {surv.mean():.0f} min {surv.min()} max {surv.max()}; "
              f"fallback heads {(route != 0).sum()}")
        assert (route == 0).all()
        assert surv.min() >= wl.top_k and surv.max() <= 4 * wl.top_k
    wl = synth.Workload("ties_all_equal", 1, 4, 1, 128, 16, 20000, 300, 64, seed=5)
    xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
    xd["codes"][:] = xd["codes"][:, :, :1]
    surv, route = _routes(wl, xd)
    assert (route != 0).all(), route


def test_streaming_route_serves_a_grid_of_shapes():
    """Over a grid of context lengths, K and head layouts the streaming route must serve every head
    (the planner's segment and sample sizes must follow from the shape, not from one workload)."""
    bad = []
    for N, K, (Bn, Hq, Hkv, M) in itertools.product((16700, 100000, 600000), (1, 256, 2048),
                                                    ((1, 4, 1, 16), (2, 14, 2, 32), (8, 32, 8, 16))):
        if 4 * K > N - 64:
            continue
        wl = synth.Workload("grid", Bn, Hq, Hkv, 128, M, N, K, 64, seed=N + K)
        xd = synth.make_decode_inputs(wl, device="cuda", with_kv=False)
        surv, route = _routes(wl, xd)
        H.log(f"N={N} K={K} B{Bn} Hq{Hq} Hkv{Hkv} M{M}: survivors mean {surv.mean():.0f} max {surv.max()} "
              f"routes {np.bincount(route.ravel(), minlength=5)}")
        if (route != 0).any() or surv.max() > 8192:
            bad.append((N, K, Bn, Hq, Hkv, M))
        del xd
        torch.cuda.empty_cache()
    assert not bad, bad


@pytest.mark.parametrize("calls", ["four calls", "decode_select"])
def test_decode_step_in_a_hip_graph(calls):
    """A captured decode step must replay to the eager result every time, with eager work and
    synchronisations between the replays; as the four separate calls and as a2ats_decode_select +
    a2ats_sparse_attn."""
    wl = synth.Workload("graph", 2, 8, 2, 128, 16, 30000, 900, 128, seed=8)
    xd = H.to_dev(synth.make_decode_inputs(wl))
    st = H.gpu_decode(wl, xd, want_scores=False)           # eager reference (also warms the library)
    ref = (st.topk_idx.clone(), st.out.clone())
    new_key = xd["k"][:, :, -1:, :].float().contiguous()

    def step():
        if calls == "four calls":
            B.encode_keys(st.dims, new_key, 1, wl.ctx_len - 1, xd["codebook"], None, B.W_NONE, xd["codes"], st.ws)
            st.step(xd["q"], xd["codes"], xd["k"], xd["v"], xd["codebook"])
        else:
            B.decode_select(st.dims, new_key, 1, wl.ctx_len - 1, xd["codebook"], None, B.W_NONE, xd["codes"], xd["q"],
                            st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale, wl.top_k, wl.window, 0, None,
                            st.topk_idx, st.topk_count, None, st.ws)
            B.sparse_attn(st.dims, xd["q"], st.q_rot, xd["k"], xd["v"], st.topk_idx, st.topk_count, wl.top_k,
                          wl.window, 0, st.cos_win, st.sin_win, None, st.out, st.ws)
    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for it in range(4):
        st.topk_idx.fill_(-3)
        st.out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(st.topk_idx, ref[0]), f"replay {it}: top-K differs"
        assert torch.equal(st.out.view(torch.int16), ref[1].view(torch.int16)), f"replay {it}: output differs"
        junk = torch.randn(1 << 20, device="cuda").sum().item()   # eager work between replays
        assert junk == junk


def _group_shared_step(wl, xd, n_sink=0, want_scores=True, seq_lens=None):
    """One decode step with one selection per KV head: shared tables, score/top-K on the dims of the
    table heads, attention of all G heads over the shared rows."""
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32, device="cuda")
    stride = xd["codes"].shape[2]
    dims = H.dims_of(wl, stride)
    kvw = wl.replace(n_q_heads=wl.n_kv_heads)
    dims_kv = H.dims_of(kvw, stride)
    st = B.DecodeState(dims, wl.top_k, wl.window, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    sk = B.DecodeState(dims_kv, wl.top_k, wl.window, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b,
                       want_scores=want_scores)
    sk.topk_idx.fill_(-7)
    sk.topk_count.fill_(-7)
    B.build_lut_shared(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, sk.lut, sk.lut_scale)
    B.score_topk(dims_kv, xd["codes"], sk.lut, sk.lut_scale, wl.top_k, wl.window, n_sink, sl, sk.topk_idx,
                 sk.topk_count, sk.topk_score, sk.scores, sk.ws)
    B.sparse_attn_shared(dims, xd["q"], st.q_rot, xd["k"], xd["v"], sk.topk_idx, sk.topk_count, wl.top_k,
                         wl.window, n_sink, st.cos_win, st.sin_win, sl, st.out, st.ws)
    torch.cuda.synchronize()
    return st, sk


def test_shared_decode_step_in_a_hip_graph():
    """The step with one selection per KV head as its two calls (a2ats_decode_select_shared,
    a2ats_sparse_attn_shared), captured: every replay gives the eager result of the separate calls."""
    wl = synth.Workload("graph_shared", 2, 8, 2, 128, 16, 30000, 900, 128, seed=9)
    xd = H.to_dev(synth.make_decode_inputs(wl))
    new_key = xd["k"][:, :, -1:, :].float().contiguous()
    ws = torch.empty(max(B.workspace_bytes(H.dims_of(wl), B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
    B.encode_keys(H.dims_of(wl), new_key, 1, wl.ctx_len - 1, xd["codebook"], None, B.W_NONE, xd["codes"], ws)
    st, sk = _group_shared_step(wl, xd, want_scores=False)   # eager reference (also warms the library)
    ref = (sk.topk_idx.clone(), st.out.clone())

    def step():
        B.decode_select_shared(st.dims, new_key, 1, wl.ctx_len - 1, xd["codebook"], None, B.W_NONE, xd["codes"],
                               xd["q"], st.cos_b, st.sin_b, st.q_rot, sk.lut, sk.lut_scale, wl.top_k, wl.window, 0,
                               None, sk.topk_idx, sk.topk_count, None, sk.ws)
        B.sparse_attn_shared(st.dims, xd["q"], st.q_rot, xd["k"], xd["v"], sk.topk_idx, sk.topk_count, wl.top_k,
                             wl.window, 0, st.cos_win, st.sin_win, None, st.out, st.ws)
    step()
    torch.cuda.synchronize()
    assert torch.equal(sk.topk_idx, ref[0]) and torch.equal(st.out.view(torch.int16), ref[1].view(torch.int16))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for it in range(4):
        sk.topk_idx.fill_(-3)
        st.out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(sk.topk_idx, ref[0]), f"replay {it}: top-K differs"
        assert torch.equal(st.out.view(torch.int16), ref[1].view(torch.int16)), f"replay {it}: output differs"
        junk = torch.randn(1 << 20, device="cuda").sum().item()   # eager work between replays
        assert junk == junk


@pytest.mark.parametrize("shape", [(2, 8, 2, 16, 9000, 300, 64), (1, 14, 2, 32, 5000, 64, 32),
                                   (2, 8, 2, 16, 40000, 512, 128), (1, 3, 3, 16, 700, 700, 16),
                                   (2, 8, 2, 1, 9000, 300, 64), (1, 7, 1, 1, 40000, 512, 128),
                                   (2, 8, 2, 16, 9000, 300, 64, "f32"), (3, 16, 2, 16, 3000, 2500, 200)])
def test_group_shared_selection(oracle, shape):
    """One selection per KV head (sum of the group's scores), against the oracle: rotated queries per
    head, group scores, the shared top-K, and the attention of every head over the shared rows (bf16
    caches with up to 8 heads per KV head: the matrix-core kernel; float32 caches: the per-head kernel)."""
    Bn, Hq, Hkv, M, N, K, w = shape[:7]
    if M == 1:   # the single codebook of 4096
        wl = _single("shared_single", Bn, Hq, Hkv, N, K, w, seed=N + Hq)
    else:
        wl = synth.Workload("shared", Bn, Hq, Hkv, 128, M, N, K, w, seed=N + Hq,
                            kv_dtype=shape[7] if len(shape) > 7 else "bf16")
    x = synth.make_decode_inputs(wl)
    xd = H.to_dev(x)
    n_sink = 4 if N < 6000 else 0
    st, sk = _group_shared_step(wl, xd, n_sink=n_sink)
    G = wl.group
    qrot = oracle.rope(x["q"], x["inv_freq"], wl.wrope_b)
    err = np.abs(st.q_rot.cpu().numpy() - qrot)
    assert (err <= 2e-6 * np.maximum(1.0, np.abs(qrot))).all()
    grp = oracle.group_scores(oracle.scores_explicit(qrot, x["codebook"], x["codes"], N), Hkv)
    H.check_scores(sk.scores.cpu().numpy()[:, :, :N].astype(np.float64), grp, "group scores")
    idx, cnt, kth = oracle.topk(grp, K, w, n_sink)
    exc, slots = H.compare_topk(sk.topk_idx.cpu().numpy(), sk.topk_count.cpu().numpy(), idx, cnt, grp, kth)
    H.log(f"shared {shape}: {exc} near-tie exclusions in {slots} slots")
    # every head of a group attends the group's rows (the GPU's own selection, so that a near-tie
    # exclusion above does not leak into the attention comparison)
    g_idx = np.repeat(sk.topk_idx.cpu().numpy(), G, axis=1)
    g_cnt = np.repeat(sk.topk_count.cpu().numpy(), G, axis=1)
    want = oracle.sparse_attn(x["q"], x["k"], x["v"], g_idx, g_cnt, N, w, n_sink, x["inv_freq"], float(wl.wrope_b))
    aerr = np.abs(st.out.float().cpu().numpy().astype(np.float64) - want).max()
    H.log(f"shared {shape}: attention max error {aerr:.3e}")
    assert aerr <= (2e-2 if wl.kv_dtype == "bf16" else 2e-4), aerr


def test_group_shared_selection_ragged(oracle):
    """Shared selection with ragged lengths (a full sequence, one shorter than window + top-K, one shorter
    than the window, an empty one) and sinks: the matrix-core attention against the oracle."""
    wl = synth.Workload("shared_ragged", 4, 8, 2, 128, 16, 20000, 600, 128, seed=88)
    lens = [20000, 500, 90, 0]
    x = synth.make_decode_inputs(wl)
    st, sk = _group_shared_step(wl, H.to_dev(x), n_sink=4, want_scores=False, seq_lens=lens)
    sl = np.asarray(lens, dtype=np.int32)
    qrot = oracle.rope(x["q"], x["inv_freq"], wl.wrope_b)
    grp = oracle.group_scores(oracle.scores_explicit(qrot, x["codebook"], x["codes"], wl.ctx_len), wl.n_kv_heads)
    idx, cnt, kth = oracle.topk(grp, wl.top_k, wl.window, 4, sl)
    exc, slots = H.compare_topk(sk.topk_idx.cpu().numpy(), sk.topk_count.cpu().numpy(), idx, cnt, grp, kth)
    g_idx = np.repeat(sk.topk_idx.cpu().numpy(), wl.group, axis=1)
    g_cnt = np.repeat(sk.topk_count.cpu().numpy(), wl.group, axis=1)
    want = oracle.sparse_attn(x["q"], x["k"], x["v"], g_idx, g_cnt, wl.ctx_len, wl.window, 4, x["inv_freq"],
                              float(wl.wrope_b), sl)
    got = st.out.float().cpu().numpy().astype(np.float64)
    aerr = np.abs(got - want).max()
    H.log(f"shared ragged: {exc} near-tie exclusions in {slots} slots, attention max error {aerr:.3e}")
    assert aerr <= 2e-2, aerr
    assert np.abs(got[3]).max() == 0.0


def test_second_moment(oracle):
    """H = E[q~^T q~] per KV head from rotated query samples (heads of a KV head pooled), ragged sample
    counts included, against the oracle; it is positive definite enough for the encoder's Cholesky."""
    for Hq, Hkv, n in ((8, 2, 777), (3, 3, 1), (14, 2, 5000), (4, 1, 0)):
        wl = synth.Workload("moment", 1, Hq, Hkv, 128, 16, 64, 1, 1, seed=n)
        dims = H.dims_of(wl, 64)
        g = torch.Generator().manual_seed(n + Hq)
        q = torch.randn(max(n, 1), Hq, 128, generator=g) * torch.linspace(0.2, 3.0, 128)
        ws = torch.empty(B.workspace_bytes(dims, B.OP_FIT), dtype=torch.uint8, device="cuda")
        out = torch.full((Hkv, 128, 128), float("nan"), device="cuda")
        B.second_moment(dims, q.cuda(), n, out, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        if n == 0:
            assert (got == 0).all()
            continue
        want = oracle.second_moment(q[:n].numpy(), Hkv)
        err = np.abs(got - want)
        assert (err <= 2e-7 * np.maximum(1.0, np.abs(want))).all(), err.max()


@pytest.mark.parametrize("geometry", ["single", "pq16"])
def test_lloyd_iterations(oracle, geometry):
    """k-means under the query-aware distortion, three iterations of a2ats_encode_keys +
    a2ats_codebook_update from the same start as the oracle: assignments (near-ties excluded), counts
    and centroids agree at every iteration, empty codewords keep their value, and the query-aware
    objective J' never rises."""
    if geometry == "single":
        wl = _single("lloyd_single", 2, 4, 2, 3000, 1, 1, seed=12)
        mode, wkey = B.W_BLOCK, "h_block"
    else:
        wl = synth.Workload("lloyd_pq", 2, 4, 2, 128, 16, 3000, 1, 1, seed=12)
        mode, wkey = B.W_BLOCK, "h_block"
    hm = synth.make_query_second_moment(wl)
    n = 3000
    keys = synth.make_encode_keys(wl, n, stress=True)           # far from the start codebook: clusters move
    cb = synth.make_codebook(wl) * 0.5
    dims = H.dims_of(wl, n)
    ws_e = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(B.workspace_bytes(dims, B.OP_FIT), dtype=torch.uint8, device="cuda")
    kd, wd = keys.cuda(), hm[wkey].cuda()
    cb_g = cb.cuda()
    cb_o = cb.numpy().copy()
    cdt = torch.int16 if geometry == "single" else torch.uint8
    prev = None
    for it in range(3):
        codes = torch.zeros(wl.batch, wl.n_kv_heads, n, wl.n_sub, dtype=cdt, device="cuda")
        B.encode_keys(dims, kd, n, 0, cb_g, wd, mode, codes, ws_e)
        new_g = torch.empty_like(cb_g)
        counts = torch.empty(wl.n_kv_heads, wl.n_sub, wl.n_centroids, dtype=torch.int32, device="cuda")
        B.codebook_update(dims, kd, n, 0, codes, cb_g, new_g, counts, ws_f)
        torch.cuda.synchronize()
        got_codes = codes.cpu().numpy()
        got_codes = got_codes.view(np.uint16) if geometry == "single" else got_codes
        # the oracle's iteration from the GPU's current codebook (float32, as both sides store it)
        cur = cb_g.cpu().numpy()
        if geometry == "single":
            want_codes, b1, b2 = oracle.encode_cholesky(keys, cur, hm[wkey], want_margins=True)
        else:
            want_codes, b1, b2 = oracle.encode(keys, cur, hm[wkey], mode, want_margins=True)
        n_near = H.compare_codes(got_codes, want_codes, b1, b2)
        # centroid step checked on the GPU's own assignment, so that an excluded near-tie does not leak
        if geometry == "single":
            want_cb, want_counts = oracle.lloyd_update(keys, got_codes, cur)
        else:
            want_cb = np.empty(cur.shape, dtype=np.float64)
            want_counts = np.empty((wl.n_kv_heads, wl.n_sub, 256), dtype=np.int64)
            ds = wl.sub_dim
            for m in range(wl.n_sub):   # a product quantiser is M independent k-means problems
                c_m, n_m = oracle.lloyd_update(keys[..., m * ds:(m + 1) * ds], got_codes[..., m:m + 1], cur[:, m:m + 1])
                want_cb[:, m], want_counts[:, m] = c_m[:, 0], n_m
        np.testing.assert_array_equal(counts.cpu().numpy().reshape(want_counts.shape), want_counts)
        err = np.abs(new_g.cpu().numpy().astype(np.float64) - want_cb.reshape(cur.shape))
        assert (err <= 1e-6 * np.maximum(1.0, np.abs(want_cb.reshape(cur.shape)))).all(), err.max()
        empty = want_counts.reshape(-1) == 0
        assert geometry != "single" or empty.any()   # 6000 keys per KV head leave some of 4096 codewords without keys
        assert (new_g.cpu().numpy().reshape(empty.size, -1)[empty] == cur.reshape(empty.size, -1)[empty]).all()
        if geometry == "single":
            j = oracle.distortion(keys, new_g.cpu().numpy(), got_codes, hm["H"].numpy())
            if prev is not None:
                assert (j <= prev * (1 + 1e-6)).all(), (j, prev)
            prev = j
        H.log(f"{wl.name} iteration {it}: near-tie exclusions {n_near}, codewords in use {(~empty).sum()}")
        cb_g = new_g


def test_kv_cache_in_pinned_host_memory(oracle):
    """Heterogeneous placement (section 4.3 keeps the KV cache in host memory): the attention kernels
    read K and V rows straight from pinned host memory over PCIe; everything else stays in HBM."""
    wl = synth.Workload("kv_on_host", 2, 8, 2, 128, 16, 6000, 96, 64, seed=9)
    x = synth.make_decode_inputs(wl)
    xd = H.to_dev({k: v for k, v in x.items() if k not in ("k", "v")})
    kh, vh = x["k"].pin_memory(), x["v"].pin_memory()
    for t in (kh, vh):   # the address the device uses must be the one the call is given
        assert B.host_device_pointer(t) == t.data_ptr()
    dims = H.dims_of(wl, 6000)
    st = B.DecodeState(dims, wl.top_k, wl.window, 0, kh.dtype, x["inv_freq"], wl.wrope_b)
    B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
    B.score_topk(dims, xd["codes"], st.lut, st.lut_scale, wl.top_k, wl.window, 0, None, st.topk_idx, st.topk_count,
                 None, None, st.ws)
    B.sparse_attn(dims, xd["q"], st.q_rot, kh, vh, st.topk_idx, st.topk_count, wl.top_k, wl.window, 0, st.cos_win,
                  st.sin_win, None, st.out, st.ws)
    torch.cuda.synchronize()
    want = oracle.sparse_attn(x["q"], x["k"], x["v"], st.topk_idx.cpu().numpy(), st.topk_count.cpu().numpy(),
                              wl.ctx_len, wl.window, 0, x["inv_freq"], float(wl.wrope_b))
    aerr = np.abs(st.out.float().cpu().numpy().astype(np.float64) - want).max()
    assert aerr <= 2e-2, aerr


@pytest.mark.parametrize("mode", ["block", "none"])
def test_kmeanspp_seeding(oracle, mode):
    """The 4096 sequential k-means++ draws under the query-aware distortion follow the definition
    (same uniform numbers), and the seed codebook is exactly the drawn keys; duplicated keys included,
    so that zero distortions occur.  The oracle evaluates the definition in float64; the kernel rounds
    z = k L once to float32, which moves a distortion by at most 2.4e-7 of itself, hence a prefix sum
    and the target u * sum(d) by at most 5e-7 * sum(d) together.  The draws are sequential, so every
    draw is judged given the library's earlier draws (oracle.kmeanspp_check); a draw that differs from
    the definition's is excluded iff the target lies within 5e-7 * sum(d) of the library row's prefix
    interval.  Exclusions are counted and printed."""
    wl = _single("seed", 2, 4, 2, 2600, 1, 1, seed=17)
    hm = synth.make_query_second_moment(wl)
    n = 2600
    keys = synth.make_encode_keys(wl, n, stress=True)
    keys[:, :, 100:140] = keys[:, :, 60:100]                     # 40 duplicated keys per sequence
    g = torch.Generator().manual_seed(3)
    u = torch.rand(wl.n_kv_heads, 4096, generator=g, dtype=torch.float64)
    u[0, 7] = 0.0
    dims = H.dims_of(wl, n)
    ws = torch.empty(B.workspace_bytes(dims, B.OP_SEED), dtype=torch.uint8, device="cuda")
    out = torch.full((wl.n_kv_heads, 1, 4096, 128), float("nan"), device="cuda")
    picks = torch.full((wl.n_kv_heads, 4096), -1, dtype=torch.int32, device="cuda")
    w = hm["h_block"].cuda() if mode == "block" else None
    B.kmeanspp_seed(dims, keys.cuda(), n, w, B.W_BLOCK if mode == "block" else B.W_NONE, u.cuda(), out, picks, ws)
    torch.cuda.synchronize()
    hfull = hm["h_block"].numpy().astype(np.float64)[:, 0] if mode == "block" else None
    got = picks.cpu().numpy()
    n_equal, n_near, wrong = oracle.kmeanspp_check(keys, hfull, u.numpy(), got, 5e-7)
    print(f"k-means++ seeding ({mode}): draws compared {got.size}/{got.size}, equal {n_equal}, "
          f"excluded on a prefix boundary {n_near}, wrong {len(wrong)}")
    assert not wrong, f"draws that do not follow the definition: {wrong[:5]}"
    assert n_near <= got.size // 1000
    pooled = keys.permute(1, 0, 2, 3).reshape(wl.n_kv_heads, wl.batch * n, 128)
    for kv in range(wl.n_kv_heads):
        assert torch.equal(out[kv, 0].cpu(), pooled[kv][torch.as_tensor(got[kv].astype(np.int64))])


def test_query_aware_codebook_lowers_the_query_aware_distortion_on_a_mixture(oracle):
    """Section 4.2 end to end on the GPU (k-means++ seeding, then Lloyd iterations = a2ats_encode_keys +
    a2ats_codebook_update), once under the query-aware distortion with the full matrix H and once under
    the Euclidean one, on keys drawn from a mixture with correlated within-cluster spread.  The objective
    J' = sum (k - c) H (k - c)^T, evaluated by the oracle on each codebook's own final assignment, must
    not rise over the query-aware iterations and must end below the Euclidean codebook's."""
    wl = _single("fit_mixture", 4, 8, 2, 16384, 1, 1, seed=51)
    hm = synth.make_query_second_moment(wl)
    n = wl.ctx_len
    g = torch.Generator().manual_seed(9)
    centres = torch.randn(wl.n_kv_heads, 512, 128, generator=g)
    mix = torch.randn(128, 128, generator=g) / 128 ** 0.5
    which = torch.randint(0, 512, (wl.batch, wl.n_kv_heads, n), generator=g)
    keys = torch.stack([centres[kv][which[:, kv]] for kv in range(wl.n_kv_heads)], dim=1)
    keys = (keys + 0.6 * torch.randn(wl.batch, wl.n_kv_heads, n, 128, generator=g) @ mix).float().contiguous()
    u = torch.rand(wl.n_kv_heads, 4096, generator=g, dtype=torch.float64).cuda()
    dims = H.dims_of(wl, n)
    kd = keys.cuda()
    ws_e = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(B.workspace_bytes(dims, B.OP_FIT), dtype=torch.uint8, device="cuda")
    ws_s = torch.empty(B.workspace_bytes(dims, B.OP_SEED), dtype=torch.uint8, device="cuda")
    Hm = hm["H"].numpy()
    final = {}
    for name, mode, w in (("query-aware", B.W_BLOCK, hm["h_block"].cuda()), ("euclidean", B.W_NONE, None)):
        cb = torch.empty(wl.n_kv_heads, 1, 4096, 128, device="cuda")
        B.kmeanspp_seed(dims, kd, n, w, mode, u, cb, None, ws_s)
        trace = []
        codes = torch.zeros(wl.batch, wl.n_kv_heads, n, 1, dtype=torch.int16, device="cuda")
        for it in range(5):
            B.encode_keys(dims, kd, n, 0, cb, w, mode, codes, ws_e)
            torch.cuda.synchronize()
            trace.append(oracle.distortion(keys, cb.cpu().numpy(), codes.cpu().numpy().view(np.uint16), Hm))
            if it < 4:
                new = torch.empty_like(cb)
                B.codebook_update(dims, kd, n, 0, codes, cb, new, None, ws_f)
                cb = new
        final[name] = trace
        H.log(f"fit_mixture {name}: J' per KV head over the iterations {[t.round(1).tolist() for t in trace]}")
    aware, euclid = final["query-aware"], final["euclidean"]
    for a, b in zip(aware[1:], aware[:-1]):
        assert (a <= b * (1 + 1e-9)).all()          # assignment + mean under H never raise J'
    assert (aware[-1] < 0.98 * euclid[-1]).all(), (aware[-1], euclid[-1])   # measured 0.967


def test_single_codebook_step_in_a_hip_graph():
    """The decode step of the single-codebook geometry (append of one key on a prepared workspace, tables,
    selection, attention) and a prefill-sized encode, captured in HIP graphs: every replay must give the
    eager result, with eager work and synchronisations between the replays."""
    wl = _single("single_graph", 2, 8, 2, 40000, 700, 128, seed=6)
    xd = H.to_dev(synth.make_decode_inputs(wl))
    hm = synth.make_query_second_moment(wl)
    w = hm["h_block"].cuda()
    dims = H.dims_of(wl, 40000)
    st = B.DecodeState(dims, wl.top_k, wl.window, 0, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
    enc_ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    B.encode_prepare(dims, xd["codebook"], w, B.W_BLOCK, enc_ws)
    new_key = xd["k"][:, :, -1:, :].float().contiguous()
    many = synth.make_encode_keys(wl, 2000, stress=True).cuda()
    many_codes = torch.zeros(wl.batch, wl.n_kv_heads, 40000, 1, dtype=torch.int16, device="cuda")

    def step():
        B.encode_keys(dims, new_key, 1, wl.ctx_len - 1, xd["codebook"], w, B.W_BLOCK | B.W_PREPARED, xd["codes"], enc_ws)
        st.step(xd["q"], xd["codes"], xd["k"], xd["v"], xd["codebook"])
        B.encode_keys(dims, many, 2000, 5, xd["codebook"], w, B.W_BLOCK | B.W_PREPARED, many_codes, enc_ws)
    step()
    torch.cuda.synchronize()
    ref = (st.topk_idx.clone(), st.out.clone(), xd["codes"].clone(), many_codes.clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for it in range(3):
        st.topk_idx.fill_(-3)
        st.out.zero_()
        many_codes.zero_()
        xd["codes"][:, :, -1].fill_(0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(st.topk_idx, ref[0]), f"replay {it}: top-K differs"
        assert torch.equal(st.out.view(torch.int16), ref[1].view(torch.int16)), f"replay {it}: output differs"
        assert torch.equal(xd["codes"], ref[2]) and torch.equal(many_codes, ref[3]), f"replay {it}: codes differ"
        junk = torch.randn(1 << 20, device="cuda").sum().item()   # eager work between replays
        assert junk == junk


@pytest.mark.parametrize("page_size", [16, 256])
def test_paged_kv_cache(oracle, page_size):
    """K and V in pools of pages reached through a page table (pages of a sequence scattered over the pool,
    pools larger than needed, ragged lengths): the attention output must equal the contiguous layout's bit
    for bit, and so the oracle's within tolerance."""
    wl = synth.Workload("paged", 3, 8, 2, 128, 16, 5000, 200, 100, n_sink=4, seed=14)
    stride = 5120 if page_size == 256 else 5008
    x = synth.make_decode_inputs(wl, ctx_stride=stride)
    xd = H.to_dev(x)
    lens = [5000, 1234, 40]
    st = H.gpu_decode(wl, xd, seq_lens=lens, want_scores=False, ctx_stride=stride)
    ref = st.out.clone()
    n_pages_seq = stride // page_size
    n_phys = wl.batch * n_pages_seq + 7
    g = torch.Generator().manual_seed(page_size)
    perm = torch.randperm(n_phys, generator=g)[: wl.batch * n_pages_seq].reshape(wl.batch, n_pages_seq)
    pools = []
    for name in ("k", "v"):
        pool = torch.full((n_phys, wl.n_kv_heads, page_size, 128), float("nan"), dtype=x[name].dtype)
        pages = x[name].reshape(wl.batch, wl.n_kv_heads, n_pages_seq, page_size, 128).permute(0, 2, 1, 3, 4)
        pool[perm.reshape(-1)] = pages.reshape(-1, wl.n_kv_heads, page_size, 128)
        pools.append(pool.cuda())
    table = perm.to(torch.int32).cuda()
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    st.out.zero_()
    B.sparse_attn_paged(st.dims, xd["q"], st.q_rot, pools[0], pools[1], table, page_size, st.topk_idx, st.topk_count,
                        wl.top_k, wl.window, 4, st.cos_win, st.sin_win, sl, st.out, st.ws)
    torch.cuda.synchronize()
    assert torch.equal(st.out.view(torch.int16), ref.view(torch.int16))
    want = oracle.sparse_attn(x["q"], x["k"], x["v"], st.topk_idx.cpu().numpy(), st.topk_count.cpu().numpy(),
                              wl.ctx_len, wl.window, 4, x["inv_freq"], float(wl.wrope_b), np.asarray(lens, dtype=np.int32))
    assert np.abs(st.out.float().cpu().numpy().astype(np.float64) - want).max() <= 2e-2


def _page_codes(codes_cpu, page_size, seed, spare=5):
    """Scatter a contiguous code matrix [B, Hkv, stride, M] over a pool of pages [page][Hkv][page_size][M]
    (a random page per (sequence, slot), the pool larger than needed and poisoned elsewhere)."""
    Bn, Hkv, stride, M = codes_cpu.shape
    n_slots = stride // page_size
    n_phys = Bn * n_slots + spare
    perm = torch.randperm(n_phys, generator=torch.Generator().manual_seed(seed))[: Bn * n_slots].reshape(Bn, n_slots)
    pool = torch.full((n_phys, Hkv, page_size, M), 0xEE, dtype=torch.uint8)
    pages = codes_cpu.reshape(Bn, Hkv, n_slots, page_size, M).permute(0, 2, 1, 3, 4)
    pool[perm.reshape(-1)] = pages.reshape(-1, Hkv, page_size, M)
    return pool.cuda(), perm.to(torch.int32).cuda()


@pytest.mark.gpu
@pytest.mark.parametrize("case", ["exact_route", "stream_m16", "stream_m32_two_groups", "stream_long_chunks"])
def test_paged_code_matrix(case):
    """The code matrix in a pool of pages reached through a page table (the page table of the paged key/value
    cache): indices, counts, scores of the winners, the dense scores and the survivor statistics must equal
    those of the contiguous layout bit for bit -- on the exact route, on the streaming route with the page
    numbers staged in LDS (M = 16; M = 32 with two head groups per KV head) and with page numbers read from
    the table (chunks longer than the staged slice), with sinks and ragged lengths."""
    if case == "exact_route":
        wl, stride, lens, page_sizes = synth.Workload("pg1", 3, 8, 2, 128, 16, 5000, 200, 100, n_sink=4, seed=31), 5120, [5000, 1234, 40], (16, 256)
    elif case == "stream_m16":
        wl, stride, lens, page_sizes = synth.Workload("pg2", 3, 8, 2, 128, 16, 40000, 512, 128, n_sink=4, seed=32), 40960, [40000, 21111, 300], (16, 256)
    elif case == "stream_m32_two_groups":
        wl, stride, lens, page_sizes = synth.Workload("pg3", 2, 14, 2, 128, 32, 36000, 256, 64, n_sink=0, seed=33), 36864, [36000, 17000], (64,)
    else:   # 512 problems, so one chunk of 35984 rows each: 2250 pages of 16 tokens, more than the staged slice
        wl, stride, lens, page_sizes = synth.Workload("pg4", 64, 8, 8, 128, 16, 36000, 64, 16, n_sink=0, seed=34), 36864, None, (16,)
    x = synth.make_decode_inputs(wl, with_kv=False, ctx_stride=stride)
    xd = H.to_dev(x)
    want_scores = case != "stream_long_chunks"
    dims = H.dims_of(wl, stride)
    st = B.DecodeState(dims, wl.top_k, wl.window, wl.n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b,
                       want_scores=want_scores)
    sl = None if lens is None else torch.tensor(lens, dtype=torch.int32, device="cuda")
    B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
    B.score_topk(dims, xd["codes"], st.lut, st.lut_scale, wl.top_k, wl.window, wl.n_sink, sl, st.topk_idx,
                 st.topk_count, st.topk_score, st.scores if want_scores else None, st.ws)
    plan = B.score_topk_plan(st.dims, wl.top_k, wl.window, wl.n_sink)
    assert bool(plan["fast"]) == (case != "exact_route")
    heads = wl.batch * wl.n_q_heads
    ref_stats = torch.zeros(heads, dtype=torch.int32, device="cuda")
    B.score_topk_stats(st.dims, wl.top_k, wl.window, wl.n_sink, st.ws, ref_stats)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (st.topk_idx, st.topk_count, st.topk_score)] + [st.scores.clone() if want_scores else None]
    if case == "stream_long_chunks":
        assert plan["chunks"] == 1 and plan["rows_per_chunk"] // 16 > 2048
    for page_size in page_sizes:
        pool, table = _page_codes(x["codes"], page_size, seed=page_size)
        H.log(f"paged codes {case}: page size {page_size}, pool {tuple(pool.shape)}, plan {plan}")
        st.topk_idx.fill_(-7); st.topk_count.fill_(-7); st.topk_score.fill_(-7.0)
        if want_scores:
            st.scores.fill_(float("nan"))
        st.ws.zero_()
        B.score_topk_paged(st.dims, pool, table, page_size, st.lut, st.lut_scale, wl.top_k, wl.window, wl.n_sink, sl,
                           st.topk_idx, st.topk_count, st.topk_score, st.scores if want_scores else None, st.ws)
        stats = torch.zeros(heads, dtype=torch.int32, device="cuda")
        B.score_topk_stats(st.dims, wl.top_k, wl.window, wl.n_sink, st.ws, stats)
        torch.cuda.synchronize()
        assert torch.equal(st.topk_count, ref[1])
        assert torch.equal(st.topk_idx, ref[0])
        assert torch.equal(st.topk_score.view(torch.int32), ref[2].view(torch.int32))
        assert torch.equal(stats, ref_stats)
        if want_scores:
            n = torch.tensor(lens if lens is not None else [wl.ctx_len] * wl.batch, device="cuda")
            live = (torch.arange(stride, device="cuda")[None, :] < n[:, None])[:, None, :].expand_as(st.scores)
            assert torch.equal(st.scores[live].view(torch.int32), ref[3][live].view(torch.int32))


@pytest.mark.gpu
def test_paged_code_matrix_random_shapes():
    """Twelve seeded random shapes (batch, head grouping, M, context length, K, window, sinks, ragged lengths,
    page size): a2ats_score_topk_paged equals a2ats_score_topk bit for bit."""
    rng = np.random.default_rng(2024)
    for case in range(12):
        Bn = int(rng.integers(1, 4))
        Hkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 2, 4, 7]))
        M = int(rng.choice([16, 32]))
        N = int(rng.integers(17000, 45000))
        K = int(rng.choice([1, 64, 500, 2048]))
        w = int(rng.choice([0, 16, 128, 300]))
        n_sink = int(rng.choice([0, 4]))
        page = int(rng.choice([16, 32, 64, 128]))
        stride = (N + page - 1) // page * page
        lens = [int(N if i == 0 else rng.integers(0, N + 1)) for i in range(Bn)]
        wl = synth.Workload(f"pgr{case}", Bn, Hkv * G, Hkv, 128, M, N, K, w, n_sink=n_sink, seed=100 + case)
        x = synth.make_decode_inputs(wl, with_kv=False, ctx_stride=stride)
        xd = H.to_dev(x)
        dims = H.dims_of(wl, stride)
        st = B.DecodeState(dims, K, w, n_sink, xd["q"].dtype, xd["inv_freq"], wl.wrope_b)
        sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
        B.build_lut(dims, xd["q"], st.cos_b, st.sin_b, xd["codebook"], st.q_rot, st.lut, st.lut_scale)
        B.score_topk(dims, xd["codes"], st.lut, st.lut_scale, K, w, n_sink, sl, st.topk_idx, st.topk_count,
                     st.topk_score, None, st.ws)
        torch.cuda.synchronize()
        ref = [t.clone() for t in (st.topk_idx, st.topk_count, st.topk_score)]
        pool, table = _page_codes(x["codes"], page, seed=case)
        st.topk_idx.fill_(-7); st.topk_count.fill_(-7); st.topk_score.fill_(-7.0)
        B.score_topk_paged(dims, pool, table, page, st.lut, st.lut_scale, K, w, n_sink, sl, st.topk_idx,
                           st.topk_count, st.topk_score, None, st.ws)
        torch.cuda.synchronize()
        what = f"case {case}: B {Bn} Hkv {Hkv} G {G} M {M} N {N} K {K} w {w} sinks {n_sink} page {page} lens {lens}"
        assert torch.equal(st.topk_count, ref[1]), what
        assert torch.equal(st.topk_idx, ref[0]), what
        assert torch.equal(st.topk_score.view(torch.int32), ref[2].view(torch.int32)), what
        H.log("paged ok: " + what)


@pytest.mark.gpu
def test_codes_to_pages_append():
    """The append path of the paged code matrix: rows encoded into a staging buffer and copied through the
    page table land where the contiguous layout has them."""
    wl = synth.Workload("pg5", 3, 8, 2, 128, 16, 1000, 16, 16, seed=35)
    stride, page_size, n_new, pos0 = 1024, 16, 5, 990
    x = synth.make_decode_inputs(wl, ctx_stride=stride)
    pool, table = _page_codes(x["codes"], page_size, seed=7)
    fresh = torch.randint(0, 256, (wl.batch, wl.n_kv_heads, n_new, wl.n_sub), dtype=torch.uint8, device="cuda")
    dims = H.dims_of(wl, stride)
    B.codes_to_pages(dims, fresh, n_new, pos0, pool, table, page_size)
    torch.cuda.synchronize()
    want = x["codes"].clone()
    want[:, :, pos0:pos0 + n_new] = fresh.cpu()
    want_pool, _ = _page_codes(want, page_size, seed=7)
    assert torch.equal(pool, want_pool)
