#!/usr/bin/env python3
"""Benchmark of the A2ATS decode-time retrieval path on one MI355X.

A step is one pass of the whole hot path for one transformer layer over one batch:
encode the current token's key (query-aware distortion, one key per sequence and KV head),
rotate the query and build the lookup tables, score every cached token and select the top-K,
run selective attention.  Inputs are synthetic (seeded) and resident in HBM before the timed
region.  To keep the 256 MB Infinity Cache from serving the code matrix, the step rotates
over R independent replicas of every input (R "layers"), so consecutive touches of one
replica are separated by the other replicas' traffic.

Prints ONE JSON line (see the keys below); `value` is scored key rows per second over whole
steps.  The `roofline` object is for the code-streaming kernel, timed with HIP events
recorded by the library immediately around that launch.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


class HipEvents:
    """Raw hipEvent_t pairs (the library records them on the stream it launches on)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.ev = []
        for _ in range(2 * n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            assert rc == 0, rc
            self.ev.append(e)

    def pair(self, i):
        return self.ev[2 * i].value, self.ev[2 * i + 1].value

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[2 * i], self.ev[2 * i + 1])
        assert rc == 0, rc
        return ms.value


def _summary_commit(path):
    """The 'source commit:' line a summary under profiles/ carries (the commit whose build it profiled)."""
    try:
        for line in open(path):
            if line.lower().startswith("source commit:"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def measured_traffic(workload):
    """HBM bytes per launch of the streaming kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what it reads for a plain copy of known size).
    Counters cannot be collected from inside this process, so the figure is the one of the
    profile of this same command; (None, None) if there is no summary for the workload.
    Returns (bytes, where the figure comes from)."""
    rel = os.path.join("profiles", f"stream_select_{workload}_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    try:
        for line in open(path):
            if line.startswith("stream_select traffic_bytes_per_launch ="):
                return float(line.split("=")[1]), (f"{rel} (rocprofv3 --pmc runs of this command at commit "
                                                   f"{_summary_commit(path)}; read from the file, not measured "
                                                   "in this run)")
    except OSError:
        pass
    return None, None


def profiled_kernel_us(workload):
    """Average duration of the streaming kernel in the committed rocprofv3 --kernel-trace summary of
    this command ((None, None) if there is none): the event pair above also covers the dispatch
    between two commands, which the profiler's kernel time does not.  Returns (us, source)."""
    rel = os.path.join("profiles", f"decode_step_{workload}_kernel_stats.txt")
    path = os.path.join(ROOT, rel)
    try:
        for line in open(path):
            if line.startswith("a2ats::stream_select_kernel"):
                return float(line.split()[2]), (f"{rel} (rocprofv3 --kernel-trace --stats of this command at commit "
                                                f"{_summary_commit(path)}; read from the file, not measured in "
                                                "this run)")
    except (OSError, ValueError, IndexError):
        pass
    return None, None


def measured_machine_peaks(torch):
    """What this machine sustains on the two access patterns of the path, measured in this run with
    plain library kernels (for scale beside the nominal 8 TB/s): a 1 GiB device-to-device copy (bytes
    read + written) and a gather of 2^20 random 256-byte rows out of 4 GiB (bytes read + written)."""
    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * reps)]
        for r in range(reps):
            ev[2 * r].record()
            fn()
            ev[2 * r + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[2 * r].elapsed_time(ev[2 * r + 1]) for r in range(reps))[reps // 2] * 1e-3
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    t_copy = timed(lambda: dst.copy_(src))
    del dst
    rows = torch.empty((1 << 24, 128), dtype=torch.bfloat16, device="cuda")
    rows.view(torch.int16).random_(0, 100)
    idx = torch.randint(0, 1 << 24, (1 << 20,), device="cuda")
    out = torch.empty((1 << 20, 128), dtype=torch.bfloat16, device="cuda")
    t_gather = timed(lambda: torch.index_select(rows, 0, idx, out=out))
    del src, rows, idx, out
    return {"copy_1GiB_read_plus_write_GBps": 2 * (1 << 30) / t_copy / 1e9,
            "gather_256B_rows_read_plus_write_GBps": 2 * (1 << 20) * 256 / t_gather / 1e9,
            "note": "torch library kernels, measured in this run; nominal peak 8000 GB/s"}


def encode_prefill(args, torch, B, synth):
    """Prefill side: a2ats_encode_keys over whole sequences under the per-dimension query-aware
    distortion.  One step = one call over all keys; the bound is the vector ALU."""
    wl = synth.WORKLOADS["c5_qwen7b_64k"]   # all 32 sequences: 8.4 M keys, 4.3 GB of float32 keys
    N, M = wl.ctx_len, wl.n_sub
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl, "cuda")
    keys = synth.make_encode_keys(wl, N, device="cuda")
    dims = B.make_dims(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sub, wl.ctx_len)
    ws = torch.empty(max(B.workspace_bytes(dims, B.OP_ENCODE), 16), dtype=torch.uint8, device="cuda")
    codes = torch.empty(wl.batch, wl.n_kv_heads, N, M, dtype=torch.uint8, device="cuda")
    w = hm["h_diag"].cuda()
    n_keys = wl.batch * wl.n_kv_heads * N
    steps, warmup = min(args.steps, 8), min(args.warmup, 2)
    for _ in range(warmup):
        B.encode_keys(dims, keys, N, 0, cb, w, B.W_DIAG, codes, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.encode_keys(dims, keys, N, 0, cb, w, B.W_DIAG, codes, ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    evals = n_keys * M * 256                       # (key subvector, centroid) distance evaluations
    # instruction mix of the inner loop (from the kernel's ISA, ds = 4): per evaluation 4 subtract,
    # 1 multiply + 3 fused multiply-add, and + add (index into the low mantissa bits), median-of-3,
    # minimum = 12 vector instructions; peak issue rate taken as the published 157.3 TFLOP/s / 2 flop
    # per FMA lane
    ops_per_eval = 12.0
    peak = 157.3e12 / 2 / 1e12
    achieved = evals * ops_per_eval / (ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "encoded keys/s (prefill-side query-aware key encoding, per-dimension weights)",
        "value": n_keys / (ms * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 distances, f64 re-check of near ties", "data": "synthetic",
        "config": {"workload": "c5_qwen7b_64k encode, all 32 sequences", "keys": n_keys, "n_sub": M,
                   "sub_dim": wl.sub_dim, "weights": "W_DIAG"},
        "roofline": {"kernel": "encode_kernel", "bound": "alu", "achieved": achieved, "peak": peak,
                     "unit": "T vector lane-instructions/s", "frac": achieved / peak, "traffic": None,
                     "distance_evaluations_per_s": evals / (ms * 1e-3)},
    }))


def paged_codes_phase(args, torch, B, synth, wl):
    """The score/top-K phase over a paged code matrix (pages of --paged-codes tokens scattered over a
    pool) beside the same phase over the contiguous matrix: same tables, same results, timed by events
    around the call, replicas cycled."""
    R = max(1, min(args.replicas, 4))
    page = args.paged_codes
    dims = B.make_dims(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sub, wl.ctx_len)
    N, K, w = wl.ctx_len, wl.top_k, wl.window
    assert N % page == 0, "--paged-codes must divide the context length"
    sts, reps = [], []
    for r in range(R):
        x = synth.make_decode_inputs(wl.replace(seed=wl.seed + r), device="cuda", with_kv=False)
        n_slots = N // page
        n_phys = wl.batch * n_slots + 3
        perm = torch.randperm(n_phys, device="cuda")[: wl.batch * n_slots].reshape(wl.batch, n_slots)
        pool = torch.zeros(n_phys, wl.n_kv_heads, page, wl.n_sub, dtype=torch.uint8, device="cuda")
        pool[perm.reshape(-1)] = x["codes"].reshape(wl.batch, wl.n_kv_heads, n_slots, page, wl.n_sub) \
            .permute(0, 2, 1, 3, 4).reshape(-1, wl.n_kv_heads, page, wl.n_sub)
        x["pool"], x["table"] = pool, perm.to(torch.int32)
        st = B.DecodeState(dims, K, w, wl.n_sink, x["q"].dtype, x["inv_freq"], wl.wrope_b)
        B.build_lut(dims, x["q"], st.cos_b, st.sin_b, x["codebook"], st.q_rot, st.lut, st.lut_scale)
        reps.append(x)
        sts.append(st)
    torch.cuda.synchronize()

    def timed(fn):
        ts = []
        for i in range(args.warmup + args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn(i % R)
            b.record()
            b.synchronize()
            if i >= args.warmup:
                ts.append(a.elapsed_time(b) * 1e3)
        return sorted(ts)[len(ts) // 2]

    def flat(r):
        x, st = reps[r], sts[r]
        B.score_topk(dims, x["codes"], st.lut, st.lut_scale, K, w, wl.n_sink, None, st.topk_idx, st.topk_count,
                     st.topk_score, None, st.ws)

    def paged(r):
        x, st = reps[r], sts[r]
        B.score_topk_paged(dims, x["pool"], x["table"], page, st.lut, st.lut_scale, K, w, wl.n_sink, None,
                           st.topk_idx, st.topk_count, st.topk_score, None, st.ws)

    flat(0)
    torch.cuda.synchronize()
    want = sts[0].topk_idx.clone()
    paged(0)
    torch.cuda.synchronize()
    same = bool(torch.equal(want, sts[0].topk_idx))
    t_flat, t_paged = timed(flat), timed(paged)
    rows = wl.batch * wl.n_kv_heads * N
    print(json.dumps({
        "metric": "scored keys/s, score/top-K phase over a PAGED code matrix (events around the call)",
        "value": rows / (t_paged * 1e-6), "unit": "keys/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_paged * 1e-3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 fixed-point scores", "data": "synthetic",
        "config": {"workload": wl.name + " score/top-K phase", "page_size": page, "replicas_cycled": R},
        "us_paged": t_paged, "us_contiguous": t_flat, "indices_equal_to_contiguous": same}))


def host_attention_step(args, torch, B, synth, wl):
    """The placement of section 4.3: K/V caches in (pinned) host memory, selection on the GPU, attention over
    the retrieved rows on the host CPU (a2ats_sparse_attn_host).  A step = a2ats_decode_select on the GPU,
    indices / counts / rotated queries to the host, host attention, output back to the GPU; wall clock per
    step, with the host kernel's share timed separately."""
    R = max(1, min(args.replicas, 2))
    dims = B.make_dims(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sub, wl.ctx_len)
    N, K, w = wl.ctx_len, wl.top_k, wl.window
    hm = synth.make_query_second_moment(wl)
    h_diag = hm["h_diag"].cuda()
    reps = []
    for r in range(R):
        x = synth.make_decode_inputs(wl.replace(seed=wl.seed + r), device="cuda")
        x["new_key"] = x["k"][:, :, N - 1:N, :].float().contiguous()
        for name in ("k", "v"):
            x[name] = x[name].cpu().pin_memory()
        x["q_h"] = x["q"].cpu().pin_memory()
        reps.append(x)
    st = B.DecodeState(dims, K, w, wl.n_sink, reps[0]["q"].dtype, reps[0]["inv_freq"], wl.wrope_b)
    pin = lambda t: torch.empty_like(t, device="cpu").pin_memory()
    idx_h, cnt_h, qrot_h, out_h = pin(st.topk_idx), pin(st.topk_count), pin(st.q_rot), pin(st.out)
    cos_h, sin_h = st.cos_win.cpu(), st.sin_win.cpu()
    t_host = []

    def step(i):
        x = reps[i % R]
        B.decode_select(dims, x["new_key"], 1, N - 1, x["codebook"], h_diag, B.W_DIAG, x["codes"], x["q"],
                        st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale, K, w, wl.n_sink, None, st.topk_idx,
                        st.topk_count, None, st.ws)
        idx_h.copy_(st.topk_idx, non_blocking=True)
        cnt_h.copy_(st.topk_count, non_blocking=True)
        qrot_h.copy_(st.q_rot, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.sparse_attn_host(dims, x["q_h"], qrot_h, x["k"], x["v"], idx_h, cnt_h, K, w, wl.n_sink, cos_h, sin_h,
                           None, out_h, args.host_threads)
        t_host.append(time.perf_counter() - t0)
        st.out.copy_(out_h, non_blocking=True)

    steps, warmup = min(args.steps, 16), min(args.warmup, 4)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t_host.clear()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    e = 2 if wl.kv_dtype == "bf16" else 4
    attn_bytes = wl.batch * wl.n_q_heads * (min(K, N - w) + w) * 2 * wl.head_dim * e   # rows each head reads
    host_ms = sorted(t_host)[len(t_host) // 2] * 1e3
    print(json.dumps({
        "metric": "scored keys/s, whole decode step with the K/V caches in host memory and the attention on the host CPU",
        "value": wl.batch * wl.n_kv_heads * N / (ms * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 fixed-point scores on the GPU; bf16 K/V with f32 accumulate on the CPU", "data": "synthetic",
        "config": {"workload": wl.name, "kv_cache": "pinned host memory", "attention": "host CPU",
                   "host_threads": args.host_threads or "OpenMP default", "replicas_cycled": R},
        "host_attention_ms_median": host_ms, "host_attention_bytes": attn_bytes,
        "host_attention_GBps": attn_bytes / (host_ms * 1e-3) / 1e9}))


def single_codebook_encode_prefill(args, torch, B, synth, wl):
    """Prefill side in the paper's own geometry: a2ats_encode_keys over whole sequences under the full
    D x D query-aware distortion (4096 distances over 128 dimensions per key, on the matrix cores)."""
    N, Hkv = wl.ctx_len, wl.n_kv_heads
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl, "cuda")
    keys = synth.make_encode_keys(wl, N, device="cuda")
    dims = B.make_dims(wl.batch, wl.n_q_heads, Hkv, wl.head_dim, 1, N, n_centroids=wl.n_centroids)
    ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    codes = torch.empty(wl.batch, Hkv, N, 1, dtype=torch.int16, device="cuda")
    w = hm["h_block"].cuda()
    n_keys = wl.batch * Hkv * N
    steps, warmup = min(args.steps, 8), min(args.warmup, 2)
    for _ in range(warmup):
        B.encode_keys(dims, keys, N, 0, cb, w, B.W_BLOCK, codes, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.encode_keys(dims, keys, N, 0, cb, w, B.W_BLOCK, codes, ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flop = n_keys * 4096.0 * 128.0 * 2.0           # the contraction [keys x 128] . [128 x 4096]
    achieved = flop / (ms * 1e-3) / 1e12
    peak = 2500.0                                  # dense bf16 matrix-core peak, TFLOP/s
    print(json.dumps({
        "metric": "encoded keys/s (prefill-side query-aware key encoding, one codebook of 4096, full D x D matrix H)",
        "value": n_keys / (ms * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 hi/lo split products with f32 accumulate; f64 transform and f64 re-check of near ties",
        "data": "synthetic",
        "config": {"workload": wl.name + " encode", "keys": n_keys, "codewords": 4096, "weights": "W_BLOCK"},
        "roofline": {"kernel": "encode_single_kernel (+ float64 transform, factor, codeword and re-check kernels)",
                     "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": None,
                     "executed_bf16_TFLOPs": 3.0 * achieved, "executed_frac": 3.0 * achieved / peak,
                     "note": "algorithmic flops; each term takes three bf16 products (hi.hi + hi.lo + lo.hi)"},
    }))


def single_codebook_step(args, torch, B, synth, wl):
    """Decode step in the paper's own geometry (one codebook of 4096 codewords per KV head, 16-bit codes,
    full D x D matrix H for the appended key)."""
    R = max(1, args.replicas)
    N, Bn, Hq, Hkv, D, K, w = wl.ctx_len, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.top_k, wl.window
    dims = B.make_dims(Bn, Hq, Hkv, D, 1, N, n_centroids=wl.n_centroids)
    reps = []
    for r in range(R):
        x = synth.make_decode_inputs(wl.replace(seed=wl.seed + r), device="cuda")
        x["new_key"] = x["k"][:, :, N - 1:N, :].float().contiguous()
        reps.append(x)
    hm = synth.make_query_second_moment(wl)
    h_block = hm["h_block"].cuda()
    st = B.DecodeState(dims, K, w, wl.n_sink, reps[0]["q"].dtype, reps[0]["inv_freq"], wl.wrope_b)
    enc_ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    # the factor of H and the transformed codewords depend on neither the step nor the sequence:
    # derived once per codebook, outside the steps (every input replica has a codebook of its own)
    for x in reps:
        x["enc_ws"] = torch.empty_like(enc_ws)
        B.encode_prepare(dims, x["codebook"], h_block, B.W_BLOCK, x["enc_ws"])

    def step(i, timed):
        x = reps[i % R]
        if timed:
            ev[i][0].record()
        if args.separate_prologue:
            B.encode_keys(dims, x["new_key"], 1, N - 1, x["codebook"], h_block, B.W_BLOCK | B.W_PREPARED,
                          x["codes"], x["enc_ws"])
            if timed:
                ev[i][1].record()
            B.build_lut(dims, x["q"], st.cos_b, st.sin_b, x["codebook"], st.q_rot, st.lut, st.lut_scale)
        else:   # the sweep of the key encoder, then the table build that also picks the code
            if timed:
                ev[i][1].record()
            B.decode_prologue(dims, x["new_key"], 1, N - 1, x["codebook"], h_block, B.W_BLOCK | B.W_PREPARED,
                              x["codes"], x["q"], st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale, x["enc_ws"])
        if timed:
            ev[i][2].record()
        B.score_topk(dims, x["codes"], st.lut, st.lut_scale, K, w, wl.n_sink, None, st.topk_idx, st.topk_count,
                     None, None, st.ws)
        if timed:
            ev[i][3].record()
        B.sparse_attn(dims, x["q"], st.q_rot, x["k"], x["v"], st.topk_idx, st.topk_count, K, w, wl.n_sink,
                      st.cos_win, st.sin_win, None, st.out, st.ws)
        if timed:
            ev[i][4].record()

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, False)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    med = lambda v: float(sorted(v)[len(v) // 2])
    ph = [med([ev[i][p].elapsed_time(ev[i][p + 1]) * 1e3 for i in range(args.steps)]) for p in range(4)]
    rows = Bn * Hkv * N
    kernel_bytes = rows * 2 + Bn * Hq * 4096 * 4 + Bn * Hq * K * 4   # codes once, tables, selected positions
    achieved = kernel_bytes / (ph[2] * 1e-6) / 1e9
    out = {
        "metric": "scored keys/s (whole decode step, single codebook of 4096: encode 1 key + WRoPE/LUT + score/top-K "
                  "+ sparse attention)",
        "value": rows / (ms * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "launch": "eager", "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 scores as ordered int32 keys; bf16 K/V with f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "batch": Bn, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "n_sub": 1,
                   "codewords": 4096, "ctx_len": N, "top_k": K, "window": w, "replicas_cycled": R},
        "us_per_decode_step": ms * 1e3,
        "prologue": "encode_keys + build_lut" if args.separate_prologue else "decode_prologue (two launches)",
        "phase_us_median": ({"encode_1key": ph[0], "wrope_lut": ph[1]} if args.separate_prologue else
                            {"encode_1key_and_wrope_lut": ph[1]}) | {"score_topk": ph[2], "sparse_attn": ph[3]},
        "roofline": {"kernel": "select_single_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": kernel_bytes,
                     "avg_launch_us": ph[2],
                     "note": "duration = events around the a2ats_score_topk call (one kernel)"},
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        x = reps[0]
        xc = {k: x[k].cpu() for k in ("q", "codes", "k", "v")}
        cb, inv, nk = x["codebook"].cpu(), x["inv_freq"], x["new_key"].cpu()
        n_rep, t0 = 0, time.perf_counter()
        while True:
            orc.encode_cholesky(nk, cb, hm["h_block"])
            qrot = orc.rope(xc["q"], inv, wl.wrope_b)
            sc = orc.scores_explicit(qrot, cb, xc["codes"], N)
            idx, cnt, kth = orc.topk(sc, K, w, wl.n_sink)
            orc.sparse_attn(xc["q"], xc["k"], xc["v"], idx, cnt, N, w, wl.n_sink, inv, float(wl.wrope_b))
            n_rep += 1
            dt = time.perf_counter() - t0
            if dt >= args.cpu_baseline_seconds or n_rep >= 64:
                break
        out["cpu_baseline"] = {"value": n_rep * rows / dt, "unit": "keys/s", "cores": orc.threads(), "kind": "oracle",
                               "sample": f"{n_rep} whole decode steps over the full batch of one input replica "
                                         f"({Bn * Hkv} (sequence, KV head) problems of {N} keys), {dt:.1f} s"}
    print(json.dumps(out))


def group_shared_step(args, torch, B, synth, wl):
    """Decode step with ONE selection per KV head (the group's summed score): shared tables, score/top-K
    over Hkv table heads, attention of all query heads over the shared rows."""
    R = max(1, args.replicas)
    N, Bn, Hq, Hkv, M, D, K, w = wl.ctx_len, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.n_sub, wl.head_dim, \
        wl.top_k, wl.window
    dims = B.make_dims(Bn, Hq, Hkv, D, M, N)
    dims_kv = B.make_dims(Bn, Hkv, Hkv, D, M, N)
    reps = []
    for r in range(R):
        x = synth.make_decode_inputs(wl.replace(seed=wl.seed + r), device="cuda")
        x["new_key"] = x["k"][:, :, N - 1:N, :].float().contiguous()
        reps.append(x)
    h_diag = synth.make_query_second_moment(wl)["h_diag"].cuda()
    st = B.DecodeState(dims, K, w, wl.n_sink, reps[0]["q"].dtype, reps[0]["inv_freq"], wl.wrope_b)
    sk = B.DecodeState(dims_kv, K, w, wl.n_sink, reps[0]["q"].dtype, reps[0]["inv_freq"], wl.wrope_b)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    kev = HipEvents(args.steps)

    def step(i, timed):
        # the steps timed for `value` make two calls (a2ats_decode_select_shared: append, shared tables and
        # threshold sampling in one launch, then the streaming and final kernels; a2ats_sparse_attn_shared);
        # the steps with events between the phases make the four separate calls
        x = reps[i % R]
        if not timed:
            B.decode_select_shared(dims, x["new_key"], 1, N - 1, x["codebook"], h_diag, B.W_DIAG, x["codes"], x["q"],
                                   st.cos_b, st.sin_b, st.q_rot, sk.lut, sk.lut_scale, K, w, wl.n_sink, None,
                                   sk.topk_idx, sk.topk_count, None, sk.ws)
            B.sparse_attn_shared(dims, x["q"], st.q_rot, x["k"], x["v"], sk.topk_idx, sk.topk_count, K, w,
                                 wl.n_sink, st.cos_win, st.sin_win, None, st.out, st.ws)
            return
        ev[i][0].record()
        B.encode_keys(dims, x["new_key"], 1, N - 1, x["codebook"], h_diag, B.W_DIAG, x["codes"], st.ws)
        ev[i][1].record()
        B.build_lut_shared(dims, x["q"], st.cos_b, st.sin_b, x["codebook"], st.q_rot, sk.lut, sk.lut_scale)
        ev[i][2].record()
        B.score_topk_profiled(dims_kv, x["codes"], sk.lut, sk.lut_scale, K, w, wl.n_sink, None, sk.topk_idx,
                              sk.topk_count, None, None, sk.ws, *kev.pair(i))
        ev[i][3].record()
        B.sparse_attn_shared(dims, x["q"], st.q_rot, x["k"], x["v"], sk.topk_idx, sk.topk_count, K, w, wl.n_sink,
                             st.cos_win, st.sin_win, None, st.out, st.ws)
        ev[i][4].record()

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, False)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    med = lambda v: float(sorted(v)[len(v) // 2])
    ph = [med([ev[i][p].elapsed_time(ev[i][p + 1]) * 1e3 for i in range(args.steps)]) for p in range(4)]
    k_us = sum(kev.elapsed_ms(i) * 1e3 for i in range(args.steps)) / args.steps
    rows = Bn * Hkv * N
    kernel_bytes = rows * M + Bn * Hkv * M * 256 * 4
    e = 2 if wl.kv_dtype == "bf16" else 4
    attn_bytes = Bn * Hkv * min(K, N - w) * 2 * D * e + Bn * Hkv * w * 2 * D * e   # rows once per KV head
    achieved = kernel_bytes / (k_us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "scored keys/s (whole decode step, one selection per KV head: encode 1 key + WRoPE/shared LUT + "
                  "score/top-K + sparse attention over shared rows)",
        "value": rows / (ms * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "launch": "eager", "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 fixed-point scores; bf16 K/V with f32 accumulate" if wl.kv_dtype == "bf16" else
                 "int32 fixed-point scores; f32 K/V",
        "data": "synthetic",
        "config": {"workload": wl.name + ", selection shared by the query heads of a KV head", "batch": Bn,
                   "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "n_sub": M, "ctx_len": N, "top_k": K,
                   "window": w, "replicas_cycled": R},
        "us_per_decode_step": ms * 1e3,
        "calls_per_step": "decode_select_shared (append, shared tables and threshold sampling in one launch, then the "
                          "streaming and final kernels), sparse_attn_shared",
        "phase_us_median": {"encode_1key": ph[0], "wrope_shared_lut": ph[1], "score_topk": ph[2], "sparse_attn": ph[3],
                            "note": "from steps made of encode_keys + build_lut_shared + score_topk + "
                                    "sparse_attn_shared with events between"},
        "sparse_attn_phase": {"algorithmic_bytes": attn_bytes, "GBps": attn_bytes / (ph[3] * 1e-6) / 1e9},
        "roofline": {"kernel": "stream_select_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": kernel_bytes, "avg_launch_us": k_us},
    }))


def codebook_fit(args, torch, B, synth, wl):
    """Offline codebook construction: one Lloyd iteration under the query-aware distortion (assignment by
    a2ats_encode_keys with the full matrix H, centroid step by a2ats_codebook_update) over whole sequences,
    and the second moment H itself from as many rotated query rows."""
    N, Hkv = wl.ctx_len, wl.n_kv_heads
    hm = synth.make_query_second_moment(wl)
    cb = synth.make_codebook(wl, "cuda")
    keys = synth.make_encode_keys(wl, N, device="cuda", stress=True)
    dims = B.make_dims(wl.batch, wl.n_q_heads, Hkv, wl.head_dim, wl.n_sub, N, n_centroids=wl.n_centroids)
    ws = torch.empty(B.workspace_bytes(dims, B.OP_ENCODE), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(B.workspace_bytes(dims, B.OP_FIT), dtype=torch.uint8, device="cuda")
    codes = torch.empty(wl.batch, Hkv, N, wl.n_sub, dtype=synth.code_dtype(wl), device="cuda")
    new_cb = torch.empty_like(cb)
    w = hm["h_block"].cuda()
    n_keys = wl.batch * Hkv * N
    q_rows = torch.randn(N, wl.n_q_heads, wl.head_dim, device="cuda")
    h_out = torch.empty(Hkv, wl.head_dim, wl.head_dim, device="cuda")
    steps, warmup = min(args.steps, 8), min(args.warmup, 2)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]

    def it(i, timed):
        if timed:
            ev[i][0].record()
        B.encode_keys(dims, keys, N, 0, cb, w, B.W_BLOCK, codes, ws)
        if timed:
            ev[i][1].record()
        B.codebook_update(dims, keys, N, 0, codes, cb, new_cb, None, ws_f)
        if timed:
            ev[i][2].record()
        B.second_moment(dims, q_rows, N, h_out, ws_f)
        if timed:
            ev[i][3].record()

    for i in range(warmup):
        it(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        it(i, False)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    for i in range(steps):
        it(i, True)
    torch.cuda.synchronize()
    med = lambda v: float(sorted(v)[len(v) // 2])
    ph = [med([ev[i][p].elapsed_time(ev[i][p + 1]) for i in range(steps)]) for p in range(3)]
    flop = n_keys * 4096.0 * 128.0 * 2.0
    # k-means++ seeding (4096 sequential draws, one workgroup per KV head) on a calibration-sized subset
    n_seed = 8192
    dims_s = B.make_dims(wl.batch, wl.n_q_heads, Hkv, wl.head_dim, wl.n_sub, n_seed, n_centroids=wl.n_centroids)
    ws_s = torch.empty(B.workspace_bytes(dims_s, B.OP_SEED), dtype=torch.uint8, device="cuda")
    u = torch.rand(Hkv, 4096, dtype=torch.float64, device="cuda")
    seed_keys = keys[:, :, :n_seed].contiguous()
    seed_cb = torch.empty_like(cb)
    B.kmeanspp_seed(dims_s, seed_keys, n_seed, w, B.W_BLOCK, u, seed_cb, None, ws_s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    B.kmeanspp_seed(dims_s, seed_keys, n_seed, w, B.W_BLOCK, u, seed_cb, None, ws_s)
    torch.cuda.synchronize()
    seed_ms = (time.perf_counter() - t0) * 1e3
    print(json.dumps({
        "metric": "keys/s per Lloyd iteration (query-aware k-means: assignment under the full matrix H + centroid "
                  "step; plus one second-moment accumulation)",
        "value": n_keys / (ms * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 split products / f64 re-check for the assignment; f64 sums for means and moments",
        "data": "synthetic",
        "config": {"workload": wl.name + " codebook construction", "keys": n_keys, "codewords": wl.n_centroids,
                   "query_rows": N * wl.n_q_heads},
        "phase_ms_median": {"assign": ph[0], "centroid_step": ph[1], "second_moment": ph[2]},
        "kmeanspp_seed_ms": {"keys_per_kv_head": wl.batch * n_seed, "ms": seed_ms},
        "roofline": {"kernel": "encode_single_kernel", "bound": "mfma", "achieved": flop / (ph[0] * 1e-3) / 1e12,
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": flop / (ph[0] * 1e-3) / 1e12 / 2500.0,
                     "traffic": None, "note": "algorithmic flops of the assignment over its whole call"},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="c4_long_128k")
    ap.add_argument("--replicas", type=int, default=8, help="independent input sets cycled through (cold cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-seconds", type=float, default=10.0,
                    help="the oracle repeats whole steps until this much time has passed")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP-graph replays")
    ap.add_argument("--separate-prologue", action="store_true",
                    help="a2ats_encode_keys and a2ats_build_lut as two launches instead of a2ats_decode_prologue")
    ap.add_argument("--two-calls", action="store_true",
                    help="a2ats_decode_prologue and a2ats_score_topk as two calls instead of a2ats_decode_select")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run 3 plain float32 copies (out = in + 0) of this many MiB, so that a "
                         "rocprofv3 --pmc run of this command holds a kernel of known HBM traffic")
    ap.add_argument("--group-shared", action="store_true",
                    help="one selection per KV head (sum of the group's scores) instead of one per query head; "
                         "prints a line of its own")
    ap.add_argument("--kv-on-host", action="store_true",
                    help="keep the K/V caches in pinned host memory; the attention kernels read the selected rows "
                         "over PCIe (codes, tables and everything else stay in HBM)")
    ap.add_argument("--codebook-fit", action="store_true",
                    help="offline codebook construction (single-codebook workloads): one Lloyd iteration and one "
                         "second-moment accumulation; prints a line of its own")
    ap.add_argument("--host-attention", action="store_true",
                    help="K/V caches in pinned host memory, selection on the GPU, attention on the host CPU "
                         "(a2ats_sparse_attn_host); prints a line of its own")
    ap.add_argument("--host-threads", type=int, default=0, help="threads of --host-attention (0: OpenMP default)")
    ap.add_argument("--paged-codes", type=int, default=0,
                    help="time the score/top-K phase over a code matrix in pages of this many tokens beside the "
                         "contiguous one; prints a line of its own")
    ap.add_argument("--encode-prefill", action="store_true",
                    help="measure the prefill-side key encoder (configuration 5 geometry, 8 of its 32 "
                         "sequences) instead of the decode step, and print its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_12665_amd import binding as B
    from paper_2502_12665_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    if wl.n_centroids == 4096:   # the paper's own quantiser geometry: lines of its own
        if args.codebook_fit:
            codebook_fit(args, torch, B, synth, wl)
        elif args.encode_prefill:
            single_codebook_encode_prefill(args, torch, B, synth, wl)
        else:
            single_codebook_step(args, torch, B, synth, wl)
        return
    if args.encode_prefill:
        encode_prefill(args, torch, B, synth)
        return
    if args.group_shared:
        group_shared_step(args, torch, B, synth, wl)
        return
    if args.paged_codes:
        paged_codes_phase(args, torch, B, synth, wl)
        return
    if args.host_attention:
        host_attention_step(args, torch, B, synth, wl)
        return
    R = max(1, args.replicas)
    dims = B.make_dims(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sub, wl.ctx_len)
    N, Bn, Hq, Hkv, M, D, K, w = wl.ctx_len, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.n_sub, wl.head_dim, \
        wl.top_k, wl.window

    # ---- inputs, resident in HBM
    reps = []
    for r in range(R):
        x = synth.make_decode_inputs(wl.replace(seed=wl.seed + r), device="cuda")
        x["new_key"] = x["k"][:, :, N - 1:N, :].float().contiguous()
        if args.kv_on_host:
            for name in ("k", "v"):
                host = x[name].cpu().pin_memory()
                assert B.host_device_pointer(host) == host.data_ptr()
                x[name + "_hbm"], x[name] = x[name], host
        reps.append(x)
    hm = synth.make_query_second_moment(wl)
    h_diag = hm["h_diag"].cuda()
    st = B.DecodeState(dims, K, w, wl.n_sink, reps[0]["q"].dtype, reps[0]["inv_freq"], wl.wrope_b)
    cand_counts = torch.empty(Bn, Hq, dtype=torch.int32, device="cuda")

    n_ev = args.steps
    kev = HipEvents(n_ev)
    phase_ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]

    def step(i, timed, stats=False):
        # The timed-for-`value` steps make two calls (a2ats_decode_select, a2ats_sparse_attn); the steps
        # that carry events between the phases use a2ats_decode_prologue + a2ats_score_topk instead (same
        # kernels except that the threshold sampling is a launch of its own), so that the phases can be
        # told apart.
        x = reps[i % R]
        fused = not (args.separate_prologue or args.two_calls or timed)
        if timed:
            phase_ev[i][0].record()
        if fused:
            B.decode_select(dims, x["new_key"], 1, N - 1, x["codebook"], h_diag, B.W_DIAG, x["codes"], x["q"],
                            st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale, K, w, wl.n_sink, None,
                            st.topk_idx, st.topk_count, None, st.ws)
        else:
            if args.separate_prologue:
                B.encode_keys(dims, x["new_key"], 1, N - 1, x["codebook"], h_diag, B.W_DIAG, x["codes"], st.ws)
                if timed:
                    phase_ev[i][1].record()
                B.build_lut(dims, x["q"], st.cos_b, st.sin_b, x["codebook"], st.q_rot, st.lut, st.lut_scale)
            else:   # the key encode and the table build in one launch
                if timed:
                    phase_ev[i][1].record()
                B.decode_prologue(dims, x["new_key"], 1, N - 1, x["codebook"], h_diag, B.W_DIAG, x["codes"],
                                  x["q"], st.cos_b, st.sin_b, st.q_rot, st.lut, st.lut_scale)
            if timed:
                phase_ev[i][2].record()
                B.score_topk_profiled(dims, x["codes"], st.lut, st.lut_scale, K, w, wl.n_sink, None, st.topk_idx,
                                      st.topk_count, None, None, st.ws, *kev.pair(i))
            else:
                B.score_topk(dims, x["codes"], st.lut, st.lut_scale, K, w, wl.n_sink, None, st.topk_idx,
                             st.topk_count, None, None, st.ws)
        if timed:
            phase_ev[i][3].record()
        elif stats:   # candidate-list sizes, read before the attention reuses the workspace
            B.score_topk_stats(dims, K, w, wl.n_sink, st.ws, cand_counts)
        B.sparse_attn(dims, x["q"], st.q_rot, x["k"], x["v"], st.topk_idx, st.topk_count, K, w, wl.n_sink,
                      st.cos_win, st.sin_win, None, st.out, st.ws)
        if timed:
            phase_ev[i][4].record()

    if args.calibration_copy_mib > 0:
        n = args.calibration_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i, False, stats=(i == 0))
    torch.cuda.synchronize()

    # ---- timed region 1: K whole steps, launched eagerly (the host runs ahead of the GPU) and, unless
    # --no-graph, also as replays of one captured HIP graph per replica; `value` takes the faster
    # of the two and `launch` says which.  Both regions time exactly K steps between two
    # device synchronisations.
    def timed_steps(run_one):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            run_one(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_eager = timed_steps(lambda i: step(i, False))
    ms_graph = None
    if not args.no_graph:
        graphs = []
        for r in range(R):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(r, False)
            graphs.append(g)
        for r in range(R):
            graphs[r].replay()
        ms_graph = timed_steps(lambda i: graphs[i % R].replay())
    # One graph holding R consecutive steps (one per replica), as a serving stack would capture the layers
    # of a model: the gap between two graph launches is then paid once per R steps.
    ms_graph_multi = None
    if not args.no_graph and R > 1 and args.steps % R == 0:
        big = torch.cuda.CUDAGraph()
        with torch.cuda.graph(big):
            for r in range(R):
                step(r, False)
        big.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // R):
            big.replay()
        torch.cuda.synchronize()
        ms_graph_multi = (time.perf_counter() - t0) * 1e3 / args.steps
    choices = [(ms_eager, "eager")]
    if ms_graph is not None:
        choices.append((ms_graph, "hip-graph replay"))
    if ms_graph_multi is not None:
        choices.append((ms_graph_multi, f"replay of one hip graph holding {R} steps"))
    ms_per_step, launch_name = min(choices)

    # ---- timed region 2: the same K steps launched eagerly with events between the phases and
    # around the streaming kernel (events cannot be read back from inside a graph)
    torch.cuda.synchronize()
    te0 = time.perf_counter()
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    te1 = time.perf_counter()

    ph = [[phase_ev[i][p].elapsed_time(phase_ev[i][p + 1]) * 1e3 for i in range(args.steps)] for p in range(4)]
    med = lambda v: float(sorted(v)[len(v) // 2])
    mean = lambda v: float(sum(v) / len(v))
    raw = cand_counts.cpu().numpy().astype("int64") & 0xFFFFFFFF
    fast_route = bool((raw != 0xFFFFFFFF).all())   # the exact-only route reports 0xFFFFFFFF
    cc, routes = raw & 0x0FFFFFFF, raw >> 28
    kern_us = [kev.elapsed_ms(i) * 1e3 for i in range(args.steps)] if fast_route else [float("nan")]

    rows = Bn * Hkv * N
    code_bytes = rows * M
    lut_bytes = Bn * Hq * M * 256 * 4
    idx_bytes = Bn * Hq * K * 4
    phase_bytes = code_bytes + lut_bytes + idx_bytes          # score + top-K phase
    kernel_bytes = code_bytes + lut_bytes                      # what the streaming kernel must read
    e = 2 if wl.kv_dtype == "bf16" else 4
    attn_bytes = Bn * Hq * min(K, N - w) * 2 * D * e + Bn * Hkv * w * 2 * D * e
    k_us = mean(kern_us)
    prof_us, prof_src = profiled_kernel_us(wl.name)
    traffic, traffic_src = measured_traffic(wl.name)
    achieved = kernel_bytes / (k_us * 1e-6) / 1e9 if k_us == k_us else None

    out = {
        "metric": "scored keys/s = B * Hkv * N code rows / time of the WHOLE decode step (encode 1 key + WRoPE/LUT + "
                  "score/top-K + sparse attention); the rate over the score/top-K phase alone is in score_topk_phase",
        "value": rows / (ms_per_step * 1e-3),
        "unit": "keys/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "launch": launch_name,
        "ms_per_step_eager": ms_eager, "ms_per_step_graph_replay": ms_graph,
        "ms_per_step_graph_of_R_steps": ms_graph_multi,
        "ms_per_step_eager_with_events": (te1 - te0) * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 fixed-point scores; bf16 K/V with f32 accumulate" if wl.kv_dtype == "bf16" else
                 "int32 fixed-point scores; f32 K/V",
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": Bn, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D,
                   "n_sub": M, "ctx_len": N, "top_k": K, "window": w, "replicas_cycled": R,
                   "kv_cache": "pinned host memory, read by the attention kernels over PCIe" if args.kv_on_host
                   else "HBM"},
        "us_per_decode_step": ms_per_step * 1e3,
        "calls_per_step": "encode_keys, build_lut, score_topk, sparse_attn" if args.separate_prologue else
                          ("decode_prologue, score_topk, sparse_attn" if args.two_calls else
                           "decode_select (prologue and threshold sampling in one launch, then the streaming and "
                           "final kernels), sparse_attn"),
        "phase_us_median": ({"encode_1key": med(ph[0]), "wrope_lut": med(ph[1])} if args.separate_prologue else
                            {"encode_1key_and_wrope_lut": med(ph[1])}) |
                           {"score_topk": med(ph[2]), "sparse_attn": med(ph[3]),
                            "note": "from steps made of decode_prologue + score_topk + sparse_attn with events between"},
        "score_topk_phase": {"scored_keys_per_s": rows / (med(ph[2]) * 1e-6),
                             "query_head_scores_per_s": Bn * Hq * N / (med(ph[2]) * 1e-6),
                             "algorithmic_bytes": phase_bytes,
                             "GBps": phase_bytes / (med(ph[2]) * 1e-6) / 1e9,
                             "frac_of_hbm_peak": phase_bytes / (med(ph[2]) * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "sparse_attn_phase": {"algorithmic_bytes": attn_bytes,
                              "GBps": attn_bytes / (med(ph[3]) * 1e-6) / 1e9,
                              "frac_of_hbm_peak": attn_bytes / (med(ph[3]) * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "survivors_per_head": {"mean": float(cc.mean()), "max": int(cc.max()), "min": int(cc.min()),
                               "heads_on_exact_fallback": int((routes != 0).sum())}
        if fast_route else None,
        "roofline": {"kernel": "stream_select_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": kernel_bytes,
                     "avg_launch_us": k_us if k_us == k_us else None,
                     "avg_launch_us_source": "HIP event pair attached to the kernel's dispatch, measured in this run",
                     "avg_launch_us_rocprofv3": prof_us, "rocprofv3_source": prof_src,
                     "frac_rocprofv3": (kernel_bytes / (prof_us * 1e-6) / 1e9 / HBM_PEAK_GBS) if prof_us else None},
        "measured_machine_peaks": measured_machine_peaks(torch),
    }

    if not args.no_cpu_baseline:
        # The oracle as it stands, on the host cores: whole decode steps over the full batch of one
        # replica, repeated until about ten seconds of CPU work have been spent.
        from oracle import oracle as orc
        x = reps[0]
        xc = {k: x[k].cpu() for k in ("q", "codes", "k", "v")}
        cb = x["codebook"].cpu()
        inv = x["inv_freq"]
        nk = x["new_key"].cpu()
        n_rep, t0 = 0, time.perf_counter()
        phase_s = [0.0] * 5
        while True:
            ts = [time.perf_counter()]
            orc.encode(nk, cb, hm["h_diag"], orc.W_DIAG)
            ts.append(time.perf_counter())
            qrot = orc.rope(xc["q"], inv, wl.wrope_b)
            ts.append(time.perf_counter())
            sc = orc.scores_explicit(qrot, cb, xc["codes"], N)
            ts.append(time.perf_counter())
            idx, cnt, kth = orc.topk(sc, K, w, wl.n_sink)
            ts.append(time.perf_counter())
            orc.sparse_attn(xc["q"], xc["k"], xc["v"], idx, cnt, N, w, wl.n_sink, inv, float(wl.wrope_b))
            ts.append(time.perf_counter())
            for i in range(5):
                phase_s[i] += ts[i + 1] - ts[i]
            n_rep += 1
            dt = time.perf_counter() - t0
            if dt >= args.cpu_baseline_seconds or n_rep >= 64:
                break
        out["cpu_baseline"] = {"value": n_rep * rows / dt, "unit": "keys/s", "cores": orc.threads(),
                               "kind": "oracle",
                               "phase_ms_per_step": dict(zip(("encode_1key", "rope", "scores_explicit", "topk_full_sort",
                                                              "sparse_attn"), (1e3 * v / n_rep for v in phase_s))),
                               "sample": f"{n_rep} whole decode steps (encode 1 key, rotate query, explicit-"
                                         f"reconstruction scores, full-sort top-K, selective attention) over the "
                                         f"full batch of one input replica ({Bn * Hkv} (sequence, KV head) "
                                         f"problems of {N} keys), {dt:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
