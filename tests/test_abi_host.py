"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
plans workspaces, builds rotation tables, and rejects bad arguments before touching a GPU."""
import ctypes
import itertools
import math
import os
import re

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2502_12665_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2502_12665_amd import build
        build.build()
    return b


def test_every_declared_symbol_is_exported(binding):
    header = open(os.path.join(ROOT, "include", "a2ats.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(a2ats_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert binding.version() >= 100
    assert binding.status_string(0) == "ok" and "workspace" in binding.status_string(-3)


def test_dims_validation_and_plans(binding):
    good = binding.make_dims(4, 32, 8, 128, 16, 131072)
    assert binding.lut_elems(good) == 4 * 32 * 16 * 256 + 4 * 8 * 1 * 256 * 16 * 2 + 4 * 32 * 4
    g7 = binding.make_dims(2, 28, 4, 128, 32, 65536)
    assert binding.lut_elems(g7) == 2 * 28 * 32 * 256 + 2 * 4 * 2 * 256 * 32 * 2 + 2 * 28 * 4
    assert binding.workspace_bytes(good, binding.OP_LUT) == 0
    assert binding.workspace_bytes(good, binding.OP_SCORE_TOPK, 2048, 256) > 128 * 2048 * 24
    small = binding.make_dims(1, 4, 1, 128, 16, 4096)
    assert binding.workspace_bytes(small, binding.OP_SCORE_TOPK, 128, 64) == 0
    assert binding.workspace_bytes(good, binding.OP_ENCODE) == 8 * 16 * (64 + 256 * 8) * 4
    L = binding.lib()
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(16)      # non-NULL, aligned, never dereferenced: validation fails first

    def topk(d, top_k=8, window=4, n_sink=0, codes=one, ws=null, ws_bytes=0):
        return L.a2ats_score_topk(ctypes.byref(d), codes, one, one, top_k, window, n_sink, null, one, one,
                                  null, null, ws, ws_bytes, null)

    bad = binding.make_dims(1, 4, 3, 128, 16, 64)              # Hq % Hkv != 0
    assert topk(bad) == -1
    bad = binding.make_dims(1, 4, 1, 128, 16, 64, sub_dim=4)   # M * ds != D
    assert topk(bad) == -1
    bad = binding.make_dims(1, 4, 1, 128, 16, 64, ctx_stride=32)
    assert topk(bad) == -1
    assert topk(binding.make_dims(1, 4, 1, 64, 8, 64)) == -2           # head_dim 64 not compiled
    assert topk(binding.make_dims(1, 4, 1, 128, 16, 64, n_centroids=128, sub_dim=8)) == -2
    assert topk(binding.make_dims(1, 16, 1, 128, 16, 64)) == -2        # group of 16
    assert topk(small, top_k=-1) == -1
    assert topk(small, window=-1) == -1
    assert topk(small, codes=null) == -1
    assert topk(small, codes=ctypes.c_void_p(8)) == -1                 # misaligned code matrix
    assert topk(small, top_k=5000) == -2
    assert topk(good, top_k=2048, window=256) == -3                    # fast route needs a workspace
    assert topk(good, top_k=2048, window=256, ws=one, ws_bytes=1024) == -3
    rc = L.a2ats_build_lut(ctypes.byref(small), one, 7, one, one, one, one, one, one, null)
    assert rc == -1
    rc = L.a2ats_encode_keys(ctypes.byref(small), one, 4, 4094, one, null, 0, one, null, 0, null)
    assert rc == -1                                                     # pos0 + n_new > ctx_stride
    rc = L.a2ats_encode_keys(ctypes.byref(small), one, 4, 0, one, null, 1, one, null, 0, null)
    assert rc == -1                                                     # weighted mode without weights
    rc = L.a2ats_encode_keys(ctypes.byref(small), one, 4, 0, one, one, 2, one, null, 0, null)
    assert rc == -3
    rc = L.a2ats_sparse_attn(ctypes.byref(small), one, one, one, one, 3, one, one, 8, 4, 0, one, one, null,
                             one, null, 0, null)
    assert rc == -1                                                     # unknown dtype
    rc = L.a2ats_sparse_attn(ctypes.byref(good), one, one, one, one, 1, one, one, 2048, 256, 0, one, one,
                             null, one, null, 0, null)
    assert rc == -3                                                     # split attention needs a workspace
    with pytest.raises(binding.A2atsError):
        binding.workspace_bytes(bad, binding.OP_LUT)


def test_score_topk_plan_invariants(binding):
    """Host logic of a2ats_score_topk over a grid of shapes: whatever the batch, context, K and window,
    the plan must cover every candidate row exactly once with chunks of whole loop iterations, keep
    every survivor segment within what the 10-bit ranks address, keep the segments of a problem within
    what the final kernel handles (512), and ask for a workspace that holds them."""
    n_fast = 0
    for Bn, (Hq, Hkv, M), N, K, w, n_sink in itertools.product(
            (1, 2, 4, 16, 32, 64), ((4, 1, 16), (32, 8, 16), (28, 4, 32), (8, 8, 16), (64, 8, 32)),
            (4096, 16384 + 300, 32768, 65536, 131072, 500000, 1 << 20), (1, 64, 1024, 2048, 4096), (16, 256), (0, 4)):
        d = binding.make_dims(Bn, Hq, Hkv, 128, M, N)
        p = binding.score_topk_plan(d, K, w, n_sink)
        ncand = max(0, N - w - n_sink)
        ws = binding.workspace_bytes(d, binding.OP_SCORE_TOPK, K, w)
        if not p["fast"]:
            assert ncand < 16384 or K > 2048 or 4 * K > ncand or K < 1, (Bn, Hq, N, K, p)
            continue
        n_fast += 1
        G = Hq // Hkv
        assert ncand >= 16384 and 1 <= K <= 2048 and 4 * K <= ncand
        assert p["head_groups"] == (G + 3) // 4
        assert 1 <= p["sample_parts"] <= 8 and p["sample_rows"] <= 8192
        assert p["sample_parts"] * p["sample_rows"] <= ncand
        rpc, chunks, subs, sub_rows = p["rows_per_chunk"], p["chunks"], p["segments_per_wave"], p["rows_per_segment"]
        assert rpc % 512 == 0 and 1 <= chunks <= 64
        assert chunks * rpc >= ncand > (chunks - 1) * rpc                  # every row in exactly one chunk, none empty
        assert subs == 1 and sub_rows == rpc // 8                          # one survivor segment per wave
        assert chunks * 8 <= 512                                           # segments per problem
        cap = p["segment_capacity"]
        assert 64 <= cap and cap % 32 == 0 and cap <= sub_rows
        assert p["survivor_capacity"] >= 2 * K
        problems = Bn * Hkv * p["head_groups"]
        segs = problems * chunks * 8 * subs
        assert ws >= segs * (cap * (4 + M) + 32) + Bn * Hq * (4 * p["sample_parts"] + 4)
    assert n_fast > 500


def test_score_topk_workspace_covers_sink_counts(binding):
    """a2ats_workspace_bytes(OP_SCORE_TOPK) promises to cover every call with up to 64 sinks: over a grid
    of shapes it is at least what the plan of each such call asks for, and a call with one byte less
    than its plan is refused with the workspace status before anything else happens to `ws`."""
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)
    n = 0
    for Bn, (Hq, Hkv, M), N, K, w in itertools.product(
            (1, 4, 16), ((32, 8, 16), (28, 4, 32)), (16384 + 300, 16448, 32768, 32768 + 37, 65536, 131072, 1 << 20),
            (1, 1024, 2048), (0, 64, 256)):
        d = binding.make_dims(Bn, Hq, Hkv, 128, M, N)
        ws = binding.workspace_bytes(d, binding.OP_SCORE_TOPK, K, w)
        for n_sink in (0, 1, 3, 4, 17, 63, 64):
            p = binding.score_topk_plan(d, K, w, n_sink)
            need = p["workspace_bytes_div_256"] * 256 if p["fast"] else 0
            assert ws >= need, (Bn, Hq, N, K, w, n_sink, ws, p)
            if p["fast"]:
                n += 1
                rc = L.a2ats_score_topk(ctypes.byref(d), one, one, one, K, w, n_sink, null, one, one, null, null,
                                        one, need - 1, null)
                assert rc == -3
    assert n > 500


def test_decode_select_checks_every_argument_before_launching(binding):
    """a2ats_decode_select validates the union of the arguments of its two halves before the prologue is
    enqueued (shape of the fused route, then of the two-call route)."""
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)

    def call(d, top_k=2048, window=256, n_sink=0, codes=one, idx=one, cnt=one, ws=one, ws_bytes=1 << 40, n_new=1,
             pos0=None, keys=one):
        pos0 = d.ctx_len - 1 if pos0 is None else pos0
        return L.a2ats_decode_select(ctypes.byref(d), keys, n_new, pos0, one, null, 0, codes, one, 0, one, one, one,
                                     one, one, top_k, window, n_sink, null, idx, cnt, null, ws, ws_bytes, null)
    for d in (binding.make_dims(4, 32, 8, 128, 16, 131072), binding.make_dims(1, 4, 1, 128, 16, 4096)):
        assert call(d, top_k=-1) == -1
        assert call(d, window=-1) == -1
        assert call(d, n_sink=-1) == -1
        assert call(d, top_k=5000) == -2
        assert call(d, codes=null) == -1
        assert call(d, idx=null) == -1
        assert call(d, cnt=null) == -1
        assert call(d, n_new=33, pos0=0) == -2
        assert call(d, keys=null) == -1
        assert call(d, pos0=d.ctx_len) == -1
    big = binding.make_dims(4, 32, 8, 128, 16, 131072)
    assert call(big, ws=null, ws_bytes=0) == -3
    assert call(big, ws_bytes=1024) == -3


def test_decode_select_shared_checks_every_argument_before_launching(binding):
    """a2ats_decode_select_shared validates the union of the arguments of the three calls it stands for before
    anything is enqueued; the single codebook is not served."""
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)

    def call(d, top_k=2048, window=256, n_sink=0, codes=one, idx=one, cnt=one, ws=one, ws_bytes=1 << 40, n_new=1,
             pos0=None, keys=one, mode=0):
        pos0 = d.ctx_len - 1 if pos0 is None else pos0
        return L.a2ats_decode_select_shared(ctypes.byref(d), keys, n_new, pos0, one, null, mode, codes, one, 0, one,
                                            one, one, one, one, top_k, window, n_sink, null, idx, cnt, null, ws,
                                            ws_bytes, null)
    for d in (binding.make_dims(4, 32, 8, 128, 16, 131072), binding.make_dims(1, 4, 1, 128, 16, 4096)):
        assert call(d, top_k=-1) == -1
        assert call(d, window=-1) == -1
        assert call(d, n_sink=-1) == -1
        assert call(d, top_k=5000) == -2
        assert call(d, codes=null) == -1
        assert call(d, idx=null) == -1
        assert call(d, cnt=null) == -1
        assert call(d, n_new=33, pos0=0) == -2
        assert call(d, keys=null) == -1
        assert call(d, pos0=d.ctx_len) == -1
        assert call(d, mode=binding.W_DIAG) == -1      # weights missing
        assert call(d, mode=7) == -1
    big = binding.make_dims(4, 32, 8, 128, 16, 131072)
    assert call(big, ws=null, ws_bytes=0) == -3
    assert call(big, ws_bytes=1024) == -3
    assert call(binding.make_dims(2, 8, 2, 128, 1, 4096, n_centroids=4096)) == -2


def test_validation_of_the_single_codebook_and_construction_calls(binding):
    """Argument checks of the entry points added for the paper's own geometry (one codebook of 4096,
    16-bit codes), the selection shared per KV head and the offline construction: all on the host,
    before any launch."""
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)
    pq = binding.make_dims(2, 8, 2, 128, 16, 4096)
    sc = binding.make_dims(2, 8, 2, 128, 1, 4096, n_centroids=4096)
    assert binding.lut_elems(sc) == 2 * 8 * 4096
    assert binding.workspace_bytes(sc, binding.OP_SCORE_TOPK, 64, 16) == 0
    for op in (binding.OP_ENCODE, binding.OP_FIT, binding.OP_SEED):
        assert binding.workspace_bytes(sc, op) > 0
    assert binding.workspace_bytes(sc, binding.OP_SEED) > binding.workspace_bytes(sc, binding.OP_ENCODE)
    with pytest.raises(binding.A2atsError):
        binding.workspace_bytes(pq, binding.OP_SEED)                       # seeding: single codebook only
    # a codebook of 4096 needs M = 1, ds = 128
    assert L.a2ats_build_lut(ctypes.byref(binding.make_dims(1, 4, 1, 128, 16, 64, n_centroids=4096, sub_dim=8)),
                             one, 0, one, one, one, one, one, one, null) == -2
    # encoder: every mode needs the workspace; prepared flag accepted; bad mode refused
    assert L.a2ats_encode_keys(ctypes.byref(sc), one, 4, 0, one, null, 0, one, null, 0, null) == -3
    assert L.a2ats_encode_keys(ctypes.byref(sc), one, 4, 0, one, null, 0x100, one, one, 64, null) == -3
    assert L.a2ats_encode_keys(ctypes.byref(sc), one, 4, 0, one, null, 0x103, one, one, 1 << 40, null) == -1
    assert L.a2ats_encode_prepare(ctypes.byref(sc), one, null, 2, one, 1 << 40, null) == -1   # weights missing
    assert L.a2ats_encode_prepare(ctypes.byref(sc), one, one, 2, null, 0, null) == -3
    assert L.a2ats_encode_prepare(ctypes.byref(pq), one, one, 2, null, 0, null) == 0          # nothing to keep
    # fused prologue: at most 8 appended keys, and the encoder's workspace
    def prologue(d, n_new, ws, ws_bytes):
        return L.a2ats_decode_prologue(ctypes.byref(d), one, n_new, 0, one, null, 0, one, one, 0, one, one, one, one,
                                       one, ws, ws_bytes, null)
    assert prologue(sc, 9, one, 1 << 40) == -2
    assert prologue(sc, 1, null, 0) == -3 and prologue(sc, 1, one, 64) == -3
    assert prologue(pq, 33, null, 0) == -2
    # shared selection
    assert L.a2ats_build_lut_shared(ctypes.byref(pq), one, 0, one, one, one, null, one, one, null) == -1
    assert L.a2ats_sparse_attn_shared(ctypes.byref(pq), one, one, one, one, 1, one, one, 64, 16, 0, one, one, null,
                                      one, null, 0, null) == -3
    # paged key/value cache: a page table and a power-of-two page size of at least 16 tokens
    def paged(table, page_size):
        return L.a2ats_sparse_attn_paged(ctypes.byref(pq), one, one, one, one, 1, table, page_size, one, one, 64, 16, 0,
                                         one, one, null, one, one, 1 << 40, null)
    assert paged(null, 64) == -1 and paged(one, 48) == -1 and paged(one, 8) == -1
    # construction
    assert L.a2ats_second_moment(ctypes.byref(pq), one, -1, one, one, 1 << 40, null) == -1
    assert L.a2ats_second_moment(ctypes.byref(pq), one, 10, one, null, 0, null) == -3
    assert L.a2ats_codebook_update(ctypes.byref(pq), one, 4, 4094, one, one, one, null, one, 1 << 40, null) == -1
    assert L.a2ats_codebook_update(ctypes.byref(pq), one, 4, 0, one, one, null, null, one, 1 << 40, null) == -1
    assert L.a2ats_codebook_update(ctypes.byref(pq), one, 4, 0, one, one, one, null, one, 8, null) == -3
    assert L.a2ats_kmeanspp_seed(ctypes.byref(pq), one, 4, null, 0, one, one, null, one, 1 << 40, null) == -2
    assert L.a2ats_kmeanspp_seed(ctypes.byref(sc), one, 0, null, 0, one, one, null, one, 1 << 40, null) == -1
    assert L.a2ats_kmeanspp_seed(ctypes.byref(sc), one, 4, null, 2, one, one, null, one, 1 << 40, null) == -1
    assert L.a2ats_kmeanspp_seed(ctypes.byref(sc), one, 4, null, 0, one, one, null, one, 64, null) == -3


def test_rope_tables_against_numpy(binding):
    from paper_2502_12665_amd import synth
    inv = synth.inv_freq(128, 500000.0)
    cb, sb, cw, sw = binding.rope_tables(128, inv, 2048, 64)
    ang = 2048.0 * inv.numpy()
    np.testing.assert_array_equal(cb.numpy(), np.cos(ang).astype(np.float32))
    np.testing.assert_array_equal(sb.numpy(), np.sin(ang).astype(np.float32))
    d = np.arange(64, dtype=np.float64)[:, None] * inv.numpy()[None, :]
    np.testing.assert_array_equal(cw.numpy(), np.cos(d).astype(np.float32))
    np.testing.assert_array_equal(sw.numpy(), np.sin(d).astype(np.float32))
    assert cw[0].eq(1).all() and sw[0].eq(0).all()


def test_product_path_does_not_touch_the_oracle():
    """The package must not import or reference anything under oracle/ (no CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2502_12665_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", f
    text = open(os.path.join(pkg, "synth.py")).read()
    assert "import oracle" not in text and "from oracle" not in text


def test_static_scratch_entry_point_refuses_what_does_not_fit(binding):
    """a2ats_sparse_attn_static keeps its partial states in an 8 MiB array of the library: a shape that
    needs more is refused with the workspace status, and bad arguments with theirs, before any GPU call."""
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)

    def call(d, top_k=64, window=1024, n_sink=0, q=one):
        return L.a2ats_sparse_attn_static(ctypes.byref(d), q, one, one, one, 1, one, one, top_k, window, n_sink,
                                          one, one, null, one, null)
    huge = binding.make_dims(64, 64, 8, 128, 16, 8192)
    assert binding.workspace_bytes(huge, binding.OP_ATTN, 64, 1024) > 8 << 20
    assert call(huge) == -3
    assert call(huge, top_k=-1) == -1
    assert call(binding.make_dims(1, 4, 3, 128, 16, 64)) == -1



def test_paged_code_entry_points_check_their_arguments(binding):
    """a2ats_score_topk_paged and a2ats_codes_to_pages refuse a missing page table, a page size that is
    not a power of two of at least 16, the single-codebook geometry and rows outside the token capacity --
    all on the host, before any GPU call."""
    L = binding.lib()
    null, one = ctypes.c_void_p(0), ctypes.c_void_p(16)
    d = binding.make_dims(1, 8, 2, 128, 16, 4096)

    def topk(d, table=one, page=16, top_k=64):
        return L.a2ats_score_topk_paged(ctypes.byref(d), one, table, page, one, one, top_k, 64, 0, null, one, one,
                                        null, null, null, ctypes.c_size_t(0), null)
    assert topk(d, table=null) == -1
    for bad in (0, 8, 24, 100, -16):
        assert topk(d, page=bad) == -1
    assert topk(d, top_k=-1) == -1
    single = binding.make_dims(1, 8, 2, 128, 1, 4096, n_centroids=4096)
    assert topk(single) == -2
    big = binding.make_dims(4, 32, 8, 128, 16, 131072)       # streaming route: the workspace is checked too
    assert topk(big, top_k=2048) == -3

    def scatter(d, n_new=1, pos0=0, table=one, page=16, rows=one, pool=one):
        return L.a2ats_codes_to_pages(ctypes.byref(d), rows, n_new, pos0, pool, table, page, null)
    assert scatter(d, table=null) == -1
    assert scatter(d, page=48) == -1
    assert scatter(d, n_new=2, pos0=4095) == -1
    assert scatter(d, n_new=-1) == -1
    assert scatter(d, rows=null) == -1
    assert scatter(single) == -2


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: --gpus 2 exits with a message and a non-zero status before touching a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr
