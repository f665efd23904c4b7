"""a2ats_sparse_attn_static (the entry point that allocates nothing: its partial attention states
live in an array inside the library) against a2ats_sparse_attn, through the C ABI: same inputs, same
kernels, so the outputs must be bit for bit equal.  Two calls in a row, the second on a smaller
input, so that what the first call left in the array cannot leak into the second."""
import pytest
import torch

from paper_2502_12665_amd import binding as B
from paper_2502_12665_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _both(wl, n_sink, seq_lens=None):
    x = synth.make_decode_inputs(wl)
    xd = H.to_dev(x)
    st = H.gpu_decode(wl, xd, seq_lens=seq_lens, n_sink=n_sink, want_scores=False)   # sparse_attn with a caller workspace
    want = st.out.clone()
    assert torch.isfinite(want.float()).all()
    sl = None if seq_lens is None else torch.as_tensor(seq_lens, dtype=torch.int32, device="cuda")
    got = torch.full_like(st.out, float("nan"))
    B.sparse_attn_static(st.dims, xd["q"], st.q_rot, xd["k"], xd["v"], st.topk_idx, st.topk_count, wl.top_k,
                         wl.window, n_sink, st.cos_win, st.sin_win, sl, got)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                       want.view(torch.int16 if want.dtype == torch.bfloat16 else torch.int32)), wl.name
    return int(B.workspace_bytes(st.dims, B.OP_ATTN, wl.top_k, wl.window))


def test_static_scratch_matches_the_caller_workspace_twice():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    big = synth.Workload("static_big", 4, 32, 8, 128, 16, 40000, 1024, 128, n_sink=4, seed=41)
    small = synth.Workload("static_small", 2, 8, 2, 128, 16, 3000, 64, 32, n_sink=0, kv_dtype="f32", seed=42)
    b1 = _both(big, 4, seq_lens=[40000, 31000, 40000, 777])
    b2 = _both(small, 0)
    H.log(f"static scratch: {b1} and {b2} bytes of partial states, both outputs bit-identical")
    assert b2 < b1 <= 8 << 20
