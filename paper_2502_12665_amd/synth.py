"""Seeded synthetic inputs for the A2ATS decode-time retrieval path.

This module only draws random numbers, gathers and casts.  It contains none of
the method's arithmetic (no rotation, no scoring, no selection, no attention, no
nearest-centroid search): the CPU oracle and the HIP library both consume the
arrays produced here and share nothing else.

The shapes follow the model geometry the paper evaluates (Llama-3.1-8B: 32 query
/ 8 KV heads, head dim 128; contexts of 16K-128K tokens; top-K of about 3% of
the context; a recent window of the order of 64 tokens; WRoPE offset b = 2048,
paper section 5.1 "Implementation Details" and appendix A).  The paper's own
workloads (RULER / LongBench prompts run through trained models) are not
available, so keys are "codeword + small noise" and queries / values are
standard normal, which gives uniformly random code bytes (the worst case for an
LDS gather) and near-Gaussian approximate scores.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch

N_CENTROIDS = 256


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_sub: int            # M
    ctx_len: int          # N, including the current token
    top_k: int
    window: int
    n_sink: int = 0
    kv_dtype: str = "bf16"   # "f32" or "bf16": dtype of q, K, V and of the output
    rope_base: float = 500000.0
    wrope_b: int = 2048      # paper section 5.1: b = 2048
    seed: int = 0
    n_centroids: int = 256   # codewords per subspace; above 256 the codes are 16 bits wide

    @property
    def sub_dim(self) -> int:
        return self.head_dim // self.n_sub

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations.
WORKLOADS: Dict[str, Workload] = {
    "c1_tiny": Workload("c1_tiny", 1, 4, 1, 128, 16, 4096, 128, 64,
                        kv_dtype="f32", rope_base=10000.0),
    "c2_llama8b_32k": Workload("c2_llama8b_32k", 1, 32, 8, 128, 16, 32768, 1024, 128),
    "c3_batched_32k": Workload("c3_batched_32k", 16, 32, 8, 128, 16, 32768, 1024, 128),
    "c4_long_128k": Workload("c4_long_128k", 4, 32, 8, 128, 16, 131072, 2048, 256),
    "c5_qwen7b_64k": Workload("c5_qwen7b_64k", 32, 28, 4, 128, 32, 65536, 2048, 128,
                              rope_base=1000000.0),
    # The paper's own vector-quantisation geometry (section 5.1): one codebook of 4096 codewords
    # per head over all 128 dimensions, on the shape of configuration 4.
    "p4_single_codebook_128k": Workload("p4_single_codebook_128k", 4, 32, 8, 128, 1, 131072, 2048, 256,
                                        n_centroids=4096),
}


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + stream)
    return g


def _torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def inv_freq(head_dim: int, base: float) -> torch.Tensor:
    """Per-pair inverse frequencies base^(-2t/D), t in [0, D/2), as float64 (CPU)."""
    t = torch.arange(head_dim // 2, dtype=torch.float64)
    return torch.exp(-(2.0 * t / head_dim) * math.log(base))


def code_dtype(wl: Workload) -> torch.dtype:
    """uint8 codes for up to 256 codewords, else 16-bit codes (stored as int16: values stay below 2^15)."""
    assert wl.n_centroids <= 32768
    return torch.uint8 if wl.n_centroids <= 256 else torch.int16


def make_codebook(wl: Workload, device="cpu") -> torch.Tensor:
    """[Hkv, M, L, ds] float32, standard normal."""
    g = _gen(wl.seed, 1, device)
    return torch.randn(wl.n_kv_heads, wl.n_sub, wl.n_centroids, wl.sub_dim,
                       generator=g, device=device, dtype=torch.float32)


def reconstruct(codebook: torch.Tensor, codes: torch.Tensor) -> torch.Tensor:
    """Concatenate the centroids a code row points at: [B,Hkv,n,M] -> [B,Hkv,n,D] float32.

    Pure gather; used to build "codeword + noise" keys."""
    B, Hkv, n, M = codes.shape
    ds = codebook.shape[-1]
    out = torch.empty(B, Hkv, n, M * ds, dtype=torch.float32, device=codes.device)
    m_idx = torch.arange(M, device=codes.device)[None, :]
    for b in range(B):
        for h in range(Hkv):
            out[b, h] = codebook[h][m_idx, codes[b, h].long()].reshape(n, M * ds)
    return out


def make_decode_inputs(wl: Workload, device="cpu", with_kv: bool = True,
                       ctx_stride: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """All tensors of one decode step.

    codebook [Hkv,M,L,ds] f32 ; codes [B,Hkv,S,M] u8 (i16 for L > 256) ; k,v [B,Hkv,S,D] kv_dtype ;
    q [B,Hq,D] kv_dtype ; inv_freq [D/2] f64 (CPU).  S = ctx_stride >= N; rows past N
    are filled with a recognisable pattern that must never be read as data."""
    dt = _torch_dtype(wl.kv_dtype)
    B, Hkv, N, M, D = wl.batch, wl.n_kv_heads, wl.ctx_len, wl.n_sub, wl.head_dim
    S = N if ctx_stride is None else int(ctx_stride)
    assert S >= N
    out: Dict[str, torch.Tensor] = {}
    cb = make_codebook(wl, device)
    out["codebook"] = cb
    cdt = code_dtype(wl)
    codes = torch.full((B, Hkv, S, M), wl.n_centroids - 1, dtype=cdt, device=device)
    codes[:, :, :N] = torch.randint(0, wl.n_centroids, (B, Hkv, N, M), generator=_gen(wl.seed, 2, device),
                                    device=device, dtype=torch.int32).to(cdt)
    out["codes"] = codes
    if with_kv:
        k = torch.full((B, Hkv, S, D), 7.0, dtype=dt, device=device)
        v = torch.full((B, Hkv, S, D), -7.0, dtype=dt, device=device)
        gk, gv = _gen(wl.seed, 3, device), _gen(wl.seed, 4, device)
        for b in range(B):   # per-sequence slices keep the float32 temporaries small
            rec = reconstruct(cb, codes[b:b + 1, :, :N])
            rec += 0.1 * torch.randn(rec.shape, generator=gk, device=device, dtype=torch.float32)
            k[b:b + 1, :, :N] = rec.to(dt)
            v[b:b + 1, :, :N] = torch.randn(1, Hkv, N, D, generator=gv, device=device,
                                            dtype=torch.float32).to(dt)
        out["k"], out["v"] = k, v
    out["q"] = torch.randn(B, wl.n_q_heads, D, generator=_gen(wl.seed, 5, device), device=device,
                           dtype=torch.float32).to(dt)
    out["inv_freq"] = inv_freq(D, wl.rope_base)
    return out


def make_query_second_moment(wl: Workload, device="cpu") -> Dict[str, torch.Tensor]:
    """A seeded positive-definite "query second moment" per KV head, H = A A^T / D + 0.05 I
    (dense, non-uniform, non-diagonal, like the matrices the paper's figure 2 describes),
    plus the two restrictions of it the encoder accepts:
      h_diag  [Hkv, D]          the diagonal of H
      h_block [Hkv, M, ds, ds]  the diagonal ds x ds blocks of H
    All float32 (H itself is returned in float64)."""
    D, M, ds = wl.head_dim, wl.n_sub, wl.sub_dim
    g = _gen(wl.seed, 6, "cpu")
    A = torch.randn(wl.n_kv_heads, D, D, generator=g, dtype=torch.float64)
    H = A @ A.transpose(1, 2) / D + 0.05 * torch.eye(D, dtype=torch.float64)
    h_diag = torch.diagonal(H, dim1=1, dim2=2).to(torch.float32).contiguous()
    h_block = torch.stack([H[:, m * ds:(m + 1) * ds, m * ds:(m + 1) * ds] for m in range(M)], dim=1)
    return {"H": H, "h_diag": h_diag.to(device), "h_block": h_block.to(torch.float32).contiguous().to(device)}


def make_encode_keys(wl: Workload, n_new: int, device="cpu", stress: bool = False,
                     batch: Optional[int] = None) -> torch.Tensor:
    """Pre-RoPE float32 keys to encode, [B, Hkv, n_new, D].

    Default: codeword + N(0, 0.1^2) noise around uniformly drawn codes.  stress=True
    draws keys ~ N(0,1), far from every centroid, where weighted and Euclidean
    assignments differ often."""
    B = wl.batch if batch is None else batch
    if stress:
        return torch.randn(B, wl.n_kv_heads, n_new, wl.head_dim, generator=_gen(wl.seed, 8, device),
                           device=device, dtype=torch.float32)
    cb = make_codebook(wl, device)
    codes = torch.randint(0, wl.n_centroids, (B, wl.n_kv_heads, n_new, wl.n_sub),
                          generator=_gen(wl.seed, 7, device), device=device, dtype=torch.int32).to(code_dtype(wl))
    keys = reconstruct(cb, codes)
    keys += 0.1 * torch.randn(keys.shape, generator=_gen(wl.seed, 9, device), device=device,
                              dtype=torch.float32)
    return keys
