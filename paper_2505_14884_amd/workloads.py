"""Seeded synthetic workloads for batched decode-step Selective Head Attention.

This module only *produces inputs*: shapes, head layouts and sequence-length
mixes of the models the paper evaluates (OPT, LLaMA-2, LLaMA-3; Section 5,
"Experiment Setting", and the decode-shape description in Section 3.2), filled
with seeded Gaussian values.  It holds none of the method's arithmetic (no
router product, no top-k, no softmax) and is imported by the tests and the
bench on behalf of both the HIP path and the CPU oracle; neither of those two
imports the other.

Values are drawn in fp32 by ``torch.Generator`` on the requested device and
rounded to nearest-even to the storage type (fp16 or bf16).  The CPU and the
GPU generators produce different streams; a case is always generated once and
the *same bits* are handed to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import torch

_TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16}
DTYPE_CODE = {"f16": 0, "bf16": 1}  # values of polar_dtype in include/polar.h


@dataclass(frozen=True)
class ShaWorkload:
    """One decode-attention layer call: B requests, Hq query heads, Hkv KV heads."""

    name: str
    B: int          # requests in the batch
    Hq: int         # query heads
    Hkv: int        # key/value heads (selection units: heads for MHA, groups for GQA)
    d: int          # head dimension
    S: int          # KV-cache capacity per request, in rows
    k: int          # selection units kept per request
    D: int          # router input width (model hidden size)
    dtype: str      # "f16" | "bf16": storage type of q/K/V/hidden/Wr
    seq_lo: int = 0     # 0 => every request holds S rows; else n_b ~ U{seq_lo..S}
    peaky: float = 0.0  # fraction of key rows scaled by 8 before rounding
    seed: int = 0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def torch_dtype(self) -> torch.dtype:
        return _TORCH_DTYPE[self.dtype]

    @property
    def dtype_code(self) -> int:
        return DTYPE_CODE[self.dtype]

    def scaled(self, **kw) -> "ShaWorkload":
        return replace(self, **kw)


# The five configurations of the baseline description, in its order.
CONFIGS: Dict[str, ShaWorkload] = {
    "C1_tiny": ShaWorkload("C1_tiny", B=4, Hq=8, Hkv=8, d=64, S=256, k=4, D=512,
                           dtype="f16", seed=101),
    "C2_llama2_7b": ShaWorkload("C2_llama2_7b", B=32, Hq=32, Hkv=32, d=128, S=1920, k=16,
                                D=4096, dtype="f16", seed=102),
    "C3_llama3_8b_gqa": ShaWorkload("C3_llama3_8b_gqa", B=64, Hq=32, Hkv=8, d=128, S=4096,
                                    k=4, D=4096, dtype="bf16", seed=103),
    "C4_opt66b": ShaWorkload("C4_opt66b", B=128, Hq=72, Hkv=72, d=128, S=1920, k=36,
                             D=9216, dtype="f16", seed=104),
    "C5_ragged": ShaWorkload("C5_ragged", B=256, Hq=32, Hkv=32, d=128, S=8192, k=8,
                             D=4096, dtype="bf16", seq_lo=512, peaky=0.05, seed=105),
}

# Further decode shapes of the paper's evaluation (Section 5 and the kernel figures) used by the
# bench sweeps only: a 64-query-head / 8-group model at long context.
EXTRA_SHAPES: Dict[str, ShaWorkload] = {
    "X1_gqa8_s8192": ShaWorkload("X1_gqa8_s8192", B=32, Hq=64, Hkv=8, d=128, S=8192, k=4,
                                 D=8192, dtype="bf16", seed=106),
}


@dataclass(frozen=True)
class MlpWorkload:
    """First (up-projection) layer of a sparsified MLP at decode: B requests, hidden width K,
    N neurons of which the batch union of predicted-active ones is computed."""

    name: str
    B: int          # requests
    K: int          # model hidden size (contraction length)
    N: int          # feed-forward width (neurons)
    density: float  # target fraction of neurons in the batch union
    dtype: str
    seed: int = 0

    @property
    def torch_dtype(self) -> torch.dtype:
        return _TORCH_DTYPE[self.dtype]


# OPT-66B feed-forward shape (hidden 9216, 4x expansion) at the paper's kernel-figure batch size.
MLP_CONFIGS: Dict[str, MlpWorkload] = {
    "M1_tiny": MlpWorkload("M1_tiny", B=8, K=256, N=1024, density=0.3, dtype="f16", seed=201),
    "M2_opt66b_ffn": MlpWorkload("M2_opt66b_ffn", B=64, K=9216, N=36864, density=0.3,
                                 dtype="f16", seed=202),
}


def make_mlp_inputs(w: MlpWorkload, device="cpu"):
    """x [B,K] ~ N(0,1), W1 [N,K] ~ N(0,1/K) (one row per neuron) and per-request predicted
    neuron ids [B,kn]: every request draws kn = 5 % of a seeded "hot set" of density*N neurons,
    so the batch union covers most of the hot set (the union grows with B as in the paper's
    batch-activation study, while each request alone is sparse)."""
    g = _gen(device, w.seed * 7919 + 1)
    x = torch.randn((w.B, w.K), generator=g, device=device, dtype=torch.float32).to(w.torch_dtype)
    W1 = torch.empty((w.N, w.K), device=device, dtype=w.torch_dtype)
    step = max(1, (1 << 27) // w.K)
    for n0 in range(0, w.N, step):
        n1 = min(w.N, n0 + step)
        blk = torch.randn((n1 - n0, w.K), generator=g, device=device, dtype=torch.float32)
        W1[n0:n1] = (blk * (1.0 / math.sqrt(w.K))).to(w.torch_dtype)
    gc = _gen("cpu", w.seed * 7919 + 2)
    hot = torch.randperm(w.N, generator=gc)[: max(1, int(round(w.density * w.N)))]
    kn = max(1, int(round(0.05 * hot.numel())))
    rows = [hot[torch.randperm(hot.numel(), generator=gc)[:kn]] for _ in range(w.B)]
    topk = torch.stack(rows).to(torch.int32).to(device)
    return x, W1, topk


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_seqlens(w: ShaWorkload, device="cpu") -> torch.Tensor:
    """int32 [B]: S for every request, or integers uniform on [seq_lo, S] inclusive."""
    if w.seq_lo <= 0:
        return torch.full((w.B,), w.S, dtype=torch.int32, device=device)
    g = _gen("cpu", w.seed * 7919 + 3)
    n = torch.randint(w.seq_lo, w.S + 1, (w.B,), generator=g, dtype=torch.int32)
    return n.to(device)


def make_router_inputs(w: ShaWorkload, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """hidden [B, D] ~ N(0, 1) and Wr [D, Hkv] ~ N(0, 1/D) (variance), storage dtype."""
    g = _gen(device, w.seed * 7919 + 1)
    hidden = torch.randn((w.B, w.D), generator=g, device=device, dtype=torch.float32)
    Wr = torch.randn((w.D, w.Hkv), generator=g, device=device, dtype=torch.float32)
    Wr *= 1.0 / math.sqrt(w.D)
    return hidden.to(w.torch_dtype), Wr.to(w.torch_dtype)


def make_attention_inputs(w: ShaWorkload, device="cpu", poison_padding: bool = False,
                          seqlens: Optional[torch.Tensor] = None):
    """q [B, Hq, d], K and V [B, Hkv, S, d] in the storage dtype, seqlens int32 [B].

    Values are N(0, 1); with ``w.peaky`` > 0 that fraction of key rows (chosen
    i.i.d. per (request, head, row)) is multiplied by 8 before rounding, which
    makes the softmax peaky.  Rows at or beyond a request's length are zero, or
    NaN when ``poison_padding`` is set (nothing may read them).
    Generated one request at a time so the fp32 temporaries stay small.
    """
    dt = w.torch_dtype
    if seqlens is None:
        seqlens = make_seqlens(w, device)
    g = _gen(device, w.seed * 7919 + 2)
    q = torch.randn((w.B, w.Hq, w.d), generator=g, device=device, dtype=torch.float32).to(dt)
    K = torch.empty((w.B, w.Hkv, w.S, w.d), device=device, dtype=dt)
    V = torch.empty((w.B, w.Hkv, w.S, w.d), device=device, dtype=dt)
    n_host = seqlens.cpu().tolist()
    pad = float("nan") if poison_padding else 0.0
    for b in range(w.B):
        n = max(0, min(int(n_host[b]), w.S))
        if n > 0:
            kb = torch.randn((w.Hkv, n, w.d), generator=g, device=device, dtype=torch.float32)
            if w.peaky > 0.0:
                hot = torch.rand((w.Hkv, n, 1), generator=g, device=device) < w.peaky
                kb = torch.where(hot, kb * 8.0, kb)
            K[b, :, :n] = kb.to(dt)
            del kb
            vb = torch.randn((w.Hkv, n, w.d), generator=g, device=device, dtype=torch.float32)
            V[b, :, :n] = vb.to(dt)
            del vb
        if n < w.S:
            K[b, :, n:] = pad
            V[b, :, n:] = pad
    return q, K, V, seqlens


def random_head_idx(w: ShaWorkload, device="cpu", seed_offset: int = 0) -> torch.Tensor:
    """int32 [B, k]: an independent uniformly random k-subset of the Hkv units per request."""
    g = _gen("cpu", w.seed * 7919 + 4 + seed_offset)
    rows = [torch.randperm(w.Hkv, generator=g)[: w.k] for _ in range(w.B)]
    return torch.stack(rows).to(torch.int32).to(device)


def selected_kv_bytes(w: ShaWorkload, seqlens: torch.Tensor, k: Optional[int] = None) -> int:
    """Bytes of K and V rows that k selected units per request oblige a kernel to read."""
    k = w.k if k is None else k
    n = seqlens.to(torch.int64).clamp(0, w.S).sum().item()
    return int(n) * k * 2 * w.d * 2


def bits_u16(t: torch.Tensor):
    """The 16-bit patterns of an fp16/bf16 CPU tensor as a numpy uint16 array (no copy of values)."""
    import numpy as np

    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy().view(np.uint16)
