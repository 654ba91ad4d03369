"""The allocation-free attention entry point (polar_sha_decode_static: split-KV scratch in the
library's own static device array) against polar_sha_decode with a caller's workspace: same
kernels, same plan, so the outputs must be equal bit for bit, and each must match the oracle to
the attention bar (2e-3 max-abs, skipped heads exactly +0.0).  Two calls in a row share the
array; the second is smaller, so stale records of the first lie beyond and between its own."""
import numpy as np
import pytest
import torch

import paper_2505_14884_amd as polar
from oracle import polar_oracle as orc
from paper_2505_14884_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-3


def one_call(w):
    print("\ncase no-alloc", w, flush=True)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV, poison_padding=True)
    head_idx = wl.random_head_idx(w, DEV)
    need = polar.sha_workspace_bytes(w.B, w.Hq, w.Hkv, w.S, w.d, w.k)
    assert 0 < need <= polar.binding.STATIC_SCRATCH_BYTES
    assert polar.sha_launches(w.B, w.Hq, w.Hkv, w.S, w.d, w.k) == 2      # the scratch is really used
    out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device=DEV)
    before = torch.cuda.memory_allocated()
    polar.sha_decode_static(q, K, V, seqlens, head_idx, w.k, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    ref = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)              # caller-owned workspace
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
    want = orc.sha_decode(wl.bits_u16(q), wl.bits_u16(K), wl.bits_u16(V), seqlens.cpu().numpy(),
                          head_idx.cpu().numpy(), w.k, w.dtype)
    got = out.cpu().numpy()
    err = float(np.abs(got - want).max())
    print("   max-abs error %.3e" % err, flush=True)
    assert np.isfinite(got).all() and err <= TOL
    assert (got.view(np.uint32)[(want == 0.0).all(axis=2)] == 0).all()


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    first = wl.ShaWorkload("static-1", B=7, Hq=24, Hkv=6, d=128, S=9000, k=3, D=64, dtype="bf16", seq_lo=100, seed=71)
    second = wl.ShaWorkload("static-2", B=3, Hq=8, Hkv=8, d=128, S=2500, k=5, D=64, dtype="f16", seq_lo=1, seed=72)
    one_call(first)
    one_call(second)       # smaller, right after: the array still holds the first call's records


def test_static_scratch_entry_point_under_graph_capture():
    """The callers it is for: a step recorded into a HIP graph with no workspace to hand over.  The
    first call on the GPU was made above (outside any capture); every replay, with eager work in
    between, must equal the eager result of the workspace entry point bit for bit."""
    w = wl.ShaWorkload("static-graph", B=5, Hq=8, Hkv=8, d=128, S=3000, k=3, D=64, dtype="f16", seq_lo=500, seed=73)
    print("\ncase no-alloc graph", w, flush=True)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV)
    head_idx = wl.random_head_idx(w, DEV)
    out = torch.zeros((w.B, w.Hq, w.d), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        polar.sha_decode_static(q, K, V, seqlens, head_idx, w.k, out)        # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        polar.sha_decode_static(q, K, V, seqlens, head_idx, w.k, out)
    gen = torch.Generator(device=DEV).manual_seed(9)
    for rep in range(3):
        q.copy_(torch.randn(q.shape, generator=gen, device=DEV).to(q.dtype))
        head_idx.copy_(wl.random_head_idx(w, DEV, seed_offset=rep + 1))
        ref = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)              # eager work in between, own workspace
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32)), "replay %d" % rep


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    # 256 requests x 32 heads x 8 chunks of 1024 rows x 130 floats: 34 MB of records
    B, Hq, Hkv, S, d, k = 256, 32, 32, 8192, 128, 32
    assert polar.sha_workspace_bytes(B, Hq, Hkv, S, d, k) > polar.binding.STATIC_SCRATCH_BYTES
    a = torch.zeros(16, dtype=torch.float16, device=DEV)
    L = polar.binding.lib()
    p = a.data_ptr()
    assert L.polar_sha_decode_static(p, p, p, p, p, p, B, Hq, Hkv, S, d, k, 0, 0.0, None) == -3    # POLAR_EWORKSPACE
