"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments with the documented status before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2505_14884_amd as polar
from paper_2505_14884_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, EINVAL, EUNSUPPORTED, EWORKSPACE = 0, -1, -2, -3
FAKE = ctypes.c_void_p(0x1000)          # a non-NULL pointer that is never dereferenced on the host
ALIGNED = ctypes.c_void_p(0x10000)


def declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(polar_[a-z0-9_]+)\s*\(", text)))


def test_libraries_export_every_declared_symbol():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["polar.h", "polar_probe.h"]
    for header, L, exports in (("polar.h", binding.lib(), binding.EXPORTS),
                               ("polar_probe.h", binding.probe_lib(), binding.PROBE_EXPORTS)):
        names = declared_functions(header)
        assert set(names) == set(exports)
        for name in names:
            assert getattr(L, name) is not None
    assert binding.lib().polar_version() >= 2000
    # the yardsticks live in their own library, not in the product
    for name in binding.PROBE_EXPORTS:
        assert not hasattr(binding.lib(), name)


def test_library_is_built_from_the_sources_in_the_tree():
    from paper_2505_14884_amd import build
    assert binding.lib().polar_source_hash().decode() == build.source_hash()


def test_options():
    L = binding.lib()
    v = ctypes.c_int(-1)
    for name, opt in binding.OPTIONS.items():
        assert L.polar_get_option(opt, ctypes.byref(v)) == OK and v.value == 0, name     # all automatic
    assert L.polar_set_option(8, 0) == EINVAL and L.polar_set_option(-1, 0) == EINVAL
    assert L.polar_get_option(8, ctypes.byref(v)) == EINVAL
    assert L.polar_get_option(0, None) == EINVAL
    bad = {"sha_chunk_rows": [-1, 1, 127, (1 << 20) + 1], "sha_form": [-1, 3], "sha_grouped_kernel": [2, -1],
           "router_path": [3, -1], "router_phase1": [3], "gemm_form": [2], "gemm_workgroups": [257, -1],
           "union_form": [3, -1]}
    for name, values in bad.items():
        for value in values:
            assert L.polar_set_option(binding.OPTIONS[name], value) == EINVAL, (name, value)
            assert polar.get_option(name) == 0
    # options change the plan, and the workspace query follows; leaving the block restores them
    free = polar.sha_chunk_rows(32, 32, 32, 1920, 128, 16)
    size = polar.sha_workspace_bytes(32, 32, 32, 1920, 128, 16)
    with polar.options(sha_chunk_rows=200, sha_form=2):
        assert polar.get_option("sha_chunk_rows") == 200
        assert polar.sha_chunk_rows(32, 32, 32, 1920, 128, 16) == 256          # rounded up to 128 rows
        assert polar.sha_workspace_bytes(32, 32, 32, 1920, 128, 16) > size
        assert polar.sha_launches(32, 32, 32, 1920, 128, 16) == 2
    assert polar.sha_chunk_rows(32, 32, 32, 1920, 128, 16) == free and polar.get_option("sha_form") == 0
    assert polar.sha_launches(32, 32, 32, 1920, 128, 16) == 1
    # the vector-ALU grouped kernel exists for groups of 2, 4 and 8 only: forcing it elsewhere is a clean status
    with polar.options(sha_grouped_kernel=1):
        assert polar.sha_workspace_bytes(4, 24, 8, 256, 128, 4) == 0
        assert decode(L, Hq=24, Hkv=8, d=128, ws=None, ws_bytes=0) == EUNSUPPORTED
        assert decode(L, Hq=32, Hkv=8, d=128, ws=None, ws_bytes=0) == EWORKSPACE     # sizes pass, no launch
    assert polar.sha_workspace_bytes(4, 24, 8, 256, 128, 4) > 0


def test_strerror_covers_every_status():
    L = binding.lib()
    seen = {L.polar_strerror(s) for s in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and all(seen)
    assert L.polar_strerror(-99)
    assert L.polar_last_hip_error() == 0


def router(L, hidden=FAKE, Wr=FAKE, B=4, D=512, H=8, k=4, dt=0, idx=FAKE, ws=None, ws_bytes=0):
    return L.polar_router_topk(hidden, Wr, B, D, H, k, dt, idx, None, ws, ws_bytes, None)


def test_router_argument_errors():
    L = binding.lib()
    assert router(L, k=0) == EINVAL
    assert router(L, k=9) == EINVAL
    assert router(L, D=0) == EINVAL
    assert router(L, H=0) == EINVAL
    assert router(L, B=-1) == EINVAL
    assert router(L, dt=2) == EINVAL
    assert router(L, hidden=None) == EINVAL
    assert router(L, Wr=None) == EINVAL
    assert router(L, idx=None) == EINVAL
    assert router(L, H=257, k=4) == EUNSUPPORTED
    assert router(L, D=16385) == EUNSUPPORTED
    assert router(L, B=0, hidden=None, Wr=None, idx=None) == OK      # empty batch: no-op
    need = L.polar_router_workspace_bytes(4, 512, 8)
    assert need >= 4 * 8 * 8 and need % 256 == 0
    assert router(L, ws=ALIGNED, ws_bytes=need - 1) == EWORKSPACE
    assert router(L, ws=ctypes.c_void_p(0x10010), ws_bytes=need) == EWORKSPACE
    assert L.polar_router_workspace_bytes(4, 0, 8) == 0
    assert L.polar_router_workspace_bytes(4, 512, 257) == 0


def decode(L, q=ALIGNED, K=ALIGNED, V=ALIGNED, n=FAKE, idx=FAKE, out=ALIGNED, B=4, Hq=8, Hkv=8, S=256, d=64,
           k=4, dt=0, scale=0.0, ws=ALIGNED, ws_bytes=None):
    if ws_bytes is None:
        ws_bytes = L.polar_sha_workspace_bytes(B, Hq, Hkv, S, d, k)
    return L.polar_sha_decode(q, K, V, n, idx, out, B, Hq, Hkv, S, d, k, dt, scale, ws, ws_bytes, None)


def test_sha_argument_errors():
    L = binding.lib()
    assert decode(L, k=0) == EINVAL
    assert decode(L, k=9) == EINVAL
    assert decode(L, Hq=12, Hkv=8) == EINVAL                # Hq not a multiple of Hkv
    assert decode(L, S=0) == EINVAL
    assert decode(L, B=-2) == EINVAL
    assert decode(L, dt=7) == EINVAL
    assert decode(L, scale=-1.0) == EINVAL
    assert decode(L, scale=float("nan")) == EINVAL
    assert decode(L, scale=float("inf")) == EINVAL
    assert decode(L, idx=None, k=4) == EINVAL               # dense needs k == Hkv
    for name in ("q", "K", "V", "n", "out"):
        assert decode(L, **{name: None}) == EINVAL
    for name in ("q", "K", "V", "out"):                      # 16-byte accesses: misaligned pointers are refused
        assert decode(L, **{name: ctypes.c_void_p(0x10008)}) == EINVAL
    assert L.polar_sha_merge(FAKE, FAKE, ctypes.c_void_p(0x10004), 4, 8, 8, 256, 64, 4, ALIGNED, 1 << 20, None) == EINVAL
    assert decode(L, d=96) == EUNSUPPORTED
    assert decode(L, d=256) == EUNSUPPORTED
    assert decode(L, Hq=136, Hkv=8) == EUNSUPPORTED         # G = 17
    assert decode(L, Hq=24, Hkv=8, d=64) == EUNSUPPORTED    # G = 3 at d = 64
    assert decode(L, Hq=128, Hkv=8, d=64) == EUNSUPPORTED   # G = 16 at d = 64
    assert decode(L, ws=None) == EWORKSPACE
    assert decode(L, ws=ctypes.c_void_p(0x10010)) == EWORKSPACE   # not 256-byte aligned
    assert decode(L, ws_bytes=255) == EWORKSPACE
    assert decode(L, B=0, q=None, K=None, V=None, n=None, out=None, ws=None) == OK   # empty batch


def test_static_scratch_entry_point_argument_errors():
    """polar_sha_decode_static: polar_sha_decode's checks, plus the size limit of the library's own
    scratch array, all before any HIP call."""
    L = binding.lib()
    f = lambda q=ALIGNED, K=ALIGNED, V=ALIGNED, n=FAKE, idx=FAKE, out=ALIGNED, B=4, Hq=8, Hkv=8, S=256, d=64, k=4, dt=0, \
        scale=0.0: L.polar_sha_decode_static(q, K, V, n, idx, out, B, Hq, Hkv, S, d, k, dt, scale, None)
    assert f(k=0) == EINVAL and f(k=9) == EINVAL and f(Hq=12) == EINVAL and f(S=0) == EINVAL and f(B=-1) == EINVAL
    assert f(dt=5) == EINVAL and f(scale=-1.0) == EINVAL and f(idx=None) == EINVAL
    for name in ("q", "K", "V", "n", "out"):
        assert f(**{name: None}) == EINVAL
    assert f(q=ctypes.c_void_p(0x10008)) == EINVAL and f(out=ctypes.c_void_p(0x10004)) == EINVAL
    assert f(d=96) == EUNSUPPORTED and f(Hq=136) == EUNSUPPORTED
    assert f(B=0, q=None, K=None, V=None, n=None, out=None) == OK
    # 256 requests x 32 heads x 8 chunks x 130 floats of records do not fit 32 MiB; 24 heads do
    assert polar.sha_workspace_bytes(256, 32, 32, 8192, 128, 32) > binding.STATIC_SCRATCH_BYTES
    assert f(B=256, Hq=32, Hkv=32, S=8192, d=128, k=32) == EWORKSPACE
    assert polar.sha_workspace_bytes(256, 32, 32, 8192, 128, 24) <= binding.STATIC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "polar.h")).read()
    assert "#define POLAR_STATIC_SCRATCH_BYTES (32u << 20)" in text and binding.STATIC_SCRATCH_BYTES == 32 << 20


def test_layout_entry_points_share_the_checks():
    L = binding.lib()
    args = lambda layout, **kw: L.polar_sha_decode_layout(
        kw.get("q", ALIGNED), ALIGNED, ALIGNED, FAKE, FAKE, ALIGNED, 4, 8, 8, 256, kw.get("d", 64), 4, 0, layout,
        0.0, ALIGNED, L.polar_sha_workspace_bytes(4, 8, 8, 256, 64, 4), None)
    assert args(2) == EINVAL and args(-1) == EINVAL           # unknown layout
    assert args(1, q=None) == EINVAL
    assert args(1, d=96) == EUNSUPPORTED
    assert args(1, q=ctypes.c_void_p(0x10002)) == EINVAL
    assert L.polar_sha_partial_layout(ALIGNED, ALIGNED, ALIGNED, FAKE, FAKE, 4, 8, 8, 256, 64, 4, 0, 5, 0.0,
                                      ALIGNED, 1 << 20, None) == EINVAL


def test_head_norm_topk_argument_errors():
    L = binding.lib()
    f = lambda out=FAKE, B=4, Hq=8, Hkv=8, d=64, k=4, idx=FAKE: L.polar_head_norm_topk(
        out, B, Hq, Hkv, d, k, idx, None, None)
    assert f(k=0) == EINVAL and f(k=9) == EINVAL
    assert f(Hq=12) == EINVAL
    assert f(d=0) == EINVAL
    assert f(out=None) == EINVAL and f(idx=None) == EINVAL
    assert f(Hq=512, Hkv=512, k=4) == EUNSUPPORTED
    assert f(B=0, out=None, idx=None) == OK


def test_head_labels_argument_errors():
    L = binding.lib()
    need = L.polar_sha_workspace_bytes(4, 8, 8, 256, 64, 8)
    f = lambda q=ALIGNED, K=ALIGNED, V=ALIGNED, n=FAKE, labels=FAKE, out=None, B=4, Hq=8, Hkv=8, S=256, d=64, k=3, dt=0, \
        layout=0, scale=0.0, ws=ALIGNED, wsb=need: L.polar_head_labels(q, K, V, n, labels, None, out, B, Hq, Hkv, S, d, k,
                                                                      dt, layout, scale, ws, wsb, None)
    assert f(k=0) == EINVAL and f(k=9) == EINVAL and f(Hq=12) == EINVAL and f(S=0) == EINVAL and f(B=-1) == EINVAL
    assert f(dt=2) == EINVAL and f(layout=2) == EINVAL and f(scale=-1.0) == EINVAL
    assert f(labels=None) == EINVAL and f(out=ctypes.c_void_p(0x10008)) == EINVAL
    for name in ("q", "K", "V", "n"):
        assert f(**{name: None}) == EINVAL
    assert f(d=96) == EUNSUPPORTED and f(Hq=512, Hkv=512, k=4) == EUNSUPPORTED
    assert f(ws=None) == EWORKSPACE and f(wsb=need - 1) == EWORKSPACE
    assert f(B=0, q=None, K=None, V=None, n=None, labels=None, ws=None) == OK


def test_select_gemm_and_union_argument_errors():
    L = binding.lib()
    A16 = ctypes.c_void_p(0x1000)
    g = lambda A=A16, W=A16, idx=FAKE, C=FAKE, M=4, K=256, N=64, cap=32, dt=0: L.polar_select_gemm(
        A, W, idx, None, C, M, K, N, cap, dt, 1, None)
    assert g(M=-1) == EINVAL and g(K=0) == EINVAL and g(N=0) == EINVAL and g(cap=-1) == EINVAL
    assert g(dt=3) == EINVAL
    assert g(K=200) == EUNSUPPORTED                       # K must be a multiple of 128
    assert g(A=None) == EINVAL and g(W=None) == EINVAL and g(idx=None) == EINVAL and g(C=None) == EINVAL
    assert g(A=ctypes.c_void_p(0x1008)) == EINVAL         # 16-byte alignment
    assert g(M=0, A=None, W=None, idx=None, C=None) == OK
    assert g(cap=0, idx=None, C=None) == OK
    # the workspace form checks the same things, and its workspace's alignment
    gw = lambda A=A16, W=A16, idx=FAKE, C=FAKE, M=4, K=256, N=64, cap=32, dt=0, ws=None, wsb=0: \
        L.polar_select_gemm_ws(A, W, idx, None, C, M, K, N, cap, dt, 1, ws, wsb, None)
    assert gw(M=-1) == EINVAL and gw(K=0) == EINVAL and gw(N=0) == EINVAL and gw(cap=-1) == EINVAL
    assert gw(dt=3) == EINVAL and gw(K=200) == EUNSUPPORTED
    assert gw(A=None) == EINVAL and gw(W=None) == EINVAL and gw(idx=None) == EINVAL and gw(C=None) == EINVAL
    assert gw(ws=ctypes.c_void_p(0x1004), wsb=1 << 20) == EINVAL
    assert gw(M=0, A=None, W=None, idx=None, C=None) == OK and gw(cap=0, idx=None, C=None) == OK
    assert L.polar_select_gemm_workspace_bytes(-1) == 0 and L.polar_select_gemm_workspace_bytes(0) == 0
    sizes = [L.polar_select_gemm_workspace_bytes(M) for M in (1, 16, 17, 32, 33, 64, 65, 128, 129, 4096)]
    assert sizes[0] == sizes[1] > 0 and sizes[2] == sizes[3] == 2 * sizes[0]
    assert sizes[4] == sizes[5] == 4 * sizes[0] and sizes[6] == sizes[7] == 8 * sizes[0]
    assert sizes[8] == sizes[9] == 8 * sizes[0]         # beyond 128 rows: passes of 128 share it
    assert polar.select_gemm_workspace_bytes(64) == sizes[5]
    u = lambda topk=FAKE, B=2, kn=3, N=64, cap=6, idx=FAKE, cnt=FAKE: L.polar_neuron_union(
        topk, B, kn, N, cap, idx, cnt, None)
    assert u(B=-1) == EINVAL and u(N=0) == EINVAL and u(cap=-1) == EINVAL
    assert u(cnt=None) == EINVAL and u(idx=None) == EINVAL and u(topk=None) == EINVAL
    assert u(N=524289) == EUNSUPPORTED
    uw = lambda topk=FAKE, B=2, kn=3, N=64, cap=6, idx=FAKE, cnt=FAKE, ws=None, wsb=0: L.polar_neuron_union_ws(
        topk, B, kn, N, cap, idx, cnt, ws, wsb, None)
    assert uw(B=-1) == EINVAL and uw(N=0) == EINVAL and uw(cap=-1) == EINVAL
    assert uw(cnt=None) == EINVAL and uw(idx=None) == EINVAL and uw(topk=None) == EINVAL
    assert uw(N=524289) == EUNSUPPORTED
    assert uw(ws=ctypes.c_void_p(0x1002), wsb=1 << 20) == EINVAL
    assert L.polar_neuron_union_workspace_bytes(-1, 3, 64) == 0                # invalid sizes: nothing to allocate
    assert L.polar_neuron_union_workspace_bytes(64, 1843, 524289) == 0
    assert polar.neuron_union_workspace_bytes(2, 3, 64) == 0                 # too few ids to split
    assert polar.neuron_union_workspace_bytes(64, 1843, 36864) == 8 * 1152 * 4
    assert polar.neuron_union_workspace_bytes(4, 1024, 36864) == 0              # 4096 ids: the one-launch kernel is faster
    assert polar.neuron_union_workspace_bytes(16, 1024, 36864) == 8 * 1152 * 4
    with polar.options(union_form=2):                                           # pinned: split whenever there are two shares
        assert polar.neuron_union_workspace_bytes(4, 1024, 36864) == 2 * 1152 * 4
    with polar.options(union_form=1):
        assert polar.neuron_union_workspace_bytes(64, 1843, 36864) == 0


def test_select_gemm_down_argument_errors():
    L = binding.lib()
    A16 = ctypes.c_void_p(0x1000)
    big = 1 << 30
    d = lambda H=A16, W2=A16, idx=FAKE, Y=A16, M=4, Kout=256, N=64, cap=32, dt=0, ws=A16, wsb=big: \
        L.polar_select_gemm_down(H, W2, idx, None, Y, M, Kout, N, cap, dt, ws, wsb, None)
    assert d(M=-1) == EINVAL and d(Kout=0) == EINVAL and d(N=0) == EINVAL and d(cap=-1) == EINVAL
    assert d(dt=2) == EINVAL
    assert d(Kout=384) == EUNSUPPORTED
    assert d(W2=None) == EINVAL and d(Y=None) == EINVAL and d(ws=None) == EINVAL
    assert d(H=None) == EINVAL and d(idx=None) == EINVAL
    assert d(H=ctypes.c_void_p(0x1002)) == EINVAL and d(Y=ctypes.c_void_p(0x1008)) == EINVAL
    assert d(wsb=16) == EWORKSPACE
    assert d(M=0, H=None, W2=None, idx=None, Y=None, ws=None) == OK
    q = L.polar_select_gemm_down_workspace_bytes
    # the ranges' sums (ranges x padded rows x Kout floats) and the prepared 16-bit activations
    assert q(4, 256, 33) > 0 and (q(4, 256, 33) - 4 * 64 * 2) % (16 * 256 * 4) == 0
    assert q(64, 9216, 36864) == 7 * 64 * 9216 * 4 + 64 * 36864 * 2      # 36 column groups x 7 ranges
    assert (q(64, 9216, 400000) - 64 * 400000 * 2) // (64 * 9216 * 4) >= 49
    assert q(0, 256, 32) == 0
    assert q(4, 300, 32) == 0 and q(-1, 256, 32) == 0                    # sizes the call rejects
    # beyond 64 rows: passes of up to 128 rows (72 column blocks x 3 ranges) and a remainder share it
    assert q(300, 9216, 36864) == max(7 * 64, 3 * 128) * 9216 * 4 + 128 * 36864 * 2
    assert q(65, 9216, 36864) == max(7 * 64, 3 * 128) * 9216 * 4 + 128 * 36864 * 2


def test_sparse_mlp_argument_errors():
    L = binding.lib()
    A16 = ctypes.c_void_p(0x1000)
    big = 1 << 32
    m = lambda X=A16, W1=A16, W2=A16, idx=FAKE, Y=A16, M=4, D=256, N=64, cap=32, dt=0, ws=A16, wsb=big: \
        L.polar_sparse_mlp(X, W1, W2, idx, None, Y, M, D, N, cap, dt, 1, ws, wsb, None)
    assert m(M=-1) == EINVAL and m(D=0) == EINVAL and m(N=0) == EINVAL and m(cap=-1) == EINVAL
    assert m(dt=2) == EINVAL
    assert m(D=384) == EUNSUPPORTED and m(D=128) == EUNSUPPORTED
    assert m(X=None) == EINVAL and m(W1=None) == EINVAL and m(W2=None) == EINVAL and m(idx=None) == EINVAL
    assert m(Y=None) == EINVAL and m(ws=None) == EINVAL
    assert m(X=ctypes.c_void_p(0x1008)) == EINVAL and m(ws=ctypes.c_void_p(0x1010)) == EINVAL   # 16 and 256 bytes
    assert m(wsb=4096) == EWORKSPACE
    assert m(M=0, X=None, W1=None, W2=None, idx=None, Y=None, ws=None) == OK
    q = L.polar_sparse_mlp_workspace_bytes
    # four regions, each a multiple of 256 bytes: the first factor's workspace (up to 128 rows a pass),
    # the second factor's partial sums, the 16-bit hidden activations of one pass (128 rows of them
    # beyond 64 rows), and the hidden activations of one pass as floats (the fallback's)
    for (M, D, cap) in [(64, 9216, 36864), (4, 256, 33), (100, 512, 700), (300, 1024, 5000)]:
        rows, h16_rows, cap32 = min(M, 128), (M if M <= 64 else 128), (cap + 31) // 32 * 32
        g = L.polar_select_gemm_workspace_bytes(rows)
        partial = L.polar_select_gemm_down_workspace_bytes(M, D, cap) - h16_rows * cap32 * 2
        up = lambda v: (v + 255) // 256 * 256
        assert q(M, D, cap) == up(g) + up(partial) + up(h16_rows * cap32 * 2) + up(rows * cap * 4)
    assert q(0, 256, 32) == 0
    assert q(4, 300, 32) == 0 and q(-1, 256, 32) == 0


def test_workspace_size_is_consistent_with_the_chunking():
    L = binding.lib()
    for (B, Hq, Hkv, S, d, k) in [(4, 8, 8, 256, 64, 4), (32, 32, 32, 1920, 128, 16),
                                  (64, 32, 8, 4096, 128, 4), (128, 72, 72, 1920, 128, 36),
                                  (256, 32, 32, 8192, 128, 8), (1, 8, 8, 1, 64, 8)]:
        chunk = polar.sha_chunk_rows(B, Hq, Hkv, S, d, k)
        assert chunk > 0 and chunk % 128 == 0
        nsplit = -(-S // chunk)
        need = B * k * (Hq // Hkv) * nsplit * (d + 2) * 4
        got = polar.sha_workspace_bytes(B, Hq, Hkv, S, d, k)
        assert need <= got <= need + 512 and got % 256 == 0
    assert polar.sha_workspace_bytes(4, 8, 8, 256, 96, 4) == 0
    assert polar.sha_chunk_rows(4, 12, 8, 256, 64, 4) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros((1, 8, 64), dtype=torch.float16)
    K = torch.zeros((1, 8, 128, 64), dtype=torch.float16)
    n = torch.ones(1, dtype=torch.int32)
    ws = torch.zeros(1 << 16, dtype=torch.uint8)
    out = torch.zeros((1, 8, 64))
    with pytest.raises(ValueError, match="no CPU fallback"):
        polar.sha_decode(q, K, K, n, None, 8, out=out, workspace=ws)
    with pytest.raises(ValueError, match="no CPU fallback"):
        polar.router_topk(torch.zeros((1, 16), dtype=torch.float16),
                          torch.zeros((16, 4), dtype=torch.float16), 2,
                          head_idx=torch.zeros((1, 2), dtype=torch.int32))
    with pytest.raises(polar.PolarError):
        polar.alloc_workspace(4, 8, 8, 256, 96, 4, "cpu")


def test_probe_and_launch_query_argument_checks():
    L = binding.probe_lib()
    assert L.polar_probe_last_hip_error() == 0
    assert L.polar_probe_read(FAKE, 4, 8, 1, FAKE, None) == EINVAL          # slab under 16 bytes
    assert L.polar_probe_read(FAKE, 4, 4100, 1, FAKE, None) == EINVAL       # not a multiple of 16
    assert L.polar_probe_read(None, 4, 4096, 1, FAKE, None) == EINVAL
    assert L.polar_probe_read(FAKE, 4, 4096, 1, None, None) == EINVAL
    assert L.polar_probe_read(ctypes.c_void_p(0x10008), 4, 4096, 1, FAKE, None) == EINVAL   # misaligned
    assert L.polar_probe_read(None, 0, 4096, 1, None, None) == OK           # nothing to read
    # launches of polar_sha_decode: 1 for a moderate unsplit cache, 2 when split or very large, 0 if invalid
    assert polar.sha_launches(32, 32, 32, 1920, 128, 16) == 1
    assert polar.sha_launches(64, 32, 8, 4096, 128, 4) == 1
    assert polar.sha_launches(128, 72, 72, 1920, 128, 36) == 2
    assert polar.sha_launches(256, 32, 32, 8192, 128, 8) == 2
    assert polar.sha_launches(4, 8, 8, 256, 96, 4) == 0


def test_gather_probe_argument_checks():
    L = binding.probe_lib()
    A16 = ctypes.c_void_p(0x1000)
    g = lambda W=A16, idx=FAKE, n=100, N=64, K=1536, slices=3, depth=1, sink=FAKE: L.polar_probe_gather_read(
        W, idx, n, N, K, slices, depth, 1, sink, None)
    assert g(n=-1) == EINVAL and g(N=0) == EINVAL and g(K=0) == EINVAL and g(slices=0) == EINVAL
    assert g(depth=3) == EINVAL and g(depth=0) == EINVAL and g(depth=2) == EINVAL
    assert g(K=1500) == EUNSUPPORTED and g(K=1536, slices=5) == EUNSUPPORTED and g(K=1536, depth=4, slices=2) == EUNSUPPORTED
    assert g(W=None) == EINVAL and g(idx=None) == EINVAL and g(sink=None) == EINVAL
    assert g(W=ctypes.c_void_p(0x1008)) == EINVAL
    assert g(n=0, W=None, idx=None, sink=None) == OK


def test_bench_refuses_more_than_one_gpu():
    """The benchmark runs on one GPU only and says so before it touches torch or the GPU."""
    import subprocess
    import sys
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                          capture_output=True, text=True, timeout=120)
    assert proc.returncode == 2
    assert "one GPU" in proc.stderr and proc.stdout.strip() == ""
