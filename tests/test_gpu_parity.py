"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle on the same bits.

Bar: head_idx bit-exact; attention output max-abs error <= 2e-3 (16-bit inputs, float
accumulation); skipped heads exactly +0.0.  Inputs are seeded and synthetic, shaped like the
configurations the bench uses.  Every case prints its name before it touches the GPU.
"""
import numpy as np
import pytest
import torch

import paper_2505_14884_amd as polar
from oracle import polar_oracle as orc
from paper_2505_14884_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-3
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def host_bits(t):
    return wl.bits_u16(t)


def check_against_oracle(w, q, K, V, seqlens, head_idx, out, rows=None, max_host_bytes=2 << 30):
    """Compare `out` (GPU, float32 [B,Hq,d]) with the oracle, element by element, for the requests
    in `rows` (default: every request).  Large batches go to the host a slice of requests at a
    time, so that the host copy of K and V stays under max_host_bytes."""
    rows = list(range(w.B)) if rows is None else list(rows)
    per_request = 2 * w.Hkv * w.S * w.d * 2
    step = max(1, min(len(rows) or 1, max_host_bytes // per_request))
    worst = 0.0
    for r0 in range(0, len(rows), step):
        sel = torch.tensor(rows[r0:r0 + step], device=q.device)
        idx_host = None if head_idx is None else head_idx[sel].cpu().numpy()
        want = orc.sha_decode(host_bits(q[sel]), host_bits(K[sel]), host_bits(V[sel]),
                              seqlens[sel].cpu().numpy(), idx_host, w.k, w.dtype)
        got32 = out[sel].cpu().numpy()
        got = got32.astype(np.float64)
        assert np.isfinite(got).all()
        err = np.abs(got - want).max() if got.size else 0.0
        assert err <= TOL, (err, rows[r0:r0 + step])
        # heads the oracle leaves at zero must be +0.0 bit for bit
        zero = (want == 0.0).all(axis=2)
        assert (got32.view(np.uint32)[zero] == 0).all()
        worst = max(worst, float(err))
        if len(rows) > step:
            say("   requests %d..%d: max-abs error %.3e" % (rows[r0], rows[min(r0 + step, len(rows)) - 1], err))
    say("   max-abs error %.3e over %d requests" % (worst, len(rows)))
    return worst


def poison_unselected(w, q, K, V, head_idx):
    """NaN into q/K/V of every head a request did not select (nothing may read them)."""
    keep = torch.zeros((w.B, w.Hkv), dtype=torch.bool, device=K.device)
    valid = (head_idx >= 0) & (head_idx < w.Hkv)
    b_ix = torch.arange(w.B, device=K.device)[:, None].expand_as(head_idx)
    keep[b_ix[valid], head_idx[valid].long()] = True
    K[~keep] = float("nan")
    V[~keep] = float("nan")
    q.view(w.B, w.Hkv, w.G, w.d)[~keep] = float("nan")


# (pass a workspace?, router_path option, router_phase1 option): without a workspace the one-kernel
# path runs; with one the library picks the faster path for the shape unless the option forces the
# split-D kernels (2), whose first phase runs on the vector ALU (1) or the fp64 matrix cores (2).
ROUTER_MODES = [(False, None, None), (True, 2, 1), (True, 2, 2), (True, None, None)]


def router_path(path, phase1=None):
    return polar.options(router_path=path, router_phase1=phase1)


def run_router(w):
    hidden, Wr = wl.make_router_inputs(w, DEV)
    ref_logits = orc.router_logits(host_bits(hidden), host_bits(Wr), w.dtype)
    want = orc.topk(ref_logits, w.k)
    for ws, path, mfma in ROUTER_MODES:
        logits = torch.full((w.B, w.Hkv), float("nan"), dtype=torch.float32, device=DEV)
        got = torch.full((w.B, w.k), -7, dtype=torch.int32, device=DEV)
        with router_path(path, mfma):          # the workspace size depends on the phase-1 kernel
            rws = polar.alloc_router_workspace(w.B, w.D, w.Hkv, DEV).fill_(0xFF) if ws else None
            polar.router_topk(hidden, Wr, w.k, head_idx=got, logits_out=logits, workspace=rws)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want), "head_idx differs from the oracle"
        np.testing.assert_allclose(logits.cpu().numpy(), ref_logits, rtol=2e-7, atol=1e-7)
    srt = -np.sort(-ref_logits, axis=1)
    say("   router ok; smallest gap among the top-(k+1) logits: %.3e"
        % np.diff(-srt[:, : min(w.k + 1, w.Hkv)], axis=1).min(initial=np.inf))
    return got


def run_attention(w, head_idx, rows=None, poison=True, check_dense_rows=None):
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV, poison_padding=poison)
    if poison and head_idx is not None:
        poison_unselected(w, q, K, V, head_idx)
    out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device=DEV)
    ws = polar.alloc_workspace(w.B, w.Hq, w.Hkv, w.S, w.d, w.k, DEV)
    ws.fill_(0xFF)                                  # NaN bit patterns: stale partials would show
    polar.sha_decode(q, K, V, seqlens, head_idx, w.k, out=out, workspace=ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all(), "a NaN canary or an unwritten element reached the output"
    check_against_oracle(w, q, K, V, seqlens, head_idx, out, rows)
    # bit-reproducible: no atomics, fixed merge order
    out2 = torch.empty_like(out)
    polar.sha_decode(q, K, V, seqlens, head_idx, w.k, out=out2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))
    return out


# ----------------------------------------------------------------------------- the five configs
@pytest.mark.parametrize("name", ["C1_tiny", "C2_llama2_7b", "C3_llama3_8b_gqa"])
def test_config_full_parity(name):
    w = wl.CONFIGS[name]
    say("\ncase", name, w)
    head_idx = run_router(w)
    run_attention(w, head_idx)


@pytest.mark.parametrize("name", ["C4_opt66b", "C5_ragged", "X1_gqa8_s8192"])
def test_config_full_size_whole_batch_parity(name):
    """Full-size launch exactly as the bench times it (same sizes, same plan, NaN-poisoned
    padding and unselected heads); the oracle recomputes EVERY request, a slice of the batch at
    a time, and every element and every skipped head's bit pattern is compared."""
    w = wl.CONFIGS.get(name) or wl.EXTRA_SHAPES[name]
    say("\ncase", name, w)
    head_idx = run_router(w)
    out = run_attention(w, head_idx, poison=True)
    selected = torch.zeros((w.B, w.Hkv), dtype=torch.bool, device=DEV)
    selected[torch.arange(w.B, device=DEV)[:, None], head_idx.long()] = True
    skipped = ~selected.repeat_interleave(w.G, dim=1)
    assert (out.view(torch.int32)[skipped] == 0).all()
    assert (out[~skipped].abs().sum(dim=-1) > 0).all()


# ----------------------------------------------------------------------------- dense path
@pytest.mark.parametrize("dtype,d,G", [("f16", 128, 1), ("bf16", 64, 1), ("bf16", 128, 4),
                                       ("f16", 64, 2), ("f16", 128, 8)])
def test_dense_null_index_and_identity_index(dtype, d, G):
    w = wl.ShaWorkload("dense", B=3, Hq=4 * G, Hkv=4, d=d, S=700, k=4, D=64, dtype=dtype,
                       seq_lo=1, seed=7 + d + G)
    say("\ncase dense", w)
    out_null = run_attention(w, None)
    ident = torch.arange(4, dtype=torch.int32, device=DEV).repeat(w.B, 1)
    out_ident = run_attention(w, ident, poison=False)
    assert torch.equal(out_null.view(torch.int32), out_ident.view(torch.int32))


# ----------------------------------------------------------------------------- edge shapes
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("d,G", [(128, 1), (64, 1), (128, 4), (64, 8), (128, 2), (128, 8), (128, 3),
                                 (128, 7), (128, 16)])
def test_ragged_lengths_and_tails(dtype, d, G):
    """Lengths 0, 1, around every tile boundary (rows per load, per wave step, per workgroup
    step, per chunk) and the full capacity."""
    lens = [0, 1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 127, 128, 129, 255, 256,
            257, 300, 511, 512, 513, 640, 1000, 1023]
    w = wl.ShaWorkload("ragged", B=len(lens), Hq=6 * G, Hkv=6, d=d, S=1023, k=3, D=64,
                       dtype=dtype, seed=11 * d + G)
    say("\ncase ragged", w)
    seqlens = torch.tensor(lens, dtype=torch.int32, device=DEV)
    q, K, V, _ = wl.make_attention_inputs(w, DEV, poison_padding=True, seqlens=seqlens)
    head_idx = wl.random_head_idx(w, DEV)
    poison_unselected(w, q, K, V, head_idx)
    out = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    check_against_oracle(w, q, K, V, seqlens, head_idx, out)
    assert (out[0].view(torch.int32) == 0).all()          # length 0 -> zeros


def test_invalid_and_duplicate_head_ids_and_clamped_lengths():
    w = wl.ShaWorkload("ids", B=4, Hq=8, Hkv=8, d=128, S=300, k=4, D=64, dtype="f16", seed=5)
    say("\ncase ids", w)
    seqlens = torch.tensor([300, 9999, -7, 150], dtype=torch.int32, device=DEV)
    q, K, V, _ = wl.make_attention_inputs(w, DEV, seqlens=seqlens.clamp(0, w.S))
    head_idx = torch.tensor([[2, -1, 2, 8], [7, 7, 7, 7], [0, 1, 2, 3], [-5, 100, 3, 0]],
                            dtype=torch.int32, device=DEV)
    out = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)
    torch.cuda.synchronize()
    check_against_oracle(w, q, K, V, seqlens, head_idx, out)
    assert (out[2].view(torch.int32) == 0).all()


def test_peaky_softmax_and_explicit_scale():
    w = wl.ShaWorkload("peaky", B=2, Hq=4, Hkv=4, d=128, S=2048, k=2, D=64, dtype="bf16",
                       peaky=0.05, seed=9)
    say("\ncase peaky", w)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV)
    head_idx = wl.random_head_idx(w, DEV)
    for scale in (0.0, 0.25, 0.01):
        out = polar.sha_decode(q, K, V, seqlens, head_idx, w.k, scale=scale)
        torch.cuda.synchronize()
        want = orc.sha_decode(host_bits(q), host_bits(K), host_bits(V), seqlens.cpu().numpy(),
                              head_idx.cpu().numpy(), w.k, w.dtype, scale=scale)
        err = np.abs(out.cpu().numpy() - want).max()
        say("   scale %.3g max-abs error %.3e" % (scale, err))
        assert err <= TOL


@pytest.mark.parametrize("name,dtype,G,d", [("f16-mha", "f16", 1, 128), ("bf16-gqa", "bf16", 4, 128),
                                            ("f16-d64", "f16", 2, 64)])
def test_sequence_major_cache_layout(name, dtype, G, d):
    """K/V stored [B, S, Hkv, d] (the footnote layout of Section 3.2): same result as the
    head-major layout, and the oracle (which reads head-major) agrees."""
    w = wl.ShaWorkload("bshd-" + name, B=5, Hq=6 * G, Hkv=6, d=d, S=777, k=3, D=64, dtype=dtype,
                       seq_lo=1, seed=31 + G)
    say("\ncase", w)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV, poison_padding=True)
    head_idx = wl.random_head_idx(w, DEV)
    poison_unselected(w, q, K, V, head_idx)
    Kt, Vt = K.permute(0, 2, 1, 3).contiguous(), V.permute(0, 2, 1, 3).contiguous()
    out = polar.sha_decode(q, Kt, Vt, seqlens, head_idx, w.k, kv_layout="bshd")
    ref = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
    check_against_oracle(w, q, K, V, seqlens, head_idx, out)
    dense = polar.sha_decode(q, Kt, Vt, seqlens, None, w.Hkv, kv_layout="bshd")
    torch.cuda.synchronize()
    wd = w.scaled(k=w.Hkv)
    K2, V2 = K.nan_to_num(0.0), V.nan_to_num(0.0)   # dense reads every head: un-poison a copy
    dense2 = polar.sha_decode(q.nan_to_num(0.0), K2.permute(0, 2, 1, 3).contiguous(),
                              V2.permute(0, 2, 1, 3).contiguous(), seqlens, None, w.Hkv,
                              kv_layout="bshd")
    torch.cuda.synchronize()
    check_against_oracle(wd, q.nan_to_num(0.0), K2, V2, seqlens, None, dense2)
    del dense


def two_kernel_form():
    """Keep the streaming + merge pair even where an unsplit cache would take the one-kernel form."""
    return polar.options(sha_form=2)


@pytest.mark.parametrize("dtype,Hkv,G,d,k,S", [("f16", 8, 1, 128, 3, 250), ("bf16", 6, 4, 128, 2, 256),
                                               ("f16", 128, 1, 64, 100, 130), ("bf16", 72, 1, 128, 7, 200),
                                               ("f16", 5, 3, 128, 5, 255), ("bf16", 4, 8, 64, 1, 90)])
def test_one_kernel_form_for_unsplit_caches(dtype, Hkv, G, d, k, S):
    """A cache that is not split is finished by the streaming kernel alone (it normalises, and
    zero-fills the unselected heads).  Same bits as the streaming + merge pair, and parity with the
    oracle, with -1 padding, duplicates, an empty request and rows of more than 64 ids."""
    w = wl.ShaWorkload("direct", B=6, Hq=Hkv * G, Hkv=Hkv, d=d, S=S, k=k, D=64, dtype=dtype,
                       seq_lo=1, seed=900 + Hkv + G)
    say("\ncase one-kernel form", w)
    assert polar.sha_launches(w.B, w.Hq, w.Hkv, w.S, w.d, w.k) == 1          # really one kernel
    with two_kernel_form():
        assert polar.sha_launches(w.B, w.Hq, w.Hkv, w.S, w.d, w.k) == 2
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV, poison_padding=True)
    seqlens[2] = 0
    K[2], V[2] = float("nan"), float("nan")
    head_idx = wl.random_head_idx(w, DEV)
    head_idx[1, 0] = -1                                   # an empty slot
    if k > 1:
        head_idx[3, 1] = head_idx[3, 0]                   # a duplicate
        head_idx[4, :] = -1                               # a request with nothing selected
    poison_unselected(w, q, K, V, head_idx)
    out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device=DEV)
    polar.sha_decode(q, K, V, seqlens, head_idx, w.k, out=out)
    with two_kernel_form():
        ref = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
    assert (out[2].view(torch.int32) == 0).all()
    assert k == 1 or (out[4].view(torch.int32) == 0).all()
    check_against_oracle(w, q, K, V, seqlens, head_idx, out)
    # dense call (NULL index) on clean inputs, with an empty request
    q2, K2, V2, n2 = wl.make_attention_inputs(w, DEV, poison_padding=True)
    n2[0] = 0
    dense = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device=DEV)
    polar.sha_decode(q2, K2, V2, n2, None, w.Hkv, out=dense)
    with two_kernel_form():
        dref = polar.sha_decode(q2, K2, V2, n2, None, w.Hkv)
    torch.cuda.synchronize()
    assert torch.equal(dense.view(torch.int32), dref.view(torch.int32))
    assert (dense[0].view(torch.int32) == 0).all()


def test_random_shapes_against_the_oracle():
    """Forty seeded random valid shapes (group size, head dimension, lengths, k, dtype, cache layout,
    padded and duplicate ids, forced chunk sizes): every one element by element against the oracle."""
    rng = np.random.default_rng(20250514)
    for case in range(40):
        d = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 2, 4, 8])) if d == 64 else int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 12, 16]))
        Hkv = int(rng.integers(1, 13))
        k = int(rng.integers(1, Hkv + 1))
        B = int(rng.integers(1, 9))
        S = int(rng.integers(1, 1400))
        dtype = str(rng.choice(["f16", "bf16"]))
        layout = str(rng.choice(["bhsd", "bshd"]))
        chunk = int(rng.choice([0, 128, 256, 384, 1024]))        # 0: the library's own choice
        w = wl.ShaWorkload("rnd%d" % case, B=B, Hq=Hkv * G, Hkv=Hkv, d=d, S=S, k=k, D=64, dtype=dtype,
                           seq_lo=1, seed=5000 + case)
        say("\ncase", case, w, layout, "chunk", chunk)
        seqlens = wl.make_seqlens(w, DEV)
        seqlens[int(rng.integers(0, B))] = int(rng.choice([0, 1, S]))
        q, K, V, _ = wl.make_attention_inputs(w, DEV, poison_padding=True, seqlens=seqlens)
        head_idx = wl.random_head_idx(w, DEV, seed_offset=case)
        if k > 1 and rng.random() < 0.5:
            head_idx[int(rng.integers(0, B)), int(rng.integers(0, k))] = -1
        if k > 1 and rng.random() < 0.3:
            head_idx[0, 1] = head_idx[0, 0]
        poison_unselected(w, q, K, V, head_idx)
        Kc, Vc = (K, V) if layout == "bhsd" else (K.permute(0, 2, 1, 3).contiguous(),
                                                  V.permute(0, 2, 1, 3).contiguous())
        with polar.options(sha_chunk_rows=chunk or None):
            out = torch.full((B, w.Hq, d), float("nan"), dtype=torch.float32, device=DEV)
            polar.sha_decode(q, Kc, Vc, seqlens, head_idx, k, out=out, kv_layout=layout)
            torch.cuda.synchronize()
        check_against_oracle(w, q, K, V, seqlens, head_idx, out)


def test_per_request_k_through_padding():
    """Requests keep different numbers of heads: unused slots hold -1 (the adaptive routing the
    paper lists as future work needs nothing else from the kernel)."""
    w = wl.ShaWorkload("padk", B=6, Hq=8, Hkv=8, d=128, S=500, k=5, D=64, dtype="f16", seq_lo=50,
                       seed=77)
    say("\ncase", w)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV, poison_padding=True)
    head_idx = wl.random_head_idx(w, DEV)
    keep = torch.tensor([5, 0, 1, 3, 2, 4], device=DEV)          # per-request k, 0 = nothing kept
    pad = torch.arange(w.k, device=DEV)[None, :] >= keep[:, None]
    head_idx[pad] = -1
    poison_unselected(w, q, K, V, head_idx)
    out = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)
    torch.cuda.synchronize()
    check_against_oracle(w, q, K, V, seqlens, head_idx, out)
    assert (out[1].view(torch.int32) == 0).all()
    assert int((out.abs().sum(-1) > 0).sum()) == int(keep.sum())


def test_hip_graph_replays_match_eager():
    """Router + attention recorded into one HIP graph (as the paper's runs used CUDA graphs):
    every replay, with eager work and synchronisation in between, equals the eager result."""
    w = wl.ShaWorkload("graph", B=16, Hq=32, Hkv=8, d=128, S=900, k=3, D=1024, dtype="bf16",
                       seq_lo=100, seed=55)
    say("\ncase", w)
    hidden, Wr = wl.make_router_inputs(w, DEV)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV)
    idx = torch.zeros((w.B, w.k), dtype=torch.int32, device=DEV)
    out = torch.zeros((w.B, w.Hq, w.d), dtype=torch.float32, device=DEV)
    ws = polar.alloc_workspace(w.B, w.Hq, w.Hkv, w.S, w.d, w.k, DEV)
    rws = polar.alloc_router_workspace(w.B, w.D, w.Hkv, DEV)

    def step(idx_buf, out_buf):
        polar.router_topk(hidden, Wr, w.k, head_idx=idx_buf, workspace=rws)
        polar.sha_decode(q, K, V, seqlens, idx_buf, w.k, out=out_buf, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        step(idx, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(idx, out)
    gen = torch.Generator(device=DEV).manual_seed(4242)
    for rep in range(4):
        hidden.copy_(torch.randn(hidden.shape, generator=gen, device=DEV).to(hidden.dtype))
        q.copy_(torch.randn(q.shape, generator=gen, device=DEV).to(q.dtype))
        idx_e, out_e = torch.empty_like(idx), torch.empty_like(out)
        step(idx_e, out_e)                             # eager, same workspaces, before the replay
        torch.cuda.synchronize()
        idx.fill_(-3)
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, idx_e), "replay %d: head_idx" % rep
        assert torch.equal(out.view(torch.int32), out_e.view(torch.int32)), "replay %d: out" % rep
    check_against_oracle(w, q, K, V, seqlens, idx, out)


@pytest.mark.parametrize("name", ["C1_tiny", "C2_llama2_7b", "C3_llama3_8b_gqa"])
def test_head_importance_labels(name):
    """Labeller = dense attention + per-group output norm + top-k (Section 3.2 head-sparsity study,
    Section 4.2 router targets).  Labels are index work, so the bar is bit-exact:
    (1) the ranking kernel, fed the GPU's own dense attention output, must give on EVERY row the
        labels the oracle's score and top-k routines give on those same float bits;
    (2) end to end (oracle attention in double against GPU attention in float) the labels must be
        identical on every row whose neighbouring oracle scores among the top k+1 differ by more
        than the float attention's error can move them; rows with a nearer tie are counted and
        reported, never accepted on a weaker check (they are covered by (1), and the attention
        that feeds them by the parity tests above)."""
    w = wl.CONFIGS[name]
    say("\ncase labels", name)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV)
    dense = polar.sha_decode(q, K, V, seqlens, None, w.Hkv)
    norms = torch.empty((w.B, w.Hkv), dtype=torch.float32, device=DEV)
    got = polar.head_norm_topk(dense, w.Hkv, w.k, norms_out=norms).cpu().numpy()
    torch.cuda.synchronize()
    # (1) same bits in, same labels out: the oracle ranks the GPU's float attention output
    same_bits = dense.cpu().numpy().astype(np.float64)               # float -> double is exact
    score_same, norm_same = orc.head_scores(same_bits, w.Hkv)
    want_same = orc.topk(score_same, w.k)
    assert np.array_equal(got, want_same), "labels differ from the oracle's on the same attention output"
    np.testing.assert_allclose(norms.cpu().numpy(), norm_same, rtol=2e-7)
    # the one-call labeller (norm and ranking as the dense merge's epilogue): the same labels, and
    # the very attention output polar_sha_decode gives, with poisoned outputs and workspace
    out2 = torch.full_like(dense, float("nan"))
    norms2 = torch.full_like(norms, float("nan"))
    labels2 = torch.full((w.B, w.k), -9, dtype=torch.int32, device=DEV)
    ws = polar.alloc_workspace(w.B, w.Hq, w.Hkv, w.S, w.d, w.Hkv, DEV).fill_(0xFF)
    polar.head_labels(q, K, V, seqlens, w.k, labels=labels2, norms_out=norms2, attn_out=out2, workspace=ws)
    labels3 = polar.head_labels(q, K, V, seqlens, w.k)                 # no output, no norms wanted
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int32), dense.view(torch.int32))
    assert np.array_equal(labels2.cpu().numpy(), want_same) and np.array_equal(labels3.cpu().numpy(), want_same)
    np.testing.assert_allclose(norms2.cpu().numpy(), norm_same, rtol=2e-7)
    # (2) end to end
    want, score = orc.head_importance_labels(host_bits(q), host_bits(K), host_bits(V),
                                             seqlens.cpu().numpy(), w.k, w.dtype)
    srt = -np.sort(-score, axis=1)
    top = srt[:, : min(w.k + 1, w.Hkv)]
    gaps = (top[:, :-1] - top[:, 1:]) / top[:, :-1]
    # a float attention output within 2e-6 relative of the double one moves a sum of squares by
    # at most 4e-6 relative, hence neighbouring scores towards each other by at most 8e-6
    separated = gaps.min(axis=1, initial=1.0) > 1e-5
    assert np.array_equal(got[separated], want[separated])
    differ = int((got != want).any(axis=1).sum())
    say("   %d of %d rows have every top-(k+1) gap above 1e-5 and match exactly; %d rows hold a nearer tie; "
        "%d rows differ from the double-precision labels; smallest relative gap %.2e"
        % (int(separated.sum()), w.B, int((~separated).sum()), differ, gaps.min(initial=1.0)))
    assert differ <= int((~separated).sum())


@pytest.mark.parametrize("dtype,Hkv,G,d,S,layout", [("f16", 5, 1, 64, 300, "bhsd"), ("bf16", 7, 3, 128, 2600, "bshd"),
                                                      ("f16", 72, 1, 128, 130, "bhsd"), ("bf16", 4, 8, 64, 9000, "bhsd"),
                                                      ("f16", 256, 1, 64, 40, "bhsd")])
def test_head_labels_one_call_edge_shapes(dtype, Hkv, G, d, S, layout):
    """polar_head_labels on ragged lengths (an empty request included), both layouts, split and
    unsplit caches, several heads per merge pass: labels equal the oracle's ranking of the very
    output it stores, which equals polar_sha_decode's dense output bit for bit."""
    w = wl.ShaWorkload("labels", B=5, Hq=Hkv * G, Hkv=Hkv, d=d, S=S, k=max(1, Hkv // 2), D=64, dtype=dtype,
                       seq_lo=1, seed=300 + Hkv)
    say("\ncase one-call labels", w, layout)
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV, poison_padding=True)
    seqlens[3] = 0
    Kc, Vc = (K, V) if layout == "bhsd" else (K.permute(0, 2, 1, 3).contiguous(), V.permute(0, 2, 1, 3).contiguous())
    out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device=DEV)
    norms = torch.full((w.B, w.Hkv), float("nan"), dtype=torch.float32, device=DEV)
    labels = polar.head_labels(q, Kc, Vc, seqlens, w.k, norms_out=norms, attn_out=out, kv_layout=layout)
    dense = polar.sha_decode(q, Kc, Vc, seqlens, None, w.Hkv, kv_layout=layout)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), dense.view(torch.int32))
    score, norm = orc.head_scores(out.cpu().numpy().astype(np.float64), w.Hkv)
    assert np.array_equal(labels.cpu().numpy(), orc.topk(score, w.k))
    np.testing.assert_allclose(norms.cpu().numpy(), norm, rtol=2e-7)
    assert labels[3].cpu().tolist() == list(range(w.k))              # empty request: all norms 0, ids in order
    check_against_oracle(w.scaled(k=w.Hkv), q, K, V, seqlens, None, out)


# ----------------------------------------------------------------------------- selective GEMM
GEMM_TOL = 1e-4      # float accumulation of K <= 9216 products whose sum is O(1): ~sqrt(K) * 2^-24 * |sum| ~ 1e-5


def gemm_workgroups(G):
    """Pin the launch width of the wide-tile GEMM form (None: the library's own)."""
    return polar.options(gemm_workgroups=G)


def gemm_case(M, K, N, idx_host, dtype, relu, count=None, seed=0, ws=False, G=None, ws_bytes=None):
    """ws: call the workspace entry point (wide-tile form for M <= 128); G pins its launch width;
    ws_bytes shrinks the workspace below the recommended size."""
    g = torch.Generator(device=DEV).manual_seed(1000 + seed)
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    A = torch.randn((M, K), generator=g, device=DEV).to(tdt)
    W = (torch.randn((N, K), generator=g, device=DEV) / K ** 0.5).to(tdt)
    idx = torch.tensor(idx_host, dtype=torch.int32, device=DEV)
    cnt = None if count is None else torch.tensor([count], dtype=torch.int32, device=DEV)
    out = torch.full((M, len(idx_host)), float("nan"), dtype=torch.float32, device=DEV)
    workspace = None
    if ws:
        nbytes = polar.select_gemm_workspace_bytes(M) if ws_bytes is None else ws_bytes
        # poisoned: the kernels must write every slot they later read; a zero-size request still
        # goes through the workspace entry point, with a token buffer
        workspace = torch.full((max(nbytes, 16) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    with gemm_workgroups(G):
        polar.select_gemm(A, W, idx, count=cnt, relu=relu, out=out, workspace=workspace)
    torch.cuda.synchronize()
    live = len(idx_host) if count is None else max(0, min(count, len(idx_host)))
    want = orc.select_gemm(host_bits(A), host_bits(W), np.array(idx_host[:live], np.int32), dtype, relu)
    got = out.cpu().numpy()
    assert np.isfinite(got[:, :live]).all()
    err = np.abs(got[:, :live] - want).max() if want.size else 0.0
    assert err <= GEMM_TOL, err
    assert np.isnan(got[:, live:]).all()                   # columns beyond the live count untouched
    return err


@pytest.mark.parametrize("ws", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M", [1, 5, 17, 33, 64, 65, 100, 128, 130, 256, 300])
def test_select_gemm_shapes(dtype, M, ws):
    say("\ncase select_gemm", dtype, M, "workspace" if ws else "")
    rng = np.random.default_rng(M)
    N, K = 500, (512 if ws else 384)                       # the wide form needs K % 256 == 0
    idx = rng.permutation(N)[:77].tolist()                 # 77: two full 32-neuron tiles and a ragged one
    say("   err %.2e" % gemm_case(M, K, N, idx, dtype, relu=True, seed=M, ws=ws))
    say("   err %.2e" % gemm_case(M, K, N, idx, dtype, relu=False, seed=M + 1, ws=ws))


@pytest.mark.parametrize("G", [1, 2, 3, 5, 7, 11, 12, None])
def test_select_gemm_wide_form_spans(G):
    """The evenly split form cuts 3 tiles x 4 units (pairs of K blocks) into G spans: whole tiles
    finished in place (G = 1, 3), tiles shared by several workgroups (first / last slot), spans of
    unequal length, and spans left empty when the live count is below the capacity."""
    say("\ncase select_gemm spans G =", G)
    rng = np.random.default_rng(77)
    N, K = 700, 1024
    idx = rng.permutation(N)[:300].tolist()                # 3 tiles of 128, the last ragged
    idx[5], idx[200] = -1, N                               # invalid ids give zero columns
    for M, dtype in ((64, "f16"), (20, "bf16"), (3, "f16"), (128, "bf16"), (70, "f16")):
        gemm_case(M, K, N, idx, dtype, relu=True, seed=3, ws=True, G=G)
        gemm_case(M, K, N, idx, dtype, relu=False, seed=4, ws=True, G=G, count=130)   # 2 live tiles
        gemm_case(M, K, N, idx, dtype, relu=False, seed=5, ws=True, G=G, count=0)


def test_select_gemm_small_workspace_narrows_the_launch():
    say("\ncase select_gemm small workspace")
    rng = np.random.default_rng(78)
    idx = rng.permutation(700)[:300].tolist()
    full = polar.select_gemm_workspace_bytes(64)
    assert full > 0 and polar.select_gemm_workspace_bytes(300) == polar.select_gemm_workspace_bytes(128) == 2 * full
    one = 2 * 8 * 4 * 64 * 16          # a workgroup's two slots: 8 waves x 4 accumulator tiles x 64 lanes x 16 B
    assert full % one == 0
    for nbytes in (one, 3 * one, one - 16, 0):             # launch of 1 workgroup, of 3, narrow kernel, narrow kernel
        gemm_case(64, 1024, 700, idx, "f16", relu=True, seed=6, ws=True, ws_bytes=nbytes)


def test_select_gemm_capacity_at_and_beyond_the_even_split_limit():
    """The evenly split form keeps the row ids of at most 8 tiles per span in LDS: with 256
    workgroups that holds up to 1536 tiles (196608 ids).  At the limit every span touches 6 to 8
    tiles; one tile more and the workspace call runs the one-launch kernel instead, as does the
    one-call MLP (with the conversion launch)."""
    say("\ncase select_gemm capacity limit")
    rng = np.random.default_rng(5)
    N = 200100
    for cap in (196608, 196608 + 128):
        idx = rng.permutation(N)[:cap].tolist()
        say("   cap", cap, "err %.2e" % gemm_case(3, 256, N, idx, "f16", relu=True, seed=cap % 1000, ws=True))
    mlp_case(3, 256, N, rng.permutation(N)[:196608 + 128].tolist(), "bf16", count=196700, seed=77)


def test_select_gemm_invalid_ids_count_and_long_k():
    say("\ncase select_gemm ids")
    idx = [3, -1, 3, 99, 100, 7, 0, 42] * 5                # invalid ids (-1, 100) and repeats
    gemm_case(9, 128, 100, idx, "f16", relu=True)
    gemm_case(9, 128, 100, idx, "bf16", relu=False, count=17)   # device-side live count
    gemm_case(9, 128, 100, idx, "bf16", relu=False, count=0)
    gemm_case(9, 128, 100, idx, "f16", relu=True, count=1000)   # count beyond capacity is clamped
    gemm_case(33, 9216, 64, list(range(64)), "f16", relu=True)  # the OPT-66B contraction length
    for ws in (False, True):
        gemm_case(9, 128, 100, idx, "bf16", relu=False, count=17, ws=ws)
        gemm_case(64, 9216, 300, list(range(299, -1, -1)), "bf16", relu=True, ws=ws)


@pytest.mark.parametrize("ws", [False, True, "split"])
def test_neuron_union_matches_oracle(ws):
    """ws False: the one-launch kernel (sixteen workgroups mark everything and share the emit phase); True: the
    workspace entry point with the library's choice of form; "split": the split form pinned for every size."""
    say("\ncase neuron union", ws)
    with polar.options(union_form=2 if ws == "split" else None):
        union_cases(bool(ws))


def union_cases(ws):
    g = torch.Generator(device="cpu").manual_seed(5)
    for (B, kn, N) in [(1, 1, 1), (7, 12, 50), (64, 1843, 36864), (3, 5, 524288), (16, 100, 33),
                       (5, 1000, 524288), (128, 300, 4097)]:
        topk = torch.randint(-2, N + 2, (B, kn), generator=g, dtype=torch.int32).to(DEV)
        workspace = None
        if ws:        # poisoned, and at least a token buffer so that the workspace entry point is the one called
            nbytes = polar.neuron_union_workspace_bytes(B, kn, N)
            workspace = torch.full((max(nbytes, 4) // 4,), -1, dtype=torch.int32, device=DEV)
        idx, count = polar.neuron_union(topk, N, workspace=workspace)
        torch.cuda.synchronize()
        want = orc.neuron_union(topk.cpu().numpy(), N)
        c = int(count.item())
        assert c == len(want)
        assert idx[:c].cpu().numpy().tolist() == want.tolist()
    # a capacity smaller than the union truncates the ascending list
    topk = torch.arange(40, dtype=torch.int32, device=DEV).reshape(4, 10)
    idx, count = polar.neuron_union(topk, 64, cap=25)
    torch.cuda.synchronize()
    assert int(count.item()) == 25 and idx.cpu().tolist() == list(range(25))
    # a workspace that holds fewer bitmaps than the library wants narrows the launch; one that
    # holds fewer than two falls back to the one-launch kernel
    B, kn, N = 64, 1843, 36864
    topk = torch.randint(0, N, (B, kn), generator=g, dtype=torch.int32).to(DEV)
    want = orc.neuron_union(topk.cpu().numpy(), N)
    one = (N + 31) // 32 * 4
    for nbytes in (3 * one, 2 * one, one, 4):
        workspace = torch.full((nbytes // 4,), -1, dtype=torch.int32, device=DEV)
        idx, count = polar.neuron_union(topk, N, cap=len(want) - 7, workspace=workspace)
        torch.cuda.synchronize()
        assert int(count.item()) == len(want) - 7
        assert idx.cpu().numpy().tolist() == want[:-7].tolist()


@pytest.mark.parametrize("ws", [False, True])
@pytest.mark.parametrize("name", ["M1_tiny", "M2_opt66b_ffn"])
def test_sparse_mlp_first_layer(name, ws):
    """Union index built on the device feeds the selective GEMM without a host round trip;
    the oracle recomputes a sample of the selected neurons."""
    w = wl.MLP_CONFIGS[name]
    say("\ncase", w)
    x, W1, topk = wl.make_mlp_inputs(w, DEV)
    workspace = polar.alloc_select_gemm_workspace(w.B, DEV) if ws else None
    union_ws = (torch.empty(max(polar.neuron_union_workspace_bytes(w.B, topk.shape[1], w.N), 4), dtype=torch.uint8,
                            device=DEV) if ws else None)
    idx, count = polar.neuron_union(topk, w.N, workspace=union_ws)
    out = polar.select_gemm(x, W1, idx, count=count, relu=True, workspace=workspace)
    torch.cuda.synchronize()
    S = orc.neuron_union(topk.cpu().numpy(), w.N)
    c = int(count.item())
    assert c == len(S) and np.array_equal(idx[:c].cpu().numpy(), S)
    say("   union %d of %d neurons (%.1f %%)" % (c, w.N, 100.0 * c / w.N))
    cols = np.unique(np.linspace(0, c - 1, num=min(c, 192)).astype(np.int64))
    want = orc.select_gemm(host_bits(x), host_bits(W1[torch.from_numpy(S[cols]).long().to(DEV)]),
                           np.arange(len(cols), dtype=np.int32), w.dtype, True)
    got = out[:, torch.from_numpy(cols).to(DEV)].cpu().numpy()
    err = np.abs(got - want).max()
    say("   max-abs error %.3e on %d sampled neurons" % (err, len(cols)))
    assert err <= GEMM_TOL
    assert (out[:, :c] >= 0).all() and torch.isfinite(out[:, :c]).all()
    assert 0.3 < float((out[:, :c] > 0).float().mean()) < 0.7      # ReLU of a symmetric pre-activation
    if ws:
        # every element, not only the sampled columns: the two forms differ in the order of the
        # float additions only; and the split form is reproducible bit for bit
        narrow = polar.select_gemm(x, W1, idx, count=count, relu=True)
        again = polar.select_gemm(x, W1, idx, count=count, relu=True, workspace=workspace)
        torch.cuda.synchronize()
        diff = float((out[:, :c] - narrow[:, :c]).abs().max())
        say("   max-abs difference between the forms %.3e over %d x %d outputs" % (diff, w.B, c))
        assert diff <= GEMM_TOL
        assert torch.equal(out[:, :c], again[:, :c])


# ----------------------------------------------------------------------------- second MLP factor
def down_case(M, Kout, N, idx_host, dtype, count=None, seed=0, scale=1.0, sample_cols=None):
    """sample_cols: compare that many evenly spaced output columns instead of all (large cases:
    every workgroup's column block is hit, the oracle's work stays small)."""
    g = torch.Generator(device=DEV).manual_seed(2000 + seed)
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    cap = len(idx_host)
    # activations like the first factor's output: ReLU of a symmetric value; NaN beyond the live
    # count (those columns are never written by the first factor and must not be read)
    H = torch.relu(torch.randn((M, max(cap, 1)), generator=g, device=DEV))[:, :cap].contiguous() * scale
    live = cap if count is None else max(0, min(count, cap))
    H[:, live:] = float("nan")
    W2 = (torch.randn((N, Kout), generator=g, device=DEV) / max(live, 1) ** 0.5).to(tdt)
    idx = torch.tensor(idx_host, dtype=torch.int32, device=DEV)
    cnt = None if count is None else torch.tensor([count], dtype=torch.int32, device=DEV)
    out = torch.full((M, Kout), float("nan"), dtype=torch.float32, device=DEV)
    nbytes = polar.select_gemm_down_workspace_bytes(M, Kout, cap)
    workspace = torch.full((max(nbytes, 16) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    polar.select_gemm_down(H, W2, idx, count=cnt, out=out, workspace=workspace)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    if sample_cols:
        cols = torch.from_numpy(np.unique(np.linspace(0, Kout - 1, num=sample_cols).astype(np.int64))).to(DEV)
        W2, got = W2[:, cols].contiguous(), got[:, cols.cpu().numpy()]
    want = orc.select_gemm_down(H[:, :live].cpu().numpy(), host_bits(W2), np.array(idx_host[:live], np.int32), dtype)
    err = np.abs(got - want).max()
    assert err <= GEMM_TOL * max(scale, 1.0), err
    return err


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("M", [1, 5, 16, 17, 33, 64, 65, 100, 127, 128, 129, 150, 200])
def test_select_gemm_down_shapes(dtype, M):
    say("\ncase select_gemm_down", dtype, M)
    rng = np.random.default_rng(100 + M)
    N = 500
    for Kout, n in ((256, 77), (512, 300), (1024, 1), (256, 33)):      # ragged blocks of 32, a single neuron
        idx = rng.permutation(N)[:n].tolist()
        say("   Kout %d, %d neurons: err %.2e" % (Kout, n, down_case(M, Kout, N, idx, dtype, seed=M + n)))


def test_select_gemm_down_ids_counts_and_long_contraction():
    say("\ncase select_gemm_down ids")
    idx = [3, -1, 3, 99, 100, 7, 0, 42] * 5                # invalid ids (-1, 100) and repeats
    down_case(9, 256, 100, idx, "f16")
    down_case(9, 256, 100, idx, "bf16", count=17)          # device-side live count
    down_case(9, 256, 100, idx, "bf16", count=1000)        # beyond the capacity: clamped
    down_case(9, 256, 100, idx, "f16", count=0)            # nothing live: zeros
    down_case(4, 512, 100, [], "f16")                      # no capacity at all: zeros
    rng = np.random.default_rng(9)
    down_case(64, 512, 40000, rng.permutation(40000)[:12000].tolist(), "f16", seed=1)   # many ranges, long sums
    down_case(33, 256, 20000, rng.permutation(20000)[:9000].tolist(), "bf16", count=8191, seed=2)
    down_case(64, 256, 300, list(range(299, -1, -1)), "f16", scale=50.0)       # activations that round coarsely
    # the kernel for 65 to 128 rows: ids, counts, ranges of several chunks
    down_case(70, 256, 100, idx, "f16")
    down_case(128, 256, 100, idx, "bf16", count=17)
    down_case(90, 512, 100, idx, "bf16", count=1000)
    down_case(128, 256, 100, idx, "f16", count=0)
    down_case(65, 512, 100, [], "f16")
    down_case(100, 1024, 40000, rng.permutation(40000)[:20000].tolist(), "f16", seed=3, sample_cols=64)
    down_case(128, 4096, 9000, rng.permutation(9000)[:5000].tolist(), "bf16", count=4999, seed=4, sample_cols=96)


@pytest.mark.parametrize("B", [64, 128])
def test_sparsified_mlp_both_factors(B):
    """Union -> first factor -> second factor on one stream, no host round trip, against the
    oracle on sampled output columns (OPT-66B FFN shape); the one-call form gives the same bits."""
    w = wl.MLP_CONFIGS["M2_opt66b_ffn"]
    w = wl.MlpWorkload(w.name, B, w.K, w.N, w.density, w.dtype, w.seed)       # 128: the kernels for 65 to 128 rows
    say("\ncase both factors", w)
    x, W1, topk = wl.make_mlp_inputs(w, DEV)
    g = torch.Generator(device=DEV).manual_seed(w.seed + 1)
    W2 = (torch.randn((w.N, w.K), generator=g, device=DEV) / 100.0).to(W1.dtype)
    idx, count = polar.neuron_union(topk, w.N)
    hidden = polar.select_gemm(x, W1, idx, count=count, relu=True,
                               workspace=polar.alloc_select_gemm_workspace(w.B, DEV))
    y = polar.select_gemm_down(hidden, W2, idx, count=count)
    again = polar.select_gemm_down(hidden, W2, idx, count=count)
    one_call = polar.sparse_mlp(x, W1, W2, idx, count=count, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(y, one_call), "both factors in one call, at the size the bench times"
    c = int(count.item())
    cols = np.unique(np.linspace(0, w.K - 1, num=48).astype(np.int64))
    S = idx[:c].long()
    want = orc.select_gemm_down(hidden[:, :c].cpu().numpy(), host_bits(W2[S][:, torch.from_numpy(cols).to(DEV)]),
                                np.arange(c, dtype=np.int32), w.dtype)
    got = y[:, torch.from_numpy(cols).to(DEV)].cpu().numpy()
    err = np.abs(got - want).max()
    say("   %d live neurons, max-abs error %.3e on %d sampled columns, |y| up to %.2f" % (c, err, len(cols), np.abs(want).max()))
    assert err <= GEMM_TOL
    assert torch.isfinite(y).all() and torch.equal(y, again)


def gemm_form(form):
    """Force the first factor's one-launch kernel ("narrow") or leave the choice to the library (None)."""
    return polar.options(gemm_form=1 if form == "narrow" else None)


def mlp_case(M, D, N, idx_host, dtype, count=None, relu=True, seed=0, form=None):
    """polar_sparse_mlp against the two calls it stands for (bit for bit: same kernels, same order
    of additions) and against the oracle's two definitions applied one after the other.  The
    hidden activations are rounded to 16 bits between the factors; where the GPU's float sum and
    the oracle's double sum fall on different sides of a rounding boundary the hidden value differs
    by one unit in the last place: those cases are counted, and the tolerance is widened by exactly
    what they can contribute."""
    g = torch.Generator(device=DEV).manual_seed(4000 + seed)
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    X = torch.randn((M, D), generator=g, device=DEV).to(tdt)
    W1 = (torch.randn((N, D), generator=g, device=DEV) / D ** 0.5).to(tdt)
    W2 = (torch.randn((N, D), generator=g, device=DEV) / 30.0).to(tdt)
    cap = len(idx_host)
    idx = torch.tensor(idx_host, dtype=torch.int32, device=DEV)
    cnt = None if count is None else torch.tensor([count], dtype=torch.int32, device=DEV)
    nbytes = polar.sparse_mlp_workspace_bytes(M, D, cap)
    ws = torch.full((max(nbytes, 256) // 4,), float("nan"), dtype=torch.float32, device=DEV)   # poisoned
    y = torch.full((M, D), float("nan"), dtype=torch.float32, device=DEV)
    with gemm_form(form):
        polar.sparse_mlp(X, W1, W2, idx, count=cnt, relu=relu, out=y, workspace=ws)
        again = polar.sparse_mlp(X, W1, W2, idx, count=cnt, relu=relu, workspace=ws)
        hidden = torch.full((M, cap), float("nan"), dtype=torch.float32, device=DEV)
        for m0 in range(0, M if cap > 0 else 0, 128):       # as the one call does: 128 rows at a time (the order
            rows = min(128, M - m0)                          # of the additions depends on the pass's row count)
            polar.select_gemm(X[m0:m0 + rows], W1, idx, count=cnt, relu=relu, out=hidden[m0:m0 + rows],
                              workspace=polar.alloc_select_gemm_workspace(rows, DEV))
        two = polar.select_gemm_down(hidden, W2, idx, count=cnt)
    torch.cuda.synchronize()
    assert torch.isfinite(y).all()
    assert torch.equal(y, again) and torch.equal(y, two)
    live = cap if count is None else max(0, min(count, cap))
    ids = np.array(idx_host[:live], np.int32)
    H = orc.select_gemm(host_bits(X), host_bits(W1), ids, dtype, relu)
    want = orc.select_gemm_down(H.astype(np.float32), host_bits(W2), ids, dtype)
    # Where do the GPU's 16-bit hidden values differ from the oracle's?  `hidden` holds the float
    # sums the GPU rounds (the two-call form is bit-identical to the one call); round both sides'
    # values to the storage type on the host and count, per request, the neurons whose 16-bit
    # value differs and by how much.  Each such neuron moves every output of its row by at most
    # |difference| * max|W2 row|: that sum, not a guessed multiple of an ulp, widens the bound.
    got_h16 = hidden[:, :live].to(tdt).float().cpu().numpy().astype(np.float64)
    want_h16 = torch.from_numpy(H.astype(np.float32)).to(tdt).float().numpy().astype(np.float64)
    valid = (ids >= 0) & (ids < N)
    w2max = np.zeros(live)
    if live:
        w2max[valid] = W2[torch.from_numpy(ids[valid]).long().to(DEV)].abs().max(dim=1).values.float().cpu().numpy()
    delta = np.abs(got_h16 - want_h16) * valid[None, :]
    flips = int((delta > 0).sum())
    allowance = float((delta * w2max[None, :]).sum(axis=1).max()) if live and M else 0.0
    tol = GEMM_TOL + allowance
    err = np.abs(y.cpu().numpy() - want).max()
    say("   M=%d D=%d N=%d cap=%d live=%d %s relu=%s form=%s: max-abs error %.3e; %d of %d hidden values round "
        "differently, worth at most %.2e per output (tolerance %.1e)"
        % (M, D, N, cap, live, dtype, relu, form, err, flips, M * live, allowance, tol))
    assert flips <= max(4, (M * live) // 50)           # rounding-boundary cases are rare, not the rule
    assert err <= tol


def test_sparse_mlp_one_call():
    """Both factors in one call, hidden activations kept in 16-bit form in the workspace."""
    say("\ncase sparse_mlp one call")
    rng = np.random.default_rng(31)
    mlp_case(64, 512, 4000, sorted(rng.permutation(4000)[:1500].tolist()), "f16")
    mlp_case(33, 256, 900, rng.permutation(900)[:333].tolist(), "bf16", seed=1)          # ragged rows, odd count
    mlp_case(1, 1024, 700, sorted(rng.permutation(700)[:129].tolist()), "f16", seed=2)
    mlp_case(16, 512, 3000, rng.permutation(3000)[:1000].tolist(), "bf16", count=517, seed=3)
    mlp_case(48, 256, 600, [5, -1, 7, 600, 9] + list(range(100, 300)), "f16", seed=4)     # ids outside [0, N)
    mlp_case(20, 256, 500, list(range(64)), "f16", count=0, seed=5)                       # nothing live: zeros
    mlp_case(24, 512, 500, list(range(200)), "f16", relu=False, seed=6)
    mlp_case(100, 512, 2000, sorted(rng.permutation(2000)[:700].tolist()), "f16", seed=7)   # two passes of rows
    mlp_case(150, 256, 1000, rng.permutation(1000)[:400].tolist(), "bf16", count=390, seed=8)
    mlp_case(40, 512, 2000, sorted(rng.permutation(2000)[:900].tolist()), "f16", seed=9, form="narrow")   # one-launch first factor
    mlp_case(8, 256, 300, [], "f16", seed=10)                                             # cap = 0


def test_sparse_mlp_random_shapes():
    """Seeded random batch sizes, widths, capacities, live counts and id lists (repeats and ids
    outside [0, N) included) through the one-call form, the two calls and the oracle."""
    say("\ncase sparse_mlp random shapes")
    rng = np.random.default_rng(2024)
    for case in range(24):
        M = int(rng.choice([1, 2, 7, 16, 17, 31, 32, 48, 64, 65, 90, 128, 129, 200]))
        D = int(rng.choice([256, 512, 768, 1024]))
        N = int(rng.integers(40, 3000))
        cap = int(rng.integers(1, min(N, 1200) + 1))
        ids = rng.integers(-2, N + 2, size=cap)                  # a few invalid ones at either end
        if case % 3 == 0:
            ids = np.sort(ids)
        count = None if case % 4 == 0 else int(rng.integers(0, cap + 40))
        mlp_case(M, D, N, ids.tolist(), "f16" if case % 2 == 0 else "bf16", count=count, relu=case % 5 != 0,
                 seed=100 + case)


def test_hip_graph_replays_of_the_sparsified_mlp_match_eager():
    """Neuron index -> first factor -> second factor recorded into one HIP graph: the live count
    never leaves the device, so one recording serves whatever ids the requests predict; every
    replay, with eager work in between, equals the eager result bit for bit.  A second graph holds
    the index and the one-call form of both factors."""
    B, K, N, kn = 24, 512, 3000, 90
    say("\ncase sparsified MLP graph", B, K, N, kn)
    g = torch.Generator(device=DEV).manual_seed(77)
    x = torch.randn((B, K), generator=g, device=DEV).half()
    W1 = (torch.randn((N, K), generator=g, device=DEV) / K ** 0.5).half()
    W2 = (torch.randn((N, K), generator=g, device=DEV) / 30.0).half()
    topk = torch.randint(0, N, (B, kn), generator=g, device=DEV, dtype=torch.int32)
    cap = min(N, B * kn)
    ws_union = torch.empty(max(polar.neuron_union_workspace_bytes(B, kn, N), 4), dtype=torch.uint8, device=DEV)
    ws_up = polar.alloc_select_gemm_workspace(B, DEV)
    ws_down = torch.empty(polar.select_gemm_down_workspace_bytes(B, K, cap), dtype=torch.uint8, device=DEV)
    ws_mlp = torch.empty(polar.sparse_mlp_workspace_bytes(B, K, cap), dtype=torch.uint8, device=DEV)

    def bufs():
        return (torch.full((cap,), -1, dtype=torch.int32, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV),
                torch.zeros((B, cap), dtype=torch.float32, device=DEV), torch.zeros((B, K), dtype=torch.float32, device=DEV))

    def step(idx, count, hidden, y):
        polar.neuron_union(topk, N, workspace=ws_union, out=(idx, count))
        polar.select_gemm(x, W1, idx, count=count, relu=True, out=hidden, workspace=ws_up)
        polar.select_gemm_down(hidden, W2, idx, count=count, out=y, workspace=ws_down)

    def one_call_step(idx, count, hidden, y):
        polar.neuron_union(topk, N, workspace=ws_union, out=(idx, count))
        polar.sparse_mlp(x, W1, W2, idx, count=count, relu=True, out=y, workspace=ws_mlp)

    rec, rec1 = bufs(), bufs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        step(*rec)
        one_call_step(*rec1)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph, graph1 = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(*rec)
    with torch.cuda.graph(graph1):
        one_call_step(*rec1)
    for rep in range(4):
        # other ids (and with them another live count) and other activations every time
        hot = max(kn, N // (rep + 2))
        topk.copy_(torch.randint(0, hot, (B, kn), generator=g, device=DEV, dtype=torch.int32))
        x.copy_(torch.randn((B, K), generator=g, device=DEV).half())
        eager = bufs()
        step(*eager)
        torch.cuda.synchronize()
        rec[3].fill_(float("nan"))
        rec1[3].fill_(float("nan"))
        graph.replay()
        graph1.replay()
        torch.cuda.synchronize()
        c = int(eager[1].item())
        assert int(rec[1].item()) == c and torch.equal(rec[0][:c], eager[0][:c]), "replay %d: index" % rep
        assert torch.equal(rec[2][:, :c], eager[2][:, :c]), "replay %d: first factor" % rep
        assert torch.equal(rec[3].view(torch.int32), eager[3].view(torch.int32)), "replay %d: second factor" % rep
        assert torch.equal(rec1[3].view(torch.int32), eager[3].view(torch.int32)), "replay %d: one call" % rep
    S = orc.neuron_union(topk.cpu().numpy(), N)
    assert c == len(S)
    hid = orc.select_gemm(host_bits(x), host_bits(W1), S, "f16", True)
    assert np.abs(rec[2][:, :c].cpu().numpy() - hid).max() <= GEMM_TOL
    want = orc.select_gemm_down(rec[2][:, :c].cpu().numpy(), host_bits(W2), S, "f16")
    assert np.abs(rec[3].cpu().numpy() - want).max() <= GEMM_TOL


def test_read_probe_folds_every_word_of_every_slab():
    """The bandwidth yardstick really reads what it claims: each slab's result is the XOR of its
    words (slabs of whole 16 KiB wave steps, so no clamped tail load repeats a word)."""
    g = torch.Generator(device=DEV).manual_seed(3)
    slab_bytes, slabs = 3 * 16384, 37
    data = torch.randint(-2 ** 31, 2 ** 31 - 1, (slabs, slab_bytes // 4), generator=g, device=DEV,
                         dtype=torch.int32)
    want = np.bitwise_xor.reduce(data.cpu().numpy().view(np.uint32), axis=1)
    for nt in (True, False):
        got = polar.probe_read(data, slab_bytes, nt)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want)


def test_empty_batch_is_a_noop():
    e16 = torch.empty((0, 8, 64), dtype=torch.float16, device=DEV)
    kv = torch.empty((0, 8, 128, 64), dtype=torch.float16, device=DEV)
    n = torch.empty((0,), dtype=torch.int32, device=DEV)
    idx = torch.empty((0, 4), dtype=torch.int32, device=DEV)
    out = polar.sha_decode(e16, kv, kv, n, idx, 4)
    assert tuple(out.shape) == (0, 8, 64)
    got = polar.router_topk(torch.empty((0, 64), dtype=torch.float16, device=DEV),
                            torch.zeros((64, 8), dtype=torch.float16, device=DEV), 4)
    assert tuple(got.shape) == (0, 4)
    torch.cuda.synchronize()


def test_phases_compose_to_the_single_call():
    w = wl.CONFIGS["C1_tiny"]
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV)
    head_idx = wl.random_head_idx(w, DEV)
    ws = polar.alloc_workspace(w.B, w.Hq, w.Hkv, w.S, w.d, w.k, DEV)
    a = polar.sha_decode(q, K, V, seqlens, head_idx, w.k, workspace=ws)
    out = torch.empty_like(a)
    polar.sha_partial(q, K, V, seqlens, head_idx, w.k, ws)
    polar.sha_merge(seqlens, head_idx, out, w.Hkv, w.S, w.k, ws)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int32), out.view(torch.int32))


def test_non_default_stream():
    w = wl.CONFIGS["C1_tiny"]
    q, K, V, seqlens = wl.make_attention_inputs(w, DEV)
    hidden, Wr = wl.make_router_inputs(w, DEV)
    torch.cuda.synchronize()
    rws = polar.alloc_router_workspace(w.B, w.D, w.Hkv, DEV)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        head_idx = polar.router_topk(hidden, Wr, w.k, workspace=rws)
        out = polar.sha_decode(q, K, V, seqlens, head_idx, w.k)
    s.synchronize()
    check_against_oracle(w, q, K, V, seqlens, head_idx, out)


# ----------------------------------------------------------------------------- router edge cases
def router_case(hidden, Wr, k, dtype):
    want = orc.router_topk(host_bits(hidden), host_bits(Wr), k, dtype)
    B, D = hidden.shape
    for ws, path, mfma in ROUTER_MODES:
        with router_path(path, mfma):
            rws = polar.alloc_router_workspace(B, D, Wr.shape[1], DEV).fill_(0xFF) if ws else None
            got = polar.router_topk(hidden, Wr, k, workspace=rws)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want), (ws, path, mfma)
    return want


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,D,H,k", [(1, 1, 1, 1), (3, 17, 5, 2), (5, 1000, 72, 36),
                                     (2, 4096, 256, 256), (7, 333, 100, 1), (4, 16384, 8, 4),
                                     (2, 3, 200, 50), (9, 777, 6, 3), (130, 640, 32, 8),
                                     (6, 513, 255, 17)])
def test_router_shapes(dtype, B, D, H, k):
    say("\ncase router", dtype, B, D, H, k)
    g = torch.Generator(device=DEV).manual_seed(B * 1000 + D + H)
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    hidden = torch.randn((B, D), generator=g, device=DEV).to(tdt)
    Wr = (torch.randn((D, H), generator=g, device=DEV) / D ** 0.5).to(tdt)
    router_case(hidden, Wr, k, dtype)


def test_router_ties():
    say("\ncase router ties")
    g = torch.Generator(device=DEV).manual_seed(77)
    D, H = 512, 16
    Wr = (torch.randn((D, H), generator=g, device=DEV) / D ** 0.5).to(torch.float16)
    Wr[:, 9] = Wr[:, 4]
    Wr[:, 15] = Wr[:, 4]                                       # three identical columns
    hidden = torch.randn((32, D), generator=g, device=DEV).to(torch.float16)
    want = router_case(hidden, Wr, H, "f16")
    for row in want.tolist():
        assert row.index(9) == row.index(4) + 1 and row.index(15) == row.index(9) + 1
    zero = torch.zeros((3, D), dtype=torch.float16, device=DEV)
    assert router_case(zero, Wr, 5, "f16").tolist() == [[0, 1, 2, 3, 4]] * 3
    # small integers: every partial sum is exact, so many exact ties between different columns
    hi = torch.randint(-2, 3, (16, 64), generator=g, device=DEV).to(torch.bfloat16)
    Wi = torch.randint(-1, 2, (64, 24), generator=g, device=DEV).to(torch.bfloat16)
    router_case(hi, Wi, 12, "bf16")
    # signed zeros: +0 and -0 logits tie and fall back to the id order
    hz = torch.zeros((1, 8), dtype=torch.float16, device=DEV)
    hz[0, 0] = 1.0
    Wz = torch.zeros((8, 6), dtype=torch.float16, device=DEV)
    Wz[0] = torch.tensor([0.0, -0.0, 0.0, -0.0, 0.0, -0.0])
    assert router_case(hz, Wz, 6, "f16").tolist() == [[0, 1, 2, 3, 4, 5]]


@pytest.mark.parametrize("depth", [1, 4])
def test_gather_probe_folds_every_word_of_every_gathered_row(depth):
    """The gathered-row yardstick really reads what it claims: each wave's result is the XOR of
    its 32 rows' words in its slice of K (ids out of range read row 0; a ragged last tile repeats
    its last entry)."""
    g = torch.Generator(device=DEV).manual_seed(11)
    N, K, slices = 300, 1536, 3
    W = torch.randint(-2 ** 15, 2 ** 15 - 1, (N, K), generator=g, device=DEV, dtype=torch.int16)
    ids = torch.randint(0, N, (150,), generator=g, device=DEV, dtype=torch.int32)
    ids[7], ids[99] = -1, N
    for nt in (False, True):
        sink = polar.probe_gather_read(W, ids, slices=slices, depth=depth, nontemporal=nt)
        torch.cuda.synchronize()
        got = sink.cpu().numpy().view(np.uint32)
        words = W.cpu().numpy().view(np.uint32).reshape(N, K // 2)
        idh = ids.cpu().numpy().copy()
        idh[(idh < 0) | (idh >= N)] = 0
        per = K // 2 // slices
        for tile in range(3):
            for sl in range(slices):
                for wave in range(2):
                    first = tile * 64 + wave * 32
                    if first >= len(idh):
                        continue
                    rows = [idh[min(first + r, len(idh) - 1)] for r in range(32)]
                    want = np.bitwise_xor.reduce(words[rows, sl * per:(sl + 1) * per].reshape(-1))
                    assert got[2 * (tile * slices + sl) + wave] == want, (depth, nt, tile, sl, wave)

