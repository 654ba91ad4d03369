"""Pins of the fp64 CPU oracle against what the paper's definitions and the mathematics fix.

The paper prints no worked numeric example for the router or the attention
kernel, so every pin here is a closed form, an invariant, a brute force on a
tiny input, or a library routine (numpy / torch CPU in float64) evaluating the
same definition by a different route.  None of these tests touches the HIP
library.
"""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import polar_oracle as orc

RNG = np.random.default_rng(20250514)


# ----------------------------------------------------------------------------- helpers
def f16_bits(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def bf16_bits(a):
    t = torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.float32))).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bits_of(a, dtype):
    return f16_bits(a) if dtype == "f16" else bf16_bits(a)


def as_f64(bits, dtype):
    """Independent widening: numpy for fp16, integer shift into a float32 for bf16."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def dense_reference(q, K, V, n, scale=None):
    """softmax(q K^T / sqrt(d)) V by torch's CPU attention routine in float64.
    q [Hq,d], K/V [Hkv,S,d] float64, first n rows valid; Hq == Hkv here."""
    qt = torch.from_numpy(q)[:, None, :]                 # [H,1,d]
    kt = torch.from_numpy(K[:, :n])
    vt = torch.from_numpy(V[:, :n])
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=scale)
    return o[:, 0, :].numpy()


def random_case(B, Hq, Hkv, S, d, dtype, lo=1):
    q = bits_of(RNG.standard_normal((B, Hq, d)), dtype)
    K = bits_of(RNG.standard_normal((B, Hkv, S, d)), dtype)
    V = bits_of(RNG.standard_normal((B, Hkv, S, d)), dtype)
    n = RNG.integers(lo, S + 1, size=B).astype(np.int32)
    return q, K, V, n


# ----------------------------------------------------------------------------- storage decoding
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_widening_of_every_bit_pattern(dtype):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.widen16(bits, dtype)
    want = as_f64(bits, dtype)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ----------------------------------------------------------------------------- router
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,D,H", [(3, 17, 5), (4, 512, 8), (2, 4096, 32)])
def test_router_logits_equal_matrix_product(dtype, B, D, H):
    hid = bits_of(RNG.standard_normal((B, D)), dtype)
    Wr = bits_of(RNG.standard_normal((D, H)) / math.sqrt(D), dtype)
    got = orc.router_logits(hid, Wr, dtype)
    want = as_f64(hid, dtype) @ as_f64(Wr, dtype)
    assert got.shape == (B, H)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    # a transposed weight layout ([H,D] read as [D,H]) must not pass by accident
    wrong = as_f64(hid, dtype) @ as_f64(Wr, dtype).reshape(H, D).T
    assert not np.allclose(got, wrong, rtol=1e-3, atol=1e-3)


def test_router_small_integer_inputs_are_exact():
    hid = f16_bits(RNG.integers(-3, 4, size=(5, 64)))
    Wr = f16_bits(RNG.integers(-3, 4, size=(64, 6)))
    got = orc.router_logits(hid, Wr, "f16")
    want = as_f64(hid, "f16").astype(np.int64) @ as_f64(Wr, "f16").astype(np.int64)
    assert np.array_equal(got, want.astype(np.float64))


# ----------------------------------------------------------------------------- top-k
def brute_force_topk(row, k):
    """The unique k-subset in which every member beats every non-member under
    (larger logit, then lower id), listed best first.  NaN-free rows only."""
    H = len(row)

    def beats(a, b):
        return row[a] > row[b] or (row[a] == row[b] and a < b)

    for sub in itertools.combinations(range(H), k):
        rest = [h for h in range(H) if h not in sub]
        if all(beats(a, b) for a in sub for b in rest):
            order = list(sub)
            for i in range(len(order)):           # selection sort under the same relation
                for j in range(i + 1, len(order)):
                    if beats(order[j], order[i]):
                        order[i], order[j] = order[j], order[i]
            return order
    raise AssertionError("no dominating subset")


def test_topk_brute_force_tiny():
    for H in (1, 2, 5, 8):
        for k in range(1, H + 1):
            x = RNG.standard_normal((6, H))
            x[1] = np.round(x[1])                 # many ties
            x[2] = 0.0
            got = orc.topk(x, k)
            for b in range(x.shape[0]):
                assert got[b].tolist() == brute_force_topk(x[b], k), (H, k, b)


def test_topk_equals_stable_argsort():
    x = RNG.standard_normal((64, 72))
    x[:, 10] = x[:, 3]                            # duplicated columns -> exact ties
    x[5] = np.round(x[5] * 2) / 2
    for k in (1, 7, 36, 72):
        got = orc.topk(x, k)
        want = np.argsort(-x, axis=1, kind="stable")[:, :k]
        assert np.array_equal(got, want.astype(np.int32))


def test_topk_tie_rules():
    assert orc.topk(np.zeros((2, 8)), 3).tolist() == [[0, 1, 2], [0, 1, 2]]
    # -0.0 and +0.0 are one value: order by id
    assert orc.topk(np.array([[-0.0, 0.0, -0.0, 0.0]]), 4).tolist() == [[0, 1, 2, 3]]
    assert orc.topk(np.array([[0.0, -0.0, 1.0]]), 2).tolist() == [[2, 0]]
    # NaN ranks after every number (even -inf), NaNs among themselves by id
    x = np.array([[np.nan, -np.inf, 2.0, np.nan, 1.0]])
    assert orc.topk(x, 5).tolist() == [[2, 4, 1, 0, 3]]
    # k == H is a full ordering, k == 1 an argmax with lowest-id tie-break
    assert orc.topk(np.array([[1.0, 3.0, 3.0, 2.0]]), 1).tolist() == [[1]]


def test_router_topk_all_zero_hidden_and_duplicate_columns():
    D, H = 128, 8
    Wr = RNG.standard_normal((D, H)) / math.sqrt(D)
    Wr[:, 5] = Wr[:, 2]
    Wrb = f16_bits(Wr)
    zero = f16_bits(np.zeros((2, D)))
    assert orc.router_topk(zero, Wrb, 4, "f16").tolist() == [[0, 1, 2, 3]] * 2
    hid = f16_bits(RNG.standard_normal((16, D)))
    logits = orc.router_logits(hid, Wrb, "f16")
    assert np.array_equal(logits[:, 5], logits[:, 2])          # bit-identical sums
    idx = orc.router_topk(hid, Wrb, H, "f16")
    for row in idx.tolist():                                   # 2 always directly before 5
        assert row.index(5) == row.index(2) + 1


# ----------------------------------------------------------------------------- attention, k = H
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("B,H,S,d", [(2, 3, 37, 16), (4, 8, 256, 64), (1, 2, 1920, 128)])
def test_dense_equals_library_softmax_attention(dtype, B, H, S, d):
    q, K, V, n = random_case(B, H, H, S, d, dtype)
    got = orc.sha_decode(q, K, V, n, None, H, dtype)
    ident = np.tile(np.arange(H, dtype=np.int32), (B, 1))
    got_idx = orc.sha_decode(q, K, V, n, ident, H, dtype)
    assert np.array_equal(got, got_idx)
    for b in range(B):
        want = dense_reference(as_f64(q[b], dtype), as_f64(K[b], dtype), as_f64(V[b], dtype), int(n[b]))
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-13)


def test_explicit_scale_and_default_scale():
    q, K, V, n = random_case(1, 2, 2, 50, 32, "f16")
    got = orc.sha_decode(q, K, V, n, None, 2, "f16", scale=0.3)
    want = dense_reference(as_f64(q[0], "f16"), as_f64(K[0], "f16"), as_f64(V[0], "f16"), int(n[0]), scale=0.3)
    np.testing.assert_allclose(got[0], want, rtol=1e-11, atol=1e-13)
    dflt = orc.sha_decode(q, K, V, n, None, 2, "f16")
    expl = orc.sha_decode(q, K, V, n, None, 2, "f16", scale=1.0 / math.sqrt(32))
    np.testing.assert_allclose(dflt, expl, rtol=1e-15)
    assert not np.allclose(dflt, got)


def test_numpy_softmax_written_out():
    """Same definition through numpy: softmax(q K^T / sqrt(d)) V."""
    q, K, V, n = random_case(3, 4, 4, 100, 64, "bf16")
    got = orc.sha_decode(q, K, V, n, None, 4, "bf16")
    qf, Kf, Vf = as_f64(q, "bf16"), as_f64(K, "bf16"), as_f64(V, "bf16")
    for b in range(3):
        nb = int(n[b])
        s = np.einsum("hd,hjd->hj", qf[b], Kf[b, :, :nb]) / math.sqrt(64)
        w = np.exp(s - s.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        want = np.einsum("hj,hjd->hd", w, Vf[b, :, :nb])
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------- closed forms
def test_geometric_scores_closed_form():
    """d = 64 so 1/sqrt(d) = 1/8.  q = 8 e_0 and K_j = j e_0 give scores s_j = j exactly;
    V_j = e_j then makes out[j] = e^j (e - 1) / (e^n - 1), a geometric series.
    Fails if the scale, the exponent's sign or the normalisation is wrong."""
    d, n = 64, 12
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 8.0
    K = np.zeros((1, 1, n, d)); K[0, 0, :, 0] = np.arange(n)
    V = np.zeros((1, 1, n, d)); V[0, 0, np.arange(n), np.arange(n)] = 1.0
    out = orc.sha_decode(f16_bits(q), f16_bits(K), f16_bits(V), np.array([n], np.int32), None, 1, "f16")
    want = np.zeros(d)
    want[:n] = [math.exp(j) * (math.e - 1.0) / (math.exp(n) - 1.0) for j in range(n)]
    np.testing.assert_allclose(out[0, 0], want, rtol=1e-13, atol=1e-18)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_equal_keys_give_mean_of_values(dtype):
    B, H, S, d = 2, 3, 40, 32
    q, K, V, n = random_case(B, H, H, S, d, dtype, lo=5)
    K[:] = K[:, :, :1, :]                                    # every row of a head identical
    got = orc.sha_decode(q, K, V, n, None, H, dtype)
    Vf = as_f64(V, dtype)
    for b in range(B):
        np.testing.assert_allclose(got[b], Vf[b, :, : n[b]].mean(axis=1), rtol=1e-14, atol=1e-15)


def test_dominant_key_returns_its_value_row():
    d, S, n = 64, 64, 50
    q, K, V, _ = random_case(1, 1, 1, S, d, "f16")
    qf = as_f64(q, "f16")[0, 0]
    Kf = as_f64(K, "f16")
    star = 17
    # key = c*q with c making its scaled score exceed every other by at least 50
    others = (Kf[0, 0, :n] @ qf) / 8.0
    c = (np.abs(others).max() + 60.0) * 8.0 / (qf @ qf)
    K[0, 0, star] = f16_bits(c * qf)
    Kf = as_f64(K, "f16")
    gap = (Kf[0, 0, star] @ qf) / 8.0 - np.delete((Kf[0, 0, :n] @ qf) / 8.0, star).max()
    assert gap >= 50.0
    got = orc.sha_decode(q, K, V, np.array([n], np.int32), None, 1, "f16")
    Vf = as_f64(V, "f16")
    err = np.abs(got[0, 0] - Vf[0, 0, star]).max()
    assert err <= n * math.exp(-50.0) * 2 * np.abs(Vf[0, 0, :n]).max()


def test_length_one_and_length_zero():
    q, K, V, _ = random_case(2, 2, 2, 8, 16, "bf16")
    n = np.array([1, 0], np.int32)
    got = orc.sha_decode(q, K, V, n, None, 2, "bf16")
    assert np.array_equal(got[0], as_f64(V, "bf16")[0, :, 0, :])
    assert np.array_equal(got[1].view(np.uint64), np.zeros_like(got[1]).view(np.uint64))
    # lengths beyond the capacity are clamped to it, negative ones to zero
    a = orc.sha_decode(q, K, V, np.array([99, -5], np.int32), None, 2, "bf16")
    b = orc.sha_decode(q, K, V, np.array([8, 0], np.int32), None, 2, "bf16")
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------- invariants
def test_skipped_heads_are_exactly_positive_zero_and_selected_match_dense():
    B, H, S, d, k = 3, 8, 33, 16, 3
    q, K, V, n = random_case(B, H, H, S, d, "f16")
    idx = np.stack([RNG.permutation(H)[:k] for _ in range(B)]).astype(np.int32)
    got = orc.sha_decode(q, K, V, n, idx, k, "f16")
    dense = orc.sha_decode(q, K, V, n, None, H, "f16")
    for b in range(B):
        for h in range(H):
            if h in idx[b]:
                assert np.array_equal(got[b, h], dense[b, h])
            else:
                assert np.array_equal(got[b, h].view(np.uint64), np.zeros(d, np.uint64))


def test_nan_canaries_in_padding_and_unselected_heads_never_reach_output():
    B, H, S, d, k = 2, 6, 20, 16, 2
    q, K, V, n = random_case(B, H, H, S, d, "bf16")
    n[:] = [7, 13]
    idx = np.array([[4, 1], [0, 5]], np.int32)
    clean = orc.sha_decode(q, K, V, n, idx, k, "bf16")
    nanbits = np.uint16(0x7FC0)
    for b in range(B):
        K[b, :, n[b]:] = nanbits
        V[b, :, n[b]:] = nanbits
        for h in range(H):
            if h not in idx[b]:
                K[b, h] = nanbits
                V[b, h] = nanbits
                q[b, h] = nanbits
    got = orc.sha_decode(q, K, V, n, idx, k, "bf16")
    assert np.isfinite(got).all()
    assert np.array_equal(got, clean)


def test_out_of_range_and_duplicate_ids():
    B, H, S, d = 1, 4, 10, 8
    q, K, V, n = random_case(B, H, H, S, d, "f16")
    dense = orc.sha_decode(q, K, V, n, None, H, "f16")
    got = orc.sha_decode(q, K, V, n, np.array([[2, -1, 2, 7]], np.int32), 4, "f16")
    assert np.array_equal(got[0, 2], dense[0, 2])
    assert not got[0, [0, 1, 3]].any()


def test_joint_row_permutation_leaves_output_unchanged():
    q, K, V, _ = random_case(1, 2, 2, 64, 32, "f16")
    n = np.array([64], np.int32)
    perm = RNG.permutation(64)
    a = orc.sha_decode(q, K, V, n, None, 2, "f16")
    b = orc.sha_decode(q, K[:, :, perm], V[:, :, perm], n, None, 2, "f16")
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    # permuting K alone is a different problem: the pairing of key and value rows matters
    c = orc.sha_decode(q, K[:, :, perm], V, n, None, 2, "f16")
    assert not np.allclose(a, c, atol=1e-3)


def test_adding_one_vector_to_every_key_leaves_output_unchanged():
    """softmax shift invariance; values on a 1/8 grid so the shifted keys are exact in fp16."""
    d, n = 32, 48
    q = RNG.integers(-8, 9, size=(1, 1, d)) / 8.0
    K = RNG.integers(-16, 17, size=(1, 1, n, d)) / 8.0
    V = RNG.standard_normal((1, 1, n, d))
    u = RNG.integers(-16, 17, size=d) / 8.0
    nn = np.array([n], np.int32)
    a = orc.sha_decode(f16_bits(q), f16_bits(K), f16_bits(V), nn, None, 1, "f16")
    b = orc.sha_decode(f16_bits(q), f16_bits(K + u), f16_bits(V), nn, None, 1, "f16")
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_output_lies_in_the_convex_hull_of_value_rows():
    q, K, V, n = random_case(2, 3, 3, 70, 16, "bf16", lo=3)
    got = orc.sha_decode(q, K, V, n, None, 3, "bf16")
    Vf = as_f64(V, "bf16")
    for b in range(2):
        lo = Vf[b, :, : n[b]].min(axis=1)
        hi = Vf[b, :, : n[b]].max(axis=1)
        assert (got[b] >= lo - 1e-12).all() and (got[b] <= hi + 1e-12).all()


# ----------------------------------------------------------------------------- GQA
@pytest.mark.parametrize("Hq", [8, 6, 14])          # groups of 4, 3 and 7 query heads
def test_group_selection_equals_mha_on_repeated_kv(Hq):
    B, Hkv, S, d, k = 2, 2, 30, 16, 1
    G = Hq // Hkv
    q, K, V, n = random_case(B, Hq, Hkv, S, d, "bf16")
    idx = np.array([[1], [0]], np.int32)
    got = orc.sha_decode(q, K, V, n, idx, k, "bf16")
    Krep = np.repeat(K, G, axis=1)
    Vrep = np.repeat(V, G, axis=1)
    idx_q = np.stack([np.concatenate([np.arange(g * G, (g + 1) * G) for g in row]) for row in idx])
    want = orc.sha_decode(q, Krep, Vrep, n, idx_q.astype(np.int32), k * G, "bf16")
    assert np.array_equal(got, want)
    assert not got[0, :G].any() and got[0, G:].all()        # request 0 skips group 0
    assert got[1, :G].all() and not got[1, G:].any()


# ----------------------------------------------------------------------------- Algorithm 1
@pytest.mark.parametrize("Bc", [1, 7, 16, 64, 100, 1000])
def test_algorithm1_recurrence_equals_two_pass_definition(Bc):
    n, d = 100, 32
    q, K, V, _ = random_case(1, 1, 1, n, d, "f16")
    K[0, 0, 40] = f16_bits(as_f64(K[0, 0, 40], "f16") * 6.0)   # a late, much larger score
    two_pass = orc.sha_decode(q, K, V, np.array([n], np.int32), None, 1, "f16")[0, 0]
    tiled = orc.alg1_tiled(as_f64(q, "f16")[0, 0], as_f64(K, "f16")[0, 0], as_f64(V, "f16")[0, 0],
                           Bc, 1.0 / math.sqrt(d))
    np.testing.assert_allclose(tiled, two_pass, rtol=1e-12, atol=1e-14)


def test_partition_merge_algebra():
    """Splitting the rows into parts, keeping (max, sum, unnormalised output) per part and
    combining them with the running-max rescale reproduces the whole; empty parts drop out.
    This is the identity the split-KV GPU kernel relies on (same recurrence as Algorithm 1)."""
    n, d = 90, 16
    q, K, V, _ = random_case(1, 1, 1, n, d, "f16")
    whole = orc.sha_decode(q, K, V, np.array([n], np.int32), None, 1, "f16")[0, 0]
    qf, Kf, Vf = as_f64(q, "f16")[0, 0], as_f64(K, "f16")[0, 0], as_f64(V, "f16")[0, 0]
    for cuts in ([0, 90], [0, 1, 90], [0, 30, 30, 64, 90], [0, 17, 55, 89, 90]):
        parts = []
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            if hi == lo:
                parts.append((-np.inf, 0.0, np.zeros(d)))
                continue
            s = Kf[lo:hi] @ qf / math.sqrt(d)
            m = s.max()
            p = np.exp(s - m)
            parts.append((m, p.sum(), p @ Vf[lo:hi]))
        m_star = max(m for m, _, _ in parts)
        l_star = sum(l * math.exp(m - m_star) for m, l, _ in parts)
        o_star = sum(o * math.exp(m - m_star) for m, _, o in parts) / l_star
        np.testing.assert_allclose(o_star, whole, rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------------------- head importance
def test_head_scores_equal_numpy_norms_and_group_pooling():
    B, Hq, Hkv, d = 3, 12, 4, 16
    attn = RNG.standard_normal((B, Hq, d))
    score, norms = orc.head_scores(attn, Hkv)
    want = np.linalg.norm(attn.reshape(B, Hkv, (Hq // Hkv) * d), axis=2)
    np.testing.assert_allclose(norms, want, rtol=1e-14)
    np.testing.assert_allclose(score, want ** 2, rtol=1e-13)
    # MHA: one score per head
    score1, norms1 = orc.head_scores(attn, Hq)
    np.testing.assert_allclose(norms1, np.linalg.norm(attn, axis=2), rtol=1e-14)
    # a wrong grouping (strided instead of contiguous heads) must not pass by accident
    wrong = np.linalg.norm(attn.reshape(B, Hq // Hkv, Hkv, d).transpose(0, 2, 1, 3).reshape(B, Hkv, -1), axis=2)
    assert not np.allclose(norms, wrong)


def test_head_importance_labels_closed_form():
    """Value rows of head h are all h+1 times a fixed unit vector, so every head's attention
    output is (h+1)*u whatever the scores are, its norm is h+1, and the labels are the k
    highest head ids in descending order."""
    B, H, S, d, k = 2, 6, 20, 16, 3
    q, K, V, n = random_case(B, H, H, S, d, "f16")
    u = np.zeros(d); u[3] = 1.0
    Vf = np.zeros((B, H, S, d))
    for h in range(H):
        Vf[:, h, :, :] = (h + 1) * u
    labels, score = orc.head_importance_labels(q, K, f16_bits(Vf), n, k, "f16")
    assert labels.tolist() == [[5, 4, 3]] * B
    np.testing.assert_allclose(score, np.tile((np.arange(H) + 1.0) ** 2, (B, 1)), rtol=1e-12)
    # equal norms: ties go to the lower id
    Vf[:] = u
    labels, _ = orc.head_importance_labels(q, K, f16_bits(Vf), n, k, "f16")
    assert labels.tolist() == [[0, 1, 2]] * B


def test_head_importance_labels_equal_numpy_route():
    B, Hq, Hkv, S, d, k = 3, 8, 4, 50, 16, 2
    q, K, V, n = random_case(B, Hq, Hkv, S, d, "bf16")
    labels, score = orc.head_importance_labels(q, K, V, n, k, "bf16")
    attn = orc.sha_decode(q, K, V, n, None, Hkv, "bf16")
    norms = np.linalg.norm(attn.reshape(B, Hkv, -1), axis=2)
    want = np.argsort(-norms, axis=1, kind="stable")[:, :k]
    assert np.array_equal(labels, want.astype(np.int32))


# ----------------------------------------------------------------------------- selective GEMM
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("relu", [True, False])
def test_select_gemm_equals_gathered_matrix_product(dtype, relu):
    M, K, N = 5, 96, 40
    A = bits_of(RNG.standard_normal((M, K)), dtype)
    W = bits_of(RNG.standard_normal((N, K)) / math.sqrt(K), dtype)
    idx = RNG.permutation(N)[:13].astype(np.int32)
    got = orc.select_gemm(A, W, idx, dtype, relu=relu)
    want = as_f64(A, dtype) @ as_f64(W, dtype)[idx].T
    if relu:
        want = np.maximum(want, 0.0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    assert relu == bool((got >= 0).all())
    # reading W as [K,N] (input-major) instead of one row per neuron must not pass
    wrong = as_f64(A, dtype) @ as_f64(W, dtype).reshape(K, N)[:, idx]
    assert not np.allclose(got, np.maximum(wrong, 0.0) if relu else wrong, atol=1e-3)


def test_select_gemm_one_hot_rows_pick_activation_columns():
    """Neuron n's weight row is e_{n mod K}: its pre-activation is A[:, n mod K] exactly."""
    M, K, N = 4, 16, 32
    A = RNG.integers(-5, 6, size=(M, K)).astype(np.float64)
    W = np.zeros((N, K)); W[np.arange(N), np.arange(N) % K] = 1.0
    idx = np.array([3, 19, 0, 31, 19], np.int32)                  # a repeated id repeats the column
    got = orc.select_gemm(f16_bits(A), f16_bits(W), idx, "f16", relu=True)
    assert np.array_equal(got, np.maximum(A[:, idx % K], 0.0))
    got_lin = orc.select_gemm(f16_bits(A), f16_bits(W), idx, "f16", relu=False)
    assert np.array_equal(got_lin, A[:, idx % K])


def test_select_gemm_invalid_ids_and_empty_selection():
    M, K, N = 3, 8, 6
    A = f16_bits(RNG.standard_normal((M, K)))
    W = f16_bits(RNG.standard_normal((N, K)))
    got = orc.select_gemm(A, W, np.array([2, -1, 6, 5], np.int32), "f16", relu=False)
    full = orc.select_gemm(A, W, np.arange(N, dtype=np.int32), "f16", relu=False)
    assert np.array_equal(got[:, 0], full[:, 2]) and np.array_equal(got[:, 3], full[:, 5])
    assert not got[:, 1:3].any()
    assert orc.select_gemm(A, W, np.zeros(0, np.int32), "f16").shape == (M, 0)


def test_neuron_union_is_the_sorted_set_of_valid_ids():
    B, kn, N = 7, 12, 50
    topk = RNG.integers(-3, N + 3, size=(B, kn)).astype(np.int32)
    got = orc.neuron_union(topk, N)
    want = sorted({int(v) for v in topk.ravel() if 0 <= v < N})
    assert got.tolist() == want
    assert orc.neuron_union(np.full((2, 3), -1, np.int32), N).tolist() == []
    assert orc.neuron_union(np.array([[4, 4, 4]], np.int32), N).tolist() == [4]


def test_select_gemm_on_union_equals_masked_dense_layer():
    """Section 3.1: with S_B the union of the requests' active sets, sigma(x W_{1,S_B}) is the
    dense layer's activation restricted to the columns in S_B."""
    B, K, N, kn = 6, 64, 48, 5
    x = bf16_bits(RNG.standard_normal((B, K)))
    W1 = bf16_bits(RNG.standard_normal((N, K)) / 8.0)
    dense = np.maximum(as_f64(x, "bf16") @ as_f64(W1, "bf16").T, 0.0)
    topk = np.argsort(-dense, axis=1)[:, :kn].astype(np.int32)       # each request's top neurons
    S = orc.neuron_union(topk, N)
    got = orc.select_gemm(x, W1, S, "bf16", relu=True)
    np.testing.assert_allclose(got, dense[:, S], rtol=1e-12, atol=1e-14)
    assert len(S) >= kn and len(S) <= min(N, B * kn)


# ----------------------------------------------------------------------------- second MLP factor
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_select_gemm_down_equals_library_product_of_rounded_activations(dtype):
    """The definition against library routines: the activations cast to the storage type by
    numpy (binary16) or torch (bfloat16), the gathered rows multiplied by numpy in double."""
    import torch
    M, n_sel, N, Kout = 7, 37, 50, 24
    H = (RNG.standard_normal((M, n_sel)) * 3.0).astype(np.float32)
    H[0, :4] = [0.0, 1e-7, 70000.0 if dtype == "bf16" else 60000.0, -2.5]
    W2 = (f16_bits if dtype == "f16" else bf16_bits)(RNG.standard_normal((N, Kout)))
    idx = RNG.integers(0, N, n_sel).astype(np.int32)
    if dtype == "f16":
        h16 = H.astype(np.float16).astype(np.float64)
    else:
        h16 = torch.from_numpy(H).to(torch.bfloat16).double().numpy()
    want = h16 @ as_f64(W2, dtype)[idx]
    got = orc.select_gemm_down(H, W2, idx, dtype)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_select_gemm_down_rounds_activations_to_nearest_even():
    """One-hot weight rows hand the rounded activation through: halfway cases of binary16 go to
    the even neighbour, also among subnormals; bfloat16 keeps 8 significant bits."""
    cases16 = [(1.0 + 2.0 ** -11, 1.0), (1.0 + 2.0 ** -11 + 2.0 ** -20, 1.0 + 2.0 ** -10),
               (1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -9), (2.0 ** -25, 0.0), (3 * 2.0 ** -25, 2.0 ** -23),
               (2.0 ** -24, 2.0 ** -24), (65519.0, 65504.0), (-0.3, float(np.float16(-0.3)))]
    H = np.array([[c[0] for c in cases16]], np.float32)
    n = H.shape[1]
    eye = f16_bits(np.eye(n))
    got = orc.select_gemm_down(H, eye, np.arange(n, dtype=np.int32), "f16")
    assert got[0].tolist() == [c[1] for c in cases16]
    casesb = [(1.0 + 2.0 ** -8, 1.0), (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6),
              (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7), (-7.0, -7.0), (2.0 ** -130, 2.0 ** -130)]
    Hb = np.array([[c[0] for c in casesb]], np.float32)
    nb = Hb.shape[1]
    gotb = orc.select_gemm_down(Hb, bf16_bits(np.eye(nb)), np.arange(nb, dtype=np.int32), "bf16")
    assert gotb[0].tolist() == [c[1] for c in casesb]


def test_select_gemm_down_ids_and_empty_selection():
    M, N, Kout = 3, 8, 5
    H = RNG.standard_normal((M, 4)).astype(np.float32)
    W2 = f16_bits(RNG.standard_normal((N, Kout)))
    w = as_f64(W2, "f16")
    h = H.astype(np.float16).astype(np.float64)
    got = orc.select_gemm_down(H, W2, np.array([2, -1, 8, 5], np.int32), "f16")     # -1 and 8 are skipped
    np.testing.assert_allclose(got, np.outer(h[:, 0], w[2]) + np.outer(h[:, 3], w[5]), rtol=1e-13, atol=1e-15)
    twice = orc.select_gemm_down(H[:, :2], W2, np.array([3, 3], np.int32), "f16")    # a repeated id adds twice
    np.testing.assert_allclose(twice, np.outer(h[:, 0] + h[:, 1], w[3]), rtol=1e-13, atol=1e-15)
    empty = orc.select_gemm_down(np.zeros((M, 0), np.float32), W2, np.zeros(0, np.int32), "f16")
    assert empty.shape == (M, Kout) and not empty.any()


def test_sparsified_mlp_over_all_neurons_is_the_dense_mlp():
    """Section 3.1: with S_B = every neuron, sigma(x W_1) W_2^T restricted to S_B is the dense
    two-layer block (numpy in double, activations held in the storage type)."""
    B, K, N = 5, 32, 24
    x = f16_bits(RNG.standard_normal((B, K)))
    W1 = f16_bits(RNG.standard_normal((N, K)) / 6.0)
    W2 = f16_bits(RNG.standard_normal((N, K)) / 5.0)                 # one row per neuron: W_2^T row-major
    hidden = np.maximum(as_f64(x, "f16") @ as_f64(W1, "f16").T, 0.0)
    dense = hidden.astype(np.float32).astype(np.float16).astype(np.float64) @ as_f64(W2, "f16")
    all_ids = np.arange(N, dtype=np.int32)
    up = orc.select_gemm(x, W1, all_ids, "f16", relu=True)
    got = orc.select_gemm_down(up.astype(np.float32), W2, all_ids, "f16")
    np.testing.assert_allclose(got, dense, rtol=1e-12, atol=1e-13)
    # and over a subset S it is the dense block with the other neurons' activations zeroed
    S = np.array([1, 4, 5, 11, 20], np.int32)
    masked = np.zeros_like(hidden)
    masked[:, S] = hidden[:, S]
    want = masked.astype(np.float32).astype(np.float16).astype(np.float64) @ as_f64(W2, "f16")
    got_s = orc.select_gemm_down(orc.select_gemm(x, W1, S, "f16", relu=True).astype(np.float32), W2, S, "f16")
    np.testing.assert_allclose(got_s, want, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- threads
def test_result_does_not_depend_on_thread_count():
    q, K, V, n = random_case(4, 4, 4, 50, 16, "f16")
    idx = np.stack([RNG.permutation(4)[:2] for _ in range(4)]).astype(np.int32)
    before = orc.num_threads()
    orc.set_num_threads(1)
    a = orc.sha_decode(q, K, V, n, idx, 2, "f16")
    orc.set_num_threads(max(before, 4))
    b = orc.sha_decode(q, K, V, n, idx, 2, "f16")
    orc.set_num_threads(before)
    assert np.array_equal(a, b)
