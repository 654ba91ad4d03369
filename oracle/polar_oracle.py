"""ctypes binding of the fp64 CPU oracle (``polar_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT: only ``tests/``, the smoke check and the
bench's ``cpu_baseline`` leg import this.  It knows nothing of the HIP library
and takes numpy arrays of raw 16-bit patterns (uint16) plus a dtype name.

The shared object is compiled from the C file beside it with gcc; it is rebuilt
here when missing or older than its source (a one-second gcc run).  The
environment variable POLAR_ORACLE_LIBRARY names another build of the same
source to load instead (the sanitizer test uses it).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "polar_oracle.c")
_SO = os.path.join(_HERE, "libpolar_oracle.so")
_DT = {"f16": 0, "bf16": 1}
_lib = None


def build(force: bool = False, out_path: str = _SO, extra_flags=("-O2",)) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp by default).  Returns the path of the shared object."""
    stale = (not os.path.exists(out_path)) or os.path.getmtime(out_path) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = out_path + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *extra_flags, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                        "-Wextra", "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, out_path)
    return out_path


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(os.environ.get("POLAR_ORACLE_LIBRARY") or build())
        c_int, c_long, c_dbl, vp = ctypes.c_int, ctypes.c_long, ctypes.c_double, ctypes.c_void_p
        L.oracle_num_threads.restype = c_int
        L.oracle_set_num_threads.argtypes = [c_int]
        L.oracle_widen16.argtypes = [vp, c_long, c_int, vp]
        L.oracle_router_logits.argtypes = [vp, vp, c_int, c_int, c_int, c_int, vp]
        L.oracle_topk.argtypes = [vp, c_int, c_int, c_int, vp]
        L.oracle_sha_decode.argtypes = [vp, vp, vp, vp, vp, vp] + [c_int] * 7 + [c_dbl]
        L.oracle_head_scores.argtypes = [vp, c_int, c_int, c_int, c_int, vp, vp]
        L.oracle_neuron_union.argtypes = [vp, c_int, c_int, c_int, vp, vp]
        L.oracle_select_gemm.argtypes = [vp, vp, vp] + [c_int] * 6 + [vp]
        L.oracle_select_gemm_down.argtypes = [vp, vp, vp] + [c_int] * 5 + [vp]
        L.oracle_alg1_tiled.argtypes = [vp, vp, vp, c_int, c_int, c_int, c_dbl, vp]
        _lib = L
    return _lib


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("expected raw 16-bit patterns as uint16, got %s" % a.dtype)
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(int(n))


def widen16(bits, dtype: str) -> np.ndarray:
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    rc = lib().oracle_widen16(_ptr(bits), bits.size, _DT[dtype], _ptr(out))
    assert rc == 0, rc
    return out


def router_logits(hidden_bits, Wr_bits, dtype: str) -> np.ndarray:
    """hidden [B,D], Wr [D,H] as uint16 patterns -> float64 logits [B,H]."""
    hidden_bits, Wr_bits = _u16(hidden_bits), _u16(Wr_bits)
    B, D = hidden_bits.shape
    D2, H = Wr_bits.shape
    assert D == D2
    out = np.empty((B, H), dtype=np.float64)
    rc = lib().oracle_router_logits(_ptr(hidden_bits), _ptr(Wr_bits), B, D, H, _DT[dtype], _ptr(out))
    assert rc == 0, rc
    return out


def topk(logits, k: int) -> np.ndarray:
    """float64 logits [B,H] -> int32 [B,k], descending logit, ties to the lower id."""
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    B, H = logits.shape
    out = np.empty((B, k), dtype=np.int32)
    rc = lib().oracle_topk(_ptr(logits), B, H, k, _ptr(out))
    assert rc == 0, rc
    return out


def router_topk(hidden_bits, Wr_bits, k: int, dtype: str) -> np.ndarray:
    return topk(router_logits(hidden_bits, Wr_bits, dtype), k)


def sha_decode(q_bits, K_bits, V_bits, seqlens, head_idx, k: int, dtype: str,
               scale: float = 0.0) -> np.ndarray:
    """q [B,Hq,d], K/V [B,Hkv,S,d] uint16 patterns, seqlens [B], head_idx [B,k] or None
    (dense, k == Hkv) -> float64 out [B,Hq,d]; unselected heads are +0.0."""
    q_bits, K_bits, V_bits = _u16(q_bits), _u16(K_bits), _u16(V_bits)
    B, Hq, d = q_bits.shape
    B2, Hkv, S, d2 = K_bits.shape
    assert (B, d) == (B2, d2) and V_bits.shape == K_bits.shape
    seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
    assert seqlens.shape == (B,)
    if head_idx is not None:
        head_idx = np.ascontiguousarray(head_idx, dtype=np.int32)
        assert head_idx.shape == (B, k)
    out = np.empty((B, Hq, d), dtype=np.float64)
    rc = lib().oracle_sha_decode(_ptr(q_bits), _ptr(K_bits), _ptr(V_bits), _ptr(seqlens),
                                 _ptr(head_idx), _ptr(out), B, Hq, Hkv, S, d, k, _DT[dtype],
                                 float(scale))
    assert rc == 0, rc
    return out


def alg1_tiled(q, K, V, Bc: int, scale: float) -> np.ndarray:
    """Algorithm 1's tile-by-tile recurrence for one head: q [d], K/V [n,d] float64 -> [d]."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    n, d = K.shape
    out = np.empty(d, dtype=np.float64)
    rc = lib().oracle_alg1_tiled(_ptr(q), _ptr(K), _ptr(V), n, d, int(Bc), float(scale), _ptr(out))
    assert rc == 0, rc
    return out


def head_scores(attn, Hkv: int):
    """Dense attention output float64 [B,Hq,d] -> (sum of squares [B,Hkv], L2 norms [B,Hkv])."""
    attn = np.ascontiguousarray(attn, dtype=np.float64)
    B, Hq, d = attn.shape
    score = np.empty((B, Hkv), dtype=np.float64)
    norms = np.empty((B, Hkv), dtype=np.float64)
    rc = lib().oracle_head_scores(_ptr(attn), B, Hq, Hkv, d, _ptr(score), _ptr(norms))
    assert rc == 0, rc
    return score, norms


def head_importance_labels(q_bits, K_bits, V_bits, seqlens, k: int, dtype: str):
    """The router's training labels: dense attention, per-group output norm, top-k.
    Returns (labels int32 [B,k], scores float64 [B,Hkv])."""
    Hkv = K_bits.shape[1]
    attn = sha_decode(q_bits, K_bits, V_bits, seqlens, None, Hkv, dtype)
    score, _ = head_scores(attn, Hkv)
    return topk(score, k), score


def neuron_union(topk_idx, N: int) -> np.ndarray:
    """Per-request neuron ids int32 [B,kn] -> ascending distinct ids in [0,N) (int32 [count])."""
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    B, kn = topk_idx.shape
    out = np.empty(max(1, min(N, B * kn)), dtype=np.int32)
    count = np.zeros(1, dtype=np.int32)
    rc = lib().oracle_neuron_union(_ptr(topk_idx), B, kn, N, _ptr(out), _ptr(count))
    assert rc == 0, rc
    return out[: int(count[0])].copy()


def select_gemm(A_bits, W_bits, idx, dtype: str, relu: bool = True) -> np.ndarray:
    """A [M,K], W [N,K] uint16 patterns, idx int32 [n_sel] -> float64 [M,n_sel]:
    act(A @ W[idx].T); ids outside [0,N) give zero columns."""
    A_bits, W_bits = _u16(A_bits), _u16(W_bits)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    M, K = A_bits.shape
    N, K2 = W_bits.shape
    assert K == K2 and idx.ndim == 1
    C = np.empty((M, idx.shape[0]), dtype=np.float64)
    rc = lib().oracle_select_gemm(_ptr(A_bits), _ptr(W_bits), _ptr(idx), M, K, N, idx.shape[0],
                                  _DT[dtype], 1 if relu else 0, _ptr(C))
    assert rc == 0, rc
    return C


def select_gemm_down(H, W2_bits, idx, dtype: str) -> np.ndarray:
    """H float32 [M,n_sel], W2 [N,Kout] uint16 patterns, idx int32 [n_sel] -> float64 [M,Kout]:
    sum_j h16(H[:,j]) * W2[idx[j],:] with H rounded to the storage type; ids outside [0,N) are skipped."""
    H = np.ascontiguousarray(H, dtype=np.float32)
    W2_bits = _u16(W2_bits)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    M, n_sel = H.shape
    N, Kout = W2_bits.shape
    assert idx.shape == (n_sel,)
    Y = np.empty((M, Kout), dtype=np.float64)
    rc = lib().oracle_select_gemm_down(_ptr(H), _ptr(W2_bits), _ptr(idx), M, Kout, N, n_sel, _DT[dtype], _ptr(Y))
    assert rc == 0, rc
    return Y
