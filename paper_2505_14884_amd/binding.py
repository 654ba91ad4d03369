"""Thin ctypes binding of ``libpolar.so`` (see ``include/polar.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch tensors are used as handles to device memory, and the current
torch stream is the stream the kernels are enqueued on.  There is no CPU or
PyTorch fallback: if the library cannot be loaded, or a tensor is not on the
GPU, the call raises.
"""
from __future__ import annotations

import contextlib
import ctypes
import os
from typing import Optional, Tuple

import torch

from .build import LIB_PATH, PROBE_LIB_PATH, build_library, source_hash

F16, BF16 = 0, 1
KV_LAYOUT = {"bhsd": 0, "bshd": 1}   # [B,Hkv,S,d] (default) / [B,S,Hkv,d]
_STATUS = {0: "POLAR_OK", -1: "POLAR_EINVAL", -2: "POLAR_EUNSUPPORTED", -3: "POLAR_EWORKSPACE",
           -4: "POLAR_EHIP"}
EXPORTS = ("polar_router_topk", "polar_router_workspace_bytes", "polar_sha_workspace_bytes", "polar_sha_decode",
           "polar_sha_decode_static", "polar_sha_decode_layout", "polar_sha_partial", "polar_sha_partial_layout", "polar_sha_merge",
           "polar_sha_chunk_rows", "polar_sha_launches", "polar_head_norm_topk", "polar_head_labels", "polar_select_gemm",
           "polar_select_gemm_ws", "polar_select_gemm_workspace_bytes", "polar_select_gemm_down",
           "polar_select_gemm_down_workspace_bytes", "polar_sparse_mlp", "polar_sparse_mlp_workspace_bytes",
           "polar_neuron_union", "polar_neuron_union_ws", "polar_neuron_union_workspace_bytes",
           "polar_set_option", "polar_get_option", "polar_strerror", "polar_last_hip_error", "polar_version",
           "polar_source_hash")
PROBE_EXPORTS = ("polar_probe_read", "polar_probe_gather_read", "polar_probe_last_hip_error")
# polar_option in include/polar.h
OPTIONS = {"sha_chunk_rows": 0, "sha_form": 1, "sha_grouped_kernel": 2, "router_path": 3, "router_phase1": 4,
           "gemm_form": 5, "gemm_workgroups": 6, "union_form": 7}

_lib: Optional[ctypes.CDLL] = None
_probe_lib: Optional[ctypes.CDLL] = None


class PolarError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        text = lib().polar_strerror(status).decode()
        extra = ""
        if status == -4:
            extra = " (hipError %d)" % lib().polar_last_hip_error()
        super().__init__("%s: %s: %s%s" % (where, _STATUS.get(status, str(status)), text, extra))


def _load_checked() -> ctypes.CDLL:
    """The in-tree library, built from exactly the sources in the tree: it is compiled when no
    built copy exists, and compiled again when the copy's baked-in source hash differs from the
    hash of the sources and headers now on disk (an edit since the last build).  A library named
    by POLAR_LIBRARY (a tuning variant) is loaded as it is."""
    path = os.environ.get("POLAR_LIBRARY")
    if path:
        return ctypes.CDLL(path)
    if not (os.path.exists(LIB_PATH) and os.path.exists(PROBE_LIB_PATH)):
        build_library()
    L = ctypes.CDLL(LIB_PATH)
    want = source_hash()
    try:
        L.polar_source_hash.restype = ctypes.c_char_p
        have = L.polar_source_hash().decode()
    except AttributeError:
        have = "(a build without a source hash)"
    if have != want:
        raise RuntimeError(
            "%s was built from other sources than the ones in the tree (library %s, tree %s): run "
            "`python -c 'import __graft_entry__ as g; g.build()'` (a stale binary is never used "
            "silently, and a loaded one cannot be replaced in this process)" % (LIB_PATH, have, want))
    return L


def lib() -> ctypes.CDLL:
    """Load the shared library (see _load_checked) and declare its signatures."""
    global _lib
    if _lib is None:
        L = _load_checked()
        i, vp, f, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_size_t
        L.polar_router_topk.argtypes = [vp, vp, i, i, i, i, i, vp, vp, vp, sz, vp]
        L.polar_router_topk.restype = i
        L.polar_router_workspace_bytes.argtypes = [i, i, i]
        L.polar_router_workspace_bytes.restype = sz
        L.polar_sha_workspace_bytes.argtypes = [i] * 6
        L.polar_sha_workspace_bytes.restype = sz
        L.polar_sha_chunk_rows.argtypes = [i] * 6
        L.polar_sha_chunk_rows.restype = i
        L.polar_sha_launches.argtypes = [i] * 6
        L.polar_sha_launches.restype = i
        L.polar_sha_decode.argtypes = [vp] * 6 + [i] * 7 + [f, vp, sz, vp]
        L.polar_sha_decode.restype = i
        L.polar_sha_decode_static.argtypes = [vp] * 6 + [i] * 7 + [f, vp]
        L.polar_sha_decode_static.restype = i
        L.polar_sha_partial.argtypes = [vp] * 5 + [i] * 7 + [f, vp, sz, vp]
        L.polar_sha_partial.restype = i
        L.polar_sha_decode_layout.argtypes = [vp] * 6 + [i] * 8 + [f, vp, sz, vp]
        L.polar_sha_decode_layout.restype = i
        L.polar_sha_partial_layout.argtypes = [vp] * 5 + [i] * 8 + [f, vp, sz, vp]
        L.polar_sha_partial_layout.restype = i
        L.polar_sha_merge.argtypes = [vp] * 3 + [i] * 6 + [vp, sz, vp]
        L.polar_sha_merge.restype = i
        L.polar_head_norm_topk.argtypes = [vp, i, i, i, i, i, vp, vp, vp]
        L.polar_head_norm_topk.restype = i
        L.polar_head_labels.argtypes = [vp] * 7 + [i] * 8 + [f, vp, sz, vp]
        L.polar_head_labels.restype = i
        L.polar_select_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
        L.polar_select_gemm.restype = i
        L.polar_select_gemm_ws.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, vp, ctypes.c_size_t, vp]
        L.polar_select_gemm_ws.restype = i
        L.polar_select_gemm_workspace_bytes.argtypes = [i]
        L.polar_select_gemm_workspace_bytes.restype = sz
        L.polar_select_gemm_down.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp, ctypes.c_size_t, vp]
        L.polar_select_gemm_down.restype = i
        L.polar_select_gemm_down_workspace_bytes.argtypes = [i, i, i]
        L.polar_select_gemm_down_workspace_bytes.restype = sz
        L.polar_sparse_mlp.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp, ctypes.c_size_t, vp]
        L.polar_sparse_mlp.restype = i
        L.polar_sparse_mlp_workspace_bytes.argtypes = [i, i, i]
        L.polar_sparse_mlp_workspace_bytes.restype = sz
        L.polar_neuron_union.argtypes = [vp, i, i, i, i, vp, vp, vp]
        L.polar_neuron_union.restype = i
        L.polar_neuron_union_ws.argtypes = [vp, i, i, i, i, vp, vp, vp, ctypes.c_size_t, vp]
        L.polar_neuron_union_ws.restype = i
        L.polar_neuron_union_workspace_bytes.argtypes = [i, i, i]
        L.polar_neuron_union_workspace_bytes.restype = sz
        L.polar_set_option.argtypes = [i, i]
        L.polar_set_option.restype = i
        L.polar_get_option.argtypes = [i, ctypes.POINTER(ctypes.c_int)]
        L.polar_get_option.restype = i
        L.polar_strerror.argtypes = [i]
        L.polar_strerror.restype = ctypes.c_char_p
        L.polar_last_hip_error.restype = i
        L.polar_version.restype = i
        L.polar_source_hash.restype = ctypes.c_char_p
        _lib = L
    return _lib


def probe_lib() -> ctypes.CDLL:
    """The read yardsticks' own library (include/polar_probe.h); built with the product library."""
    global _probe_lib
    if _probe_lib is None:
        lib()                                            # builds both when needed, checks the source hash
        P = ctypes.CDLL(os.environ.get("POLAR_PROBE_LIBRARY", PROBE_LIB_PATH))
        i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        P.polar_probe_read.argtypes = [vp, sz, sz, i, vp, vp]
        P.polar_probe_read.restype = i
        P.polar_probe_gather_read.argtypes = [vp, vp, i, i, i, i, i, i, vp, vp]
        P.polar_probe_gather_read.restype = i
        P.polar_probe_last_hip_error.restype = i
        _probe_lib = P
    return _probe_lib


def set_option(name: str, value: int) -> None:
    """Set a process-wide option of the library (see polar_option in include/polar.h); 0 = automatic."""
    _check(lib().polar_set_option(OPTIONS[name], int(value)), "polar_set_option(%s, %d)" % (name, value))


def get_option(name: str) -> int:
    v = ctypes.c_int(0)
    _check(lib().polar_get_option(OPTIONS[name], ctypes.byref(v)), "polar_get_option(%s)" % name)
    return int(v.value)


@contextlib.contextmanager
def options(**values):
    """Pin options for the duration of a block (tests and sweeps): options(sha_form=2, router_path=2).
    None leaves an option as it is."""
    saved = {}
    try:
        for name, value in values.items():
            if value is not None:
                saved[name] = get_option(name)
                set_option(name, value)
        yield
    finally:
        for name, old in saved.items():
            set_option(name, old)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("expected a float16 or bfloat16 tensor, got %s" % t.dtype)


def _dev(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU; this path has no CPU fallback" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise PolarError(rc, where)


def router_workspace_bytes(B: int, D: int, H: int) -> int:
    return int(lib().polar_router_workspace_bytes(B, D, H))


def alloc_router_workspace(B: int, D: int, H: int, device) -> torch.Tensor:
    nbytes = router_workspace_bytes(B, D, H)
    if nbytes == 0:
        raise PolarError(-2, "polar_router_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def router_topk(hidden: torch.Tensor, Wr: torch.Tensor, k: int,
                head_idx: Optional[torch.Tensor] = None,
                logits_out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """hidden [B,D], Wr [D,H] (fp16/bf16, GPU) -> head_idx int32 [B,k].
    With a workspace (alloc_router_workspace) the library uses its split-D kernels."""
    B, D = hidden.shape
    D2, H = Wr.shape
    if D != D2 or hidden.dtype != Wr.dtype:
        raise ValueError("hidden [B,D] and Wr [D,H] must agree in D and dtype")
    if head_idx is None:
        head_idx = torch.empty((B, max(k, 0)), dtype=torch.int32, device=hidden.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().polar_router_topk(_dev(hidden, "hidden"), _dev(Wr, "Wr"), B, D, H, k,
                                 _dtype_code(hidden), _dev(head_idx, "head_idx", torch.int32),
                                 _dev(logits_out, "logits_out", torch.float32),
                                 _dev(workspace, "workspace"), ws_bytes, _stream())
    _check(rc, "polar_router_topk")
    return head_idx


def sha_workspace_bytes(B: int, Hq: int, Hkv: int, S: int, d: int, k: int) -> int:
    return int(lib().polar_sha_workspace_bytes(B, Hq, Hkv, S, d, k))


def sha_chunk_rows(B: int, Hq: int, Hkv: int, S: int, d: int, k: int) -> int:
    return int(lib().polar_sha_chunk_rows(B, Hq, Hkv, S, d, k))


def sha_launches(B: int, Hq: int, Hkv: int, S: int, d: int, k: int) -> int:
    """Kernels sha_decode launches for these sizes (1: streaming kernel alone, 2: + merge)."""
    return int(lib().polar_sha_launches(B, Hq, Hkv, S, d, k))


def alloc_workspace(B: int, Hq: int, Hkv: int, S: int, d: int, k: int, device) -> torch.Tensor:
    nbytes = sha_workspace_bytes(B, Hq, Hkv, S, d, k)
    if nbytes == 0:
        # sizes the library rejects: ask the size check itself for the status to report
        rc = lib().polar_sha_merge(None, None, None, B, Hq, Hkv, S, d, k, None, 0, None)
        raise PolarError(rc if rc != 0 else -1, "polar_sha_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _sha_shapes(q, K, V, seqlens, head_idx, k, kv_layout="bhsd"):
    if kv_layout not in KV_LAYOUT:
        raise ValueError("kv_layout must be 'bhsd' or 'bshd'")
    B, Hq, d = q.shape
    if kv_layout == "bhsd":
        B2, Hkv, S, d2 = K.shape
    else:
        B2, S, Hkv, d2 = K.shape
    if (B, d) != (B2, d2) or V.shape != K.shape or q.dtype != K.dtype or V.dtype != K.dtype:
        raise ValueError("q [B,Hq,d] and K/V ([B,Hkv,S,d] or [B,S,Hkv,d]) must agree in B, d and dtype")
    if tuple(seqlens.shape) != (B,):
        raise ValueError("seqlens must be [B]")
    if head_idx is not None and tuple(head_idx.shape) != (B, k):
        raise ValueError("head_idx must be [B,k]")
    return B, Hq, Hkv, S, d


def sha_decode(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, seqlens: torch.Tensor,
               head_idx: Optional[torch.Tensor], k: int, out: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, scale: float = 0.0,
               kv_layout: str = "bhsd") -> torch.Tensor:
    """Selective head attention, decode step -> out float32 [B,Hq,d] (unselected heads zero).
    K/V are [B,Hkv,S,d] (kv_layout "bhsd") or [B,S,Hkv,d] ("bshd")."""
    B, Hq, Hkv, S, d = _sha_shapes(q, K, V, seqlens, head_idx, k, kv_layout)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(B, Hq, Hkv, S, d, k, q.device)
    ptrs = (_dev(q, "q"), _dev(K, "K"), _dev(V, "V"), _dev(seqlens, "seqlens", torch.int32),
            _dev(head_idx, "head_idx", torch.int32), _dev(out, "out", torch.float32))
    tail = (float(scale), _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream())
    if kv_layout == "bhsd":       # the main-text layout goes through the plain entry point
        rc = lib().polar_sha_decode(*ptrs, B, Hq, Hkv, S, d, k, _dtype_code(q), *tail)
        _check(rc, "polar_sha_decode")
    else:
        rc = lib().polar_sha_decode_layout(*ptrs, B, Hq, Hkv, S, d, k, _dtype_code(q), KV_LAYOUT[kv_layout], *tail)
        _check(rc, "polar_sha_decode_layout")
    return out


STATIC_SCRATCH_BYTES = 32 << 20      # POLAR_STATIC_SCRATCH_BYTES in include/polar.h


def sha_decode_static(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, seqlens: torch.Tensor,
                      head_idx: Optional[torch.Tensor], k: int, out: torch.Tensor, scale: float = 0.0) -> torch.Tensor:
    """sha_decode through the entry point that allocates nothing: the caller passes `out`, the
    split-KV scratch is the library's own static device array (sizes beyond it raise)."""
    B, Hq, Hkv, S, d = _sha_shapes(q, K, V, seqlens, head_idx, k)
    rc = lib().polar_sha_decode_static(_dev(q, "q"), _dev(K, "K"), _dev(V, "V"), _dev(seqlens, "seqlens", torch.int32),
                                       _dev(head_idx, "head_idx", torch.int32), _dev(out, "out", torch.float32),
                                       B, Hq, Hkv, S, d, k, _dtype_code(q), float(scale), _stream())
    _check(rc, "polar_sha_decode_static")
    return out


def sha_partial(q, K, V, seqlens, head_idx, k: int, workspace: torch.Tensor,
                scale: float = 0.0, kv_layout: str = "bhsd") -> None:
    """The KV-streaming phase of sha_decode alone (leaves per-chunk partials in workspace)."""
    B, Hq, Hkv, S, d = _sha_shapes(q, K, V, seqlens, head_idx, k, kv_layout)
    ptrs = (_dev(q, "q"), _dev(K, "K"), _dev(V, "V"), _dev(seqlens, "seqlens", torch.int32),
            _dev(head_idx, "head_idx", torch.int32))
    tail = (float(scale), _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream())
    if kv_layout == "bhsd":
        rc = lib().polar_sha_partial(*ptrs, B, Hq, Hkv, S, d, k, _dtype_code(q), *tail)
        _check(rc, "polar_sha_partial")
    else:
        rc = lib().polar_sha_partial_layout(*ptrs, B, Hq, Hkv, S, d, k, _dtype_code(q), KV_LAYOUT[kv_layout], *tail)
        _check(rc, "polar_sha_partial_layout")


def sha_merge(seqlens, head_idx, out: torch.Tensor, Hkv: int, S: int, k: int,
              workspace: torch.Tensor) -> torch.Tensor:
    """The merge / zero-fill phase of sha_decode alone."""
    B, Hq, d = out.shape
    rc = lib().polar_sha_merge(_dev(seqlens, "seqlens", torch.int32),
                               _dev(head_idx, "head_idx", torch.int32),
                               _dev(out, "out", torch.float32), B, Hq, Hkv, S, d, k,
                               _dev(workspace, "workspace"),
                               workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "polar_sha_merge")
    return out


def probe_read(src: torch.Tensor, slab_bytes: int, nontemporal: bool = True,
               sink: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Streaming-read yardstick over the whole slabs of `src` (see polar_probe_read)."""
    nbytes = src.numel() * src.element_size()
    slabs = nbytes // slab_bytes
    if sink is None:
        sink = torch.empty(max(slabs, 1), dtype=torch.int32, device=src.device)
    rc = probe_lib().polar_probe_read(_dev(src, "src"), slabs, slab_bytes, 1 if nontemporal else 0,
                                      _dev(sink, "sink"), _stream())
    _check(rc, "polar_probe_read")
    return sink


def probe_gather_read(W: torch.Tensor, idx: torch.Tensor, slices: int = 3, depth: int = 1,
                      nontemporal: bool = True, sink: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Read yardstick for gathered weight rows (see polar_probe_gather_read)."""
    N, K = W.shape
    n_idx = idx.shape[0]
    if sink is None:
        sink = torch.empty(max(2 * ((n_idx + 63) // 64) * slices, 1), dtype=torch.int32, device=W.device)
    rc = probe_lib().polar_probe_gather_read(_dev(W, "W"), _dev(idx, "idx", torch.int32), n_idx, N, K, slices,
                                             depth, 1 if nontemporal else 0, _dev(sink, "sink"), _stream())
    _check(rc, "polar_probe_gather_read")
    return sink


def head_norm_topk(attn_out: torch.Tensor, Hkv: int, k: int,
                   head_idx: Optional[torch.Tensor] = None,
                   norms_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Dense attention output float32 [B,Hq,d] -> int32 [B,k]: the k KV groups with the largest
    output L2 norm per request, best first (the router's training labels)."""
    B, Hq, d = attn_out.shape
    if head_idx is None:
        head_idx = torch.empty((B, max(k, 0)), dtype=torch.int32, device=attn_out.device)
    rc = lib().polar_head_norm_topk(_dev(attn_out, "attn_out", torch.float32), B, Hq, Hkv, d, k,
                                    _dev(head_idx, "head_idx", torch.int32),
                                    _dev(norms_out, "norms_out", torch.float32), _stream())
    _check(rc, "polar_head_norm_topk")
    return head_idx


def head_labels(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, seqlens: torch.Tensor, k: int,
                labels: Optional[torch.Tensor] = None, norms_out: Optional[torch.Tensor] = None,
                attn_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                scale: float = 0.0, kv_layout: str = "bhsd") -> torch.Tensor:
    """Head-importance labels straight from the caches: dense decode attention with the norm and the
    ranking as the merge kernel's epilogue -> int32 [B,k] (the k KV groups with the largest output
    norm per request, best first).  attn_out (float32 [B,Hq,d]) receives the dense output if given."""
    B, Hq, Hkv, S, d = _sha_shapes(q, K, V, seqlens, None, 0, kv_layout)
    if labels is None:
        labels = torch.empty((B, max(k, 0)), dtype=torch.int32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(B, Hq, Hkv, S, d, Hkv, q.device)
    rc = lib().polar_head_labels(_dev(q, "q"), _dev(K, "K"), _dev(V, "V"), _dev(seqlens, "seqlens", torch.int32),
                                 _dev(labels, "labels", torch.int32), _dev(norms_out, "norms_out", torch.float32),
                                 _dev(attn_out, "attn_out", torch.float32), B, Hq, Hkv, S, d, k, _dtype_code(q),
                                 KV_LAYOUT[kv_layout], float(scale), _dev(workspace, "workspace"),
                                 workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "polar_head_labels")
    return labels


def select_gemm_workspace_bytes(M: int) -> int:
    """Workspace size at which polar_select_gemm_ws launches as wide as it wants."""
    return int(lib().polar_select_gemm_workspace_bytes(M))


def alloc_select_gemm_workspace(M: int, device) -> Optional[torch.Tensor]:
    n = select_gemm_workspace_bytes(M)
    return torch.empty(n, dtype=torch.uint8, device=device) if n else None


def select_gemm(A: torch.Tensor, W: torch.Tensor, idx: torch.Tensor,
                count: Optional[torch.Tensor] = None, relu: bool = True,
                out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """act(A @ W[idx].T): A [M,K], W [N,K] (fp16/bf16, one row per neuron), idx int32 [cap],
    count int32 [1] on the device (None: all of idx is live) -> float32 [M,cap].  With a
    workspace (alloc_select_gemm_workspace) the call goes to polar_select_gemm_ws."""
    M, K = A.shape
    N, K2 = W.shape
    if K != K2 or A.dtype != W.dtype:
        raise ValueError("A [M,K] and W [N,K] must agree in K and dtype")
    cap = idx.shape[0]
    if out is None:
        out = torch.zeros((M, cap), dtype=torch.float32, device=A.device)
    if workspace is not None:
        rc = lib().polar_select_gemm_ws(_dev(A, "A"), _dev(W, "W"), _dev(idx, "idx", torch.int32),
                                        _dev(count, "count", torch.int32), _dev(out, "out", torch.float32),
                                        M, K, N, cap, _dtype_code(A), 1 if relu else 0,
                                        _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream())
        _check(rc, "polar_select_gemm_ws")
        return out
    rc = lib().polar_select_gemm(_dev(A, "A"), _dev(W, "W"), _dev(idx, "idx", torch.int32),
                                 _dev(count, "count", torch.int32), _dev(out, "out", torch.float32),
                                 M, K, N, cap, _dtype_code(A), 1 if relu else 0, _stream())
    _check(rc, "polar_select_gemm")
    return out


def select_gemm_down_workspace_bytes(M: int, Kout: int, cap: int) -> int:
    """Workspace size polar_select_gemm_down requires."""
    return int(lib().polar_select_gemm_down_workspace_bytes(M, Kout, cap))


def select_gemm_down(H: torch.Tensor, W2: torch.Tensor, idx: torch.Tensor,
                     count: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """h16(H) @ W2[idx]: H float32 [M,cap] (select_gemm's output), W2 [N,Kout] fp16/bf16 (one row per
    neuron), idx int32 [cap], count int32 [1] on the device (None: all live) -> float32 [M,Kout].
    A workspace is allocated when none is given."""
    M, cap = H.shape
    N, Kout = W2.shape
    if idx.shape[0] != cap:
        raise ValueError("idx must have one entry per column of H")
    if out is None:
        out = torch.empty((M, Kout), dtype=torch.float32, device=W2.device)
    if workspace is None:
        workspace = torch.empty(max(select_gemm_down_workspace_bytes(M, Kout, cap), 16), dtype=torch.uint8,
                                device=W2.device)
    rc = lib().polar_select_gemm_down(_dev(H, "H", torch.float32), _dev(W2, "W2"), _dev(idx, "idx", torch.int32),
                                      _dev(count, "count", torch.int32), _dev(out, "out", torch.float32),
                                      M, Kout, N, cap, _dtype_code(W2), _dev(workspace, "workspace"),
                                      workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "polar_select_gemm_down")
    return out


def sparse_mlp_workspace_bytes(M: int, D: int, cap: int) -> int:
    """Workspace size polar_sparse_mlp requires."""
    return int(lib().polar_sparse_mlp_workspace_bytes(M, D, cap))


def sparse_mlp(X: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor, idx: torch.Tensor,
               count: Optional[torch.Tensor] = None, relu: bool = True, out: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """h16(act(X @ W1[idx].T)) @ W2[idx] in one call: X [M,D], W1 and W2 [N,D] fp16/bf16 (one row per
    neuron), idx int32 [cap], count int32 [1] on the device (None: all live) -> float32 [M,D].
    A workspace is allocated when none is given."""
    M, D = X.shape
    N = W1.shape[0]
    if W1.shape != W2.shape or W1.shape[1] != D or W1.dtype != X.dtype or W2.dtype != X.dtype:
        raise ValueError("X [M,D], W1 [N,D] and W2 [N,D] must agree in D and dtype")
    cap = idx.shape[0]
    if out is None:
        out = torch.empty((M, D), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty(max(sparse_mlp_workspace_bytes(M, D, cap), 256), dtype=torch.uint8, device=X.device)
    rc = lib().polar_sparse_mlp(_dev(X, "X"), _dev(W1, "W1"), _dev(W2, "W2"), _dev(idx, "idx", torch.int32),
                                _dev(count, "count", torch.int32), _dev(out, "out", torch.float32),
                                M, D, N, cap, _dtype_code(X), int(bool(relu)), _dev(workspace, "workspace"),
                                workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "polar_sparse_mlp")
    return out


def neuron_union_workspace_bytes(B: int, kn: int, N: int) -> int:
    """Workspace size polar_neuron_union_ws wants for this input (0: too small to split)."""
    return int(lib().polar_neuron_union_workspace_bytes(B, kn, N))


def neuron_union(topk: torch.Tensor, N: int, cap: Optional[int] = None,
                 workspace: Optional[torch.Tensor] = None,
                 out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None):
    """Per-request neuron ids int32 [B,kn] -> (idx int32 [cap] ascending distinct ids, count int32 [1]).
    With a workspace (neuron_union_workspace_bytes) the call goes to polar_neuron_union_ws; `out`
    = (idx, count) reuses existing outputs."""
    B, kn = topk.shape
    if out is not None:
        idx, count = out
        cap = idx.shape[0]
    else:
        cap = min(N, B * kn) if cap is None else cap
        idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=topk.device)[:cap]
        count = torch.zeros(1, dtype=torch.int32, device=topk.device)
    if workspace is not None:
        rc = lib().polar_neuron_union_ws(_dev(topk, "topk", torch.int32), B, kn, N, cap,
                                         _dev(idx, "idx", torch.int32), _dev(count, "count", torch.int32),
                                         _dev(workspace, "workspace"),
                                         workspace.numel() * workspace.element_size(), _stream())
        _check(rc, "polar_neuron_union_ws")
        return idx, count
    rc = lib().polar_neuron_union(_dev(topk, "topk", torch.int32), B, kn, N, cap,
                                  _dev(idx, "idx", torch.int32), _dev(count, "count", torch.int32),
                                  _stream())
    _check(rc, "polar_neuron_union")
    return idx, count
