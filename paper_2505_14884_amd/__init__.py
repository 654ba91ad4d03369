"""MI355X-native Selective Head Attention decode path (router + top-k + selective decode attention).

The compute runs in hand-written HIP kernels behind a C-ABI library (``include/polar.h``);
``binding`` marshals torch device tensors into it and ``workloads`` generates seeded inputs.
"""
from . import binding, workloads  # noqa: F401
from .binding import (PolarError, alloc_router_workspace, alloc_select_gemm_workspace, alloc_workspace,  # noqa: F401
                      get_option, head_labels, head_norm_topk, neuron_union, neuron_union_workspace_bytes, options,
                      probe_gather_read, probe_read, router_topk, router_workspace_bytes, select_gemm,
                      select_gemm_down, select_gemm_down_workspace_bytes, select_gemm_workspace_bytes,
                      set_option, sha_chunk_rows, sha_decode, sha_decode_static, sha_launches, sha_merge, sha_partial,
                      sha_workspace_bytes, sparse_mlp, sparse_mlp_workspace_bytes)

__all__ = ["binding", "workloads", "PolarError", "alloc_router_workspace", "alloc_select_gemm_workspace",
           "alloc_workspace", "get_option", "head_labels", "head_norm_topk", "neuron_union", "neuron_union_workspace_bytes",
           "options", "probe_gather_read", "probe_read", "router_topk", "router_workspace_bytes", "select_gemm",
           "select_gemm_down", "select_gemm_down_workspace_bytes", "select_gemm_workspace_bytes", "set_option",
           "sha_chunk_rows", "sha_decode", "sha_decode_static", "sha_launches", "sha_merge", "sha_partial", "sha_workspace_bytes",
           "sparse_mlp", "sparse_mlp_workspace_bytes"]
