#!/usr/bin/env python3
"""Benchmark of the Selective Head Attention decode path on one MI355X.

A step is one pass of the whole hot path over one batch: router GEMV + per-request top-k,
then selective decode attention (KV streaming + split merge + zero fill) for the heads the
router just chose.  Inputs are seeded synthetic tensors already resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line.  `value` is the effective KV bandwidth of the whole step: bytes of
K and V the selected heads oblige a kernel to read, divided by the wall time of a step
(router included).  The K timed steps are replayed from HIP graphs, as a decode loop would
run them (`config.launch` says how; --no-graph launches them one by one, and that time is
always reported beside it as `breakdown_us.eager_us_per_layer`).  `roofline` is for the dominant kernel alone (the KV-streaming kernel),
timed with events on the launch stream; its `traffic` is read from the hardware counters in
this very run: before it touches the GPU, the benchmark runs itself four times as a child
process under `rocprofv3 --pmc` (FETCH_SIZE and WRITE_SIZE of the streaming kernel, and of a
plain device copy of known size that scales them).  --no-traffic skips those passes (traffic is
then null), --traffic-from DIR reads passes made earlier, --traffic-dir DIR keeps the CSV files.
`cpu_baseline` is the fp64 oracle on the host cores over a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
DEFAULT_WORKLOAD = "C4_opt66b"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed time the GPU is kept busy with the same steps before warm-up and timing (clocks settle)")
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--k", type=int, default=0, help="override the number of selected units")
    ap.add_argument("--B", type=int, default=0, help="override the batch size")
    ap.add_argument("--Hq", type=int, default=0, help="override the number of query heads")
    ap.add_argument("--Hkv", type=int, default=0, help="override the number of KV heads")
    ap.add_argument("--S", type=int, default=0, help="override the KV-cache capacity (rows per request)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=0,
                    help="threads the oracle is timed with (0: all host cores)")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense (k = H) comparison run, so a kernel trace of this command "
                         "holds selective launches only")
    ap.add_argument("--cpu-sample", type=int, default=0,
                    help="requests the oracle is timed on (0: the whole batch, capped so that the "
                         "host copy of their K and V stays under 12 GB)")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the timing of the step replayed from a HIP graph")
    ap.add_argument("--no-traffic", action="store_true",
                    help="do not run the rocprofv3 counter passes (roofline.traffic is then null)")
    ap.add_argument("--traffic-from", default="",
                    help="directory of counter passes made earlier by this program (--traffic-dir): read "
                         "roofline.traffic from them instead of running the passes again")
    ap.add_argument("--traffic-dense-pass", action="store_true",
                    help="with the counter passes, also read FETCH_SIZE of the dense run of the same kernel (k = Hkv), "
                         "for the selective / dense traffic ratio")
    ap.add_argument("--traffic-dir", default="",
                    help="keep the counter passes' CSV files and logs in this directory (default: a "
                         "temporary one that is removed)")
    ap.add_argument("--kv-layout", choices=["bhsd", "bshd"], default="bhsd",
                    help="cache layout: [B,Hkv,S,d] (default) or the sequence-major [B,S,Hkv,d]")
    ap.add_argument("--mlp-workload", default="M2_opt66b_ffn",
                    help="workload of --phase select_gemm (see workloads.MLP_CONFIGS)")
    ap.add_argument("--density", type=float, default=0.0,
                    help="--phase select_gemm: override the target union density")
    ap.add_argument("--mlp-layers", type=int, default=3,
                    help="--phase select_gemm: copies of the weight matrices the launches rotate through, so that "
                         "no launch finds its rows in the 256 MB last-level cache left there by the one before "
                         "(a model streams another layer's weights every time)")
    ap.add_argument("--gemm-form", choices=["wide", "narrow"], default="wide",
                    help="--phase select_gemm: 'wide' passes a workspace (128-neuron tiles, evenly split "
                         "fixed-size launch + reduction), 'narrow' calls the 32-neuron one-launch kernel")
    ap.add_argument("--phase", choices=["all", "partial", "copy", "select_gemm", "select_gemm_only"],
                    default="all",
                    help="'partial' launches only the KV-streaming kernel (for counter runs); "
                         "'copy' runs a plain device copy of known size, the yardstick the "
                         "FETCH_SIZE / WRITE_SIZE counters are scaled by; 'select_gemm' benchmarks "
                         "the selective fused-gather GEMM (union index + GEMM) instead of the "
                         "attention path; 'select_gemm_only' launches just that GEMM (counter runs)")
    return ap.parse_args()


def workload_args(args):
    """The command-line arguments that select the workload, for the child runs of this program."""
    if args.phase in ("select_gemm", "select_gemm_only"):
        flags = (("--mlp-workload", args.mlp_workload), ("--B", args.B), ("--density", args.density),
                 ("--mlp-layers", args.mlp_layers), ("--gemm-form", args.gemm_form))
    else:
        flags = (("--workload", args.workload), ("--k", args.k), ("--B", args.B), ("--Hq", args.Hq), ("--Hkv", args.Hkv),
                 ("--S", args.S), ("--kv-layout", args.kv_layout if args.kv_layout != "bhsd" else ""))
    out = []
    for flag, value in flags:
        if value:
            out += [flag, str(value)]
    return out


def hbm_traffic(args, phase, kernels):
    """roofline.traffic for the kernels named: HBM bytes per launch from `rocprofv3 --pmc FETCH_SIZE`
    and `--pmc WRITE_SIZE` runs of this program's --phase <phase> (only those kernels launch), each
    scaled by the same counter's reading for a plain 4 GiB device copy (--phase copy).  Returns
    (dict or None, note).  Must run before this process touches the GPU."""
    from paper_2505_14884_amd import rocprof

    if args.traffic_from:
        with open(os.path.join(args.traffic_from, "commands.txt"), "a") as f:
            f.write("python3 bench.py %s\n" % " ".join(sys.argv[1:]))
        t = rocprof.traffic_from(args.traffic_from, kernels)
        return t, "read from %s" % args.traffic_from if t else "no usable counter passes in %s" % args.traffic_from
    if args.no_traffic:
        return None, "counter passes skipped (--no-traffic)"
    if not rocprof.rocprofv3():
        return None, "rocprofv3 not found"
    if any(name.startswith(("ROCPROF", "ROCP_")) for name in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return None, "this run is itself under a profiler: counter passes skipped (use --traffic-from)"
    import shutil
    import tempfile

    keep = bool(args.traffic_dir)
    out_dir = os.path.abspath(args.traffic_dir) if keep else tempfile.mkdtemp(prefix="polar_pmc_")
    try:
        phase_args = workload_args(args) + ["--phase", phase, "--steps", "5", "--warmup", "2"]
        dense_args = None
        if args.traffic_dense_pass and phase == "partial":
            from paper_2505_14884_amd import workloads as wl

            w0 = wl.CONFIGS.get(args.workload) or wl.EXTRA_SHAPES[args.workload]
            dense_args = [a for a in phase_args] + ["--k", str(args.Hkv or w0.Hkv)]
        t = rocprof.collect_traffic(out_dir, phase_args, kernels, dense_args)
        if keep:
            with open(os.path.join(out_dir, "commands.txt"), "a") as f:
                f.write("python3 bench.py %s\n" % " ".join(sys.argv[1:]))
        return t, "four rocprofv3 --pmc passes made by this run" if t else "counter passes held no dispatch of %s" % (kernels,)
    except Exception as e:                       # a failed profiler pass must not cost the benchmark
        return None, "counter passes failed: %s" % (str(e)[-300:],)
    finally:
        if not keep:
            shutil.rmtree(out_dir, ignore_errors=True)


def bench_select_gemm(args, torch, np, polar, wl, dev, traffic, traffic_note):
    """Step = batch union of the predicted neuron ids + selective GEMM with ReLU over the union
    (first layer of the sparsified MLP).  value = bytes of the gathered weight rows / step time."""
    w = wl.MLP_CONFIGS[args.mlp_workload]
    if args.density:
        w = wl.MlpWorkload(w.name, w.B, w.K, w.N, args.density, w.dtype, w.seed)
    if args.B:
        w = wl.MlpWorkload(w.name, args.B, w.K, w.N, w.density, w.dtype, w.seed)
    x, W1, topk = wl.make_mlp_inputs(w, dev)
    cap = min(w.N, topk.numel())
    idx = torch.full((cap,), -1, dtype=torch.int32, device=dev)
    count = torch.zeros(1, dtype=torch.int32, device=dev)
    out = torch.zeros((w.B, cap), dtype=torch.float32, device=dev)
    L = polar.binding.lib()
    st = lambda: torch.cuda.current_stream().cuda_stream

    wide = args.gemm_form == "wide"
    workspace = polar.alloc_select_gemm_workspace(w.B, dev) if wide else None    # None beyond 128 rows
    union_ws = None
    if wide:
        nbytes = polar.neuron_union_workspace_bytes(w.B, topk.shape[1], w.N)
        union_ws = torch.empty(nbytes, dtype=torch.uint8, device=dev) if nbytes else None

    def union():
        polar.neuron_union(topk, w.N, workspace=union_ws, out=(idx, count))

    layers = max(1, args.mlp_layers)
    W1s = [W1] + [W1.clone() for _ in range(layers - 1)]
    turn = [0]

    def gemm(i=0):
        turn[0] += 1
        polar.select_gemm(x, W1s[turn[0] % layers], idx, count=count, relu=True, out=out, workspace=workspace)

    union()
    torch.cuda.synchronize()
    n_sel = int(count.item())
    bytes_sel = n_sel * w.K * 2
    all_idx = torch.arange(w.N, dtype=torch.int32, device=dev)
    dense_out = torch.empty((w.B, w.N), dtype=torch.float32, device=dev)

    if args.phase == "select_gemm_only":       # counter runs: both factors, nothing else
        W2o = [torch.zeros_like(W1) for _ in range(layers)]
        yo = torch.empty((w.B, w.K), dtype=torch.float32, device=dev)
        wso = torch.empty(polar.select_gemm_down_workspace_bytes(w.B, w.K, cap), dtype=torch.uint8, device=dev)
        for i in range(args.warmup + args.steps):
            gemm()
            polar.select_gemm_down(out, W2o[i % layers], idx, count=count, out=yo, workspace=wso)
        torch.cuda.synchronize()
        print(json.dumps({"phase": "select_gemm_only", "workload": w.name,
                          "launches": args.warmup + args.steps,
                          "algorithmic_bytes_per_launch": bytes_sel}))
        return

    t_busy = time.perf_counter()               # let the clocks of a freshly initialised GPU settle (see main)
    while time.perf_counter() - t_busy < args.settle_ms * 1e-3:
        union(); gemm()
        torch.cuda.synchronize()
    for i in range(args.warmup):
        union(); gemm()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        union(); gemm()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    def ev(fn, n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    n_ev = max(10, min(args.steps, 100))
    gemm_ms = ev(gemm, n_ev)
    union_ms = ev(union, n_ev)
    dense_ms = float("nan") if args.no_dense else ev(
        lambda: polar.select_gemm(x, W1, all_idx, relu=True, out=dense_out, workspace=workspace), max(5, n_ev // 4))
    # (all rows of one matrix are 680 MB: more than the last-level cache holds, no rotation needed)
    achieved = bytes_sel / (gemm_ms * 1e-3) / 1e9
    # second factor of the sparsified MLP on the same index: Y = h16(hidden) W2[idx,:]
    g2 = torch.Generator(device=dev).manual_seed(w.seed + 1)
    W2 = (torch.randn((w.N, w.K), generator=g2, device=dev) / 100.0).to(W1.dtype)
    W2s = [W2] + [W2.clone() for _ in range(layers - 1)]
    y = torch.empty((w.B, w.K), dtype=torch.float32, device=dev)
    down_ws = torch.empty(polar.select_gemm_down_workspace_bytes(w.B, w.K, cap), dtype=torch.uint8, device=dev)

    def down():
        turn[0] += 1
        polar.select_gemm_down(out, W2s[turn[0] % layers], idx, count=count, out=y, workspace=down_ws)

    down_ms = ev(down, n_ev)
    mlp_ms = ev(lambda: (union(), gemm(), down()), n_ev)
    # the same two factors through the one-call entry point (hidden activations stay 16-bit in its workspace)
    mlp_ws = torch.empty(polar.sparse_mlp_workspace_bytes(w.B, w.K, cap), dtype=torch.uint8, device=dev)

    def fused():
        turn[0] += 1
        polar.sparse_mlp(x, W1s[turn[0] % layers], W2s[turn[0] % layers], idx, count=count, relu=True, out=y,
                         workspace=mlp_ws)

    fused_ms = ev(fused, n_ev)
    mlp1_ms = ev(lambda: (union(), fused()), n_ev)
    # what the bare access pattern reaches: the same gathered rows, read and nothing else
    probe_sink = torch.empty(2 * ((n_sel + 63) // 64) * 3, dtype=torch.int32, device=dev)
    live_idx = idx[:n_sel].contiguous()

    def probe(depth):
        def run():
            turn[0] += 1
            polar.probe_gather_read(W1s[turn[0] % layers], live_idx, slices=3, depth=depth, nontemporal=True,
                                    sink=probe_sink)
        for _ in range(3):                        # first launches of a kernel are not representative
            run()
        torch.cuda.synchronize()
        return round(bytes_sel / (min(ev(run, max(5, n_ev // 4)) for _ in range(2)) * 1e-3) / 1e9, 1)
    gather_probe = {"one_block_in_flight": probe(1), "four_blocks_in_flight": probe(4)}
    result = {
        "metric": "selective fused-gather GEMM effective weight HBM GB/s (gathered rows' bytes / step "
                  "time; step = batch neuron union + GEMM with ReLU)",
        "value": round(bytes_sel / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d K=%d N=%d %s weights, union %d neurons (%.1f %%)"
                               % (w.name, w.B, w.K, w.N, w.dtype, n_sel, 100.0 * n_sel / w.N),
                   "weight_copies_rotated": layers,
                   "selected_weight_bytes": bytes_sel, "dense_weight_bytes": w.N * w.K * 2},
        "breakdown_us": {"neuron_union": round(union_ms * 1e3, 2), "select_gemm": round(gemm_ms * 1e3, 2),
                         "dense_gemm_all_rows": None if args.no_dense else round(dense_ms * 1e3, 2),
                         "select_gemm_down": round(down_ms * 1e3, 2),
                         "sparse_mlp_one_call": round(fused_ms * 1e3, 2),
                         "union_and_sparse_mlp_one_call": round(mlp1_ms * 1e3, 2),
                         "union_and_both_factors": round(mlp_ms * 1e3, 2)},
        # the second factor streams the same number of weight bytes (one row of W2 per live neuron)
        "second_factor": {"kernel": "select_gemm_down_kernel + select_gemm_down_reduce_kernel", "bound": "hbm",
                          "achieved": round(bytes_sel / (down_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": round(bytes_sel / (down_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          "avg_us": round(down_ms * 1e3, 2)},
        "dense_over_selective": None if args.no_dense else round(dense_ms / gemm_ms, 3),
        "ideal_N_over_selected": round(w.N / max(n_sel, 1), 3),
        "roofline": {"kernel": "select_gemm_stream_kernel + select_gemm_reduce_kernel" if workspace is not None else "select_gemm_kernel",
                     "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "avg_us": round(gemm_ms * 1e3, 2),
                     "mfma_tflops": round(2.0 * w.B * w.K * n_sel / (gemm_ms * 1e-3) / 1e12, 1),
                     "gathered_read_probe_GBps": gather_probe,
                     # HBM bytes per launch of the first factor read from the counters by this run, or null
                     "traffic": traffic["bytes"] if traffic else None,
                     "traffic_over_algorithmic": round(traffic["bytes"] / max(bytes_sel, 1), 4) if traffic else None,
                     "traffic_detail": dict(traffic, note=traffic_note) if traffic else {"note": traffic_note}},
    }
    if not args.no_cpu_baseline:
        from oracle import polar_oracle as orc

        ncol = min(n_sel, 1024)
        cols = idx[:ncol].long()
        c0 = time.perf_counter()
        ref = orc.select_gemm(wl.bits_u16(x), wl.bits_u16(W1[cols]), np.arange(ncol, dtype=np.int32),
                              w.dtype, True)
        c1 = time.perf_counter()
        gemm()
        torch.cuda.synchronize()
        err = float(np.abs(out[:, :ncol].cpu().numpy() - ref).max())
        result["cpu_baseline"] = {
            "value": round(ncol * w.K * 2 / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": 1,
            "kind": "oracle",
            "sample": "first %d of the %d selected neurons, all %d requests, %.2f s" % (ncol, n_sel, w.B, c1 - c0),
            "parity_on_sample": {"out_max_abs_err": err}}
    print(json.dumps(result))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2505_14884_amd as polar
    from paper_2505_14884_amd import workloads as wl

    # Counter passes first, as child processes, while this process has not touched the GPU yet.
    traffic, traffic_note = None, "not applicable to this phase"
    if args.phase == "all":
        w0 = wl.CONFIGS.get(args.workload) or wl.EXTRA_SHAPES[args.workload]
        Hq0, Hkv0 = args.Hq or w0.Hq, args.Hkv or w0.Hkv
        grouped0 = Hq0 // Hkv0 > 1 and w0.d == 128
        traffic, traffic_note = hbm_traffic(args, "partial", ["sha_partial_gqa_kernel<" if grouped0 else "sha_partial_kernel<"])
    elif args.phase == "select_gemm":
        traffic, traffic_note = hbm_traffic(args, "select_gemm_only", ["select_gemm_stream_kernel<", "select_gemm_reduce_kernel<", "select_gemm_kernel<"])

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.phase == "copy":
        nbytes = 4 << 30
        src = torch.full((nbytes // 4,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"phase": "copy", "launches": args.warmup + args.steps,
                          "bytes_read_per_launch": nbytes, "bytes_written_per_launch": nbytes}))
        return

    if args.phase in ("select_gemm", "select_gemm_only"):
        bench_select_gemm(args, torch, np, polar, wl, dev, traffic, traffic_note)
        return

    w = wl.CONFIGS.get(args.workload) or wl.EXTRA_SHAPES[args.workload]
    if args.k:
        w = w.scaled(k=args.k)
    if args.B:
        w = w.scaled(B=args.B)
    if args.Hq:
        w = w.scaled(Hq=args.Hq)
    if args.Hkv:
        w = w.scaled(Hkv=args.Hkv)
    if args.S:
        w = w.scaled(S=args.S, seq_lo=min(w.seq_lo, args.S))

    hidden, Wr = wl.make_router_inputs(w, dev)
    q, K, V, seqlens = wl.make_attention_inputs(w, dev)
    if args.kv_layout == "bshd":
        K, V = K.permute(0, 2, 1, 3).contiguous(), V.permute(0, 2, 1, 3).contiguous()
    lay = args.kv_layout
    bytes_sel = wl.selected_kv_bytes(w, seqlens)
    bytes_dense = wl.selected_kv_bytes(w, seqlens, k=w.Hkv)

    # Small workloads: rotate over R copies of the KV cache so the footprint of consecutive
    # steps exceeds the 256 MB memory-side cache and repeats cannot be served from it.
    R = 1 if bytes_dense >= (2 << 30) else int(math.ceil((2 << 30) / max(bytes_dense, 1)))
    R = min(R, 64)
    caches = [(K, V)] + [(K.clone(), V.clone()) for _ in range(R - 1)]

    head_idx = torch.empty((w.B, w.k), dtype=torch.int32, device=dev)
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
    # one workspace for the selective and the dense call: the chunking depends on k, so neither
    # requirement bounds the other
    ws_sel = polar.alloc_workspace(w.B, w.Hq, w.Hkv, w.S, w.d, w.k, dev)
    ws_dense = polar.alloc_workspace(w.B, w.Hq, w.Hkv, w.S, w.d, w.Hkv, dev)
    ws = ws_sel if ws_sel.numel() >= ws_dense.numel() else ws_dense
    del ws_sel, ws_dense
    rws = polar.alloc_router_workspace(w.B, w.D, w.Hkv, dev)
    chunk = polar.sha_chunk_rows(w.B, w.Hq, w.Hkv, w.S, w.d, w.k)

    def step(i):
        Ki, Vi = caches[i % R]
        polar.router_topk(hidden, Wr, w.k, head_idx=head_idx, workspace=rws)
        polar.sha_decode(q, Ki, Vi, seqlens, head_idx, w.k, out=out, workspace=ws, kv_layout=lay)

    grouped = w.G > 1 and w.d == 128 and polar.get_option("sha_grouped_kernel") == 0   # the matrix-core kernel runs
    # An unsplit cache is finished by the streaming kernel alone (it normalises and zero-fills,
    # no merge kernel): then the attention call itself is one launch of the dominant kernel.
    one_kernel = polar.sha_launches(w.B, w.Hq, w.Hkv, w.S, w.d, w.k) == 1

    def partial_only(i):
        Ki, Vi = caches[i % R]
        if one_kernel:
            polar.sha_decode(q, Ki, Vi, seqlens, head_idx, w.k, out=out, workspace=ws, kv_layout=lay)
        else:
            polar.sha_partial(q, Ki, Vi, seqlens, head_idx, w.k, ws, kv_layout=lay)

    def dense_step(i):
        Ki, Vi = caches[i % R]
        polar.sha_decode(q, Ki, Vi, seqlens, None, w.Hkv, out=out, workspace=ws, kv_layout=lay)

    polar.router_topk(hidden, Wr, w.k, head_idx=head_idx, workspace=rws)
    torch.cuda.synchronize()

    if args.phase == "partial":
        for i in range(args.warmup + args.steps):
            partial_only(i)
        torch.cuda.synchronize()
        print(json.dumps({"phase": "partial", "workload": w.name, "launches": args.warmup + args.steps,
                          "algorithmic_bytes_per_launch": bytes_sel}))
        return

    # ---- whole-step wall time: W untimed, then exactly K timed steps.
    # The steps are replayed from HIP graphs (Section 5: the paper runs its router and kernels
    # under CUDA graphs; a decode step of a model replays one graph that holds all its layers):
    # a graph of L consecutive steps, each on the next cache copy (L = 8, or the number of copies
    # rotated if that is larger, but at most K), replayed K // L times; the K % L steps left over
    # are launched one by one, on the next copies.  With --no-graph all steps are launched one
    # by one, which is also timed below (`eager_us_per_layer`): there the time depends on how
    # fast the host gets its launches out (0 to 20 us of gaps per step between runs of the same
    # binary).  A graph of one step is timed for the breakdown.
    L = max(1, min(max(8, R), args.steps))
    layers_graph = one_graph = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)                                   # warm-up outside any capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        layers_graph, one_graph = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(layers_graph):
            for i in range(L):
                step(i)
        with torch.cuda.graph(one_graph):
            step(0)
        for _ in range(2):                            # a graph's first launches upload it; not part of any step
            layers_graph.replay()
            one_graph.replay()
        torch.cuda.synchronize()

    def run_steps(n):
        if layers_graph is None:
            for i in range(n):
                step(i)
            return
        for _ in range(n // L):
            layers_graph.replay()
        for i in range(n % L):
            step(i)

    def wall_time(run, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(n)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    # A freshly initialised GPU runs its first few hundred milliseconds of work about 3 % slower than the
    # steady state a decode loop lives in (the same binary measured 658 or 682 us per step on C5 depending on
    # how early in the process the timed steps fell).  So the card is kept busy with the same steps for a
    # quarter of a second before the W warm-up steps and the K timed ones.
    t_busy = time.perf_counter()
    while time.perf_counter() - t_busy < args.settle_ms * 1e-3:
        run_steps(L)
        torch.cuda.synchronize()
    run_steps(args.warmup)
    ms_per_step = wall_time(run_steps, args.steps)
    value = bytes_sel / (ms_per_step * 1e-3) / 1e9
    for i in range(min(args.warmup, 5)):
        step(i)
    eager_ms = wall_time(lambda n: [step(i) for i in range(n)], args.steps)

    def event_time(fn, n):
        """Duration of one launch of fn from events on the launch stream: the average over n
        back-to-back launches inside one event bracket, and median / minimum over n separately
        bracketed launches (those include the dispatch latency of a cold queue)."""
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            fn(i)
        b.record()
        pairs = []
        for i in range(n):
            c, d = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c.record()
            fn(i)
            d.record()
            pairs.append((c, d))
        torch.cuda.synchronize()
        ts = sorted(c.elapsed_time(d) for c, d in pairs)
        return a.elapsed_time(b) / n, ts[len(ts) // 2], ts[0]

    n_ev = max(10, min(args.steps, 100))
    part_avg, part_med, part_min = event_time(partial_only, n_ev)
    router_avg, _, _ = event_time(lambda i: polar.router_topk(hidden, Wr, w.k, head_idx=head_idx, workspace=rws), n_ev)
    sha_avg, _, _ = event_time(
        lambda i: polar.sha_decode(q, caches[i % R][0], caches[i % R][1], seqlens, head_idx, w.k,
                                   out=out, workspace=ws, kv_layout=lay), n_ev)
    if args.no_dense:
        dense_avg = float("nan")
    else:
        for i in range(3):
            dense_step(i)
        dense_avg, _, _ = event_time(dense_step, max(5, n_ev // 4))
    achieved = bytes_sel / (part_avg * 1e-3) / 1e9

    # the graphs by events on the stream, for the breakdown
    graph_avg = graph1_avg = float("nan")
    if layers_graph is not None:
        n_rep = max(3, n_ev // L)
        graph_avg = event_time(lambda i: layers_graph.replay(), n_rep)[0] / L
        graph1_avg = event_time(lambda i: one_graph.replay(), n_ev)[0]

    # Read-only yardstick over the same K cache with the streaming kernel's launch shape: what this
    # GPU gives a kernel that does nothing but read, with non-temporal and with plain loads.
    slab = w.S * w.d * 2          # bytes of one head's rows; the probe reads contiguous slabs of that size
    probe_bytes = (K.numel() * 2) // slab * slab
    sink = torch.empty(probe_bytes // slab, dtype=torch.int32, device=dev)
    probe = {}
    for label, nt in (("nontemporal", True), ("plain", False)):
        run_probe = lambda i: polar.probe_read(caches[i % R][0], slab, nt, sink)
        for i in range(3):                        # the first launches of a kernel are not representative
            run_probe(i)
        torch.cuda.synchronize()
        t_avg = min(event_time(run_probe, max(10, n_ev // 4))[0] for _ in range(2))
        probe[label] = round(probe_bytes / (t_avg * 1e-3) / 1e9, 1)

    result = {
        "metric": "selective-head decode attention effective KV HBM GB/s "
                  "(selected-head K+V bytes / step time; us per layer = 1000*ms_per_step)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # the arithmetic of the kernel that ran: scores, softmax statistics and the output accumulate in
        # float; the grouped-head kernel feeds each probability to the second matrix product as two
        # 16-bit terms (rounded value + rounded remainder), the per-head kernel keeps it a float
        "dtype": "f32 (P as 2x16-bit terms into MFMA)" if grouped else "f32",
        "data": "synthetic",
        "config": {
            "workload": "%s: B=%d Hq=%d Hkv=%d d=%d S=%d k=%d %s KV, router D=%d"
                        % (w.name, w.B, w.Hq, w.Hkv, w.d, w.S, w.k, w.dtype, w.D),
            "seqlens": "all %d" % w.S if w.seq_lo <= 0 else "uniform integers in [%d, %d]" % (w.seq_lo, w.S),
            "selected_kv_bytes": bytes_sel,
            "dense_kv_bytes": bytes_dense,
            "kv_layout": lay,
            "chunk_rows": chunk,
            "attention_kernels": "streaming kernel only (unsplit cache)" if one_kernel
                                 else "streaming kernel + merge kernel",
            "kv_copies_rotated": R,
            "settle_ms_before_warmup": args.settle_ms,
            "launch": "eager launches" if layers_graph is None else
                      "HIP graph of %d consecutive steps replayed %d times + %d steps launched one by one"
                      % (L, args.steps // L, args.steps % L),
        },
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "us_per_layer": round(ms_per_step * 1e3, 2),
        "breakdown_us": {
            "router_topk": round(router_avg * 1e3, 2),
            "sha_decode": round(sha_avg * 1e3, 2),
            "streaming_kernel": round(part_avg * 1e3, 2),
            "eager_us_per_layer": round(eager_ms * 1e3, 2),
            "step_in_hip_graph_of_%d_layers" % L: None if args.no_graph else round(graph_avg * 1e3, 2),
            "step_in_hip_graph_of_1_layer": None if args.no_graph else round(graph1_avg * 1e3, 2),
            "dense_k_eq_H": None if args.no_dense else round(dense_avg * 1e3, 2),
        },
        "dense_over_selective": None if args.no_dense else round(dense_avg / sha_avg, 3),
        "ideal_H_over_k": round(w.Hkv / w.k, 3),
        "roofline": {
            "kernel": "sha_partial_gqa_kernel" if grouped else "sha_partial_kernel",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "avg_us": round(part_avg * 1e3, 2),
            "median_us": round(part_med * 1e3, 2),
            "min_us": round(part_min * 1e3, 2),
            "read_probe_GBps": probe,
            # HBM bytes per launch read from the counters by this run (see hbm_traffic), or null
            "traffic": traffic["bytes"] if traffic else None,
            "traffic_over_algorithmic": round(traffic["bytes"] / bytes_sel, 4) if traffic else None,
            "traffic_detail": dict(traffic, note=traffic_note) if traffic else {"note": traffic_note},
        },
    }

    if not args.no_cpu_baseline:
        from oracle import polar_oracle as orc

        if args.cpu_threads > 0:
            orc.set_num_threads(args.cpu_threads)
        nb = w.B if args.cpu_sample <= 0 else max(1, min(args.cpu_sample, w.B))
        nb = max(1, min(nb, int(12e9) // (2 * w.Hkv * w.S * w.d * 2)))
        hb, Wb = wl.bits_u16(hidden[:nb]), wl.bits_u16(Wr)
        Ks, Vs = (K[:nb], V[:nb]) if lay == "bhsd" else (K[:nb].permute(0, 2, 1, 3), V[:nb].permute(0, 2, 1, 3))
        qb, Kb, Vb = wl.bits_u16(q[:nb]), wl.bits_u16(Ks), wl.bits_u16(Vs)
        nh = seqlens[:nb].cpu().numpy()
        step(0)                       # leave the selective result of copy 0 in `out`
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        idx = orc.router_topk(hb, Wb, w.k, w.dtype)
        ref = orc.sha_decode(qb, Kb, Vb, nh, idx, w.k, w.dtype)
        c1 = time.perf_counter()
        sample_bytes = int(np.clip(nh, 0, w.S).astype(np.int64).sum()) * w.k * 2 * w.d * 2
        gpu_idx = head_idx[:nb].cpu().numpy()
        err = float(np.abs(out[:nb].cpu().numpy() - ref).max())
        result["cpu_baseline"] = {
            "value": round(sample_bytes / (c1 - c0) / 1e9, 4),
            "unit": "GB/s",
            "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": "first %d of %d requests of the same workload (router + top-k + selected "
                      "heads' attention), %.2f s" % (nb, w.B, c1 - c0),
            "seconds_per_layer_extrapolated": round((c1 - c0) * bytes_sel / max(sample_bytes, 1), 3),
            "parity_on_sample": {"head_idx_equal": bool(np.array_equal(gpu_idx, idx)),
                                 "out_max_abs_err": err},
        }

    print(json.dumps(result))


if __name__ == "__main__":
    main()
