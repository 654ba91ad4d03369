"""rocprofv3 plumbing for the benchmark: run counter passes, read their CSV files, write the
short summaries kept under ``profiles/``.

Nothing here computes anything of the method; it only drives the profiler and reads what it wrote.

Layout of a profile directory ``D`` (every part is optional; readers use what is there):

    D/fetch/       rocprofv3 --pmc FETCH_SIZE  ... -- python3 bench.py <workload> --phase partial
    D/write/       rocprofv3 --pmc WRITE_SIZE  ... -- python3 bench.py <workload> --phase partial
    D/copy_fetch/  rocprofv3 --pmc FETCH_SIZE  ... -- python3 bench.py --phase copy
    D/copy_write/  rocprofv3 --pmc WRITE_SIZE  ... -- python3 bench.py --phase copy
    D/dense_fetch/ the fetch pass again with k = Hkv (the dense run of the same kernel)
    D/trace/       rocprofv3 --kernel-trace --stats ... -- python3 bench.py <workload> ...
    D/*.json       the JSON line each of those bench.py runs printed
    D/commands.txt the full command of every pass, as it was run

``bench.py`` fills fetch, write, copy_* itself (``collect_traffic``) and reads them back
(``traffic_from``), so its ``roofline.traffic`` is a counter reading of the kernels it has just
timed, not a stored constant.  The copy passes are the yardstick: FETCH_SIZE and WRITE_SIZE are
scaled by what the same counter reads for a plain device copy of known size.

    python -m paper_2505_14884_amd.rocprof attention D --out profiles/<name>.md
    python -m paper_2505_14884_amd.rocprof mlp D --out profiles/<name>.md
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import shutil
import subprocess
import sys
from typing import Dict, List, Optional, Sequence, Tuple

COPY_KERNEL = "copyBuffer"        # substring of the runtime's device-to-device copy kernel


def rocprofv3() -> Optional[str]:
    return shutil.which("rocprofv3") or ("/opt/rocm/bin/rocprofv3" if os.path.exists("/opt/rocm/bin/rocprofv3") else None)


def _one(pattern_dir: str, suffix: str) -> Optional[str]:
    hits = sorted(glob.glob(os.path.join(pattern_dir, "**", "*" + suffix), recursive=True))
    return hits[0] if hits else None


def short_name(kernel: str) -> str:
    """`void polar::(anonymous namespace)::foo<A, B>(args)` -> `foo<A, B>`."""
    name = kernel.replace("void ", "").replace("polar::(anonymous namespace)::", "").replace("polar::", "")
    depth = 0
    for i, ch in enumerate(name):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return name[:i]
    return name


def kernel_stats(trace_dir: str, only: str = "polar") -> List[dict]:
    """Rows of `*_kernel_stats.csv` (rocprofv3 --kernel-trace --stats) whose name contains `only`."""
    path = _one(trace_dir, "kernel_stats.csv")
    if not path:
        return []
    rows = []
    for r in csv.DictReader(open(path, newline="")):
        if only in r["Name"]:
            rows.append({"kernel": short_name(r["Name"]), "calls": int(r["Calls"]),
                         "avg_us": float(r["AverageNs"]) / 1e3, "min_us": float(r["MinNs"]) / 1e3,
                         "max_us": float(r["MaxNs"]) / 1e3})
    return sorted(rows, key=lambda r: -r["avg_us"] * r["calls"])


def counter_per_dispatch(pmc_dir: str, counter: str) -> Dict[str, Tuple[float, int]]:
    """{short kernel name: (mean counter value per dispatch, dispatches)} from `*_counter_collection.csv`."""
    path = _one(pmc_dir, "counter_collection.csv")
    if not path:
        return {}
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path, newline="")):
        if r["Counter_Name"] == counter:
            agg[short_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in agg.items()}


def last_json(path: str) -> Optional[dict]:
    if not os.path.exists(path):
        return None
    lines = [ln for ln in open(path).read().splitlines() if ln.startswith("{")]
    return json.loads(lines[-1]) if lines else None


def copy_factors(profile_dir: str) -> Optional[dict]:
    """Scale factors of FETCH_SIZE and WRITE_SIZE (KiB per dispatch) from the plain-copy passes."""
    meta = last_json(os.path.join(profile_dir, "copy_fetch.json")) or last_json(os.path.join(profile_dir, "copy_write.json"))
    cf = counter_per_dispatch(os.path.join(profile_dir, "copy_fetch"), "FETCH_SIZE")
    cw = counter_per_dispatch(os.path.join(profile_dir, "copy_write"), "WRITE_SIZE")
    kf = [k for k in cf if COPY_KERNEL in k]
    kw = [k for k in cw if COPY_KERNEL in k]
    if not (meta and kf and kw):
        return None
    fetch_kib, write_kib = cf[kf[0]][0], cw[kw[0]][0]
    if fetch_kib <= 0 or write_kib <= 0:
        return None
    return {"copy_kernel": kf[0], "copy_bytes": meta["bytes_read_per_launch"],
            "fetch_kib": fetch_kib, "write_kib": write_kib,
            "fetch_factor": meta["bytes_read_per_launch"] / 1024.0 / fetch_kib,
            "write_factor": meta["bytes_written_per_launch"] / 1024.0 / write_kib}


def traffic_from(profile_dir: str, kernels: Sequence[str], fetch_sub: str = "fetch", write_sub: str = "write") -> Optional[dict]:
    """HBM bytes per launch of the kernels whose short name starts with one of `kernels`, summed:
    FETCH_SIZE and WRITE_SIZE per dispatch (KiB), each scaled by the copy yardstick's factor.
    None when a pass is missing."""
    fac = copy_factors(profile_dir)
    F = counter_per_dispatch(os.path.join(profile_dir, fetch_sub), "FETCH_SIZE")
    W = counter_per_dispatch(os.path.join(profile_dir, write_sub), "WRITE_SIZE")
    if not (fac and F and W):
        return None
    per = []
    for want in kernels:
        names = [k for k in F if k.startswith(want) and k in W]
        for name in names:
            rd = F[name][0] * 1024.0 * fac["fetch_factor"]
            wr = W[name][0] * 1024.0 * fac["write_factor"]
            per.append({"kernel": name, "dispatches": F[name][1], "fetch_kib_raw": round(F[name][0], 1),
                        "write_kib_raw": round(W[name][0], 1), "read_bytes": int(round(rd)),
                        "written_bytes": int(round(wr))})
    if not per:
        return None
    return {"bytes": sum(p["read_bytes"] + p["written_bytes"] for p in per),
            "read_bytes": sum(p["read_bytes"] for p in per),
            "written_bytes": sum(p["written_bytes"] for p in per),
            "fetch_factor": round(fac["fetch_factor"], 4), "write_factor": round(fac["write_factor"], 4),
            "kernels": per}


def run_pmc_pass(out_dir: str, name: str, counter: str, bench_args: Sequence[str], timeout_s: int = 180) -> dict:
    """One `rocprofv3 --pmc <counter> -- python3 bench.py <bench_args>` run as a child process; CSVs
    go to out_dir/name, the child's JSON line to out_dir/name.json.  The program itself follows
    `--` (no shell, no wrapper).  Raises on failure."""
    exe = rocprofv3()
    if not exe:
        raise RuntimeError("rocprofv3 not found")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sub = os.path.join(out_dir, name)
    shutil.rmtree(sub, ignore_errors=True)
    os.makedirs(sub, exist_ok=True)
    cmd = [exe, "--pmc", counter, "-f", "csv", "-d", sub, "-o", "p", "--", sys.executable,
           os.path.join(root, "bench.py")] + list(bench_args)
    env = dict(os.environ, TMPDIR="/tmp")
    proc = subprocess.run(cmd, cwd="/tmp", env=env, capture_output=True, text=True, timeout=timeout_s)
    with open(os.path.join(out_dir, "commands.txt"), "a") as f:
        f.write("rocprofv3 --pmc %s -f csv -d %s -o p -- python3 bench.py %s\n" % (counter, sub, " ".join(bench_args)))
    if proc.returncode != 0:
        raise RuntimeError("%s pass failed (exit %d): %s" % (name, proc.returncode, proc.stderr[-400:]))
    lines = [ln for ln in proc.stdout.splitlines() if ln.startswith("{")]
    with open(os.path.join(out_dir, name + ".json"), "w") as f:
        f.write((lines[-1] if lines else "{}") + "\n")
    return json.loads(lines[-1]) if lines else {}


def collect_traffic(out_dir: str, phase_args: Sequence[str], kernels: Sequence[str], dense_args: Optional[Sequence[str]] = None) -> Optional[dict]:
    """The four counter passes of a workload (and, with dense_args, a fifth over the dense run),
    then `traffic_from`.  Called before the calling process has touched the GPU."""
    os.makedirs(out_dir, exist_ok=True)
    open(os.path.join(out_dir, "commands.txt"), "w").close()
    run_pmc_pass(out_dir, "fetch", "FETCH_SIZE", phase_args)
    run_pmc_pass(out_dir, "write", "WRITE_SIZE", phase_args)
    copy_args = ["--phase", "copy", "--steps", "3", "--warmup", "1"]
    run_pmc_pass(out_dir, "copy_fetch", "FETCH_SIZE", copy_args)
    run_pmc_pass(out_dir, "copy_write", "WRITE_SIZE", copy_args)
    if dense_args:
        run_pmc_pass(out_dir, "dense_fetch", "FETCH_SIZE", dense_args)
    return traffic_from(out_dir, kernels)


# ------------------------------------------------------------------------------------- summaries
def _commands(profile_dir: str) -> List[str]:
    path = os.path.join(profile_dir, "commands.txt")
    lines = [ln.strip() for ln in open(path).read().splitlines()] if os.path.exists(path) else []
    lines = [ln.replace(os.path.abspath(profile_dir), "<dir>").replace(profile_dir, "<dir>") for ln in lines if ln]
    # the run that reads the passes back (--traffic-from) is the traced one: it was started under the profiler
    return [("rocprofv3 --kernel-trace --stats -f csv -d <dir>/trace -o t -- " + ln + " > <dir>/trace.json")
            if "--traffic-from" in ln else (ln + " > <dir>/bench.json" if ln.startswith("python3 bench.py") else ln)
            for ln in lines]


def _trace_table(rows: List[dict]) -> List[str]:
    out = ["| kernel | calls | avg us | min us | max us |", "|---|---|---|---|---|"]
    for r in rows:
        out.append("| `%s` | %d | %.2f | %.2f | %.2f |" % (r["kernel"], r["calls"], r["avg_us"], r["min_us"], r["max_us"]))
    return out


def _traffic_lines(t: dict, alg: Optional[int], what: str) -> List[str]:
    out = ["Copy yardstick: FETCH_SIZE x %.4f, WRITE_SIZE x %.4f (a plain device copy of known size read by the same counters)." % (t["fetch_factor"], t["write_factor"]), "",
           "| kernel | dispatches | FETCH_SIZE KiB (raw) | read bytes (scaled) | WRITE_SIZE KiB (raw) | written bytes (scaled) |",
           "|---|---|---|---|---|---|"]
    for p in t["kernels"]:
        out.append("| `%s` | %d | %.1f | %.4e | %.1f | %.4e |" % (p["kernel"], p["dispatches"], p["fetch_kib_raw"], p["read_bytes"], p["write_kib_raw"], p["written_bytes"]))
    out.append("")
    if alg:
        out.append("Algorithmic bytes per launch (%s): %d = %.4e." % (what, alg, alg))
        out.append("Measured HBM traffic per launch: %.4e bytes = %.4f x algorithmic (reads %.4f x)." % (t["bytes"], t["bytes"] / alg, t["read_bytes"] / alg))
    return out


def summarize_attention(profile_dir: str) -> str:
    bench = last_json(os.path.join(profile_dir, "bench.json"))
    trace = last_json(os.path.join(profile_dir, "trace.json"))
    fetch = last_json(os.path.join(profile_dir, "fetch.json")) or {}
    name = (bench or trace or {}).get("config", {}).get("workload", fetch.get("workload", "?"))
    out = ["# rocprofv3 summary: %s, whole step (router + selective decode attention)" % name.split(":")[0], "",
           "Commands (from the repository root on the MI355X box; `<dir>` is any scratch directory; `bench.py` runs the",
           "`--pmc` passes itself, as child processes with `cwd=/tmp`, `TMPDIR=/tmp`, and logs them in `<dir>/commands.txt`):", "", "```"]
    out += _commands(profile_dir) + ["python3 -m paper_2505_14884_amd.rocprof attention <dir> --out profiles/<this file>", "```", ""]
    rows = kernel_stats(os.path.join(profile_dir, "trace"))
    if rows:
        out += ["## Kernel trace (`rocprofv3 --kernel-trace --stats`, this library's kernels)", ""] + _trace_table(rows) + [""]
    for label, js in (("untraced run", bench), ("the traced run's own event timing", trace)):
        if js and "roofline" in js:
            r, b = js["roofline"], js["breakdown_us"]
            out.append("bench.py, %s: `%s` avg %.2f us (median %.2f, min %.2f) by events on the launch stream = %.1f GB/s = %.2f %% of 8 TB/s; "
                       "router %.2f us; step %.2f us = %.1f GB/s (%.2f %%; %s; launched one by one: %s us); dense (k = H) / selective %s "
                       "(ideal %s); read yardstick (GB/s) %s."
                       % (label, r["kernel"], r["avg_us"], r["median_us"], r["min_us"], r["achieved"], 100 * r["frac"], b["router_topk"],
                          js["us_per_layer"], js["value"], js["pct_of_hbm_peak"], js.get("config", {}).get("launch", "eager launches"),
                          b.get("eager_us_per_layer"), js.get("dense_over_selective"), js.get("ideal_H_over_k"),
                          json.dumps(r.get("read_probe_GBps"))))
            out.append("")
    kern = ((bench or trace or {}).get("roofline") or {}).get("kernel")
    t = traffic_from(profile_dir, [kern + "<"] if kern else ["sha_partial"])
    if t:
        out += ["## HBM traffic counters (KiB per dispatch; `--phase partial` launches the streaming kernel only)", ""]
        out += _traffic_lines(t, fetch.get("algorithmic_bytes_per_launch"), "selected heads' K+V rows") + [""]
    dense = last_json(os.path.join(profile_dir, "dense_fetch.json"))
    td = traffic_from(profile_dir, [kern + "<"] if kern else ["sha_partial"], fetch_sub="dense_fetch")
    if t and td and dense:
        alg_d = dense["algorithmic_bytes_per_launch"]
        out += ["## Dense run of the same kernel (k = H), for the selective / dense traffic ratio", "",
                "Dense reads %.4e bytes per launch (%.4f x its %d algorithmic bytes); selective reads %.4e: selective / dense = %.4f "
                "(k / H = %.4f), i.e. the unselected heads' K/V is physically never fetched." %
                (td["read_bytes"], td["read_bytes"] / alg_d, alg_d, t["read_bytes"], t["read_bytes"] / td["read_bytes"],
                 fetch.get("algorithmic_bytes_per_launch", 0) / alg_d), ""]
    return "\n".join(out) + "\n"


def summarize_mlp(profile_dir: str) -> str:
    bench = last_json(os.path.join(profile_dir, "bench.json"))
    trace = last_json(os.path.join(profile_dir, "trace.json"))
    fetch = last_json(os.path.join(profile_dir, "fetch.json")) or {}
    name = (bench or trace or {}).get("config", {}).get("workload", "?")
    out = ["# rocprofv3 summary: sparsified MLP (batch neuron index, selective fused-gather GEMM, second factor), %s" % name, "",
           "Commands (from the repository root on the MI355X box; `<dir>` is any scratch directory; `bench.py` runs the",
           "`--pmc` passes itself, as child processes with `cwd=/tmp`, `TMPDIR=/tmp`, and logs them in `<dir>/commands.txt`):", "", "```"]
    out += _commands(profile_dir) + ["python3 -m paper_2505_14884_amd.rocprof mlp <dir> --out profiles/<this file>", "```", ""]
    rows = kernel_stats(os.path.join(profile_dir, "trace"))
    if rows:
        out += ["## Kernel trace (`rocprofv3 --kernel-trace --stats`, this library's kernels)", ""] + _trace_table(rows) + [""]
    for label, js in (("untraced run", bench), ("the traced run's own event timing", trace)):
        if js and "breakdown_us" in js:
            out.append("bench.py, %s: breakdown (us, events on the launch stream) %s; first factor %s GB/s (%.1f %% of 8 TB/s), second factor %s GB/s (%.1f %%); "
                       "gathered-read yardstick %s GB/s; dense / selective %s (ideal %s)."
                       % (label, json.dumps(js["breakdown_us"]), js["roofline"]["achieved"], 100 * js["roofline"]["frac"],
                          js["second_factor"]["achieved"], 100 * js["second_factor"]["frac"],
                          js["roofline"].get("gathered_read_probe_GBps"), js.get("dense_over_selective"), js.get("ideal_N_over_selected")))
            out.append("")
    alg = fetch.get("algorithmic_bytes_per_launch")
    for title, kernels in (("first factor", ["select_gemm_stream_kernel<", "select_gemm_reduce_kernel<", "select_gemm_kernel<"]),
                           ("second factor", ["select_gemm_down"])):
        t = traffic_from(profile_dir, kernels)
        if t:
            out += ["## HBM traffic counters, %s (`--phase select_gemm_only`)" % title, ""]
            out += _traffic_lines(t, alg, "gathered weight rows of one factor") + [""]
    return "\n".join(out) + "\n"


def summarize_kernels(labelled_dirs: Sequence[str], match: str, title: str, note: str) -> str:
    """One table of a kernel's duration across several traced runs (`label=trace_dir` each): used for
    builds of the library with parts of a kernel switched off."""
    out = ["# %s" % title, ""]
    if note:
        out += [note, ""]
    out += ["| run | kernel | calls | avg us | min us | max us |", "|---|---|---|---|---|---|"]
    for item in labelled_dirs:
        label, _, d = item.partition("=")
        for r in kernel_stats(d):
            if match in r["kernel"]:
                out.append("| %s | `%s` | %d | %.2f | %.2f | %.2f |" % (label, r["kernel"], r["calls"], r["avg_us"], r["min_us"], r["max_us"]))
    return "\n".join(out) + "\n"


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("kind", choices=["attention", "mlp", "kernels"])
    ap.add_argument("dir", nargs="+", help="profile directory; for `kernels`: label=trace_dir pairs")
    ap.add_argument("--out", default="")
    ap.add_argument("--match", default="", help="kernels: substring of the kernel name")
    ap.add_argument("--title", default="rocprofv3 kernel trace")
    ap.add_argument("--note", default="", help="kernels: text (or @file) placed under the title: commands, what the runs are")
    a = ap.parse_args(argv)
    if a.kind == "kernels":
        note = open(a.note[1:]).read().rstrip() if a.note.startswith("@") else a.note
        text = summarize_kernels(a.dir, a.match, a.title, note)
    else:
        text = summarize_attention(a.dir[0]) if a.kind == "attention" else summarize_mlp(a.dir[0])
    if a.out:
        with open(a.out, "w") as f:
            f.write(text)
    print(text)


if __name__ == "__main__":
    main()
