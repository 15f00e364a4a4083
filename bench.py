#!/usr/bin/env python3
"""Benchmark of the sub-sampled Newton hot path on one MI355X.

A step is one full SSN iteration on the wide dense workload (50000 x 3072, C = 10: the largest of the
benchmark's workloads, 1.23 GB in fp64): full gradient and objective, Hessian sample of 5 % of the rows,
<= 10 CG products H_S v, Armijo line search, update.  Headline value: sub-sampled Hessian-vector products per
second (back-to-back ssn_hess_apply on resident data).  Also reported in the same JSON line: time per SSN
iteration, the HBM roofline of the dominant STREAMING kernel (the gradient pass over all rows; HIP events inside
the library on its own stream) next to the cache-resident sampled product, call-level effective bandwidth of
objective / gradient / H_S v, the same figures for the other workloads, and the CPU oracle timed on one core
and on all cores.
"""
import argparse
import json
import os
import platform
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X datasheet HBM3E bandwidth

# HBM bytes per launch (fetched + written) measured with `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` and scaled by
# the calibration kernels: kept in profiles/hbm_traffic.json next to the summaries they come from (counters cannot
# be read from inside this script).  A kernel without an entry reports null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(workload, dtype, kernel):
    try:
        with open(TRAFFIC_FILE) as fh:
            table = json.load(fh)
    except OSError:
        return None
    ent = table.get(workload, {}).get(dtype, {}).get(kernel)
    return None if ent is None else ent["fetch_bytes"] + ent["write_bytes"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dtype", choices=["f64", "f32"], default="f64")
    ap.add_argument("--config", type=int, default=2, help="index into the workload list (2 = wide dense, the largest)")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the summary of the other workloads")
    ap.add_argument("--n", type=int, default=None, help="override the number of rows (debugging)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-other-dtype", action="store_true", help="skip the secondary-dtype figures")
    ap.add_argument("--hv-calls", type=int, default=200)
    ap.add_argument("--pmc", action="store_true",
                    help="counter-collection mode for `rocprofv3 --pmc`: a few launches of every hot kernel, a plain "
                         "streaming read of X and a plain copy of X (calibration), nothing else")
    return ap.parse_args()


def csr_kernel_bytes(n, p, K, nS, e, nnz, nnzS):
    """CSR: stored entries cost value + column index in the rows kernels, value + row position in the
    column-sorted gather; W / V is read once (gathers beyond that are cache traffic)."""
    touched, touched_S = min(p, nnz), min(p, nnzS)          # rows of the p x K block a gather can reach
    return {
        0: nnz * (e + 4) + 4 * (n + 1) + 4 * n + p * K * e,
        1: nnz * (e + 4) + 4 * (n + 1) + 4 * n + p * K * e + n * K * e,
        2: nnz * (e + 4) + n * K * e + 2 * touched * K * e,         # gather by column, read-modify-write of the result
        3: nnzS * (e + 4) + 8 * nS + 2 * nS * K * e + touched_S * K * e,
        4: nnzS * (e + 4) + nS * K * e + 2 * touched_S * K * e,
    }


def kernel_bytes(n, p, K, nS, e, path):
    """Algorithmic bytes one launch of each timed kernel has to move (X counted once per kernel).
    path 1: margins kernel then X^T U kernel; path 2: one sweep does both, kernel 2 / 4 only add up the
    per-workgroup partial sums (no pass over X: no HBM roofline entry)."""
    if path == 2:
        return {
            0: n * p * e + 4 * n + p * K * e,                       # margins + loss
            1: n * p * e + 4 * n + p * K * e,                       # margins + U + X^T U partials, one sweep
            2: None,
            3: nS * p * e + 4 * nS + nS * K * e + p * K * e,        # sampled: margins, P in, X_S^T U partials
            4: None,
        }
    return {
        0: n * p * e + 4 * n + p * K * e,                       # margins + loss
        1: n * p * e + 4 * n + p * K * e + n * K * e,           # margins + U out
        2: n * p * e + n * K * e,                               # X^T U (full)
        3: nS * p * e + 4 * nS + p * K * e + 2 * nS * K * e,    # sampled margins, P in, U out
        4: nS * p * e + 4 * nS + nS * K * e,                    # sampled X^T U
    }


def call_bytes(n, p, K, nS, e, nnz=None, nnzS=None):
    """Algorithmic bytes per call: X is counted ONCE per call whatever the kernel count."""
    if nnz is not None:
        return {
            "objective": nnz * (e + 4) + 4 * (n + 1) + 4 * n + p * K * e,
            "gradient": nnz * (e + 4) + 4 * (n + 1) + 4 * n + 2 * p * K * e,
            "hess_apply": nnzS * (e + 4) + 8 * nS + nS * K * e + 2 * p * K * e,
        }
    return {
        "objective": n * p * e + 4 * n + p * K * e,
        "gradient": n * p * e + 4 * n + 2 * p * K * e,
        "hess_apply": nS * p * e + 4 * nS + nS * K * e + 2 * p * K * e,
    }


KERNEL_NAMES = {
    0: {0: "csr_rows_kernel<OBJ>", 1: "csr_rows_kernel<GRAD>", 2: "csc_piece_kernel + csc_run_kernel + csc_combine_kernel (n rows)",
        3: "csr_rows_kernel<APPLY>", 4: "csc_piece_kernel + csc_combine_kernel (|S| rows)"},
    1: {0: "dense_rows_kernel<OBJ>", 1: "dense_rows_kernel<GRAD>", 2: "dense_xtu_kernel (n rows)",
        3: "dense_rows_kernel<APPLY>", 4: "dense_xtu_kernel (|S| rows)"},
    2: {0: "dense_fused_kernel<OBJ>", 1: "dense_fused_kernel<GRAD>", 2: "finalize_kernel (gradient partials)",
        3: "dense_fused_kernel<APPLY>", 4: "finalize_kernel (H_S v partials)"},
    3: {0: "binary_rows_kernel<OBJ>", 1: "binary_rows_kernel<GRAD>", 2: "binary_xtu_kernel (n rows)",
        3: "binary_rows_kernel<APPLY>", 4: "binary_xtu_kernel (|S| rows)"},
}


def measure(data, dtype_name, steps, warmup, hv_calls, full_step=True):
    import numpy as np
    import torch
    from paper_1802_09113_amd import synth
    from paper_1802_09113_amd.binding import Context

    tdt = torch.float64 if dtype_name == "f64" else torch.float32
    e = 8 if dtype_name == "f64" else 4
    n, p, C, K, nS = data["n"], data["p"], data["C"], data["K"], data["nS"]
    dev = "cuda:0"
    labels = torch.from_numpy(data["labels"]).to(dev)
    sparse = data["layout"] == "csr"
    if sparse:
        csr = (torch.from_numpy(data["rowptr"].astype(np.int32)).to(dev), torch.from_numpy(data["colidx"]).to(dev),
               torch.from_numpy(data["vals"]).to(dev).to(tdt))
        ctx = Context(labels, C, data["lam"], csr=csr, p=p)
        nnz = int(data["nnz"])
    else:
        X = torch.from_numpy(data["X"]).to(dev).to(tdt)
        ctx = Context(labels, C, data["lam"], X=X)
        nnz = None
    W = torch.zeros((p, K), dtype=tdt, device=dev)
    out = {}
    S_all = torch.from_numpy(synth.sample_schedule(n, nS, warmup + steps)).to(dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    if full_step:
        if warmup > 0:
            ctx.ssn_solve(W, S_all[:warmup].contiguous(), theta=1e-4, T=data["T"])
        torch.cuda.synchronize()
        W_start = W.clone()
        # the timed steps run without the stream events behind the per-phase times (six records per iteration,
        # a few microseconds of device time each); the same steps are then repeated with them for the breakdown
        t0 = time.perf_counter()
        recs_timed, done = ctx.ssn_solve(W, S_all[warmup:].contiguous(), theta=1e-4, T=data["T"], phase_times=False)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        assert done == steps
        out["ms_per_step"] = (t1 - t0) * 1e3 / steps
        W_timed = W.clone()
        W.copy_(W_start)
        t0 = time.perf_counter()
        recs, done = ctx.ssn_solve(W, S_all[warmup:].contiguous(), theta=1e-4, T=data["T"])
        torch.cuda.synchronize()
        out["ms_per_step_with_phase_events"] = (time.perf_counter() - t0) * 1e3 / steps
        assert done == steps and torch.equal(W, W_timed) and [r["f"] for r in recs] == [r["f"] for r in recs_timed]
        out["products_in_steps"] = sum(r["cg_iters"] for r in recs)
        out["hv_per_s_inside_cg"] = out["products_in_steps"] / max(sum(r["ms_cg"] for r in recs) * 1e-3, 1e-12)
        out["phase_ms"] = {k: statistics.mean(r[k] for r in recs)
                           for k in ("ms_grad", "ms_prepare", "ms_cg", "ms_linesearch", "ms_update")}
        out["ls_evals_mean"] = statistics.mean(r["ls_evals"] for r in recs)
        out["final_f"] = recs[-1]["f"]
    else:
        W.copy_(torch.from_numpy(synth.probe(p, K, sub=1, scale=0.05)).to(dev).to(tdt))

    # back-to-back H_S v: rotating direction / result buffers, 5 batches, median
    S = S_all[-1].contiguous()
    ctx.ssn_hess_prepare(W, S)
    V = [torch.from_numpy(synth.probe(p, K, sub=10 + i)).to(dev).to(tdt) for i in range(2)]
    HV = [torch.empty_like(V[0]) for _ in range(2)]
    for i in range(10):
        ctx.ssn_hess_apply(V[i & 1], HV[i & 1])
    torch.cuda.synchronize()
    rates = []
    for b in range(5):
        a, z = ev(), ev()
        a.record()
        for i in range(hv_calls):
            ctx.ssn_hess_apply(V[i & 1], HV[i & 1])
        z.record()
        torch.cuda.synchronize()
        rates.append(hv_calls / (a.elapsed_time(z) * 1e-3))
    out["hv_per_s"] = statistics.median(rates)

    # gradient (asynchronous, no scalar read-back) and objective (returns a scalar: includes one sync)
    G = torch.empty_like(W)
    for _ in range(3):
        ctx.ssn_gradient(W, G, want_f=False)
    torch.cuda.synchronize()
    a, z = ev(), ev()
    a.record()
    for _ in range(20):
        ctx.ssn_gradient(W, G, want_f=False)
    z.record()
    torch.cuda.synchronize()
    ms_grad = a.elapsed_time(z) / 20
    t0 = time.perf_counter()
    for _ in range(20):
        ctx.ssn_objective(W)
    ms_obj = (time.perf_counter() - t0) * 1e3 / 20
    nnzS = None
    if sparse:
        rl = data["rowptr"][1:] - data["rowptr"][:-1]
        nnzS = int(rl[S.cpu().numpy()].sum())
    cb = call_bytes(n, p, K, nS, e, nnz, nnzS)
    ms_call = {"objective": ms_obj, "gradient": ms_grad, "hess_apply": 1e3 / out["hv_per_s"]}
    out["calls"] = {k: {"ms": ms_call[k], "algorithmic_GB": cb[k] / 1e9,
                        "GBps": cb[k] / ms_call[k] / 1e6, "frac_of_hbm_peak": cb[k] / ms_call[k] / 1e6 / HBM_PEAK_GBS}
                    for k in cb}

    # per-kernel durations from HIP events recorded by the library on its own stream
    path = ctx.ssn_dense_path()
    out["dense_path"] = path
    kb = csr_kernel_bytes(n, p, K, nS, e, nnz, nnzS) if sparse else kernel_bytes(n, p, K, nS, e, path)
    names = dict(KERNEL_NAMES[path])
    if (path == 2 and p <= 64 and p % 2 == 0 and K <= 10 and n >= 16384 and (e == 4 or K <= 9 or n <= 100000)
            and os.environ.get("SSN_NARROW_PATH") != "off"):
        # long gradient / product passes over a narrow matrix go through the vector-unit kernel (dense_narrow.hip)
        names[1] = "dense_narrow_kernel<GRAD>"
    if sparse and K == 1:
        # one weight column: full passes and the column-sorted product run with a lane per stored entry
        names[0] = "csr1_flat_kernel + csr1_rowwork_kernel<OBJ>"
        names[1] = "csr1_flat_kernel + csr1_rowwork_kernel<GRAD>"
        names[2] = "csc1_window_kernel + csc1_combine_kernel (n rows)"
        names[4] = "csc1_window_kernel + csc1_combine_kernel (|S| rows)"
    kern = {}
    for which in (0, 1, 2, 3, 4):
        reps = 20 if which < 3 else 200
        ctx.ssn_time_kernel(which, V[0] if which >= 3 else W, 3)
        ms = ctx.ssn_time_kernel(which, V[0] if which >= 3 else W, reps)
        if which == 3 and ctx.ssn_sampled_slices() > 0:
            # sampled product on a wide matrix: margins per (row block, feature slice), U formed by the second kernel
            sl = ctx.ssn_sampled_slices()
            out["sampled_slices"] = sl
            names[3], names[4] = "dense_zpart_kernel (|S| rows)", "dense_xtu_kernel<from partial margins> (|S| rows)"
            kb[3] = nS * p * e + 4 * nS + p * K * e + sl * nS * 16 * e
            kb[4] = nS * p * e + sl * nS * 16 * e + nS * K * e
        ent = {"kernel": names[which], "ms": ms}
        if kb[which] is not None:
            ent.update({"algorithmic_GB": kb[which] / 1e9, "GBps": kb[which] / ms / 1e6,
                        "frac": kb[which] / ms / 1e6 / HBM_PEAK_GBS})
        kern[which] = ent
    out["kernels"] = kern
    # plain streaming read of X (no arithmetic): what this chip delivers to a trivial kernel
    ctx.ssn_time_kernel(5, W, 3)
    ms = ctx.ssn_time_kernel(5, W, 20)
    sbytes = (nnz if sparse else n * p) * e
    out["stream_read"] = {"ms": ms, "GBps": sbytes / ms / 1e6, "frac": sbytes / ms / 1e6 / HBM_PEAK_GBS}
    # the product kernels on ALL rows (the FullNewton shape, |S| = n): the streaming data point of H_S v
    S_full = torch.arange(n, dtype=torch.int32, device=dev)
    ctx.ssn_hess_prepare(W, S_full)
    for _ in range(3):
        ctx.ssn_hess_apply(V[0], HV[0])
    torch.cuda.synchronize()
    a, z = ev(), ev()
    a.record()
    for _ in range(10):
        ctx.ssn_hess_apply(V[0], HV[0])
    z.record()
    torch.cuda.synchronize()
    ms_full = a.elapsed_time(z) / 10
    cbf = call_bytes(n, p, K, n, e, nnz, nnz)["hess_apply"]
    out["hess_apply_all_rows"] = {"ms": ms_full, "algorithmic_GB": cbf / 1e9, "GBps": cbf / ms_full / 1e6,
                                  "frac_of_hbm_peak": cbf / ms_full / 1e6 / HBM_PEAK_GBS}
    ctx.close()
    return out


def pmc_sequence(data, dtype_name):
    """Three launches of each hot kernel plus two calibration kernels of known traffic (read n*p*e bytes;
    read and write n*p*e bytes), for per-dispatch hardware counters."""
    import numpy as np
    import torch
    from paper_1802_09113_amd import synth
    from paper_1802_09113_amd.binding import Context
    tdt = torch.float64 if dtype_name == "f64" else torch.float32
    n, p, C, K, nS = data["n"], data["p"], data["C"], data["K"], data["nS"]
    labels = torch.from_numpy(data["labels"]).to("cuda:0")
    if data["layout"] == "csr":
        # calibration kernels: a streaming read of the values, and a copy of them
        X = torch.from_numpy(data["vals"]).to("cuda:0").to(tdt)
        csr = (torch.from_numpy(data["rowptr"].astype(np.int32)).to("cuda:0"), torch.from_numpy(data["colidx"]).to("cuda:0"), X)
        ctx = Context(labels, C, data["lam"], csr=csr, p=p)
    else:
        X = torch.from_numpy(data["X"]).to("cuda:0").to(tdt)
        ctx = Context(labels, C, data["lam"], X=X)
    W = torch.from_numpy(synth.probe(p, K, sub=1, scale=0.05)).to("cuda:0").to(tdt)
    V = torch.from_numpy(synth.probe(p, K, sub=2)).to("cuda:0").to(tdt)
    ctx.ssn_hess_prepare(W, torch.from_numpy(synth.sample_rows(n, nS)).to("cuda:0"))
    for which in (0, 1, 2, 3, 4, 5):
        ctx.ssn_time_kernel(which, V if which in (3, 4) else W, 3)
    Y = torch.empty_like(X)
    for _ in range(3):
        Y.copy_(X)
    torch.cuda.synchronize()
    ctx.close()


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return platform.processor() or "unknown"


def cpu_baseline(data):
    """The oracle as it stands on the GPU machine's host, on a bounded sample of the workload: the plain single-thread
    build, and the OpenMP build of the same source on all the cores the process is given.  Median of 3 repetitions
    of each call; gradient and objective on the first n/8 rows (scaled to n for the per-call figures)."""
    import numpy as np
    from oracle import oracle
    from oracle.oracle import Problem
    from paper_1802_09113_amd import synth
    n, nS = data["n"], data["nS"]
    sub = max(nS, n // 8)
    S = synth.sample_rows(n, nS)

    def problem(rows, threads):
        if data["layout"] == "csr":
            rp = data["rowptr"][: rows + 1]
            return Problem(data["labels"][:rows], data["C"], data["lam"], threads=threads, p=data["p"],
                           csr=(rp, data["colidx"][: rp[-1]], data["vals"][: rp[-1]]))
        return Problem(data["labels"][:rows], data["C"], data["lam"], X=data["X"][:rows], threads=threads)

    def med3(fn):
        ts = []
        for _ in range(3):
            t0 = time.perf_counter()
            fn()
            ts.append(time.perf_counter() - t0)
        return statistics.median(ts)

    legs = {}
    for name, threads in (("single_thread", False), ("all_cores", True)):
        full, part = problem(n, threads), problem(sub, threads)
        W = np.zeros((full.p, full.K))
        V = synth.probe(full.p, full.K, sub=10)
        t_hv = med3(lambda: full.hessvec(W, S, V))
        t_grad = med3(lambda: part.gradient(W)) * n / sub
        t_obj = med3(lambda: part.objective(W)) * n / sub
        legs[name] = {"cores": oracle.threads_of(threads), "hessvec_s": t_hv, "hv_per_s": 1.0 / t_hv,
                      "gradient_s_scaled_to_n": t_grad, "objective_s_scaled_to_n": t_obj,
                      # one SSN iteration = gradient + T products + one line-search trial (the usual case)
                      "ssn_iteration_s_estimate": t_grad + data["T"] * t_hv + t_obj}
    one = legs["single_thread"]
    return {"value": one["hv_per_s"], "unit": "Hess-vec products/s", "cores": 1, "kind": "oracle",
            "sample": f"median of 3: product H_S v on the workload's sample (|S|={nS} of n={n}, p={data['p']}, C={data['C']}) "
                      f"at W=0; gradient and objective on the first {sub} rows, scaled to n",
            "single_thread": one, "all_cores": legs["all_cores"],
            "nproc": os.cpu_count(), "cpu_model": _cpu_model(),
            "compiler": "gcc " + " ".join(oracle.CFLAGS) + " (no fast-math; all-cores build adds -fopenmp), fp64 with "
                        "long-double row sums"}


def summary(data, res, dtype):
    """The headline figures of one workload, for the list of the other workloads."""
    return {"workload": f"{data['name']}: {data['layout']} {data['n']}x{data['p']}, C={data['C']}, |S|={data['nS']}",
            "dtype": dtype, "hv_per_s": res["hv_per_s"], "hv_per_s_inside_cg": res["hv_per_s_inside_cg"],
            "ms_per_ssn_iteration": res["ms_per_step"], "calls": res["calls"],
            "hess_apply_all_rows": res["hess_apply_all_rows"], "stream_read": res["stream_read"],
            "kernels": {v["kernel"]: {kk: vv for kk, vv in v.items() if kk != "kernel"} for v in res["kernels"].values()}}


def kernel_roofline(data, dtype, k, which, note):
    ent = k[which]
    return {"bound": "hbm", "kernel": ent["kernel"], "achieved": ent["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ent["frac"], "traffic": measured_traffic(data["name"], dtype, ent["kernel"]),
            "ms_per_launch": ent["ms"], "algorithmic_bytes_per_launch": ent["algorithmic_GB"] * 1e9, "what": note}


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1\n")
        sys.exit(2)
    import torch
    from paper_1802_09113_amd import synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    t_gen = time.perf_counter()
    data = synth.make(args.config, n=args.n)
    sys.stderr.write(f"[bench] generated {data['name']} {data['n']}x{data['p']} C={data['C']} in "
                     f"{time.perf_counter() - t_gen:.1f}s\n")
    if args.pmc:
        pmc_sequence(data, args.dtype)
        return
    main_res = measure(data, args.dtype, args.steps, args.warmup, args.hv_calls)
    sys.stderr.write(f"[bench] {args.dtype} measured\n")
    other = None
    if not args.no_other_dtype:
        od = "f32" if args.dtype == "f64" else "f64"
        other = measure(data, od, args.steps, args.warmup, args.hv_calls)
        sys.stderr.write(f"[bench] {od} measured\n")
    cpu = None if args.no_cpu else cpu_baseline(data)
    sys.stderr.write("[bench] cpu baseline done\n")
    others = []
    if not args.no_other_workloads and args.n is None:
        for cfg in range(1, len(synth.CONFIGS)):
            if cfg == args.config:
                continue
            od = synth.make(cfg)
            others.append(summary(od, measure(od, args.dtype, min(args.steps, 5), min(args.warmup, 2), 100), args.dtype))
            sys.stderr.write(f"[bench] workload {od['name']} measured\n")
            del od

    # The roofline entry is the dominant STREAMING kernel of a step: the pass over all rows with the largest share
    # of the step's kernel time (gradient or objective; on the one-pass path the gradient kernel reads X once for
    # both products).  The sampled product runs on |S| rows that stay cache-resident between the products of an
    # iteration: its figure is reported beside it and is a latency figure, not an HBM stream.
    k = main_res["kernels"]
    per_step = {0: main_res["ls_evals_mean"] * k[0]["ms"], 1: k[1]["ms"], 2: k[2]["ms"],
                3: data["T"] * k[3]["ms"], 4: data["T"] * k[4]["ms"]}
    stream = max((w for w in (0, 1, 2) if "GBps" in k[w]), key=per_step.get)
    roof = kernel_roofline(data, args.dtype, k, stream,
                           "dominant streaming kernel of an SSN iteration (all n rows from HBM)")
    roof.update({"share_of_step_kernel_time": per_step[stream] / sum(per_step.values()),
                 "stream_read_GBps": main_res["stream_read"]["GBps"],
                 "frac_of_stream_read": k[stream]["GBps"] / main_res["stream_read"]["GBps"]})
    sampled = max((w for w in (3, 4) if "GBps" in k[w]), key=per_step.get)
    roof_sampled = kernel_roofline(data, args.dtype, k, sampled,
                                   "sampled product kernel: X_S is cache-resident after the first product of an iteration, "
                                   "so this is a latency figure, not an HBM stream")
    roof_sampled["share_of_step_kernel_time"] = per_step[sampled] / sum(per_step.values())
    line = {
        "metric": "sub-sampled Hess-vec products/s", "value": main_res["hv_per_s"], "unit": "products/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{data['name']}: {data['layout']} {data['n']}x{data['p']}"
                               + (f" nnz={data['nnz']}" if data["layout"] == "csr" else "")
                               + f", C={data['C']}, lambda={data['lam']}, "
                               f"|S|={data['nS']} (5%), CG T={data['T']}, theta=1e-4, Armijo beta=1e-4 rho=0.5; "
                               f"step = one SSN iteration", "config_index": args.config},
        "roofline": roof,
        "roofline_sampled_product": roof_sampled,
        "cpu_baseline": cpu,
        "time_per_ssn_iteration_ms": main_res["ms_per_step"],
        "hv_per_s_inside_cg": main_res["hv_per_s_inside_cg"],
        "phase_ms": main_res["phase_ms"],
        "phase_ms_note": "from a repeat of the timed steps with stream events on (ms_per_step_with_phase_events); "
                         "the line search phase holds the next iteration's gradient pass (look-ahead)",
        "ms_per_step_with_phase_events": main_res["ms_per_step_with_phase_events"],
        "calls": main_res["calls"],
        "dense_path": main_res["dense_path"],
        "stream_read": main_res["stream_read"],
        "hess_apply_all_rows": main_res["hess_apply_all_rows"],
        "kernels": {v["kernel"]: {kk: vv for kk, vv in v.items() if kk != "kernel"} for v in k.values()},
        "final_f": main_res["final_f"],
    }
    if other is not None:
        od = "f32" if args.dtype == "f64" else "f64"
        line["other_dtype"] = summary(data, other, od)
    if others:
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
