#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch: Lanczos with
full reorthogonalisation (m steps on the planted-spectrum operator), Ritz
extraction of the k largest / l smallest pairs, and one model update.  The
default workload is the ResNet-50-sized block: n = 25.6 M, r = 128, m = 80,
k = 20, l = 10, all inputs resident in HBM before the timed region.

Prints ONE JSON line: whole-step throughput in algorithmic GB/s (`value`), the
step time, a roofline entry for the dominant kernel (measured with HIP events
on the library's stream) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


REORTH_MODES = {"single": 1, "twice": 2, "local_full": 3, "selective": 4}


def algorithmic_vectors(m_eff: int, r: int, r_v: int, reorth: str, with_pi: bool, second_passes: int = 0) -> dict:
    """Vectors (4n bytes each) the variant that is run must move, per phase.
    Per Lanczos step with c = i+1 live columns: operator (r+1) + (r+2); a
    Gram-Schmidt pass against all columns (c+1) + (c+2) -- "single": once,
    "twice": two times; "local_full": the local pass rides on the operator's
    expand sweep (+1 vector, q_{i-1}, when i > 0), the full pass reads h, q_i and
    q_{i-1} to form its vector (c + 2 + [i > 0]) and one subtraction follows
    (c+2) that also normalises (the other schemes: a normalisation sweep, 2); "selective": a pass whose
    subtraction normalises, and in `second_passes` of the steps a second one (which steps is decided on the
    device: priced at the average pass).  Start vector 3.  Ritz vectors m_eff + r_v.  Update:
    3 sweeps of V-hat plus 7 vector accesses (+2 with a dual variable)."""
    hvp = m_eff * (2 * r + 3)
    if reorth == "local_full":
        hvp += max(0, m_eff - 1)

    def gs(c):
        full = 2 * c + 3
        if reorth == "local_full":
            return full + 1 + (1 if c > 1 else 0)
        return {"single": full, "twice": 2 * full, "selective": full}[reorth]
    reorth_name = reorth
    reorth = sum(gs(i + 1) for i in range(m_eff))
    if reorth_name == "selective" and m_eff > 0:
        reorth += round(reorth * second_passes / m_eff)
    norm = (0 if reorth_name in ("local_full", "selective") else 2 * m_eff) + 3   # those normalise inside the subtraction
    ritz = m_eff + r_v
    step = 3 * r_v + 7 + (2 if with_pi else 0)
    return dict(hvp=hvp, reorth=reorth, normalise=norm, ritz=ritz, step=step,
                total=hvp + reorth + norm + ritz + step)


def device_name(torch) -> str:
    """Marketing name if the driver's id table has one, else the architecture string (e.g. gfx950)."""
    name = torch.cuda.get_device_name(0)
    if not name:
        props = torch.cuda.get_device_properties(0)
        name = f"{getattr(props, 'gcnArchName', 'unknown arch')}, {props.multi_processor_count} CUs, " \
               f"{props.total_memory / 2**30:.0f} GiB"
    return name


def cpu_baseline(cfg_id: int, n_sample: int, fo=None, reorth: str = "local_full") -> dict:
    """The CPU oracle, as it stands, on a reduced-n copy of the same workload (host Philox generator) -- and, when
    the binding is handed in, the HIP path on exactly those host-generated inputs, uploaded, so that one row of the
    report times both sides on identical data.  Why a reduced n: the oracle's time is linear in n (about 6 us per
    row for m = 80 on 16 cores: ~10 s at 1.6 M rows, ~155 s and ~32 GB at the full 25.6 M), and the whole bench has
    to finish within minutes; 1/16 of the block keeps the leg inside the 10-30 s it is given."""
    import numpy as np

    import oracle
    import workloads as wl
    n_sample = min(int(n_sample), wl.CONFIGS[cfg_id]["n"])
    w = wl.planted_workload(cfg_id, n=n_sample)
    op = lambda v: oracle.hvp_planted(w.U, w.lam, float(w.shift), v)
    p = w.params
    g = w.grad(0)
    t0 = time.perf_counter()
    res = oracle.lanczos(op, w.v1, w.m)
    t1 = time.perf_counter()
    rz = oracle.ritz(res.Q, res.alpha, res.beta, res.m_eff, w.k, w.l)
    t2 = time.perf_counter()
    oracle.fosi_step(w.w0, g, rz.V, rz.evals, np.zeros(w.n), float(p.alpha), float(p.lr), float(p.momentum))
    t3 = time.perf_counter()
    dt = t3 - t0
    vecs = algorithmic_vectors(res.m_eff, w.r, w.k + w.l, "single", False)   # the oracle does one Gram-Schmidt pass
    gbs = vecs["total"] * 4.0 * n_sample / dt / 1e9
    try:
        from threadpoolctl import threadpool_info
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    frac = max(1, wl.CONFIGS[cfg_id]["n"] // n_sample)
    out = {"value": round(gbs, 3), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
           "sample": f"numpy fp64 oracle, same workload with n={n_sample} rows ("
                     + (f"1/{frac} of the block: the oracle's time is linear in n and the full block would take ~{frac}x this"
                        if frac > 1 else "the whole block") + f"), full m={w.m}, one "
                     f"Lanczos+Ritz+update pass, {dt:.1f} s; bytes counted as fp32 algorithmic traffic of its single-pass variant",
           "seconds": round(dt, 2),
           "phase_seconds": {"lanczos": round(t1 - t0, 2), "ritz": round(t2 - t1, 2), "step": round(t3 - t2, 3)}}
    if fo is not None:
        import torch
        ctx = fo.Context(0)
        ld = wl.padded_ld(w.n)
        U = fo.ColMajor.from_numpy(w.U, ld)
        hop = ctx.hvp_planted(U, torch.from_numpy(w.lam).cuda(), float(w.shift))
        Q, V = fo.ColMajor(w.n, w.m + 1, ld), fo.ColMajor(w.n, w.k + w.l, ld)
        v1, gd = torch.from_numpy(w.v1).cuda(), torch.from_numpy(g).cuda()
        sp = fo.StepParams(float(p.alpha), float(p.lr), float(p.momentum), float(p.sigma), 0)
        times = []
        for _ in range(4):                                   # first pass warms up; median of the rest
            wa, mom = torch.from_numpy(w.w0).cuda(), torch.zeros(w.n, device="cuda")
            Q.col(0).copy_(v1)
            torch.cuda.synchronize()
            s0 = time.perf_counter()
            alpha, beta, m_eff = fo.fosi_lanczos(ctx, hop, Q, w.m, reorth_mode=REORTH_MODES[reorth])
            evals, _ = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, w.k, w.l, V)
            fo.fosi_step(ctx, V, w.k + w.l, evals, gd, None, mom, wa, sp)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - s0)
        gpu_s = sorted(times[1:])[1]
        rel = float(np.max(np.abs(evals - rz.evals) / np.abs(rz.evals)))
        out["same_inputs"] = {"n": n_sample, "oracle_seconds": round(dt, 2), "gpu_ms": round(gpu_s * 1e3, 3),
                              "ratio": round(dt / gpu_s, 1),
                              "max_rel_diff_ritz_values": rel,
                              "note": "the HIP path on exactly the host-generated inputs the oracle was timed on (uploaded "
                                      "beforehand); same Lanczos+Ritz+update pass"}
        hop.close()
        ctx.close()
    return out


def bench_ggn(args, fo, torch, np) -> int:
    """Workloads 3 and 6: softmax-GGN operator (the MFMA path), Lanczos m = 60 + Ritz k = 20, no update.
    3: batch 512, fp32 data, fp32 matrix cores.  6: batch 8192, bf16 data, bf16 matrix cores with the fp32
    operand split in two bf16 parts (two matrix instructions per product)."""
    import workloads as wl
    bf16 = args.config == 6
    g = wl.ggn_workload(cfg_id=args.config)
    ctx = fo.Context(0)
    W = torch.from_numpy(g.W).cuda()
    if bf16:
        X = torch.from_numpy(g.X).cuda().to(torch.bfloat16).contiguous()
        op = ctx.hvp_softmax_ggn_bf16(X, W)
    else:
        X = torch.from_numpy(g.X).cuda()
        op = ctx.hvp_softmax_ggn(X, W)
    ld = wl.padded_ld(g.n)
    Q = fo.ColMajor(g.n, g.m + 1, ld)
    V = fo.ColMajor(g.n, g.k, ld)
    v1 = torch.from_numpy(g.v1).cuda()
    state = {}

    def one_step():
        Q.col(0).copy_(v1)
        alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, g.m, reorth_mode=REORTH_MODES[args.reorth],
                                             reorth_eta=args.reorth_eta)
        fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, g.k, 0, V)
        state["m_eff"] = m_eff

    for _ in range(args.warmup):
        one_step()
    # timed region: HIP events around the operator only (events around every kernel would add ~5 us of
    # stream time per event to a step of a few hundred short kernels)
    ctx.profile_enable("hvp_ggn")
    ctx.profile_reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    cnt, ms, flops = ctx.profile_read("hvp_ggn")
    tf = flops / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
    peak = 2500.0 if bf16 else 157.3
    # per-class breakdown from one more, untimed step with events around every kernel class
    ctx.profile_enable(True)
    ctx.profile_reset()
    one_step()
    ctx.profile_enable(False)
    phases = {"note": "one extra untimed step with events around every kernel class"}
    for name in ("hvp_ggn", "reorth_dot", "reorth_sub", "normalise", "ritz_vectors"):
        c, m_, by = ctx.profile_read(name)
        if c:
            phases[name] = {"launches": c, "ms_total": round(m_, 3), "avg_ms": round(m_ / c, 4)}
            if name != "hvp_ggn":
                phases[name]["GBps"] = round(by / (m_ * 1e-3) / 1e9, 1)
    out = {"metric": "Lanczos+Ritz on the softmax-GGN operator: step time (ms); MFMA TFLOP/s of the operator",
           "value": round(dt / args.steps * 1e3, 3), "unit": "ms", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 3), "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16 x2 (split fp32 operand), f32 accumulate" if bf16 else "f32",
           "data": "synthetic",
           "config": {"workload": f"cfg{args.config}: softmax-GGN, X {g.B}x{g.d}{' bf16' if bf16 else ''}, W {g.d}x{g.C} "
                                  f"(n={g.n}), Lanczos m={g.m}, k={g.k}", "m_eff": state["m_eff"]},
           "roofline": {"bound": "mfma",
                        "kernel": ("softmax-GGN apply (2 split-operand bf16-MFMA GEMMs + softmax Jacobian), whole apply; "
                                   "achieved counts the 4*B*d*C algorithmic flops, the matrix cores execute twice that")
                        if bf16 else "softmax-GGN apply (2 fp32-MFMA GEMMs + softmax Jacobian), whole apply",
                        "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4),
                        "traffic": None, "avg_launch_ms": round(ms / cnt, 4) if cnt else None,
                        "flops_per_apply": 4.0 * g.B * g.d * g.C},
           "phases": phases}
    print(json.dumps(out))
    op.close()
    ctx.close()
    return 0


def bench_blocks(args, fo, torch, np) -> int:
    """K independent parameter blocks of the chosen planted workload at once: one context per block, each on a
    stream of its own, each driven by a host thread (the per-layer blocks of the ADMM-like variant are
    independent problems).  Below a few million rows a single block is bound by the latency between its
    dependent kernels; blocks on separate streams fill those gaps.  Prints the aggregate rate."""
    import threading

    from workloads.device import planted_workload_device
    K = args.blocks
    blocks = []
    for _ in range(K):
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            w = planted_workload_device(args.config, args.n)
            if args.m is not None:
                w.m = args.m
            ctx = fo.Context(0, stream=stream)
            U = fo.ColMajor(w.n, w.r, w.ld, buf=w.U)
            op = ctx.hvp_planted(U, w.lam, w.shift)
            r_v = w.k + w.l
            b = dict(w=w, ctx=ctx, op=op, stream=stream, Q=fo.ColMajor(w.n, w.m + 1, w.ld), V=fo.ColMajor(w.n, r_v, w.ld),
                     wa=w.w0.clone(), mom=torch.zeros_like(w.w0), g=w.grad(0), m_eff=0,
                     pi=torch.zeros_like(w.w0) if w.admm else None, anchor=torch.zeros_like(w.w0) if w.admm else None)
            p = w.params
            b["sp"] = fo.StepParams(float(p.alpha), float(p.lr), float(p.momentum), float(p.sigma), 0)
        blocks.append(b)
    torch.cuda.synchronize()

    def run(b, steps):
        w, ctx = b["w"], b["ctx"]
        with torch.cuda.stream(b["stream"]):
            for _ in range(steps):
                b["Q"].col(0).copy_(w.v1)
                alpha, beta, m_eff = fo.fosi_lanczos(ctx, b["op"], b["Q"], w.m, reorth_mode=REORTH_MODES[args.reorth],
                                                     graph_mode=int(args.graph), reorth_eta=args.reorth_eta)
                evals, _ = fo.fosi_ritz(ctx, b["Q"], m_eff, alpha, beta, w.k, w.l, b["V"])
                if w.admm:
                    fo.fosi_admm_begin(ctx, b["sp"].sigma, b["pi"], b["anchor"], b["wa"])
                fo.fosi_step(ctx, b["V"], w.k + w.l, evals, b["g"], b["pi"], b["mom"], b["wa"], b["sp"])
                if w.admm:
                    fo.fosi_admm_end(ctx, b["sp"].sigma, b["anchor"], b["wa"], b["pi"])
                b["m_eff"] = m_eff

    def run_single_thread(steps):
        # one host thread: start every block's Lanczos run (nothing waits for the GPU), then collect them in turn
        for _ in range(steps):
            for b in blocks:
                with torch.cuda.stream(b["stream"]):
                    b["Q"].col(0).copy_(b["w"].v1)
                    fo.fosi_lanczos_begin(b["ctx"], b["op"], b["Q"], b["w"].m, reorth_mode=REORTH_MODES[args.reorth],
                                          graph_mode=int(args.graph), reorth_eta=args.reorth_eta)
            for b in blocks:
                w, ctx = b["w"], b["ctx"]
                with torch.cuda.stream(b["stream"]):
                    alpha, beta, m_eff = fo.fosi_lanczos_end(ctx, w.m)
                    evals, _ = fo.fosi_ritz(ctx, b["Q"], m_eff, alpha, beta, w.k, w.l, b["V"])
                    if w.admm:
                        fo.fosi_admm_begin(ctx, b["sp"].sigma, b["pi"], b["anchor"], b["wa"])
                    fo.fosi_step(ctx, b["V"], w.k + w.l, evals, b["g"], b["pi"], b["mom"], b["wa"], b["sp"])
                    if w.admm:
                        fo.fosi_admm_end(ctx, b["sp"].sigma, b["anchor"], b["wa"], b["pi"])
                    b["m_eff"] = m_eff

    def run_all(steps):
        if args.block_driver == "begin_end":
            run_single_thread(steps)
            torch.cuda.synchronize()
            return
        th = [threading.Thread(target=run, args=(b, steps)) for b in blocks]
        for t in th:
            t.start()
        for t in th:
            t.join()
        torch.cuda.synchronize()

    run_all(args.warmup)
    t0 = time.perf_counter()
    run_all(args.steps)
    dt = time.perf_counter() - t0
    w = blocks[0]["w"]
    vecs = algorithmic_vectors(blocks[0]["m_eff"], w.r, w.k + w.l, args.reorth, w.admm)
    if w.admm:
        vecs["total"] += 8
    step_bytes = vecs["total"] * 4.0 * w.n
    ms_per_step = dt / args.steps * 1e3
    value = K * step_bytes / (ms_per_step * 1e-3) / 1e9
    print(json.dumps({
        "metric": "Lanczos+FOSI step on K independent blocks at once: aggregate algorithmic HBM GB/s",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"cfg{args.config} x {K} blocks on {K} streams: planted spectrum n={w.n}, r={w.r}, "
                               f"Lanczos m={w.m} with '{args.reorth}' Gram-Schmidt, k={w.k}, l={w.l}, one update each",
                   "blocks": K, "driver": args.block_driver, "graph": bool(args.graph), "ms_per_block_step": round(ms_per_step / K, 3),
                   "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4)},
        "roofline": None}))
    for b in blocks:
        b["op"].close()
        b["ctx"].close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = n 25.6M headline; 2 = n 1M; 5 = n 125M; 3 = softmax-GGN batch 512 fp32; "
                         "6 = softmax-GGN batch 8192, bf16 data)")
    ap.add_argument("--n", type=int, default=None, help="override the row count (debugging)")
    ap.add_argument("--reorth", choices=sorted(REORTH_MODES), default="local_full",
                    help="Gram-Schmidt scheme of the Lanczos run (library default: local_full)")
    ap.add_argument("--reorth-eta", type=float, default=0.0,
                    help="threshold of the second pass of --reorth selective (0: the library's 1/sqrt 2)")
    ap.add_argument("--m", type=int, default=None, help="override the number of Lanczos steps")
    ap.add_argument("--accuracy", action="store_true",
                    help="also report max|Q^T Q - I| of the last Lanczos basis (library float64 matmuls, untimed)")
    ap.add_argument("--blocks", type=int, default=1,
                    help="run this many independent copies of a planted workload at once, one stream each (aggregate rate)")
    ap.add_argument("--block-driver", choices=["threads", "begin_end"], default="threads",
                    help="with --blocks: one host thread per block (blocking calls), or one thread that starts every "
                         "block's Lanczos run with fosi_lanczos_begin and collects them with fosi_lanczos_end")
    ap.add_argument("--graph", action="store_true",
                    help="with --blocks: replay each block's Lanczos run from a captured HIP graph (library option graph_mode)")
    ap.add_argument("--outer", action="store_true",
                    help="time whole outer iterations of Algorithm 3 instead of single-update steps: curvature refresh, "
                         "anchor, the workload's number of updates (10) with the dual variable and a fresh gradient each, "
                         "multiplier rule (workloads 2 and 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=1_600_000)
    ap.add_argument("--pmc-probe", action="store_true",
                    help="short run for hardware-counter collection: 3 plain copies of 1 GiB (calibration), then a "
                         "Lanczos run of 6 steps, Ritz vectors and one update on the chosen workload; no timing")
    ap.add_argument("--traffic-model", action="store_true",
                    help="instead of the timed steps: the library's memory-only sweep (fosi_traffic_model) on the chosen "
                         "workload's column counts -- Ritz vectors (m read, k + l written), an update sweep (k + l + 2 "
                         "read, 1 written), read-only and write-only -- beside the real kernels of one step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2505_00982_amd as fo
    if not os.path.exists(fo.library_path()):
        from paper_2505_00982_amd.build import build_library
        build_library(verbose=False)
    from workloads.device import planted_workload_device

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.config in (3, 6):
        return bench_ggn(args, fo, torch, np)
    if args.blocks > 1:
        return bench_blocks(args, fo, torch, np)
    w = planted_workload_device(args.config, args.n)
    if args.m is not None:
        w.m = args.m
    ctx = fo.Context(0)
    U = fo.ColMajor(w.n, w.r, w.ld, buf=w.U)
    op = ctx.hvp_planted(U, w.lam, w.shift)
    Q = fo.ColMajor(w.n, w.m + 1, w.ld)
    r_v = w.k + w.l
    V = fo.ColMajor(w.n, r_v, w.ld)
    wa = w.w0.clone()
    mom = torch.zeros_like(wa)
    pi = torch.zeros_like(wa) if w.admm else None
    anchor = torch.zeros_like(wa) if w.admm else None
    if args.outer and not w.admm:
        print("bench.py: --outer needs a workload with the ADMM-like rule (--config 2 or 5)", file=sys.stderr)
        return 2
    updates = w.steps if args.outer else 1
    grads = [w.grad(t) for t in range(updates)]     # resident before the timed region, one per update
    g = grads[0]
    p = w.params
    sp = fo.StepParams(float(p.alpha), float(p.lr), float(p.momentum), float(p.sigma), 0)
    state = {}

    def one_step():
        Q.col(0).copy_(w.v1)
        alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, w.m, reorth_mode=REORTH_MODES[args.reorth],
                                             reorth_eta=args.reorth_eta)
        state.update(second_passes=fo.fosi_lanczos_second_passes(ctx))
        evals, resid = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, w.k, w.l, V)
        if w.admm:
            fo.fosi_admm_begin(ctx, sp.sigma, pi, anchor, wa)
        for t in range(updates):
            fo.fosi_step(ctx, V, r_v, evals, grads[t], pi, mom, wa, sp)
        if w.admm:
            fo.fosi_admm_end(ctx, sp.sigma, anchor, wa, pi)
        state.update(m_eff=m_eff, evals=evals, resid=resid)

    if args.pmc_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)            # reads 1 GiB, writes 1 GiB: the counters' calibration point
        Q.col(0).copy_(w.v1)
        alpha, beta, m_eff = fo.fosi_lanczos(ctx, op, Q, 6, reorth_mode=REORTH_MODES[args.reorth])
        evals, _ = fo.fosi_ritz(ctx, Q, m_eff, alpha, beta, 3, 2, V)
        fo.fosi_step(ctx, V, r_v, np.linspace(10.0, 1.0, r_v), g, pi, mom, wa, sp)
        ctx.synchronize()
        print(json.dumps({"pmc_probe": "done", "n": w.n, "r": w.r, "copy_bytes_each_way": 4 << 28}))
        return 0

    if args.traffic_model:
        def phase(names):
            out = {}
            for name in names:
                c_, m_, b_ = ctx.profile_read(name)
                if c_:
                    out[name] = {"launches": c_, "avg_ms": round(m_ / c_, 4), "GBps": round(b_ / (m_ * 1e-3) / 1e9, 1)}
            return out
        one_step()                                           # warm-up, and real Ritz pairs for the update
        ctx.profile_enable(["ritz_vectors", "step_project", "step_complement", "step_apply"])
        ctx.profile_reset()
        one_step()
        kernels = phase(["ritz_vectors", "step_project", "step_complement", "step_apply"])
        ctx.profile_enable("traffic_model")
        m_e = state["m_eff"]
        cases = [("ritz_vectors: m read, k+l written", Q, m_e, V, r_v), ("update sweep: k+l+2 read, 1 written", Q, r_v + 2, V, 1),
                 ("read only, m columns", Q, m_e, None, 0), ("read only, r columns", U, w.r, None, 0),
                 ("write only, k+l columns", None, 0, V, r_v)]
        model = {}
        for label, A_, ci, B_, co in cases:
            for _ in range(2):
                fo.fosi_traffic_model(ctx, A_, ci, B_, co, w.n)
            ctx.profile_reset()
            for _ in range(5):
                fo.fosi_traffic_model(ctx, A_, ci, B_, co, w.n)
            c_, m_, b_ = ctx.profile_read("traffic_model")
            model[label] = {"cols_in": ci, "cols_out": co, "avg_ms": round(m_ / c_, 4), "GBps": round(b_ / (m_ * 1e-3) / 1e9, 1),
                            "frac_of_hbm_peak": round(b_ / (m_ * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        ctx.profile_enable(False)
        print(json.dumps({"traffic_model": model, "kernels_of_one_step": kernels, "unit": "algorithmic GB/s",
                          "workload": f"cfg{args.config}: n={w.n}, m={w.m}, k+l={r_v}, r={w.r}"}))
        return 0

    for _ in range(args.warmup):
        one_step()
    # Timed region: HIP events (on the library's stream) around the dominant kernel only -- the operator's expand
    # sweep (k_combine_columns<false,true,false,false,LDOT,...>: U, the current and, from the second Lanczos step
    # on in 'local_full' mode, the previous Lanczos vector, one store).  Events around every kernel would add
    # ~5 us of stream time per event, which matters for the small workloads.
    ctx.profile_enable("hvp_expand")
    ctx.profile_reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    cnt, ms, by = ctx.profile_read("hvp_expand")
    achieved = by / (ms * 1e-3) / 1e9 if ms > 0 else 0.0

    ms_per_step = dt / args.steps * 1e3
    vec_bytes = 4.0 * w.n
    vecs = algorithmic_vectors(state["m_eff"], w.r, r_v, args.reorth, w.admm, state["second_passes"])
    if w.admm:
        vecs["total"] += 8
    vecs["total"] += (updates - 1) * vecs["step"]
    step_bytes = vecs["total"] * vec_bytes
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # per-class breakdown from one more, untimed step with events around every kernel class
    ctx.profile_enable(True)
    ctx.profile_reset()
    one_step()
    ctx.profile_enable(False)
    phases = {"note": "one extra untimed step with events around every kernel class"}
    for name in ("hvp_project", "hvp_expand", "reorth_dot", "reorth_sub", "normalise", "ritz_vectors", "step", "admm"):
        c_, m_, b_ = ctx.profile_read(name)
        if c_:
            phases[name] = {"launches": c_, "ms_total": round(m_, 3), "avg_ms": round(m_ / c_, 4),
                            "GBps": round(b_ / (m_ * 1e-3) / 1e9, 1) if m_ > 0 else None}
    # the three sweeps of the update one by one (one more untimed update; the whole-update bracket above and these
    # three are alternatives inside the library)
    ctx.profile_enable(["step_project", "step_complement", "step_apply"])
    ctx.profile_reset()
    fo.fosi_step(ctx, V, r_v, state["evals"], g, pi, mom, wa, sp)
    for name in ("step_project", "step_complement", "step_apply"):
        c_, m_, b_ = ctx.profile_read(name)
        if c_:
            phases[name] = {"launches": c_, "ms_total": round(m_, 3), "avg_ms": round(m_ / c_, 4),
                            "GBps": round(b_ / (m_ * 1e-3) / 1e9, 1) if m_ > 0 else None}
    ctx.profile_enable(False)
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"hvp_expand_cfg{args.config}_pmc.txt")
    if os.path.exists(tfile) and args.n is None:
        for line in open(tfile):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                traffic = float(line.split("=", 1)[1])
    roofline = {"bound": "hbm", "kernel": "k_combine_columns<false,true,false,false,...> (planted operator, expand sweep)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": (f"profiles/hvp_expand_cfg{args.config}_pmc.txt: FETCH_SIZE and WRITE_SIZE of this kernel from two "
                                   "rocprofv3 --pmc runs of `bench.py --pmc-probe`, scaled by a 1 GiB copy; not measured in this run")
                if traffic is not None else None,
                "avg_launch_ms": round(ms / cnt, 4) if cnt else None,
                "algorithmic_bytes_per_launch": round(by / cnt) if cnt else None, "launches": cnt}

    out = {
        "metric": "Lanczos+FOSI step: achieved algorithmic HBM GB/s (step time in ms_per_step)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"cfg{args.config}: planted spectrum n={w.n}, r={w.r}, Lanczos m={w.m} with "
                               f"'{args.reorth}' Gram-Schmidt, k={w.k}, l={w.l}, "
                               + (f"one outer iteration of Algorithm 3 per step: curvature refresh, anchor, {updates} updates "
                                  f"with the dual variable and fresh gradients, multiplier rule" if args.outer else
                                  f"one update{' with ADMM begin/end' if w.admm else ''}"),
                   "accumulation": "f64 products and sums, one rounding per stored fp32 vector",
                   "m_eff": state["m_eff"], "algorithmic_GB_per_step": round(step_bytes / 1e9, 1),
                   **({"second_passes": state["second_passes"], "reorth_eta": args.reorth_eta or round(2 ** -0.5, 4)}
                      if args.reorth == "selective" else {}),
                   "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
                   "device": device_name(torch), "hip": getattr(torch.version, "hip", None)},
        "roofline": roofline,
        "phases": phases,
    }
    if args.accuracy:
        me = state["m_eff"]
        Qm = Q.buf[: me * w.ld].view(me, w.ld)
        gram = torch.zeros(me, me, dtype=torch.float64, device="cuda")
        for lo in range(0, w.n, 1 << 20):
            blk = Qm[:, lo:min(w.n, lo + (1 << 20))].double()
            gram += blk @ blk.T
        out["accuracy"] = {"max_abs_QtQ_minus_I": float((gram - torch.eye(me, dtype=torch.float64, device="cuda")).abs().max()),
                           "ritz_values": [float(x) for x in state["evals"]],
                           "ritz_residual_estimates": [float(x) for x in state["resid"]]}
    if not args.no_cpu_baseline:
        op.close()
        ctx.close()
        del U, Q, V, op, ctx
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(args.config, args.cpu_sample_rows, fo, args.reorth)
        print(json.dumps(out))
        return 0
    print(json.dumps(out))
    op.close()
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
