#!/usr/bin/env python3
"""Benchmark of the SLA hot path on one MI355X.

One step = sla_build_mask + sla_forward + sla_backward over one batch of the seeded synthetic
Wan-1.3B-shaped layer (bf16, 12 heads x 128, N = 32760 on a 21x30x52 grid, 64x64 blocks,
k_h = 5 %, k_l = 10 %), inputs resident in HBM.  Prints ONE JSON line: executed TFLOP/s on the
critical blocks over the whole step, ms per step, the roofline of the dominant kernel
(per-kernel durations from HIP events recorded on the launch stream inside the library), and
the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
from dataclasses import replace
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# algorithmic work of each kernel per launch, as a function of the workload's counts:
#   ("mfma", flops) for the contractions over critical pairs, ("hbm", bytes) for streaming kernels
def kernel_work(name, c):
    pair = c["pair_elems"] * c["d"]          # sum over critical pairs of r*c*d
    nd2 = c["BH"] * c["N"] * c["d"] * c["d"]
    table = {
        "forward": ("mfma", 4 * pair),              # S = Q K^T and P V per critical pair
        "fwd_sparse": ("mfma", 4 * pair),
        "bwd_sparse_kv": ("mfma", 8 * pair),        # S, dP, dV, dK
        "bwd_sparse_q": ("mfma", 2 * pair),         # dQ (S and dP are recomputed there)
        "bwd_query": ("mfma", 2 * pair),            # the same, preceded by the linear branch's query side
        "bwd_sparse": ("mfma", 10 * pair),
        # indicator GEMM: priced against whichever of its two floors is the higher one
        "aggregate": max(("mfma", 2 * c["BH"] * c["T"] * c["T"] * (c["d"] * c["d"] + c["d"])),
                         ("hbm", c["BH"] * c["T"] * (c["d"] * c["d"] + c["d"]) * 2 * c["esize"]),
                         key=lambda kw: kw[1] / (PEAK_BF16_TFLOPS * 1e12 if kw[0] == "mfma" else PEAK_HBM_GBS * 1e9)),
        "states": ("mfma", 2 * nd2),
        "pool": ("hbm", c["BH"] * c["N"] * c["d"] * c["esize"]),
    }
    return table.get(name)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="wan")
    ap.add_argument("--k-h", type=float, default=None)
    ap.add_argument("--k-l", type=float, default=None, help="fraction of negligible blocks (changes the density of the linear branch's marginal blocks)")
    ap.add_argument("--dense-steps", type=int, default=5, help="timed iterations of the dense reference run (after one warm-up); 0 skips it")
    ap.add_argument("--sub-runs", default="sweep,long",
                    help="bounded extra runs whose results ride in the same JSON line: 'sweep' = k_h 2.5 / 10 / 20 %% on the "
                         "same layer, 'long' = the 40-head N = 75600 layer; '' or 'none' skips them (default workload only)")
    ap.add_argument("--cpu-heads", type=int, default=4, help="0 skips the CPU oracle baseline")
    ap.add_argument("--settle-ms", type=float, default=200.0,
                    help="before the warm-up steps, run untimed steps for this long so that the GPU's clock "
                         "has left its idle state (a cold start runs the same kernels at about 1.6 instead of "
                         "2.0 GHz); 0 disables")
    ap.add_argument("--bq", type=int, default=64, help="query block size of the mask (64, 128, 192, 256)")
    ap.add_argument("--wide-query-tiles", action="store_true",
                    help="with --bq 128 / 256: the eight-wave kernels (one workgroup per pair of query tiles)")
    ap.add_argument("--agg-compare", action="store_true",
                    help="also time the accumulation line of Alg. 1 alone (random bf16 states, this workload's mask) "
                         "by the product the library uses and by the three forms the paper describes")
    ap.add_argument("--dq-atomics-probe", action="store_true",
                    help="also time the float atomics that accumulating dQ inside the column-wise backward kernel "
                         "would issue (one 64 x d tile per critical pair), next to the row-wise dQ kernel's time")
    ap.add_argument("--token-major", action="store_true",
                    help="hand the library [B,N,H,d] tensors (SLA_BNHD) instead of [B,H,N,d]")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="run one float add over this many MiB first: a kernel of known HBM traffic that "
                         "calibrates the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every step is per head, so heads would shard trivially); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2509_24006_amd import binding as sla
    from paper_2509_24006_amd import flops as fl
    from paper_2509_24006_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    w = wl.WORKLOADS[args.workload]
    if args.k_h is not None:
        w = wl.sweep(args.k_h) if args.workload == "wan" else w
    if args.k_l is not None:
        w = replace(w, name=f"{w.name}_kl{args.k_l:g}", k_l=args.k_l)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    t0 = time.time()
    x = wl.make_inputs(w)
    dev = {k: torch.from_numpy(v).to(tdt).cuda() for k, v in x.items()}
    if args.token_major:
        dev = {k: (v.transpose(1, 2).contiguous() if v.ndim == 4 else v) for k, v in dev.items()}
    Q, K, V, W, dO = dev["Q"], dev["K"], dev["V"], dev["Proj"], dev["dO"]
    t_gen = time.time() - t0

    lay = sla.SLA_BNHD if args.token_major else sla.SLA_BHND

    def buffers(p):
        z = sla.sla_sizes(p)
        u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda")
        return dict(z=z, Mc=torch.empty((p.B, p.H, z.Tq, z.T), dtype=torch.int8, device="cuda"),
                    luts=u8(z.luts_bytes), ws_m=u8(z.ws_mask_bytes), ws_f=u8(z.ws_forward_bytes),
                    ws_b=u8(z.ws_backward_bytes), saved=u8(z.saved_bytes), O=torch.empty_like(Q),
                    out=(torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V),
                         torch.empty((p.d, p.d), dtype=torch.float32, device="cuda")))

    def phases(p, b):
        def mask():
            sla.sla_build_mask(p, Q, K, workspace=b["ws_m"], Mc=b["Mc"], luts=b["luts"])
        def fwd():
            sla.sla_forward(p, Q, K, V, W, b["Mc"], b["luts"], O=b["O"], saved=b["saved"],
                            workspace=b["ws_f"])
        def bwd():
            sla.sla_backward(p, Q, K, V, W, b["Mc"], b["luts"], b["saved"], dO, workspace=b["ws_b"],
                             out=b["out"])
        return mask, fwd, bwd

    def timed_all(fn, n):
        """n iterations bracketed by synchronisations; one event between consecutive iterations.
        Returns (host ms per iteration, event ms per iteration over the whole region, per-iteration ms)."""
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        t = time.perf_counter()
        ev[0].record()
        for k in range(n):
            fn()
            ev[k + 1].record()
        torch.cuda.synchronize()
        host = (time.perf_counter() - t) * 1e3 / n
        return host, ev[0].elapsed_time(ev[n]) / n, [ev[k].elapsed_time(ev[k + 1]) for k in range(n)]

    def timed(fn, n):
        h, e, _ = timed_all(fn, n)
        return h, e

    def spread(per):
        return {"mean": float(np.mean(per)), "median": float(np.median(per)), "min": float(np.min(per)),
                "max": float(np.max(per))}

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)    # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    sla.sla_wide_query_tiles(args.wide_query_tiles)
    p = sla.make_params(w.B, w.H, w.N, w.d, w.k_h, w.k_l, tdt, layout=lay, bq=args.bq)
    b = buffers(p)
    mask, fwd, bwd = phases(p, b)

    def step():
        mask(); fwd(); bwd()

    settle_steps = 0
    if args.settle_ms > 0:
        t_end = time.perf_counter() + args.settle_ms * 1e-3
        while time.perf_counter() < t_end:
            step()
            torch.cuda.synchronize()
            settle_steps += 1
    for _ in range(args.warmup):
        step()
    ms_step, ms_step_ev, per_step = timed_all(step, args.steps)
    _, ms_mask, per_mask = timed_all(mask, args.steps)
    _, ms_fwd, per_fwd = timed_all(fwd, args.steps)
    _, ms_bwd, per_bwd = timed_all(bwd, args.steps)
    peak_measured = sla.sla_profile_mfma_peak(4096)

    # per-kernel durations (events inside the library, on the same stream)
    sla.sla_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = sla.sla_profile_read()
    sla.sla_profile_enable(False)
    kernels = {n: {"launches_per_step": c / args.steps, "ms_per_step": ms / args.steps,
                   "ms_per_launch": ms / c} for n, (c, ms) in prof.items()}

    Mc = b["Mc"].cpu().numpy()
    z = b["z"]
    f_fwd, f_bwd = fl.executed_flops(Mc, w.N, w.d, bq=args.bq)
    d_fwd, d_bwd = fl.dense_flops(w.B * w.H, w.N, w.d)
    counts = dict(pair_elems=fl.critical_pair_elems(Mc, w.N, bq=args.bq), d=w.d, BH=w.B * w.H, N=w.N, T=z.T,
                  esize=2 if w.dtype == "bf16" else 4)

    # roofline of the dominant kernel (largest share of the step)
    roof = None
    for name, k in sorted(kernels.items(), key=lambda kv: -kv[1]["ms_per_step"]):
        work = kernel_work(name, counts)
        if work is None:
            continue
        kind, amount = work
        sec = k["ms_per_launch"] * 1e-3
        if kind == "mfma":
            ach = amount / sec / 1e12
            roof = {"kernel": name, "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": None,
                    "ms_per_launch": k["ms_per_launch"]}
        else:
            ach = amount / sec / 1e9
            roof = {"kernel": name, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None,
                    "ms_per_launch": k["ms_per_launch"]}
        break

    # HBM traffic of that kernel per launch, from the committed counter summary (two rocprofv3 --pmc
    # runs of this command, FETCH_SIZE and WRITE_SIZE, scaled by the calibration kernel), if present
    if roof is not None and args.bq == 64:
        tpath = os.path.join(ROOT, "profiles", f"pmc_traffic_{roof['kernel']}_{w.name}.txt")
        if os.path.exists(tpath):
            src = {"file": os.path.relpath(tpath, ROOT)}
            for line in open(tpath):
                if line.startswith("traffic_bytes_per_launch:"):
                    roof["traffic"] = float(line.split(":")[1])
                if line.startswith("collected_at_commit:"):
                    src["collected_at_commit"] = line.split(":")[1].strip()
            roof["traffic_source"] = src
    if roof is not None:
        roof["peak_measured"] = peak_measured
        if roof["bound"] == "mfma":
            roof["frac_of_measured_peak"] = roof["achieved"] / peak_measured

    # dense reference on the same GPU: the same library with every block critical
    dense = None
    if args.dense_steps > 0 and w.k_h < 1.0:
        pd = sla.make_params(w.B, w.H, w.N, w.d, 1.0, 0.0, tdt, layout=lay)
        bd = buffers(pd)
        dm, df, db = phases(pd, bd)
        dm(); df(); db(); torch.cuda.synchronize()      # one warm-up iteration
        _, dfw, per_df = timed_all(df, args.dense_steps)
        _, dbw, per_db = timed_all(db, args.dense_steps)
        dense = {"iterations": args.dense_steps, "fwd_ms": dfw, "bwd_ms": dbw,
                 "fwd_ms_spread": spread(per_df), "bwd_ms_spread": spread(per_db),
                 "fwd_tflops": d_fwd / dfw / 1e9,
                 "bwd_tflops": d_bwd / dbw / 1e9, "speedup_fwd": dfw / ms_fwd,
                 "speedup_bwd": dbw / ms_bwd, "speedup_fwd_bwd": (dfw + dbw) / (ms_fwd + ms_bwd)}
        del bd

    # the accumulation line alone, by every method (same mask, random states: the time does not
    # depend on the values)
    agg = None
    if args.agg_compare and w.dtype == "bf16":
        hst = torch.randn((p.B, p.H, z.T, w.d * w.d + w.d), device="cuda").to(torch.bfloat16)
        agg = {}
        for method, name in ((sla.SLA_AGG_GEMM, "product"), (sla.SLA_AGG_ADD, "additions"),
                             (sla.SLA_AGG_PREAGG, "pre_aggregation"), (sla.SLA_AGG_FOUR_RUSSIANS, "four_russians")):
            need = sla.sla_aggregate_ws_bytes(p, method)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
            outb = sla.sla_aggregate_states(p, method, b["luts"], hst, workspace=ws)
            run = lambda: sla.sla_aggregate_states(p, method, b["luts"], hst, workspace=ws, out=outb)
            run(); torch.cuda.synchronize()
            agg[name] = {"ms": timed(run, 5)[1], "workspace_bytes": need}
            del ws, outb
        del hst

    atomics = None
    if args.dq_atomics_probe and args.bq == 64:
        accb = torch.zeros((p.B, p.H, p.N, p.d), dtype=torch.float32, device="cuda")
        sla.sla_profile_dq_atomics(p, b["luts"], accb)      # warm-up
        accb.zero_()
        ms_a = [sla.sla_profile_dq_atomics(p, b["luts"], accb) for _ in range(5)]
        ok = bool((accb[:, :, :, 0] == 5.0 * z.n_h).all().item())   # every row got n_h additions per launch
        atomics = {"ms": spread(ms_a), "adds_per_launch": w.B * w.H * w.N * z.n_h * w.d, "counts_ok": ok,
                   "bwd_sparse_q_ms": kernels.get("bwd_sparse_q", {}).get("ms_per_launch")}
        del accb

    # CPU oracle on a bounded sample: the first heads of the same workload, one thread per head
    cpu = None
    if args.cpu_heads > 0:
        from oracle import sla_oracle as orc
        hs = list(range(min(args.cpu_heads, w.H)))
        xs = {k: (v[:, hs] if v.ndim == 4 else v) for k, v in x.items()}
        os.environ.setdefault("OMP_NUM_THREADS", str(len(hs)))
        t = time.perf_counter()
        Mo = orc.build_mask(xs["Q"], xs["K"], w.k_h, w.k_l, bq=args.bq)
        fo = orc.forward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo, bq=args.bq, dtype=np.float32)
        orc.backward(xs["Q"], xs["K"], xs["V"], xs["Proj"], Mo, fo, xs["dO"], bq=args.bq, dtype=np.float32)
        sec = time.perf_counter() - t
        sf, sb = fl.executed_flops(Mo, w.N, w.d, bq=args.bq)
        cpu = {"value": (sf + sb) / sec / 1e12, "unit": "TFLOP/s", "cores": len(hs) * w.B,
               "kind": "oracle", "seconds": sec, "nproc": os.cpu_count(),
               "OMP_NUM_THREADS": os.environ.get("OMP_NUM_THREADS"),
               "sample": f"heads 0..{len(hs) - 1} of {w.H} (mask + forward + backward, float), "
                         f"one thread per head; full workload would take ~{sec * w.H / len(hs):.0f} s "
                         f"on {len(hs)} threads"}

    # bounded sub-runs on the other configurations (their own buffers; the default workload's are freed first)
    subs = [t for t in args.sub_runs.split(",") if t and t != "none"] if args.workload == "wan" and args.k_h is None else []
    sweep_res, long_res = None, None

    def sub_run(ws_, Qs, Ks, Vs, Ws, dOs, n_warm, n_steps):
        ps = sla.make_params(ws_.B, ws_.H, ws_.N, ws_.d, ws_.k_h, ws_.k_l, tdt)
        zs = sla.sla_sizes(ps)
        u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda")
        bs = dict(Mc=torch.empty((ps.B, ps.H, zs.Tq, zs.T), dtype=torch.int8, device="cuda"), luts=u8(zs.luts_bytes),
                  ws_m=u8(zs.ws_mask_bytes), ws_f=u8(zs.ws_forward_bytes), ws_b=u8(zs.ws_backward_bytes),
                  saved=u8(zs.saved_bytes), O=torch.empty_like(Qs),
                  out=(torch.empty_like(Qs), torch.empty_like(Ks), torch.empty_like(Vs),
                       torch.empty((ps.d, ps.d), dtype=torch.float32, device="cuda")))
        def m_(): sla.sla_build_mask(ps, Qs, Ks, workspace=bs["ws_m"], Mc=bs["Mc"], luts=bs["luts"])
        def f_(): sla.sla_forward(ps, Qs, Ks, Vs, Ws, bs["Mc"], bs["luts"], O=bs["O"], saved=bs["saved"], workspace=bs["ws_f"])
        def b_(): sla.sla_backward(ps, Qs, Ks, Vs, Ws, bs["Mc"], bs["luts"], bs["saved"], dOs, workspace=bs["ws_b"], out=bs["out"])
        def st_():
            m_(); f_(); b_()
        for _ in range(n_warm):
            st_()
        _, ms_s, per_s = timed_all(st_, n_steps)
        _, ms_f = timed(f_, n_steps)
        _, ms_b = timed(b_, n_steps)
        ff, fb = fl.executed_flops(bs["Mc"].cpu().numpy(), ws_.N, ws_.d)
        return {"k_h": ws_.k_h, "n_h": zs.n_h, "steps": n_steps, "ms_per_step": ms_s, "ms_per_step_spread": spread(per_s),
                "forward_ms": ms_f, "backward_ms": ms_b, "executed_tflop": (ff + fb) / 1e12,
                "tflops_step": (ff + fb) / ms_s / 1e9, "tflops_forward": ff / ms_f / 1e9,
                "tflops_backward": fb / ms_b / 1e9,
                "frac_of_bf16_peak_excl_mask": (ff + fb) / (ms_f + ms_b) / 1e9 / PEAK_BF16_TFLOPS}

    if "sweep" in subs and not args.token_major and args.bq == 64:
        sweep_res = {}
        for kh in (0.025, 0.10, 0.20):
            sweep_res[f"k_h={kh:g}"] = sub_run(wl.sweep(kh), Q, K, V, W, dO, 2, 5)
            if dense is not None:
                r_ = sweep_res[f"k_h={kh:g}"]
                r_["speedup_fwd_bwd_vs_dense"] = (dense["fwd_ms"] + dense["bwd_ms"]) / (r_["forward_ms"] + r_["backward_ms"])
    if "long" in subs:
        del b, Q, K, V, dO, dev
        torch.cuda.empty_cache()
        wlng = wl.WORKLOADS["long"]
        t1 = time.time()
        xl = wl.make_inputs(wlng)
        dl = {k: torch.from_numpy(v).to(tdt).cuda() for k, v in xl.items()}
        del xl
        long_res = sub_run(wlng, dl["Q"], dl["K"], dl["V"], dl["Proj"], dl["dO"], 1, 3)
        long_res["workload"] = f"long: B={wlng.B} H={wlng.H} d={wlng.d} N={wlng.N} grid={wlng.grid} k_h={wlng.k_h} k_l={wlng.k_l}"
        long_res["input_gen_s"] = time.time() - t1
        del dl

    out = {
        "metric": "SLA fwd+bwd executed TFLOPS on critical blocks (mask + forward + backward per step)",
        "value": (f_fwd + f_bwd) / (ms_step_ev * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step_ev,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} d={w.d} N={w.N} grid={w.grid} block={args.bq}x64 "
                               f"tensors={'[B,N,H,d]' if args.token_major else '[B,H,N,d]'} "
                               f"k_h={w.k_h} k_l={w.k_l} phi=softmax; n_h={z.n_h} n_l={z.n_l} "
                               f"n_0={z.n_0}; seeded Fourier-feature Q/K/V stand in for Wan2.1 activations"},
        "ms": {"step_wall": ms_step, "mask": ms_mask, "forward": ms_fwd, "backward": ms_bwd},
        "ms_spread": {"step": spread(per_step), "mask": spread(per_mask), "forward": spread(per_fwd),
                      "backward": spread(per_bwd)},
        "mfma_peak_tflops": {"nominal": PEAK_BF16_TFLOPS, "measured_register_only_loop": peak_measured},
        "executed_tflop": {"forward": f_fwd / 1e12, "backward": f_bwd / 1e12},
        "tflops": {"forward": f_fwd / ms_fwd / 1e9, "backward": f_bwd / ms_bwd / 1e9,
                   "fwd_bwd_excl_mask": (f_fwd + f_bwd) / (ms_fwd + ms_bwd) / 1e9,
                   "frac_of_bf16_peak_excl_mask": (f_fwd + f_bwd) / (ms_fwd + ms_bwd) / 1e9 / PEAK_BF16_TFLOPS,
                   "frac_of_measured_peak_excl_mask": (f_fwd + f_bwd) / (ms_fwd + ms_bwd) / 1e9 / peak_measured,
                   "paper_style_effective_fwd_bwd": (d_fwd + d_bwd) / (ms_fwd + ms_bwd) / 1e9},
        "dense_reference": dense,
        "sweep": sweep_res,
        "long": long_res,
        "kernels": kernels,
        "roofline": roof,
        "cpu_baseline": cpu,
        "settle_steps": settle_steps,
        "aggregation_methods": agg,
        "dq_atomics_probe": atomics,
        "input_gen_s": t_gen,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
