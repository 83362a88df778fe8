#!/usr/bin/env python3
"""Benchmark of the PACT token-reduction hot path on one MI355X.

One "step" = one pact_reduce (score -> prune -> DBDPC -> recovery -> merge) over one
synthetic LLaVA-OneVision-7B-shaped anyres image: N = 7290 tokens, hidden 3584, keys 512
(4 KV heads x 128), bf16, lambda = 0.45, d_c calibrated for ~71% total reduction.  Inputs,
outputs and workspace are resident in HBM before the timed region; the timed region is K
back-to-back calls bracketed by device synchronisation.

Prints ONE JSON line: whole-job images/s, ms per step, the roofline record of the dominant
kernel (per-kernel durations measured with HIP events recorded by the library on the launch
stream, in a separate pass right after the timed one), the bandwidth-bound stages with cold
caches first, the other workload shapes (a 729-token fp32 image, the same image with the
model's 28 query heads, 8 videos, 16 ragged images, a 16384-token video with fp32 keys, with
and without pruning), each with its density pass against the matrix-core peak and its merge
against the HBM peak, and the CPU oracle timed on this machine's host cores on the same image.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def algorithmic_work(kernel: str, n, h, dk, q, C, n_reinc, key_bytes, hid_bytes, out_bytes, n_q, d_h):
    """(bound, work, unit) of one launch of `kernel`: algorithmic flops or HBM bytes."""
    if kernel == "gram_density":          # unique pairs: q^2/2 dot products of length dk, 2 flops each
        return "mfma", float(q) * q * dk, "flop"
    if kernel == "gram_candidates":
        return "mfma", 2.0 * (n - q) * C * dk, "flop"
    if kernel == "qglobal_hnorm":         # read H once (norms) and the query partials, write norms and the global query
        return "hbm", n * h * hid_bytes + 512 * n_q * d_h * 8 + n * 8 + n_q * d_h * 8, "B"
    if kernel == "merge_mean":            # read member rows once, write C merged rows
        return "hbm", (q + n_reinc) * h * hid_bytes + C * h * out_bytes, "B"
    if kernel == "prep":                  # keys and queries read, the kept x kept bitmap cleared
        return "hbm", n * dk * key_bytes + n * n_q * d_h * key_bytes + q * ((q + 63) // 64) * 8, "B"
    return None, 0.0, ""


def _profile_table(name):
    """Rows `| kernel | a | b | ...` of a committed rocprofv3 summary under profiles/ -> {kernel: [cells]}."""
    path = os.path.join(ROOT, "profiles", name)
    rows = {}
    if os.path.exists(path):
        for ln in open(path):
            cells = [c.strip() for c in ln.strip().strip("|").split("|")]
            if len(cells) >= 3 and re.fullmatch(r"[a-z_]+", cells[0] or ""):
                rows[cells[0]] = cells[1:]
    return rows


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` (read + write) from the committed rocprofv3 --pmc summary."""
    cells = _profile_table("pact_reduce_img7b_hbm_traffic.md").get(kernel)
    try:
        return float(cells[0]) + float(cells[1])
    except (TypeError, ValueError, IndexError):
        return None


def rocprof_us(kernel: str):
    """Average duration of `kernel` in the committed rocprofv3 kernel trace of this command (us)."""
    cells = _profile_table("pact_reduce_img7b_kernel_stats.md").get(kernel)
    try:
        return float(cells[1])
    except (TypeError, ValueError, IndexError):
        return None


def kernel_times(P, torch, fn, steps):
    """us per call of every kernel (the library's event brackets), and launches per call."""
    P.pact_profile_enable(True)
    P.pact_profile_reset()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    recs = P.pact_profile_read(steps * 64)
    P.pact_profile_enable(False)
    tot, cnt = {}, {}
    for k, ms in recs:
        tot[k] = tot.get(k, 0.0) + ms
        cnt[k] = cnt.get(k, 0) + 1
    return {k: v / steps * 1e3 for k, v in tot.items()}, {k: c // steps for k, c in cnt.items()}


def other_configs(P, gen, torch, np, only=None, steps_override=None):
    """us per call of the other workload shapes (warm, back to back), with their counts, the
    algorithmic matrix-core fraction of their density pass and HBM fraction of their merge.
    only: run just that shape (for a profiler run of one shape), steps_override calls of it."""
    with open(os.path.join(ROOT, "pact_synth", "manifest.json")) as f:
        man = json.load(f)

    def dev(x, dt):
        t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        return t.to(torch.bfloat16) if dt == "bf16" else t

    def entry(sm):
        grids = sm.n // (sm.config.gh * sm.config.gw)
        heads = "" if sm.queries.shape[1] == sm.config.n_kv else f":q{sm.queries.shape[1]}"
        return man[f"{sm.config.name}:s{sm.seed}:g{grids}:l{sm.lam:.2f}{heads}"]

    def timeit(fn, steps):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e6

    def fractions(kus, reps, ns, h, dk):
        """density pass: unique pairs of all samples against the bf16 matrix-core peak (fp32 keys run on the
        bf16 instruction as three parts, six passes: their algorithmic flops are still q^2 dk); merge: member
        rows read + merged rows written against the HBM peak."""
        out = {}
        if "gram_density" in kus:
            fl = sum(float(r["n_kept"]) ** 2 * dk for r in reps)
            out["density_pass"] = {"us": round(kus["gram_density"], 1), "algorithmic_GFLOP": round(fl / 1e9, 2),
                                   "frac_of_bf16_mfma_peak": round(fl / (kus["gram_density"] * 1e-6) / 1e12 / PEAK_MFMA_TFLOPS["bf16"], 4)}
        if "merge_mean" in kus:
            by = sum((r["n_kept"] + r["n_reincorporated"]) * h * 2 + r["n_centers"] * h * 4 for r in reps)
            out["merge"] = {"us": round(kus["merge_mean"], 1), "algorithmic_MB": round(by / 1e6, 1),
                            "frac_of_hbm_peak": round(by / (kus["merge_mean"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)}
        return out

    out = {}
    singles = (("img_0p5b", dict(), 200), ("img_7b_q28", dict(n_q=28), 100), ("vid_long", dict(), 20),
               ("vid_long_lambda0", dict(lam=0.0), 10))
    for name, kw, steps in singles:
        if only is not None and name != only:
            continue
        steps = steps_override or steps
        base = {"img_7b_q28": "img_7b", "vid_long_lambda0": "vid_long"}.get(name, name)
        cfg = gen.CONFIGS[base]
        sm = gen.make_sample(cfg, 0, **kw)
        m = entry(sm)
        n_q = sm.queries.shape[1]
        hid = dev(sm.hidden, cfg.hidden_dtype)
        ks = dev(sm.keys.reshape(sm.n, -1), cfg.key_dtype)
        qs = dev(sm.queries.reshape(sm.n, -1), cfg.key_dtype)
        prm = P.PactParams(sm.lam, m["d_c"], 2.0, 1.5)
        ws = P.alloc_workspace(sm.n, 1, cfg.dk, n_q, cfg.d_h, key_dtype=ks.dtype)
        o = P.pact_reduce(hid, ks, ks, qs, cfg.n_kv, cfg.d_h, n_q, prm, ws=ws)
        call = lambda: P.pact_reduce(hid, ks, ks, qs, cfg.n_kv, cfg.d_h, n_q, prm, ws=ws, out=o)
        us = timeit(call, steps)
        r = P.read_report(o["rep"])
        assert r["n_kept"] == m["q"] and r["n_centers"] == m["C"], (name, r, m)
        kus, _ = kernel_times(P, torch, call, min(steps, 10))
        out[name] = {"n": sm.n, "batch": 1, "key_dtype": cfg.key_dtype, "query_heads": n_q, "lambda": sm.lam,
                     "us_per_call": round(us, 1), "samples_per_s": round(1e6 / us, 1), "q": r["n_kept"],
                     "C": r["n_centers"], "rho_rechecked": r["rho_rechecked"], **fractions(kus, [r], [sm.n], cfg.hidden, cfg.dk),
                     "kernels_us": {k: round(v, 1) for k, v in sorted(kus.items(), key=lambda kv: -kv[1])}}
        del hid, ks, qs, ws, o
    if only in (None, "img_7b_hidden_dbdpc"):
        # DBDPC alone on the hidden states of the benchmark image (the ablation that clusters hidden states
        # instead of keys): 7290 vectors of width 3584, nothing pruned
        sm = gen.make_sample("img_7b", 0)
        m = man["img_7b:s0:g10:hidden"]
        hid = dev(sm.hidden, "bf16")
        ws = P.alloc_workspace(sm.n, 1, sm.config.hidden, 1, 1, key_dtype=hid.dtype)
        o = P.dbdpc_cluster(hid, m["d_c"], 2.0, ws=ws)
        call = lambda: P.dbdpc_cluster(hid, m["d_c"], 2.0, ws=ws)
        us = timeit(call, steps_override or 50)
        r = P.read_report(o["rep"])
        assert r["n_centers"] == m["C"], (r, m)
        kus, _ = kernel_times(P, torch, call, 10)
        fl = float(sm.n) ** 2 * sm.config.hidden
        out["img_7b_hidden_dbdpc"] = {
            "n": sm.n, "width": sm.config.hidden, "us_per_call": round(us, 1), "C": r["n_centers"],
            "density_pass": {"us": round(kus["gram_density"], 1), "algorithmic_GFLOP": round(fl / 1e9, 1),
                             "frac_of_bf16_mfma_peak": round(fl / (kus["gram_density"] * 1e-6) / 1e12 / PEAK_MFMA_TFLOPS["bf16"], 4)},
            "kernels_us": {k: round(v, 1) for k, v in sorted(kus.items(), key=lambda kv: -kv[1])}}
        del hid, ws, o
    for name, make, steps in (("vid_7b_batch8", lambda: gen.make_batch("vid_7b", 0), 30),
                              ("varlen16", lambda: gen.make_varlen_batch(0), 30)):
        if only is not None and name != only:
            continue
        steps = steps_override or steps
        samples = make()
        cu = [0]
        for sm in samples:
            cu.append(cu[-1] + sm.n)
        cfg0 = samples[0].config
        hid = dev(np.concatenate([sm.hidden for sm in samples]), "bf16")
        ks = dev(np.concatenate([sm.keys.reshape(sm.n, -1) for sm in samples]), "bf16")
        qs = dev(np.concatenate([sm.queries.reshape(sm.n, -1) for sm in samples]), "bf16")
        prms = [P.PactParams(sm.lam, entry(sm)["d_c"], 2.0, 1.5) for sm in samples]
        exp = [(entry(sm)["q"], entry(sm)["C"]) for sm in samples]
        n_max = max(sm.n for sm in samples)
        ws = P.alloc_workspace(n_max, len(samples), cfg0.dk, cfg0.n_kv, cfg0.d_h, key_dtype=ks.dtype)
        o = P.pact_reduce_varlen(hid, ks, ks, qs, cfg0.n_kv, cfg0.d_h, cfg0.n_kv, cu, prms, ws=ws)
        call = lambda: P.pact_reduce_varlen(hid, ks, ks, qs, cfg0.n_kv, cfg0.d_h, cfg0.n_kv, cu, prms, ws=ws, out=o)
        us = timeit(call, steps)
        reps = P.read_report(o["rep"])
        assert [(r["n_kept"], r["n_centers"]) for r in reps] == exp, (name, reps, exp)
        kus, _ = kernel_times(P, torch, call, min(steps, 10))
        out[name] = {"n_total": cu[-1], "batch": len(samples), "us_per_call": round(us, 1),
                     "us_per_sample": round(us / len(samples), 1),
                     "samples_per_s": round(len(samples) * 1e6 / us, 1),
                     "rho_rechecked": sum(r["rho_rechecked"] for r in reps),
                     **fractions(kus, reps, [sm.n for sm in samples], cfg0.hidden, cfg0.dk),
                     "kernels_us": {k: round(v, 1) for k, v in sorted(kus.items(), key=lambda kv: -kv[1])}}
        del hid, ks, qs, ws, o
    return out


def cpu_baseline(s, d_c):
    """The oracle as it stands on this machine's host cores, on the benchmark image: once with every
    numerical library held to one thread, once with the threads they take by themselves."""
    from oracle import pact_oracle as po
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
    except Exception:
        threadpool_info, threadpool_limits = None, None

    def run(budget_s, max_reps):
        reps, t_cpu = 0, 0.0
        while reps < 2 or (t_cpu < budget_s and reps < max_reps):
            t1 = time.perf_counter()
            po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, d_c, 2.0, 1.5)
            t_cpu += time.perf_counter() - t1
            reps += 1
        return reps, t_cpu

    pool = max([i.get("num_threads", 1) for i in threadpool_info()] + [1]) if threadpool_info else 1
    reps_all, t_all = run(8.0, 30)
    one = None
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            reps_1, t_1 = run(10.0, 4)
        one = {"value": round(reps_1 / t_1, 4), "unit": "images/s", "cores": 1, "ms_per_step": round(t_1 / reps_1 * 1e3, 1),
               "sample": f"{reps_1} runs, every numerical library held to one thread"}
    return {"value": round(reps_all / t_all, 4), "unit": "images/s", "cores": pool, "kind": "oracle",
            "sample": f"{reps_all} runs of the fp64 numpy oracle's pact_reduce on the benchmark image (matmuls on the "
                      f"{pool} BLAS threads numpy takes by itself, the rest on one thread)",
            "ms_per_step": round(t_all / reps_all * 1e3, 1), "host_cpu_count": os.cpu_count(), "one_thread": one}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-table", action="store_true", help="print per-kernel averages to stderr")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache passes (profiling runs)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the other workload shapes (single image, 28 query heads, video batch, ragged batch, "
                         "long video); by default they are timed after the benchmark image and reported under other_configs")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also launch the library's plain copy kernel once over this many MiB "
                         "(a dispatch of known HBM traffic for rocprofv3 --pmc runs)")
    ap.add_argument("--only-config", choices=["img_0p5b", "img_7b_q28", "vid_long", "vid_long_lambda0", "img_7b_hidden_dbdpc",
                                              "vid_7b_batch8", "varlen16"], default=None,
                    help="run --steps calls of that workload shape alone and print its record (a profiler run of "
                         "one shape; the benchmark line is not printed)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (samples are independent and "
              "would be sharded one group per GPU, with no communication). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2504_08966_amd as P
    from pact_synth import gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    P.load_library()

    if args.only_config:
        rec = other_configs(P, gen, torch, np, only=args.only_config, steps_override=args.steps)
        print(json.dumps({"workload": args.only_config, **rec[args.only_config]}))
        return

    cfg = gen.CONFIGS["img_7b"]
    s = gen.make_sample(cfg, args.seed)
    with open(os.path.join(ROOT, "pact_synth", "manifest.json")) as f:
        man = json.load(f)[f"img_7b:s{args.seed}:g{cfg.grids}:l{cfg.lam:.2f}"]
    d_c = man["d_c"]
    n, h, dk = s.n, cfg.hidden, cfg.dk

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda().to(torch.bfloat16)

    hidden, keys, q = dev(s.hidden), dev(s.keys.reshape(n, -1)), dev(s.queries.reshape(n, -1))
    prm = P.PactParams(s.lam, d_c, 2.0, 1.5)
    ws = P.alloc_workspace(n, 1, dk, cfg.n_kv, cfg.d_h, key_dtype=keys.dtype)
    out = P.pact_reduce(hidden, keys, keys, q, cfg.n_kv, cfg.d_h, cfg.n_kv, prm, ws=ws)

    def step():
        P.pact_reduce(hidden, keys, keys, q, cfg.n_kv, cfg.d_h, cfg.n_kv, prm, ws=ws, out=out)

    if args.calibration_copy_mib > 0:
        src = torch.full((args.calibration_copy_mib << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        P.pact_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    rep = P.read_report(out["rep"])
    assert rep["n_kept"] == man["q"] and rep["n_centers"] == man["C"], (rep, man)

    # per-kernel durations: library-side HIP events on the launch stream, separate pass
    prof_steps = min(args.steps, 50)
    per_step_us, launches = kernel_times(P, torch, step, prof_steps)
    per_launch_us = {k: per_step_us[k] / max(launches[k], 1) for k in per_step_us}
    if args.kernel_table:
        for k in sorted(per_step_us, key=per_step_us.get, reverse=True):
            print(f"  {k:18s} {per_step_us[k]:9.2f} us/step  {launches[k]} launch(es)  {per_launch_us[k]:9.2f} us/launch",
                  file=sys.stderr)
        print(f"  sum of kernels      {sum(per_step_us.values()):9.2f} us/step; wall {ms_per_step * 1e3:.2f} us/step",
              file=sys.stderr)

    # distribution over steps (events on the launch stream around each step), warm and cold:
    # "cold" writes a 512 MiB scrub buffer between steps, so that neither the L2s nor the 256 MB
    # Infinity Cache still hold the inputs (the hidden states alone are 52 MB)
    # A second cold figure reads a 1 GiB buffer between steps instead: the caches then hold clean
    # lines of other data, and the step's reads do not compete with write-backs of the scrub.
    def step_times(n_steps, scrub):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_steps)]
        for a, b in evs:
            if scrub is not None:
                scrub()
            a.record()
            step()
            b.record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) * 1e3 for a, b in evs])      # us

    def cold_pass(scrub):
        us = step_times(dist_steps, scrub)

        def scrubbed_step():
            scrub()
            step()
        tab, cnt = kernel_times(P, torch, scrubbed_step, 30)
        return us, {k: tab[k] / max(cnt[k], 1) for k in tab}

    dist_steps = min(max(args.steps, 100), 300)
    warm_us = step_times(dist_steps, None)
    cold_us, cold_per_launch = None, {}
    coldr_us, coldr_per_launch = None, {}
    if not args.no_cold:
        buf = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
        cold_us, cold_per_launch = cold_pass(lambda: buf.fill_(1))
        del buf
        buf = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB, only ever read
        coldr_us, coldr_per_launch = cold_pass(lambda: torch.max(buf))
        del buf
    pct = lambda a: {"p10": round(float(np.percentile(a, 10)), 2), "p50": round(float(np.percentile(a, 50)), 2),
                     "p90": round(float(np.percentile(a, 90)), 2)}

    q_kept, C, n_re = rep["n_kept"], rep["n_centers"], rep["n_reincorporated"]
    roof = None
    for k in sorted(per_step_us, key=per_step_us.get, reverse=True):
        bound, work, unit = algorithmic_work(k, n, h, dk, q_kept, C, n_re, 2, 2, 4, cfg.n_kv, cfg.d_h)
        if bound is None:
            continue
        sec = per_launch_us[k] * 1e-6
        if bound == "mfma":
            ach, peak, u = work / sec / 1e12, PEAK_MFMA_TFLOPS["bf16"], "TFLOP/s"
        else:
            ach, peak, u = work / sec / 1e9, PEAK_HBM_GBS, "GB/s"
        roof = {"kernel": k, "bound": bound, "achieved": round(ach, 3), "peak": peak, "unit": u,
                "frac": round(ach / peak, 4), "traffic": measured_traffic(k), "us_per_launch": round(sec * 1e6, 2),
                "work_per_launch": work, "work_unit": unit,
                "share_of_step": round(per_step_us[k] / sum(per_step_us.values()), 3)}
        # the same kernel's average in the committed rocprofv3 kernel trace (begin/end timestamps; the event
        # brackets above include the dispatch overhead inside the bracket, about 2.5 us)
        rp = rocprof_us(k)
        if rp:
            roof["us_per_launch_rocprof"] = rp
            roof["frac_rocprof"] = round(work / (rp * 1e-6) / (1e12 if bound == "mfma" else 1e9) / peak, 4)
        if k == "gram_density":
            # the kernel computes the full (symmetric) matrix: executed flops are twice the algorithmic ones
            roof["executed_flop_per_launch"] = 2.0 * work
            roof["frac_executed"] = round(2.0 * ach / peak, 4)
        break

    # the bandwidth-bound stages: cold first (nothing of the inputs in any cache), then warm (inputs still in the
    # caches from the previous step)
    hbm_stages = {}
    for k in ("qglobal_hnorm", "merge_mean", "prep"):
        bound, work, unit = algorithmic_work(k, n, h, dk, q_kept, C, n_re, 2, 2, 4, cfg.n_kv, cfg.d_h)
        if k not in per_launch_us:
            continue
        ent = {"bytes_algorithmic": work, "traffic_measured": measured_traffic(k)}
        for tag, tbl in (("cold", cold_per_launch), ("cold_read_scrub", coldr_per_launch), ("warm", per_launch_us)):
            if k in tbl:
                gbs = work / (tbl[k] * 1e-6) / 1e9
                ent[tag] = {"us": round(tbl[k], 2), "GB/s": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4)}
        hbm_stages[k] = ent

    # what a plain copy reaches on this machine (the library's copy kernel; bytes read + bytes written per
    # second): the yardstick for stages that read and write, next to the 8 TB/s data-sheet peak
    hbm_reference = {}
    for mib in (32, 256):
        src = torch.full((mib << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            P.pact_calibration_copy(dst, src)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(20):
            P.pact_calibration_copy(dst, src)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t1) / 20 * 1e6
        hbm_reference[f"copy_{mib}MiB"] = {"us": round(us, 1), "GB/s_moved": round(2 * (mib << 20) / us / 1e3, 1)}
        del src, dst
    for k, ent in hbm_stages.items():
        ref = hbm_reference["copy_32MiB"]["GB/s_moved"]
        for tag in ("cold", "cold_read_scrub", "warm"):
            if tag in ent:
                ent[tag]["frac_of_copy_rate"] = round(ent[tag]["GB/s"] / ref, 4)

    cpu = None if args.no_cpu_baseline else cpu_baseline(s, d_c)

    line = {
        "metric": "images/sec per pact_reduce at N=7290, Dk=512", "value": round(args.steps / dt, 2),
        "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "us_per_pact_reduce": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "LLaVA-OV-7B-shaped anyres image, N=7290 (10x729), H=3584, Dk=512 (4x128) bf16, "
                               "lambda=0.45, d_n=2, alpha=1.5, d_c=%.6f (71%% reduction), batch 1" % d_c,
                   "seed": args.seed, "q": q_kept, "C": C, "n_reincorporated": n_re, "launches_per_call": sum(launches.values()),
                   "rounds": rep["rounds"], "dc_checked_pairs": rep["dc_checked_pairs"], "dc_near_ties": rep["dc_near_ties"],
                   "rho_rechecked": rep["rho_rechecked"], "rho_near_ties": rep["rho_near_ties"],
                   "score_near_ties": rep["score_near_ties"], "nonfinite_seen": rep["nonfinite_seen"],
                   "refine_overflow": rep["refine_overflow"]},
        "roofline": roof,
        "cpu_baseline": cpu,
        "us_per_step_cold": pct(cold_us) if cold_us is not None else None,
        "us_per_step_cold_read_scrub": pct(coldr_us) if coldr_us is not None else None,
        "us_per_step_warm": pct(warm_us),
        "hbm_stages": hbm_stages,
        "hbm_reference": hbm_reference,
        "kernels_us_per_step": {k: round(v, 2) for k, v in sorted(per_step_us.items(), key=lambda kv: -kv[1])},
        "kernels_us_per_step_cold": {k: round(v, 2) for k, v in sorted(cold_per_launch.items(), key=lambda kv: -kv[1])},
        "kernels_us_per_step_cold_read_scrub": {k: round(v, 2) for k, v in sorted(coldr_per_launch.items(), key=lambda kv: -kv[1])},
    }
    if not args.no_other_configs:
        line["other_configs"] = other_configs(P, gen, torch, np)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
