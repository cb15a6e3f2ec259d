#!/usr/bin/env python3
"""Benchmark of the Dion step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4a] [--no-cpu-baseline]

A "step" is one full Dion step (Z = (M+G)Q, CholeskyQR2, R = (M+G)^T P, ColNorm, fused M and X
update) of the workload's matrices, inputs resident in HBM.  Prints ONE JSON line: ms per step as
`value`, the roofline of the dominant kernel (stage durations from HIP events recorded by the
library on the step's stream) and the CPU oracle timed on the host cores as `cpu_baseline`.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2504_05295_amd import inputs  # noqa: E402

PEAK_BF16 = 2.5e15   # dense bf16 MFMA FLOP/s
PEAK_F32 = 157.3e12  # fp32 MFMA FLOP/s
PEAK_HBM = 8.0e12    # B/s

WORKLOAD_NAMES = {
    "C1": "C1: 256x256 r=64, fp32 G, fp32 math",
    "C2": "C2: 2048x2048 r=512, bf16 G, fp32 math",
    "C2b": "C2: 2048x2048 r=512, bf16 G, bf16 operands",
    "C3a": "C3: 8192x8192 r=2048, bf16 G, bf16 operands, fp32 state",
    "C3b": "C3: 8192x8192 r=512, bf16 G, bf16 operands, fp32 state",
    "C4a": "C4: 16384x53248 r=1024 (Llama-3-405B MLP shape), bf16 G, bf16 operands",
    "C4b": "C4: 16384x53248 r=4096 (Llama-3-405B MLP shape), bf16 G, bf16 operands",
    "C5": "C5: 196 matrices of a 3B decoder (28 layers, d=3072, ffn=8192), r=768, batched",
}


PROFILE_TAGS = {"C3a": "C3_8192x8192_r2048", "C3b": "C3_8192x8192_r512", "C4a": "C4_16384x53248_r1024",
                "C4b": "C4_16384x53248_r4096", "C5": "C5_3B_decoder_196", "C2b": "C2_2048x2048_r512"}


def measured_traffic(workload):
    """HBM-side bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, calibrated against
    a plain copy), as recorded in the committed summary of this workload; {} if there is none."""
    tag = PROFILE_TAGS.get(workload)
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % tag) if tag else None
    out = {}
    if path and os.path.exists(path):
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch":
                out[f[1]] = float(f[2])
    return out


def kernel_models(shapes, g_bytes, math):
    """Algorithmic FLOPs and HBM bytes of the three large kernels, summed over the workload."""
    peak = PEAK_BF16 if math == "bf16" else PEAK_F32
    out = {}
    k1f = k1b = k2f = k2b = k5f = k5b = 0.0
    for (m, n, r) in shapes:
        mn, mr, nr = float(m) * n, float(m) * r, float(n) * r
        k1f += 2 * mn * r
        k1b += (4 + g_bytes) * mn + 4 * nr + 4 * mr            # read M, G, Q; write Z
        k2f += 2 * mn * r
        k2b += (4 + g_bytes) * mn + 4 * mr + 4 * nr            # read M, G, P; write R
        k5f += 4 * mn * r
        k5b += (16 + g_bytes) * mn + 4 * mr + 8 * nr           # read M, G, X; write M, X; read P, R, Q
    for name, fl, by in (("k1_BQ", k1f, k1b), ("k2_BtP", k2f, k2b), ("k5_update", k5f, k5b)):
        bound = "mfma" if fl / peak > by / PEAK_HBM else "hbm"
        out[name] = dict(flops=fl, bytes=by, bound=bound, peak=peak if bound == "mfma" else PEAK_HBM)
    # Orthonormalisation (CholeskyQR2): two Gram matrices without symmetry (4 m r^2), two triangular solves
    # (2 m r^2), two Cholesky factorisations (2/3 r^3); about five passes over the m x r factor.  Its products want
    # fp32 accuracy.  In fp32 mode they run on the fp32 matrix pipe and are priced against its peak; in bf16 mode the
    # library runs each as three bf16 products of split operands (x = hi + lo), so the same FLOP count is priced
    # against a third of the bf16 peak, with the fraction of the fp32 peak stated beside it (`vs_fp32_mfma`: it can
    # exceed 1, the split products being faster than the fp32 pipe, and the second pass being cut short when the
    # first one's result is orthonormal to 1e-3).
    of = ob = 0.0
    for (m, n, r) in shapes:
        of += 6.0 * m * r * r + 2.0 / 3.0 * float(r) ** 3
        ob += 20.0 * m * r
    out["orth"] = dict(flops=of, bytes=ob, bound="mfma", peak=PEAK_BF16 / 3.0 if math == "bf16" else PEAK_F32, f32_peak=PEAK_F32)
    return out


_HOST_CACHE = {}   # (m, n, g_bf16, n_grads) -> (X, [G_t]) host draws of the last shape built


def build_problem(cfg, seed=0, n_grads=2, form="standard"):
    import torch
    from paper_2504_05295_amd import binding as B
    shapes = cfg["shapes"]
    dev = "cuda"
    X, M, Q, G = [], [], [], []
    uniq = {}
    cache = _HOST_CACHE if seed == 0 else {}
    forms = [B.DION_FORM_TRANSPOSED if (form == "transposed" or (form == "short-side" and n < m)) else B.DION_FORM_STANDARD
             for (m, n, r) in shapes]
    for i, (m, n, r) in enumerate(shapes):
        # one host draw per distinct shape is enough for timing; every matrix still gets its own buffers
        if (m, n, r) not in uniq:
            key = (m, n, cfg["g_bf16"], n_grads)
            if key not in cache:
                cache.clear()      # one shape's draws at a time: the large ones take gigabytes of host memory
                cache[key] = (inputs.weight(m, n, seed + 1, 0),
                              [inputs.gradient(m, n, t, seed, 0, bf16=cfg["g_bf16"]) for t in range(n_grads)])
            uniq[(m, n, r)] = (cache[key][0], inputs.right_factor_raw(n, r, seed + 2, 0), cache[key][1])
        x, q, gs = uniq[(m, n, r)]
        X.append(torch.from_numpy(x).to(dev))
        M.append(torch.empty((m, n), dtype=torch.float32, device=dev))
        if forms[i] == B.DION_FORM_TRANSPOSED:
            q = inputs.right_factor_raw(m, r, seed + 2, 0)
        Q.append(torch.from_numpy(q).to(dev))
        if cfg["g_bf16"]:
            G.append([torch.from_numpy(g.view(np.int16)).view(torch.bfloat16).to(dev) for g in gs])
        else:
            G.append([torch.from_numpy(g).to(dev) for g in gs])
    state = B.dion_init_state(shapes, B.DION_G_BF16 if cfg["g_bf16"] else B.DION_G_F32,
                              B.DION_MATH_BF16 if cfg["math"] == "bf16" else B.DION_MATH_F32, M, Q, q_is_filled=True,
                              forms=None if form == "standard" else forms)
    return dict(B=B, shapes=shapes, X=X, M=M, Q=Q, G=G, state=state, uniq=uniq)


def do_step(p, t):
    B = p["B"]
    ng = len(p["G"][0])
    if p.get("variant") == "lazy":
        refresh = t % p["refresh_every"] == 0
        if len(p["shapes"]) == 1:
            B.dion_lazy_step(p["state"], p["X"][0], p["G"][0][t % ng], p["M"][0], p["Q"][0], inputs.MU, inputs.ETA, refresh)
        else:
            B.dion_lazy_step_batched(p["state"], p["X"], [g[t % ng] for g in p["G"]], p["M"], p["Q"], inputs.MU, inputs.ETA,
                                     refresh)
    elif len(p["shapes"]) == 1:
        B.dion_step(p["state"], p["X"][0], p["G"][0][t % ng], p["M"][0], p["Q"][0], inputs.MU, inputs.ETA)
    else:
        B.dion_step_batched(p["state"], p["X"], [g[t % ng] for g in p["G"]], p["M"], p["Q"], inputs.MU, inputs.ETA)


def cpu_baseline(cfg, p, budget_s=30.0, variant="dion", refresh_every=1):
    """Times the CPU oracle (as it stands, fp64 numpy) on a bounded sample of the workload."""
    from oracle import dion_oracle as orc
    shapes = cfg["shapes"]
    # sample: one step of the largest-work distinct matrix that fits the budget, else one smaller square matrix
    (m, n, r) = max(set(shapes), key=lambda s: s[0] * s[1] * s[2])
    est = (8.0 * m * n * r + 4.0 * m * r * r) / 1.5e11
    sample = "one full oracle step of %dx%d r=%d" % (m, n, r)
    scale = 1.0
    if est > budget_s:
        m2 = n2 = 4096
        r2 = max(1, int(round(4096 * r / min(m, n))))
        scale = (8.0 * m * n * r + 4.0 * m * r * r) / (8.0 * m2 * n2 * r2 + 4.0 * m2 * r2 * r2)
        sample = "one oracle step of %dx%d r=%d, scaled by FLOP count (x%.1f) to %dx%d r=%d" % (m2, n2, r2, scale, m, n, r)
        x = inputs.weight(m2, n2, 1, 0)
        q = inputs.right_factor_raw(n2, r2, 2, 0)
        g = inputs.gradient(m2, n2, 0, 0, 0, bf16=cfg["g_bf16"])
    else:
        x, q, gs = p["uniq"][(m, n, r)]
        g = gs[0]
    g32 = inputs.bf16_bits_to_f32(g) if cfg["g_bf16"] else g
    M0, Q0 = orc.init_state(x.shape[0], x.shape[1], q)
    # repeat the step (state carried on) until about 10 s of CPU work have been measured
    X0, steps_done, t0 = x, 0, time.perf_counter()
    while True:
        if variant == "lazy":
            res = orc.lazy_dion_step(X0, g32, M0, Q0, inputs.MU, inputs.ETA, steps_done % refresh_every == 0, method="lapack")
            assert res["status"] == 0
            X0, M0, Q0 = res["X"], res["M"], res["V"]
        else:
            res = orc.dion_step(X0, g32, M0, Q0, inputs.MU, inputs.ETA, method="lapack")
            assert res["status"] == 0
            X0, M0, Q0 = res["X"], res["M"], res["Q"]
        steps_done += 1
        dt = time.perf_counter() - t0
        if (dt >= 10.0 and steps_done % refresh_every == 0) or steps_done >= 400 * refresh_every:
            break
    sample += " (%d step%s timed)" % (steps_done, "" if steps_done == 1 else "s")
    dt /= steps_done
    per_matrix_ms = dt * 1e3 * scale
    # whole workload: every matrix costs the same FLOP-scaled time
    total = 0.0
    ref = 8.0 * m * n * r + 4.0 * m * r * r
    for (a, b, c) in shapes:
        total += per_matrix_ms * (8.0 * a * b * c + 4.0 * a * c * c) / ref
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS") or os.environ.get("OPENBLAS_NUM_THREADS")
    if env:
        cores = min(cores, int(env))
    return dict(value=total, unit="ms/step", cores=cores, kind="oracle", sample=sample, measured_s=dt * steps_done)


def run_workload(tag, steps, warmup, stage_timing=True, variant="dion", refresh_every=1, form="standard",
                 calibration_copy=False, orth_mode=0):
    """Builds the workload, runs `warmup` untimed and exactly `steps` timed steps (inputs resident in HBM, host clock
    bracketed by device synchronisations).  Returns the problem, ms per step and the per-stage ms."""
    import torch
    cfg = inputs.CONFIGS[tag]
    p = build_problem(cfg, form=form)
    p["variant"], p["refresh_every"] = variant, max(1, refresh_every)
    B = p["B"]
    if orth_mode:
        B.dion_set_orth_mode(p["state"], orth_mode)
    for t in range(warmup):
        do_step(p, t)
    status, bad = B.dion_last_status(p["state"])
    assert status == 0, "warm-up step of %s reported numerical status %d" % (tag, status)
    if calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    B.dion_set_stage_timing(p["state"], stage_timing)
    stage_sum = {k: 0.0 for k in B.STAGES}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if not stage_timing:
        for t in range(steps):
            do_step(p, warmup + t)
    else:
        # stage events are read back after each step (a host wait, also inside the timed region)
        for t in range(steps):
            do_step(p, warmup + t)
            for k, v in B.dion_stage_times(p["state"]).items():
                stage_sum[k] += v
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    status, bad = B.dion_last_status(p["state"])
    assert status == 0, "timed step of %s reported numerical status %d" % (tag, status)
    return p, (t1 - t0) * 1e3 / steps, {k: v / steps for k, v in stage_sum.items()}


def stage_rooflines(tag, stages, ceilings):
    """Achieved rate of every stage against its bound, from the algorithmic FLOPs / bytes of kernel_models."""
    cfg = inputs.CONFIGS[tag]
    models = kernel_models(cfg["shapes"], 2 if cfg["g_bf16"] else 4, cfg["math"])
    traffic = measured_traffic(tag)
    tsrc = "profiles/hbm_traffic_%s.txt" % PROFILE_TAGS[tag] if traffic else None
    out = {}
    for name, mdl in models.items():
        ms = stages.get(name, 0.0)
        if ms <= 0:
            continue
        work = mdl["flops"] if mdl["bound"] == "mfma" else mdl["bytes"]
        ach = work / (ms * 1e-3)
        unit = "TFLOP/s" if mdl["bound"] == "mfma" else "GB/s"
        div = 1e12 if mdl["bound"] == "mfma" else 1e9
        rf = dict(bound=mdl["bound"], achieved=ach / div, peak=mdl["peak"] / div, unit=unit, frac=ach / mdl["peak"],
                  traffic=traffic.get(name), traffic_source=tsrc if traffic.get(name) is not None else None, ms=ms,
                  tflops=mdl["flops"] / (ms * 1e-3) / 1e12, gbps=mdl["bytes"] / (ms * 1e-3) / 1e9)
        if name == "orth":
            rf["peak_of"] = "fp32 MFMA" if mdl["peak"] == mdl["f32_peak"] else "bf16 MFMA / 3 (three split-bf16 products per fp32 product)"
            rf["vs_fp32_mfma"] = dict(peak=mdl["f32_peak"] / 1e12, unit="TFLOP/s", frac=ach / mdl["f32_peak"])
        elif ceilings:
            top = ceilings["mfma_tflops"] if rf["bound"] == "mfma" else ceilings["stream_gbps"]
            rf["frac_of_measured"] = rf["achieved"] / top
        out[name] = rf
    return out


# workloads reported next to the headline one: (tag, timed steps, warm-up steps)
ALSO = (("C4b", 3, 2), ("C3a", 10, 3), ("C3b", 10, 3), ("C5", 2, 1), ("C2", 20, 3), ("C2b", 20, 3))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C4a", choices=sorted(inputs.CONFIGS))
    ap.add_argument("--variant", default="dion", choices=["dion", "lazy"],
                    help="dion: the Dion step (default); lazy: Lazy-Dion with a refresh every --refresh-every steps")
    ap.add_argument("--refresh-every", type=int, default=8)
    ap.add_argument("--form", default="standard", choices=["standard", "transposed", "short-side"],
                    help="power iteration on M (standard), on M^T (transposed), or per matrix on whichever side makes the "
                         "orthonormalised factor shorter (transposed where n < m)")
    ap.add_argument("--orth-mode", type=int, default=0, choices=[0, 1, 2],
                    help="0 CholeskyQR2 (default), 1 shifted CholeskyQR3, 2 CholeskyQR2 with the on-device fallback passes enqueued")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stage-timing", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the two micro-kernels that measure this GPU's MFMA and streaming ceilings")
    ap.add_argument("--no-also", action="store_true", help="time the headline workload only")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    cfg = inputs.CONFIGS[args.workload]
    if args.form != "standard" and (args.variant != "dion"):
        print("--form applies to the Dion step only", file=sys.stderr)
        sys.exit(2)
    refresh_every = max(1, args.refresh_every) if args.variant == "lazy" else 1
    if args.variant == "lazy":
        # the first step must refresh (V starts column-normalised, not orthonormal); time whole refresh periods
        args.warmup = max(1, args.warmup)
        args.warmup += (-args.warmup) % refresh_every
        args.steps += (-args.steps) % refresh_every
    p, ms_per_step, stages = run_workload(args.workload, args.steps, args.warmup, not args.no_stage_timing, args.variant,
                                          refresh_every, args.form, args.calibration_copy, args.orth_mode)
    B = p["B"]
    # measured ceilings of this GPU, in the same run: bf16 MFMA issue loop, 18-byte-per-element streaming pass
    ceilings = None
    if not args.no_ceilings:
        scratch = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        ceilings = B.dion_measure_ceilings(scratch)
        del scratch
    rooflines = stage_rooflines(args.workload, stages, ceilings)
    dominant = max(rooflines, key=lambda k: rooflines[k]["ms"]) if rooflines else None
    out = {
        "metric": "ms per Dion step per m x n matrix at rank r" if args.variant == "dion"
                  else "ms per Lazy-Dion step per m x n matrix at rank r (refresh every %d steps)" % refresh_every,
        "value": ms_per_step, "unit": "ms/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["math"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.workload], "matrices": len(cfg["shapes"]),
                   "shape": list(cfg["shapes"][0]) if len(set(cfg["shapes"])) == 1 else "mixed",
                   "mu": inputs.MU, "eta": inputs.ETA, "g_dtype": "bf16" if cfg["g_bf16"] else "f32",
                   "variant": args.variant, "form": args.form, "orth_mode": args.orth_mode},
        "stage_ms": stages,
        "roofline": dict(rooflines[dominant], kernel=dominant) if dominant else None,
        "rooflines": rooflines,
        "ceilings": ceilings,
    }
    p = dict(uniq=p["uniq"], refresh_every=refresh_every)   # drop the device buffers, keep the host inputs for the oracle
    torch.cuda.empty_cache()
    if args.variant == "dion" and args.form == "standard" and not args.calibration_copy and not args.no_also:
        # the other configurations of the benchmark list, each timed the same way (fewer steps), in the same run
        also = {}
        for tag, k, w in ALSO:
            if tag == args.workload:
                continue
            q, ms, st = run_workload(tag, k, w, not args.no_stage_timing)
            del q
            torch.cuda.empty_cache()
            rf = stage_rooflines(tag, st, ceilings)
            also[WORKLOAD_NAMES[tag]] = {"ms_per_step": ms, "steps": k, "warmup": w, "stage_ms": st,
                                         "rooflines": {k2: {f: v[f] for f in ("bound", "achieved", "peak", "unit", "frac", "ms")}
                                                       for k2, v in rf.items()}}
        out["also"] = also
    if not args.no_cpu_baseline and args.form == "standard":
        out["cpu_baseline"] = cpu_baseline(cfg, p, variant=args.variant, refresh_every=refresh_every)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
