#!/usr/bin/env python3
"""Benchmark of the locally connected autoencoder hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-sae]

One "step" is one pass of the whole hot path over one synthetic mini-batch of workload cfg3 (one GPU's
share of a first layer: B=128, 200x200x3 pink-noise images, 20x20x3 fields at stride 4, 32 filters per
location), inputs already resident in HBM:

    lc_forward -> l2pool_lcn_fwd (L2 pooling, then LCN) -> lcn_l2pool_bwd (their gradients)
               -> lc_backward_data -> lc_backward_weights

`value` is the algorithmic flop of the three layer contractions (3 x 2*B*K*F*L) divided by the time of
the whole step.  The JSON line also carries per-kernel times (HIP events on the launch stream, in untimed
steps of their own), the roofline of the dominant kernel (events around it inside the timed steps), the three-stage RICA training step of workload cfg5 (images/s), and
the fp64 CPU oracle timed on the host cores as a scale reference.
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

FP32_MFMA_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sae", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the per-kernel timings of the other workloads (cfg2, cfg4 fp32/bf16, the paper's layer 1)")
    ap.add_argument("--hbm-calibration", action="store_true",
                    help="only run a plain device-to-device copy of 1 GiB five times (reference for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc) and exit")
    return ap.parse_args()


def main() -> int:
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (one GPU's share of a layer at its real shape); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_1502_03409_amd as lc
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback for the product path.", file=sys.stderr)
        return 3
    lc.lib()
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    if args.hbm_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"hbm_calibration": "copy", "bytes_read": src.numel() * 4, "bytes_written": dst.numel() * 4}))
        return 0

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # ---------------------------------------------------------------- workload cfg3
    g = wl.CONFIG_GEOM["cfg3"]
    G = lc.geom(*g.as_tuple())
    x, w, dy = wl.lc_inputs(g, wl.CONFIG_IMAGE_KIND["cfg3"], seed=0)
    xd, wd = dev(x), dev(w)
    Hp, Wp = g.LH - wl.POOL_KSIZE + 1, g.LW - wl.POOL_KSIZE + 1
    y = torch.empty((g.B, g.LH, g.LW, g.F), device="cuda")
    p = torch.empty((g.B, Hp, Wp, g.F), device="cuda")
    n = torch.empty_like(p)
    mu = torch.empty((g.B, Hp, Wp), device="cuda")
    rstd = torch.empty_like(mu)
    dn = dev(np.random.default_rng(1).standard_normal(tuple(p.shape)).astype(np.float32))  # upstream gradient
    dp = torch.empty_like(p)
    dyd = torch.empty_like(y)
    dx = torch.empty((g.B, g.H, g.W, g.C), device="cuda")
    dw = torch.empty((g.LH, g.LW, g.K, g.F), device="cuda")

    names = ["lc_forward", "l2pool_lcn_fwd", "lcn_l2pool_bwd", "lc_backward_data", "lc_backward_weights"]
    calls = [
        lambda: lc.lc_forward(G, xd, wd, None, 1.0, y),
        lambda: lc.l2pool_lcn_fwd(y, p, n, mu, rstd, wl.POOL_KSIZE, wl.POOL_STRIDE, wl.POOL_EPS, wl.LCN_KSIZE,
                                  wl.LCN_SIGMA, wl.LCN_EPS),
        lambda: lc.lcn_l2pool_bwd(y, p, mu, rstd, dn, dp, dyd, wl.POOL_KSIZE, wl.POOL_STRIDE, wl.LCN_KSIZE, wl.LCN_SIGMA),
        lambda: lc.lc_backward_data(G, dyd, wd, dx),
        lambda: lc.lc_backward_weights(G, xd, dyd, 0.0, dw),
    ]

    def step(events=None, only=None):
        """One pass of the hot path.  events: len(calls)+1 events recorded between the calls, or, with `only`,
        two events recorded around call number `only`."""
        for i, c in enumerate(calls):
            if events is not None and only is None:
                events[i].record(stream)
            elif events is not None and i == only:
                events[0].record(stream)
            c()
            if events is not None and i == only:
                events[1].record(stream)
        if events is not None and only is None:
            events[len(calls)].record(stream)

    # The GPU's clocks need some tens of milliseconds of load to settle (the first steps of a process run 10-15 %
    # slower): at least 60 ms of the same work, outside every timed region, then the warm-up steps asked for.
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < 60.0:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # per-entry-point breakdown: its own untimed steps with an event between every two calls (each event costs the
    # stream a microsecond or two, which is why the timed region below carries only the dominant kernel's pair)
    nb = max(1, min(200, args.steps))
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(nb)]
    for s_ in range(nb):
        step(evs[s_])
    torch.cuda.synchronize()
    kern_ms = {nm: float(np.mean([evs[s_][i].elapsed_time(evs[s_][i + 1]) for s_ in range(nb)]))
               for i, nm in enumerate(names)}
    dom = max(("lc_forward", "lc_backward_data", "lc_backward_weights"), key=lambda k: kern_ms[k])
    idom = names.index(dom)
    # the timed region: exactly args.steps steps, HIP events on the launch stream around the dominant kernel only
    devs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s_ in range(args.steps):
        step(devs[s_], idom)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    dom_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in devs]))

    flop_pass = g.flop_per_pass
    lc_flop = 3 * flop_pass
    value = lc_flop / (ms_per_step * 1e-3) / 1e9
    lc_ms = kern_ms["lc_forward"] + kern_ms["lc_backward_data"] + kern_ms["lc_backward_weights"]
    lc_tflops = lc_flop / (lc_ms * 1e-3) / 1e12

    # roofline of the dominant kernel (largest share of the step)
    achieved = flop_pass / (dom_ms * 1e-3) / 1e12
    # HBM bytes per launch: not measurable from inside this process (rocprofv3 --pmc counters); taken from the
    # committed counter summary of the same kernels and workload, and labelled so
    traffic, traffic_source = None, None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic_cfg3.json")
    if os.path.exists(tfile):
        traffic = json.load(open(tfile)).get(dom)
        traffic_source = "profiles/hbm_traffic_cfg3.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, earlier run)"
    roofline = {"kernel": dom, "bound": "mfma", "launch_ms": round(dom_ms, 4), "achieved": round(achieved, 3), "peak": FP32_MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / FP32_MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                "traffic_source": traffic_source}
    # the dominant kernel as the per-kernel breakdown saw it and as the timed region saw it must agree
    warnings = []
    if abs(kern_ms[dom] - dom_ms) > 0.03 * dom_ms:
        warnings.append(f"{dom}: {kern_ms[dom]:.4f} ms in the per-kernel breakdown against {dom_ms:.4f} ms in the "
                        "timed region (more than 3 % apart: clocks not settled, or another process on the GPU)")
    nbytes = {
        "l2pool_lcn_fwd": 4 * (y.numel() + 2 * p.numel() + 2 * mu.numel()),     # y read; p, n, mu, rstd written
        # p, dn, mu, rstd and y read, dy written (the intermediate between the two gradients is not counted)
        "lcn_l2pool_bwd": 4 * (2 * p.numel() + 2 * mu.numel() + 2 * y.numel()),
    }
    kernels = {}
    for nm in names:
        e = {"ms": round(kern_ms[nm], 4)}
        if nm in nbytes:
            gbs = nbytes[nm] / (kern_ms[nm] * 1e-3) / 1e9
            e.update({"GB/s": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)})
        else:
            tf = flop_pass / (kern_ms[nm] * 1e-3) / 1e12
            e.update({"TFLOP/s": round(tf, 2), "frac_fp32_mfma": round(tf / FP32_MFMA_PEAK_TFLOPS, 4)})
        kernels[nm] = e

    out = {
        "metric": "LC layer fwd+bwd GFLOP/s (3 x 2BKFL flop per whole hot-path step)",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg3: B=128 200x200x3 pink-noise, R=20 S=4 F=32 (L=2116, K=1200), "
                               "then 3x3/1 L2 pool and 5x5 LCN, forward and backward",
                   "B": g.B, "H": g.H, "W": g.W, "C": g.C, "R": g.R, "S": g.S, "F": g.F},
        "images_per_s": round(g.B / (ms_per_step * 1e-3), 1),
        "lc_fwd_bwd": {"ms": round(lc_ms, 4), "TFLOP/s": round(lc_tflops, 2),
                       "frac_fp32_mfma_peak": round(lc_tflops / FP32_MFMA_PEAK_TFLOPS, 4)},
        "kernels": kernels,
        "roofline": roofline,
    }
    if warnings:
        out["warnings"] = warnings
    del dw, dx, dyd, dp, dn, n, p, y, xd, wd

    # ---------------------------------------------------------------- workload cfg5: three-stage RICA step
    if not args.no_sae:
        out["sae_step"] = bench_sae(lc, wl, np, torch, dev, max(3, args.steps // 2), max(2, args.warmup // 2))

    # ---------------------------------------------------------------- the three contractions on the other shapes
    if not args.no_others:
        out["other_workloads"] = bench_others(lc, wl, torch, min(50, max(3, args.steps // 4)))

    # ---------------------------------------------------------------- CPU oracle, as a scale reference
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(np, wl, x, w, dy)

    print(json.dumps(out), flush=True)
    return 0


def bench_sae(lc, wl, np, torch, dev, steps, warmup):
    """cfg5: all three stages take one SGD step on the same mini-batch; stage s+1 reads
    l2pool_lcn_fwd(h_s).  Returns images/s of the whole three-stage step: the sequential schedule (flags 0 as
    the workload states it, and with row projection and learned alpha), and the layer pipeline of Sec. 3.1 with a
    forward-only copy of each stage refreshed every P steps."""
    from paper_1502_03409_amd.pipeline import SaePipeline

    keys = ("cfg5_s1", "cfg5_s2", "cfg5_s3")
    geoms = [wl.CONFIG_GEOM[k] for k in keys]
    flop = sum(5 * g.flop_per_pass for g in geoms)
    x1 = dev(wl.pink_images(np.random.default_rng(0), 128, 128, 128, 3))

    def weights():
        out = []
        for si, g in enumerate(geoms):
            rw = np.random.default_rng(100 + si)
            out.append(dev((rw.standard_normal((g.LH, g.LW, g.K, g.F)) / np.sqrt(g.K)).astype(np.float32)))
        return out

    def timed(step, join=None):
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < 60.0:      # settle the clocks on this very work
            for _ in range(4):
                step()
            torch.cuda.synchronize()
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        if join:
            join()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def line(ms, extra=None):
        tf = flop / (ms * 1e-3) / 1e12
        e = {"ms_per_step": round(ms, 4), "images_per_s": round(128 / (ms * 1e-3), 1), "TFLOP/s": round(tf, 2),
             "frac_fp32_mfma_peak": round(tf / FP32_MFMA_PEAK_TFLOPS, 4)}
        e.update(extra or {})
        return e

    # ---- sequential: every stage trains on the features its predecessor's training instance just produced
    def sequential(flags):
        # a learned alpha sums its gradient over every unit of a layer: it needs a far smaller step to stay stable
        lr = wl.SAE_LR if not flags & 2 else 1e-2 * wl.SAE_LR
        stages, inp = [], x1
        for g, w in zip(geoms, weights()):
            G = lc.geom(*g.as_tuple())
            st = {"G": G, "x": inp, "w": w, "b": torch.zeros((g.H, g.W, g.C), device="cuda"),
                  "alpha": torch.ones(1, device="cuda"), "cost": torch.zeros(1, device="cuda"),
                  "h": torch.empty((g.B, g.LH, g.LW, g.F), device="cuda"),
                  "ws": torch.empty(lc.workspace_bytes(G, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device="cuda"),
                  "p": torch.empty((g.B, g.LH - 2, g.LW - 2, g.F), device="cuda")}
            st["n"] = torch.empty_like(st["p"])
            st["mu"] = torch.empty(st["p"].shape[:3], device="cuda")
            st["rstd"] = torch.empty_like(st["mu"])
            stages.append(st)
            inp = st["n"]

        def step():
            for st in stages:
                lc.sae_step(st["G"], st["x"], st["w"], st["b"], st["alpha"], wl.SAE_LAMBDA, wl.SAE_EPS, lr, flags,
                            st["h"], st["cost"], st["ws"])
                lc.l2pool_lcn_fwd(st["h"], st["p"], st["n"], st["mu"], st["rstd"], wl.POOL_KSIZE, wl.POOL_STRIDE,
                                  wl.POOL_EPS, wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS)

        ms = timed(step)
        return line(ms, {"flags": flags, "lr": lr, "costs": [round(float(st["cost"].item()), 4) for st in stages]})

    res = {"workload": "cfg5: three-stage RICA step, B=128 128x128x3", "steps": steps}
    res.update(sequential(0))
    res["project_rows_learn_alpha"] = sequential(3)

    # ---- the layer pipeline of Sec. 3.1: training instance + forward-only instance per stage, one stream per stage
    for P in (1, 10):
        pipe = SaePipeline([lc.geom(*g.as_tuple()) for g in geoms], weights(),
                           [torch.zeros((g.H, g.W, g.C), device="cuda") for g in geoms], [1.0] * 3, [wl.SAE_LAMBDA] * 3,
                           sync_period=P, eps_sparse=wl.SAE_EPS, lr=wl.SAE_LR, flags=0,
                           pool=(wl.POOL_KSIZE, wl.POOL_STRIDE, wl.POOL_EPS), lcn=(wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS))
        ms = timed(lambda: pipe.step(x1), pipe.join)
        res[f"pipeline_sync{P}"] = line(ms, {
            "schedule": f"one stream per stage; forward-only copy of stages 1-2 refreshed every {P} step(s) feeds the "
                        "next stage (one more forward pass per stage than the sequential schedule; TFLOP/s still "
                        "counts 5 passes per stage)"})
        del pipe
        torch.cuda.empty_cache()
    return res


BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak


def timed_ms(torch, stream, f, iters, warm_ms=60.0):
    """Average duration of f() in ms between two HIP events on `stream`, after at least warm_ms of the same work:
    the GPU's clocks take some tens of milliseconds of load to settle, and the first calls run up to 15 % slower."""
    f()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < warm_ms:
        for _ in range(4):
            f()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(iters):
        f()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def bench_others(lc, wl, torch, iters):
    """lc_forward / lc_backward_data / lc_backward_weights alone on the other workloads (random device
    tensors of the workload's shape; parity at these shapes is the tests' business), HIP events on the
    launch stream.  bf16 lines also give the time the mandatory HBM traffic would take at 8 TB/s."""
    stream = torch.cuda.current_stream()
    shapes = [("cfg3", wl.CONFIG_GEOM["cfg3"], "bf16"),
              ("cfg2", wl.CONFIG_GEOM["cfg2"], "f32"), ("cfg2", wl.CONFIG_GEOM["cfg2"], "bf16"),
              ("cfg4", wl.CONFIG_GEOM["cfg4"], "f32"),
              ("cfg4", wl.CONFIG_GEOM["cfg4"], "bf16"), ("paper_layer1", wl.PAPER_LAYER1, "f32"), ("paper_layer3_dense", wl.PAPER_LAYER3, "f32")]
    res = {}
    for name, g, dt in shapes:
        G = lc.geom(*g.as_tuple())
        x = torch.randn((g.B, g.H, g.W, g.C), device="cuda")
        w = torch.randn((g.LH, g.LW, g.K, g.F), device="cuda") / g.K ** 0.5
        dy = torch.randn((g.B, g.LH, g.LW, g.F), device="cuda")
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        code = lc.LC_F32
        if dt == "bf16":
            x, w, dy, code = x.bfloat16(), w.bfloat16(), dy.bfloat16(), lc.LC_BF16
        nws = lc.workspace_bytes(G, lc.LC_OP_FORWARD, code)      # optional: layers with very few fields
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
        fns = {"lc_forward": lambda: lc.lc_forward(G, x, w, None, 1.0, y, code, ws),
               "lc_backward_data": lambda: lc.lc_backward_data(G, dy, w, dx, code),
               "lc_backward_weights": lambda: lc.lc_backward_weights(G, x, dy, 0.0, dw, code)}
        esz = 2 if dt == "bf16" else 4
        min_bytes = {"lc_forward": esz * (w.numel() + x.numel()) + 4 * y.numel(),
                     "lc_backward_data": esz * (w.numel() + dy.numel()) + 4 * dx.numel(),
                     "lc_backward_weights": esz * (x.numel() + dy.numel()) + 4 * dw.numel()}
        peak = BF16_MFMA_PEAK_TFLOPS if dt == "bf16" else FP32_MFMA_PEAK_TFLOPS
        entry, total = {}, 0.0
        for kn, f in fns.items():
            ms = timed_ms(torch, stream, f, iters)
            total += ms
            tf = g.flop_per_pass / (ms * 1e-3) / 1e12
            entry[kn] = {"ms": round(ms, 4), "TFLOP/s": round(tf, 1), "frac_mfma_peak": round(tf / peak, 4),
                         "frac_hbm_roof": round(min_bytes[kn] / (HBM_PEAK_GBS * 1e9) / (ms * 1e-3), 4)}
        tf = 3 * g.flop_per_pass / (total * 1e-3) / 1e12
        entry["fwd_bwd"] = {"ms": round(total, 4), "TFLOP/s": round(tf, 1), "frac_mfma_peak": round(tf / peak, 4)}
        # the three passes back to back, as a training step runs them: a kernel timed alone in a loop finds operands
        # that fit the 256 MB Infinity Cache still there from its own previous call, behind the other passes it does not
        seq = timed_ms(torch, stream, lambda: [f() for f in fns.values()], max(iters // 2, 5))
        tf = 3 * g.flop_per_pass / (seq * 1e-3) / 1e12
        entry["fwd_bwd_in_sequence"] = {"ms": round(seq, 4), "TFLOP/s": round(tf, 1),
                                        "frac_mfma_peak": round(tf / peak, 4)}
        entry["shape"] = dict(zip("BHWCRSF", g.as_tuple()))
        res[f"{name}_{dt}"] = entry
        del x, w, dy, y, dx, dw
        torch.cuda.empty_cache()

    # one whole RICA step (Eq. 1) on the paper's first layer: 1.53e9 weights trained in place on one GPU
    g = wl.PAPER_LAYER1
    G = lc.geom(*g.as_tuple())
    x = torch.randn((g.B, g.H, g.W, g.C), device="cuda")
    w = torch.randn((g.LH, g.LW, g.K, g.F), device="cuda") / g.K ** 0.5
    b = torch.zeros((g.H, g.W, g.C), device="cuda")
    a, cost = torch.ones(1, device="cuda"), torch.zeros(1, device="cuda")
    h = torch.empty((g.B, g.LH, g.LW, g.F), device="cuda")
    ws = torch.empty(lc.workspace_bytes(G, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device="cuda")
    f = lambda: lc.sae_step(G, x, w, b, a, wl.SAE_LAMBDA, wl.SAE_EPS, wl.SAE_LR, 0, h, cost, ws)
    ms = timed_ms(torch, stream, f, iters)
    tf = 5 * g.flop_per_pass / (ms * 1e-3) / 1e12
    res["paper_layer1_sae_step"] = {"ms": round(ms, 3), "images_per_s": round(g.B / (ms * 1e-3), 1),
                                    "TFLOP/s": round(tf, 1), "frac_mfma_peak": round(tf / FP32_MFMA_PEAK_TFLOPS, 4),
                                    "shape": dict(zip("BHWCRSF", g.as_tuple()))}
    del x, w, b, h, ws
    torch.cuda.empty_cache()

    # RICA as Eq. 1 prints it (unit-norm rows, learned alpha) on the paper's first layer and on its dense last layer
    # (lambda = 0.01 there)
    for name, g, lam in (("paper_layer1_sae_step_project_alpha", wl.PAPER_LAYER1, wl.SAE_LAMBDA),
                         ("paper_layer3_dense_sae_step_project_alpha", wl.PAPER_LAYER3, wl.SAE_LAMBDA_DENSE)):
        G = lc.geom(*g.as_tuple())
        x = torch.randn((g.B, g.H, g.W, g.C), device="cuda").abs()
        w = torch.randn((g.LH, g.LW, g.K, g.F), device="cuda") / g.K ** 0.5
        b = torch.zeros((g.H, g.W, g.C), device="cuda")
        a, cost = torch.ones(1, device="cuda"), torch.zeros(1, device="cuda")
        h = torch.empty((g.B, g.LH, g.LW, g.F), device="cuda")
        ws = torch.empty(lc.workspace_bytes(G, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device="cuda")
        f = lambda: lc.sae_step(G, x, w, b, a, lam, wl.SAE_EPS, 1e-5, 3, h, cost, ws)
        ms = timed_ms(torch, stream, f, iters)
        tf = 5 * g.flop_per_pass / (ms * 1e-3) / 1e12
        res[name] = {"ms": round(ms, 3), "images_per_s": round(g.B / (ms * 1e-3), 1), "TFLOP/s": round(tf, 1),
                     "frac_mfma_peak": round(tf / FP32_MFMA_PEAK_TFLOPS, 4), "lambda": lam, "flags": 3,
                     "shape": dict(zip("BHWCRSF", g.as_tuple()))}
        del x, w, b, h, ws
        torch.cuda.empty_cache()

    # the LCN variants at cfg3's shape (flags: 1 per-channel statistics, 2 zero-padded borders, 4 two stages)
    g = wl.CONFIG_GEOM["cfg3"]
    shape = (g.B, (g.LH - wl.POOL_KSIZE) // wl.POOL_STRIDE + 1, (g.LW - wl.POOL_KSIZE) // wl.POOL_STRIDE + 1, g.F)
    x, dy = torch.randn(shape, device="cuda"), torch.randn(shape, device="cuda")
    y, dx = torch.empty_like(x), torch.empty_like(x)
    entry = {"shape": list(shape), "ksize": wl.LCN_KSIZE}
    for flags in range(8):
        stat = shape if flags & lc.LCN_PER_CHANNEL else shape[:3]
        mu, rstd = torch.empty(stat, device="cuda"), torch.empty(stat, device="cuda")
        nws = lc.lcn_variant_workspace_bytes(shape, flags)
        ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
        fns = {"fwd": (lambda: lc.lcn_variant_fwd(x, y, mu, rstd, wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS, flags),
                       4 * (2 * x.numel() + 2 * mu.numel())),
               "bwd": (lambda: lc.lcn_variant_bwd(x, mu, rstd, dy, dx, wl.LCN_KSIZE, wl.LCN_SIGMA, flags, ws),
                       4 * (3 * x.numel() + 2 * mu.numel()))}
        e = {}
        for kn, (f, nbytes) in fns.items():
            ms = timed_ms(torch, stream, f, iters)
            e[kn] = {"us": round(ms * 1e3, 1), "frac_hbm_roof": round(nbytes / (HBM_PEAK_GBS * 1e9) / (ms * 1e-3), 4)}
        entry[f"flags{flags}"] = e
    res["lcn_variants_cfg3"] = entry
    return res


def cpu_baseline(np, wl, x, w, dy):
    """The fp64 oracle as it stands, on the host cores, over whole cfg3 steps (every primitive once per
    step, B=128), repeated until about ten seconds have passed (at most 8 steps).  A scale reference, not a
    target."""
    import oracle

    g = wl.CONFIG_GEOM["cfg3"]
    t = g.as_tuple()
    xd, wd, dyd = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    reps, t0 = 0, time.perf_counter()
    while reps < 8 and (reps == 0 or time.perf_counter() - t0 < 10.0):
        y = oracle.lc_forward(t, xd, wd)
        p = oracle.l2pool_fwd(y, wl.POOL_KSIZE, wl.POOL_STRIDE, wl.POOL_EPS)
        n, mu, rstd = oracle.lcn_fwd(p, wl.LCN_KSIZE, wl.LCN_SIGMA, wl.LCN_EPS)
        dp = oracle.lcn_bwd(p, mu, rstd, n, wl.LCN_KSIZE, wl.LCN_SIGMA)
        oracle.l2pool_bwd(y, p, dp, wl.POOL_KSIZE, wl.POOL_STRIDE)
        oracle.lc_backward_data(t, dyd, wd)
        oracle.lc_backward_weights(t, xd, dyd)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": round(3 * g.flop_per_pass / dt / 1e9, 2), "unit": "GFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds_per_step": round(dt, 2), "steps": reps,
            "sample": f"{reps} whole cfg3 steps (all seven primitives, B=128), fp64 naive loops, OpenMP"}


if __name__ == "__main__":
    sys.exit(main())
