#!/usr/bin/env python3
"""Benchmark of the MGRIT-GRU hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch: input
projection, `fwd_iters` MGRIT cycles of forward propagation, the loss head
(cross-entropy through a linear layer, outside the library), `bwd_iters` MGRIT
cycles of the adjoint and the parameter gradients.  All inputs are resident in
HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3]
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

MI355X_PEAK = {"hbm_GBps": 8000.0, "fp32_TFLOPs": 157.3, "bf16_TFLOPs": 2500.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3",
                    help="C1..C5 (the benchmark configurations in order); P1: the paper's HMDB51 shape")
    ap.add_argument("--fwd-iters", type=int, default=None)
    ap.add_argument("--bwd-iters", type=int, default=None)
    ap.add_argument("--fine-relax", choices=["FCF", "F"], default="FCF",
                    help="relaxation on the fine level (Alg. 2 as printed uses FCF; the paper notes "
                         "that F-relaxation is often used there)")
    ap.add_argument("--until-converged", action="store_true",
                    help="forward only: first find the number of cycles after which the level-0 "
                         "residual, relative to the norm of the serial solution, is below 1e-8 or has "
                         "stopped decreasing (fp32 floor), then time that many cycles")
    ap.add_argument("--layers", type=int, default=1,
                    help="2: a stack of two GRU layers (layer 2 reads the states of layer 1; "
                         "fp32 workloads only), each solved by its own MGRIT solve")
    ap.add_argument("--study", choices=["convergence", "training", "ode", "lstm"], default=None,
                    help="convergence: residual per cycle, forward and backward, for the paper's "
                         "hierarchies at T = 128 (cf 2 / 4 / 8 with 6 / 3 / 2 levels) and for the "
                         "Classic coarse propagator.  training: the training loop of Alg. 3 with Adam "
                         "on a synthetic classification task, MGRIT (2 forward / 1 backward cycles) "
                         "against serial propagation from the same start.  ode: the appendix's "
                         "demonstration ODE (Eq. 17) as the propagator of the forward cycle, at the "
                         "sizes of --workload, against its serial propagation.  lstm: the same for the LSTM "
                         "step.  One JSON line each")
    ap.add_argument("--train-steps", type=int, default=300)
    ap.add_argument("--operands", choices=["stored", "bf16x3"], default="stored",
                    help="stored: the workload's own form (fp32 or bf16 MFMA).  bf16x3 (fp32 "
                         "workloads): the tile kernels contract the fp32 operands as three bf16 "
                         "terms each on the bf16 matrix pipe (same inputs, same parity bar)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-serial", action="store_true")
    ap.add_argument("--no-side-workloads", action="store_true",
                    help="default run only: do not time C4 and C5 after the C3 headline")
    ap.add_argument("--print-kernel-sources-hash", action="store_true",
                    help="print the hash that stamps the counter records under profiles/ and exit")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="run one 1 GiB device-to-device copy first: the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    return ap.parse_args()


def kernel_sources_sha256():
    """Hash of the code the forward step kernel is built from (stamps the counter records):
    the sources with comments and white space taken out, so that an edited comment does not
    disown a measurement."""
    import hashlib
    import re
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2203_04738_amd", "csrc")
    for f in ("common.h", "gates.h", "gemm_core.h", "gemm_core_bf16.h", "kernels_forward.hip"):
        text = open(os.path.join(csrc, f), "r").read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update("".join(text.split()).encode())
    return h.hexdigest()


def cpu_baseline(wl, fwd_iters, bwd_iters, fcf=True):
    """The CPU oracle as it stands, single-threaded (BLAS pool limited to one thread), timed on a
    reduced twin of the workload (same B, D, H, cf, levels; T a multiple of cf^(levels-1)); work is
    linear in T.  The same sample with the BLAS pool at its default size is reported beside it."""
    import numpy as np
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import mgrit_gru_oracle as orc
    from synthetic_inputs import make_inputs
    all_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])

    def run(tw):
        d = make_inputs(tw)
        P = (d["W"], d["U"], d["b_i"], d["b_h"])
        z = np.zeros((tw.T + 1, tw.B, tw.H))
        t0 = time.perf_counter()
        h, _ = orc.mgrit_forward(*P, d["x"], d["h0"], z, tw.cf, tw.levels, fwd_iters,
                                 fine_relax_fcf=fcf)
        if bwd_iters > 0:
            _, g = orc.cross_entropy_head(h[-1], d["W_o"], d["b_o"], d["labels"])
            orc.mgrit_backward(*P, d["x"], h, g, z, tw.cf, tw.levels, bwd_iters,
                               fine_relax_fcf=fcf)
        return time.perf_counter() - t0

    unit = wl.cf ** (wl.levels - 1)
    n_max = wl.T // unit
    with threadpool_limits(limits=1):
        n = min(2, n_max)
        tw = wl.twin(n)
        dt = run(tw)
        if dt < 8.0 and n < n_max:
            # enlarge the sample towards ~15 s of CPU work (never beyond the full workload)
            n = int(min(n_max, max(n + 1, n * 15.0 / max(dt, 1e-3))))
            tw = wl.twin(n)
            dt = run(tw)
    dt_all = run(tw)
    sample = (f"reduced-T twin of {wl.name}: T={tw.T} (of {wl.T}), B={tw.B}, D={tw.D}, H={tw.H}, "
              f"cf={tw.cf}, levels={tw.levels}, {fwd_iters} fwd + {bwd_iters} bwd cycles, numpy float64")
    return {"value": tw.T * tw.B / dt, "unit": "time-steps*batch/s", "cores": 1, "kind": "oracle",
            "sample": sample + f", {dt:.1f} s",
            "all_threads": {"value": tw.T * tw.B / dt_all, "cores": int(all_threads),
                            "seconds": dt_all}}


def stack_cpu_baseline(wl, layers, fwd_iters, bwd_iters, fcf=True):
    """The oracle's stacked solve on the reduced twin (T = 8*cf^(levels-1))."""
    import numpy as np
    from oracle import mgrit_gru_oracle as orc
    from synthetic_inputs import layer_workload, make_inputs
    from threadpoolctl import threadpool_limits
    tw = wl.twin(min(8, wl.T // wl.cf ** (wl.levels - 1)))
    ds = [make_inputs(layer_workload(tw, j)) for j in range(layers)]
    params = [(d["W"], d["U"], d["b_i"], d["b_h"]) for d in ds]
    z = np.zeros((tw.T + 1, tw.B, tw.H))

    def bwd(j, W, U, bi, bh, x, h, s):
        out = orc.mgrit_backward(W, U, bi, bh, x, h, None, z, tw.cf, tw.levels, bwd_iters,
                                 fine_relax_fcf=fcf, dL_dh=s)
        return (out[0],) + tuple(out[2:7])

    with threadpool_limits(limits=1):      # one host thread, as the single-layer baseline
        t0 = time.perf_counter()
        hs = orc.stacked_forward(
            params, ds[0]["x"], [d["h0"] for d in ds],
            lambda j, W, U, bi, bh, x, h0: orc.mgrit_forward(W, U, bi, bh, x, h0, z, tw.cf,
                                                             tw.levels, fwd_iters,
                                                             fine_relax_fcf=fcf)[0])
        top = ds[-1]
        _, g = orc.cross_entropy_head(hs[-1][-1], top["W_o"], top["b_o"], top["labels"])
        src = np.zeros_like(z)
        src[-1] = g
        orc.stacked_backward(params, ds[0]["x"], hs, src, bwd)
        dt = time.perf_counter() - t0
    return {"value": tw.T * tw.B / dt, "unit": "time-steps*batch/s", "cores": 1,
            "kind": "oracle",
            "sample": f"reduced-T twin of {wl.name}, {layers} layers: T={tw.T} (of {wl.T}), "
                      f"B={tw.B}, D={tw.D}, H={tw.H}, cf={tw.cf}, levels={tw.levels}, {fwd_iters} fwd + "
                      f"{bwd_iters} bwd cycles per layer, numpy float64, {dt:.1f} s"}


def stack_main(args):
    """--layers L: one training step of a stack of L GRU layers.  Forward: the layers
    in order, each by MGRIT, layer j+1 reading the states of layer j.  Backward: the
    loss head on the top layer's h_T, then the layers in reverse order, each layer's
    input gradient being the source term of the layer below."""
    import numpy as np
    import torch

    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import (MGRIT_KEEP_COEFFS, MGRIT_REUSE_COEFFS,
                                              MGRIT_REUSE_PROJECTION, MGRIT_ZERO_ADJOINT_GUESS,
                                              MGRIT_ZERO_STATE_GUESS, MgritGruCfg)
    from synthetic_inputs import WORKLOADS, layer_workload, make_inputs

    wl = WORKLOADS[args.workload]
    if wl.dtype != "fp32":
        print("bench.py: --layers needs an fp32 workload (upper layers read fp32 states)",
              file=sys.stderr)
        sys.exit(2)
    L = args.layers
    x3 = args.operands == "bf16x3"
    dtype_code = 2 if x3 else 0
    fwd_iters = wl.fwd_iters if args.fwd_iters is None else args.fwd_iters
    bwd_iters = max(1, wl.bwd_iters if args.bwd_iters is None else args.bwd_iters)
    fine_relax = 1 if args.fine_relax == "FCF" else 0
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T, B, H = wl.T, wl.B, wl.H
    lay = []
    for j in range(L):
        wj = layer_workload(wl, j)
        d = make_inputs(wj)
        t = {k: torch.from_numpy(v).to(dev) for k, v in d.items() if k != "x" or j == 0}
        cfgj = (lambda wj: lambda iters, flags=0: MgritGruCfg(
            T, B, wj.D, H, cf=wl.cf, levels=wl.levels, iters=iters, fine_relax=fine_relax,
            propagator=0, dtype=dtype_code, flags=flags))(wj)
        lay.append({
            "t": t, "cfg": cfgj, "D": wj.D,
            "ws": torch.empty(mg.mgrit_gru_workspace_bytes(cfgj(max(fwd_iters, bwd_iters))),
                              dtype=torch.uint8, device=dev),
            "h": torch.zeros(T + 1, B, H, device=dev), "w": torch.zeros(T + 1, B, H, device=dev),
            "src": torch.zeros(T + 1, B, H, device=dev),
            "g": (torch.empty(3 * H, wj.D, device=dev), torch.empty(3 * H, H, device=dev),
                  torch.empty(3 * H, device=dev), torch.empty(3 * H, device=dev)),
        })
    top = lay[-1]["t"]
    x0 = lay[0]["t"]["x"]

    def inp(j):
        return x0 if j == 0 else lay[j - 1]["h"][1:]

    def P(j):
        t = lay[j]["t"]
        return t["W"], t["U"], t["b_i"], t["b_h"], inp(j)

    def head():
        logits = lay[-1]["h"][T] @ top["W_o"].T + top["b_o"]
        p = torch.softmax(logits, dim=1)
        p[torch.arange(B, device=dev), top["labels"]] -= 1.0
        lay[-1]["src"][T] = (p / B) @ top["W_o"]

    def dx_of(j):
        # the input gradient of layer j lands in rows 1..T of the source term of layer j-1
        return lay[j - 1]["src"][1:] if j > 0 else None

    def mgrit_step():
        for j in range(L):
            lay[j]["h"].zero_()
            mg.mgrit_gru_forward(lay[j]["cfg"](fwd_iters, MGRIT_KEEP_COEFFS | MGRIT_ZERO_STATE_GUESS),
                                 *P(j),
                                 lay[j]["t"]["h0"], lay[j]["h"], None, lay[j]["ws"])
        head()
        for j in range(L - 1, -1, -1):
            lay[j]["w"].zero_()
            # the top layer's source term is zero below row T and its adjoint starts from zero:
            # its first cycle may skip what is still zero
            top_flag = MGRIT_ZERO_ADJOINT_GUESS if j == L - 1 else 0
            mg.mgrit_gru_backward_steps(lay[j]["cfg"](bwd_iters, MGRIT_REUSE_PROJECTION |
                                                      MGRIT_REUSE_COEFFS | top_flag), *P(j),
                                        lay[j]["h"], lay[j]["src"], lay[j]["w"], None,
                                        *lay[j]["g"], dx_of(j), lay[j]["ws"])

    def serial_step():
        for j in range(L):
            mg.gru_serial_scan(lay[j]["cfg"](1, MGRIT_KEEP_COEFFS), *P(j), lay[j]["t"]["h0"],
                               lay[j]["h"], lay[j]["ws"])
        head()
        for j in range(L - 1, -1, -1):
            mg.gru_serial_scan_backward_steps(lay[j]["cfg"](1, MGRIT_REUSE_PROJECTION |
                                                            MGRIT_REUSE_COEFFS), *P(j),
                                              lay[j]["h"], lay[j]["src"], lay[j]["w"],
                                              *lay[j]["g"], dx_of(j), lay[j]["ws"])

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    sec = timed(mgrit_step, args.steps, args.warmup)
    mg.mgrit_gru_profile_enable(True)
    for _ in range(args.steps):
        mgrit_step()
    torch.cuda.synchronize()
    mg.mgrit_gru_profile_enable(False)
    names = {0: "phi_step (fused forward level step, MFMA tiles)",
             1: "adj_step (fused adjoint level step, MFMA tiles)",
             2: "projection GEMM", 3: "weight-gradient GEMMs + bias sums",
             4: "phi_skinny (few-row forward step, coarsest level)",
             5: "adj_skinny (few-row adjoint step, coarsest level)",
             6: "input-gradient GEMM"}
    kernels = {}
    for kind, nm in names.items():
        n, ms, fl, by = mg.mgrit_gru_profile_read(kind)
        if n:
            kernels[nm] = {"launches_per_step": n / args.steps, "ms_per_step": ms / args.steps,
                           "avg_launch_us": 1e3 * ms / n, "TFLOPs": fl / ms / 1e9,
                           "algorithmic_GBps": by / ms / 1e6}
    peak = MI355X_PEAK["bf16_TFLOPs"] if x3 else MI355X_PEAK["fp32_TFLOPs"]
    step_flops = sum(v["TFLOPs"] * v["ms_per_step"] * 1e9 for v in kernels.values())
    dom = kernels.get(names[0])
    roofline = None
    if dom:
        roofline = {"kernel": names[0], "bound": "mfma", "achieved": dom["TFLOPs"], "peak": peak,
                    "unit": "TFLOP/s", "frac": dom["TFLOPs"] / peak, "traffic": None,
                    "avg_launch_us": dom["avg_launch_us"],
                    "launches_per_step": dom["launches_per_step"]}
    serial = None
    if not args.no_serial:
        ssec = timed(serial_step, max(1, min(args.steps, 3)), 1)
        serial = {"value": T * B / ssec, "unit": "time-steps*batch/s", "ms_per_step": 1e3 * ssec,
                  "what": "gru_serial_scan + gru_serial_scan_backward_steps per layer on the same GPU",
                  "mgrit_speedup": ssec / sec}
    out = {
        "metric": f"GRU time-steps x batch / sec, {L}-layer MGRIT fwd+bwd (1 GPU)",
        "value": T * B / sec, "unit": "time-steps*batch/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * sec, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 as 3 bf16 terms (bf16 MFMA, f32 accumulate)" if x3 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name} x {L} layers: T={T} B={B} D={wl.D} H={H} cf={wl.cf} "
                               f"levels={wl.levels} fwd_iters={fwd_iters} bwd_iters={bwd_iters} per layer, "
                               f"fine-level {args.fine_relax} relaxation, implicit GRU",
                   "operands": args.operands, "seed": wl.seed},
        "roofline": roofline, "kernels": kernels,
        "whole_step": {"TFLOPs": step_flops / sec / 1e12,
                       "frac_of_mfma_peak": step_flops / sec / 1e12 / peak},
        "serial_gpu": serial,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = stack_cpu_baseline(wl, L, fwd_iters, bwd_iters, fcf=bool(fine_relax))
    print(json.dumps(out))


def study_convergence(args):
    """Residual history of MGRIT on the paper-shaped workload P1 (one layer): the study
    behind the paper's choice of cf = 4 and of 2 forward / 1 backward iterations
    (Sec. 4.2, residual figure), on synthetic stand-in data, and the Implicit against the
    Classic coarse propagator (Sec. 3.3)."""
    import torch

    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import MgritGruCfg
    from synthetic_inputs import WORKLOADS, make_inputs

    wl = WORKLOADS["P1"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    d = make_inputs(wl)
    t = {k: torch.from_numpy(v).to(dev) for k, v in d.items()}
    T, B, D, H = wl.T, wl.B, wl.D, wl.H
    P = (t["W"], t["U"], t["b_i"], t["b_h"], t["x"])
    cycles = 8
    rows = []
    for cf, levels, prop in ((2, 6, 0), (4, 3, 0), (8, 2, 0), (2, 6, 1), (4, 3, 1), (8, 2, 1)):
        cfg = MgritGruCfg(T, B, D, H, cf=cf, levels=levels, iters=cycles, fine_relax=1,
                          propagator=prop, dtype=0)
        ws = torch.empty(mg.mgrit_gru_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
        hs = torch.zeros(T + 1, B, H, device=dev)
        mg.gru_serial_scan(cfg, *P, t["h0"], hs, ws)
        h = torch.zeros(T + 1, B, H, device=dev)
        rf = torch.zeros(cycles, device=dev)
        mg.mgrit_gru_forward(cfg, *P, t["h0"], h, rf, ws)
        err = float(torch.max(torch.abs(h - hs)) / torch.max(torch.abs(hs)))
        # adjoint around the serial states, terminal loss gradient from the seeded draw
        w = torch.zeros(T + 1, B, H, device=dev)
        rb = torch.zeros(cycles, device=dev)
        mg.mgrit_gru_backward(cfg, *P, hs, t["dL_dhT"], w, rb, None, None, None, None, ws)
        torch.cuda.synchronize()
        rows.append({"cf": cf, "levels": levels,
                     "propagator": "implicit" if prop == 0 else "classic",
                     "forward_residuals": rf.cpu().tolist(), "backward_residuals": rb.cpu().tolist(),
                     "forward_max_rel_error_after_%d_cycles" % cycles: err})
        del ws
    print(json.dumps({"study": "convergence",
                      "workload": f"P1: T={T} B={B} D={D} H={H}, one layer, FCF relaxation, fp32, "
                                  f"synthetic stand-in for the HMDB51 features",
                      "cycles": cycles, "rows": rows}))


def study_ode(args):
    """Forward MGRIT with the demonstration ODE of the appendix (Eq. 17; forward Euler,
    step size dt on level 0) as propagator, at the sizes and hierarchy of --workload,
    against serial propagation on the same GPU.  A step is one forward solve (projection
    included) over one batch of synthetic data."""
    import numpy as np
    import torch

    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import MgritGruCfg
    from synthetic_inputs import WORKLOADS, random_ode

    wl = WORKLOADS[args.workload]
    if wl.dtype != "fp32":
        print("bench.py: --study ode runs fp32 workloads", file=sys.stderr)
        sys.exit(2)
    T, B, D, H = wl.T, wl.B, wl.D, wl.H
    iters = wl.fwd_iters if args.fwd_iters is None else args.fwd_iters
    fine_relax = 1 if args.fine_relax == "FCF" else 0
    # forward Euler must stay stable on the coarsest level (step size cf^(levels-1) dt;
    # the decay term alone needs it below 4): the coarsest step is at most 1
    dt = min(1.0 / 16, 1.0 / wl.cf ** (wl.levels - 1))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = random_ode(0, T, B, D, H, h0_random=False)
    t = {k: torch.from_numpy(v).to(dev) for k, v in p.items()}
    P = (t["A"], t["Bw"], t["b"], t["d"], t["h0"])

    def cfg(n, levels=wl.levels):
        return MgritGruCfg(T, B, D, H, cf=wl.cf, levels=levels, iters=n, fine_relax=fine_relax)

    ws = torch.empty(mg.mgrit_gru_workspace_bytes(cfg(max(iters, 1))), dtype=torch.uint8,
                     device=dev)
    h = torch.zeros(T + 1, B, H, device=dev)
    hs = torch.zeros(T + 1, B, H, device=dev)
    res = torch.zeros(max(iters, 1), device=dev)

    def mgrit_step():
        h[1:].zero_()
        mg.mgrit_ode_forward(cfg(iters), dt, *P, h, res, ws)

    def serial_step():
        mg.ode_serial_scan(cfg(1), dt, *P, hs, ws)

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    sec = timed(mgrit_step, args.warmup, args.steps)
    residuals = res.cpu().tolist()
    ssec = None if args.no_serial else timed(serial_step, 1, max(2, args.steps // 3))
    err = None
    if ssec is not None:
        err = float(torch.max(torch.abs(h - hs)) / torch.max(torch.abs(hs)))

    # event-timed pass: the level-0 relaxation launches of the ODE step kernel
    rows0 = (T // wl.cf) * B
    mg.mgrit_gru_profile_enable(True)
    for _ in range(args.steps):
        mgrit_step()
    torch.cuda.synchronize()
    mg.mgrit_gru_profile_enable(False)
    n0, ms0, fl0, _ = mg.mgrit_gru_profile_read_shape(8, rows0, 0)
    nall, msall, flall, _ = mg.mgrit_gru_profile_read(8)
    npj, mspj, flpj, _ = mg.mgrit_gru_profile_read(2)
    roof = None
    if n0:
        ach = fl0 / ms0 / 1e9
        roof = {"kernel": f"ode_step (fused forward-Euler level step, MFMA tiles), level-0 "
                          f"relaxation launches ({rows0} rows x H={H})",
                "bound": "mfma", "achieved": ach, "peak": MI355X_PEAK["fp32_TFLOPs"],
                "unit": "TFLOP/s", "frac": ach / MI355X_PEAK["fp32_TFLOPs"], "traffic": None,
                "algorithmic_flops_per_launch": fl0 / n0, "avg_launch_us": 1e3 * ms0 / n0,
                "launches_per_step": n0 / args.steps}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import demo_ode_oracle as ode
        from threadpoolctl import threadpool_limits
        unit = wl.cf ** (wl.levels - 1)

        def run(Tt):
            q = random_ode(0, Tt, B, D, H, h0_random=False)
            with threadpool_limits(limits=1):      # one host thread, as the other baselines
                t0 = time.perf_counter()
                ode.ode_mgrit_forward(q["A"], q["Bw"], q["b"], q["d"], q["h0"],
                                      np.zeros((Tt + 1, B, H)), dt, wl.cf, wl.levels, iters,
                                      fine_relax_fcf=bool(fine_relax))
                return time.perf_counter() - t0

        n, n_max = min(16, T // unit), T // unit
        Tt = n * unit
        el = run(Tt)
        if el < 8.0 and n < n_max:     # enlarge the sample towards ~15 s of CPU work
            n = int(min(n_max, max(n + 1, n * 15.0 / max(el, 1e-3))))
            Tt = n * unit
            el = run(Tt)
        cpu = {"value": Tt * B / el, "unit": "time-steps*batch/s", "cores": 1,
               "kind": "oracle",
               "sample": f"T={Tt} (of {T}), B={B}, D={D}, H={H}, cf={wl.cf}, levels={wl.levels}, "
                         f"{iters} cycles, numpy float64, {el:.1f} s"}

    out = {"study": "ode",
           "metric": "time-steps*batch/sec, MGRIT forward propagation of the demonstration ODE vs "
                     "serial propagation (1 GPU); % roofline",
           "value": T * B / sec, "unit": "time-steps*batch/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": 1e3 * sec, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"demonstration ODE (Eq. 17), forward Euler dt={dt}, sizes of "
                                  f"{wl.name}: T={T} B={B} D={D} H={H} cf={wl.cf} "
                                  f"levels={wl.levels} cycles={iters} fine-level "
                                  f"{args.fine_relax} relaxation, zero initial guess", "seed": 0},
           "residual_fwd": residuals,
           "max_rel_difference_from_serial_propagation": err,
           "roofline": roof,
           "ode_step_all_launches": ({"launches_per_step": nall / args.steps,
                                      "ms_per_step": msall / args.steps,
                                      "TFLOPs": flall / msall / 1e9} if nall else None),
           "projection": ({"ms_per_step": mspj / args.steps, "TFLOPs": flpj / mspj / 1e9}
                          if npj else None),
           "serial_gpu": (None if ssec is None else
                          {"value": T * B / ssec, "unit": "time-steps*batch/s",
                           "ms_per_step": 1e3 * ssec, "what": "ode_serial_scan on the same GPU",
                           "mgrit_speedup": ssec / sec}),
           "cpu_baseline": cpu}
    print(json.dumps(out))


def study_lstm(args):
    """Forward MGRIT with the LSTM step (implicit in the decay terms) as propagator, at the sizes
    and hierarchy of --workload, against serial propagation on the same GPU.  A step is one
    forward solve (projection included) over one batch of synthetic data."""
    import numpy as np
    import torch

    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import MgritGruCfg
    from synthetic_inputs import WORKLOADS, make_lstm_inputs

    wl = WORKLOADS[args.workload]
    if wl.dtype != "fp32":
        print("bench.py: --study lstm runs fp32 workloads", file=sys.stderr)
        sys.exit(2)
    T, B, D, H = wl.T, wl.B, wl.D, wl.H
    iters = wl.fwd_iters if args.fwd_iters is None else args.fwd_iters
    fine_relax = 1 if args.fine_relax == "FCF" else 0
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    d = make_lstm_inputs(wl)
    t = {k: torch.from_numpy(v).to(dev) for k, v in d.items()}
    P = (t["W"], t["U"], t["b_i"], t["b_h"], t["x"], t["u0"])

    def cfg(n):
        return MgritGruCfg(T, B, D, H, cf=wl.cf, levels=wl.levels, iters=n, fine_relax=fine_relax)

    ws = torch.empty(mg.mgrit_lstm_workspace_bytes(cfg(max(iters, 1))), dtype=torch.uint8,
                     device=dev)
    u = torch.zeros(T + 1, B, 2 * H, device=dev)
    us = torch.zeros(T + 1, B, 2 * H, device=dev)
    res = torch.zeros(max(iters, 1), device=dev)

    def mgrit_step():
        u[1:].zero_()
        mg.mgrit_lstm_forward(cfg(iters), *P, u, res, ws)

    def serial_step():
        mg.lstm_serial_scan(cfg(1), *P, us, ws)

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    sec = timed(mgrit_step, args.warmup, args.steps)
    residuals = res.cpu().tolist()
    ssec = None if args.no_serial else timed(serial_step, 1, max(2, args.steps // 3))
    err = None
    if ssec is not None:
        err = float(torch.max(torch.abs(u - us)) / torch.max(torch.abs(us)))

    rows0 = (T // wl.cf) * B
    mg.mgrit_gru_profile_enable(True)
    for _ in range(args.steps):
        mgrit_step()
    torch.cuda.synchronize()
    mg.mgrit_gru_profile_enable(False)
    n0, ms0, fl0, _ = mg.mgrit_gru_profile_read_shape(9, rows0, 0)
    nall, msall, flall, _ = mg.mgrit_gru_profile_read(9)
    npj, mspj, flpj, _ = mg.mgrit_gru_profile_read(2)
    roof = None
    if n0:
        ach = fl0 / ms0 / 1e9
        roof = {"kernel": f"lstm_step (fused LSTM level step, MFMA tiles), level-0 relaxation "
                          f"launches ({rows0} rows x H={H})",
                "bound": "mfma", "achieved": ach, "peak": MI355X_PEAK["fp32_TFLOPs"],
                "unit": "TFLOP/s", "frac": ach / MI355X_PEAK["fp32_TFLOPs"], "traffic": None,
                "algorithmic_flops_per_launch": fl0 / n0, "avg_launch_us": 1e3 * ms0 / n0,
                "launches_per_step": n0 / args.steps}

    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_limits
        from oracle import lstm_oracle as lo
        unit = wl.cf ** (wl.levels - 1)

        def run(n):
            q = make_lstm_inputs(wl.twin(n))
            t0 = time.perf_counter()
            lo.mgrit_lstm_forward(q["W"], q["U"], q["b_i"], q["b_h"], q["x"], q["u0"],
                                  np.zeros((n * unit + 1, B, 2 * H)), wl.cf, wl.levels, iters,
                                  fine_relax_fcf=bool(fine_relax))
            return time.perf_counter() - t0

        with threadpool_limits(limits=1):
            n, n_max = min(2, T // unit), T // unit
            el = run(n)
            if el < 8.0 and n < n_max:     # enlarge the sample towards ~15 s of CPU work
                n = int(min(n_max, max(n + 1, n * 15.0 / max(el, 1e-3))))
                el = run(n)
        cpu = {"value": n * unit * B / el, "unit": "time-steps*batch/s", "cores": 1,
               "kind": "oracle",
               "sample": f"T={n * unit} (of {T}), B={B}, D={D}, H={H}, cf={wl.cf}, "
                         f"levels={wl.levels}, {iters} cycles, numpy float64, {el:.1f} s"}

    out = {"study": "lstm",
           "metric": "time-steps*batch/sec, MGRIT forward propagation of an LSTM layer vs serial "
                     "propagation (1 GPU); % roofline",
           "value": T * B / sec, "unit": "time-steps*batch/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": 1e3 * sec, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"LSTM layer, step implicit in the decay terms, sizes of "
                                  f"{wl.name}: T={T} B={B} D={D} H={H} cf={wl.cf} "
                                  f"levels={wl.levels} cycles={iters} fine-level "
                                  f"{args.fine_relax} relaxation, zero initial guess",
                      "seed": wl.seed},
           "residual_fwd": residuals,
           "max_rel_difference_from_serial_propagation": err,
           "roofline": roof,
           "lstm_step_all_launches": ({"launches_per_step": nall / args.steps,
                                       "ms_per_step": msall / args.steps,
                                       "TFLOPs": flall / msall / 1e9} if nall else None),
           "projection": ({"ms_per_step": mspj / args.steps, "TFLOPs": flpj / mspj / 1e9}
                          if npj else None),
           "serial_gpu": (None if ssec is None else
                          {"value": T * B / ssec, "unit": "time-steps*batch/s",
                           "ms_per_step": 1e3 * ssec, "what": "lstm_serial_scan on the same GPU",
                           "mgrit_speedup": ssec / sec}),
           "cpu_baseline": cpu}
    print(json.dumps(out))


def study_training(args):
    """Alg. 3 as a training loop: a two-layer Implicit GRU with a linear head, trained
    with Adam (lr 1e-3, Sec. 3.4) on a synthetic sequence-classification task of the
    UCI-HAR shape (128 steps, 9 features padded to 12, hidden 100, 6 classes, batch 100;
    cf = 4, 3 levels, 2 forward / 1 backward cycles).  The label of a sequence is a fixed
    function of the sequence (argmax of an exponentially weighted linear read-out), so no
    dataset is needed.  Two runs from the same initial weights on the same batches: one
    with serial propagation (exact states and gradients), one with MGRIT; then the
    MGRIT-trained model is evaluated with serial and with MGRIT inference (Remark 3)."""
    import numpy as np
    import torch

    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import (MGRIT_KEEP_COEFFS, MGRIT_REUSE_COEFFS,
                                              MGRIT_REUSE_PROJECTION, MgritGruCfg)

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    from paper_2203_04738_amd.training import GruStackTrainer
    from synthetic_inputs import ClassificationTask, init_stack
    task = ClassificationTask()                       # T = 128, B = 100, 9 channels, 6 classes
    T, B, D, C, H, L = task.T, task.B, task.D, task.classes, 100, 2
    cf, levels = 4, 3
    fwd_iters = 2 if args.fwd_iters is None else args.fwd_iters
    bwd_iters = 1 if args.bwd_iters is None else max(1, args.bwd_iters)

    def batch(index):
        x, y = task.batch(index)
        return torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev)

    def accuracy(tr, parallel, seeds):
        hit = 0
        for sd in seeds:
            x, y = batch(sd)
            hit += int((tr.predict(x, parallel) == y).sum())
        return hit / (len(seeds) * B)

    def train(parallel):
        params, head = init_stack(7, D, H, C, L)
        tr = GruStackTrainer(T, B, [[torch.from_numpy(q).to(dev) for q in p] for p in params],
                             [torch.from_numpy(q).to(dev) for q in head], cf=cf, levels=levels,
                             fwd_iters=fwd_iters, bwd_iters=bwd_iters, lr=1e-3, parallel=parallel)
        losses = [tr.step(*batch(step)) for step in range(args.train_steps)]
        return tr, losses

    test_seeds = list(range(100000, 100010))
    out = {"study": "training",
           "task": f"synthetic sequence classification, T={T} B={B} features 9 (padded to {D}) H={H} "
                   f"classes={C} layers={L}; cf={cf} levels={levels} {fwd_iters} fwd / {bwd_iters} bwd "
                   f"cycles; Adam lr 1e-3, {args.train_steps} steps, fresh seeded batch every step",
           "runs": {}}
    for name, parallel in (("serial", False), ("mgrit", True)):
        t0 = time.perf_counter()
        tr, losses = train(parallel)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        k = max(1, args.train_steps // 10)
        run = {"loss_first_%d" % k: float(np.mean(losses[:k])),
               "loss_last_%d" % k: float(np.mean(losses[-k:])),
               "loss_every_%d" % k: [float(np.mean(losses[i:i + k]))
                                     for i in range(0, args.train_steps, k)],
               "test_accuracy_serial_inference": accuracy(tr, False, test_seeds),
               "seconds": dt}
        if parallel:
            run["test_accuracy_mgrit_inference"] = accuracy(tr, True, test_seeds)
        out["runs"][name] = run
    print(json.dumps(out))


def main():
    args = parse()
    if args.print_kernel_sources_hash:
        print(kernel_sources_sha256())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.study == "convergence":
        return study_convergence(args)
    if args.study == "training":
        return study_training(args)
    if args.study == "ode":
        return study_ode(args)
    if args.study == "lstm":
        return study_lstm(args)
    if args.layers > 1:
        return stack_main(args)
    out = run_workload(args)
    if (args.workload == "C3" and args.operands == "stored" and not args.until_converged
            and not args.no_side_workloads and args.fwd_iters is None and args.bwd_iters is None):
        # the other two workloads the report covers, in the same run: the image-sequence-shaped
        # long input (C4: bf16 inputs and weights, fp32 state) and the stress configuration (C5)
        out["workloads"] = {}
        for name in ("C4", "C5"):
            a = argparse.Namespace(**vars(args))
            a.workload = name
            a.steps, a.warmup = max(2, min(args.steps, 5)), max(1, min(args.warmup, 2))
            r = run_workload(a, light=True)
            rf = r["roofline"] or {}
            out["workloads"][name] = {
                "config": r["config"]["workload"], "dtype": r["dtype"], "steps": a.steps,
                "ms_per_step": r["ms_per_step"], "value": r["value"], "unit": r["unit"],
                "residual_fwd": r["residual_fwd"], "residual_bwd": r["residual_bwd"],
                "serial_gpu_ms_per_step": r["serial_gpu"]["ms_per_step"],
                "serial_gpu_value": r["serial_gpu"]["value"],
                "speedup_over_serial_scan": r["serial_gpu"]["mgrit_speedup"],
                "level0_step": {"bound": rf.get("bound"), "avg_launch_us": rf.get("avg_launch_us"),
                                "achieved": rf.get("achieved"), "peak": rf.get("peak"),
                                "unit": rf.get("unit"), "frac": rf.get("frac"),
                                "launches_per_step": rf.get("launches_per_step")},
                "few_row_steps": {k.split(" ")[0]: {"launches_per_step": v["launches_per_step"],
                                                    "avg_launch_us": v["avg_launch_us"],
                                                    "ms_per_step": v["ms_per_step"]}
                                  for k, v in r["kernels"].items() if "skinny" in k},
                "whole_step_frac_of_mfma_peak": r["whole_step"]["frac_of_mfma_peak"]}
    print(json.dumps(out))


def run_workload(args, light=False):
    """Times one workload (MGRIT step, per-kernel event times, serial scan on the same GPU) and
    returns the record.  light: no second operand form, no undeclared-guess timing, no CPU leg."""
    import numpy as np
    import torch

    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import (MGRIT_KEEP_COEFFS, MGRIT_REUSE_COEFFS,
                                              MGRIT_REUSE_PROJECTION, MGRIT_ZERO_ADJOINT_GUESS,
                                              MGRIT_ZERO_STATE_GUESS, MgritGruCfg)
    from synthetic_inputs import WORKLOADS, make_inputs

    wl = WORKLOADS[args.workload]
    fwd_iters = wl.fwd_iters if args.fwd_iters is None else args.fwd_iters
    bwd_iters = wl.bwd_iters if args.bwd_iters is None else args.bwd_iters
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    d = make_inputs(wl)
    T, B, D, H = wl.T, wl.B, wl.D, wl.H
    in_dt = torch.float32 if wl.dtype == "fp32" else torch.bfloat16
    t = {k: torch.from_numpy(v).to(dev) for k, v in d.items()}
    for k in ("x", "W", "U"):
        t[k] = t[k].to(in_dt)
    dtype_code = 0 if wl.dtype == "fp32" else 1
    x3 = args.operands == "bf16x3"
    if x3:
        if wl.dtype != "fp32":
            print("bench.py: --operands bf16x3 applies to fp32 workloads", file=sys.stderr)
            sys.exit(2)
        dtype_code = 2

    fine_relax = 1 if args.fine_relax == "FCF" else 0

    def cfg(iters, flags=0, levels=wl.levels, dtype=None):
        return MgritGruCfg(T, B, D, H, cf=wl.cf, levels=levels, iters=iters, fine_relax=fine_relax,
                           propagator=0, dtype=dtype_code if dtype is None else dtype, flags=flags)

    convergence = None
    if args.until_converged:
        # cycles are applied one call at a time; stop when the residual
        # relative to ||h_serial|| is below 1e-8, or has not halved for two cycles in a row
        # (the fp32 floor), or after N_1/2 cycles (two-level FCF is exact by then)
        bwd_iters = 0
        ws0 = torch.empty(mg.mgrit_gru_workspace_bytes(cfg(1)), dtype=torch.uint8, device=dev)
        hs = torch.zeros(T + 1, B, H, device=dev)
        mg.gru_serial_scan(cfg(1), t["W"], t["U"], t["b_i"], t["b_h"], t["x"], t["h0"], hs, ws0)
        hnorm = float(torch.linalg.vector_norm(hs[1:].double()))
        hh = torch.zeros(T + 1, B, H, device=dev)
        r1 = torch.zeros(1, device=dev)
        hist, stall, limit = [], 0, max(1, (T // wl.cf + 1) // 2)
        while len(hist) < limit:
            flags = MGRIT_REUSE_PROJECTION if hist else 0
            mg.mgrit_gru_forward(cfg(1, flags), t["W"], t["U"], t["b_i"], t["b_h"], t["x"], t["h0"],
                                 hh, r1, ws0)
            hist.append(float(r1.item()) / hnorm)
            if hist[-1] < 1e-8:
                break
            stall = stall + 1 if len(hist) > 1 and hist[-1] > 0.5 * hist[-2] else 0
            if stall >= 2:
                break
        fwd_iters = len(hist)
        err = float(torch.max(torch.abs(hh - hs)) / torch.max(torch.abs(hs)))
        convergence = {"cycles": fwd_iters, "relative_residuals": hist,
                       "max_rel_error_vs_serial_scan": err,
                       "stopped_by": "tolerance 1e-8" if hist[-1] < 1e-8 else
                                     ("fp32 floor (residual stopped halving)" if stall >= 2
                                      else "cycle limit N_1/2")}
        del ws0, hs, hh

    # the form timed beside the main one: fp32 workloads, three bf16 terms per operand; bf16
    # workloads, the fp32 state operand as two bf16 terms (MGRIT_BF16_STATE2)
    other = None
    if not x3 and not light:
        other = 2 if wl.dtype == "fp32" else 3
    ws = torch.empty(max(mg.mgrit_gru_workspace_bytes(cfg(max(fwd_iters, bwd_iters, 1), dtype=dt))
                         for dt in (None, other)), dtype=torch.uint8, device=dev)
    h = torch.zeros(T + 1, B, H, device=dev)
    w = torch.zeros(T + 1, B, H, device=dev)
    dW = torch.empty(3 * H, D, device=dev)
    dU = torch.empty(3 * H, H, device=dev)
    dbi = torch.empty(3 * H, device=dev)
    dbh = torch.empty(3 * H, device=dev)
    res_f = torch.zeros(max(fwd_iters, 1), device=dev)
    res_b = torch.zeros(max(bwd_iters, 1), device=dev)
    Wp = (t["W"], t["U"], t["b_i"], t["b_h"], t["x"])
    W_o, b_o, labels = t["W_o"], t["b_o"], t["labels"]

    def loss_head():
        # linear head + mean cross-entropy on h_T and its gradient (outside the library)
        logits = h[T] @ W_o.T + b_o
        p = torch.softmax(logits, dim=1)
        p[torch.arange(B, device=dev), labels] -= 1.0
        return (p / B) @ W_o

    def mgrit_step(dtype=None, declare_zero_guess=True):
        h.zero_()
        # the forward solve leaves the projection and the adjoint coefficients of the steps of
        # its closing relaxation in the workspace; the backward solve reuses both
        zs = MGRIT_ZERO_STATE_GUESS if declare_zero_guess else 0      # h was just zero-filled
        mg.mgrit_gru_forward(cfg(fwd_iters, (MGRIT_KEEP_COEFFS if bwd_iters > 0 else 0) | zs,
                                 dtype=dtype), *Wp, t["h0"], h, res_f, ws)
        if bwd_iters > 0:
            g = loss_head()
            w.zero_()
            # w is the zero initial guess of Alg. 3: the first cycle may skip what is still zero
            zg = MGRIT_ZERO_ADJOINT_GUESS if declare_zero_guess else 0
            mg.mgrit_gru_backward(cfg(bwd_iters, MGRIT_REUSE_PROJECTION | MGRIT_REUSE_COEFFS | zg,
                                      dtype=dtype),
                                  *Wp, h, g, w, res_b, dW, dU, dbi, dbh, ws)

    def serial_step():
        mg.gru_serial_scan(cfg(1, MGRIT_KEEP_COEFFS if bwd_iters > 0 else 0), *Wp, t["h0"], h, ws)
        if bwd_iters > 0:
            g = loss_head()
            mg.gru_serial_scan_backward(cfg(1, MGRIT_REUSE_PROJECTION | MGRIT_REUSE_COEFFS), *Wp,
                                        h, g, w, dW, dU, dbi, dbh, ws)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    if args.pmc_calibration:
        # known-size kernel for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE: a 1 GiB
        # device-to-device copy kernel whose source has been pushed out of the 256 MB
        # memory-side cache by a 1 GiB fill in between
        n = 256 << 20
        src = torch.ones(n, device=dev)
        flush = torch.zeros(n, device=dev)
        dst = torch.empty(n, device=dev)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)      # an elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst, flush

    sec = timed(mgrit_step, args.steps, args.warmup)
    resf = res_f.cpu().numpy().tolist()[:fwd_iters]
    resb = res_b.cpu().numpy().tolist()[:bwd_iters]

    # per-kernel durations from HIP events on the launch stream, over the same K steps
    mg.mgrit_gru_profile_enable(True)
    for _ in range(args.steps):
        mgrit_step()
    torch.cuda.synchronize()
    mg.mgrit_gru_profile_enable(False)
    names = {0: "phi_step (fused forward level step, MFMA tiles)",
             1: "adj_step (fused adjoint level step, MFMA tiles)",
             2: "projection GEMM", 3: "weight-gradient GEMMs + bias sums",
             4: "phi_skinny (few-row forward step, coarsest level)",
             5: "adj_skinny (few-row adjoint step, coarsest level)",
             7: "copy_points (coarse-grid correction, end conditions; HBM-bound)"}
    # dominant launch shape: the level-0 relaxation sub-step (all intervals x batch rows, epilogue
    # mode 0), read first; its launches are put back into the class total below
    dom_rows = (T // wl.cf) * B if wl.levels > 1 else B
    dn, dms, dfl, dby = mg.mgrit_gru_profile_read_shape(0, dom_rows, 0)
    kernels = {}
    for kind, nm in names.items():
        n, ms, fl, by = mg.mgrit_gru_profile_read(kind)
        if kind == 0:
            n, ms, fl, by = n + dn, ms + dms, fl + dfl, by + dby
        if n:
            kernels[nm] = {"launches_per_step": n / args.steps, "ms_per_step": ms / args.steps,
                           "avg_launch_us": 1e3 * ms / n, "TFLOPs": fl / ms / 1e9,
                           "algorithmic_GBps": by / ms / 1e6}
            if kind in (0, 1, 2, 3):
                kernels[nm]["frac_of_mfma_peak"] = fl / ms / 1e9 / (
                    MI355X_PEAK["fp32_TFLOPs"] if dtype_code == 0 else MI355X_PEAK["bf16_TFLOPs"])
                if x3:   # six bf16 MFMA products per algorithmic multiply-add
                    kernels[nm]["issued_TFLOPs"] = 6.0 * fl / ms / 1e9
                    kernels[nm]["issued_frac_of_mfma_peak"] = 6.0 * kernels[nm]["frac_of_mfma_peak"]
            if kind == 7:
                kernels[nm]["frac_of_hbm_peak"] = by / ms / 1e6 / MI355X_PEAK["hbm_GBps"]
    # whole step against the matrix-core peak: flops of all library kernels / step time
    step_flops = sum(v["TFLOPs"] * v["ms_per_step"] * 1e9 for v in kernels.values())
    dom = None
    if dn:
        dom = {"launches_per_step": dn / args.steps, "avg_launch_us": 1e3 * dms / dn,
               "TFLOPs": dfl / dms / 1e9, "flops_per_launch": dfl / dn, "bytes_per_launch": dby / dn}
    peak = MI355X_PEAK["fp32_TFLOPs"] if dtype_code == 0 else MI355X_PEAK["bf16_TFLOPs"]
    # HBM traffic of the dominant kernel per launch: measured with rocprofv3 --pmc (FETCH_SIZE,
    # WRITE_SIZE; scaled by a copy kernel of known size) and recorded in profiles/ together with
    # a hash of the kernel's sources; a record made for other sources is not reported
    traffic, traffic_note = None, "not measured for this workload / operand form"
    tf = os.path.join(ROOT, "profiles", f"phi_step_{wl.name}_hbm_traffic.txt")
    if os.path.exists(tf) and not x3:
        rec = {}
        for line in open(tf):
            if "=" in line and not line.startswith("#"):
                k, v = line.split("=", 1)
                rec[k.strip()] = v.split("#")[0].strip()
        if rec.get("kernel_sources_sha256") == kernel_sources_sha256():
            traffic = int(rec["traffic_bytes_per_launch"])
            traffic_note = ("bytes per launch at this launch shape, rocprofv3 counters "
                            "(profiles/phi_step_%s_hbm_traffic.txt, same kernel sources)" % wl.name)
        else:
            traffic_note = ("profiles/phi_step_%s_hbm_traffic.txt was measured on other kernel "
                            "sources: not reported" % wl.name)
    roofline = None
    if dom:
        roofline = {"kernel": names[0] + f", level-0 relaxation launches ({dom_rows} rows x H={H})",
                    "bound": "mfma", "achieved": dom["TFLOPs"], "peak": peak,
                    "unit": "TFLOP/s", "frac": dom["TFLOPs"] / peak, "traffic": traffic,
                    "traffic_unit": traffic_note,
                    "algorithmic_flops_per_launch": dom["flops_per_launch"],
                    "algorithmic_bytes_per_launch": dom["bytes_per_launch"],
                    "avg_launch_us": dom["avg_launch_us"],
                    "launches_per_step": dom["launches_per_step"],
                    "all_launch_shapes_TFLOPs": kernels[names[0]]["TFLOPs"]}
        if x3:
            # the pipe runs six bf16 products per algorithmic multiply-add: frac prices the
            # algorithmic flops against the bf16 peak, issued_frac the MFMA work actually done
            roofline["issued_TFLOPs"] = 6.0 * dom["TFLOPs"]
            roofline["issued_frac"] = 6.0 * dom["TFLOPs"] / peak
            roofline["frac_of_fp32_mfma_peak"] = dom["TFLOPs"] / MI355X_PEAK["fp32_TFLOPs"]

    # the same step without declaring the zero initial guesses: every pass of the first cycles
    # then runs over all rows, those that only produce (or only read) zeros included
    undeclared = None
    if bwd_iters > 0 and not light:
        usec = timed(lambda: mgrit_step(declare_zero_guess=False), args.steps, 1)
        undeclared = {"what": "same step without MGRIT_ZERO_STATE_GUESS / MGRIT_ZERO_ADJOINT_GUESS (the first "
                              "cycles also run the contractions whose result is exactly zero)",
                      "ms_per_step": 1e3 * usec, "value": T * B / usec}

    # fp32 workloads: the same step with the operands contracted as three bf16 terms
    other_form = None
    if other is not None:
        osec = timed(lambda: mgrit_step(other), args.steps, 1)
        mg.mgrit_gru_profile_enable(True)
        mgrit_step(other)
        torch.cuda.synchronize()
        mg.mgrit_gru_profile_enable(False)
        on, oms, ofl, _ = mg.mgrit_gru_profile_read_shape(0, dom_rows, 0)
        for kind in names:
            mg.mgrit_gru_profile_read(kind)
        if other == 2:
            other_form = {"what": "same step, same inputs, dtype MGRIT_F32_BF16X3: fp32 operands of the "
                                  "tile kernels contracted as three bf16 terms each (six bf16 MFMA "
                                  "products per multiply-add, fp32 accumulation; same 1e-5 parity bar)",
                          "ms_per_step": 1e3 * osec, "value": T * B / osec,
                          "speedup_over_fp32_mfma": sec / osec}
        else:
            other_form = {"what": "same step, same inputs, dtype MGRIT_BF16_STATE2: the fp32 state operand "
                                  "of the tile kernels enters the bf16 MFMAs as two terms (hi + lo, twice "
                                  "the matrix work; within 1e-4 of the oracle where the one-term form is "
                                  "within 2e-2)",
                          "ms_per_step": 1e3 * osec, "value": T * B / osec,
                          "slowdown_over_one_term": osec / sec}
        if on:
            other_form["phi_step_level0_avg_launch_us"] = 1e3 * oms / on
            other_form["phi_step_level0_TFLOPs"] = ofl / oms / 1e9
            if other == 2:
                other_form["phi_step_level0_frac_of_fp32_mfma_peak"] = (
                    ofl / oms / 1e9 / MI355X_PEAK["fp32_TFLOPs"])

    serial = None
    if not args.no_serial:
        s_steps = max(1, min(args.steps, 3))
        ssec = timed(serial_step, s_steps, 1)
        serial = {"value": T * B / ssec, "unit": "time-steps*batch/s", "ms_per_step": 1e3 * ssec,
                  "what": "gru_serial_scan + gru_serial_scan_backward on the same GPU",
                  "mgrit_speedup": ssec / sec}
        # the same comparison without the GEMMs both paths share (input projection and
        # weight gradients), from the per-kernel event times of one profiled step each
        mg.mgrit_gru_profile_enable(True)
        serial_step()
        torch.cuda.synchronize()
        mg.mgrit_gru_profile_enable(False)
        s_shared = sum(mg.mgrit_gru_profile_read(k)[1] for k in (2, 3))
        m_shared = sum(kernels[names[k]]["ms_per_step"] for k in (2, 3) if names[k] in kernels)
        m_rec, s_rec = 1e3 * sec - m_shared, 1e3 * ssec - s_shared
        serial["without_shared_gemms"] = {
            "mgrit_ms_per_step": m_rec, "serial_ms_per_step": s_rec,
            "mgrit_value": T * B / (1e-3 * m_rec), "serial_value": T * B / (1e-3 * s_rec),
            "mgrit_speedup": s_rec / m_rec}

    out = {
        "metric": "GRU time-steps×batch/sec, MGRIT fwd+bwd vs serial scan (1 GPU); % roofline",
        "value": T * B / sec,
        "unit": "time-steps*batch/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * sec,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f32 as 3 bf16 terms (bf16 MFMA, f32 accumulate)" if x3 else
                  "f32" if wl.dtype == "fp32" else "bf16-in/f32-state"),
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={T} B={B} D={D} H={H} cf={wl.cf} levels={wl.levels} "
                               f"fwd_iters={fwd_iters} bwd_iters={bwd_iters} fine-level {args.fine_relax} "
                               f"relaxation, implicit GRU, zero initial guesses (the adjoint's declared)",
                   "operands": args.operands, "seed": wl.seed},
        "convergence": convergence,
        "residual_fwd": resf,
        "residual_bwd": resb,
        "roofline": roofline,
        "kernels": kernels,
        "whole_step": {"TFLOPs": step_flops / sec / 1e12,
                       "frac_of_mfma_peak": step_flops / sec / 1e12 / peak},
        "serial_gpu": serial,
    }
    if undeclared:
        out["without_zero_guess_flag"] = undeclared
    if other_form:
        other_form["mgrit_speedup_vs_serial"] = (serial["ms_per_step"] / other_form["ms_per_step"]
                                                 if serial else None)
        out["bf16x3_operands" if other == 2 else "bf16_state_two_terms"] = other_form
    if not args.no_cpu_baseline and not light:
        out["cpu_baseline"] = cpu_baseline(wl, fwd_iters, bwd_iters, fcf=bool(fine_relax))
    del ws, h, w, t, Wp
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
