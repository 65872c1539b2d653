#!/usr/bin/env python3
"""Benchmark of the per-replica training step on one MI355X.

A "step" is one whole pass of the hot path over one synthetic minibatch: forward, softmax
cross-entropy, backward (data and weight gradients of every conv / FC layer, ReLU and max-pool
backward) and the SGD update, enqueued from the library's launch list on one stream.

Prints ONE short JSON line on stdout (its last line).  `value` is the step's algorithmic TFLOP/s
(direct-convolution FLOP count, first layer's data gradient excluded) with all inputs resident in HBM.
`roofline` describes the kernel that takes the largest share of the step, timed with HIP events inside
the timed region; `cpu_baseline` is the fp64 oracle on the host cores over a bounded sample of the same
workload; `util_table` is the step-level utilisation-versus-per-GPU-minibatch sweep for both networks
(rows of [net, minibatch, ms per step, TFLOP/s, fraction of the bf16 peak]).

Everything long goes to files, not to that line: `--detail-out` (JSON: per-kernel and per-operation
breakdown of the step, the per-layer t_c tables of both networks from wap_profile_layer, the workload
analysis decisions, the FC head as model-parallel slices, the vendor GEMM context) and `--table-out`
(the same tables as Markdown).  Progress lines go to stderr.
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

import numpy as np  # noqa: E402

import synth_inputs as si  # noqa: E402

PEAK_BF16 = 2516.6  # TFLOP/s, dense bf16 MFMA
PEAK_HBM = 8000.0   # GB/s
BOUND_NAMES = ("mfma", "hbm", "launch/occupancy")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def _arena(plan, torch):
    buf = torch.empty(plan.arena_bytes() + 256, dtype=torch.uint8, device="cuda")
    assert buf.data_ptr() % 256 == 0
    return buf


def _view(buf, tensors, name, dtype, torch):
    off, nb = tensors[name]
    return buf[off:off + nb].view(dtype)


def init_step(plan, buf, net, B, image, torch, wap, recipe):
    """Fills weights, input and labels.  recipe='numpy' uses the seeded host recipe of
    synth_inputs (the headline run); 'device' draws the same distributions with torch on the GPU
    (used for the minibatch sweep, where only timing matters)."""
    t = plan.tensors()
    convs, fcs = si.NETS[net]
    shapes = si.conv_shapes(convs, image)
    layers = [(d["name"], (d["K"], d["R"], d["S"], d["C"])) for d in shapes]
    n_in = shapes[-1]["out_hw"] ** 2 * shapes[-1]["K"]
    for (name, _, n_out, _) in fcs:
        layers.append((name, (n_out, n_in)))
        n_in = n_out
    _view(buf, t, "params.w32", torch.float32, torch).zero_()
    _view(buf, t, "params.dw", torch.float32, torch).zero_()
    for i, (name, shape) in enumerate(layers):
        w32 = _view(buf, t, name + ".w32", torch.float32, torch)
        fan_in = int(np.prod(shape[1:]))
        if recipe == "numpy":
            bits = si.he_weight_bf16(si.rng(5, 10 + i), shape)
            w = torch.from_numpy(bits.view(np.int16).ravel()).to("cuda").view(torch.bfloat16)
            w32.copy_(w.to(torch.float32))
        else:
            w32.normal_(0.0, float(np.sqrt(2.0 / fan_in)))
            w32.copy_(w32.to(torch.bfloat16).to(torch.float32))
    n = t["params.w32"][1] // 4
    wap.wap_cast_f32_bf16(n, _view(buf, t, "params.w32", torch.float32, torch),
                          _view(buf, t, "params.w", torch.bfloat16, torch))
    x = _view(buf, t, "input", torch.bfloat16, torch)
    lab = _view(buf, t, "labels", torch.int32, torch)
    if recipe == "numpy":
        bits = si.normal_bf16(si.rng(5, 0), (B, image, image, 3))
        x.copy_(torch.from_numpy(bits.view(np.int16).ravel()).to("cuda").view(torch.bfloat16))
        lab.copy_(torch.from_numpy(si.labels(si.rng(5, 1), B)).to("cuda"))
    else:
        x.copy_(torch.randn(x.numel(), device="cuda").to(torch.bfloat16))
        lab.copy_(torch.randint(0, 1000, (B,), device="cuda", dtype=torch.int32))
    torch.cuda.synchronize()


# Learning rate of the benchmark step.  The paper gives none; with the workload's recipe (He-initialised
# weights, N(0,1) images, no normalisation layers) plain SGD at 0.01 blows up within three steps and leaves
# a dead network, at 0.001 the loss on the fixed synthetic batch falls steadily (16 -> 3.5 in 30 steps), so
# consecutive timed steps are ordinary training steps and nothing has to be restored between them.
LR = 0.001


def time_plain_steps(plan, buf, steps, warmup, torch):
    for _ in range(warmup):
        plan.run(buf)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        plan.run(buf)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def vendor_gemm_reference(torch):
    """Context only (nothing of the product path runs through it): the rate of the vendor's bf16 GEMM (torch.matmul,
    i.e. hipBLASLt / rocBLAS) on this machine, for a large square problem and for the plain GEMMs that have the shapes of
    three VGG-16 layers at minibatch 64 (no im2col gather, operands already in matrix form).  It shows what this part
    sustains under its own clock management, next to the datasheet peak the roofline fractions are quoted against."""
    rows = []
    for name, (M, N, K) in (("square", (8192, 8192, 8192)), ("conv3_2 as GEMM", (200704, 256, 2304)),
                            ("conv4_2 as GEMM", (50176, 512, 4608)), ("conv5_2 as GEMM", (12544, 512, 4608))):
        x = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
        w = torch.randn(N, K, device="cuda", dtype=torch.bfloat16)
        for _ in range(10):
            y = x @ w.t()
        torch.cuda.synchronize()
        iters = 40
        t0 = time.perf_counter()
        for _ in range(iters):
            y = x @ w.t()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / iters
        rows.append({"problem": name, "M": M, "N": N, "K": K, "us": round(dt * 1e6, 1),
                     "tflops": round(2.0 * M * N * K / dt / 1e12, 1)})
        del x, w, y
    torch.cuda.empty_cache()
    return {"library": "torch.matmul bf16 (hipBLASLt / rocBLAS)", "rows": rows}


def cpu_baseline(net, image):
    """The fp64 oracle, as it stands, on a bounded sample of the headline workload (two images for VGG-16, sixteen
    for the AlexNet-style network): every conv and FC layer forward + data gradient + weight gradient (first layer's
    data gradient skipped).  Only the oracle calls are timed, not the generation of their inputs."""
    from oracle import oracle as orc
    orc.build()
    convs, fcs = si.NETS[net]
    shapes = si.conv_shapes(convs, image)
    nb = 2 if net == "vgg16" else 16
    g = np.random.default_rng(7)
    flops = 0.0
    dt = 0.0

    def timed(fn, *args, **kw):
        nonlocal dt
        t0 = time.perf_counter()
        out = fn(*args, **kw)
        dt += time.perf_counter() - t0
        return out

    x = g.standard_normal((nb, image, image, 3))
    for i, d in enumerate(shapes):
        w = g.standard_normal((d["K"], d["R"], d["S"], d["C"])) * np.sqrt(2.0 / (d["C"] * d["R"] * d["S"]))
        st, pad = (d["stride"],) * 2, (d["pad"],) * 2
        y = timed(orc.conv2d_fwd, x, w, st, pad, relu=True)
        gy = g.standard_normal(y.shape)
        timed(orc.conv2d_bwd_weight, x, gy, w.shape, st, pad)
        f = 2.0 * nb * d["P"] * d["Q"] * d["K"] * d["C"] * d["R"] * d["S"]
        flops += 2 * f
        if i > 0:
            timed(orc.conv2d_bwd_data, gy, w, x.shape, st, pad)
            flops += f
        x = y
        if d["pool"]:
            x, _ = timed(orc.maxpool_fwd, x, d["pool"][0], d["pool"][1])
    x = x.reshape(nb, -1)
    for (_, _, n_out, relu) in fcs:
        w = g.standard_normal((n_out, x.shape[1])) * np.sqrt(2.0 / x.shape[1])
        y = timed(orc.fc_fwd, x, w, relu=relu)
        gy = g.standard_normal(y.shape)
        timed(orc.fc_bwd_data, gy, w)
        timed(orc.fc_bwd_weight, gy, x)
        flops += 3 * 2.0 * nb * x.shape[1] * n_out
        x = y
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{net}, {nb} images ({image}x{image}), every conv/FC layer fwd+dgrad+wgrad in fp64, "
                      f"{flops / 1e9:.1f} GFLOP in {dt:.1f} s of oracle time"}


def load_traffic(kernel, net, B):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload (the "scaled HBM
    MB / launch" column of profiles/<net>_b<minibatch>_hbm_traffic.md), if there is one and it lists the kernel."""
    path = os.path.join(ROOT, "profiles", f"{net}_b{B}_hbm_traffic.md")
    try:
        with open(path) as f:
            for line in f:
                cells = [c.strip() for c in line.split("|")]
                if len(cells) >= 8 and cells[1].strip("`").replace(" ", "") == kernel.replace(" ", ""):
                    return float(cells[5]) * 1e6
    except (OSError, ValueError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--net", default="vgg16", choices=["vgg16", "alexnet"])
    ap.add_argument("--minibatch", type=int, default=64)
    ap.add_argument("--no-table", action="store_true", help="skip the minibatch sweep and per-layer table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--bias", action="store_true",
                    help="give every layer a bias (forward add, bias gradient, SGD); the headline runs without")
    ap.add_argument("--link-gbs", type=float, default=76.8,
                    help="one-direction bandwidth of one xGMI link, GB/s (analytic t_s of the workload analysis)")
    ap.add_argument("--link-latency-us", type=float, default=10.0, help="latency of one ring step, microseconds")
    ap.add_argument("--table-out", default=os.path.join(ROOT, "gpurun_out", "bench_tables.md"),
                    help="the tables as Markdown go to this path")
    ap.add_argument("--detail-out", default=os.path.join(ROOT, "gpurun_out", "bench_detail.json"),
                    help="the full result (breakdowns and tables) as JSON goes to this path")
    ap.add_argument("--profile-iters", type=int, default=20, help="timed samples per row of the per-layer tables")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs one replica on ONE GPU; --gpus above 1 is not supported "
              "(no collectives, no sharding in this library)", file=sys.stderr)
        return 2

    import torch
    import paper_1811_01532_amd as wap
    if not os.path.exists(os.path.join(ROOT, "paper_1811_01532_amd", "libwap.so")):
        from paper_1811_01532_amd import build
        build.build(verbose=False)
    wap.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    net, B, image = a.net, a.minibatch, 224

    plan = wap.StepPlan(net, B, lr=LR, image=image, flags=wap.WAP_STEP_BIAS if a.bias else 0)
    buf = _arena(plan, torch)
    init_step(plan, buf, net, B, image, torch, wap, "numpy")
    ops = plan.ops()
    flops_step = plan.flops()

    # Untimed: three plain device-to-device copies of a known size (256 MiB); they appear in a rocprofv3 counter run
    # as the runtime's copy kernel and calibrate FETCH_SIZE / WRITE_SIZE (see profiles/).
    cal_src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    torch.cuda.empty_cache()
    # Untimed, before the warm-up: two plain steps, then one step with an event pair around every operation.
    # That pass gives the per-operation breakdown and names the kernel with the largest share of the step.
    for _ in range(2):
        plan.run(buf)
    us, epi, pro = plan.time(buf, steps=1, with_prologue=True)
    torch.cuda.synchronize()

    def group(us_, epi_):
        kern_ = {}
        for (name, kernel, fl, by), u, ue, up in zip(ops, us_, epi_, pro):
            if up > 0:   # weight repacking in front of this operation's main kernel
                k0 = kern_.setdefault("pack_weights_kernel", {"kernel": "pack_weights_kernel", "launches": 0, "us": 0.0,
                                                              "flops": 0.0, "bytes": 0.0})
                k0["launches"] += 1
                k0["us"] += up
            k = kern_.setdefault(kernel, {"kernel": kernel, "launches": 0, "us": 0.0, "flops": 0.0, "bytes": 0.0})
            k["launches"] += 1
            k["us"] += u
            k["flops"] += fl
            k["bytes"] += by
            if ue > 0:   # split-reduction epilogue kernel of this operation, timed on its own
                ek = "reduce_f32*_kernel" if kernel.startswith("wgrad") else "reduce_bf16_kernel"
                k2 = kern_.setdefault(ek, {"kernel": ek, "launches": 0, "us": 0.0, "flops": 0.0, "bytes": 0.0})
                k2["launches"] += 1
                k2["us"] += ue
        return kern_

    kern = group(us, epi)
    klist = sorted(kern.values(), key=lambda k: -k["us"])
    # the dominant kernel is chosen among the operations' main kernels (the split-reduction epilogues and the weight
    # repacking are listed in the breakdown, but carry no algorithmic FLOP / byte count of their own to price)
    main_kernels = {kernel for (_, kernel, _, _) in ops}
    dom_entry = next(k for k in klist if k["kernel"] in main_kernels)
    dom_name = dom_entry["kernel"]
    step_us_all_events = sum(k["us"] for k in klist)

    # Timed region: exactly K steps back to back on the stream, one synchronisation on each side, HIP event
    # pairs only around the launches of the dominant kernel (the full instrumentation costs two event records
    # per operation, about 0.5 ms per step, and would be charged to the step).
    mask = [kernel == dom_name for (_, kernel, _, _) in ops]
    # W warm-up steps immediately in front of the timed region (the clock needs about four steps to settle after
    # any idle gap; the host-side bookkeeping above is such a gap)
    for _ in range(a.warmup):
        plan.run(buf)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # events in every fifth step only: each record between two kernels adds a few microseconds of launch gap, and
    # 22 of them per step made the region about 1.5 % longer than the same steps without events
    every = 5 if a.steps >= 10 else 1
    dus, _ = plan.time(buf, steps=a.steps, op_mask=mask, every=every)      # synchronises once, at its end
    dt = time.perf_counter() - t0
    ms_per_step = dt / a.steps * 1e3
    value = flops_step / (ms_per_step * 1e-3) / 1e12
    dom_us_timed = sum(dus)
    loss = float(_view(buf, plan.tensors(), "loss", torch.float32, torch)[0])
    if not np.isfinite(loss):
        print(f"bench.py: loss is not finite after the timed steps ({loss})", file=sys.stderr)
        return 4

    # ---- roofline of the dominant kernel from the events of the timed region ----
    dom = dict(dom_entry)
    dom["us"] = dom_us_timed
    dom_mfma = dom["flops"] > 0
    if dom_mfma:
        ach = dom["flops"] / (dom["us"] * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16, "unit": "TFLOP/s", "frac": ach / PEAK_BF16}
    else:
        ach = dom["bytes"] / (dom["us"] * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM, "unit": "GB/s", "frac": ach / PEAK_HBM}
    roof.update({"traffic": load_traffic(dom["kernel"], net, B), "kernel": dom["kernel"],
                 "timed_launches": dom["launches"] * ((a.steps + every - 1) // every),
                 "launches_per_step": dom["launches"], "avg_launch_us": dom["us"] / dom["launches"],
                 "alg_flops_per_launch": dom["flops"] / dom["launches"],
                 "alg_bytes_per_launch": dom["bytes"] / dom["launches"],
                 "share_of_step_time": dom["us"] / (ms_per_step * 1e3)})
    kernels = [{"kernel": k["kernel"], "launches": k["launches"], "us_per_step": round(k["us"], 2),
                "tflops": round(k["flops"] / (k["us"] * 1e-6) / 1e12, 2) if k["us"] > 0 else None,
                "gbs": round(k["bytes"] / (k["us"] * 1e-6) / 1e9, 1) if k["us"] > 0 else None} for k in klist]
    op_rows = [{"op": name, "kernel": kernel, "us": round(u, 2), "epilogue_us": round(ue, 2),
                "tflops": round(fl / ((u + ue) * 1e-6) / 1e12, 1) if u > 0 else None,
                "frac_peak": round(fl / ((u + ue) * 1e-6) / 1e12 / PEAK_BF16, 4) if u > 0 else None,
                "gbs": round(by / ((u + ue) * 1e-6) / 1e9, 1) if u > 0 else None}
               for (name, kernel, fl, by), u, ue in zip(ops, us, epi)]

    out = {
        "metric": "step TFLOP/s (bf16 MFMA utilisation) of one replica's training step",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{net} full training step (conv+FC fwd/bwd, ReLU, max-pool, softmax-CE, SGD "
                               f"lr={LR}), per-GPU minibatch {B}, 3x{image}x{image} input, 1000 classes",
                   "net": net, "minibatch": B, "bias": bool(a.bias), "lr": LR,
                   "lr_note": "config 5 names lr=0.01; 0.001 is used because 0.01 diverges on this recipe within three "
                              "steps (work per step is identical)",
                   "step_gflop": flops_step / 1e9, "ops_per_step": len(ops)},
        "frac_of_bf16_peak": value / PEAK_BF16,
        "images_per_s": B / (ms_per_step * 1e-3),
        "loss_after": loss,
        "breakdown_note": "kernels / ops: one fully instrumented warm-up step (event pair around every operation, "
                          f"{step_us_all_events / 1e3:.3f} ms of kernel time); value / ms_per_step / roofline: the timed region",
        "roofline": roof,
        "kernels": kernels,
        "ops": op_rows,
    }
    del buf, plan
    torch.cuda.empty_cache()

    # The same step in the form a replica of a data-parallel job runs (every weight gradient stored for the exchange,
    # the update a separate pass): reported beside the headline, whose one-GPU job lets the gradient kernels update
    # the weights themselves.
    p2 = wap.StepPlan(net, B, lr=LR, image=image,
                      flags=wap.WAP_STEP_STORE_GRADS | (wap.WAP_STEP_BIAS if a.bias else 0))
    b2 = _arena(p2, torch)
    init_step(p2, b2, net, B, image, torch, wap, "device")
    sec2 = time_plain_steps(p2, b2, steps=a.steps, warmup=a.warmup, torch=torch)   # as the headline: the clock settles
    out["gradients_stored"] = {"ms_per_step": sec2 * 1e3, "tflops": flops_step / sec2 / 1e12, "ops_per_step": p2.num_ops(),
                               "note": "WAP_STEP_STORE_GRADS: dw of every layer written, SGD as a separate pass (a data-"
                                       "parallel replica's share; not the headline)"}
    del b2, p2
    torch.cuda.empty_cache()

    # ---- what the matrix pipe of this device sustains (clock under load), measured beside the published peak ----
    log("measuring the MFMA ceiling")
    cs = torch.empty(wap.wap_mfma_ceiling_scratch_bytes() + 256, dtype=torch.uint8, device="cuda")
    ceil_rows = []
    for data, feed, label in ((0, 0, "constant operands, registers only"), (1, 0, "random operands, registers only"),
                              (1, 1, "random operands, LDS + L2 operand feed of the forward kernels")):
        r = wap.wap_measure_mfma_ceiling(data, feed, 6000, cs)
        ceil_rows.append({"data": "random" if data else "constant", "feed": "lds+l2" if feed else "registers",
                          "what": label, "tflops": round(r.tflops, 1), "clock_ghz": round(r.clock_ghz, 3),
                          "frac_of_bf16_peak": round(r.tflops / PEAK_BF16, 4)})
    del cs
    out["mfma_ceiling"] = {"rows": ceil_rows,
                           "note": "wap_measure_mfma_ceiling: a loop of v_mfma_f32_32x32x16_bf16 on every CU; the chip "
                                   "lowers its clock under load, so these measured rates, not the published peak, bound "
                                   "what a kernel can reach on this device"}
    fed = ceil_rows[2]["tflops"]
    if roof.get("bound") == "mfma" and fed > 0:
        roof["frac_of_measured_ceiling"] = round(roof["achieved"] / fed, 4)
        roof["measured_ceiling_tflops"] = fed

    md = []
    if not a.no_table:
        # ---- step-level utilisation versus per-GPU minibatch, both networks ----
        table = []
        for tnet in ("alexnet", "vgg16"):
            for b in (8, 16, 32, 64, 128, 256) + ((512,) if tnet == "alexnet" else ()):
                p = wap.StepPlan(tnet, b, lr=LR, image=image)
                bb = _arena(p, torch)
                init_step(p, bb, tnet, b, image, torch, wap, "device")
                sec = time_plain_steps(p, bb, steps=5, warmup=2, torch=torch)
                tf = p.flops() / sec / 1e12
                table.append({"net": tnet, "minibatch": b, "ms_per_step": round(sec * 1e3, 4),
                              "tflops": round(tf, 2), "frac_of_bf16_peak": round(tf / PEAK_BF16, 4),
                              "images_per_s": round(b / sec, 1), "ops": p.num_ops()})
                del bb, p
                torch.cuda.empty_cache()
        out["util_table"] = table
        # ---- per-layer table (t_c per pass) across the minibatch sweep: the headline network in full, the other
        # one only as input of the workload analysis below ----
        mbs = [8, 16, 32, 64, 128, 256]

        def layer_table(tnet):
            rows_out = []
            convs, fcs = si.NETS[tnet]
            descs = [(d["name"], 0, d["K"] * d["R"] * d["S"] * d["C"],
                      wap.conv_desc(1, d["H"], d["W"], d["C"], d["K"], d["R"], d["S"], d["stride"], d["pad"], relu=True))
                     for d in si.conv_shapes(convs, image)]
            descs += [(name, 1, n_in * n_out, wap.fc_desc(1, n_in, n_out, relu)) for (name, n_in, n_out, relu) in fcs]
            for (name, kind, nparam, desc) in descs:
                nbytes = wap.wap_profile_scratch_bytes(kind, desc, mbs)
                scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
                rows = wap.wap_profile_layer(kind, desc, mbs, 2, a.profile_iters, scratch)
                for r in rows:
                    rows_out.append({"layer": name, "pass": ("fwd", "dgrad", "wgrad")[r.pass_], "minibatch": r.minibatch,
                                     "us": round(r.time_us_median, 2), "tflops": round(r.tflops, 2),
                                     "frac_peak": round(r.frac_of_bf16_peak, 4), "gbs": round(r.gbytes_per_s, 1),
                                     "bound": BOUND_NAMES[r.bound], "params": nparam})
                del scratch
                torch.cuda.empty_cache()
            return rows_out

        tables = {net: layer_table(net)}
        other = "alexnet" if net == "vgg16" else "vgg16"
        tables[other] = layer_table(other)
        out["layers"] = {tn: [{k: v for k, v in r.items() if k != "params"} for r in rows] for tn, rows in tables.items()}
        log("per-layer tables done")

        # ---- workload analysis (Eq. 1): t_c(l, d) from the table at per-GPU minibatch B/d (forward + both
        # backward passes; no data gradient for the first layer), t_s from the ring all-reduce model over one
        # xGMI link; d restricted to the divisions of the global minibatch that the sweep measured ----
        link_bw, link_lat = a.link_gbs * 1e9, a.link_latency_us * 1e-6
        wau_rows = []
        for tnet, rows in tables.items():
            names = []
            for r in rows:
                if r["layer"] not in names:
                    names.append(r["layer"])
            t_of = {(r["layer"], r["pass"], r["minibatch"]): r["us"] * 1e-6 for r in rows}
            params = {r["layer"]: r["params"] for r in rows}
            for Bg in (64, 128, 256):
                G = 8
                allowed = [1 if (Bg % d == 0 and Bg // d in mbs) else 0 for d in range(1, G + 1)]
                t_c = []
                for li, name in enumerate(names):
                    row = []
                    for d in range(1, G + 1):
                        if not allowed[d - 1]:
                            row.append(0.0)
                            continue
                        b = Bg // d
                        t = t_of[(name, "fwd", b)] + t_of[(name, "wgrad", b)]
                        if li > 0:
                            t += t_of[(name, "dgrad", b)]
                        row.append(t)
                    t_c.append(row)
                gb = [4.0 * params[n] for n in names]
                best, est = wap.wap_choose_gpus(t_c, gb, link_bw, link_lat, allowed)
                wau_rows.append({"net": tnet, "global_minibatch": Bg, "best_d": best,
                                 "t_estimate_ms": {str(d): round(est[d - 1] * 1e3, 4) for d in range(1, G + 1) if allowed[d - 1]},
                                 "images_per_s": {str(d): round(Bg / est[d - 1], 1) for d in range(1, G + 1) if allowed[d - 1]}})
        out["wau"] = {"link_bytes_per_s": link_bw, "latency_s": link_lat,
                      "note": "t_c measured on this GPU at minibatch B/d (wap_profile_layer); t_s analytic (ring all-reduce "
                              "over one xGMI link, fp32 gradients); no multi-GPU run is involved",
                      "decisions": wau_rows}
        # ---- the FC head as model-parallel shards (the hybrid direction the paper's Section 2 leaves open): one GPU's
        # share is a slice of out_features / d output neurons at the FULL minibatch, through the same kernels ----
        shard_rows = []
        shard_mbs = sorted({B, 256})
        for (name, n_in, n_out, relu) in si.NETS[net][1]:
            for d in (1, 2, 4, 8):
                n_sh = (n_out + d - 1) // d
                desc = wap.fc_desc(1, n_in, n_sh, relu)
                scratch = torch.empty(wap.wap_profile_scratch_bytes(1, desc, shard_mbs) + 256, dtype=torch.uint8, device="cuda")
                for r in wap.wap_profile_layer(1, desc, shard_mbs, 2, a.profile_iters, scratch):
                    shard_rows.append({"layer": name, "d": d, "out_features": n_sh, "minibatch": r.minibatch,
                                       "pass": ("fwd", "dgrad", "wgrad")[r.pass_], "us": round(r.time_us_median, 2),
                                       "tflops": round(r.tflops, 2), "frac_peak": round(r.frac_of_bf16_peak, 4),
                                       "gbs": round(r.gbytes_per_s, 1), "bound": BOUND_NAMES[r.bound]})
                del scratch
                torch.cuda.empty_cache()
        out["fc_shards"] = {"note": "FC layers of the headline network cut into d slices of output neurons, full minibatch per "
                                    "slice (model-parallel share of one GPU); dgrad is the slice's partial dx", "rows": shard_rows}
        md.append(f"Utilisation versus per-GPU minibatch on one MI355X (bf16 MFMA, fp32 accumulation; fractions against "
                  f"{PEAK_BF16} TFLOP/s and {PEAK_HBM / 1000:.0f} TB/s).  Written by `python bench.py` "
                  f"(headline: {net}, minibatch {B}, {a.steps} timed steps; per-layer rows: wap_profile_layer, "
                  f"{a.profile_iters} samples per row, median).\n\n## Whole training step\n")
        md.append("| net | minibatch | ms/step | TFLOP/s | frac of bf16 peak | images/s |\n|---|---|---|---|---|---|")
        for r in table:
            md.append(f"| {r['net']} | {r['minibatch']} | {r['ms_per_step']} | {r['tflops']} | "
                      f"{r['frac_of_bf16_peak']} | {r['images_per_s']} |")
        md.append("\n## Measured ceiling of the matrix pipe (wap_measure_mfma_ceiling: MFMA loop on every CU, clock read in the kernel)\n")
        md.append("| operands | operand feed | TFLOP/s | clock GHz | frac of bf16 peak |\n|---|---|---|---|---|")
        for r in out["mfma_ceiling"]["rows"]:
            md.append(f"| {r['data']} | {r['feed']} | {r['tflops']} | {r['clock_ghz']} | {r['frac_of_bf16_peak']} |")
        md.append("\n## Workload analysis (Eq. 1): measured t_c at minibatch B/d, analytic ring all-reduce t_s\n")
        md.append("| net | global minibatch | t_estimate ms by d | chosen d |\n|---|---|---|---|")
        for r in wau_rows:
            md.append(f"| {r['net']} | {r['global_minibatch']} | "
                      + ", ".join(f"d={d}: {t}" for d, t in r["t_estimate_ms"].items()) + f" | {r['best_d']} |")
        md.append("\n## FC head as model-parallel slices (out_features / d per GPU, full minibatch)\n")
        md.append("| FC layer | d | out features per shard | minibatch | pass | us | TFLOP/s | GB/s | bound |\n"
                  "|---|---|---|---|---|---|---|---|---|")
        for r in shard_rows:
            md.append(f"| {r['layer']} | {r['d']} | {r['out_features']} | {r['minibatch']} | {r['pass']} | {r['us']} | "
                      f"{r['tflops']} | {r['gbs']} | {r['bound']} |")
        for tn in ("vgg16", "alexnet"):
            md.append(f"\n## Per-layer t_c(l, b), {tn}: one row per layer and pass, cells = us (fraction of the bf16 peak; "
                      f"bound m = MFMA side, h = HBM side, L = launch / occupancy)\n")
            md.append("| layer | pass | " + " | ".join(f"b={b}" for b in mbs) + " |\n|---|---|" + "---|" * len(mbs))
            cell = {(r["layer"], r["pass"], r["minibatch"]): r for r in out["layers"][tn]}
            seen = []
            for r in out["layers"][tn]:
                key = (r["layer"], r["pass"])
                if key in seen:
                    continue
                seen.append(key)
                cells = []
                for b in mbs:
                    c = cell[(r["layer"], r["pass"], b)]
                    cells.append(f"{c['us']} ({c['frac_peak']:.3f} {'mhL'[BOUND_NAMES.index(c['bound'])]})")
                md.append(f"| {r['layer']} | {r['pass']} | " + " | ".join(cells) + " |")

    if not a.no_table:
        out["vendor_gemm_reference"] = vendor_gemm_reference(torch)
    if not a.no_cpu_baseline:
        log("timing the fp64 oracle on the host cores")
        out["cpu_baseline"] = cpu_baseline(net, image)
    for path in (a.table_out, a.detail_out):
        if path:
            os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    if a.table_out and md:
        with open(a.table_out, "w") as f:
            f.write("\n".join(md) + "\n")
    if a.detail_out:
        with open(a.detail_out, "w") as f:
            json.dump(out, f)
    # the ONE line: the headline, its roofline and the CPU baseline; tables only in compact form
    short_keys = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                  "vs_baseline", "dtype", "data", "config", "frac_of_bf16_peak", "images_per_s", "loss_after", "roofline",
                  "cpu_baseline")
    line = {k: out[k] for k in short_keys if k in out}
    if "util_table" in out:
        line["util_table"] = {"columns": ["net", "minibatch", "ms_per_step", "tflops", "frac_of_bf16_peak"],
                              "rows": [[r["net"], r["minibatch"], r["ms_per_step"], r["tflops"], r["frac_of_bf16_peak"]]
                                       for r in out["util_table"]]}
    if "mfma_ceiling" in out:
        line["mfma_ceiling_tflops"] = {f"{r['data']}/{r['feed']}": [r["tflops"], r["clock_ghz"]] for r in out["mfma_ceiling"]["rows"]}
    if "gradients_stored" in out:
        line["gradients_stored_ms_per_step"] = round(out["gradients_stored"]["ms_per_step"], 4)
    line["detail"] = {"json": os.path.relpath(a.detail_out, ROOT) if a.detail_out else None,
                      "markdown": os.path.relpath(a.table_out, ROOT) if a.table_out and md else None}
    sys.stderr.flush()
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
