"""GPU checks of the per-layer time / utilisation table (wap_profile_layer): the t_c(l, b) entries that the
workload analysis of Section 3.2.1 sums in Eq. 1.  Times cannot be compared with an oracle; what is checked is
everything about a row that has a closed form (row count and order, FLOP and byte counts, derived columns, bound
class) and the sanity relations a usable table must satisfy (throughput does not fall as the minibatch grows,
the end-to-end step sits between its longest layer pass and a small multiple of the sum of its layer passes)."""
import time

import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu

MBS = [8, 16, 32, 64, 128, 256]
PEAK_TF, PEAK_GBS = 2516.6, 8000.0


def _profile(wap, kind, desc, mbs, warmup=2, iters=20):
    nbytes = wap.wap_profile_scratch_bytes(kind, desc, mbs)
    scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    rows = wap.wap_profile_layer(kind, desc, mbs, warmup, iters, scratch)
    torch.cuda.synchronize()
    return rows


def _check_common(rows, mbs, flops_of, bytes_of):
    assert len(rows) == 3 * len(mbs)                       # rows_written == 3 * n_mb
    for i, r in enumerate(rows):
        b, p = mbs[i // 3], i % 3                          # minibatch-major, passes fwd / dgrad / wgrad within
        assert r.minibatch == b and r.pass_ == p
        assert r.flops == flops_of(b)
        assert r.alg_bytes == bytes_of(b, p)
        assert 0.0 < r.time_us_min <= r.time_us_median
        assert 1 <= r.reps_per_sample <= 8
        assert r.tflops == pytest.approx(r.flops / (r.time_us_median * 1e-6) / 1e12, rel=1e-9)
        assert r.frac_of_bf16_peak == pytest.approx(r.tflops / PEAK_TF, rel=1e-9)
        assert r.gbytes_per_s == pytest.approx(r.alg_bytes / (r.time_us_median * 1e-6) / 1e9, rel=1e-9)
        assert r.frac_of_hbm_peak == pytest.approx(r.gbytes_per_s / PEAK_GBS, rel=1e-9)
        assert r.frac_of_bf16_peak < 1.0 and r.frac_of_hbm_peak < 1.5   # nothing beats its roof (cache hits may beat HBM)
        t_mfma, t_hbm = r.flops / (PEAK_TF * 1e12) * 1e6, r.alg_bytes / (PEAK_GBS * 1e9) * 1e6
        want = 2 if r.time_us_median > 4.0 * max(t_mfma, t_hbm) else (0 if t_mfma >= t_hbm else 1)
        assert r.bound == want


def test_conv_layer_table_rows(capsys):
    import paper_1811_01532_amd as wap
    H = W = 28
    C = K = 512                                            # VGG-16 conv4_2
    print("[case] profile conv4_2 over", MBS, flush=True)
    d = wap.conv_desc(1, H, W, C, K, 3, 3, 1, 1, relu=True)
    rows = _profile(wap, 0, d, MBS)
    xe, we = H * W * C, K * 9 * C
    _check_common(rows, MBS, lambda b: 2.0 * b * H * W * K * C * 9,
                  lambda b, p: 2.0 * (b * xe + we + b * H * W * K) if p < 2 else 2.0 * (b * xe + b * H * W * K) + 4.0 * we)
    for p in range(3):
        tf = [rows[3 * i + p].tflops for i in range(len(MBS))]
        # throughput is (weakly) monotone in the minibatch: allow 10 % of timing noise between neighbours
        for a, b in zip(tf, tf[1:]):
            assert b >= 0.9 * a, (p, tf)
        assert tf[-1] > 1.5 * tf[0], (p, tf)               # the small-minibatch under-utilisation is visible
    assert all(rows[3 * (len(MBS) - 1) + p].bound == 0 for p in range(3))   # b = 256: the matrix side, not class 2


def test_fc_layer_table_rows():
    import paper_1811_01532_amd as wap
    n_in, n_out = 4096, 4096                               # fc7 of both networks
    print("[case] profile fc7 over", MBS, flush=True)
    d = wap.fc_desc(1, n_in, n_out, True)
    rows = _profile(wap, 1, d, MBS)
    _check_common(rows, MBS, lambda b: 2.0 * b * n_in * n_out,
                  lambda b, p: 2.0 * (b * n_in + n_in * n_out + b * n_out) if p < 2
                  else 2.0 * (b * n_in + b * n_out) + 4.0 * n_in * n_out)
    # the FC head stays off the matrix roof for every per-GPU minibatch up to 256 (weights dominate the bytes)
    assert all(r.bound in (1, 2) for r in rows)
    for p in range(3):
        tf = [rows[3 * i + p].tflops for i in range(len(MBS))]
        for a, b in zip(tf, tf[1:]):
            assert b >= 0.9 * a, (p, tf)


def test_flops_agree_with_the_step_count():
    """The table's FLOP column summed over a network's layers (forward + both gradients, no data gradient for the
    first layer) is the step's FLOP count, and both equal the closed form of the input recipe module."""
    import paper_1811_01532_amd as wap
    b = 8
    for net in ("alexnet", "vgg16"):
        convs, fcs = si.NETS[net]
        total = 0.0
        for i, d in enumerate(si.conv_shapes(convs, 224)):
            total += (2 if i == 0 else 3) * 2.0 * b * d["P"] * d["Q"] * d["K"] * d["C"] * d["R"] * d["S"]
        for (_, n_in, n_out, _) in fcs:
            total += 3 * 2.0 * b * n_in * n_out
        plan = wap.StepPlan(net, b, lr=0.001, image=224)
        assert plan.flops() == pytest.approx(total, rel=1e-12)
        assert total == pytest.approx(b * si.step_flops_per_image(net), rel=1e-12)


def test_step_time_is_bracketed_by_its_layer_times():
    """AlexNet-style step at minibatch 32: longest single layer pass <= measured step <= 2 x sum of the layer passes
    (the step adds pools, loss and the update traffic to the layer passes and loses the isolated launches' idle gaps)."""
    import paper_1811_01532_amd as wap
    net, b = "alexnet", 32
    convs, fcs = si.NETS[net]
    descs = [(0, wap.conv_desc(1, d["H"], d["W"], d["C"], d["K"], d["R"], d["S"], d["stride"], d["pad"], relu=True))
             for d in si.conv_shapes(convs, 224)]
    descs += [(1, wap.fc_desc(1, n_in, n_out, relu)) for (_, n_in, n_out, relu) in fcs]
    print("[case] profile every alexnet layer at b=32", flush=True)
    total, longest = 0.0, 0.0
    for li, (kind, desc) in enumerate(descs):
        rows = _profile(wap, kind, desc, [b], warmup=2, iters=20)
        for r in rows:
            if li == 0 and r.pass_ == 1:
                continue                                   # the step computes no gradient w.r.t. the image
            total += r.time_us_median
            longest = max(longest, r.time_us_median)
    plan = wap.StepPlan(net, b, lr=0.001, image=224)
    buf = torch.zeros(plan.arena_bytes() + 256, dtype=torch.uint8, device="cuda")
    t = plan.tensors()
    off, nb = t["params.w32"]
    w32 = buf[off:off + nb].view(torch.float32)
    w32.normal_(0.0, 0.01)
    off, nb = t["params.w"]
    wap.wap_cast_f32_bf16(w32.numel(), w32, buf[off:off + nb].view(torch.bfloat16))
    off, nb = t["input"]
    buf[off:off + nb].view(torch.bfloat16).normal_()
    for _ in range(3):
        plan.run(buf)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    steps = 10
    for _ in range(steps):
        plan.run(buf)
    torch.cuda.synchronize()
    step_us = (time.perf_counter() - t0) / steps * 1e6
    print(f"[info] step {step_us:.1f} us, sum of layer passes {total:.1f} us, longest pass {longest:.1f} us", flush=True)
    assert longest <= step_us <= 2.0 * total


def test_mfma_ceiling_rows():
    """The measured ceiling of the matrix pipe: rates below the published peak, clocks inside the chip's range,
    constant operands no slower than random ones, register-only no slower than the LDS / L2-fed loop, and the rate
    consistent with the clock the kernel read (7 MFMAs of 32 cycles per trip, two wavefronts per SIMD)."""
    import paper_1811_01532_amd as wap
    scratch = torch.empty(wap.wap_mfma_ceiling_scratch_bytes() + 256, dtype=torch.uint8, device="cuda")
    rows = {}
    for data in (0, 1):
        for feed in (0, 1):
            print(f"[case] mfma ceiling data={data} feed={feed}", flush=True)
            r = wap.wap_measure_mfma_ceiling(data, feed, 4000, scratch)
            assert (r.data, r.feed) == (data, feed)
            assert 300.0 < r.tflops < PEAK_TF
            assert 0.8 < r.clock_ghz < 2.6
            assert r.us > 0.0
            # at most one MFMA per SIMD every 32 cycles: the rate cannot exceed what the measured clock allows
            assert r.tflops <= 1.05 * PEAK_TF * r.clock_ghz / 2.4
            rows[(data, feed)] = r
    assert rows[(1, 0)].tflops <= 1.03 * rows[(0, 0)].tflops
    assert rows[(1, 1)].tflops <= 1.03 * rows[(1, 0)].tflops
    with pytest.raises(wap.WapError):
        wap.wap_measure_mfma_ceiling(2, 0, 100, scratch)
    with pytest.raises(wap.WapError):
        wap.wap_measure_mfma_ceiling(0, 0, 100, scratch[:4096])
