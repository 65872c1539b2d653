"""GPU parity on a seeded randomised sweep of convolution shapes: whatever kernel and tiling the shape-driven
selection picks (patch / 2-D tile / flat tile / first-layer / generic kernels, split reductions, ragged tails), the
three passes, the fused forward pool and the pooled-gradient backward calls must match the fp64 oracle.  The fixed
cases in test_gpu_conv.py pin each kernel; this sweep guards the selection logic between them."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,ncase", [(7, 40), (11, 40)])
def test_random_conv_shapes_match_oracle(orc, seed, ncase):
    import paper_1811_01532_amd as wap
    rng = np.random.default_rng(seed)
    bad = []
    for ci in range(ncase):
        kind = rng.integers(0, 4)
        if kind == 0:   # channel-rich stride-1 layers (patch / tile kernels)
            C = int(rng.choice([64, 128, 192, 256])); K = int(rng.choice([64, 128, 192, 256]))
            R, S = [(3, 3), (3, 3), (5, 5), (1, 3), (3, 1), (3, 5)][rng.integers(0, 6)]
            H = int(rng.integers(7, 40)); W = int(rng.integers(7, 60)); N = int(rng.integers(1, 9))
            st = (1, 1); pad = ((R - 1) // 2, (S - 1) // 2) if rng.random() < 0.8 else (0, 0)
        elif kind == 1:  # first-layer shapes
            C = 3; K = int(rng.choice([32, 64])); R = int(rng.choice([3, 5, 7, 11])); S = R
            sw = int(rng.choice([1, 2, 4])); st = (int(rng.choice([1, 2, 4])), sw)
            H = int(rng.integers(24, 70)); W = int(rng.choice([40, 48, 56, 64, 72, 51, 67])); N = int(rng.integers(2, 10))
            pad = (int(rng.integers(0, min(R, 4))), int(rng.choice([0, 2])) if R > 2 else 0)
        elif kind == 2:  # strided / odd channels (generic)
            C = int(rng.choice([8, 24, 40, 64, 5])); K = int(rng.choice([16, 40, 64, 100, 7]))
            R, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
            st = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
            H = int(rng.integers(6, 30)); W = int(rng.integers(6, 30)); N = int(rng.integers(1, 5))
            pad = (int(rng.integers(0, R)), int(rng.integers(0, S)))
        else:            # larger pixel counts, thin channels (tile2d / wgrad_patch with many tiles)
            C = 64; K = int(rng.choice([64, 128])); R = S = 3; st = (1, 1); pad = (1, 1)
            H = int(rng.choice([28, 30, 32, 56, 26])); W = int(rng.choice([28, 32, 56, 64, 30, 112])); N = int(rng.integers(1, 5))
        P, Q = si.out_dim(H, pad[0], R, st[0]), si.out_dim(W, pad[1], S, st[1])
        if P < 1 or Q < 1: continue
        shape = (N, H, W, C, K, R, S, st, pad)
        print(f"[case] sweep seed={seed} #{ci} {shape} P={P} Q={Q}", flush=True)
        xb = si.normal_bf16(si.rng(9000 + 100 * seed + ci, 0), (N, H, W, C)); wb = si.he_weight_bf16(si.rng(9000 + 100 * seed + ci, 1), (K, R, S, C))
        gb = si.normal_bf16(si.rng(9000 + 100 * seed + ci, 2), (N, P, Q, K))
        x64, w64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(wb), orc.bf16_bits_to_f64(gb)
        xd, wd, gd = gu.dev_bf16(xb), gu.dev_bf16(wb), gu.dev_bf16(gb)
        d = wap.conv_desc(N, H, W, C, K, R, S, st, pad, relu=True)
        ws = gu.workspace(max(wap.wap_conv2d_workspace_bytes(d, p) for p in (0, 1, 2)))
        y = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
        dx = torch.full((N, H, W, C), float("nan"), dtype=torch.bfloat16, device="cuda")
        dw = torch.full((K, R, S, C), float("nan"), dtype=torch.float32, device="cuda")
        wap.wap_conv2d_fwd(d, xd, wd, None, y, ws); wap.wap_conv2d_bwd_data(d, gd, wd, dx, ws); wap.wap_conv2d_bwd_weight(d, xd, gd, dw, ws)
        torch.cuda.synchronize()
        e = [gu.rel_err(gu.host_f64(y), orc.conv2d_fwd(x64, w64, st, pad, relu=True)),
             gu.rel_err(gu.host_f64(dx), orc.conv2d_bwd_data(g64, w64, (N, H, W, C), st, pad)),
             gu.rel_err(gu.host_f64(dw), orc.conv2d_bwd_weight(x64, g64, (K, R, S, C), st, pad))]
        ok = e[0] <= gu.TOL_BF16_OUT and e[1] <= gu.TOL_BF16_OUT and e[2] <= gu.TOL_F32_OUT
        # the weight gradient with the update applied by its own kernels: bit for bit gradient + separate update
        # (the gradient itself was checked against the oracle above)
        w0 = (torch.randn((K, R, S, C), device="cuda", generator=torch.Generator(device="cuda").manual_seed(ci)) * 0.05)
        wm, wm2 = w0.clone(), w0.clone()
        wbf, wbf2 = torch.empty_like(wm, dtype=torch.bfloat16), torch.empty_like(wm, dtype=torch.bfloat16)
        scr = None if wap.wap_conv2d_bwd_weight_sgd_fused(d) else torch.empty_like(dw)
        wap.wap_conv2d_bwd_weight_sgd(d, xd, gd, wm, wbf, 0.05, scr, ws)
        wap.wap_sgd_update(K * R * S * C, wm2, dw, 0.05, wbf2)
        torch.cuda.synchronize()
        ok = ok and torch.equal(wm, wm2) and torch.equal(wbf.view(torch.int16), wbf2.view(torch.int16))
        if P % 2 == 0 and Q % 2 == 0:
            gpb = si.normal_bf16(si.rng(9000 + 100 * seed + ci, 4), (N, P // 2, Q // 2, K))
            amh = si.rng(9000 + 100 * seed + ci, 5).integers(0, 4, size=(N, P // 2, Q // 2, K), dtype=np.uint8)
            gpd, amd = gu.dev_bf16(gpb), torch.from_numpy(amh).cuda()
            routed = orc.maxpool_bwd(orc.bf16_bits_to_f64(gpb), amh, (N, P, Q, K), 2, 2)
            scratch = torch.empty((N, P, Q, K), dtype=torch.bfloat16, device="cuda")
            wap.wap_conv2d_bwd_data_pool2x2(d, gpd, amd, wd, None, dx, scratch, ws)
            wap.wap_conv2d_bwd_weight_pool2x2(d, xd, gpd, amd, dw, scratch, ws)
            yp = torch.empty((N, P // 2, Q // 2, K), dtype=torch.bfloat16, device="cuda"); am = torch.empty((N, P // 2, Q // 2, K), dtype=torch.uint8, device="cuda")
            y2 = torch.empty_like(y)
            wap.wap_conv2d_fwd_pool2x2(d, xd, wd, None, y2, yp, am, ws)
            torch.cuda.synchronize()
            e += [gu.rel_err(gu.host_f64(dx), orc.conv2d_bwd_data(routed, w64, (N, H, W, C), st, pad)),
                  gu.rel_err(gu.host_f64(dw), orc.conv2d_bwd_weight(x64, routed, (K, R, S, C), st, pad))]
            rp, ra = orc.maxpool_fwd(gu.host_f64(y2), 2, 2)
            ok = ok and e[3] <= gu.TOL_BF16_OUT and e[4] <= gu.TOL_F32_OUT and torch.equal(y2, y) and np.array_equal(gu.host_f64(yp), rp) and np.array_equal(am.cpu().numpy(), ra)
        if not ok:
            bad.append((shape, [f"{v:.2e}" for v in e]))
    assert not bad, bad


def test_random_fc_shapes_match_oracle(orc):
    """Seeded random FC shapes (batch 1..300, widths 8..5000, odd sizes included): forward with bias + ReLU, data
    gradient and weight gradient against the oracle, whatever tile and split count the shape picks."""
    import paper_1811_01532_amd as wap
    rng = np.random.default_rng(31)
    bad = []
    for ci in range(40):
        B = int(rng.choice([1, 2, 5, 8, 16, 31, 32, 64, 100, 128, 257, 300]))
        n_in = int(rng.choice([8, 24, 100, 256, 1000, 1024, 2048, 4096, 4104, 5000]))
        n_out = int(rng.choice([8, 10, 37, 64, 125, 512, 1000, 1024, 4096]))
        print(f"[case] fc sweep #{ci} B={B} in={n_in} out={n_out}", flush=True)
        xb = si.normal_bf16(si.rng(9500 + ci, 0), (B, n_in))
        Wb = si.he_weight_bf16(si.rng(9500 + ci, 1), (n_out, n_in))
        gb = si.normal_bf16(si.rng(9500 + ci, 2), (B, n_out))
        bias = si.rng(9500 + ci, 3).standard_normal(n_out).astype(np.float32)
        x64, W64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(Wb), orc.bf16_bits_to_f64(gb)
        xd, Wd, gd = gu.dev_bf16(xb), gu.dev_bf16(Wb), gu.dev_bf16(gb)
        d = wap.fc_desc(B, n_in, n_out, relu=True)
        ws = gu.workspace(max(wap.wap_fc_workspace_bytes(d, p) for p in (0, 1, 2)))
        y = torch.full((B, n_out), float("nan"), dtype=torch.bfloat16, device="cuda")
        dx = torch.full((B, n_in), float("nan"), dtype=torch.bfloat16, device="cuda")
        dW = torch.full((n_out, n_in), float("nan"), dtype=torch.float32, device="cuda")
        wap.wap_fc_fwd(d, xd, Wd, torch.from_numpy(bias).cuda(), y, ws)
        wap.wap_fc_bwd(d, xd, Wd, gd, dx, dW, ws)
        torch.cuda.synchronize()
        e = [gu.rel_err(gu.host_f64(y), orc.fc_fwd(x64, W64, bias=bias.astype(np.float64), relu=True)),
             gu.rel_err(gu.host_f64(dx), orc.fc_bwd_data(g64, W64)),
             gu.rel_err(gu.host_f64(dW), orc.fc_bwd_weight(g64, x64))]
        w0 = (torch.randn((n_out, n_in), device="cuda", generator=torch.Generator(device="cuda").manual_seed(ci)) * 0.05)
        wm, wm2 = w0.clone(), w0.clone()
        wbf, wbf2 = torch.empty_like(wm, dtype=torch.bfloat16), torch.empty_like(wm, dtype=torch.bfloat16)
        scr = None if wap.wap_fc_bwd_weight_sgd_fused(d) else torch.empty_like(dW)
        wap.wap_fc_bwd_weight_sgd(d, xd, gd, wm, wbf, 0.05, scr, ws)
        wap.wap_sgd_update(n_out * n_in, wm2, dW, 0.05, wbf2)
        torch.cuda.synchronize()
        same = torch.equal(wm, wm2) and torch.equal(wbf.view(torch.int16), wbf2.view(torch.int16))
        if not (e[0] <= gu.TOL_BF16_OUT and e[1] <= gu.TOL_BF16_OUT and e[2] <= gu.TOL_F32_OUT and same):
            bad.append(((B, n_in, n_out), [f"{v:.2e}" for v in e], same))
    assert not bad, bad
