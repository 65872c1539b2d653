"""GPU parity at the full benchmark sizes (VGG-16 layers at per-GPU minibatch 64, AlexNet-style
layers at 32, the VGG FC head), in the launch configuration bench.py times (shape-driven tile
choice, no forcing).  The full fp64 oracle is too slow at these sizes, so every output tensor is
checked on seeded sampled coordinates plus the border rows / columns of the first image, each
computed one by one by the oracle's *_at entry points (every output element is an independent
dot product)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

# name, N, H, C, K, R, stride, pad
LAYERS = [
    ("vgg_conv1_1_b64", 64, 224, 3, 64, 3, 1, 1),
    ("vgg_conv1_2_b64", 64, 224, 64, 64, 3, 1, 1),
    ("vgg_conv2_1_b64", 64, 112, 64, 128, 3, 1, 1),     # 128-channel 2-D tiles forward, 64-channel tiles backward
    ("vgg_conv3_1_b64", 64, 56, 128, 256, 3, 1, 1),
    ("vgg_conv3_2_b64", 64, 56, 256, 256, 3, 1, 1),
    ("vgg_conv4_1_b64", 64, 28, 256, 512, 3, 1, 1),
    ("vgg_conv4_2_b64", 64, 28, 512, 512, 3, 1, 1),
    ("vgg_conv5_1_b64", 64, 14, 512, 512, 3, 1, 1),
    ("alex_conv1_b32", 32, 224, 3, 64, 11, 4, 2),
    ("alex_conv2_b32", 32, 27, 64, 192, 5, 1, 2),
    ("alex_conv3_b32", 32, 13, 192, 384, 3, 1, 1),
    ("alex_conv4_b32", 32, 13, 384, 256, 3, 1, 1),
    ("alex_conv5_b32", 32, 13, 256, 256, 3, 1, 1),
    # small minibatches: the tile rules differ there (thin flat tiles, split reductions of the generic kernel)
    ("vgg_conv4_2_b8", 8, 28, 512, 512, 3, 1, 1),
    ("vgg_conv4_2_b16", 16, 28, 512, 512, 3, 1, 1),
    ("vgg_conv5_1_b8", 8, 14, 512, 512, 3, 1, 1),
    ("vgg_conv5_1_b16", 16, 14, 512, 512, 3, 1, 1),
]


def _border_indices(shape, rng, n_random):
    """Flat indices: n_random uniform ones plus first/last rows and columns of image 0 (a few channels)."""
    N, A, B, C = shape
    idx = [rng.integers(0, N * A * B * C, n_random)]
    chans = np.unique(np.array([0, C // 2, C - 1]))
    for a in (0, A - 1):
        b = np.arange(B)
        for c in chans:
            idx.append((a * B + b) * C + c)
    for b in (0, B - 1):
        a = np.arange(A)
        for c in chans:
            idx.append((a * B + b) * C + c)
    return np.unique(np.concatenate(idx)).astype(np.int64)


@pytest.mark.parametrize("name,N,H,C,K,R,stride,pad", LAYERS, ids=[l[0] for l in LAYERS])
def test_conv_layer_full_size_sampled(orc, name, N, H, C, K, R, stride, pad):
    import paper_1811_01532_amd as wap
    li = [l[0] for l in LAYERS].index(name)
    P = si.out_dim(H, pad, R, stride)
    print(f"[case] full-size {name}: x {N}x{H}x{H}x{C}, y {N}x{P}x{P}x{K}", flush=True)
    xb = si.normal_bf16(si.rng(600 + li, 0), (N, H, H, C))
    wb = si.he_weight_bf16(si.rng(600 + li, 1), (K, R, R, C))
    gb = si.normal_bf16(si.rng(600 + li, 2), (N, P, P, K))
    xd, wd, gd = gu.dev_bf16(xb), gu.dev_bf16(wb), gu.dev_bf16(gb)
    d = wap.conv_desc(N, H, H, C, K, R, R, stride, pad, relu=True)
    y = torch.empty((N, P, P, K), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((N, H, H, C), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((K, R, R, C), dtype=torch.float32, device="cuda")
    wap.wap_conv2d_fwd(d, xd, wd, None, y, gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_FWD)))
    wap.wap_conv2d_bwd_data(d, gd, wd, dx, gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_DATA)))
    wap.wap_conv2d_bwd_weight(d, xd, gd, dw, gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_WEIGHT)))
    torch.cuda.synchronize()
    yh = y.view(torch.int16).cpu().numpy().view(np.uint16).ravel()
    dxh = dx.view(torch.int16).cpu().numpy().view(np.uint16).ravel()
    dwh = dw.cpu().numpy().astype(np.float64).ravel()
    del xd, gd, y, dx
    torch.cuda.empty_cache()
    assert np.all(np.isfinite(dwh))

    x64, w64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(wb), orc.bf16_bits_to_f64(gb)
    del xb, gb
    rng = np.random.default_rng(700 + li)
    s2, p2 = (stride, stride), (pad, pad)
    # forward (+ReLU epilogue)
    iy = _border_indices((N, P, P, K), rng, 4096)
    ref = orc.conv2d_fwd_at(x64, w64, iy, s2, p2, relu=True)
    e = gu.rel_err(orc.bf16_bits_to_f64(yh[iy]), ref)
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"{name} fwd sampled rel err {e}"
    # data gradient
    ix = _border_indices((N, H, H, C), rng, 4096)
    ref = orc.conv2d_bwd_data_at(g64, w64, (N, H, H, C), ix, s2, p2)
    e = gu.rel_err(orc.bf16_bits_to_f64(dxh[ix]), ref)
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"{name} dgrad sampled rel err {e}"
    # weight gradient: each sample is a full N*P*Q reduction
    n_w = 256 if N * P * P > 500000 else 1024
    iw = np.unique(rng.integers(0, K * R * R * C, n_w)).astype(np.int64)
    ref = orc.conv2d_bwd_weight_at(x64, g64, (K, R, R, C), iw, s2, p2)
    e = gu.rel_err(dwh[iw], ref)
    assert e <= gu.TOL and e <= gu.TOL_F32_OUT, f"{name} wgrad sampled rel err {e}"


@pytest.mark.parametrize("name,B,n_in,n_out", [("vgg_fc6_b64", 64, 25088, 4096), ("alex_fc6_b32", 32, 9216, 4096),
                                                ("fc8_b64", 64, 4096, 1000), ("fc7_b512", 512, 4096, 4096)])
def test_fc_layer_full_size_sampled(orc, name, B, n_in, n_out):
    import paper_1811_01532_amd as wap
    print(f"[case] full-size {name}", flush=True)
    g = si.rng(650, n_in + B)
    xb = si.normal_bf16(g, (B, n_in))
    Wb = si.he_weight_bf16(g, (n_out, n_in))
    gb = si.normal_bf16(g, (B, n_out))
    xd, Wd, gd = gu.dev_bf16(xb), gu.dev_bf16(Wb), gu.dev_bf16(gb)
    d = wap.fc_desc(B, n_in, n_out, relu=True)
    y = torch.empty((B, n_out), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((B, n_in), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((n_out, n_in), dtype=torch.float32, device="cuda")
    need = max(wap.wap_fc_workspace_bytes(d, p) for p in (0, 1, 2))
    ws = gu.workspace(need)
    wap.wap_fc_fwd(d, xd, Wd, None, y, ws)
    wap.wap_fc_bwd(d, xd, Wd, gd, dx, dW, ws)
    torch.cuda.synchronize()
    x64, W64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(Wb), orc.bf16_bits_to_f64(gb)
    rng = np.random.default_rng(651)
    # sampled rows / columns evaluated with the oracle's own routines on sub-matrices
    rows = np.unique(rng.integers(0, B, 8))
    cols = np.unique(np.concatenate([rng.integers(0, n_out, 64), [0, n_out - 1]]))
    ref = orc.fc_fwd(x64[rows], W64[cols], relu=True)
    got = gu.host_f64(y)[np.ix_(rows, cols)]
    e = gu.rel_err(got, ref)
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"{name} fwd rel err {e}"
    icols = np.unique(np.concatenate([rng.integers(0, n_in, 64), [0, n_in - 1]]))
    ref = orc.fc_bwd_data(g64[rows], np.ascontiguousarray(W64[:, icols]))
    e = gu.rel_err(gu.host_f64(dx)[np.ix_(rows, icols)], ref)
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"{name} dx rel err {e}"
    ref = orc.fc_bwd_weight(np.ascontiguousarray(g64[:, cols]), np.ascontiguousarray(x64[:, icols]))
    e = gu.rel_err(gu.host_f64(dW)[np.ix_(cols, icols)], ref)
    assert e <= gu.TOL and e <= gu.TOL_F32_OUT, f"{name} dW rel err {e}"
    # the weight gradient that applies the SGD update itself (the form the launch list runs): bit for bit the
    # separate update with the gradient above, and the sampled weights against oracle gradient + oracle update
    lr = 0.05
    w0 = (torch.randn((n_out, n_in), device="cuda", generator=torch.Generator(device="cuda").manual_seed(652)) * 0.05)
    wm, wm2 = w0.clone(), w0.clone()
    wbf = torch.empty((n_out, n_in), dtype=torch.bfloat16, device="cuda")
    wbf2 = torch.empty((n_out, n_in), dtype=torch.bfloat16, device="cuda")
    assert wap.wap_fc_bwd_weight_sgd_fused(d)
    wap.wap_fc_bwd_weight_sgd(d, xd, gd, wm, wbf, lr, None, ws)
    wap.wap_sgd_update(n_out * n_in, wm2, dW, lr, wbf2)
    torch.cuda.synchronize()
    assert torch.equal(wm, wm2) and torch.equal(wbf.view(torch.int16), wbf2.view(torch.int16)), name + " dW+sgd"
    w0s = w0[torch.from_numpy(cols).cuda()][:, torch.from_numpy(icols).cuda()].double().cpu().numpy()
    refw = orc.sgd(w0s, ref, float(np.float32(lr)))
    gots = wm[torch.from_numpy(cols).cuda()][:, torch.from_numpy(icols).cuda()].double().cpu().numpy()
    bound = gu.TOL_F32_OUT * float(np.float32(lr)) * np.max(np.abs(ref)) + 2.0 ** -22 * np.max(np.abs(refw))
    assert np.max(np.abs(gots - refw)) <= bound, name + " dW+sgd vs oracle"


# VGG-16 layers that are followed by a 2x2 pool, at per-GPU minibatch 64: name, N, H, C, K
POOLED = [
    ("vgg_conv1_2_b64", 64, 224, 64, 64),
    ("vgg_conv2_2_b64", 64, 112, 128, 128),
    ("vgg_conv3_3_b64", 64, 56, 256, 256),
    ("vgg_conv4_3_b64", 64, 28, 512, 512),
]


@pytest.mark.parametrize("name,N,H,C,K", POOLED, ids=[l[0] for l in POOLED])
def test_pooled_layer_fused_paths_full_size(orc, name, N, H, C, K):
    """The conv -> ReLU -> 2x2 pool chain as the step plan runs it: pool taken in the forward kernel's epilogue, pool
    backward routed in the loaders of both backward kernels.  Each fused call is compared bit for bit with the
    device's own unfused chain, and the backward results on sampled coordinates with the oracle (max-pool backward,
    then one dot product per sample)."""
    import paper_1811_01532_amd as wap
    li = [l[0] for l in POOLED].index(name)
    print(f"[case] full-size fused pool paths {name}", flush=True)
    xb = si.normal_bf16(si.rng(800 + li, 0), (N, H, H, C))
    wb = si.he_weight_bf16(si.rng(800 + li, 1), (K, 3, 3, C))
    gpb = si.normal_bf16(si.rng(800 + li, 2), (N, H // 2, H // 2, K))
    amh = si.rng(800 + li, 3).integers(0, 4, size=(N, H // 2, H // 2, K), dtype=np.uint8)
    xd, wd, gpd, amd = gu.dev_bf16(xb), gu.dev_bf16(wb), gu.dev_bf16(gpb), torch.from_numpy(amh).cuda()
    d = wap.conv_desc(N, H, H, C, K, 3, 3, 1, 1, relu=True)
    ws = gu.workspace(max(wap.wap_conv2d_workspace_bytes(d, p) for p in (0, 1, 2)))
    # ---- forward + pool ----
    y = torch.empty((N, H, H, K), dtype=torch.bfloat16, device="cuda")
    yp = torch.empty((N, H // 2, H // 2, K), dtype=torch.bfloat16, device="cuda")
    am = torch.empty((N, H // 2, H // 2, K), dtype=torch.uint8, device="cuda")
    wap.wap_conv2d_fwd(d, xd, wd, None, y, ws)
    wap.wap_maxpool_fwd(N, H, H, K, 2, 2, y, yp, am)
    if wap.wap_conv2d_fwd_pool2x2_fused(d):
        yp2, am2 = torch.full_like(yp, float("nan")), torch.full_like(am, 77)
        wap.wap_conv2d_fwd_pool2x2(d, xd, wd, None, None, yp2, am2, ws)
        torch.cuda.synchronize()
        assert torch.equal(yp2, yp) and torch.equal(am2, am), f"{name}: fused forward pool differs"
        del yp2, am2
    del y, yp, am
    # ---- backward through the pool ----
    fused = (wap.wap_conv2d_bwd_pool2x2_fused(d, wap.WAP_PASS_BWD_DATA),
             wap.wap_conv2d_bwd_pool2x2_fused(d, wap.WAP_PASS_BWD_WEIGHT))
    assert fused == (True, True), f"{name}: the benchmark's launch list expects both passes fused, got {fused}"
    xact = torch.relu(xd)
    dyf = torch.empty((N, H, H, K), dtype=torch.bfloat16, device="cuda")
    wap.wap_maxpool_bwd(N, H, H, K, 2, 2, gpd, amd, None, dyf)
    dxu = torch.empty((N, H, H, C), dtype=torch.bfloat16, device="cuda")
    dwu = torch.empty((K, 3, 3, C), dtype=torch.float32, device="cuda")
    wap.wap_conv2d_bwd_data_relu(d, dyf, wd, xact, dxu, ws)
    wap.wap_conv2d_bwd_weight(d, xd, dyf, dwu, ws)
    del dyf
    dxp = torch.full_like(dxu, float("nan"))
    dwp = torch.full_like(dwu, float("nan"))
    wap.wap_conv2d_bwd_data_pool2x2(d, gpd, amd, wd, xact, dxp, None, ws)
    wap.wap_conv2d_bwd_weight_pool2x2(d, xd, gpd, amd, dwp, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(dxp, dxu), f"{name}: fused unpool + data gradient differs from the unfused chain"
    assert torch.equal(dwp, dwu), f"{name}: fused unpool + weight gradient differs from the unfused chain"
    dxh = dxp.view(torch.int16).cpu().numpy().view(np.uint16).ravel()
    dwh = dwp.cpu().numpy().astype(np.float64).ravel()
    del xd, xact, dxu, dxp, gpd, amd
    torch.cuda.empty_cache()
    # ---- oracle on samples ----
    x64, w64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(wb)
    routed = orc.maxpool_bwd(orc.bf16_bits_to_f64(gpb), amh, (N, H, H, K), 2, 2)
    rng = np.random.default_rng(900 + li)
    ix = _border_indices((N, H, H, C), rng, 4096)
    ref = orc.conv2d_bwd_data_at(routed, w64, (N, H, H, C), ix, (1, 1), (1, 1))
    ref = np.where(x64.ravel()[ix] > 0.0, ref, 0.0)
    e = gu.rel_err(orc.bf16_bits_to_f64(dxh[ix]), ref)
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"{name} unpool+dgrad sampled rel err {e}"
    iw = np.unique(rng.integers(0, K * 9 * C, 256 if N * H * H > 500000 else 1024)).astype(np.int64)
    ref = orc.conv2d_bwd_weight_at(x64, routed, (K, 3, 3, C), iw, (1, 1), (1, 1))
    e = gu.rel_err(dwh[iw], ref)
    assert e <= gu.TOL and e <= gu.TOL_F32_OUT, f"{name} unpool+wgrad sampled rel err {e}"


def test_vgg_conv5_3_with_its_separate_pool_backward_full_size(orc):
    """The last pooled VGG-16 layer keeps separate pooling kernels (its 14 x 14 map gives weight-gradient tiles that
    pooling windows would straddle): conv5_3 forward, 2x2 pool, pool backward with the ReLU mask, data gradient, at
    minibatch 64.  The pooling passes are compared with the oracle on the whole tensor, bit for bit (teacher forced on
    the device's own convolution output); the convolutions on sampled coordinates."""
    import paper_1811_01532_amd as wap
    N, H, C, K = 64, 14, 512, 512
    print("[case] full-size vgg conv5_3 + separate pool backward", flush=True)
    xb = np.maximum(si.normal_bf16(si.rng(950, 0), (N, H, H, C)).view(np.int16), 0).view(np.uint16)  # a ReLU output
    wb = si.he_weight_bf16(si.rng(950, 1), (K, 3, 3, C))
    gpb = si.normal_bf16(si.rng(950, 2), (N, H // 2, H // 2, K))
    xd, wd, gpd = gu.dev_bf16(xb), gu.dev_bf16(wb), gu.dev_bf16(gpb)
    d = wap.conv_desc(N, H, H, C, K, 3, 3, 1, 1, relu=True)
    ws = gu.workspace(max(wap.wap_conv2d_workspace_bytes(d, p) for p in (0, 1, 2)))
    y = torch.empty((N, H, H, K), dtype=torch.bfloat16, device="cuda")
    yp = torch.empty((N, H // 2, H // 2, K), dtype=torch.bfloat16, device="cuda")
    am = torch.empty((N, H // 2, H // 2, K), dtype=torch.uint8, device="cuda")
    dy = torch.empty((N, H, H, K), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((N, H, H, C), dtype=torch.bfloat16, device="cuda")
    wap.wap_conv2d_fwd(d, xd, wd, None, y, ws)
    wap.wap_maxpool_fwd(N, H, H, K, 2, 2, y, yp, am)
    wap.wap_maxpool_bwd(N, H, H, K, 2, 2, gpd, am, yp, dy)          # ReLU derivative fused: windows with y <= 0 dropped
    wap.wap_conv2d_bwd_data_relu(d, dy, wd, xd, dx, ws)
    torch.cuda.synchronize()
    y64 = gu.host_f64(y)
    ref_p, ref_am = orc.maxpool_fwd(y64, 2, 2)
    assert np.array_equal(gu.host_f64(yp), ref_p) and np.array_equal(am.cpu().numpy(), ref_am)
    g64 = orc.bf16_bits_to_f64(gpb)
    routed = orc.maxpool_bwd(np.where(ref_p > 0.0, g64, 0.0), ref_am, (N, H, H, K), 2, 2)
    assert np.array_equal(gu.host_f64(dy), routed)
    x64, w64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(wb)
    rng = np.random.default_rng(951)
    iy = _border_indices((N, H, H, K), rng, 4096)
    e = gu.rel_err(y64.ravel()[iy], orc.conv2d_fwd_at(x64, w64, iy, (1, 1), (1, 1), relu=True))
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"conv5_3 fwd sampled rel err {e}"
    ix = _border_indices((N, H, H, C), rng, 4096)
    ref = orc.conv2d_bwd_data_at(routed, w64, (N, H, H, C), ix, (1, 1), (1, 1))
    ref = np.where(x64.ravel()[ix] > 0.0, ref, 0.0)
    e = gu.rel_err(gu.host_f64(dx).ravel()[ix], ref)
    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"conv5_3 dgrad sampled rel err {e}"
