"""GPU parity: FC forward / backward and the memory-bound kernels (ReLU backward, max-pool,
softmax cross-entropy, SGD, cast) through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

FC_CASES = [
    # name, B, in, out, force(fwd cfg, wgrad cfg, nsplit)
    ("b16_256_1000", 16, 256, 1000, (-1, -1, -1)),
    ("odd_scalar_path", 5, 100, 37, (-1, -1, -1)),
    ("b64_1024_4096", 64, 1024, 4096, (-1, -1, -1)),
    ("b130_384_520", 130, 384, 520, (-1, -1, -1)),
    ("b512_128_264_big_tiles", 512, 128, 264, (0, 0, -1)),
    ("b8_2048_512_split", 8, 2048, 512, (-1, -1, -1)),
    ("b33_vec_general", 33, 72, 136, (-1, -1, -1)),
    # model-parallel shards of the VGG-16 head: out_features / 8 at the full minibatch
    ("fc8_shard_125", 64, 4096, 125, (-1, -1, -1)),
    ("fc6_shard_512", 64, 25088, 512, (-1, -1, -1)),
    # unsplit weight gradient (one tile per work-group, the update applied in its epilogue), and a row length
    # that is not a multiple of four, where the update cannot ride on the gradient kernel
    ("b64_4096_4096_unsplit", 64, 4096, 4096, (-1, -1, -1)),
    ("b16_2050_2048_update_apart", 16, 2050, 2048, (-1, -1, -1)),
]


@pytest.mark.parametrize("name,B,n_in,n_out,force", FC_CASES, ids=[c[0] for c in FC_CASES])
def test_fc_fwd_bwd_match_oracle(orc, name, B, n_in, n_out, force):
    import paper_1811_01532_amd as wap
    print(f"[case] fc {name}", flush=True)
    ci = [c[0] for c in FC_CASES].index(name)
    xb = si.normal_bf16(si.rng(200 + ci, 0), (B, n_in))
    Wb = si.he_weight_bf16(si.rng(200 + ci, 1), (n_out, n_in))
    gb = si.normal_bf16(si.rng(200 + ci, 2), (B, n_out))
    bias = si.rng(200 + ci, 3).standard_normal(n_out).astype(np.float32)
    x64, W64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(Wb), orc.bf16_bits_to_f64(gb)
    xd, Wd, gd = gu.dev_bf16(xb), gu.dev_bf16(Wb), gu.dev_bf16(gb)
    wap.lib().wap_debug_force(*force)
    try:
        for relu, b in ((False, None), (True, bias)):
            d = wap.fc_desc(B, n_in, n_out, relu=relu)
            y = torch.full((B, n_out), float("nan"), dtype=torch.bfloat16, device="cuda")
            ws = gu.workspace(wap.wap_fc_workspace_bytes(d, wap.WAP_PASS_FWD))
            wap.wap_fc_fwd(d, xd, Wd, None if b is None else torch.from_numpy(b).cuda(), y, ws)
            torch.cuda.synchronize()
            ref = orc.fc_fwd(x64, W64, bias=None if b is None else b.astype(np.float64), relu=relu)
            e = gu.rel_err(gu.host_f64(y), ref)
            assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"fc fwd relu={relu} rel err {e}"
        d = wap.fc_desc(B, n_in, n_out)
        need = max(wap.wap_fc_workspace_bytes(d, wap.WAP_PASS_BWD_DATA),
                   wap.wap_fc_workspace_bytes(d, wap.WAP_PASS_BWD_WEIGHT))
        ws = gu.workspace(need)
        dx = torch.full((B, n_in), float("nan"), dtype=torch.bfloat16, device="cuda")
        dW = torch.full((n_out, n_in), float("nan"), dtype=torch.float32, device="cuda")
        wap.wap_fc_bwd(d, xd, Wd, gd, dx, dW, ws)
        torch.cuda.synchronize()
        e = gu.rel_err(gu.host_f64(dx), orc.fc_bwd_data(g64, W64))
        assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"fc dx rel err {e}"
        e = gu.rel_err(gu.host_f64(dW), orc.fc_bwd_weight(g64, x64))
        assert e <= gu.TOL and e <= gu.TOL_F32_OUT, f"fc dW rel err {e}"
        # each half alone
        dx2 = torch.empty_like(dx)
        wap.wap_fc_bwd(d, None, Wd, gd, dx2, None, ws)
        dW2 = torch.empty_like(dW)
        wap.wap_fc_bwd(d, xd, None, gd, None, dW2, ws)
        torch.cuda.synchronize()
        assert torch.equal(dx, dx2) and torch.equal(dW, dW2)
        # weight gradient with the SGD update applied by the kernel that finishes it: bit for bit the two-call
        # chain, and the oracle's gradient followed by its update
        lr = 0.05
        w32_0 = (si.rng(200 + ci, 4).standard_normal((n_out, n_in)) * 0.05).astype(np.float32)
        wm, wm2 = torch.from_numpy(w32_0).cuda(), torch.from_numpy(w32_0).cuda()
        wbf = torch.full((n_out, n_in), float("nan"), dtype=torch.bfloat16, device="cuda")
        wbf2 = torch.full((n_out, n_in), float("nan"), dtype=torch.bfloat16, device="cuda")
        fused = wap.wap_fc_bwd_weight_sgd_fused(d)
        assert fused == (name != "b16_2050_2048_update_apart")
        wap.wap_fc_bwd_weight_sgd(d, xd, gd, wm, wbf, lr, None if fused else torch.empty_like(dW), ws)
        wap.wap_sgd_update(n_out * n_in, wm2, dW, lr, wbf2)
        torch.cuda.synchronize()
        assert torch.equal(wm, wm2) and torch.equal(wbf.view(torch.int16), wbf2.view(torch.int16))
        lr32 = float(np.float32(lr))
        refdW = orc.fc_bwd_weight(g64, x64)
        refw = orc.sgd(w32_0.astype(np.float64), refdW, lr32)
        bound = gu.TOL_F32_OUT * lr32 * np.max(np.abs(refdW)) + 2.0 ** -22 * np.max(np.abs(refw))
        assert np.max(np.abs(gu.host_f64(wm) - refw)) <= bound
        assert np.array_equal(gu.host_f64(wbf), orc.round_bf16(gu.host_f64(wm)))
        if not fused:
            with pytest.raises(wap.WapError):
                wap.wap_fc_bwd_weight_sgd(d, xd, gd, wm, wbf, lr, None, ws)
    finally:
        wap.lib().wap_debug_force(-1, -1, -1)


def test_relu_bwd(orc):
    import paper_1811_01532_amd as wap
    n = 8 * 1000 + 5
    yb = si.f32_to_bf16_bits(np.maximum(si.rng(300, 0).standard_normal(n).astype(np.float32), 0))
    gb = si.normal_bf16(si.rng(300, 1), (n,))
    yd, gd = gu.dev_bf16(yb), gu.dev_bf16(gb)
    dx = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    print("[case] relu_bwd", flush=True)
    wap.wap_relu_bwd(gd, yd, dx, n)
    torch.cuda.synchronize()
    ref = orc.relu_bwd(orc.bf16_bits_to_f64(gb), orc.bf16_bits_to_f64(yb))
    assert np.array_equal(gu.host_f64(dx), ref)
    # in place
    wap.wap_relu_bwd(gd, yd, gd, n)
    torch.cuda.synchronize()
    assert np.array_equal(gu.host_f64(gd), ref)


@pytest.mark.parametrize("shape,win,st", [((2, 14, 14, 64), 2, 2), ((2, 13, 13, 64), 3, 2),
                                           ((3, 9, 11, 3), 3, 2), ((1, 8, 6, 5), 2, 2),
                                           ((2, 55, 55, 64), 3, 2)])
def test_maxpool_fwd_bwd(orc, shape, win, st):
    import paper_1811_01532_amd as wap
    N, H, W, C = shape
    g = si.rng(310, H * 100 + C)
    # post-ReLU style input: non-negative with many exact zeros and repeated values (ties)
    x = np.maximum(np.round(g.standard_normal(shape).astype(np.float32) * 4) / 4, 0)
    xb = si.f32_to_bf16_bits(x)
    P, Q = si.out_dim(H, 0, win, st), si.out_dim(W, 0, win, st)
    gb = si.normal_bf16(g, (N, P, Q, C))
    xd, gd = gu.dev_bf16(xb), gu.dev_bf16(gb)
    y = torch.empty((N, P, Q, C), dtype=torch.bfloat16, device="cuda")
    am = torch.empty((N, P, Q, C), dtype=torch.uint8, device="cuda")
    print(f"[case] maxpool {shape} {win}/{st}", flush=True)
    wap.wap_maxpool_fwd(N, H, W, C, win, st, xd, y, am)
    torch.cuda.synchronize()
    x64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(gb)
    yref, amref = orc.maxpool_fwd(x64, win, st)
    assert np.array_equal(gu.host_f64(y), yref)
    assert np.array_equal(am.cpu().numpy(), amref)
    # backward without and with the fused ReLU mask
    dx = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    wap.wap_maxpool_bwd(N, H, W, C, win, st, gd, am, None, dx)
    torch.cuda.synchronize()
    ref = orc.maxpool_bwd(g64, amref, shape, win, st)
    got = gu.host_f64(dx)
    assert gu.rel_err(got, ref) <= gu.TOL_BF16_OUT
    assert abs(got.sum() - g64.sum()) <= 2.0 ** -8 * np.abs(g64).sum()
    dx2 = torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    wap.wap_maxpool_bwd(N, H, W, C, win, st, gd, am, y, dx2)
    torch.cuda.synchronize()
    ref2 = orc.relu_bwd(ref, x64)
    assert gu.rel_err(gu.host_f64(dx2), ref2) <= gu.TOL_BF16_OUT


@pytest.mark.parametrize("B,classes", [(16, 1000), (3, 11), (512, 1000)])
def test_softmax_xent_grad(orc, B, classes):
    import paper_1811_01532_amd as wap
    g = si.rng(320, B)
    zb = si.normal_bf16(g, (B, classes), std=3.0)
    labels = si.labels(g, B, classes)
    zd = gu.dev_bf16(zb)
    ld = torch.from_numpy(labels).cuda()
    loss = torch.zeros(4, dtype=torch.float32, device="cuda")
    rows = torch.zeros(B, dtype=torch.float32, device="cuda")
    dz = torch.empty((B, classes), dtype=torch.bfloat16, device="cuda")
    print(f"[case] softmax B={B}", flush=True)
    wap.wap_softmax_xent_grad(B, classes, zd, ld, loss, rows, dz)
    torch.cuda.synchronize()
    lref, dzref = orc.softmax_xent(orc.bf16_bits_to_f64(zb), labels)
    assert abs(float(loss[0]) - lref) <= 1e-5 * max(1.0, abs(lref))
    assert gu.rel_err(gu.host_f64(dz), dzref) <= gu.TOL_BF16_OUT


def test_softmax_zero_logits_gives_ln_classes(orc):
    import paper_1811_01532_amd as wap
    B, classes = 8, 1000
    zd = torch.zeros((B, classes), dtype=torch.bfloat16, device="cuda")
    ld = torch.arange(B, dtype=torch.int32, device="cuda")
    loss = torch.zeros(4, dtype=torch.float32, device="cuda")
    rows = torch.zeros(B, dtype=torch.float32, device="cuda")
    dz = torch.empty((B, classes), dtype=torch.bfloat16, device="cuda")
    wap.wap_softmax_xent_grad(B, classes, zd, ld, loss, rows, dz)
    torch.cuda.synchronize()
    assert abs(float(loss[0]) - np.log(1000.0)) < 1e-5


def test_sgd_and_cast(orc):
    import paper_1811_01532_amd as wap
    n = 4 * 777 + 3
    g = si.rng(330, 0)
    w = g.standard_normal(n).astype(np.float32)
    dw = g.standard_normal(n).astype(np.float32)
    wd, dwd = torch.from_numpy(w).cuda(), torch.from_numpy(dw).cuda()
    wb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    print("[case] sgd", flush=True)
    wap.wap_sgd_update(n, wd, dwd, 0.01, wb)
    torch.cuda.synchronize()
    ref = orc.sgd(w.astype(np.float64), dw.astype(np.float64), float(np.float32(0.01)))
    got = wd.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - ref)) <= 2.0 ** -23 * np.max(np.abs(ref))
    # the bf16 copy is the correctly rounded fp32 master
    assert np.array_equal(gu.host_f64(wb), orc.round_bf16(got))
    cb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    wap.wap_cast_f32_bf16(n, dwd, cb)
    torch.cuda.synchronize()
    assert np.array_equal(gu.host_f64(cb), orc.round_bf16(dw.astype(np.float64)))


@pytest.mark.parametrize("rows,cols", [(1000, 64), (37, 10), (257, 8), (5000, 4096), (200000, 64), (300001, 24), (1, 1000)])
def test_bias_grad(orc, rows, cols):
    """db = column sums of dy (fp32 accumulation of bf16 inputs) against the fp64 oracle; vector and scalar paths,
    more columns than one pass covers, chunk tails, a single row; two runs are bitwise equal."""
    import paper_1811_01532_amd as wap
    print(f"[case] bias_grad rows={rows} cols={cols}", flush=True)
    gb = si.normal_bf16(si.rng(420, rows % 1000 + cols), (rows, cols))
    gd = gu.dev_bf16(gb)
    ws = gu.workspace(wap.wap_bias_grad_workspace_bytes(rows, cols))
    db = torch.full((cols,), float("nan"), dtype=torch.float32, device="cuda")
    wap.wap_bias_grad(rows, cols, gd, db, ws)
    torch.cuda.synchronize()
    ref = orc.bias_grad(orc.bf16_bits_to_f64(gb))
    # fp32 running sums of up to rows / chunks values each: error grows like sqrt(rows) * 2^-24 of the magnitude
    scale = max(np.abs(ref).max(), np.sqrt(rows))
    assert np.max(np.abs(gu.host_f64(db) - ref)) <= 1e-5 * scale
    db2 = torch.empty_like(db)
    wap.wap_bias_grad(rows, cols, gd, db2, ws)
    torch.cuda.synchronize()
    assert torch.equal(db, db2)
