"""GPU parity: convolution forward / data gradient / weight gradient through the C ABI against the
fp64 oracle, element by element, on seeded inputs (same bf16 bits on both sides)."""
import sys

import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

# name, (N,H,W,C,K,R,S,stride,pad), (force fwd cfg, force wgrad cfg, force nsplit)
CASES = [
    ("config1_c3_k16", (4, 32, 32, 3, 16, 3, 3, 1, 1), (-1, -1, -1)),
    ("fast_128x128_ragged", (2, 20, 20, 64, 96, 3, 3, 1, 1), (-1, -1, -1)),
    ("fast_256x256_forced", (3, 19, 23, 128, 320, 3, 3, 1, 1), (0, 0, -1)),
    ("fast_256x256_forced_split3", (1, 17, 17, 192, 200, 3, 3, 1, 1), (0, 0, 3)),
    ("fast_rowthin_forced", (1, 9, 7, 64, 264, 3, 3, 1, 1), (2, 1, -1)),
    ("fast_chanthin", (2, 30, 30, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("fast_chanthin_k40", (1, 33, 31, 128, 40, 3, 3, 1, 1), (3, 2, 2)),
    ("vec_c24_k40_stride2", (2, 21, 19, 24, 40, 3, 3, 2, 1), (-1, -1, -1)),
    ("fast_stride2_dgrad_div", (2, 18, 18, 64, 128, 3, 3, 2, 1), (-1, -1, -1)),
    ("alexnet_conv1_like", (2, 35, 35, 3, 64, 11, 11, 4, 2), (-1, -1, -1)),
    ("alexnet_conv2_like_5x5", (2, 13, 13, 64, 192, 5, 5, 1, 2), (-1, -1, -1)),
    ("one_by_one", (2, 14, 14, 256, 128, 1, 1, 1, 0), (-1, -1, -1)),
    ("split_reduction_auto", (1, 8, 8, 256, 128, 3, 3, 1, 1), (-1, -1, -1)),
    ("odd_everything", (1, 7, 9, 5, 7, 3, 2, 1, 1), (-1, -1, -1)),
    ("k_not_multiple_of_4", (1, 6, 6, 8, 10, 3, 3, 1, 1), (-1, -1, -1)),
    ("rect_filter_stride_2_1", (1, 15, 12, 16, 24, 4, 3, (2, 1), (1, 0)), (-1, -1, -1)),
    # weights-in-registers kernel (ragged rows and columns, stride 2 forward, split reduction)
    ("wreg_forced_ragged", (2, 21, 23, 64, 200, 3, 3, 1, 1), (5, -1, -1)),
    ("wreg_forced_stride2_split2", (1, 30, 30, 128, 96, 3, 3, 2, 1), (5, -1, 2)),
    # a map wider than the 16-bit pixel coordinates of the weights-in-registers kernel: planned onto the generic tiles
    ("wide_map_1x1_w40000", (2, 1, 40000, 64, 256, 1, 1, 1, 0), (-1, -1, -1)),
    # patch-in-LDS kernel: chosen from the shape; ragged last tile, one and two channel slices, both widths
    ("patch_auto_k128_ragged", (2, 88, 88, 64, 128, 3, 3, 1, 1), (-1, -1, -1)),
    ("patch_auto_k256_two_slices", (1, 120, 121, 128, 256, 3, 3, 1, 1), (-1, -1, -1)),
    # 8 x 32-pixel 2-D tile kernel: chosen from the shape for 64 channels, forced for 128
    ("tile2d_auto_c64_k64", (2, 16, 64, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("tile2d_auto_c128_k64_3x2", (1, 24, 33, 128, 64, 3, 2, 1, (1, 0)), (-1, -1, -1)),
    ("tile2d_forced_c128_k128", (1, 24, 32, 128, 128, 3, 3, 1, 1), (7, -1, -1)),
    ("tile2d_auto_square_tiles_c64_k64", (2, 32, 48, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("tile2d_forced_square_tiles_c128_k128", (1, 16, 48, 128, 128, 3, 3, 1, 1), (7, -1, -1)),
    ("tile2d_forced_8x28_strip_tiles_c128_k256", (1, 16, 56, 128, 256, 3, 3, 1, 1), (7, -1, -1)),
    ("tile2d_forced_flat_tiles_w28_ragged", (3, 28, 28, 128, 256, 3, 3, 1, 1), (7, -1, -1)),
    ("tile2d_forced_flat_tiles_w14_straddling_images", (5, 14, 14, 64, 128, 3, 3, 1, 1), (7, -1, -1)),
    ("tile2d_forced_flat_192x64_tiles_5x5_w27_fwd", (3, 27, 27, 192, 64, 5, 5, 1, 2), (7, -1, -1)),
    ("tile2d_forced_flat_192x64_tiles_5x5_w27_dgrad", (3, 27, 27, 64, 192, 5, 5, 1, 2), (7, -1, -1)),
    ("tile2d_forced_flat_192x64_tiles_3x3_w30_even_unpool", (2, 30, 30, 64, 64, 3, 3, 1, 1), (7, -1, -1)),
    # patch-in-LDS weight gradient: masked surplus columns (14 -> 16), a forced uneven split, pad 0
    ("wgrad_patch_w14_masked_columns", (3, 14, 14, 128, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("wgrad_patch_w28_forced_split5", (1, 28, 28, 64, 128, 3, 3, 1, 1), (-1, 3, 5)),
    ("wgrad_patch_pad0_w30", (2, 34, 32, 64, 64, 3, 3, 1, 0), (-1, -1, -1)),
    ("wgrad_patch_w13_partly_masked_tile_rows", (3, 13, 13, 192, 128, 3, 3, 1, 1), (-1, -1, -1)),
    ("wgrad_patch_h22_w12_partly_masked_even", (2, 22, 12, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    # the remaining step maps of the patch weight gradient (block steps on 20 / 24 / 28-wide maps with 64 output
    # channels, half-row steps with 128, a ragged last tile row of the 4-row tiles), each also with the pooled dy
    ("wgrad_patch_blocks_w20_k64", (2, 12, 20, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("wgrad_patch_blocks_w24_k64_ragged_rows", (2, 10, 24, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("wgrad_patch_blocks_w28_k64", (2, 28, 28, 64, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("wgrad_patch_halfrows_w32_k128", (2, 12, 32, 64, 128, 3, 3, 1, 1), (-1, -1, -1)),
    ("wgrad_patch_blocks_w20_k128_two_tiles_per_row", (1, 12, 40, 128, 128, 3, 3, 1, 1), (-1, -1, -1)),
    # small shapes have short pixel ranges, for which the plan picks one 32-channel dy block per wavefront; the same
    # shapes with two blocks forced (the arrangement of the large layers), every step map, with and without pooled dy
    ("wgrad_patch_two_blocks_rows16_x8", (1, 8, 8, 256, 128, 3, 3, 1, 1), (-1, 5, -1)),
    ("wgrad_patch_two_blocks_blocks_w22", (2, 88, 88, 64, 128, 3, 3, 1, 1), (-1, 5, -1)),
    ("wgrad_patch_two_blocks_blocks_w28", (3, 28, 28, 128, 256, 3, 3, 1, 1), (7, 5, -1)),
    ("wgrad_patch_two_blocks_rows16_x7_w14", (5, 14, 14, 64, 128, 3, 3, 1, 1), (7, 5, -1)),
    ("wgrad_patch_two_blocks_halfrows_w32", (2, 12, 32, 64, 128, 3, 3, 1, 1), (-1, 5, -1)),
    ("wgrad_patch_two_blocks_blocks_w20", (1, 12, 40, 128, 128, 3, 3, 1, 1), (-1, 5, -1)),
    ("wgrad_patch_two_blocks_w13_masked_rows", (3, 13, 13, 192, 128, 3, 3, 1, 1), (-1, 5, -1)),
    # backward through a 2x2 pool routed in the loaders: flat data-gradient tiles, two dy blocks per wavefront
    ("unpool_flat_w14_c128_k128", (5, 14, 14, 128, 128, 3, 3, 1, 1), (7, -1, -1)),
    ("unpool_w112_c64_k128", (1, 32, 112, 64, 128, 3, 3, 1, 1), (-1, -1, -1)),
    ("unpool_5x5_flat_tiles_c64_k64", (2, 32, 32, 64, 64, 5, 5, 1, 2), (7, -1, -1)),
    ("unpool_1x3_filter_2d_tiles_c64_k64", (2, 16, 64, 64, 64, 1, 3, 1, (0, 1)), (7, -1, -1)),
    # 3-input-channel first-layer kernels: ragged last tile / step, 32 and 64 output channels, pad 0
    ("c3_k64_ragged", (3, 41, 40, 3, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("c3_k32", (2, 48, 48, 3, 32, 3, 3, 1, 1), (-1, -1, -1)),
    ("c3_k64_pad0", (2, 50, 50, 3, 64, 3, 3, 1, 0), (-1, -1, -1)),
    # ... with whole 32-pixel tiles per output row and even input rows: input rows staged in LDS (pad 1, pad 0, pad 2)
    ("c3_rows_k64_w64", (3, 21, 64, 3, 64, 3, 3, 1, 1), (-1, -1, -1)),
    ("c3_rows_k32_w66_pad0", (2, 19, 66, 3, 32, 3, 3, 1, 0), (-1, -1, -1)),
    ("c3_rows_k64_w94_pad2", (2, 12, 94, 3, 64, 3, 3, 1, 2), (-1, -1, -1)),
    ("c3_general_5x5_s2_k32", (9, 63, 61, 3, 32, 5, 5, 2, 2), (-1, -1, -1)),
    ("c3_general_11x11_s4_k64", (4, 131, 135, 3, 64, 11, 11, 4, 2), (-1, -1, -1)),
    ("c3_general_7x3_rect_stride_1_3", (3, 20, 40, 3, 64, 7, 3, (1, 3), (3, 0)), (-1, -1, -1)),
    # 3 input channels, horizontal stride 4: weight gradient from input rows held in LDS (no gather)
    ("c3_strided_wgrad_11x11_s4_k64", (5, 64, 72, 3, 64, 11, 11, 4, 2), (-1, -1, -1)),
    ("c3_strided_wgrad_7x7_s4_k32", (6, 50, 96, 3, 32, 7, 7, 4, 2), (-1, -1, -1)),
    ("c3_strided_wgrad_5x9_rect_stride_2_4_pad_1_0", (8, 30, 64, 3, 64, 5, 9, (2, 4), (1, 0)), (-1, -1, -1)),
]


def _tup(v):
    return (v, v) if isinstance(v, int) else tuple(v)


@pytest.mark.parametrize("name,shape,force", CASES, ids=[c[0] for c in CASES])
def test_conv_three_passes_match_oracle(orc, name, shape, force):
    import paper_1811_01532_amd as wap
    N, H, W, C, K, R, S, stride, pad = shape
    stride, pad = _tup(stride), _tup(pad)
    print(f"[case] {name} shape={shape} force={force}", flush=True)
    sys.stdout.flush()
    ci = [c[0] for c in CASES].index(name)
    xb = si.normal_bf16(si.rng(100 + ci, 0), (N, H, W, C))
    wb = si.he_weight_bf16(si.rng(100 + ci, 1), (K, R, S, C))
    P, Q = si.out_dim(H, pad[0], R, stride[0]), si.out_dim(W, pad[1], S, stride[1])
    gb = si.normal_bf16(si.rng(100 + ci, 2), (N, P, Q, K))
    bias = si.rng(100 + ci, 3).standard_normal(K).astype(np.float32)
    x64, w64, g64 = orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(wb), orc.bf16_bits_to_f64(gb)

    xd, wd, gd = gu.dev_bf16(xb), gu.dev_bf16(wb), gu.dev_bf16(gb)
    bd = torch.from_numpy(bias).cuda()
    wap.lib().wap_debug_force(*force)
    try:
        # ---- forward, plain ----
        d = wap.conv_desc(N, H, W, C, K, R, S, stride, pad, relu=False)
        y = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_FWD))
        wap.wap_conv2d_fwd(d, xd, wd, None, y, ws)
        torch.cuda.synchronize()
        ref = orc.conv2d_fwd(x64, w64, stride, pad)
        e = gu.rel_err(gu.host_f64(y), ref)
        assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"fwd rel err {e}"
        # ---- forward, bias + ReLU epilogue ----
        d2 = wap.conv_desc(N, H, W, C, K, R, S, stride, pad, relu=True)
        y2 = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
        wap.wap_conv2d_fwd(d2, xd, wd, bd, y2, ws)
        torch.cuda.synchronize()
        ref2 = orc.conv2d_fwd(x64, w64, stride, pad, bias=bias.astype(np.float64), relu=True)
        got2 = gu.host_f64(y2)
        e = gu.rel_err(got2, ref2)
        assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"fwd+bias+relu rel err {e}"
        assert np.all(got2 >= 0.0)
        # ---- forward + 2x2 max-pool in one call: the oracle's pool of the device's own conv output (teacher
        # forcing) bit for bit; where the kernel pools in its epilogue, also without the full-size output ----
        if P % 2 == 0 and Q % 2 == 0:
            yp = torch.full((N, P // 2, Q // 2, K), float("nan"), dtype=torch.bfloat16, device="cuda")
            am = torch.full((N, P // 2, Q // 2, K), 77, dtype=torch.uint8, device="cuda")
            y3 = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
            wap.wap_conv2d_fwd_pool2x2(d2, xd, wd, bd, y3, yp, am, ws)
            torch.cuda.synchronize()
            assert torch.equal(y3, y2)
            ref_p, ref_am = orc.maxpool_fwd(got2, 2, 2)
            assert np.array_equal(gu.host_f64(yp), ref_p) and np.array_equal(am.cpu().numpy(), ref_am)
            if wap.wap_conv2d_fwd_pool2x2_fused(d2):
                yp2 = torch.full_like(yp, float("nan"))
                am2 = torch.full_like(am, 77)
                wap.wap_conv2d_fwd_pool2x2(d2, xd, wd, bd, None, yp2, am2, ws)
                torch.cuda.synchronize()
                assert torch.equal(yp2, yp) and torch.equal(am2, am)
        # ---- data gradient ----
        dx = torch.full((N, H, W, C), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_DATA))
        wap.wap_conv2d_bwd_data(d, gd, wd, dx, ws)
        torch.cuda.synchronize()
        refdx = orc.conv2d_bwd_data(g64, w64, (N, H, W, C), stride, pad)
        e = gu.rel_err(gu.host_f64(dx), refdx)
        assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"dgrad rel err {e}"
        # ---- data gradient fused with the ReLU derivative of the producer of x (mask = relu(x) > 0);
        # bitwise the same as masking the plain data gradient afterwards ----
        xact = torch.relu(xd)
        dxm = torch.full((N, H, W, C), float("nan"), dtype=torch.bfloat16, device="cuda")
        wap.wap_conv2d_bwd_data_relu(d, gd, wd, xact, dxm, ws)
        torch.cuda.synchronize()
        refm = orc.relu_bwd(refdx, np.maximum(x64, 0.0))
        e = gu.rel_err(gu.host_f64(dxm), refm)
        assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"dgrad+relu rel err {e}"
        keep = (xact > 0)
        assert torch.equal(torch.where(keep, dx, torch.zeros_like(dx)), dxm)
        # ---- weight gradient (fp32 out) ----
        dw = torch.full((K, R, S, C), float("nan"), dtype=torch.float32, device="cuda")
        ws = gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_WEIGHT))
        wap.wap_conv2d_bwd_weight(d, xd, gd, dw, ws)
        torch.cuda.synchronize()
        refdw = orc.conv2d_bwd_weight(x64, g64, (K, R, S, C), stride, pad)
        e = gu.rel_err(gu.host_f64(dw), refdw)
        assert e <= gu.TOL and e <= gu.TOL_F32_OUT, f"wgrad rel err {e}"
        # split reductions are summed in a fixed order: bitwise reproducible
        dw2 = torch.empty_like(dw)
        wap.wap_conv2d_bwd_weight(d, xd, gd, dw2, ws)
        torch.cuda.synchronize()
        assert torch.equal(dw, dw2)
        # ---- weight gradient with the SGD update applied by the kernel that finishes it: against the oracle's
        # gradient followed by its update, and bit for bit against the device's own two-call chain ----
        lr = 0.05
        w32_0 = (si.rng(100 + ci, 6).standard_normal((K, R, S, C)) * 0.05).astype(np.float32)
        wm, wm2 = torch.from_numpy(w32_0).cuda(), torch.from_numpy(w32_0).cuda()
        wbf = torch.full((K, R, S, C), float("nan"), dtype=torch.bfloat16, device="cuda")
        wbf2 = torch.full((K, R, S, C), float("nan"), dtype=torch.bfloat16, device="cuda")
        dws = None if wap.wap_conv2d_bwd_weight_sgd_fused(d) else torch.empty_like(dw)
        wap.wap_conv2d_bwd_weight_sgd(d, xd, gd, wm, wbf, lr, dws, ws)
        wap.wap_sgd_update(K * R * S * C, wm2, dw, lr, wbf2)
        torch.cuda.synchronize()
        assert torch.equal(wm, wm2) and torch.equal(wbf.view(torch.int16), wbf2.view(torch.int16)), "wgrad+sgd vs two calls"
        lr32 = float(np.float32(lr))
        refw = orc.sgd(w32_0.astype(np.float64), refdw, lr32)
        bound = gu.TOL_F32_OUT * lr32 * np.max(np.abs(refdw)) + 2.0 ** -22 * np.max(np.abs(refw))
        assert np.max(np.abs(gu.host_f64(wm) - refw)) <= bound, "wgrad+sgd vs oracle"
        assert np.array_equal(gu.host_f64(wbf), orc.round_bf16(gu.host_f64(wm))), "bf16 copy"
        # ---- both backward passes with dy given as the gradient of the 2x2 / stride-2 pooled output plus the pool's
        # argmax: against the oracle's max-pool backward followed by its data / weight gradient, and bit for bit
        # against the device's own unfused chain; where the loader routes the gradient itself, also without the
        # full-size scratch tensor ----
        if P % 2 == 0 and Q % 2 == 0:
            gpb = si.normal_bf16(si.rng(100 + ci, 4), (N, P // 2, Q // 2, K))
            amh = si.rng(100 + ci, 5).integers(0, 4, size=(N, P // 2, Q // 2, K), dtype=np.uint8)
            gpd, amd = gu.dev_bf16(gpb), torch.from_numpy(amh).cuda()
            routed64 = orc.maxpool_bwd(orc.bf16_bits_to_f64(gpb), amh, (N, P, Q, K), 2, 2)
            dyf = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
            wap.wap_maxpool_bwd(N, P, Q, K, 2, 2, gpd, amd, None, dyf)
            torch.cuda.synchronize()
            assert np.array_equal(gu.host_f64(dyf), routed64)
            wsd = gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_DATA))
            wsw = gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_WEIGHT))
            dxu = torch.full((N, H, W, C), float("nan"), dtype=torch.bfloat16, device="cuda")
            wap.wap_conv2d_bwd_data_relu(d, dyf, wd, xact, dxu, wsd)
            dwu = torch.full((K, R, S, C), float("nan"), dtype=torch.float32, device="cuda")
            wap.wap_conv2d_bwd_weight(d, xd, dyf, dwu, wsw)
            torch.cuda.synchronize()
            refdx_p = orc.relu_bwd(orc.conv2d_bwd_data(routed64, w64, (N, H, W, C), stride, pad), np.maximum(x64, 0.0))
            refdw_p = orc.conv2d_bwd_weight(x64, routed64, (K, R, S, C), stride, pad)
            fused = (wap.wap_conv2d_bwd_pool2x2_fused(d, wap.WAP_PASS_BWD_DATA),
                     wap.wap_conv2d_bwd_pool2x2_fused(d, wap.WAP_PASS_BWD_WEIGHT))
            print(f"[case] {name} unpool fused (dgrad, wgrad) = {fused}", flush=True)
            for with_scratch in (True, False):
                scratch = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda") if with_scratch else None
                if with_scratch or fused[0]:
                    dxp = torch.full((N, H, W, C), float("nan"), dtype=torch.bfloat16, device="cuda")
                    wap.wap_conv2d_bwd_data_pool2x2(d, gpd, amd, wd, xact, dxp, scratch, wsd)
                    torch.cuda.synchronize()
                    e = gu.rel_err(gu.host_f64(dxp), refdx_p)
                    assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, f"unpool+dgrad rel err {e}"
                    assert torch.equal(dxp, dxu)
                if with_scratch or fused[1]:
                    dwp = torch.full((K, R, S, C), float("nan"), dtype=torch.float32, device="cuda")
                    wap.wap_conv2d_bwd_weight_pool2x2(d, xd, gpd, amd, dwp, scratch, wsw)
                    torch.cuda.synchronize()
                    e = gu.rel_err(gu.host_f64(dwp), refdw_p)
                    assert e <= gu.TOL and e <= gu.TOL_F32_OUT, f"unpool+wgrad rel err {e}"
                    assert torch.equal(dwp, dwu)
            if not fused[0]:
                with pytest.raises(wap.WapError):
                    wap.wap_conv2d_bwd_data_pool2x2(d, gpd, amd, wd, xact, dxu, None, wsd)
    finally:
        wap.lib().wap_debug_force(-1, -1, -1)


def test_delta_filter_is_an_exact_shift_on_the_gpu(orc):
    """The delta-filter invariant holds bit for bit on the device too (a single 1.0 weight)."""
    import paper_1811_01532_amd as wap
    N, H, W, C, K, R, S = 2, 12, 12, 64, 64, 3, 3
    xb = si.normal_bf16(si.rng(150, 0), (N, H, W, C))
    w = np.zeros((K, R, S, C), dtype=np.float32)
    w[5, 0, 2, 17] = 1.0
    wb = si.f32_to_bf16_bits(w)
    d = wap.conv_desc(N, H, W, C, K, R, S, 1, 1)
    y = torch.empty((N, H, W, K), dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_FWD))
    print("[case] delta filter", flush=True)
    wap.wap_conv2d_fwd(d, gu.dev_bf16(xb), gu.dev_bf16(wb), None, y, ws)
    torch.cuda.synchronize()
    got = gu.host_bits(y)
    want = np.zeros((N, H, W, K), dtype=np.uint16)
    # y[n,p,q,5] = x[n,p-1,q+1,17]
    want[:, 1:, :-1, 5] = xb[:, :-1, 1:, 17]
    # -0.0 inputs may surface as +0.0 after accumulation: compare values, not zero signs
    assert np.array_equal(orc.bf16_bits_to_f64(got), orc.bf16_bits_to_f64(want))
