"""GPU check of the forward-convolution entry point that allocates nothing (its workspace is a static device array
inside the library): same bits as wap_conv2d_fwd with a caller workspace, and within the parity bound of the fp64
oracle, on consecutive calls that share the static array -- the second with a smaller input."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

# (N, H, W, C, K, R, S, stride, pad): first a layer whose workspace holds packed weights AND split-reduction partials
# (12.25 MiB of the 16 MiB array), then smaller ones: packed weights only, then the generic tiles
SEQUENCE = [
    (8, 14, 14, 512, 512, 3, 3, 1, 1),
    (2, 28, 28, 128, 256, 3, 3, 1, 1),
    (1, 9, 9, 64, 96, 3, 3, 1, 1),
    (2, 13, 13, 24, 40, 3, 3, 2, 1),
]


def test_static_workspace_forward_matches_caller_workspace_and_oracle(orc):
    import paper_1811_01532_amd as wap
    for rnd in range(2):                                   # the whole sequence twice: large after small as well
        for ci, (N, H, W, C, K, R, S, st, pad) in enumerate(SEQUENCE):
            print(f"[case] static_ws round {rnd} shape {(N, H, W, C, K, R, S, st, pad)}", flush=True)
            xb = si.normal_bf16(si.rng(900 + ci, 0), (N, H, W, C))
            wb = si.he_weight_bf16(si.rng(900 + ci, 1), (K, R, S, C))
            bias = si.rng(900 + ci, 2).standard_normal(K).astype(np.float32)
            d = wap.conv_desc(N, H, W, C, K, R, S, st, pad, relu=True)
            need = wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_FWD)
            assert need <= wap.WAP_STATIC_SCRATCH_BYTES
            P, Q = si.out_dim(H, pad, R, st), si.out_dim(W, pad, S, st)
            xd, wd, bd = gu.dev_bf16(xb), gu.dev_bf16(wb), torch.from_numpy(bias).cuda()
            y_ref = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
            y_new = torch.full((N, P, Q, K), float("nan"), dtype=torch.bfloat16, device="cuda")
            wap.wap_conv2d_fwd(d, xd, wd, bd, y_ref, gu.workspace(need))
            wap.wap_conv2d_fwd_static_ws(d, xd, wd, bd, y_new)
            torch.cuda.synchronize()
            assert torch.equal(y_new.view(torch.int16), y_ref.view(torch.int16))
            if rnd == 0:
                ref = orc.conv2d_fwd(orc.bf16_bits_to_f64(xb), orc.bf16_bits_to_f64(wb), (st, st), (pad, pad),
                                     bias=bias.astype(np.float64), relu=True)
                e = gu.rel_err(gu.host_f64(y_new), ref)
                assert e <= gu.TOL and e <= gu.TOL_BF16_OUT, e


def test_static_workspace_rejects_layers_beyond_its_size():
    import paper_1811_01532_amd as wap
    d = wap.conv_desc(64, 14, 14, 1024, 1024, 3, 3, 1, 1)  # packed weights alone are 18 MiB
    assert wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_FWD) > wap.WAP_STATIC_SCRATCH_BYTES
    t = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(wap.WapError) as ei:
        wap.wap_conv2d_fwd_static_ws(d, t, t, None, t)
    assert ei.value.status == wap.WAP_EWORKSPACE
