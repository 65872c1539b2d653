"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1811_01532_amd", "libwap.so")


@pytest.fixture(scope="module")
def wap():
    import paper_1811_01532_amd as w
    if not os.path.exists(LIB):
        from paper_1811_01532_amd import build
        build.build(verbose=False)
    w.lib()
    return w


def _declared_symbols():
    names = set()
    for header in ("wap.h", "wap_testing.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(wap_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(wap):
    names = _declared_symbols()
    assert "wap_conv2d_fwd" in names and "wap_profile_layer" in names and "wap_step_run" in names
    lib = ctypes.CDLL(LIB)
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing
    assert wap.wap_version() >= 100


def test_descriptor_struct_sizes_match_the_header(wap):
    assert ctypes.sizeof(wap.ConvDesc) == 12 * 4
    assert ctypes.sizeof(wap.FcDesc) == 4 * 4
    assert ctypes.sizeof(wap.ProfileRow) == 2 * 4 + 8 * 8 + 2 * 4


def _expect(wap, status, fn, *args):
    with pytest.raises(wap.WapError) as ei:
        fn(*args)
    assert ei.value.status == status, str(ei.value)
    assert len(str(ei.value)) > 20


def test_conv_descriptor_validation(wap):
    ok = wap.conv_desc(4, 32, 32, 3, 16, 3, 3, 1, 1)
    assert wap.wap_conv2d_workspace_bytes(ok, wap.WAP_PASS_FWD) >= 0
    for bad in (wap.conv_desc(0, 32, 32, 3, 16, 3, 3, 1, 1),
                wap.conv_desc(4, 32, 32, 3, 16, 3, 3, 0, 1),
                wap.conv_desc(4, 32, 32, 3, 16, 3, 3, 1, 3),       # pad >= filter
                wap.conv_desc(4, 32, 32, 3, 16, 3, 3, 1, -1),
                wap.conv_desc(1, 2, 2, 3, 16, 7, 7, 1, 1)):        # filter larger than padded input
        _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_workspace_bytes, bad, wap.WAP_PASS_FWD)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_workspace_bytes, ok, 7)
    big = wap.conv_desc(4096, 1024, 1024, 64, 64, 3, 3, 1, 1)
    _expect(wap, wap.WAP_EUNSUPPORTED, wap.wap_conv2d_workspace_bytes, big, wap.WAP_PASS_FWD)
    flags = wap.conv_desc(4, 32, 32, 3, 16, 3, 3, 1, 1)
    flags.flags = 0x80
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_workspace_bytes, flags, wap.WAP_PASS_FWD)


def test_null_and_misaligned_pointers_are_rejected_before_any_launch(wap):
    d = wap.conv_desc(4, 32, 32, 64, 64, 3, 3, 1, 1)
    s = 0  # null stream; never reached
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_fwd, d, None, 4096, None, 8192, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_fwd, d, 4096, 4096 + 2, None, 8192, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_data, d, 4096, 4096, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_weight, d, 4096, None, 4096, None, s)
    f = wap.fc_desc(32, 256, 1000)
    _expect(wap, wap.WAP_EINVAL, wap.wap_fc_fwd, f, 4096, None, None, 4096, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_fc_bwd, f, 4096, 4096, 4096, None, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_relu_bwd, 4096, 4096, None, 10, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_relu_bwd, 4096, 4096, 4096, 0, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_maxpool_fwd, 1, 2, 2, 8, 3, 2, 4096, 4096, 4096, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_softmax_xent_grad, 0, 1000, 4096, 4096, 4096, 4096, 4096, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_sgd_update, 16, None, 4096, 0.01, None, s)


def test_workspace_too_small_is_reported(wap):
    # a shape whose weight gradient needs a split reduction
    d = wap.conv_desc(8, 28, 28, 256, 256, 3, 3, 1, 1)
    need = wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_BWD_WEIGHT)
    assert need > 0
    with pytest.raises(wap.WapError) as ei:
        wap.lib().wap_conv2d_bwd_weight  # symbol exists
        wap._check(wap.lib().wap_conv2d_bwd_weight(ctypes.byref(d), ctypes.c_void_p(4096), ctypes.c_void_p(4096),
                                                   ctypes.c_void_p(4096), ctypes.c_void_p(4096),
                                                   ctypes.c_size_t(need - 1), ctypes.c_void_p(0)))
    assert ei.value.status == wap.WAP_EWORKSPACE
    with pytest.raises(wap.WapError) as ei:
        wap._check(wap.lib().wap_conv2d_bwd_weight(ctypes.byref(d), ctypes.c_void_p(4096), ctypes.c_void_p(4096),
                                                   ctypes.c_void_p(4096), ctypes.c_void_p(0), ctypes.c_size_t(0),
                                                   ctypes.c_void_p(0)))
    assert ei.value.status == wap.WAP_EWORKSPACE


def test_step_plan_is_host_only_and_counts_flops(wap):
    import synth_inputs as si
    for net in ("alexnet", "vgg16"):
        p = wap.StepPlan(net, 32)
        assert abs(p.flops() / 32 - si.step_flops_per_image(net)) < 1e-6 * si.step_flops_per_image(net)
        t = p.tensors()
        assert "input" in t and "labels" in t and "loss" in t and "params.w32" in t and "workspace" in t
        total = p.arena_bytes()
        assert all(off + nb <= total for (off, nb) in t.values())
        assert p.num_ops() > 30
    with pytest.raises(wap.WapError):
        wap.StepPlan("resnet", 32)
    with pytest.raises(wap.WapError):
        wap.StepPlan("alexnet", 0)
    with pytest.raises(wap.WapError):
        wap.StepPlan("alexnet", 2, image=16)   # too small for the pooling chain
    # tensors of a plan never overlap unless they are views of the parameter blocks or ping-pong buffers
    p = wap.StepPlan("vgg16", 2, image=32, flags=wap.WAP_STEP_KEEP_GRADS)
    t = p.tensors()
    plain = sorted((off, nb, n) for n, (off, nb) in t.items()
                   if not (n.endswith(".w32") or n.endswith(".dw") or n.endswith(".w")) or n.startswith("params."))
    for (o1, n1, a), (o2, _, b) in zip(plain, plain[1:]):
        assert o1 + n1 <= o2, (a, b)


def test_profile_argument_checks(wap):
    d = wap.conv_desc(1, 14, 14, 64, 64, 3, 3, 1, 1)
    assert wap.wap_profile_scratch_bytes(0, d, [8, 16]) > 0
    with pytest.raises(wap.WapError):
        wap.wap_profile_scratch_bytes(2, d, [8])
    with pytest.raises(wap.WapError):
        wap.wap_profile_layer(0, d, [8], 1, 1, None, 0)


def test_pool2x2_backward_entry_points_validate_on_the_host(wap):
    """Argument checks and the fused / unfused answer of the pooled-gradient backward calls are host logic."""
    s = 0
    odd = wap.conv_desc(2, 15, 16, 64, 64, 3, 3, 1, 1)      # 15 x 16 output: no whole 2x2 windows
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_data_pool2x2, odd, 4096, 4096, 4096, None, 4096, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_weight_pool2x2, odd, 4096, 4096, 4096, 4096, None, None, s)
    d = wap.conv_desc(2, 16, 16, 64, 64, 3, 3, 1, 1)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_data_pool2x2, d, None, 4096, 4096, None, 4096, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_data_pool2x2, d, 4096, None, 4096, None, 4096, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_weight_pool2x2, d, 4096, 4096, 4096 + 8, 4096, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_pool2x2_fused, d, wap.WAP_PASS_FWD)
    # the launch list of the VGG-16 benchmark relies on these answers
    vgg = {name: wap.conv_desc(64, h, h, c, k, 3, 3, 1, 1)
           for name, h, c, k in (("conv1_2", 224, 64, 64), ("conv2_2", 112, 128, 128), ("conv3_3", 56, 256, 256),
                                 ("conv4_3", 28, 512, 512), ("conv5_3", 14, 512, 512))}
    for name, desc in vgg.items():
        got = (wap.wap_conv2d_bwd_pool2x2_fused(desc, wap.WAP_PASS_BWD_DATA),
               wap.wap_conv2d_bwd_pool2x2_fused(desc, wap.WAP_PASS_BWD_WEIGHT))
        assert got == ((True, True) if name != "conv5_3" else (True, False)), (name, got)
    # shapes outside the patch kernels: never fused, and the scratch tensor is then required
    small = wap.conv_desc(4, 32, 32, 3, 16, 3, 3, 1, 1)
    assert not wap.wap_conv2d_bwd_pool2x2_fused(small, wap.WAP_PASS_BWD_DATA)
    assert not wap.wap_conv2d_bwd_pool2x2_fused(small, wap.WAP_PASS_BWD_WEIGHT)
    if wap.wap_conv2d_workspace_bytes(small, wap.WAP_PASS_BWD_DATA) == 0:
        _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_data_pool2x2, small, 4096, 4096, 4096, None, 4096, None, None, s)


def test_fused_update_entry_points_and_launch_list_order(wap):
    """Host logic of the weight gradient that applies its own SGD update: argument checks, which shapes fuse, and
    that in a launch list such an operation runs after the data gradient that still needs the old weights."""
    s = 0
    d = wap.conv_desc(2, 16, 16, 64, 64, 3, 3, 1, 1)
    assert wap.wap_conv2d_bwd_weight_sgd_fused(d)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_weight_sgd, d, 4096, 4096, None, 4096, 0.01, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_weight_sgd, d, 4096, 4096, 4096, None, 0.01, None, None, s)
    _expect(wap, wap.WAP_EINVAL, wap.wap_conv2d_bwd_weight_sgd, d, 4096, 4096, 4096 + 4, 4096, 0.01, None, None, s)
    f = wap.fc_desc(16, 2050, 2048)          # rows of 2050 parameters: no 16-byte groups per accumulator row
    assert not wap.wap_fc_bwd_weight_sgd_fused(f)
    assert wap.wap_fc_bwd_weight_sgd_fused(wap.fc_desc(64, 25088, 4096))
    if wap.wap_fc_workspace_bytes(f, wap.WAP_PASS_BWD_WEIGHT) == 0:
        _expect(wap, wap.WAP_EINVAL, wap.wap_fc_bwd_weight_sgd, f, 4096, 4096, 4096, 4096, 0.01, None, None, s)
    for net, flags in (("vgg16", 0), ("alexnet", 0), ("alexnet", wap.WAP_STEP_BIAS), ("vgg16", wap.WAP_STEP_KEEP_GRADS),
                       ("alexnet", wap.WAP_STEP_STORE_GRADS)):
        names = [o[0] for o in wap.StepPlan(net, 32, flags=flags).ops()]
        fused = [n for n in names if n.endswith("+sgd")]
        if flags & (wap.WAP_STEP_KEEP_GRADS | wap.WAP_STEP_STORE_GRADS):
            assert not fused and names.count("sgd") == 1
            continue
        assert fused, net
        for n in fused:
            layer = n.split(".")[0]
            later = [m for m in names[names.index(n) + 1:]
                     if m.startswith(layer + ".") and ("dgrad" in m or ".dx" in m)]
            assert not later, (n, later)     # the layer's data gradient reads this step's weights: it runs first
        # a layer is updated either by its gradient kernel or by a separate pass, and biases always by a pass
        n_layers = 8 if net == "alexnet" else 16
        assert len(set(fused)) == len(fused) <= n_layers
        if len(fused) < n_layers or (flags & wap.WAP_STEP_BIAS):
            assert any(m == "sgd" for m in names)


def test_wide_maps_leave_the_16bit_coordinate_kernel(wap):
    """The weights-in-registers kernel keeps pixel coordinates in 16-bit halves: a map wider than that range must
    be planned onto the generic tiles (host-side plan query, no device work)."""
    wide = wap.conv_desc(2, 1, 40000, 64, 256, 1, 1, 1, 0)
    assert wap.wap_conv2d_kernel_name(wide, wap.WAP_PASS_FWD).startswith("igemm_kernel")
    narrow = wap.conv_desc(2, 100, 400, 64, 256, 1, 1, 1, 0)
    assert wap.wap_conv2d_kernel_name(narrow, wap.WAP_PASS_FWD) == "conv_wreg_kernel"
    assert wap.wap_conv2d_kernel_name(wap.conv_desc(64, 28, 28, 512, 512, 3, 3, 1, 1), wap.WAP_PASS_BWD_WEIGHT).startswith("wgrad_patch")


def test_patch_weight_gradient_tile_and_step_map_per_layer(wap):
    """Host-side plan of the patch weight-gradient kernel <FD, UP, step map, steps per tile>: block steps on the
    28-wide tiles of conv2_x .. conv4_x need no padded pixel, 14- and 13-wide maps run 7-row tiles of width 16,
    64-channel layers take one dy block per wavefront, and so does any layer whose pixel range is short (at most 28
    tiles per work-group: small minibatches, the 14 x 14 layers), where the fp32 partial tiles outweigh the register
    tile; the pool backward is routed in the loader exactly where tiles have even height; maps too small for a 7-row
    or 4-row tile fall to the generic kernel."""
    def name(N, H, W, C, K):
        return wap.wap_conv2d_kernel_name(wap.conv_desc(N, H, W, C, K, 3, 3, 1, 1), wap.WAP_PASS_BWD_WEIGHT)

    def fused(N, H, W, C, K):
        return wap.wap_conv2d_bwd_pool2x2_fused(wap.conv_desc(N, H, W, C, K, 3, 3, 1, 1), wap.WAP_PASS_BWD_WEIGHT)
    assert name(64, 28, 28, 512, 512) == "wgrad_patch_kernel<2,false,2,7>" and fused(64, 28, 28, 512, 512)
    assert name(64, 56, 56, 256, 256) == "wgrad_patch_kernel<2,false,2,7>" and fused(64, 56, 56, 256, 256)
    assert name(64, 14, 14, 512, 512) == "wgrad_patch_kernel<1,false,0,7>" and not fused(64, 14, 14, 512, 512)
    assert name(256, 14, 14, 512, 512) == "wgrad_patch_kernel<2,false,0,7>"
    assert name(8, 28, 28, 512, 512) == "wgrad_patch_kernel<1,false,2,7>"
    assert name(64, 112, 112, 128, 128) == "wgrad_patch_kernel<2,false,0,8>" and fused(64, 112, 112, 128, 128)
    assert name(64, 224, 224, 64, 64) == "wgrad_patch_kernel<1,false,0,8>" and fused(64, 224, 224, 64, 64)
    assert name(32, 13, 13, 384, 256) == "wgrad_patch_kernel<1,false,0,7>"
    assert name(512, 13, 13, 384, 256) == "wgrad_patch_kernel<2,false,0,7>"
    assert not name(8, 6, 12, 64, 128).startswith("wgrad_patch")     # no 7-row tile on a 6-row map
    assert not name(8, 3, 28, 64, 128).startswith("wgrad_patch")     # no 4-row tile on a 3-row map


def test_static_workspace_entry_point_rejects_oversized_layers_on_the_host(wap):
    """The entry point that allocates nothing refuses, before any device work, a layer whose workspace exceeds its
    static array (so the check runs without a GPU)."""
    d = wap.conv_desc(64, 14, 14, 1024, 1024, 3, 3, 1, 1)
    assert wap.wap_conv2d_workspace_bytes(d, wap.WAP_PASS_FWD) > wap.WAP_STATIC_SCRATCH_BYTES
    with pytest.raises(wap.WapError) as ei:
        wap.wap_conv2d_fwd_static_ws(d, 4096, 8192, None, 12288, stream=0)
    assert ei.value.status == wap.WAP_EWORKSPACE
    text = open(os.path.join(ROOT, "include", "wap.h")).read()
    assert re.search(r"#define\s+WAP_STATIC_SCRATCH_BYTES\s+\(16u\s*<<\s*20\)", text)
