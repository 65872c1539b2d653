"""GPU parity of the whole training step (forward, loss, backward, SGD) run from the launch list.

Teacher-forced: every operation's output is compared with the oracle applied to that operation's
actual device inputs, so rounding differences do not compound across layers.  Reduced image sizes
keep the fp64 oracle fast; the layer lists are the full AlexNet-style and VGG-16 ones.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

LR = 0.01


class Arena:
    def __init__(self, plan):
        self.plan = plan
        self.t = plan.tensors()
        self.buf = torch.zeros(plan.arena_bytes() + 256, dtype=torch.uint8, device="cuda")
        assert self.buf.data_ptr() % 256 == 0

    def raw(self, name):
        off, nb = self.t[name]
        return self.buf[off:off + nb]

    def bf16(self, name, shape):
        return self.raw(name).view(torch.bfloat16).view(*shape)

    def f32(self, name, shape):
        return self.raw(name).view(torch.float32).view(*shape)

    def put_bf16(self, name, bits):
        self.raw(name).view(torch.int16).copy_(torch.from_numpy(bits.view(np.int16).ravel()))

    def put_f32(self, name, arr):
        self.raw(name).view(torch.float32).copy_(torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32).ravel()))


def _setup(net, B, image, flags, seed_cfg):
    import paper_1811_01532_amd as wap
    plan = wap.StepPlan(net, B, lr=LR, image=image, flags=flags)
    ar = Arena(plan)
    convs, fcs = si.NETS[net]
    shapes = si.conv_shapes(convs, image)
    weights = {}
    for i, d in enumerate(shapes):
        wb = si.he_weight_bf16(si.rng(seed_cfg, 10 + i), (d["K"], d["R"], d["S"], d["C"]))
        weights[d["name"]] = wb
    flat = shapes[-1]["out_hw"] ** 2 * shapes[-1]["K"]
    n_in = flat
    fc_dims = []
    for j, (name, _, n_out, relu) in enumerate(fcs):
        wb = si.he_weight_bf16(si.rng(seed_cfg, 40 + j), (n_out, n_in))
        weights[name] = wb
        fc_dims.append((name, n_in, n_out, relu))
        n_in = n_out
    from oracle import oracle as orc
    for name, wb in weights.items():
        ar.put_f32(name + ".w32", orc.bf16_bits_to_f64(wb).astype(np.float32))
        ar.put_bf16(name + ".w", wb)
    # optional fp32 biases, stored under "<layer>#bias" next to the weights
    if flags & wap.WAP_STEP_BIAS:
        for j, name in enumerate(list(weights.keys())):
            b = (0.1 * si.rng(seed_cfg, 70 + j).standard_normal(weights[name].shape[0])).astype(np.float32)
            weights[name + "#bias"] = b
            ar.put_f32(name + ".b32", b)
    xb = si.normal_bf16(si.rng(seed_cfg, 0), (B, image, image, 3))
    labels = si.labels(si.rng(seed_cfg, 1), B)
    ar.put_bf16("input", xb)
    ar.raw("labels").view(torch.int32).copy_(torch.from_numpy(labels))
    return plan, ar, shapes, fc_dims, weights, xb, labels


@pytest.mark.parametrize("net,B,image,with_bias", [("vgg16", 2, 32, False), ("alexnet", 3, 67, False),
                                                    ("vgg16", 2, 32, True), ("alexnet", 3, 67, True)])
def test_step_every_operation_matches_oracle(orc, net, B, image, with_bias):
    import paper_1811_01532_amd as wap
    flags = wap.WAP_STEP_KEEP_GRADS | (wap.WAP_STEP_BIAS if with_bias else 0)
    plan, ar, shapes, fc_dims, weights, xb, labels = _setup(net, B, image, flags, 500)
    print(f"[case] step {net} B={B} image={image} bias={with_bias} ops={plan.num_ops()}", flush=True)
    plan.run(ar.buf)
    torch.cuda.synchronize()
    f64 = orc.bf16_bits_to_f64
    biases = {k[:-5]: v.astype(np.float64) for k, v in weights.items() if k.endswith("#bias")}
    weights = {k: v for k, v in weights.items() if not k.endswith("#bias")}
    w64 = {k: f64(v) for k, v in weights.items()}

    def check_db(L, g_pre):
        """bias gradient of layer L against the column sums of the device's own pre-activation gradient"""
        if not with_bias:
            return
        K = g_pre.shape[-1]
        db = gu.host_f64(ar.f32(L + ".db", (K,)))
        e = gu.rel_err(db, orc.bias_grad(g_pre))
        assert e <= gu.TOL_F32_OUT, f"{L}.bias_grad rel err {e}"

    def check_bf16(name, got_t, ref, tol=gu.TOL_BF16_OUT):
        e = gu.rel_err(gu.host_f64(got_t), ref)
        assert e <= gu.TOL and e <= tol, f"{net} {name}: rel err {e}"

    # ---------------- forward ----------------
    cur = f64(xb)
    acts = {}
    for d in shapes:
        L = d["name"]
        y = ar.bf16(L + ".y", (B, d["P"], d["Q"], d["K"]))
        ref = orc.conv2d_fwd(cur, w64[L], (d["stride"],) * 2, (d["pad"],) * 2, bias=biases.get(L), relu=True)
        check_bf16(L + ".fwd", y, ref)
        acts[L + ".in"] = cur
        cur = gu.host_f64(y)
        acts[L + ".y"] = cur
        if d["pool"]:
            win, st = d["pool"]
            o = d["out_hw"]
            py = ar.bf16(L + ".pool.y", (B, o, o, d["K"]))
            am = ar.raw(L + ".pool.argmax").view(B, o, o, d["K"]).cpu().numpy()
            yref, amref = orc.maxpool_fwd(cur, win, st)
            assert np.array_equal(gu.host_f64(py), yref), L + ".pool.fwd"
            assert np.array_equal(am, amref), L + ".pool.argmax"
            cur = yref
            acts[L + ".pool.y"] = cur
            acts[L + ".pool.am"] = am
    cur = cur.reshape(B, -1)
    for (name, n_in, n_out, relu) in fc_dims:
        y = ar.bf16(name + ".y", (B, n_out))
        ref = orc.fc_fwd(cur, w64[name], bias=biases.get(name), relu=relu)
        check_bf16(name + ".fwd", y, ref)
        acts[name + ".in"] = cur
        cur = gu.host_f64(y)
        acts[name + ".y"] = cur
    # ---------------- loss ----------------
    lref, dzref = orc.softmax_xent(cur, labels)
    loss = float(ar.f32("loss", (4,))[0])
    assert abs(loss - lref) <= 1e-5 * max(1.0, abs(lref))
    g_t = ar.bf16("g.fc8.y", (B, 1000))
    check_bf16("softmax.dz", g_t, dzref)
    # ---------------- backward: FC ----------------
    g = gu.host_f64(g_t)
    last = shapes[-1]
    last_out = last["name"] + (".pool.y" if last["pool"] else ".y")
    for idx in range(len(fc_dims) - 1, -1, -1):
        name, n_in, n_out, relu = fc_dims[idx]
        if relu:
            gm_t = ar.bf16("gm." + name + ".y", (B, n_out))
            ref = orc.relu_bwd(g, acts[name + ".y"])
            assert np.array_equal(gu.host_f64(gm_t), ref), name + ".relu_bwd"
            g = ref
        dW = ar.f32(name + ".dw", (n_out, n_in))
        e = gu.rel_err(gu.host_f64(dW), orc.fc_bwd_weight(g, acts[name + ".in"]))
        assert e <= gu.TOL_F32_OUT, f"{name}.dW rel err {e}"
        check_db(name, g)
        in_name = "g." + (fc_dims[idx - 1][0] + ".y" if idx > 0 else last_out)
        gi_t = ar.bf16(in_name, (B, n_in))
        check_bf16(name + ".dx", gi_t, orc.fc_bwd_data(g, w64[name]))
        g = gu.host_f64(gi_t)
    # ---------------- backward: conv stack ----------------
    for i in range(len(shapes) - 1, -1, -1):
        d = shapes[i]
        L = d["name"]
        yshape = (B, d["P"], d["Q"], d["K"])
        gm_t = ar.bf16("gm." + L + ".y", yshape)
        if d["pool"]:
            win, st = d["pool"]
            o = d["out_hw"]
            routed = orc.maxpool_bwd(g.reshape(B, o, o, d["K"]), acts[L + ".pool.am"], yshape, win, st)
            ref = orc.relu_bwd(routed, acts[L + ".y"])
            check_bf16(L + ".pool_relu_bwd", gm_t, ref)
        else:
            ref = orc.relu_bwd(g.reshape(yshape), acts[L + ".y"])
            assert np.array_equal(gu.host_f64(gm_t), ref), L + ".relu_bwd"
        g = gu.host_f64(gm_t)
        dw = ar.f32(L + ".dw", (d["K"], d["R"], d["S"], d["C"]))
        refdw = orc.conv2d_bwd_weight(acts[L + ".in"], g, (d["K"], d["R"], d["S"], d["C"]),
                                      (d["stride"],) * 2, (d["pad"],) * 2)
        e = gu.rel_err(gu.host_f64(dw), refdw)
        assert e <= gu.TOL_F32_OUT, f"{L}.wgrad rel err {e}"
        check_db(L, g)
        if i > 0:
            prev = shapes[i - 1]
            in_name = "g." + prev["name"] + (".pool.y" if prev["pool"] else ".y")
            xshape = (B, d["H"], d["W"], d["C"])
            gi_t = ar.bf16(in_name, xshape)
            refdx = orc.conv2d_bwd_data(g, w64[L], xshape, (d["stride"],) * 2, (d["pad"],) * 2)
            check_bf16(L + ".dgrad", gi_t, refdx)
            g = gu.host_f64(gi_t)
    # ---------------- SGD ----------------
    for name, wb in weights.items():
        shape = wb.shape
        dw = gu.host_f64(ar.f32(name + ".dw", shape))
        w_after = gu.host_f64(ar.f32(name + ".w32", shape))
        ref = orc.sgd(w64[name], dw, float(np.float32(LR)))
        assert np.max(np.abs(w_after - ref)) <= 2.0 ** -22 * max(1e-30, np.max(np.abs(ref))), name + ".sgd"
        wb_after = gu.host_f64(ar.bf16(name + ".w", shape))
        assert np.array_equal(wb_after, orc.round_bf16(w_after)), name + ".w bf16 copy"
    for name, b in biases.items():
        db = gu.host_f64(ar.f32(name + ".db", b.shape))
        b_after = gu.host_f64(ar.f32(name + ".b32", b.shape))
        ref = orc.sgd(b, db, float(np.float32(LR)))
        assert np.max(np.abs(b_after - ref)) <= 2.0 ** -22 * max(1e-30, np.max(np.abs(ref))), name + ".b32 sgd"


@pytest.mark.parametrize("net,B,image,extra", [("vgg16", 2, 32, 0), ("vgg16", 1, 256, 0), ("alexnet", 3, 67, 0),
                                                ("alexnet", 2, 224, 0), ("vgg16", 2, 64, 2), ("alexnet", 2, 131, 2)])
def test_step_without_kept_gradients_is_bitwise_the_same(orc, net, B, image, extra):
    """The production plan (ping-pong gradient buffers, pool taken in the conv epilogue, pool backward routed in the
    backward kernels' loaders, ReLU derivatives riding on data-gradient epilogues, SGD updates applied by the kernels
    that finish the weight gradients) gives the same weights, stored gradients and loss as the plan that keeps every
    intermediate, which the teacher-forced test checks against the oracle.  The larger
    images reach the fused paths the 32-pixel case is too small for.  With biases the bias gradient of a layer whose
    pool backward is routed in the loaders is summed over the pooled gradient instead of the full-size one: the same
    sum in another order, so after the first step those vectors agree to fp32 rounding and everything else bit for
    bit (the second step then starts from biases that differ in the last bits)."""
    import paper_1811_01532_amd as wap
    res = []
    steps = 1 if extra else 2
    # extra = 2: with biases; the third plan stores the weight gradients and updates in a separate pass (the form
    # of a replica whose gradients are exchanged), everything else as in production
    for flags in (wap.WAP_STEP_KEEP_GRADS | extra, extra, wap.WAP_STEP_STORE_GRADS | extra):
        plan, ar, shapes, fc_dims, weights, _, _ = _setup(net, B, image, flags, 501)
        print(f"[case] step {net} B={B} image={image} flags={flags} ops={[o[0] for o in plan.ops()] if not (flags & 1) else plan.num_ops()}", flush=True)
        for _ in range(steps):  # without biases: a second step on the updated weights
            plan.run(ar.buf)
        torch.cuda.synchronize()
        names = [k for k in weights if not k.endswith("#bias")]
        n = ar.t["params.w32"][1] // 4
        # layers whose weight-gradient kernel applies the update itself never store their gradient
        fused = {o[0].split(".")[0] for o in plan.ops() if o[0].endswith("+sgd")}
        res.append(({k: ar.f32(k + ".dw", weights[k].shape).clone() for k in names if k not in fused},
                    ar.f32("params.w32", (n,)).clone(), ar.f32("loss", (4,))[0].item(), fused,
                    {k: ar.f32(k + ".db", (weights[k].shape[0],)).clone() for k in names} if extra else {},
                    {k: ar.bf16(k + ".w", weights[k].shape).clone() for k in names}))
    assert not res[0][3] and res[1][3] and not res[2][3], "only the production plan fuses updates"
    assert set(res[2][0]) == set(res[0][0])
    for r in res[1:]:
        for k, v in r[0].items():
            assert torch.equal(res[0][0][k], v), k + ".dw"
        for k in res[0][5]:
            assert torch.equal(res[0][5][k].view(torch.int16), r[5][k].view(torch.int16)), k + ".w (bf16 copy)"
        if not extra:
            assert torch.equal(res[0][1], r[1])          # every master weight after two steps
        else:
            # weights (the leading part of the block, alignment gaps included) bit for bit, bias gradients close
            last_w = max(ar.t[k + ".w32"][0] + ar.t[k + ".w32"][1] for k in names) - ar.t["params.w32"][0]
            assert torch.equal(res[0][1][:last_w // 4], r[1][:last_w // 4])
            for k in names:
                a, b = res[0][4][k].double(), r[4][k].double()
                scale = max(float(a.abs().max()), 1e-30)
                assert float((a - b).abs().max()) <= 1e-5 * scale, f"{k}.db differs by more than fp32 summation order"
        assert res[0][2] == r[2]
    assert res[0][2] == res[1][2]
    assert np.isfinite(res[0][2])


@pytest.mark.parametrize("net,B,image", [("vgg16", 2, 64), ("alexnet", 3, 67)])
def test_step_graph_replays_match_eager_steps(orc, net, B, image):
    """The step captured as one HIP graph: every replay (several, with the program's own eager work and
    synchronisations in between) leaves the whole arena bitwise equal to the eager step from the same state;
    capturing before any eager run is rejected."""
    import paper_1811_01532_amd as wap
    plan, ar, *_ = _setup(net, B, image, 0, 520)
    print(f"[case] step graph {net} B={B} image={image}", flush=True)
    side = torch.cuda.Stream()
    with pytest.raises(wap.WapError):
        plan.graph_capture(ar.buf, side)
    start = ar.buf.clone()
    # eager reference: three consecutive steps from the initial state
    refs = []
    for _ in range(3):
        plan.run(ar.buf)
        torch.cuda.synchronize()
        refs.append(ar.buf.clone())
    ws_off, ws_nb = ar.t["workspace"]

    def same(a, b):   # the workspace holds dead partial sums of whichever split reduction ran last: compare the rest
        return torch.equal(a[:ws_off], b[:ws_off]) and torch.equal(a[ws_off + ws_nb:], b[ws_off + ws_nb:])

    ar.buf.copy_(start)
    torch.cuda.synchronize()
    plan.graph_capture(ar.buf, side)          # records only: the arena must be untouched
    torch.cuda.synchronize()
    assert torch.equal(ar.buf, start)
    for rep in range(3):
        ar.buf.copy_(start)
        scratch = torch.relu(torch.randn(1 << 16, device="cuda")).sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        side.wait_stream(torch.cuda.current_stream())
        for k in range(3):
            plan.graph_launch(side)
            side.synchronize()
            assert same(ar.buf, refs[k]), f"replay round {rep}, step {k} differs from the eager step"
        assert np.isfinite(float(scratch))


def test_step_timing_entry_points_do_the_same_work(orc):
    """wap_step_time / _masked / _sampled run the launch list exactly as wap_step_run does (the arena ends bitwise
    equal) and report a positive duration for every bracketed operation and zero for the others."""
    import paper_1811_01532_amd as wap
    plan, ar, *_ = _setup("vgg16", 2, 64, 0, 530)
    print("[case] step timing entry points", flush=True)
    start = ar.buf.clone()
    for _ in range(4):
        plan.run(ar.buf)
    torch.cuda.synchronize()
    ref = ar.buf.clone()
    ws_off, ws_nb = ar.t["workspace"]

    def same(a, b):
        return torch.equal(a[:ws_off], b[:ws_off]) and torch.equal(a[ws_off + ws_nb:], b[ws_off + ws_nb:])

    ops = plan.ops()
    mask = [o[0].endswith(".fwd") or ".fwd+" in o[0] for o in ops]
    assert any(mask) and not all(mask)
    ar.buf.copy_(start)
    us, epi = plan.time(ar.buf, steps=4, op_mask=mask, every=2)      # events in steps 0 and 2
    assert same(ar.buf, ref)
    assert all((u > 0) == m for u, m in zip(us, mask)), list(zip([o[0] for o in ops], us))
    ar.buf.copy_(start)
    us, epi, pro = plan.time(ar.buf, steps=4, with_prologue=True)    # every operation, every step
    assert same(ar.buf, ref)
    assert all(u > 0 for u in us) and all(e >= 0 for e in epi) and all(q >= 0 for q in pro)
    with pytest.raises(wap.WapError):
        plan.time(ar.buf, steps=4, every=0)
