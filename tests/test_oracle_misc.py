"""Pins for the oracle's FC, ReLU, max-pool, softmax cross-entropy, SGD and bf16 rounding (CPU only)."""
import math

import numpy as np
import torch

import synth_inputs as si


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---- fully connected ------------------------------------------------------------------------
def test_fc_matches_fp64_matmul(orc):
    x, W, dy = _rand((5, 13), 1), _rand((7, 13), 2), _rand((5, 7), 3)
    b = _rand((7,), 4)
    assert np.allclose(orc.fc_fwd(x, W), x @ W.T, rtol=0, atol=1e-13)
    assert np.allclose(orc.fc_fwd(x, W, bias=b, relu=True), np.maximum(x @ W.T + b, 0), rtol=0, atol=1e-13)
    assert np.allclose(orc.fc_bwd_data(dy, W), dy @ W, rtol=0, atol=1e-13)
    assert np.allclose(orc.fc_bwd_weight(dy, x), dy.T @ x, rtol=0, atol=1e-13)


def test_fc_adjoints(orc):
    x, W, g = _rand((4, 9), 5), _rand((6, 9), 6), _rand((4, 6), 7)
    lhs = np.sum(orc.fc_fwd(x, W) * g)
    assert abs(np.sum(x * orc.fc_bwd_data(g, W)) - lhs) < 1e-11
    assert abs(np.sum(W * orc.fc_bwd_weight(g, x)) - lhs) < 1e-11


# ---- ReLU -----------------------------------------------------------------------------------
def test_relu_bwd_derivative_at_zero_is_zero(orc):
    y = np.array([-1.0, 0.0, 0.5, 2.0, -0.0])
    dy = np.array([10.0, 20.0, 30.0, 40.0, 50.0])
    assert np.array_equal(orc.relu_bwd(dy, y), np.array([0.0, 0.0, 30.0, 40.0, 0.0]))


# ---- max-pool -------------------------------------------------------------------------------
def test_maxpool_ramp_2x2(orc):
    x = np.arange(16, dtype=np.float64).reshape(1, 4, 4, 1)
    y, am = orc.maxpool_fwd(x, 2, 2)
    assert np.array_equal(y.ravel(), [5, 7, 13, 15])
    assert np.all(am == 3)  # bottom-right of every window (r=1,s=1 -> 1*2+1)
    dx = orc.maxpool_bwd(np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 2, 2, 1), am, x.shape, 2, 2)
    want = np.zeros((4, 4)); want[1, 1], want[1, 3], want[3, 1], want[3, 3] = 1, 2, 3, 4
    assert np.array_equal(dx.reshape(4, 4), want)


def test_maxpool_ramp_3x3_stride2_overlap(orc):
    # 7x7 ramp, window 3 stride 2 -> 3x3 output; max is the bottom-right of every window
    x = np.arange(49, dtype=np.float64).reshape(1, 7, 7, 1)
    y, am = orc.maxpool_fwd(x, 3, 2)
    assert np.array_equal(y.reshape(3, 3), [[16, 18, 20], [30, 32, 34], [44, 46, 48]])
    assert np.all(am == 8)
    # decreasing ramp: the max is the top-left, shared by no two windows except via overlap
    y2, am2 = orc.maxpool_fwd(-x, 3, 2)
    assert np.all(am2 == 0)
    assert np.array_equal(y2.reshape(3, 3), -np.array([[0, 2, 4], [14, 16, 18], [28, 30, 32]]))


def test_maxpool_ties_take_first_and_sums_are_conserved(orc):
    x = np.zeros((2, 7, 7, 3))
    _, am = orc.maxpool_fwd(x, 3, 2)
    assert np.all(am == 0)
    g = np.random.default_rng(8)
    x = np.round(g.standard_normal((2, 9, 9, 4)) * 2) / 2      # many ties
    for win, st in ((2, 2), (3, 2)):
        y, am = orc.maxpool_fwd(x, win, st)
        P = y.shape[1]
        for n in range(2):
            for p in range(P):
                for q in range(P):
                    for c in range(4):
                        wdw = x[n, p * st:p * st + win, q * st:q * st + win, c]
                        assert y[n, p, q, c] == wdw.max()
                        r, s = divmod(int(am[n, p, q, c]), win)
                        assert wdw[r, s] == wdw.max()
                        first = int(np.argmax(wdw.ravel() == wdw.max()))
                        assert first == r * win + s
        dy = g.standard_normal(y.shape)
        dx = orc.maxpool_bwd(dy, am, x.shape, win, st)
        assert abs(dx.sum() - dy.sum()) < 1e-12
        assert np.allclose(dx.sum(axis=(1, 2)), dy.sum(axis=(1, 2)), rtol=0, atol=1e-12)


# ---- softmax cross-entropy ------------------------------------------------------------------
def test_softmax_zero_logits(orc):
    B, classes = 4, 1000
    labels = np.array([0, 7, 999, 500], dtype=np.int32)
    loss, dz = orc.softmax_xent(np.zeros((B, classes)), labels)
    assert abs(loss - math.log(1000.0)) < 1e-12
    want = np.full((B, classes), 1.0 / classes / B)
    want[np.arange(B), labels] -= 1.0 / B
    assert np.allclose(dz, want, rtol=0, atol=1e-15)


def test_softmax_rows_sum_to_zero_shift_invariance_and_fd(orc):
    g = np.random.default_rng(9)
    z = g.standard_normal((3, 11)) * 3
    labels = np.array([2, 10, 0], dtype=np.int32)
    loss, dz = orc.softmax_xent(z, labels)
    assert np.allclose(dz.sum(axis=1), 0, atol=1e-15)
    loss2, dz2 = orc.softmax_xent(z + 100.0, labels)
    assert abs(loss2 - loss) < 1e-12 and np.allclose(dz2, dz, atol=1e-13)
    # library pin
    t = torch.nn.functional.cross_entropy(torch.from_numpy(z), torch.from_numpy(labels).long())
    assert abs(loss - float(t)) < 1e-12
    eps = 1e-6
    for (b, j) in ((0, 2), (1, 3), (2, 10)):
        e = np.zeros_like(z); e[b, j] = eps
        fd = (orc.softmax_xent(z + e, labels)[0] - orc.softmax_xent(z - e, labels)[0]) / (2 * eps)
        assert abs(fd - dz[b, j]) < 1e-8


# ---- SGD ------------------------------------------------------------------------------------
def test_sgd_closed_form(orc):
    w = np.array([1.0, -2.0, 0.5]); dw = np.array([10.0, 4.0, -2.0])
    assert np.allclose(orc.sgd(w, dw, 0.01), [0.9, -2.04, 0.52], rtol=0, atol=1e-15)


# ---- bf16 rounding --------------------------------------------------------------------------
def test_round_bf16_known_values_and_library(orc):
    vals = np.array([1.0, 1 + 2.0**-8, 1 + 3 * 2.0**-8, 1 + 2.0**-7, -(1 + 2.0**-8 + 2.0**-20), 0.0, 3.14159265, 1e-3, 65504.0])
    want = np.array([1.0, 1.0, 1 + 2.0**-6, 1 + 2.0**-7, -(1 + 2.0**-7), 0.0, 3.140625, 0.00099945068359375, 65536.0])
    assert np.array_equal(orc.round_bf16(vals), want)
    g = np.random.default_rng(10)
    a = (g.standard_normal(20000) * np.exp(g.uniform(-20, 20, 20000))).astype(np.float32)
    lib = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_bf16(a.astype(np.float64)), lib)
    # the input generator's own rounding agrees, and widening its bits is exact
    bits = si.f32_to_bf16_bits(a)
    assert np.array_equal(orc.bf16_bits_to_f64(bits), lib)


# ---- a toy net end to end: finite-difference check of the chained backward ------------------
def test_toy_net_gradient_by_finite_differences(orc):
    g = np.random.default_rng(11)
    x = g.standard_normal((2, 8, 8, 2))
    w1 = g.standard_normal((3, 3, 3, 2)) * 0.5
    w2 = g.standard_normal((4, 3, 3, 3)) * 0.5
    wf = g.standard_normal((5, 4 * 4 * 4)) * 0.3
    labels = np.array([1, 4], dtype=np.int32)

    def forward(w1_, w2_, wf_):
        a1 = orc.conv2d_fwd(x, w1_, (1, 1), (1, 1), relu=True)
        a2 = orc.conv2d_fwd(a1, w2_, (1, 1), (1, 1), relu=True)
        p2, am = orc.maxpool_fwd(a2, 2, 2)
        z = orc.fc_fwd(p2.reshape(2, -1), wf_)
        return a1, a2, p2, am, z

    a1, a2, p2, am, z = forward(w1, w2, wf)
    loss, dz = orc.softmax_xent(z, labels)
    dwf = orc.fc_bwd_weight(dz, p2.reshape(2, -1))
    dp2 = orc.fc_bwd_data(dz, wf).reshape(p2.shape)
    da2 = orc.relu_bwd(orc.maxpool_bwd(dp2, am, a2.shape, 2, 2), a2)
    dw2 = orc.conv2d_bwd_weight(a1, da2, w2.shape, (1, 1), (1, 1))
    da1 = orc.relu_bwd(orc.conv2d_bwd_data(da2, w2, a1.shape, (1, 1), (1, 1)), a1)
    dw1 = orc.conv2d_bwd_weight(x, da1, w1.shape, (1, 1), (1, 1))

    def L(w1_, w2_, wf_):
        return orc.softmax_xent(forward(w1_, w2_, wf_)[4], labels)[0]

    eps = 1e-6
    for (arr, grad, which) in ((w1, dw1, 0), (w2, dw2, 1), (wf, dwf, 2)):
        for _ in range(4):
            i = tuple(g.integers(0, s) for s in arr.shape)
            e = np.zeros_like(arr); e[i] = eps
            args_p = [w1, w2, wf]; args_m = [w1, w2, wf]
            args_p[which] = arr + e; args_m[which] = arr - e
            fd = (L(*args_p) - L(*args_m)) / (2 * eps)
            assert abs(fd - grad[i]) <= 2e-7 * max(1.0, abs(fd)), (which, i, fd, grad[i])


def test_input_recipe_is_seeded_and_counts_match(orc):
    a = si.normal_bf16(si.rng(1, 0), (4, 32, 32, 3))
    b = si.normal_bf16(si.rng(1, 0), (4, 32, 32, 3))
    assert np.array_equal(a, b) and a.dtype == np.uint16
    w = orc.bf16_bits_to_f64(si.he_weight_bf16(si.rng(1, 1), (256, 3, 3, 64)))
    assert abs(w.var() - 2.0 / 576) < 0.05 * 2.0 / 576
    # parameter counts implied by the two layer lists (what the gradient exchange would move)
    def params(net):
        convs, fcs = si.NETS[net]
        return sum(k * r * r * c for (_, c, k, r, _, _, _) in convs) + sum(i * o for (_, i, o, _) in fcs)
    assert params("alexnet") == 61100840 - (64 + 192 + 384 + 256 + 256 + 4096 + 4096 + 1000)
    assert params("vgg16") == 138357544 - (64 * 2 + 128 * 2 + 256 * 3 + 512 * 6 + 4096 * 2 + 1000)
    assert abs(si.step_flops_per_image("alexnet") / 1e9 - 4.145) < 0.01
    assert abs(si.step_flops_per_image("vgg16") / 1e9 - 92.65) < 0.05


def test_bias_grad_is_the_derivative_of_the_loss_wrt_the_bias(orc):
    """Pins: (a) finite differences of <conv(x, w) + b, dy> in b; (b) all-ones dy gives the pixel count;
    (c) the adjoint identity <broadcast(b), dy> = <b, db>."""
    g = np.random.default_rng(31)
    x, w = g.standard_normal((2, 5, 6, 3)), g.standard_normal((4, 3, 3, 3))
    b = g.standard_normal(4)
    y0 = orc.conv2d_fwd(x, w, (1, 1), (1, 1), bias=b)
    dy = g.standard_normal(y0.shape)
    db = orc.bias_grad(dy)
    eps = 1e-6
    for k in range(4):
        bp = b.copy(); bp[k] += eps
        num = (np.sum(orc.conv2d_fwd(x, w, (1, 1), (1, 1), bias=bp) * dy) - np.sum(y0 * dy)) / eps
        assert abs(num - db[k]) <= 1e-6 * max(1.0, abs(db[k]))
    assert np.array_equal(orc.bias_grad(np.ones((3, 4, 5, 7))), np.full(7, 60.0))
    assert np.isclose(np.sum(np.broadcast_to(b, dy.shape) * dy), np.dot(b, db), rtol=1e-13)
    # plain definition on a 2-D view
    assert np.allclose(db, dy.reshape(-1, 4).sum(axis=0), rtol=0, atol=1e-12)
