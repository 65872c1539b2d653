"""Pins for the oracle's convolution forward / data-gradient / weight-gradient (CPU only).

The paper prints no worked numerical example of a convolution, so every pin is an invariant,
a closed form, a reduction to a library routine (fp64 matmul) or an independent brute force.
"""
import os

import numpy as np
import pytest

from tests import brute_force as bf

GEOMS = [
    # N, H, W, C, K, R, S, stride, pad
    (2, 5, 5, 3, 2, 3, 3, (1, 1), (1, 1)),
    (1, 7, 6, 2, 3, 3, 2, (2, 2), (0, 1)),
    (2, 9, 11, 3, 4, 5, 5, (1, 1), (2, 2)),
    (1, 21, 21, 3, 2, 11, 11, (4, 4), (2, 2)),   # floor-truncated: (21+4-11) % 4 != 0
    (1, 8, 8, 4, 3, 3, 3, (2, 2), (1, 1)),
    (2, 6, 9, 5, 2, 1, 1, (1, 1), (0, 0)),
    (1, 10, 7, 2, 2, 4, 3, (2, 1), (1, 0)),
    (1, 9, 9, 2, 3, 3, 3, (4, 4), (2, 2)),
]


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("g", GEOMS)
def test_fwd_matches_tap_sum_brute_force(orc, g):
    N, H, W, C, K, R, S, st, pad = g
    x, w = _rand((N, H, W, C), 1), _rand((K, R, S, C), 2)
    y = orc.conv2d_fwd(x, w, st, pad)
    ref = bf.conv_fwd_taps(x, w, st, pad)
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_fwd_matches_seven_loop_brute_force(orc):
    for g in GEOMS[:2] + GEOMS[6:7]:
        N, H, W, C, K, R, S, st, pad = g
        x, w = _rand((N, H, W, C), 3), _rand((K, R, S, C), 4)
        assert np.allclose(orc.conv2d_fwd(x, w, st, pad), bf.conv_fwd_loops(x, w, st, pad), rtol=0, atol=1e-12)


@pytest.mark.parametrize("g", GEOMS)
def test_delta_filter_is_a_shift_bit_exact(orc, g):
    N, H, W, C, K, R, S, st, pad = g
    x = _rand((N, H, W, C), 5)
    k0, r0, s0, c0 = K - 1, R // 2, S - 1, C - 1
    w = np.zeros((K, R, S, C))
    w[k0, r0, s0, c0] = 1.0
    y = orc.conv2d_fwd(x, w, st, pad)
    P, Q = y.shape[1], y.shape[2]
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                h, ww = p * st[0] - pad[0] + r0, q * st[1] - pad[1] + s0
                want = x[n, h, ww, c0] if (0 <= h < H and 0 <= ww < W) else 0.0
                assert y[n, p, q, k0] == want
    others = np.delete(y, k0, axis=3)
    assert np.all(others == 0.0)


def test_all_ones_counts_in_bounds_taps(orc):
    N, H, W, C, K, R, S = 1, 6, 7, 5, 2, 3, 3
    y = orc.conv2d_fwd(np.ones((N, H, W, C)), np.ones((K, R, S, C)), (1, 1), (1, 1))
    assert y.shape == (N, H, W, K)
    assert y[0, 2, 3, 0] == C * R * S            # interior
    assert y[0, 0, 0, 1] == C * (R - 1) * (S - 1)  # corner
    assert y[0, 0, 3, 0] == C * (R - 1) * S        # top edge
    assert y[0, 3, W - 1, 0] == C * R * (S - 1)    # right edge
    # stride 2, pad 0: every window fully inside
    y2 = orc.conv2d_fwd(np.ones((1, 9, 9, 4)), np.ones((3, 3, 3, 4)), (2, 2), (0, 0))
    assert y2.shape == (1, 4, 4, 3) and np.all(y2 == 36.0)


def test_1x1_conv_is_a_matmul(orc):
    x, w = _rand((2, 4, 5, 7), 6), _rand((3, 1, 1, 7), 7)
    y = orc.conv2d_fwd(x, w)
    ref = x.reshape(-1, 7) @ w.reshape(3, 7).T
    assert np.allclose(y.reshape(-1, 3), ref, rtol=0, atol=1e-13)


def test_full_window_conv_is_fc(orc):
    x, w = _rand((3, 4, 5, 2), 8), _rand((6, 4, 5, 2), 9)
    y = orc.conv2d_fwd(x, w)
    assert y.shape == (3, 1, 1, 6)
    fc = orc.fc_fwd(x.reshape(3, -1), w.reshape(6, -1))
    assert np.allclose(y.reshape(3, 6), fc, rtol=0, atol=1e-13)
    assert np.allclose(fc, x.reshape(3, -1) @ w.reshape(6, -1).T, rtol=0, atol=1e-13)


def test_linearity_bias_and_relu(orc):
    N, H, W, C, K, R, S, st, pad = GEOMS[2]
    x1, x2, w = _rand((N, H, W, C), 10), _rand((N, H, W, C), 11), _rand((K, R, S, C), 12)
    a = orc.conv2d_fwd(2.0 * x1 - 3.0 * x2, w, st, pad)
    b = 2.0 * orc.conv2d_fwd(x1, w, st, pad) - 3.0 * orc.conv2d_fwd(x2, w, st, pad)
    assert np.allclose(a, b, rtol=0, atol=1e-11)
    bias = _rand((K,), 13)
    plain = orc.conv2d_fwd(x1, w, st, pad)
    assert np.allclose(orc.conv2d_fwd(x1, w, st, pad, bias=bias), plain + bias, rtol=0, atol=1e-13)
    assert np.array_equal(orc.conv2d_fwd(x1, w, st, pad, relu=True), np.maximum(plain, 0.0))


@pytest.mark.parametrize("g", GEOMS)
def test_adjoint_identities(orc, g):
    """<conv(x,w), g> = <x, dgrad(g,w)> = <w, wgrad(x,g)>"""
    N, H, W, C, K, R, S, st, pad = g
    x, w = _rand((N, H, W, C), 14), _rand((K, R, S, C), 15)
    y = orc.conv2d_fwd(x, w, st, pad)
    gy = _rand(y.shape, 16)
    lhs = np.sum(y * gy)
    dx = orc.conv2d_bwd_data(gy, w, x.shape, st, pad)
    dw = orc.conv2d_bwd_weight(x, gy, w.shape, st, pad)
    scale = max(1.0, abs(lhs))
    assert abs(np.sum(x * dx) - lhs) <= 1e-11 * scale
    assert abs(np.sum(w * dw) - lhs) <= 1e-11 * scale


@pytest.mark.parametrize("g", GEOMS)
def test_bwd_match_scatter_brute_force(orc, g):
    N, H, W, C, K, R, S, st, pad = g
    x, w = _rand((N, H, W, C), 17), _rand((K, R, S, C), 18)
    P, Q = bf.out_dim(H, pad[0], R, st[0]), bf.out_dim(W, pad[1], S, st[1])
    gy = _rand((N, P, Q, K), 19)
    dx = orc.conv2d_bwd_data(gy, w, x.shape, st, pad)
    dw = orc.conv2d_bwd_weight(x, gy, w.shape, st, pad)
    assert np.allclose(dx, bf.conv_dgrad_taps(gy, w, x.shape, st, pad), rtol=0, atol=1e-11)
    assert np.allclose(dw, bf.conv_wgrad_taps(x, gy, w.shape, st, pad), rtol=0, atol=1e-11)


def test_dgrad_is_zero_where_forward_never_reads(orc):
    # H=21, R=11, stride 4, pad 2: P=4, the last padded row read is 3*4+10 = 22 -> input row 20;
    # W=22 gives Q=4 as well and leaves input column 21 unread.
    N, H, W, C, K, R, S = 1, 21, 22, 2, 2, 11, 11
    st, pad = (4, 4), (2, 2)
    gy = _rand((N, 4, 4, K), 20)
    dx = orc.conv2d_bwd_data(gy, _rand((K, R, S, C), 21), (N, H, W, C), st, pad)
    assert np.all(dx[:, :, 21, :] == 0.0)
    assert np.any(dx[:, :, 20, :] != 0.0)


def test_gradients_by_finite_differences(orc):
    N, H, W, C, K, R, S, st, pad = GEOMS[4]
    x, w = _rand((N, H, W, C), 22), _rand((K, R, S, C), 23)

    def f(xx, ww):
        return 0.5 * np.sum(orc.conv2d_fwd(xx, ww, st, pad) ** 2)

    y = orc.conv2d_fwd(x, w, st, pad)
    dx = orc.conv2d_bwd_data(y, w, x.shape, st, pad)
    dw = orc.conv2d_bwd_weight(x, y, w.shape, st, pad)
    eps = 1e-6
    g = np.random.default_rng(24)
    for _ in range(6):
        i = tuple(g.integers(0, s) for s in x.shape)
        e = np.zeros_like(x); e[i] = eps
        fd = (f(x + e, w) - f(x - e, w)) / (2 * eps)
        assert abs(fd - dx[i]) <= 1e-6 * max(1.0, abs(fd))
        j = tuple(g.integers(0, s) for s in w.shape)
        e = np.zeros_like(w); e[j] = eps
        fd = (f(x, w + e) - f(x, w - e)) / (2 * eps)
        assert abs(fd - dw[j]) <= 1e-6 * max(1.0, abs(fd))


@pytest.mark.parametrize("g", [GEOMS[2], GEOMS[3], GEOMS[6]])
def test_sampled_entry_points_equal_the_full_ones(orc, g):
    N, H, W, C, K, R, S, st, pad = g
    x, w = _rand((N, H, W, C), 25), _rand((K, R, S, C), 26)
    bias = _rand((K,), 27)
    y = orc.conv2d_fwd(x, w, st, pad, bias=bias, relu=True)
    gy = _rand(y.shape, 28)
    dx = orc.conv2d_bwd_data(gy, w, x.shape, st, pad)
    dw = orc.conv2d_bwd_weight(x, gy, w.shape, st, pad)
    r = np.random.default_rng(29)
    iy = r.integers(0, y.size, 50); ix = r.integers(0, dx.size, 50); iw = r.integers(0, dw.size, 50)
    assert np.array_equal(orc.conv2d_fwd_at(x, w, iy, st, pad, bias=bias, relu=True), y.ravel()[iy])
    assert np.array_equal(orc.conv2d_bwd_data_at(gy, w, x.shape, ix, st, pad), dx.ravel()[ix])
    assert np.array_equal(orc.conv2d_bwd_weight_at(x, gy, w.shape, iw, st, pad), dw.ravel()[iw])


def test_hand_worked_example_from_golden_file(orc):
    """tests/golden/conv_hand_example.txt: a 1x4x4x1 ramp under a 3x3 filter, worked by hand."""
    path = os.path.join(os.path.dirname(__file__), "golden", "conv_hand_example.txt")
    rows = [ln.split("#")[0].split() for ln in open(path) if ln.split("#")[0].strip()]
    vals = {r[0]: np.array([float(v) for v in r[1:]]) for r in rows}
    x = vals["x"].reshape(1, 4, 4, 1)
    w = vals["w"].reshape(1, 3, 3, 1)
    y = orc.conv2d_fwd(x, w, (1, 1), (1, 1))
    assert np.array_equal(y.ravel(), vals["y_pad1"])
    y0 = orc.conv2d_fwd(x, w, (1, 1), (0, 0))
    assert np.array_equal(y0.ravel(), vals["y_pad0"])
    dw = orc.conv2d_bwd_weight(x, np.ones((1, 2, 2, 1)), (1, 3, 3, 1), (1, 1), (0, 0))
    assert np.array_equal(dw.ravel(), vals["dw_pad0_ones"])
    dx = orc.conv2d_bwd_data(np.ones((1, 2, 2, 1)), w, (1, 4, 4, 1), (1, 1), (0, 0))
    assert np.array_equal(dx.ravel(), vals["dx_pad0_ones"])
