"""Second, independent evaluation of the convolution definitions, used only to pin the oracle.

Works on an explicitly zero-padded copy of the input and sums one filter tap at a time over
strided slices (a different decomposition from the oracle's per-output gather loops), plus a
pure-Python seven-deep loop for the tiniest shapes.
"""
import numpy as np


def out_dim(n_in, pad, win, stride):
    return (n_in + 2 * pad - win) // stride + 1


def conv_fwd_taps(x, w, stride, pad):
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    (sh, sw), (ph, pw) = stride, pad
    P, Q = out_dim(H, ph, R, sh), out_dim(W, pw, S, sw)
    xp = np.zeros((N, H + 2 * ph + sh, W + 2 * pw + sw, C))
    xp[:, ph:ph + H, pw:pw + W, :] = x
    y = np.zeros((N, P, Q, K))
    for r in range(R):
        for s in range(S):
            patch = xp[:, r:r + sh * (P - 1) + 1:sh, s:s + sw * (Q - 1) + 1:sw, :]
            y += np.einsum("npqc,kc->npqk", patch, w[:, r, s, :])
    return y


def conv_fwd_loops(x, w, stride, pad):
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    (sh, sw), (ph, pw) = stride, pad
    P, Q = out_dim(H, ph, R, sh), out_dim(W, pw, S, sw)
    xp = np.zeros((N, H + 2 * ph + sh, W + 2 * pw + sw, C))
    xp[:, ph:ph + H, pw:pw + W, :] = x
    y = np.zeros((N, P, Q, K))
    for k in range(K):
        for c in range(C):
            for s in range(S):
                for r in range(R):
                    for n in range(N):
                        for q in range(Q):
                            for p in range(P):
                                y[n, p, q, k] += xp[n, p * sh + r, q * sw + s, c] * w[k, r, s, c]
    return y


def conv_dgrad_taps(dy, w, x_shape, stride, pad):
    """Scatter form: every dy element is spread over the input taps it was computed from."""
    N, H, W, C = x_shape
    K, R, S, _ = w.shape
    (sh, sw), (ph, pw) = stride, pad
    P, Q = dy.shape[1], dy.shape[2]
    dxp = np.zeros((N, H + 2 * ph + sh, W + 2 * pw + sw, C))
    for r in range(R):
        for s in range(S):
            dxp[:, r:r + sh * (P - 1) + 1:sh, s:s + sw * (Q - 1) + 1:sw, :] += np.einsum(
                "npqk,kc->npqc", dy, w[:, r, s, :])
    return dxp[:, ph:ph + H, pw:pw + W, :].copy()


def conv_wgrad_taps(x, dy, w_shape, stride, pad):
    N, H, W, C = x.shape
    K, R, S, _ = w_shape
    (sh, sw), (ph, pw) = stride, pad
    P, Q = dy.shape[1], dy.shape[2]
    xp = np.zeros((N, H + 2 * ph + sh, W + 2 * pw + sw, C))
    xp[:, ph:ph + H, pw:pw + W, :] = x
    dw = np.zeros((K, R, S, C))
    for r in range(R):
        for s in range(S):
            patch = xp[:, r:r + sh * (P - 1) + 1:sh, s:s + sw * (Q - 1) + 1:sw, :]
            dw[:, r, s, :] = np.einsum("npqk,npqc->kc", dy, patch)
    return dw
