"""ctypes binding of the fp64 CPU oracle (oracle/wap_oracle.c).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import this module.  It neither imports nor is imported by the HIP package.

All tensors are C-contiguous float64 numpy arrays in the layouts the C file states
(activations NHWC, conv weights KRSC, FC weights [out][in]).  bf16 data enter as the uint16
bit patterns the device reads, widened exactly with `bf16_bits_to_f64`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wap_oracle.c")
_LIB = os.path.join(_HERE, "libwap_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict fp64, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-fno-fast-math", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _d(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _dn(a):
    return None if a is None else _d(a)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def bf16_bits_to_f64(bits):
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def out_dim(n_in, pad, win, stride):
    return (n_in + 2 * pad - win) // stride + 1


def round_bf16(a):
    """Nearest bfloat16 (ties to even) of every element, returned as float64."""
    out = _f64(a).copy()
    lib().orc_round_bf16(_d(out), ctypes.c_int64(out.size))
    return out


def conv2d_fwd(x, w, stride=(1, 1), pad=(0, 0), bias=None, relu=False):
    x, w = _f64(x), _f64(w)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    P, Q = out_dim(H, pad[0], R, stride[0]), out_dim(W, pad[1], S, stride[1])
    y = np.empty((N, P, Q, K), dtype=np.float64)
    b = None if bias is None else _f64(bias)
    lib().orc_conv2d_fwd(_d(x), _d(w), _dn(b), _d(y), N, H, W, C, K, R, S,
                         stride[0], stride[1], pad[0], pad[1], int(relu))
    return y


def conv2d_fwd_at(x, w, idx, stride=(1, 1), pad=(0, 0), bias=None, relu=False):
    x, w = _f64(x), _f64(w)
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float64)
    b = None if bias is None else _f64(bias)
    lib().orc_conv2d_fwd_at(_d(x), _d(w), _dn(b), N, H, W, C, K, R, S,
                            stride[0], stride[1], pad[0], pad[1], int(relu),
                            idx.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(idx.size), _d(out))
    return out


def conv2d_bwd_data(dy, w, x_shape, stride=(1, 1), pad=(0, 0)):
    dy, w = _f64(dy), _f64(w)
    N, H, W, C = x_shape
    K, R, S, _ = w.shape
    assert dy.shape == (N, out_dim(H, pad[0], R, stride[0]), out_dim(W, pad[1], S, stride[1]), K)
    dx = np.empty((N, H, W, C), dtype=np.float64)
    lib().orc_conv2d_bwd_data(_d(dy), _d(w), _d(dx), N, H, W, C, K, R, S,
                              stride[0], stride[1], pad[0], pad[1])
    return dx


def conv2d_bwd_data_at(dy, w, x_shape, idx, stride=(1, 1), pad=(0, 0)):
    dy, w = _f64(dy), _f64(w)
    N, H, W, C = x_shape
    K, R, S, _ = w.shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float64)
    lib().orc_conv2d_bwd_data_at(_d(dy), _d(w), N, H, W, C, K, R, S,
                                 stride[0], stride[1], pad[0], pad[1],
                                 idx.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(idx.size), _d(out))
    return out


def conv2d_bwd_weight(x, dy, w_shape, stride=(1, 1), pad=(0, 0)):
    x, dy = _f64(x), _f64(dy)
    N, H, W, C = x.shape
    K, R, S, _ = w_shape
    assert dy.shape == (N, out_dim(H, pad[0], R, stride[0]), out_dim(W, pad[1], S, stride[1]), K)
    dw = np.empty((K, R, S, C), dtype=np.float64)
    lib().orc_conv2d_bwd_weight(_d(x), _d(dy), _d(dw), N, H, W, C, K, R, S,
                                stride[0], stride[1], pad[0], pad[1])
    return dw


def conv2d_bwd_weight_at(x, dy, w_shape, idx, stride=(1, 1), pad=(0, 0)):
    x, dy = _f64(x), _f64(dy)
    N, H, W, C = x.shape
    K, R, S, _ = w_shape
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float64)
    lib().orc_conv2d_bwd_weight_at(_d(x), _d(dy), N, H, W, C, K, R, S,
                                   stride[0], stride[1], pad[0], pad[1],
                                   idx.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(idx.size), _d(out))
    return out


def fc_fwd(x, Wt, bias=None, relu=False):
    x, Wt = _f64(x), _f64(Wt)
    B, n_in = x.shape
    n_out, n_in2 = Wt.shape
    assert n_in == n_in2
    y = np.empty((B, n_out), dtype=np.float64)
    b = None if bias is None else _f64(bias)
    lib().orc_fc_fwd(_d(x), _d(Wt), _dn(b), _d(y), B, n_in, n_out, int(relu))
    return y


def fc_bwd_data(dy, Wt):
    dy, Wt = _f64(dy), _f64(Wt)
    B, n_out = dy.shape
    n_out2, n_in = Wt.shape
    assert n_out == n_out2
    dx = np.empty((B, n_in), dtype=np.float64)
    lib().orc_fc_bwd_data(_d(dy), _d(Wt), _d(dx), B, n_in, n_out)
    return dx


def fc_bwd_weight(dy, x):
    dy, x = _f64(dy), _f64(x)
    B, n_out = dy.shape
    B2, n_in = x.shape
    assert B == B2
    dW = np.empty((n_out, n_in), dtype=np.float64)
    lib().orc_fc_bwd_weight(_d(dy), _d(x), _d(dW), B, n_in, n_out)
    return dW


def bias_grad(dy):
    """db[k] = sum of dy over every axis but the last (channels)."""
    dy = _f64(dy)
    cols = dy.shape[-1]
    rows = dy.size // cols
    db = np.empty(cols, dtype=np.float64)
    lib().orc_bias_grad(_d(dy), _d(db), ctypes.c_int64(rows), ctypes.c_int64(cols))
    return db


def relu_bwd(dy, y):
    dy, y = _f64(dy), _f64(y)
    dx = np.empty_like(dy)
    lib().orc_relu_bwd(_d(dy), _d(y), _d(dx), ctypes.c_int64(dy.size))
    return dx


def maxpool_fwd(x, win, stride):
    x = _f64(x)
    N, H, W, C = x.shape
    P, Q = out_dim(H, 0, win, stride), out_dim(W, 0, win, stride)
    y = np.empty((N, P, Q, C), dtype=np.float64)
    am = np.empty((N, P, Q, C), dtype=np.uint8)
    lib().orc_maxpool_fwd(_d(x), _d(y), am.ctypes.data_as(ctypes.c_void_p), N, H, W, C, win, stride)
    return y, am


def maxpool_bwd(dy, argmax, x_shape, win, stride):
    dy = _f64(dy)
    argmax = np.ascontiguousarray(argmax, dtype=np.uint8)
    N, H, W, C = x_shape
    dx = np.empty((N, H, W, C), dtype=np.float64)
    lib().orc_maxpool_bwd(_d(dy), argmax.ctypes.data_as(ctypes.c_void_p), _d(dx), N, H, W, C, win, stride)
    return dx


def softmax_xent(z, labels):
    z = _f64(z)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    B, classes = z.shape
    assert labels.shape == (B,) and labels.min() >= 0 and labels.max() < classes
    dz = np.empty_like(z)
    loss = ctypes.c_double(0.0)
    lib().orc_softmax_xent(_d(z), labels.ctypes.data_as(ctypes.c_void_p), B, classes,
                           ctypes.byref(loss), _d(dz))
    return loss.value, dz


def sgd(w, dw, lr):
    w = _f64(w).copy()
    dw = _f64(dw)
    assert w.shape == dw.shape
    lib().orc_sgd(_d(w), _d(dw), ctypes.c_double(lr), ctypes.c_int64(w.size))
    return w
