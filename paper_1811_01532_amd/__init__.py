"""Thin Python binding of libwap (include/wap.h): argument marshalling only.

Every step of the path runs in the HIP kernels of libwap.so; this module turns torch device
tensors into raw pointers and sizes and raises on a non-zero status.  There is no CPU fallback:
if the library has not been built the import of any entry point fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwap.so")

WAP_OK, WAP_EINVAL, WAP_EUNSUPPORTED, WAP_EWORKSPACE, WAP_EHIP = 0, 1, 2, 3, 4
WAP_RELU = 1
WAP_PASS_FWD, WAP_PASS_BWD_DATA, WAP_PASS_BWD_WEIGHT = 0, 1, 2
WAP_STEP_KEEP_GRADS = 1
WAP_STEP_BIAS = 2
WAP_STEP_STORE_GRADS = 4

PEAK_BF16_TFLOPS = 2516.6
PEAK_HBM_GBS = 8000.0


class WapError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"wap status {status}: {message}")
        self.status = status


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")] + [
                    ("flags", ctypes.c_uint32)]

    @property
    def P(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1


class FcDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("in_features", ctypes.c_int32), ("out_features", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class ProfileRow(ctypes.Structure):
    _fields_ = [("pass_", ctypes.c_int32), ("minibatch", ctypes.c_int32), ("flops", ctypes.c_double),
                ("alg_bytes", ctypes.c_double), ("time_us_median", ctypes.c_double),
                ("time_us_min", ctypes.c_double), ("tflops", ctypes.c_double),
                ("frac_of_bf16_peak", ctypes.c_double), ("gbytes_per_s", ctypes.c_double),
                ("frac_of_hbm_peak", ctypes.c_double), ("bound", ctypes.c_int32), ("reps_per_sample", ctypes.c_int32)]


class MfmaCeilingRow(ctypes.Structure):
    _fields_ = [("data", ctypes.c_int32), ("feed", ctypes.c_int32), ("tflops", ctypes.c_double),
                ("clock_ghz", ctypes.c_double), ("us", ctypes.c_double)]


_lib = None


def lib():
    """The loaded libwap.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_1811_01532_amd.build`")
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.wap_last_error.restype = ctypes.c_char_p
        _lib.wap_debug_force.restype = None
        _lib.wap_step_flops.restype = ctypes.c_double
        _lib.wap_step_plan_destroy.restype = None
        _lib.wap_mfma_ceiling_scratch_bytes.restype = ctypes.c_size_t
    return _lib


def _check(rc):
    if rc != WAP_OK:
        raise WapError(rc, lib().wap_last_error().decode())


def _ptr(t):
    """Device pointer of a torch tensor (or None / int passthrough)."""
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def conv_desc(N, H, W, C, K, R, S, stride=1, pad=0, relu=False):
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return ConvDesc(N, H, W, C, K, R, S, sh, sw, ph, pw, WAP_RELU if relu else 0)


def fc_desc(B, n_in, n_out, relu=False):
    return FcDesc(B, n_in, n_out, WAP_RELU if relu else 0)


def wap_version():
    return lib().wap_version()


def wap_conv2d_workspace_bytes(desc, pass_):
    out = ctypes.c_size_t(0)
    _check(lib().wap_conv2d_workspace_bytes(ctypes.byref(desc), int(pass_), ctypes.byref(out)))
    return out.value


def wap_conv2d_kernel_name(desc, pass_):
    out = ctypes.c_char_p()
    _check(lib().wap_conv2d_kernel_name(ctypes.byref(desc), int(pass_), ctypes.byref(out)))
    return out.value.decode()


def wap_fc_workspace_bytes(desc, pass_):
    out = ctypes.c_size_t(0)
    _check(lib().wap_fc_workspace_bytes(ctypes.byref(desc), int(pass_), ctypes.byref(out)))
    return out.value


def wap_conv2d_fwd(desc, x, w, bias, y, ws=None, stream=None):
    _check(lib().wap_conv2d_fwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(ws),
                                ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


WAP_STATIC_SCRATCH_BYTES = 16 << 20


def wap_conv2d_fwd_static_ws(desc, x, w, bias, y, stream=None):
    _check(lib().wap_conv2d_fwd_static_ws(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _stream(stream)))


def wap_conv2d_fwd_pool2x2(desc, x, w, bias, y, y_pool, argmax, ws=None, stream=None):
    _check(lib().wap_conv2d_fwd_pool2x2(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(y_pool),
                                        _ptr(argmax), _ptr(ws), ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_fwd_pool2x2_fused(desc):
    out = ctypes.c_int32(0)
    _check(lib().wap_conv2d_fwd_pool2x2_fused(ctypes.byref(desc), ctypes.byref(out)))
    return bool(out.value)


def wap_conv2d_bwd_data(desc, dy, w, dx, ws=None, stream=None):
    _check(lib().wap_conv2d_bwd_data(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(dx), _ptr(ws),
                                     ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_bwd_data_relu(desc, dy, w, x_act, dx, ws=None, stream=None):
    _check(lib().wap_conv2d_bwd_data_relu(ctypes.byref(desc), _ptr(dy), _ptr(w), _ptr(x_act), _ptr(dx), _ptr(ws),
                                          ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_bwd_weight(desc, x, dy, dw, ws=None, stream=None):
    _check(lib().wap_conv2d_bwd_weight(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(dw), _ptr(ws),
                                       ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_bwd_data_pool2x2(desc, g_pool, argmax, w, x_act, dx, dy_full=None, ws=None, stream=None):
    _check(lib().wap_conv2d_bwd_data_pool2x2(ctypes.byref(desc), _ptr(g_pool), _ptr(argmax), _ptr(w), _ptr(x_act),
                                             _ptr(dx), _ptr(dy_full), _ptr(ws), ctypes.c_size_t(_nbytes(ws)),
                                             _stream(stream)))


def wap_conv2d_bwd_weight_pool2x2(desc, x, g_pool, argmax, dw, dy_full=None, ws=None, stream=None):
    _check(lib().wap_conv2d_bwd_weight_pool2x2(ctypes.byref(desc), _ptr(x), _ptr(g_pool), _ptr(argmax), _ptr(dw),
                                               _ptr(dy_full), _ptr(ws), ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_bwd_pool2x2_fused(desc, pass_):
    out = ctypes.c_int32(0)
    _check(lib().wap_conv2d_bwd_pool2x2_fused(ctypes.byref(desc), int(pass_), ctypes.byref(out)))
    return bool(out.value)


def wap_fc_fwd(desc, x, Wt, bias, y, ws=None, stream=None):
    _check(lib().wap_fc_fwd(ctypes.byref(desc), _ptr(x), _ptr(Wt), _ptr(bias), _ptr(y), _ptr(ws),
                            ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_fc_bwd(desc, x, Wt, dy, dx, dW, ws=None, stream=None):
    _check(lib().wap_fc_bwd(ctypes.byref(desc), _ptr(x), _ptr(Wt), _ptr(dy), _ptr(dx), _ptr(dW), _ptr(ws),
                            ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_bwd_weight_sgd(desc, x, dy, w32, w_bf16, lr, dw_scratch=None, ws=None, stream=None):
    _check(lib().wap_conv2d_bwd_weight_sgd(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(w32), _ptr(w_bf16),
                                           ctypes.c_float(lr), _ptr(dw_scratch), _ptr(ws),
                                           ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_fc_bwd_weight_sgd(desc, x, dy, w32, w_bf16, lr, dw_scratch=None, ws=None, stream=None):
    _check(lib().wap_fc_bwd_weight_sgd(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(w32), _ptr(w_bf16),
                                       ctypes.c_float(lr), _ptr(dw_scratch), _ptr(ws),
                                       ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_conv2d_bwd_weight_sgd_fused(desc):
    out = ctypes.c_int32(0)
    _check(lib().wap_conv2d_bwd_weight_sgd_fused(ctypes.byref(desc), ctypes.byref(out)))
    return bool(out.value)


def wap_fc_bwd_weight_sgd_fused(desc):
    out = ctypes.c_int32(0)
    _check(lib().wap_fc_bwd_weight_sgd_fused(ctypes.byref(desc), ctypes.byref(out)))
    return bool(out.value)


def wap_relu_bwd(dy, y, dx, n, stream=None):
    _check(lib().wap_relu_bwd(_ptr(dy), _ptr(y), _ptr(dx), ctypes.c_int64(n), _stream(stream)))


def wap_bias_grad_workspace_bytes(rows, cols):
    out = ctypes.c_size_t(0)
    _check(lib().wap_bias_grad_workspace_bytes(ctypes.c_int64(rows), int(cols), ctypes.byref(out)))
    return out.value


def wap_bias_grad(rows, cols, dy, db, ws, stream=None):
    _check(lib().wap_bias_grad(ctypes.c_int64(rows), int(cols), _ptr(dy), _ptr(db), _ptr(ws),
                               ctypes.c_size_t(_nbytes(ws)), _stream(stream)))


def wap_maxpool_fwd(N, H, W, C, win, st, x, y, argmax, stream=None):
    _check(lib().wap_maxpool_fwd(N, H, W, C, win, st, _ptr(x), _ptr(y), _ptr(argmax), _stream(stream)))


def wap_maxpool_bwd(N, H, W, C, win, st, dy, argmax, relu_y, dx, stream=None):
    _check(lib().wap_maxpool_bwd(N, H, W, C, win, st, _ptr(dy), _ptr(argmax), _ptr(relu_y), _ptr(dx),
                                 _stream(stream)))


def wap_softmax_xent_grad(B, classes, z, labels, loss, row_loss, dz, stream=None):
    _check(lib().wap_softmax_xent_grad(B, classes, _ptr(z), _ptr(labels), _ptr(loss), _ptr(row_loss),
                                       _ptr(dz), _stream(stream)))


def wap_sgd_update(n, w32, dw, lr, w_bf16, stream=None):
    _check(lib().wap_sgd_update(ctypes.c_int64(n), _ptr(w32), _ptr(dw), ctypes.c_float(lr), _ptr(w_bf16),
                                _stream(stream)))


def wap_cast_f32_bf16(n, src, dst, stream=None):
    _check(lib().wap_cast_f32_bf16(ctypes.c_int64(n), _ptr(src), _ptr(dst), _stream(stream)))


def wap_profile_scratch_bytes(kind, desc, minibatches):
    out = ctypes.c_size_t(0)
    n = len(minibatches)
    mbs = (ctypes.c_int32 * n)(*minibatches)
    _check(lib().wap_profile_scratch_bytes(int(kind), ctypes.byref(desc), mbs, n, ctypes.byref(out)))
    return out.value


def wap_profile_layer(kind, desc, minibatches, warmup, iters, scratch, stream=None):
    """Returns the list of ProfileRow (3 per minibatch: fwd, bwd-data, bwd-weight)."""
    n = len(minibatches)
    mbs = (ctypes.c_int32 * n)(*minibatches)
    rows = (ProfileRow * (3 * n))()
    written = ctypes.c_int32(0)
    _check(lib().wap_profile_layer(int(kind), ctypes.byref(desc), mbs, n, int(warmup), int(iters), _ptr(scratch),
                                   ctypes.c_size_t(_nbytes(scratch)), _stream(stream), rows, 3 * n,
                                   ctypes.byref(written)))
    return [rows[i] for i in range(written.value)]


def wap_mfma_ceiling_scratch_bytes():
    return int(lib().wap_mfma_ceiling_scratch_bytes())


def wap_measure_mfma_ceiling(data, feed, iters, scratch, stream=None):
    """Measured rate of the bf16 matrix pipe (data 0/1: constant / random operands; feed 0/1: registers only / the
    forward kernels' operand traffic); returns a MfmaCeilingRow."""
    row = MfmaCeilingRow()
    _check(lib().wap_measure_mfma_ceiling(int(data), int(feed), int(iters), _ptr(scratch),
                                          ctypes.c_size_t(_nbytes(scratch)), _stream(stream), ctypes.byref(row)))
    return row


class LinkModel(ctypes.Structure):
    _fields_ = [("link_bytes_per_s", ctypes.c_double), ("latency_s", ctypes.c_double)]


def wap_choose_gpus(t_c, grad_bytes, link_bytes_per_s, latency_s, allowed=None):
    """t_c: n_layers rows of max_gpus seconds; returns (best d, [t_estimate(d) for d = 1..max_gpus])."""
    n_layers, max_gpus = len(t_c), len(t_c[0])
    flat = (ctypes.c_double * (n_layers * max_gpus))(*[float(v) for row in t_c for v in row])
    gb = (ctypes.c_double * n_layers)(*[float(v) for v in grad_bytes])
    link = LinkModel(float(link_bytes_per_s), float(latency_s))
    mask = None if allowed is None else (ctypes.c_uint8 * max_gpus)(*[1 if a else 0 for a in allowed])
    est = (ctypes.c_double * max_gpus)()
    best = ctypes.c_int32(0)
    _check(lib().wap_choose_gpus(n_layers, max_gpus, flat, gb, ctypes.byref(link), mask, est, ctypes.byref(best)))
    return best.value, [float(est[i]) for i in range(max_gpus)]


class StepPlan:
    """Host-side launch list of one replica's training step (wap_step_plan_*)."""

    def __init__(self, net, minibatch, lr=0.01, image=224, flags=0):
        self._p = ctypes.c_void_p(0)
        _check(lib().wap_step_plan_create(net.encode(), int(minibatch), int(image), ctypes.c_float(lr),
                                          ctypes.c_uint32(flags), ctypes.byref(self._p)))
        self.net, self.minibatch, self.image = net, minibatch, image

    def __del__(self):
        try:
            if getattr(self, "_p", None) and self._p.value:
                lib().wap_step_plan_destroy(self._p)
                self._p = ctypes.c_void_p(0)
        except Exception:  # interpreter shutdown
            pass

    def arena_bytes(self):
        out = ctypes.c_size_t(0)
        _check(lib().wap_step_arena_bytes(self._p, ctypes.byref(out)))
        return out.value

    def tensors(self):
        """{name: (offset, bytes)} of every named tensor in the arena."""
        n = lib().wap_step_num_tensors(self._p)
        out = {}
        for i in range(n):
            name = ctypes.c_char_p()
            off, nb = ctypes.c_size_t(0), ctypes.c_size_t(0)
            _check(lib().wap_step_tensor(self._p, i, ctypes.byref(name), ctypes.byref(off), ctypes.byref(nb)))
            out[name.value.decode()] = (off.value, nb.value)
        return out

    def flops(self):
        return lib().wap_step_flops(self._p)

    def num_ops(self):
        return lib().wap_step_num_ops(self._p)

    def run(self, arena, stream=None):
        _check(lib().wap_step_run(self._p, _ptr(arena), ctypes.c_size_t(_nbytes(arena)), _stream(stream)))

    def ops(self):
        """[(name, kernel, flops, bytes)] for every operation of the launch list."""
        out = []
        for i in range(self.num_ops()):
            name, kern = ctypes.c_char_p(), ctypes.c_char_p()
            fl, by = ctypes.c_double(0), ctypes.c_double(0)
            _check(lib().wap_step_op_info(self._p, i, ctypes.byref(name), ctypes.byref(kern), ctypes.byref(fl),
                                          ctypes.byref(by)))
            out.append((name.value.decode(), kern.value.decode(), fl.value, by.value))
        return out

    def graph_capture(self, arena, stream):
        """Records the step for this arena as one HIP graph (after at least one eager run)."""
        _check(lib().wap_step_graph_capture(self._p, _ptr(arena), ctypes.c_size_t(_nbytes(arena)), _stream(stream)))

    def graph_launch(self, stream):
        _check(lib().wap_step_graph_launch(self._p, _stream(stream)))

    def time(self, arena, steps=1, stream=None, op_mask=None, with_prologue=False, every=1):
        """`steps` steps with events around every operation (or only those whose op_mask entry is true), in every
        `every`-th step: (main-kernel us, epilogue-kernel us) lists, plus the weight-repacking-kernel us list on
        request."""
        n = self.num_ops()
        us = (ctypes.c_float * n)()
        epi = (ctypes.c_float * n)()
        pro = (ctypes.c_float * n)()
        mask = None
        if op_mask is not None:
            if len(op_mask) != n:
                raise ValueError("op_mask needs one entry per operation")
            mask = (ctypes.c_uint8 * n)(*[1 if m else 0 for m in op_mask])
        _check(lib().wap_step_time_sampled(self._p, _ptr(arena), ctypes.c_size_t(_nbytes(arena)), _stream(stream),
                                           int(steps), int(every), mask, us, epi, pro))
        if with_prologue:
            return ([float(us[i]) for i in range(n)], [float(epi[i]) for i in range(n)],
                    [float(pro[i]) for i in range(n)])
        return [float(us[i]) for i in range(n)], [float(epi[i]) for i in range(n)]
