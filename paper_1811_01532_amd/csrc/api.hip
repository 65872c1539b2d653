// C ABI of libwap: argument validation (host only, before any device work), descriptor ->
// kernel-geometry translation and dispatch.  Declarations and contracts are in include/wap.h.
#include <cstdarg>
#include <cstdio>

#include "wap_internal.h"

namespace wap {

namespace {
thread_local char g_err[512] = "";
}

int g_force_fwd_cfg = -1, g_force_wgrad_cfg = -1, g_force_nsplit = -1;

int set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_error(WAP_EHIP, "%s launch failed: %s", what, hipGetErrorString(e));
    return WAP_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static const long long kMaxElems = 2147483647LL;

static int out_dim(int in, int pad, int win, int stride) { return (in + 2 * pad - win) / stride + 1; }

int validate_conv(const wap_conv_desc* d) {
    if (!d) return set_error(WAP_EINVAL, "conv descriptor is NULL");
    if (d->N < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->K < 1 || d->R < 1 || d->S < 1)
        return set_error(WAP_EINVAL, "conv descriptor: every size must be >= 1 (N=%d H=%d W=%d C=%d K=%d R=%d S=%d)",
                         d->N, d->H, d->W, d->C, d->K, d->R, d->S);
    if (d->stride_h < 1 || d->stride_w < 1) return set_error(WAP_EINVAL, "conv descriptor: stride must be >= 1");
    if (d->pad_h < 0 || d->pad_w < 0 || d->pad_h >= d->R || d->pad_w >= d->S)
        return set_error(WAP_EINVAL, "conv descriptor: need 0 <= pad < filter size (pad %d,%d filter %d,%d)",
                         d->pad_h, d->pad_w, d->R, d->S);
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S)
        return set_error(WAP_EINVAL, "conv descriptor: filter larger than the padded input");
    if (d->flags & ~WAP_RELU) return set_error(WAP_EINVAL, "conv descriptor: unknown flag bits 0x%x", d->flags);
    if (d->R > 255 || d->S > 255) return set_error(WAP_EUNSUPPORTED, "conv descriptor: filter side above 255");
    long long P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
    long long xe = (long long)d->N * d->H * d->W * d->C;
    long long ye = (long long)d->N * P * Q * d->K;
    long long we = (long long)d->K * d->R * d->S * d->C;
    long long he = (long long)d->N * d->H * d->W, pe = (long long)d->N * P * Q;
    if (xe > kMaxElems || ye > kMaxElems || we > kMaxElems || he * 1 > kMaxElems || pe > kMaxElems)
        return set_error(WAP_EUNSUPPORTED, "conv descriptor: a tensor exceeds 2^31-1 elements");
    return WAP_OK;
}

int validate_fc(const wap_fc_desc* d) {
    if (!d) return set_error(WAP_EINVAL, "fc descriptor is NULL");
    if (d->B < 1 || d->in_features < 1 || d->out_features < 1)
        return set_error(WAP_EINVAL, "fc descriptor: every size must be >= 1 (B=%d in=%d out=%d)", d->B,
                         d->in_features, d->out_features);
    if (d->flags & ~WAP_RELU) return set_error(WAP_EINVAL, "fc descriptor: unknown flag bits 0x%x", d->flags);
    long long a = (long long)d->B * d->in_features, b = (long long)d->B * d->out_features;
    long long w = (long long)d->in_features * d->out_features;
    if (a > kMaxElems || b > kMaxElems || w > kMaxElems)
        return set_error(WAP_EUNSUPPORTED, "fc descriptor: a tensor exceeds 2^31-1 elements");
    return WAP_OK;
}

GemmGeom geom_conv_fwd(const wap_conv_desc& d) {
    GemmGeom g;
    g.IH = d.H; g.IW = d.W; g.IC = d.C;
    g.OH = out_dim(d.H, d.pad_h, d.R, d.stride_h);
    g.OW = out_dim(d.W, d.pad_w, d.S, d.stride_w);
    g.R = d.R; g.S = d.S;
    g.mul_h = d.stride_h; g.mul_w = d.stride_w;
    g.div_h = 1; g.div_w = 1;
    g.pad_h = d.pad_h; g.pad_w = d.pad_w;
    g.M = d.N * g.OH * g.OW;
    g.Ncols = d.K;
    g.Kred = d.R * d.S * d.C;
    return g;
}

// rows = input pixels (n,h,w); gathered tensor = dy[N][P][Q][K]; reduction (r',s',k) with flipped taps
// r' = R-1-r: th = h - (R-1-pad) + r' = h + pad - r, p = th / stride when divisible.
GemmGeom geom_conv_dgrad(const wap_conv_desc& d) {
    GemmGeom g;
    g.IH = out_dim(d.H, d.pad_h, d.R, d.stride_h);
    g.IW = out_dim(d.W, d.pad_w, d.S, d.stride_w);
    g.IC = d.K;
    g.OH = d.H; g.OW = d.W;
    g.R = d.R; g.S = d.S;
    g.mul_h = 1; g.mul_w = 1;
    g.div_h = d.stride_h; g.div_w = d.stride_w;
    g.pad_h = d.R - 1 - d.pad_h; g.pad_w = d.S - 1 - d.pad_w;
    g.M = d.N * d.H * d.W;
    g.Ncols = d.C;
    g.Kred = d.R * d.S * d.K;
    return g;
}

WgradGeom geom_conv_wgrad(const wap_conv_desc& d) {
    WgradGeom g;
    g.N = d.N; g.H = d.H; g.W = d.W; g.C = d.C; g.K = d.K; g.R = d.R; g.S = d.S;
    g.sh = d.stride_h; g.sw = d.stride_w; g.ph = d.pad_h; g.pw = d.pad_w;
    g.P = out_dim(d.H, d.pad_h, d.R, d.stride_h);
    g.Q = out_dim(d.W, d.pad_w, d.S, d.stride_w);
    return g;
}

static wap_conv_desc fc_as_conv(const wap_fc_desc& d) {
    wap_conv_desc c;
    c.N = d.B; c.H = 1; c.W = 1; c.C = d.in_features; c.K = d.out_features; c.R = 1; c.S = 1;
    c.stride_h = 1; c.stride_w = 1; c.pad_h = 0; c.pad_w = 0; c.flags = d.flags;
    return c;
}
GemmGeom geom_fc_fwd(const wap_fc_desc& d) { return geom_conv_fwd(fc_as_conv(d)); }
GemmGeom geom_fc_dx(const wap_fc_desc& d) { return geom_conv_dgrad(fc_as_conv(d)); }
WgradGeom geom_fc_dw(const wap_fc_desc& d) { return geom_conv_wgrad(fc_as_conv(d)); }

static int check_ptr(const void* p, const char* name) {
    if (!p) return set_error(WAP_EINVAL, "%s is NULL", name);
    if (!aligned16(p)) return set_error(WAP_EINVAL, "%s is not 16-byte aligned", name);
    return WAP_OK;
}

static int check_ws(size_t need, void* ws, size_t ws_bytes) {
    if (need == 0) return WAP_OK;
    if (!ws) return set_error(WAP_EWORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (ws_bytes < need) return set_error(WAP_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    if (!aligned16(ws)) return set_error(WAP_EINVAL, "workspace is not 16-byte aligned");
    return WAP_OK;
}

}  // namespace wap

using namespace wap;

#define WAP_TRY(expr)              \
    do {                           \
        int rc__ = (expr);         \
        if (rc__ != WAP_OK) return rc__; \
    } while (0)

extern "C" {

int wap_version(void) { return 100; }

void wap_debug_force(int fwd_cfg, int wgrad_cfg, int nsplit) {
    g_force_fwd_cfg = fwd_cfg;
    g_force_wgrad_cfg = wgrad_cfg;
    g_force_nsplit = nsplit;
}
const char* wap_last_error(void) { return g_err; }

int wap_conv2d_workspace_bytes(const wap_conv_desc* d, int pass, size_t* bytes_out) {
    WAP_TRY(validate_conv(d));
    if (!bytes_out) return set_error(WAP_EINVAL, "bytes_out is NULL");
    if (pass == WAP_PASS_FWD) *bytes_out = plan_fwd_like(geom_conv_fwd(*d), false).ws_bytes;
    else if (pass == WAP_PASS_BWD_DATA) *bytes_out = plan_fwd_like(geom_conv_dgrad(*d), true).ws_bytes;
    else if (pass == WAP_PASS_BWD_WEIGHT) *bytes_out = plan_wgrad(geom_conv_wgrad(*d)).ws_bytes;
    else return set_error(WAP_EINVAL, "unknown pass %d", pass);
    return WAP_OK;
}

int wap_conv2d_kernel_name(const wap_conv_desc* d, int pass, const char** name_out) {
    WAP_TRY(validate_conv(d));
    if (!name_out) return set_error(WAP_EINVAL, "name_out is NULL");
    if (pass == WAP_PASS_FWD) {
        GemmGeom g = geom_conv_fwd(*d);
        *name_out = fwd_like_kernel_name(g, false, plan_fwd_like(g, false));
    } else if (pass == WAP_PASS_BWD_DATA) {
        GemmGeom g = geom_conv_dgrad(*d);
        *name_out = fwd_like_kernel_name(g, true, plan_fwd_like(g, true));
    } else if (pass == WAP_PASS_BWD_WEIGHT) {
        WgradGeom g = geom_conv_wgrad(*d);
        *name_out = wgrad_kernel_name(g, plan_wgrad(g));
    } else {
        return set_error(WAP_EINVAL, "unknown pass %d", pass);
    }
    return WAP_OK;
}

int wap_conv2d_fwd(const wap_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                   void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(w, "w"));
    WAP_TRY(check_ptr(y, "y"));
    if (bias && !aligned16(bias)) return set_error(WAP_EINVAL, "bias is not 16-byte aligned");
    GemmGeom g = geom_conv_fwd(*d);
    GemmPlan p = plan_fwd_like(g, false);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    return launch_fwd_like(g, false, p, (const bf16_t*)x, (const bf16_t*)w, bias, (d->flags & WAP_RELU) != 0,
                           (bf16_t*)y, ws, (hipStream_t)stream);
}

// ---- forward convolution for callers that cannot allocate: the workspace is a static device array ----
}  // extern "C" (reopened below: the array and its per-device address are file-scope objects)

// One copy of this array exists on every GPU the library runs on, from module load until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress; kernels and launches get the per-device address.
static __device__ __align__(256) unsigned char scratch[WAP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxDevices];

// device address of `scratch` on the current device, looked up once per device (with that device current)
int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_error(WAP_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return set_error(WAP_EUNSUPPORTED, "device ordinal %d above %d", dev, kMaxDevices - 1);
    void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return set_error(WAP_EHIP, "hipGetSymbolAddress(static scratch): %s", hipGetErrorString(e));
        g_scratch_addr[dev].store(p, std::memory_order_release);   // the same address whichever thread wins
    }
    *out = p;
    return WAP_OK;
}
}  // namespace

extern "C" {

int wap_conv2d_fwd_static_ws(const wap_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                             void* stream) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(w, "w"));
    WAP_TRY(check_ptr(y, "y"));
    if (bias && !aligned16(bias)) return set_error(WAP_EINVAL, "bias is not 16-byte aligned");
    GemmGeom g = geom_conv_fwd(*d);
    GemmPlan p = plan_fwd_like(g, false);
    if (p.ws_bytes > (size_t)WAP_STATIC_SCRATCH_BYTES)
        return set_error(WAP_EWORKSPACE, "conv2d_fwd_static_ws: this layer needs %zu bytes of workspace, the static scratch "
                         "holds %zu; use wap_conv2d_fwd with a caller workspace", p.ws_bytes, (size_t)WAP_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (p.ws_bytes) WAP_TRY(static_scratch(&ws));
    return launch_fwd_like(g, false, p, (const bf16_t*)x, (const bf16_t*)w, bias, (d->flags & WAP_RELU) != 0,
                           (bf16_t*)y, ws, (hipStream_t)stream);
}

int wap_conv2d_fwd_pool2x2_fused(const wap_conv_desc* d, int32_t* fused_out) {
    WAP_TRY(validate_conv(d));
    if (!fused_out) return set_error(WAP_EINVAL, "fwd_pool2x2_fused: NULL argument");
    GemmGeom g = geom_conv_fwd(*d);
    *fused_out = fwd_like_fuses_pool(g, plan_fwd_like(g, false)) ? 1 : 0;
    return WAP_OK;
}

int wap_conv2d_fwd_pool2x2(const wap_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                           void* y_pool, uint8_t* argmax, void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(w, "w"));
    WAP_TRY(check_ptr(y_pool, "y_pool"));
    WAP_TRY(check_ptr(argmax, "argmax"));
    GemmGeom g = geom_conv_fwd(*d);
    if ((g.OH & 1) || (g.OW & 1)) return set_error(WAP_EINVAL, "fwd_pool2x2: output size %dx%d is not even", g.OH, g.OW);
    GemmPlan p = plan_fwd_like(g, false);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    const bool relu = (d->flags & WAP_RELU) != 0;
    if (fwd_like_fuses_pool(g, p))
        return launch_fwd_like(g, false, p, (const bf16_t*)x, (const bf16_t*)w, bias, relu, (bf16_t*)y, ws,
                               (hipStream_t)stream, nullptr, nullptr, nullptr, nullptr, (bf16_t*)y_pool, argmax);
    if (!y) return set_error(WAP_EINVAL, "fwd_pool2x2: this shape is not fused, y is required");
    WAP_TRY(launch_fwd_like(g, false, p, (const bf16_t*)x, (const bf16_t*)w, bias, relu, (bf16_t*)y, ws,
                            (hipStream_t)stream));
    return launch_maxpool_fwd(d->N, g.OH, g.OW, d->K, 2, 2, (const bf16_t*)y, (bf16_t*)y_pool, argmax,
                              (hipStream_t)stream);
}

int wap_conv2d_bwd_data(const wap_conv_desc* d, const void* dy, const void* w, void* dx, void* ws,
                        size_t ws_bytes, void* stream) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(w, "w"));
    WAP_TRY(check_ptr(dx, "dx"));
    GemmGeom g = geom_conv_dgrad(*d);
    GemmPlan p = plan_fwd_like(g, true);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    return launch_fwd_like(g, true, p, (const bf16_t*)dy, (const bf16_t*)w, nullptr, false, (bf16_t*)dx, ws,
                           (hipStream_t)stream);
}

int wap_conv2d_bwd_data_relu(const wap_conv_desc* d, const void* dy, const void* w, const void* x_act, void* dx,
                             void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(w, "w"));
    WAP_TRY(check_ptr(x_act, "x_act"));
    WAP_TRY(check_ptr(dx, "dx"));
    GemmGeom g = geom_conv_dgrad(*d);
    GemmPlan p = plan_fwd_like(g, true);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    return launch_fwd_like(g, true, p, (const bf16_t*)dy, (const bf16_t*)w, nullptr, false, (bf16_t*)dx, ws,
                           (hipStream_t)stream, nullptr, (const bf16_t*)x_act);
}

int wap_conv2d_bwd_weight(const wap_conv_desc* d, const void* x, const void* dy, float* dw, void* ws,
                          size_t ws_bytes, void* stream) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(dw, "dw"));
    WgradGeom g = geom_conv_wgrad(*d);
    WgradPlan p = plan_wgrad(g);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    return launch_wgrad(g, p, (const bf16_t*)x, (const bf16_t*)dy, dw, ws, (hipStream_t)stream);
}

static int bwd_weight_sgd(const WgradGeom& g, const void* x, const void* dy, float* w32, void* w_bf16, float lr,
                          float* dw_scratch, void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(w32, "w32"));
    WAP_TRY(check_ptr(w_bf16, "w_bf16"));
    WgradPlan p = plan_wgrad(g);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    hipStream_t st = (hipStream_t)stream;
    if (wgrad_fuses_sgd(g, p)) {
        const SgdFuse sgd = {w32, (bf16_t*)w_bf16, lr};
        return launch_wgrad(g, p, (const bf16_t*)x, (const bf16_t*)dy, nullptr, ws, st, nullptr, nullptr, &sgd);
    }
    if (!dw_scratch) return set_error(WAP_EINVAL, "bwd_weight_sgd: dw_scratch is NULL and this shape does not fuse the update");
    if (!aligned16(dw_scratch)) return set_error(WAP_EINVAL, "dw_scratch is not 16-byte aligned");
    WAP_TRY(launch_wgrad(g, p, (const bf16_t*)x, (const bf16_t*)dy, dw_scratch, ws, st));
    return launch_sgd((size_t)g.K * g.R * g.S * g.C, w32, dw_scratch, lr, (bf16_t*)w_bf16, st);
}

int wap_conv2d_bwd_weight_sgd(const wap_conv_desc* d, const void* x, const void* dy, float* w32, void* w_bf16,
                              float lr, float* dw_scratch, void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(validate_conv(d));
    return bwd_weight_sgd(geom_conv_wgrad(*d), x, dy, w32, w_bf16, lr, dw_scratch, ws, ws_bytes, stream);
}

int wap_fc_bwd_weight_sgd(const wap_fc_desc* d, const void* x, const void* dy, float* w32, void* w_bf16,
                          float lr, float* dw_scratch, void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(validate_fc(d));
    return bwd_weight_sgd(geom_fc_dw(*d), x, dy, w32, w_bf16, lr, dw_scratch, ws, ws_bytes, stream);
}

int wap_conv2d_bwd_weight_sgd_fused(const wap_conv_desc* d, int32_t* fused_out) {
    WAP_TRY(validate_conv(d));
    if (!fused_out) return set_error(WAP_EINVAL, "fused_out is NULL");
    WgradGeom g = geom_conv_wgrad(*d);
    *fused_out = wgrad_fuses_sgd(g, plan_wgrad(g)) ? 1 : 0;
    return WAP_OK;
}

int wap_fc_bwd_weight_sgd_fused(const wap_fc_desc* d, int32_t* fused_out) {
    WAP_TRY(validate_fc(d));
    if (!fused_out) return set_error(WAP_EINVAL, "fused_out is NULL");
    WgradGeom g = geom_fc_dw(*d);
    *fused_out = wgrad_fuses_sgd(g, plan_wgrad(g)) ? 1 : 0;
    return WAP_OK;
}

static int check_pool2x2_bwd(const wap_conv_desc* d, const void* g_pool, const uint8_t* argmax) {
    WAP_TRY(validate_conv(d));
    WAP_TRY(check_ptr(g_pool, "g_pool"));
    WAP_TRY(check_ptr(argmax, "argmax"));
    const int P = out_dim(d->H, d->pad_h, d->R, d->stride_h), Q = out_dim(d->W, d->pad_w, d->S, d->stride_w);
    if ((P & 1) || (Q & 1)) return set_error(WAP_EINVAL, "bwd_pool2x2: output size %dx%d is not even", P, Q);
    return WAP_OK;
}

int wap_conv2d_bwd_pool2x2_fused(const wap_conv_desc* d, int pass, int32_t* fused_out) {
    WAP_TRY(validate_conv(d));
    if (!fused_out) return set_error(WAP_EINVAL, "bwd_pool2x2_fused: NULL argument");
    if (pass == WAP_PASS_BWD_DATA) {
        GemmGeom g = geom_conv_dgrad(*d);
        *fused_out = fwd_like_fuses_unpool(g, plan_fwd_like(g, true)) ? 1 : 0;
    } else if (pass == WAP_PASS_BWD_WEIGHT) {
        WgradGeom g = geom_conv_wgrad(*d);
        *fused_out = wgrad_fuses_unpool(g, plan_wgrad(g)) ? 1 : 0;
    } else {
        return set_error(WAP_EINVAL, "bwd_pool2x2_fused: pass %d is not a backward pass", pass);
    }
    return WAP_OK;
}

int wap_conv2d_bwd_data_pool2x2(const wap_conv_desc* d, const void* g_pool, const uint8_t* argmax, const void* w,
                                const void* x_act, void* dx, void* dy_full, void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(check_pool2x2_bwd(d, g_pool, argmax));
    WAP_TRY(check_ptr(w, "w"));
    WAP_TRY(check_ptr(dx, "dx"));
    if (x_act && !aligned16(x_act)) return set_error(WAP_EINVAL, "x_act is not 16-byte aligned");
    GemmGeom g = geom_conv_dgrad(*d);
    GemmPlan p = plan_fwd_like(g, true);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    if (fwd_like_fuses_unpool(g, p))
        return launch_fwd_like(g, true, p, (const bf16_t*)g_pool, (const bf16_t*)w, nullptr, false, (bf16_t*)dx, ws,
                               (hipStream_t)stream, nullptr, (const bf16_t*)x_act, nullptr, nullptr, nullptr, nullptr,
                               argmax);
    WAP_TRY(check_ptr(dy_full, "dy_full (this shape is not fused)"));
    WAP_TRY(launch_maxpool_bwd(d->N, g.IH, g.IW, d->K, 2, 2, (const bf16_t*)g_pool, argmax, nullptr, (bf16_t*)dy_full,
                               (hipStream_t)stream));
    return launch_fwd_like(g, true, p, (const bf16_t*)dy_full, (const bf16_t*)w, nullptr, false, (bf16_t*)dx, ws,
                           (hipStream_t)stream, nullptr, (const bf16_t*)x_act);
}

int wap_conv2d_bwd_weight_pool2x2(const wap_conv_desc* d, const void* x, const void* g_pool, const uint8_t* argmax,
                                  float* dw, void* dy_full, void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(check_pool2x2_bwd(d, g_pool, argmax));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(dw, "dw"));
    WgradGeom g = geom_conv_wgrad(*d);
    WgradPlan p = plan_wgrad(g);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    if (wgrad_fuses_unpool(g, p))
        return launch_wgrad(g, p, (const bf16_t*)x, (const bf16_t*)g_pool, dw, ws, (hipStream_t)stream, nullptr, argmax);
    WAP_TRY(check_ptr(dy_full, "dy_full (this shape is not fused)"));
    WAP_TRY(launch_maxpool_bwd(d->N, g.P, g.Q, d->K, 2, 2, (const bf16_t*)g_pool, argmax, nullptr, (bf16_t*)dy_full,
                               (hipStream_t)stream));
    return launch_wgrad(g, p, (const bf16_t*)x, (const bf16_t*)dy_full, dw, ws, (hipStream_t)stream);
}

int wap_fc_workspace_bytes(const wap_fc_desc* d, int pass, size_t* bytes_out) {
    WAP_TRY(validate_fc(d));
    if (!bytes_out) return set_error(WAP_EINVAL, "bytes_out is NULL");
    if (pass == WAP_PASS_FWD) *bytes_out = plan_fwd_like(geom_fc_fwd(*d), false).ws_bytes;
    else if (pass == WAP_PASS_BWD_DATA) *bytes_out = plan_fwd_like(geom_fc_dx(*d), true).ws_bytes;
    else if (pass == WAP_PASS_BWD_WEIGHT) *bytes_out = plan_wgrad(geom_fc_dw(*d)).ws_bytes;
    else return set_error(WAP_EINVAL, "unknown pass %d", pass);
    return WAP_OK;
}

int wap_fc_fwd(const wap_fc_desc* d, const void* x, const void* Wt, const float* bias, void* y, void* ws,
               size_t ws_bytes, void* stream) {
    WAP_TRY(validate_fc(d));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(Wt, "Wt"));
    WAP_TRY(check_ptr(y, "y"));
    if (bias && !aligned16(bias)) return set_error(WAP_EINVAL, "bias is not 16-byte aligned");
    GemmGeom g = geom_fc_fwd(*d);
    GemmPlan p = plan_fwd_like(g, false);
    WAP_TRY(check_ws(p.ws_bytes, ws, ws_bytes));
    return launch_fwd_like(g, false, p, (const bf16_t*)x, (const bf16_t*)Wt, bias, (d->flags & WAP_RELU) != 0,
                           (bf16_t*)y, ws, (hipStream_t)stream);
}

int wap_fc_bwd(const wap_fc_desc* d, const void* x, const void* Wt, const void* dy, void* dx, float* dW,
               void* ws, size_t ws_bytes, void* stream) {
    WAP_TRY(validate_fc(d));
    WAP_TRY(check_ptr(dy, "dy"));
    if (!dx && !dW) return set_error(WAP_EINVAL, "both dx and dW are NULL");
    if (dx) {
        WAP_TRY(check_ptr(Wt, "Wt"));
        if (!aligned16(dx)) return set_error(WAP_EINVAL, "dx is not 16-byte aligned");
    }
    if (dW) {
        WAP_TRY(check_ptr(x, "x"));
        if (!aligned16(dW)) return set_error(WAP_EINVAL, "dW is not 16-byte aligned");
    }
    GemmGeom gx = geom_fc_dx(*d);
    GemmPlan px = plan_fwd_like(gx, true);
    WgradGeom gw = geom_fc_dw(*d);
    WgradPlan pw = plan_wgrad(gw);
    size_t need = 0;
    if (dx) need = px.ws_bytes;
    if (dW && pw.ws_bytes > need) need = pw.ws_bytes;
    WAP_TRY(check_ws(need, ws, ws_bytes));
    if (dx)
        WAP_TRY(launch_fwd_like(gx, true, px, (const bf16_t*)dy, (const bf16_t*)Wt, nullptr, false, (bf16_t*)dx,
                                ws, (hipStream_t)stream));
    if (dW) WAP_TRY(launch_wgrad(gw, pw, (const bf16_t*)x, (const bf16_t*)dy, dW, ws, (hipStream_t)stream));
    return WAP_OK;
}

int wap_bias_grad_workspace_bytes(int64_t rows, int32_t cols, size_t* bytes_out) {
    if (!bytes_out) return set_error(WAP_EINVAL, "bias_grad: NULL argument");
    if (rows < 1 || cols < 1) return set_error(WAP_EINVAL, "bias_grad: rows and cols must be >= 1");
    if ((long long)rows * cols > kMaxElems) return set_error(WAP_EUNSUPPORTED, "bias_grad: tensor exceeds 2^31-1 elements");
    *bytes_out = (size_t)bias_grad_chunks((size_t)rows, cols) * cols * sizeof(float);
    return WAP_OK;
}

int wap_bias_grad(int64_t rows, int32_t cols, const void* dy, float* db, void* ws, size_t ws_bytes, void* stream) {
    size_t need = 0;
    WAP_TRY(wap_bias_grad_workspace_bytes(rows, cols, &need));
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(db, "db"));
    WAP_TRY(check_ws(need, ws, ws_bytes));
    return launch_bias_grad((size_t)rows, cols, (const bf16_t*)dy, db, (float*)ws, (hipStream_t)stream);
}

int wap_relu_bwd(const void* dy, const void* y, void* dx, int64_t n, void* stream) {
    if (n < 1) return set_error(WAP_EINVAL, "relu_bwd: n must be >= 1");
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(y, "y"));
    WAP_TRY(check_ptr(dx, "dx"));
    return launch_relu_bwd((const bf16_t*)dy, (const bf16_t*)y, (bf16_t*)dx, (size_t)n, (hipStream_t)stream);
}

static int validate_pool(int32_t N, int32_t H, int32_t W, int32_t C, int32_t win, int32_t st) {
    if (N < 1 || H < 1 || W < 1 || C < 1) return set_error(WAP_EINVAL, "maxpool: every size must be >= 1");
    if (win < 1 || win > 15 || st < 1) return set_error(WAP_EINVAL, "maxpool: need 1 <= window <= 15 and stride >= 1");
    if (H < win || W < win) return set_error(WAP_EINVAL, "maxpool: window larger than the input");
    if ((long long)N * H * W * C > kMaxElems) return set_error(WAP_EUNSUPPORTED, "maxpool: tensor exceeds 2^31-1 elements");
    return WAP_OK;
}

int wap_maxpool_fwd(int32_t N, int32_t H, int32_t W, int32_t C, int32_t win, int32_t st, const void* x,
                    void* y, uint8_t* argmax, void* stream) {
    WAP_TRY(validate_pool(N, H, W, C, win, st));
    WAP_TRY(check_ptr(x, "x"));
    WAP_TRY(check_ptr(y, "y"));
    WAP_TRY(check_ptr(argmax, "argmax"));
    return launch_maxpool_fwd(N, H, W, C, win, st, (const bf16_t*)x, (bf16_t*)y, argmax, (hipStream_t)stream);
}

int wap_maxpool_bwd(int32_t N, int32_t H, int32_t W, int32_t C, int32_t win, int32_t st, const void* dy,
                    const uint8_t* argmax, const void* relu_y, void* dx, void* stream) {
    WAP_TRY(validate_pool(N, H, W, C, win, st));
    WAP_TRY(check_ptr(dy, "dy"));
    WAP_TRY(check_ptr(argmax, "argmax"));
    WAP_TRY(check_ptr(dx, "dx"));
    if (relu_y && !aligned16(relu_y)) return set_error(WAP_EINVAL, "relu_y is not 16-byte aligned");
    return launch_maxpool_bwd(N, H, W, C, win, st, (const bf16_t*)dy, argmax, (const bf16_t*)relu_y,
                              (bf16_t*)dx, (hipStream_t)stream);
}

int wap_softmax_xent_grad(int32_t B, int32_t classes, const void* z, const int32_t* labels, float* loss,
                          float* row_loss, void* dz, void* stream) {
    if (B < 1 || classes < 1) return set_error(WAP_EINVAL, "softmax: B and classes must be >= 1");
    if ((long long)B * classes > kMaxElems) return set_error(WAP_EUNSUPPORTED, "softmax: tensor exceeds 2^31-1 elements");
    WAP_TRY(check_ptr(z, "z"));
    WAP_TRY(check_ptr(labels, "labels"));
    WAP_TRY(check_ptr(loss, "loss"));
    WAP_TRY(check_ptr(row_loss, "row_loss"));
    WAP_TRY(check_ptr(dz, "dz"));
    return launch_softmax_xent(B, classes, (const bf16_t*)z, labels, loss, row_loss, (bf16_t*)dz,
                               (hipStream_t)stream);
}

int wap_sgd_update(int64_t n, float* w32, const float* dw, float lr, void* w_bf16, void* stream) {
    if (n < 1) return set_error(WAP_EINVAL, "sgd: n must be >= 1");
    WAP_TRY(check_ptr(w32, "w32"));
    WAP_TRY(check_ptr(dw, "dw"));
    if (w_bf16 && !aligned16(w_bf16)) return set_error(WAP_EINVAL, "w_bf16 is not 16-byte aligned");
    return launch_sgd((size_t)n, w32, dw, lr, (bf16_t*)w_bf16, (hipStream_t)stream);
}

int wap_cast_f32_bf16(int64_t n, const float* src, void* dst, void* stream) {
    if (n < 1) return set_error(WAP_EINVAL, "cast: n must be >= 1");
    WAP_TRY(check_ptr(src, "src"));
    WAP_TRY(check_ptr(dst, "dst"));
    return launch_cast((size_t)n, src, (bf16_t*)dst, (hipStream_t)stream);
}

}  // extern "C"
