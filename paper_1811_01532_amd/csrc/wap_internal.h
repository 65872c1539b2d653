// Internal declarations shared by the HIP translation units of libwap (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "../../include/wap.h"
#include "../../include/wap_testing.h"

namespace wap {

typedef unsigned short bf16_t;  // raw bfloat16 bits in memory

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // one 16-byte load/store as an SSA value
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;  // one 8-byte load

// exact floor(x / d) for 0 <= x < 2^31 by multiply-high and shift (d >= 1)
struct FastDiv {
    uint32_t mul, shift;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    uint32_t sh = 0;
    while ((1ull << sh) < d) ++sh;
    f.shift = sh;
    f.mul = (uint32_t)((((1ull << 32) * ((1ull << sh) - d)) / d) + 1);
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t x, FastDiv f) { return (__umulhi(x, f.mul) + x) >> f.shift; }

constexpr double kPeakBf16Tflops = 2516.6;  // 256 CU x 4096 FLOP/clk x 2.4 GHz
constexpr double kPeakHbmGBs = 8000.0;
constexpr int kNumCU = 256;
constexpr int kNumXCD = 8;

// ---- SGD update fused into the kernel that produces a weight gradient ----
// Instead of storing dW, the producer applies w32 <- w32 - lr * dW to the fp32 master weights and re-derives the
// bf16 compute copy, element for element what sgd_kernel does with a stored gradient (same fused multiply-add,
// same rounding), so both routes give the same bits.
struct SgdFuse {
    float* w32;
    bf16_t* wb;
    float lr;
};
__device__ __forceinline__ float sgd_apply(float w, float g, float lr) { return __builtin_fmaf(-lr, g, w); }
// one 16-byte group of parameters (old values in `a`): write the updated master weights and four bf16 values
__device__ __forceinline__ void sgd_store4(float* w32, bf16_t* wb, float4 a, float lr, float g0, float g1, float g2,
                                           float g3) {
    a.x = sgd_apply(a.x, g0, lr); a.y = sgd_apply(a.y, g1, lr); a.z = sgd_apply(a.z, g2, lr); a.w = sgd_apply(a.w, g3, lr);
    *reinterpret_cast<float4*>(w32) = a;
    __bf16 b0 = (__bf16)a.x, b1 = (__bf16)a.y, b2 = (__bf16)a.z, b3 = (__bf16)a.w;
    uint2 pk;
    pk.x = (unsigned)__builtin_bit_cast(unsigned short, b0) | ((unsigned)__builtin_bit_cast(unsigned short, b1) << 16);
    pk.y = (unsigned)__builtin_bit_cast(unsigned short, b2) | ((unsigned)__builtin_bit_cast(unsigned short, b3) << 16);
    *reinterpret_cast<uint2*>(wb) = pk;
}
__device__ __forceinline__ void sgd_apply4(float* w32, bf16_t* wb, float lr, float g0, float g1, float g2, float g3) {
    sgd_store4(w32, wb, *reinterpret_cast<const float4*>(w32), lr, g0, g1, g2, g3);
}

// ---- test hook: force a tile configuration / split count (-1 = choose from the shape) ----
extern int g_force_fwd_cfg, g_force_wgrad_cfg, g_force_nsplit;

// ---- error reporting (thread local) ----
int set_error(int code, const char* fmt, ...);
int check_launch(const char* what);

// ---- implicit-GEMM problem, in the form the kernels consume ----
// Rows m = (n, oh, ow) of the "row space"; reduction index kk = (r, s, ic) with ic innermost;
// the gathered element is A[n][ih][iw][ic] with th = oh*mul_h - pad_h + r, ih = th/div_h
// (valid when th >= 0, th % div_h == 0, ih < IH), likewise for the width.
struct GemmGeom {
    int IH, IW, IC;
    int OH, OW;
    int R, S;
    int mul_h, mul_w, div_h, div_w, pad_h, pad_w;
    int M;      // N * OH * OW
    int Ncols;  // output channels of this product
    int Kred;   // R * S * IC
};

// How a forward-type product (rows = pixels, reduction = filter taps x channels) is tiled.
struct GemmPlan {
    int cfg;     // tile configuration id
    int nsplit;  // reduction splits (1 = direct epilogue)
    size_t ws_bytes;
};

// Weight operand addressing.
//  NT : Bw[n][kk]               (forward conv / FC forward): row pitch Kred
//  TR : Bw[k][R-1-r][S-1-s][n]  (data gradient: reduction (r,s,k), k innermost): n contiguous
GemmPlan plan_fwd_like(const GemmGeom& g, bool b_tr);
int launch_fwd_like(const GemmGeom& g, bool b_tr, const GemmPlan& plan, const bf16_t* A,
                    const bf16_t* Bw, const float* bias, bool relu, bf16_t* out, void* ws,
                    hipStream_t st, hipEvent_t ev_mid = nullptr,  // ev_mid: recorded between kernel and split epilogue
                    const bf16_t* relu_mask = nullptr,   // out = relu_mask > 0 ? out : 0 (same shape as out)
                    hipEvent_t ev_packed = nullptr,      // recorded after the weight repacking, if the plan has one
                    const void* prepacked = nullptr,     // weights already in packed order: skip the repacking
                    bf16_t* pool_y = nullptr,            // 2x2 / stride-2 max-pool of the output from the same epilogue
                    uint8_t* pool_am = nullptr,          // (only where fwd_like_fuses_pool; `out` may then be NULL)
                    const uint8_t* unpool_am = nullptr,  // A is the gradient of the 2x2 / stride-2 pooled tensor and this the
                                                         // pool's argmax (only where fwd_like_fuses_unpool)
                    float* colsum = nullptr);            // column sums of the stored output, one partial row per pixel
                                                         // tile (only where fwd_like_colsum_rows > 0; not with pool_y)
int fwd_like_colsum_rows(const GemmGeom& g, const GemmPlan& plan);  // 0: the plan's kernel cannot emit column sums
// Fixed-order column sums of fp32 matrices [rows][cols] (cols % 4 == 0), all of a step in one pair of launches; byte
// offsets are relative to one base pointer; part2 holds colsum_f32_chunks(rows) x cols floats per matrix.
struct ColsumJob {
    int rows, cols, chunks;
    size_t part_off, part2_off, out_off;
};
constexpr int kMaxColsumJobs = 24;
struct ColsumJobs {
    int n;
    int first[kMaxColsumJobs + 1];  // first work-group of each job in the first-stage grid
    ColsumJob job[kMaxColsumJobs];
};
int colsum_f32_chunks(size_t rows);
int colsum_jobs_add(ColsumJobs& js, int rows, int cols, size_t part_off, size_t part2_off, size_t out_off);  // -1: full / bad
int launch_colsum_f32_multi(const ColsumJobs& js, void* base, hipStream_t st);
bool fwd_like_fuses_unpool(const GemmGeom& g, const GemmPlan& plan);
bool fwd_like_fuses_pool(const GemmGeom& g, const GemmPlan& plan);
bool fwd_like_packs_weights(const GemmPlan& plan);
bool fwd_like_fuses_mask(const GemmGeom& g, const GemmPlan& plan);  // mask applied in the kernel's own epilogue?

// Weight-gradient product: dw[k][(r,s,c)] = sum over pixels of dy[pix][k] * x[pix @ (r,s)][c].
struct WgradGeom {
    int N, H, W, C, K, R, S, sh, sw, ph, pw, P, Q;
};
struct WgradPlan {
    int cfg;
    int nsplit;
    size_t ws_bytes;
};
WgradPlan plan_wgrad(const WgradGeom& g);
// unpool_am: dy is the gradient of the 2x2 / stride-2 max-pooled output (N x P/2 x Q/2 x K) and unpool_am the pool's
// argmax; only where wgrad_fuses_unpool() says so.
// sgd: apply the update to the parameters instead of storing dW (dw may then be NULL); only where wgrad_fuses_sgd()
// says so.
int launch_wgrad(const WgradGeom& g, const WgradPlan& plan, const bf16_t* x, const bf16_t* dy,
                 float* dw, void* ws, hipStream_t st, hipEvent_t ev_mid = nullptr, const uint8_t* unpool_am = nullptr,
                 const SgdFuse* sgd = nullptr);
bool wgrad_fuses_unpool(const WgradGeom& g, const WgradPlan& plan);
bool wgrad_fuses_sgd(const WgradGeom& g, const WgradPlan& plan);
const char* wgrad_kernel_name(const WgradGeom& g, const WgradPlan& plan, bool unpool);

// stride-1 3x3 weight gradient with the input patch resident in LDS (wgrad_patch.hip)
bool wgrad_patch_supported(const WgradGeom& g);
int wgrad_patch_nsplit(const WgradGeom& g);
bool wgrad_patch_fuses_unpool(const WgradGeom& g);
const char* wgrad_patch_kernel_name(const WgradGeom& g, bool unpool);
int launch_wgrad_patch(const WgradGeom& g, int nsplit, const bf16_t* x, const bf16_t* dy, float* out, hipStream_t st,
                       const uint8_t* unpool_am = nullptr);

// 3-input-channel 3x3 stride-1 first layer (conv_c3.hip)
bool conv_c3_fwd_supported(const GemmGeom& g);
const char* conv_c3_fwd_kernel_name(const GemmGeom& g);
int launch_conv_c3_fwd(const GemmGeom& g, const bf16_t* x, const bf16_t* w, const float* bias, bool relu, bf16_t* y,
                       hipStream_t st);
bool wgrad_c3_supported(const WgradGeom& g);
const char* wgrad_c3_kernel_name(const WgradGeom& g);
int wgrad_c3_nsplit(const WgradGeom& g);
int launch_wgrad_c3(const WgradGeom& g, int nsplit, const bf16_t* x, const bf16_t* dy, float* part, hipStream_t st);

// data gradient with at most four output columns, on the vector ALUs (dgrad_thin.hip); g = data-gradient geometry
bool dgrad_thin_supported(const GemmGeom& g);
size_t dgrad_thin_ws_bytes(const GemmGeom& g);
int launch_dgrad_thin(const GemmGeom& g, const bf16_t* dy, const bf16_t* w, bf16_t* dx, void* ws, hipStream_t st);

// weights-in-registers large-tile kernel (conv_wreg.hip)
bool wreg_supported(const GemmGeom& g);
inline size_t wreg_wt_bytes(const GemmGeom& g) { return (size_t)((g.Ncols + 31) / 32) * 32 * g.Kred * 2; }  // packed copy
int launch_pack_weights(const GemmGeom& g, bool flip, const bf16_t* w, void* Wp, hipStream_t st);
// All packing jobs of a launch list in one kernel (offsets are relative to one base pointer).
struct PackJob {
    size_t w_off, out_off;  // byte offsets of the source weights and of the packed copy
    int Ncols, Kred, IC, R, S, flip;
};
constexpr int kMaxPackJobs = 32;
struct PackJobs {
    int n;
    size_t first[kMaxPackJobs + 1];  // first 16-byte vector of each job in the concatenated index space
    PackJob job[kMaxPackJobs];
};
void pack_jobs_add(PackJobs& js, const GemmGeom& g, bool flip, size_t w_off, size_t out_off);
int launch_pack_weights_multi(const PackJobs& js, void* base, hipStream_t st);
int launch_wreg(const GemmGeom& g, int nsplit, const bf16_t* A, const bf16_t* Bw, const float* bias, bool relu,
                void* out, bool partial, hipStream_t st);

// stride-1 convolution with the input patch resident in LDS (conv_patch.hip)
int patch_supported(const GemmGeom& g);
const char* patch_kernel_name(const GemmGeom& g);
int launch_patch(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                 hipStream_t st, const bf16_t* mask = nullptr);

// stride-1 convolution on 256-pixel 2-D tiles x 64 output channels, three work-groups per CU (conv_tile64.hip)
int tile64_width(const GemmGeom& g);  // 0: not applicable
const char* tile64_kernel_name(const GemmGeom& g, bool unpool);
bool tile64_fuses_unpool(const GemmGeom& g);
int launch_tile64(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                  hipStream_t st, const bf16_t* mask, bf16_t* pool_y, uint8_t* pool_am, const uint8_t* unpool_am,
                  float* colsum = nullptr);

// stride-1 convolution with double-buffered 32-channel patch slices: 2-D, strip and flat tiles (conv_tile2d.hip;
// it hands the shapes of conv_tile64.hip on to that kernel)
int tile2d_supported(const GemmGeom& g);
bool tile2d_preferred(const GemmGeom& g);
const char* tile2d_kernel_name(const GemmGeom& g, bool unpool);
int launch_tile2d(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                  hipStream_t st, const bf16_t* mask = nullptr, bf16_t* pool_y = nullptr, uint8_t* pool_am = nullptr,
                  const uint8_t* unpool_am = nullptr,
                  float* colsum = nullptr);  // [tile2d_colsum_rows][Ncols] column sums of the stored (masked) output
int tile2d_colsum_rows(const GemmGeom& g);
bool tile2d_fuses_pool(const GemmGeom& g);
bool tile2d_fuses_unpool(const GemmGeom& g);

const char* fwd_like_kernel_name(const GemmGeom& g, bool b_tr, const GemmPlan& plan, bool unpool = false);
const char* wgrad_kernel_name(const WgradGeom& g, const WgradPlan& plan);

// split-reduction epilogues (fixed summation order)
int launch_reduce_bf16(const float* part, int nsplit, size_t elems, int ncols, const float* bias,
                       bool relu, bf16_t* out, hipStream_t st);
// with `sgd`, the sums update the parameters (see SgdFuse) instead of being stored; `out` is then unused
int launch_reduce_f32(const float* part, int nsplit, size_t elems, float* out, hipStream_t st,
                      const SgdFuse* sgd = nullptr);

// fill helpers used by the profiler
int launch_fill_bf16(bf16_t* p, size_t n, uint32_t seed, hipStream_t st);

// memory-bound kernels
int launch_relu_bwd(const bf16_t* dy, const bf16_t* y, bf16_t* dx, size_t n, hipStream_t st);
int bias_grad_chunks(size_t rows, int cols);  // row chunks (= partial sums per column) of the first stage
int launch_bias_grad(size_t rows, int cols, const bf16_t* dy, float* db, float* part, hipStream_t st);
int launch_maxpool_fwd(int N, int H, int W, int C, int win, int stp, const bf16_t* x, bf16_t* y,
                       uint8_t* am, hipStream_t st);
int launch_maxpool_bwd(int N, int H, int W, int C, int win, int stp, const bf16_t* dy, const uint8_t* am,
                       const bf16_t* ry, bf16_t* dx, hipStream_t st);
int launch_softmax_xent(int B, int classes, const bf16_t* z, const int32_t* labels, float* loss,
                        float* row_loss, bf16_t* dz, hipStream_t st);
int launch_sgd(size_t n, float* w, const float* dw, float lr, bf16_t* wb, hipStream_t st);
int launch_cast(size_t n, const float* src, bf16_t* dst, hipStream_t st);

// descriptor -> kernel geometry (after validation)
GemmGeom geom_conv_fwd(const wap_conv_desc& d);
GemmGeom geom_conv_dgrad(const wap_conv_desc& d);
WgradGeom geom_conv_wgrad(const wap_conv_desc& d);
GemmGeom geom_fc_fwd(const wap_fc_desc& d);
GemmGeom geom_fc_dx(const wap_fc_desc& d);
WgradGeom geom_fc_dw(const wap_fc_desc& d);
int validate_conv(const wap_conv_desc* d);
int validate_fc(const wap_fc_desc* d);

}  // namespace wap
