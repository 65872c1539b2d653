/*
 * wap.h -- C ABI of the MI355X (gfx950) per-replica training-step kernels.
 *
 * The library implements the compute side of one data-parallel replica (Section 2.1): the
 * forward and backward processing of every layer, i.e. the t_c(l_i, d) term of the run-time
 * estimate of Eq. 1 (Section 3.2.1), for the layer types the paper's parser extracts --
 * convolution and fully-connected "primary" nodes plus the activation / loss "auxiliary"
 * nodes (Section 3.2.2) and the weight update that follows gradient aggregation
 * (Section 3.2.3) -- and the measured per-layer time / utilisation table versus per-GPU
 * minibatch that the workload analysis unit evaluates Eq. 1 over.
 *
 * Conventions (all entry points):
 *   - extern "C"; return a wap_status; never throw, never abort.
 *   - Every tensor pointer is DEVICE memory owned by the caller, 16-byte aligned, and must stay
 *     alive until the work enqueued on `stream` has finished.  The library keeps no reference
 *     after return, allocates and frees no device memory and (except wap_profile_layer,
 *     wap_measure_mfma_ceiling and the step-plan timing helper) never synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - bf16 tensors are arrays of 16-bit bfloat16 bit patterns.  Accumulation is fp32.
 *     Conversions to bf16 round to nearest, ties to even.
 *   - Layouts: activations x[N][H][W][C] and y[N][P][Q][K]; conv weights w[K][R][S][C];
 *     FC weights Wt[out][in]; all row-major and dense.  P = floor((H + 2*pad_h - R)/stride_h) + 1.
 *   - Outputs are fully overwritten (no accumulate-into semantics).
 *   - Arguments are validated on the host before any device work: WAP_EINVAL for null
 *     pointers, non-positive sizes, pad >= filter size, misalignment; WAP_EUNSUPPORTED for
 *     sizes whose element counts exceed 2^31-1; WAP_EWORKSPACE when `ws_bytes` is below the
 *     matching *_workspace_bytes query; WAP_EHIP when a launch fails.  wap_last_error() gives
 *     the text of the last failure on the calling thread.
 *   - `ws` is scratch the caller provides (device memory, 256-byte aligned); it holds split
 *     reduction partials and may be NULL when the query returns 0.
 *   - Threads: calls may come from several host threads as long as each uses its own stream and
 *     buffers; one-time kernel attribute set-up is guarded.  wap_last_error() is per thread.
 */
#ifndef WAP_H
#define WAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WAP_OK = 0,
    WAP_EINVAL = 1,
    WAP_EUNSUPPORTED = 2,
    WAP_EWORKSPACE = 3,
    WAP_EHIP = 4
} wap_status;

/* flags */
#define WAP_RELU 1u /* forward epilogue applies max(.,0) after the optional bias */

/* One convolution layer's workload record (what the neural-net parser of Section 3.2.2
 * extracts: layer shape including the minibatch N).  Dilation 1, one group. */
typedef struct {
    int32_t N, H, W, C;       /* input  x[N][H][W][C] */
    int32_t K, R, S;          /* filter w[K][R][S][C] */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
    uint32_t flags;           /* WAP_RELU */
} wap_conv_desc;

/* One fully-connected layer's workload record: y[B][out] = x[B][in] * Wt[out][in]^T. */
typedef struct {
    int32_t B, in_features, out_features;
    uint32_t flags;           /* WAP_RELU */
} wap_fc_desc;

typedef enum { WAP_PASS_FWD = 0, WAP_PASS_BWD_DATA = 1, WAP_PASS_BWD_WEIGHT = 2 } wap_pass;

int wap_version(void);
const char* wap_last_error(void);

/* ---- convolution (primary node, Section 3.2.2; forward and backward halves of t_c, Eq. 1) ---- */

/* Scratch bytes the given pass needs for this descriptor (0 is possible). */
int wap_conv2d_workspace_bytes(const wap_conv_desc* d, int pass, size_t* bytes_out);

/* The kernel instantiation the shape-driven dispatch launches for this descriptor and pass (the main kernel;
 * host only, no device work).  The string is static. */
int wap_conv2d_kernel_name(const wap_conv_desc* d, int pass, const char** name_out);

/* y[n,p,q,k] = act( bias[k] + sum_{r,s,c} x[n, p*stride_h-pad_h+r, q*stride_w-pad_w+s, c] * w[k,r,s,c] ),
 * taps outside the image contribute zero.  x, w, y: bf16 device; bias: fp32 device [K] or NULL. */
int wap_conv2d_fwd(const wap_conv_desc* d, const void* x, const void* w, const float* bias,
                   void* y, void* ws, size_t ws_bytes, void* stream);

/* wap_conv2d_fwd for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus `ws`: the packed-weight
 * copy and split-reduction partials that wap_conv2d_fwd keeps in the caller's workspace live in a static device
 * array of WAP_STATIC_SCRATCH_BYTES inside the library (every GPU the process uses holds its own copy until the
 * process ends; its address is looked up once per device on the first call there, with that device current).
 * Same kernels, bit-identical y.  No hipMalloc / hipFree / allocating library call, no synchronisation.
 * WAP_EWORKSPACE (before any device work) when the layer's wap_conv2d_workspace_bytes(FWD) exceeds
 * WAP_STATIC_SCRATCH_BYTES (every convolution of the two networks at minibatches 8..256 fits).
 * All calls on one GPU share the one array and it keeps the last call's contents (each call overwrites what it
 * reads, nothing needs clearing): calls that can overlap on one GPU -- different streams, or several host
 * threads -- race on it; serialise them on one stream. */
#define WAP_STATIC_SCRATCH_BYTES (16u << 20)
int wap_conv2d_fwd_static_ws(const wap_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                             void* stream);

/* Convolution forward followed by a 2x2 / stride-2 max-pool of its (bias / ReLU applied) output, the
 * conv -> ReLU -> pool chain of a VGG block (primary node plus its auxiliary nodes, Section 3.2.2):
 * y_pool[n,p/2,q/2,k] and argmax (uint8, r*2+s of the first maximum in window scan order) exactly as
 * wap_conv2d_fwd followed by wap_maxpool_fwd(win 2, stride 2) would produce them.  P and Q must be even.
 * Where the tile kernel allows it (wap_conv2d_fwd_pool2x2_fused reports 1) the pool is taken from the
 * convolution's own epilogue and y may be NULL (the full-size output is then never written); otherwise
 * y is required and the two kernels run back to back. */
int wap_conv2d_fwd_pool2x2(const wap_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                           void* y_pool, uint8_t* argmax, void* ws, size_t ws_bytes, void* stream);
int wap_conv2d_fwd_pool2x2_fused(const wap_conv_desc* d, int32_t* fused_out);

/* dx[n,h,w,c] = sum_{k,r,s} dy[n,p,q,k] * w[k,r,s,c] over the (p,q) whose tap (r,s) reads (h,w).
 * dy: bf16 [N][P][Q][K]; dx: bf16 [N][H][W][C], every element written (zeros where the forward
 * pass never reads). */
int wap_conv2d_bwd_data(const wap_conv_desc* d, const void* dy, const void* w, void* dx,
                        void* ws, size_t ws_bytes, void* stream);

/* The same product followed by the ReLU derivative of the layer that produced x (the backward half of
 * t_c, Eq. 1, of a conv whose input is another layer's ReLU output): dx = (x_act > 0) ? dx : 0, with
 * x_act the bf16 [N][H][W][C] activation the forward pass consumed.  Where the tile kernel allows it the
 * mask is applied in the convolution's own epilogue, saving one read and one write of dx. */
int wap_conv2d_bwd_data_relu(const wap_conv_desc* d, const void* dy, const void* w, const void* x_act,
                             void* dx, void* ws, size_t ws_bytes, void* stream);

/* dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride_h-pad_h+r, q*stride_w-pad_w+s, c].
 * dw: fp32 [K][R][S][C] (the tensor a gradient all-reduce would move, Section 3.2.3).
 * The split reduction is summed in a fixed order: results are bitwise reproducible. */
int wap_conv2d_bwd_weight(const wap_conv_desc* d, const void* x, const void* dy, float* dw,
                          void* ws, size_t ws_bytes, void* stream);

/* Backward passes of a convolution whose (ReLU) output went through a 2x2 / stride-2 max-pool (the
 * conv -> ReLU -> pool chain of a VGG block; the pool's backward is an auxiliary node between two primary
 * nodes, Section 3.2.2).  Instead of the full-size dy the caller passes g_pool, the bf16 gradient w.r.t. the
 * POOLED output [N][P/2][Q/2][K], and argmax (uint8, same shape, r*2+s as written by wap_maxpool_fwd or
 * wap_conv2d_fwd_pool2x2); the operand the product sees is
 *     dy[n,p,q,k] = (argmax[n,p/2,q/2,k] == (p%2)*2 + q%2) ? g_pool[n,p/2,q/2,k] : 0,
 * i.e. wap_maxpool_bwd(win 2, stride 2, no ReLU mask) followed by wap_conv2d_bwd_data(_relu) /
 * wap_conv2d_bwd_weight, bit for bit.  P and Q must be even.  The ReLU derivative of the pooled layer
 * itself belongs in g_pool (mask it with the pooled activation > 0: the routed value is the window's
 * maximum).  Where the kernel's loader can do the routing (wap_conv2d_bwd_pool2x2_fused reports 1 for the
 * pass) the full-size dy never exists and dy_full may be NULL; otherwise dy_full (bf16 [N][P][Q][K]
 * device scratch) is required and the two kernels run back to back.  x_act of the data gradient is
 * optional (NULL: no ReLU derivative of the layer below). */
int wap_conv2d_bwd_data_pool2x2(const wap_conv_desc* d, const void* g_pool, const uint8_t* argmax, const void* w,
                                const void* x_act, void* dx, void* dy_full, void* ws, size_t ws_bytes, void* stream);
int wap_conv2d_bwd_weight_pool2x2(const wap_conv_desc* d, const void* x, const void* g_pool, const uint8_t* argmax,
                                  float* dw, void* dy_full, void* ws, size_t ws_bytes, void* stream);
/* pass: WAP_PASS_BWD_DATA or WAP_PASS_BWD_WEIGHT */
int wap_conv2d_bwd_pool2x2_fused(const wap_conv_desc* d, int pass, int32_t* fused_out);

/* ---- fully connected (primary node, Section 3.2.2) ---- */
int wap_fc_workspace_bytes(const wap_fc_desc* d, int pass, size_t* bytes_out);

/* y[b,o] = act( bias[o] + sum_i x[b,i] * Wt[o,i] );  x bf16 [B][in], Wt bf16 [out][in], y bf16 [B][out]. */
int wap_fc_fwd(const wap_fc_desc* d, const void* x, const void* Wt, const float* bias,
               void* y, void* ws, size_t ws_bytes, void* stream);

/* dx[b,i] = sum_o dy[b,o] * Wt[o,i] (bf16, skipped when dx is NULL);
 * dW[o,i] = sum_b dy[b,o] * x[b,i]  (fp32, skipped when dW is NULL).  dy bf16 [B][out].
 * `ws` must satisfy the larger of the BWD_DATA and BWD_WEIGHT queries. */
int wap_fc_bwd(const wap_fc_desc* d, const void* x, const void* Wt, const void* dy,
               void* dx, float* dW, void* ws, size_t ws_bytes, void* stream);

/* ---- auxiliary nodes (activation, pooling, loss: Section 3.2.2) and the weight update
 *      (Section 3.2.3).  The paper names them without formulas; the definitions are the
 *      standard ones, with the tie and zero-point rules stated here. ---- */

/* Bias gradient of a primary node whose epilogue adds bias[k] to every output pixel (rows = N*P*Q) or batch
 * row (rows = B) of channel k:  db[k] = sum over rows of dy[row][k].  dy: bf16 device [rows][cols];
 * db: fp32 device [cols]; ws: device scratch of wap_bias_grad_workspace_bytes.  Two-stage reduction in a
 * fixed order: bitwise reproducible. */
int wap_bias_grad_workspace_bytes(int64_t rows, int32_t cols, size_t* bytes_out);
int wap_bias_grad(int64_t rows, int32_t cols, const void* dy, float* db, void* ws, size_t ws_bytes, void* stream);

/* dx[i] = y[i] > 0 ? dy[i] : 0  (derivative at zero is zero).  bf16, n elements; dx may alias dy. */
int wap_relu_bwd(const void* dy, const void* y, void* dx, int64_t n, void* stream);

/* Max-pool, square window `win` (2 or 3), stride `st`, no padding, floor output size.
 * y bf16 [N][P][Q][C]; argmax uint8 [N][P][Q][C] = r*win+s of the FIRST maximum in (r, s) scan order. */
int wap_maxpool_fwd(int32_t N, int32_t H, int32_t W, int32_t C, int32_t win, int32_t st,
                    const void* x, void* y, uint8_t* argmax, void* stream);

/* dx[n,h,w,c] = sum of dy over the windows whose argmax is (h,w); every dx element written.
 * If relu_y is not NULL it is the pooled forward output y (bf16): contributions of windows with
 * y <= 0 are dropped, which fuses the backward of a ReLU placed just before the pool. */
int wap_maxpool_bwd(int32_t N, int32_t H, int32_t W, int32_t C, int32_t win, int32_t st,
                    const void* dy, const uint8_t* argmax, const void* relu_y, void* dx, void* stream);

/* Softmax cross-entropy, mean over the minibatch: p = softmax(z[b,:]) in fp32,
 * row_loss[b] = -log p[b,label_b] (fp32 [B]), loss = (1/B) sum_b row_loss[b] (one fp32 on device,
 * fixed summation order), dz[b,j] = (p[b,j] - [j == label_b]) / B stored bf16.
 * z bf16 [B][classes]; labels int32 [B], each in [0, classes); a label outside that range gives its row
 * no one-hot term and a row loss of 0 (never an out-of-range read). */
int wap_softmax_xent_grad(int32_t B, int32_t classes, const void* z, const int32_t* labels,
                          float* loss, float* row_loss, void* dz, void* stream);

/* Plain SGD on fp32 master weights: w32 <- w32 - lr*dw (fp32), then w_bf16 <- bf16(w32).
 * n elements; w_bf16 may be NULL. */
int wap_sgd_update(int64_t n, float* w32, const float* dw, float lr, void* w_bf16, void* stream);

/* Weight gradient and SGD update of one layer in one call (the weight-gradient half of t_c, Eq. 1,
 * followed by the weight update of Section 3.2.3): w32 <- w32 - lr * dw, w_bf16 <- bf16(w32), with dw exactly what wap_conv2d_bwd_weight / wap_fc_bwd
 * compute, and the same fused multiply-add and rounding as wap_sgd_update: bit for bit the result of those
 * two calls.  w32: fp32 master weights, w_bf16: bf16 compute copy (both required, 16-byte aligned, layout of
 * the layer's weights).  Where the kernel that finishes the gradient applies the update itself (the matching
 * *_sgd_fused query reports 1) the gradient is never stored and dw_scratch may be NULL; otherwise dw_scratch
 * (fp32, one element per weight, device) is required and the two kernels run back to back.  The caller must
 * have finished every product that reads this step's weights (the layer's data gradient) first. */
int wap_conv2d_bwd_weight_sgd(const wap_conv_desc* d, const void* x, const void* dy, float* w32, void* w_bf16,
                              float lr, float* dw_scratch, void* ws, size_t ws_bytes, void* stream);
int wap_fc_bwd_weight_sgd(const wap_fc_desc* d, const void* x, const void* dy, float* w32, void* w_bf16,
                          float lr, float* dw_scratch, void* ws, size_t ws_bytes, void* stream);
int wap_conv2d_bwd_weight_sgd_fused(const wap_conv_desc* d, int32_t* fused_out);
int wap_fc_bwd_weight_sgd_fused(const wap_fc_desc* d, int32_t* fused_out);

/* fp32 -> bf16 copy of n elements (used to derive the compute copy of freshly set master weights). */
int wap_cast_f32_bf16(int64_t n, const float* src, void* dst, void* stream);

/* ---- the per-layer time / utilisation table (the t_c(l_i, d) entries of Eq. 1 that the
 *      workload analysis unit of Section 3.2.1 sums and minimises over d) ---- */
typedef struct {
    int32_t pass;              /* wap_pass */
    int32_t minibatch;         /* per-GPU minibatch this row was timed at */
    double flops;              /* algorithmic: 2*N*P*Q*K*C*R*S (padding taps included) or 2*B*in*out */
    double alg_bytes;          /* every operand read once + output written once */
    double time_us_median;
    double time_us_min;
    double tflops;             /* flops / median time */
    double frac_of_bf16_peak;  /* against 2516.6 TFLOP/s */
    double gbytes_per_s;       /* alg_bytes / median time */
    double frac_of_hbm_peak;   /* against 8000 GB/s */
    int32_t bound;             /* 0 = MFMA side of the ridge, 1 = HBM side, 2 = launch / occupancy: the median
                                  time is more than 4x the time of BOTH roofs (flops / 2516.6 TFLOP/s and
                                  alg_bytes / 8 TB/s), i.e. too little work per launch to fill the chip -- the
                                  small-minibatch under-utilisation of Section 2.2 */
    int32_t reps_per_sample;   /* back-to-back launches one timed sample brackets (passes under 100 us: up to 8) */
} wap_profile_row;

/* Device scratch needed to profile the layer at every listed minibatch (inputs, outputs, workspace). */
int wap_profile_scratch_bytes(int kind /*0 conv, 1 fc*/, const void* desc, const int32_t* minibatches,
                              int32_t n_mb, size_t* bytes_out);

/* Times fwd, bwd-data and bwd-weight of one layer at each minibatch in `minibatches`
 * (the descriptor's N / B is replaced by the minibatch) with HIP events on `stream`:
 * `warmup` untimed launches (at least one), then `iters` timed samples per row, enqueued back to back
 * with one event between consecutive samples and a single host synchronisation at the end, so that
 * the host's launch latency is not inside a sample.  A sample is one pass (every kernel the pass
 * launches: weight repacking, main kernel, split reduction), or several back-to-back passes when
 * one is shorter than 100 us (reps_per_sample; times are per pass).  Writes 3*n_mb rows, ordered by
 * minibatch and within a minibatch by pass (fwd, bwd-data, bwd-weight).  Operands are a fixed
 * pseudo-random fill pattern generated on the device (times do not depend on values); this call
 * synchronises the stream. */
int wap_profile_layer(int kind, const void* desc, const int32_t* minibatches, int32_t n_mb,
                      int32_t warmup, int32_t iters, void* scratch, size_t scratch_bytes,
                      void* stream, wap_profile_row* rows_out, int32_t rows_cap, int32_t* rows_written);

/* What the bf16 matrix pipe of this device sustains, measured: the yardstick beside the published peak for the
 * utilisation figures above (Table 1; the measured t_c of Eq. 1, Section 3.2.1).  The chip lowers its clock under
 * load, by an amount that depends on the operand values and on what else runs per MFMA, so no kernel can reach
 * clock_max x units; this times a loop of v_mfma_f32_32x32x16_bf16 on every CU (two work-groups of four
 * wavefronts per CU, 7 independent accumulators per wavefront) and reports its rate and the average shader clock.
 *   data: 0 = every operand 1.0; 1 = pseudo-random bf16 operands (random sign and mantissa, exponents 2^-3 .. 2^0).
 *   feed: 0 = operands stay in registers; 1 = the operand traffic of the forward / data-gradient kernels' main
 *         loop (per 7 MFMAs seven 16-byte LDS reads and one 16-byte L2-resident global load).
 *   iters: loop trips per wavefront (7 MFMAs each), 1 .. 2^20; a warm-up launch of iters / 8 + 1 trips runs first.
 * `scratch`: device memory, wap_mfma_ceiling_scratch_bytes() bytes, 256-byte aligned (overwritten).  Synchronises
 * `stream` before returning.  WAP_EINVAL for arguments outside the ranges above, WAP_EWORKSPACE for the scratch. */
typedef struct wap_mfma_ceiling_row {
    int32_t data, feed;
    double tflops;     /* 2 * 32 * 32 * 16 FLOP per MFMA over the timed launch */
    double clock_ghz;  /* shader clock counter against the constant 100 MHz counter, read inside the kernel */
    double us;         /* duration of the timed launch (HIP events) */
} wap_mfma_ceiling_row;
size_t wap_mfma_ceiling_scratch_bytes(void);
int wap_measure_mfma_ceiling(int32_t data, int32_t feed, int32_t iters, void* scratch, size_t scratch_bytes,
                             void* stream, wap_mfma_ceiling_row* out);

/* ---- the workload analysis unit's decision (Section 3.2.1): how many GPUs to divide the workload over ----
 * Evaluates Eq. 1, t_estimate(d) = sum over layers of { t_c(l, d) + t_s(l, d) }, for d = 1..max_gpus and
 * returns the d with the smallest estimate.  Host arithmetic only (fp64); no device work, no stream.
 *   t_c          host, [n_layers][max_gpus] seconds: entry (l, d-1) is the forward + backward time of layer l
 *                at the divided workload (per-GPU minibatch B/d), e.g. summed from wap_profile_layer rows;
 *   grad_bytes   host, [n_layers]: bytes of layer l's weight gradient (what the aggregation moves);
 *   link         ring all-reduce model of Section 3.2.3: t_s(l, d) = 0 for d = 1, otherwise
 *                2 (d-1)/d * grad_bytes[l] / link_bytes_per_s + 2 (d-1) * latency_s;
 *   allowed      host, [max_gpus] or NULL: non-zero where d is a usable division (e.g. d divides the minibatch);
 *   t_estimate_out  host, [max_gpus]: the estimates (+infinity where d is not allowed);
 *   best_d_out   the minimiser; an exact tie goes to the smaller d (fewer GPUs for the same time).
 * WAP_EINVAL for NULL / non-positive sizes, negative or non-finite times or bytes, a non-positive bandwidth,
 * a negative latency, or no allowed d. */
typedef struct {
    double link_bytes_per_s;
    double latency_s;
} wap_link_model;
int wap_choose_gpus(int32_t n_layers, int32_t max_gpus, const double* t_c, const double* grad_bytes,
                    const wap_link_model* link, const uint8_t* allowed, double* t_estimate_out,
                    int32_t* best_d_out);

/* ---- whole training step of one replica: forward, loss, backward, SGD (host-side launch list) ---- */
typedef struct wap_step_plan wap_step_plan;

/* net: "alexnet" or "vgg16" (layer lists of Section 4.1's two networks, 224x224x3 inputs,
 * 1000 classes).  The plan is host memory only.
 * flags: WAP_STEP_KEEP_GRADS keeps every intermediate gradient in a tensor of its own and every operation
 * unfused (for inspection); WAP_STEP_BIAS gives every conv / FC layer an fp32 bias (tensors "<layer>.b32",
 * gradient "<layer>.db"): added in the forward epilogues, its gradient (column sums of the gradient w.r.t. the
 * layer's pre-activation output) computed by one extra operation per layer, updated by the same SGD launch.
 * Without the flag the layers have no bias, which is how the benchmark runs.
 * By default the kernel that finishes a layer's weight gradient applies the SGD update itself (the gradient
 * tensor "<layer>.dw" is then not written): the form of a job on one GPU, where nothing else needs the
 * gradient.  WAP_STEP_STORE_GRADS stores every weight gradient and updates in a separate pass at the end of
 * the step instead: the form a replica of a data-parallel job needs, whose gradients are exchanged
 * (Section 2.1) between the backward pass and the update. */
#define WAP_STEP_KEEP_GRADS 1u
#define WAP_STEP_BIAS 2u
#define WAP_STEP_STORE_GRADS 4u
int wap_step_plan_create(const char* net, int32_t minibatch, int32_t image, float lr, uint32_t flags,
                         wap_step_plan** out);
void wap_step_plan_destroy(wap_step_plan* p);
/* Bytes of the single device arena the step runs in (weights, activations, gradients, workspace). */
int wap_step_arena_bytes(const wap_step_plan* p, size_t* bytes_out);
/* Number of named tensors in the arena and their placement; names are e.g. "conv1_1.w32",
 * "conv1_1.w", "conv1_1.y", "pool1.y", "fc6.dW", "input", "labels", "loss". */
int wap_step_num_tensors(const wap_step_plan* p);
int wap_step_tensor(const wap_step_plan* p, int32_t index, const char** name, size_t* offset,
                    size_t* bytes);
/* Enqueues one full step on `stream`: no allocation, no synchronisation. */
int wap_step_run(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream);
/* The same step as one HIP graph: wap_step_graph_capture records the launch list for this arena on `stream`
 * (stream capture; nothing executes) and instantiates it, replacing any graph captured before;
 * wap_step_graph_launch replays it.  The list holds kernel launches only (no memset or copy nodes).  At least
 * one wap_step_run on this plan must have completed before the capture (first launches set kernel
 * attributes, which capture does not allow): WAP_EINVAL otherwise.  The graph is bound to the arena address
 * it was captured with and is released by wap_step_plan_destroy. */
int wap_step_graph_capture(wap_step_plan* p, void* arena, size_t arena_bytes, void* stream);
int wap_step_graph_launch(const wap_step_plan* p, void* stream);
/* Algorithmic FLOPs of one step (direct-convolution count, first layer's data gradient excluded). */
double wap_step_flops(const wap_step_plan* p);
/* Number of operations in the launch list (an operation is one kernel, or a kernel plus its
 * split-reduction epilogue). */
int wap_step_num_ops(const wap_step_plan* p);
/* Operation `index` of the launch list: its name (e.g. "conv3_2.wgrad"), the kernel instantiation
 * it launches, and its algorithmic FLOPs and bytes (operands read once, outputs written once).
 * Strings are owned by the plan. */
int wap_step_op_info(const wap_step_plan* p, int32_t index, const char** name, const char** kernel,
                     double* flops, double* bytes);
/* Runs `steps` steps back to back with a HIP event pair around every operation (events are created
 * on first use and cached in the plan); fills us_out[num_ops] with the mean duration in microseconds
 * of each operation's main kernel and us_epilogue_out[num_ops] with that of its split-reduction
 * epilogue kernel (0 where the operation has none).  The weight-repacking kernel that precedes some
 * convolution kernels is outside both (see wap_step_time_masked).  Synchronises the stream once, at
 * the end. */
int wap_step_time(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream, int32_t steps,
                  float* us_out, float* us_epilogue_out);
/* The same with events only around the operations whose op_mask[index] is non-zero (host array of
 * num_ops bytes, NULL = all): the other operations run unbracketed and report 0, so that a timed
 * region can carry the events of one kernel without the launch gaps the full instrumentation adds
 * (two event records per operation, about 0.5 ms per VGG-16 step). */
int wap_step_time_masked(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream, int32_t steps,
                         const uint8_t* op_mask, float* us_out, float* us_epilogue_out, float* us_prologue_out);
/* us_prologue_out (host, num_ops floats, may be NULL): mean duration of the weight-repacking kernel an
 * operation launches before its main kernel (0 where it has none). */
/* The same with the events only in steps 0, every, 2 * every, ... of the `steps` back-to-back steps (means over
 * those steps): an event record between two kernels costs a few microseconds of launch gap, so a timed region
 * that brackets a kernel in every step is measurably longer than the plain region (VGG-16 step: 22 records,
 * about 1.5 %); sampled steps keep the live measurement and leave the region all but undisturbed. */
int wap_step_time_sampled(const wap_step_plan* p, void* arena, size_t arena_bytes, void* stream, int32_t steps,
                          int32_t every, const uint8_t* op_mask, float* us_out, float* us_epilogue_out,
                          float* us_prologue_out);

#ifdef __cplusplus
}
#endif
#endif /* WAP_H */
