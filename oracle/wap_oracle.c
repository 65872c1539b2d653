/*
 * wap_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU definitions of every operation on the per-replica training step
 * (the t_c term of Eq. 1, Section 3.2.1: forward and backward processing of each layer):
 * convolution forward / data-gradient / weight-gradient, fully-connected forward / backward,
 * ReLU backward, max-pool forward / backward, softmax cross-entropy with its gradient, and the
 * SGD weight update (the "primary" and "auxiliary" computation nodes of Section 3.2.2 and the
 * weight update of Section 3.2.3).  The paper names these node types and gives no formula for
 * any of them, so each function below is the textbook definition written out as loops, with
 * the readings listed beside it.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call this file; it shares no code with the HIP library and never includes its headers.
 *
 * Layouts: activations x[N][H][W][C], y[N][P][Q][K]; conv weights w[K][R][S][C];
 * FC weights Wt[out][in]; everything double, row-major.  P = floor((H+2*ph-R)/sh)+1.
 * Convolution means cross-correlation (no filter flip).  Taps that fall in the zero padding
 * contribute nothing.
 *
 * Pins (see tests/test_oracle_*.py): independent NumPy brute force over an explicitly padded
 * array, delta-filter shift (bit exact), all-ones closed form, 1x1 conv and FC against fp64
 * matmul, full-window conv == FC, adjoint identities <conv(x,w),g> = <x,dgrad(g,w)> =
 * <w,wgrad(x,g)>, finite differences, pool sum conservation, ln(classes) loss at zero logits.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

static int out_dim(int in, int pad, int win, int stride) { return (in + 2 * pad - win) / stride + 1; }

int orc_out_dim(int in, int pad, int win, int stride) { return out_dim(in, pad, win, stride); }

/* ---- convolution forward: y[n,p,q,k] = bias[k] + sum_{r,s,c} x[n,p*sh-ph+r,q*sw-pw+s,c] * w[k,r,s,c] ---- */
static double conv_fwd_one(const double* x, const double* w, const double* bias, int H, int W, int C,
                           int R, int S, int sh, int sw, int ph, int pw, int relu,
                           int n, int p, int q, int k) {
    double acc = bias ? bias[k] : 0.0;
    for (int r = 0; r < R; ++r) {
        int h = p * sh - ph + r;
        if (h < 0 || h >= H) continue;
        for (int s = 0; s < S; ++s) {
            int ww = q * sw - pw + s;
            if (ww < 0 || ww >= W) continue;
            const double* xp = x + (((size_t)n * H + h) * W + ww) * C;
            const double* wp = w + (((size_t)k * R + r) * S + s) * C;
            for (int c = 0; c < C; ++c) acc += xp[c] * wp[c];
        }
    }
    if (relu && !(acc > 0.0)) acc = 0.0;
    return acc;
}

void orc_conv2d_fwd(const double* x, const double* w, const double* bias, double* y,
                    int N, int H, int W, int C, int K, int R, int S,
                    int sh, int sw, int ph, int pw, int relu) {
    int P = out_dim(H, ph, R, sh), Q = out_dim(W, pw, S, sw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < K; ++k)
                    y[(((size_t)n * P + p) * Q + q) * K + k] =
                        conv_fwd_one(x, w, bias, H, W, C, R, S, sh, sw, ph, pw, relu, n, p, q, k);
}

/* same definition, evaluated only at the listed flat indices of y */
void orc_conv2d_fwd_at(const double* x, const double* w, const double* bias,
                       int N, int H, int W, int C, int K, int R, int S,
                       int sh, int sw, int ph, int pw, int relu,
                       const int64_t* idx, int64_t n_idx, double* out) {
    int P = out_dim(H, ph, R, sh), Q = out_dim(W, pw, S, sw);
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        int k = (int)(f % K); f /= K;
        int q = (int)(f % Q); f /= Q;
        int p = (int)(f % P); f /= P;
        int n = (int)f;
        out[i] = conv_fwd_one(x, w, bias, H, W, C, R, S, sh, sw, ph, pw, relu, n, p, q, k);
    }
}

/* ---- data gradient, written as a gather from the dx side:
 *      dx[n,h,w,c] = sum_{k,r,s} dy[n,p,q,k] * w[k,r,s,c]  over the (p,q) with p*sh-ph+r = h, q*sw-pw+s = w ---- */
static double conv_dgrad_one(const double* dy, const double* w, int C, int K, int R, int S,
                             int sh, int sw, int ph, int pw, int P, int Q,
                             int n, int h, int ww, int c) {
    double acc = 0.0;
    for (int k = 0; k < K; ++k)
        for (int r = 0; r < R; ++r) {
            int hp = h + ph - r;
            if (hp < 0 || hp % sh != 0) continue;
            int p = hp / sh;
            if (p >= P) continue;
            for (int s = 0; s < S; ++s) {
                int wq = ww + pw - s;
                if (wq < 0 || wq % sw != 0) continue;
                int q = wq / sw;
                if (q >= Q) continue;
                acc += dy[(((size_t)n * P + p) * Q + q) * K + k] * w[(((size_t)k * R + r) * S + s) * C + c];
            }
        }
    return acc;
}

void orc_conv2d_bwd_data(const double* dy, const double* w, double* dx,
                         int N, int H, int W, int C, int K, int R, int S,
                         int sh, int sw, int ph, int pw) {
    int P = out_dim(H, ph, R, sh), Q = out_dim(W, pw, S, sw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int h = 0; h < H; ++h)
            for (int ww = 0; ww < W; ++ww)
                for (int c = 0; c < C; ++c)
                    dx[(((size_t)n * H + h) * W + ww) * C + c] =
                        conv_dgrad_one(dy, w, C, K, R, S, sh, sw, ph, pw, P, Q, n, h, ww, c);
}

void orc_conv2d_bwd_data_at(const double* dy, const double* w,
                            int N, int H, int W, int C, int K, int R, int S,
                            int sh, int sw, int ph, int pw,
                            const int64_t* idx, int64_t n_idx, double* out) {
    int P = out_dim(H, ph, R, sh), Q = out_dim(W, pw, S, sw);
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        int c = (int)(f % C); f /= C;
        int ww = (int)(f % W); f /= W;
        int h = (int)(f % H); f /= H;
        int n = (int)f;
        out[i] = conv_dgrad_one(dy, w, C, K, R, S, sh, sw, ph, pw, P, Q, n, h, ww, c);
    }
}

/* ---- weight gradient: dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n,p*sh-ph+r,q*sw-pw+s,c] ---- */
static double conv_wgrad_one(const double* x, const double* dy, int N, int H, int W, int C, int K,
                             int sh, int sw, int ph, int pw, int P, int Q,
                             int k, int r, int s, int c) {
    double acc = 0.0;
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p) {
            int h = p * sh - ph + r;
            if (h < 0 || h >= H) continue;
            for (int q = 0; q < Q; ++q) {
                int ww = q * sw - pw + s;
                if (ww < 0 || ww >= W) continue;
                acc += dy[(((size_t)n * P + p) * Q + q) * K + k] * x[(((size_t)n * H + h) * W + ww) * C + c];
            }
        }
    return acc;
}

void orc_conv2d_bwd_weight(const double* x, const double* dy, double* dw,
                           int N, int H, int W, int C, int K, int R, int S,
                           int sh, int sw, int ph, int pw) {
    int P = out_dim(H, ph, R, sh), Q = out_dim(W, pw, S, sw);
    int64_t total = (int64_t)K * R * S * C;
#pragma omp parallel for schedule(static)
    for (int64_t f = 0; f < total; ++f) {
        int64_t g = f;
        int c = (int)(g % C); g /= C;
        int s = (int)(g % S); g /= S;
        int r = (int)(g % R); g /= R;
        int k = (int)g;
        dw[f] = conv_wgrad_one(x, dy, N, H, W, C, K, sh, sw, ph, pw, P, Q, k, r, s, c);
    }
}

void orc_conv2d_bwd_weight_at(const double* x, const double* dy,
                              int N, int H, int W, int C, int K, int R, int S,
                              int sh, int sw, int ph, int pw,
                              const int64_t* idx, int64_t n_idx, double* out) {
    int P = out_dim(H, ph, R, sh), Q = out_dim(W, pw, S, sw);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t g = idx[i];
        int c = (int)(g % C); g /= C;
        int s = (int)(g % S); g /= S;
        int r = (int)(g % R); g /= R;
        int k = (int)g;
        out[i] = conv_wgrad_one(x, dy, N, H, W, C, K, sh, sw, ph, pw, P, Q, k, r, s, c);
    }
}

/* ---- fully connected: y[b,o] = bias[o] + sum_i x[b,i] * Wt[o,i] ---- */
void orc_fc_fwd(const double* x, const double* Wt, const double* bias, double* y,
                int B, int in, int out, int relu) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < out; ++o) {
            double acc = bias ? bias[o] : 0.0;
            for (int i = 0; i < in; ++i) acc += x[(size_t)b * in + i] * Wt[(size_t)o * in + i];
            if (relu && !(acc > 0.0)) acc = 0.0;
            y[(size_t)b * out + o] = acc;
        }
}

/* dx[b,i] = sum_o dy[b,o] * Wt[o,i] */
void orc_fc_bwd_data(const double* dy, const double* Wt, double* dx, int B, int in, int out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < in; ++i) {
            double acc = 0.0;
            for (int o = 0; o < out; ++o) acc += dy[(size_t)b * out + o] * Wt[(size_t)o * in + i];
            dx[(size_t)b * in + i] = acc;
        }
}

/* dW[o,i] = sum_b dy[b,o] * x[b,i] */
void orc_fc_bwd_weight(const double* dy, const double* x, double* dW, int B, int in, int out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < out; ++o)
        for (int i = 0; i < in; ++i) {
            double acc = 0.0;
            for (int b = 0; b < B; ++b) acc += dy[(size_t)b * out + o] * x[(size_t)b * in + i];
            dW[(size_t)o * in + i] = acc;
        }
}

/* ---- bias gradient of a layer y = act(conv(x, w) + bias[k]) (or FC): the bias is added to every output
 *      pixel / row of channel k, so db[k] = sum over rows r of dy[r][k], dy viewed as [rows][cols] ---- */
void orc_bias_grad(const double* dy, double* db, int64_t rows, int64_t cols) {
    for (int64_t c = 0; c < cols; ++c) {
        double s = 0.0;
        for (int64_t r = 0; r < rows; ++r) s += dy[r * cols + c];
        db[c] = s;
    }
}

/* ---- ReLU backward; the derivative at zero is taken as zero: dx = dy where y > 0 ---- */
void orc_relu_bwd(const double* dy, const double* y, double* dx, int64_t n) {
    for (int64_t i = 0; i < n; ++i) dx[i] = (y[i] > 0.0) ? dy[i] : 0.0;
}

/* ---- max-pool, square window `win`, stride `st`, no padding, floor output size.
 *      Ties: the first maximum in (r, then s) scan order wins; argmax stores r*win+s. ---- */
void orc_maxpool_fwd(const double* x, double* y, uint8_t* argmax,
                     int N, int H, int W, int C, int win, int st) {
    int P = out_dim(H, 0, win, st), Q = out_dim(W, 0, win, st);
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int c = 0; c < C; ++c) {
                    double best = 0.0;
                    int bi = -1;
                    for (int r = 0; r < win; ++r)
                        for (int s = 0; s < win; ++s) {
                            double v = x[(((size_t)n * H + p * st + r) * W + q * st + s) * C + c];
                            if (bi < 0 || v > best) { best = v; bi = r * win + s; }
                        }
                    size_t o = (((size_t)n * P + p) * Q + q) * C + c;
                    y[o] = best;
                    argmax[o] = (uint8_t)bi;
                }
}

/* scatter: every dy goes to the single input its argmax names; dx starts at zero */
void orc_maxpool_bwd(const double* dy, const uint8_t* argmax, double* dx,
                     int N, int H, int W, int C, int win, int st) {
    int P = out_dim(H, 0, win, st), Q = out_dim(W, 0, win, st);
    memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int c = 0; c < C; ++c) {
                    size_t o = (((size_t)n * P + p) * Q + q) * C + c;
                    int r = argmax[o] / win, s = argmax[o] % win;
                    dx[(((size_t)n * H + p * st + r) * W + q * st + s) * C + c] += dy[o];
                }
}

/* ---- softmax cross-entropy, mean over the minibatch:
 *      p = softmax(z_b);  L = -(1/B) sum_b log p[b,label_b];  dz = (p - onehot)/B ---- */
void orc_softmax_xent(const double* z, const int32_t* labels, int B, int classes,
                      double* loss, double* dz) {
    double total = 0.0;
    for (int b = 0; b < B; ++b) {
        const double* zb = z + (size_t)b * classes;
        double m = zb[0];
        for (int j = 1; j < classes; ++j) if (zb[j] > m) m = zb[j];
        double sum = 0.0;
        for (int j = 0; j < classes; ++j) sum += exp(zb[j] - m);
        total += -(zb[labels[b]] - m - log(sum));
        for (int j = 0; j < classes; ++j) {
            double pj = exp(zb[j] - m) / sum;
            dz[(size_t)b * classes + j] = (pj - (j == labels[b] ? 1.0 : 0.0)) / (double)B;
        }
    }
    *loss = total / (double)B;
}

/* ---- plain SGD: w <- w - lr * dw ---- */
void orc_sgd(double* w, const double* dw, double lr, int64_t n) {
    for (int64_t i = 0; i < n; ++i) w[i] -= lr * dw[i];
}

/* ---- round every element to the nearest bfloat16 (ties to even), in place.
 *      Used where a chained computation must see the values a bf16 store would keep. ---- */
void orc_round_bf16(double* a, int64_t n) {
    for (int64_t i = 0; i < n; ++i) {
        double v = a[i];
        if (v == 0.0 || isnan(v) || isinf(v)) continue;
        int e;
        double m = frexp(v, &e);            /* v = m * 2^e, 0.5 <= |m| < 1 */
        if (e < -125) {                     /* below the smallest normal 2^-126: fixed quantum 2^-133 */
            double q = ldexp(1.0, -133);
            a[i] = nearbyint(v / q) * q;
            continue;
        }
        double scaled = ldexp(m, 8);        /* 8 significant bits: 128 <= |scaled| < 256 */
        double r = nearbyint(scaled);       /* default rounding mode: nearest, ties to even */
        double out = ldexp(r, e - 8);
        if (fabs(out) > 3.3895313892515355e38) out = (v > 0) ? INFINITY : -INFINITY;
        a[i] = out;
    }
}
