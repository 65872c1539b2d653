// Memory-bound kernels of the training step (gfx950): split-reduction epilogues, ReLU backward,
// max-pool forward / backward, softmax cross-entropy, SGD, casts.  These are the "auxiliary
// computation nodes" of Section 3.2.2 and the weight update of Section 3.2.3; all are streaming
// kernels with 16-byte accesses where the shape allows and a grid sized to cover the chip.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int kThreads = 256;

inline int grid_for(size_t work_items) {
    size_t b = (work_items + kThreads - 1) / kThreads;
    size_t cap = (size_t)kNumCU * 16;
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

__device__ __forceinline__ float bf2f(unsigned short h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ unsigned short f2bf(float f) {
    __bf16 b = (__bf16)f;  // round to nearest even
    return __builtin_bit_cast(unsigned short, b);
}

// ---- out[i] = bf16(act(bias[i % ncols] + sum_s part[s][i])) , summed in split order ----
__global__ void reduce_bf16_kernel(const float* __restrict__ part, int nsplit, size_t elems, int ncols,
                                   const float* __restrict__ bias, int relu, bf16_t* __restrict__ out) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    if ((ncols & 3) == 0) {
        size_t n4 = elems / 4;
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
            float4 s = reinterpret_cast<const float4*>(part)[i];
            for (int k = 1; k < nsplit; ++k) {
                float4 t = reinterpret_cast<const float4*>(part + (size_t)k * elems)[i];
                s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
            }
            if (bias) {
                int c = (int)((i * 4) % (size_t)ncols);
                s.x += bias[c]; s.y += bias[c + 1]; s.z += bias[c + 2]; s.w += bias[c + 3];
            }
            if (relu) {
                s.x = s.x > 0.f ? s.x : 0.f; s.y = s.y > 0.f ? s.y : 0.f;
                s.z = s.z > 0.f ? s.z : 0.f; s.w = s.w > 0.f ? s.w : 0.f;
            }
            uint2 pk;
            pk.x = (unsigned)f2bf(s.x) | ((unsigned)f2bf(s.y) << 16);
            pk.y = (unsigned)f2bf(s.z) | ((unsigned)f2bf(s.w) << 16);
            reinterpret_cast<uint2*>(out)[i] = pk;
        }
    } else {
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < elems; i += stride) {
            float s = part[i];
            for (int k = 1; k < nsplit; ++k) s += part[(size_t)k * elems + i];
            if (bias) s += bias[i % (size_t)ncols];
            if (relu) s = s > 0.f ? s : 0.f;
            out[i] = f2bf(s);
        }
    }
}

// With a parameter block (sgd.w32 != NULL) the sums update the parameters instead of being stored.
__global__ void reduce_f32_kernel(const float* __restrict__ part, int nsplit, size_t elems,
                                  float* __restrict__ out, const SgdFuse sgd) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    if ((elems & 3) == 0) {
        size_t n4 = elems / 4;
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
            float4 s = reinterpret_cast<const float4*>(part)[i];
            for (int k = 1; k < nsplit; ++k) {
                float4 t = reinterpret_cast<const float4*>(part + (size_t)k * elems)[i];
                s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
            }
            if (sgd.w32) sgd_apply4(sgd.w32 + i * 4, sgd.wb + i * 4, sgd.lr, s.x, s.y, s.z, s.w);
            else reinterpret_cast<float4*>(out)[i] = s;
        }
    } else {
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < elems; i += stride) {
            float s = part[i];
            for (int k = 1; k < nsplit; ++k) s += part[(size_t)k * elems + i];
            if (sgd.w32) {
                float a = sgd_apply(sgd.w32[i], s, sgd.lr);
                sgd.w32[i] = a;
                sgd.wb[i] = f2bf(a);
            } else {
                out[i] = s;
            }
        }
    }
}

// Many splits of a small tensor: G groups of threads each add the splits k = g, g + G, g + 2G, ... of one
// 16-byte column in increasing k (four independent loads in flight), then the G partial sums are added in
// group order through LDS.  The summation tree is fixed by (nsplit, G), so results are bitwise reproducible.
template <int G>
__global__ __launch_bounds__(256) void reduce_f32_grouped_kernel(const float* __restrict__ part, int nsplit, size_t elems,
                                                               float* __restrict__ out, const SgdFuse sgd) {
    constexpr int COLS = 256 / G;
    __shared__ float4 sm[G][COLS];
    const int col = threadIdx.x % COLS, grp = threadIdx.x / COLS;
    const size_t n4 = elems / 4;
    const size_t i = (size_t)blockIdx.x * COLS + col;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n4) {
        const float4* p = reinterpret_cast<const float4*>(part) + i;
        int k = grp;
        for (; k + 3 * G < nsplit; k += 4 * G) {
            float4 t0 = p[(size_t)k * n4], t1 = p[(size_t)(k + G) * n4], t2 = p[(size_t)(k + 2 * G) * n4],
                   t3 = p[(size_t)(k + 3 * G) * n4];
            s.x += t0.x; s.y += t0.y; s.z += t0.z; s.w += t0.w;
            s.x += t1.x; s.y += t1.y; s.z += t1.z; s.w += t1.w;
            s.x += t2.x; s.y += t2.y; s.z += t2.z; s.w += t2.w;
            s.x += t3.x; s.y += t3.y; s.z += t3.z; s.w += t3.w;
        }
        for (; k < nsplit; k += G) {
            float4 t = p[(size_t)k * n4];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
    }
    sm[grp][col] = s;
    __syncthreads();
    if (grp == 0 && i < n4) {
#pragma unroll
        for (int g2 = 1; g2 < G; ++g2) {
            float4 t = sm[g2][col];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        if (sgd.w32) sgd_apply4(sgd.w32 + i * 4, sgd.wb + i * 4, sgd.lr, s.x, s.y, s.z, s.w);
        else reinterpret_cast<float4*>(out)[i] = s;
    }
}

// ---- bias gradient, first stage: column sums of a chunk of rows (blockIdx.x) for a block of up to 256 column
// vectors (blockIdx.y).  A thread owns one 8-channel vector (or one channel) and every RP-th row of the chunk; the
// RP partial sums per column are then added in thread order. ----
template <int VEC>
__global__ __launch_bounds__(256) void bias_grad_kernel(const bf16_t* __restrict__ dy, float* __restrict__ part,
                                                        size_t rows, int cols, size_t rows_per_chunk) {
    __shared__ float red[256][VEC + 1];
    const int cv = (cols + VEC - 1) / VEC;         // vectors per row
    const int vpb = cv < 256 ? cv : 256;           // vectors handled side by side by this work-group
    const int rp = 256 / vpb;                      // rows in flight per pass
    const int vec = threadIdx.x % vpb, rsub = threadIdx.x / vpb;
    const size_t r0 = (size_t)blockIdx.x * rows_per_chunk;
    size_t r1 = r0 + rows_per_chunk;
    if (r1 > rows) r1 = rows;
    {
        const int v = blockIdx.y * vpb + vec;
        float s[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] = 0.f;
        if (rsub < rp && v < cv) {
            for (size_t r = r0 + rsub; r < r1; r += rp) {
                if (VEC == 8) {
                    const uint4 u = *reinterpret_cast<const uint4*>(dy + r * cols + (size_t)v * 8);
                    const unsigned w4[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        s[2 * k] += __uint_as_float(w4[k] << 16);
                        s[2 * k + 1] += __uint_as_float(w4[k] & 0xffff0000u);
                    }
                } else {
                    s[0] += bf2f(dy[r * cols + v]);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) red[threadIdx.x][e] = s[e];
        __syncthreads();
        if (rsub == 0 && v < cv) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                float t = red[vec][e];
                for (int k = 1; k < rp; ++k) t += red[k * vpb + vec][e];
                if (v * VEC + e < cols) part[(size_t)blockIdx.x * cols + v * VEC + e] = t;
            }
        }
        __syncthreads();
    }
}

// ---- ReLU backward ----
__global__ void relu_bwd_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ y,
                                bf16_t* dx, size_t n) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t n8 = n / 8;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
        uint4 g = reinterpret_cast<const uint4*>(dy)[i];
        uint4 v = reinterpret_cast<const uint4*>(y)[i];
        unsigned gg[4] = {g.x, g.y, g.z, g.w}, vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            unsigned lo = (bf2f((unsigned short)(vv[k] & 0xffff)) > 0.f) ? (gg[k] & 0xffffu) : 0u;
            unsigned hi = (bf2f((unsigned short)(vv[k] >> 16)) > 0.f) ? (gg[k] & 0xffff0000u) : 0u;
            gg[k] = lo | hi;
        }
        reinterpret_cast<uint4*>(dx)[i] = make_uint4(gg[0], gg[1], gg[2], gg[3]);
    }
    for (size_t i = n8 * 8 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        dx[i] = (bf2f(y[i]) > 0.f) ? dy[i] : (bf16_t)0;
}

// ---- max-pool forward: VEC channels per thread ----
template <int VEC>
__global__ void maxpool_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                                   uint8_t* __restrict__ am, int N, int H, int W, int C, int P, int Q,
                                   int win, int st) {
    const int CV = C / VEC;
    size_t total = (size_t)N * P * Q * CV;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int cv = (int)(i % CV);
        size_t t = i / CV;
        int q = (int)(t % Q); t /= Q;
        int p = (int)(t % P);
        int n = (int)(t / P);
        float best[VEC];
        unsigned short bestbits[VEC];
        uint8_t bi[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) { best[e] = 0.f; bestbits[e] = 0; bi[e] = 255; }
        for (int r = 0; r < win; ++r)
            for (int s = 0; s < win; ++s) {
                const bf16_t* src = x + (((size_t)n * H + p * st + r) * W + q * st + s) * C + (size_t)cv * VEC;
                unsigned short v[VEC];
                if (VEC == 8) {
                    uint4 u = *reinterpret_cast<const uint4*>(src);
                    v[0] = u.x & 0xffff; v[1] = u.x >> 16; v[2] = u.y & 0xffff; v[3] = u.y >> 16;
                    v[4] = u.z & 0xffff; v[5] = u.z >> 16; v[6] = u.w & 0xffff; v[7] = u.w >> 16;
                } else {
                    v[0] = src[0];
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    float f = bf2f(v[e]);
                    if (bi[e] == 255 || f > best[e]) { best[e] = f; bestbits[e] = v[e]; bi[e] = (uint8_t)(r * win + s); }
                }
            }
        size_t o = (((size_t)n * P + p) * Q + q) * C + (size_t)cv * VEC;
        if (VEC == 8) {
            *reinterpret_cast<uint4*>(y + o) = make_uint4(
                (unsigned)bestbits[0] | ((unsigned)bestbits[1] << 16), (unsigned)bestbits[2] | ((unsigned)bestbits[3] << 16),
                (unsigned)bestbits[4] | ((unsigned)bestbits[5] << 16), (unsigned)bestbits[6] | ((unsigned)bestbits[7] << 16));
            uint2 a;
            a.x = bi[0] | (bi[1] << 8) | (bi[2] << 16) | ((unsigned)bi[3] << 24);
            a.y = bi[4] | (bi[5] << 8) | (bi[6] << 16) | ((unsigned)bi[7] << 24);
            *reinterpret_cast<uint2*>(am + o) = a;
        } else {
            y[o] = bestbits[0];
            am[o] = bi[0];
        }
    }
}

// ---- max-pool backward as a gather over the windows covering each input element ----
template <int VEC>
__global__ void maxpool_bwd_kernel(const bf16_t* __restrict__ dy, const uint8_t* __restrict__ am,
                                   const bf16_t* __restrict__ ry, bf16_t* __restrict__ dx, int N, int H,
                                   int W, int C, int P, int Q, int win, int st) {
    const int CV = C / VEC;
    size_t total = (size_t)N * H * W * CV;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        int cv = (int)(i % CV);
        size_t t = i / CV;
        int w = (int)(t % W); t /= W;
        int h = (int)(t % H);
        int n = (int)(t / H);
        float sum[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum[e] = 0.f;
        int p_lo = (h - win + 1 + st - 1);
        p_lo = p_lo > 0 ? p_lo / st : 0;
        int p_hi = h / st; if (p_hi > P - 1) p_hi = P - 1;
        int q_lo = (w - win + 1 + st - 1);
        q_lo = q_lo > 0 ? q_lo / st : 0;
        int q_hi = w / st; if (q_hi > Q - 1) q_hi = Q - 1;
        for (int p = p_lo; p <= p_hi; ++p)
            for (int q = q_lo; q <= q_hi; ++q) {
                int code = (h - p * st) * win + (w - q * st);
                size_t o = (((size_t)n * P + p) * Q + q) * C + (size_t)cv * VEC;
                if (VEC == 8) {
                    uint2 a = *reinterpret_cast<const uint2*>(am + o);
                    uint4 g = *reinterpret_cast<const uint4*>(dy + o);
                    unsigned gg[4] = {g.x, g.y, g.z, g.w};
                    unsigned yy[4] = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
                    if (ry) {
                        uint4 v = *reinterpret_cast<const uint4*>(ry + o);
                        yy[0] = v.x; yy[1] = v.y; yy[2] = v.z; yy[3] = v.w;
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        unsigned ai = ((e < 4 ? a.x : a.y) >> ((e & 3) * 8)) & 0xff;
                        unsigned short gb = (unsigned short)((gg[e >> 1] >> ((e & 1) * 16)) & 0xffff);
                        unsigned short yb = (unsigned short)((yy[e >> 1] >> ((e & 1) * 16)) & 0xffff);
                        if ((int)ai == code && bf2f(yb) > 0.f) sum[e] += bf2f(gb);
                    }
                } else {
                    bool pass = ry ? (bf2f(ry[o]) > 0.f) : true;
                    if ((int)am[o] == code && pass) sum[0] += bf2f(dy[o]);
                }
            }
        size_t o = (((size_t)n * H + h) * W + w) * C + (size_t)cv * VEC;
        if (VEC == 8) {
            *reinterpret_cast<uint4*>(dx + o) = make_uint4(
                (unsigned)f2bf(sum[0]) | ((unsigned)f2bf(sum[1]) << 16), (unsigned)f2bf(sum[2]) | ((unsigned)f2bf(sum[3]) << 16),
                (unsigned)f2bf(sum[4]) | ((unsigned)f2bf(sum[5]) << 16), (unsigned)f2bf(sum[6]) | ((unsigned)f2bf(sum[7]) << 16));
        } else {
            dx[o] = f2bf(sum[0]);
        }
    }
}

// ---- softmax cross-entropy: one work-group per example ----
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(256) void softmax_xent_kernel(const bf16_t* __restrict__ z,
                                                           const int32_t* __restrict__ labels, int B,
                                                           int classes, float* __restrict__ row_loss,
                                                           bf16_t* __restrict__ dz) {
    __shared__ float red[4];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bf16_t* zb = z + (size_t)b * classes;
    float m = -3.0e38f;
    for (int j = tid; j < classes; j += 256) m = fmaxf(m, bf2f(zb[j]));
    m = wave_max(m);
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float s = 0.f;
    for (int j = tid; j < classes; j += 256) s += expf(bf2f(zb[j]) - m);
    s = wave_sum(s);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    s = (red[0] + red[1]) + (red[2] + red[3]);
    const float inv = 1.f / s, invB = 1.f / (float)B;
    // a label outside [0, classes) names no class: the row gets no one-hot term and contributes no loss (and no
    // out-of-range read)
    const int lab = labels[b];
    const bool lab_ok = (unsigned)lab < (unsigned)classes;
    for (int j = tid; j < classes; j += 256) {
        float p = expf(bf2f(zb[j]) - m) * inv;
        dz[(size_t)b * classes + j] = f2bf((p - (j == lab ? 1.f : 0.f)) * invB);
    }
    if (tid == 0) row_loss[b] = lab_ok ? -(bf2f(zb[lab]) - m - logf(s)) : 0.f;
}

// fixed-order mean of B row losses (single work-group tree)
__global__ __launch_bounds__(256) void loss_mean_kernel(const float* __restrict__ row_loss, int B,
                                                        float* __restrict__ loss) {
    __shared__ float sh[256];
    float s = 0.f;
    for (int j = threadIdx.x; j < B; j += 256) s += row_loss[j];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = sh[0] / (float)B;
}

// ---- SGD on fp32 master weights, re-deriving the bf16 compute copy ----
__global__ void sgd_kernel(size_t n, float* __restrict__ w, const float* __restrict__ dw, float lr,
                           bf16_t* __restrict__ wb) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t n4 = n / 4;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 a = reinterpret_cast<float4*>(w)[i];
        float4 g = reinterpret_cast<const float4*>(dw)[i];
        a.x = sgd_apply(a.x, g.x, lr); a.y = sgd_apply(a.y, g.y, lr);
        a.z = sgd_apply(a.z, g.z, lr); a.w = sgd_apply(a.w, g.w, lr);
        reinterpret_cast<float4*>(w)[i] = a;
        if (wb) {
            uint2 pk;
            pk.x = (unsigned)f2bf(a.x) | ((unsigned)f2bf(a.y) << 16);
            pk.y = (unsigned)f2bf(a.z) | ((unsigned)f2bf(a.w) << 16);
            reinterpret_cast<uint2*>(wb)[i] = pk;
        }
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float a = sgd_apply(w[i], dw[i], lr);
        w[i] = a;
        if (wb) wb[i] = f2bf(a);
    }
}

__global__ void cast_kernel(size_t n, const float* __restrict__ src, bf16_t* __restrict__ dst) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t n4 = n / 4;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 a = reinterpret_cast<const float4*>(src)[i];
        uint2 pk;
        pk.x = (unsigned)f2bf(a.x) | ((unsigned)f2bf(a.y) << 16);
        pk.y = (unsigned)f2bf(a.z) | ((unsigned)f2bf(a.w) << 16);
        reinterpret_cast<uint2*>(dst)[i] = pk;
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        dst[i] = f2bf(src[i]);
}

// deterministic small values in (-1, 1) for profiling buffers
__global__ void fill_kernel(bf16_t* p, size_t n, uint32_t seed) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint32_t h = (uint32_t)i * 2654435761u + seed;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        float f = ((float)(h & 0xffff) - 32768.f) * (1.f / 32768.f);
        p[i] = f2bf(f);
    }
}

}  // namespace

int launch_reduce_bf16(const float* part, int nsplit, size_t elems, int ncols, const float* bias,
                       bool relu, bf16_t* out, hipStream_t st) {
    hipLaunchKernelGGL(reduce_bf16_kernel, dim3(grid_for(elems / 4 + 1)), dim3(kThreads), 0, st, part,
                       nsplit, elems, ncols, bias, relu ? 1 : 0, out);
    return check_launch("reduce_bf16");
}

int launch_reduce_f32(const float* part, int nsplit, size_t elems, float* out, hipStream_t st, const SgdFuse* sgdp) {
    SgdFuse sgd = {nullptr, nullptr, 0.f};
    if (sgdp) sgd = *sgdp;
    if ((elems & 3) == 0 && nsplit >= 8) {
        const size_t n4 = elems / 4;
        if (nsplit >= 64) {
            hipLaunchKernelGGL(reduce_f32_grouped_kernel<32>, dim3((unsigned)((n4 + 7) / 8)), dim3(256), 0, st, part, nsplit,
                               elems, out, sgd);
        } else {
            hipLaunchKernelGGL(reduce_f32_grouped_kernel<8>, dim3((unsigned)((n4 + 31) / 32)), dim3(256), 0, st, part, nsplit,
                               elems, out, sgd);
        }
        return check_launch("reduce_f32_grouped");
    }
    hipLaunchKernelGGL(reduce_f32_kernel, dim3(grid_for(elems / 4 + 1)), dim3(kThreads), 0, st, part,
                       nsplit, elems, out, sgd);
    return check_launch("reduce_f32");
}

int launch_fill_bf16(bf16_t* p, size_t n, uint32_t seed, hipStream_t st) {
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n)), dim3(kThreads), 0, st, p, n, seed);
    return check_launch("fill");
}

// ---- fixed-order column sums of fp32 matrices [rows][cols], cols % 4 == 0 (the per-tile partial sums the convolution
// epilogues leave for the bias gradients), every matrix of a step in one launch.  First stage: a work-group adds one
// chunk of rows of one matrix, thread (row sub-index, 16-byte column vector) every RP-th row, then the RP partial sums
// in order.  Second stage: a thread adds the chunks of one column vector in order. ----
__global__ __launch_bounds__(256) void colsum_f32_multi_kernel(const ColsumJobs js, unsigned char* __restrict__ base) {
    __shared__ float4 red[256];
    int j = 0;
    while (j + 1 < js.n && (int)blockIdx.x >= js.first[j + 1]) ++j;
    const ColsumJob& jb = js.job[j];
    const int local = (int)blockIdx.x - js.first[j];
    const int cv = jb.cols / 4;
    const int vpb = cv < 256 ? cv : 256;
    const int colblocks = (cv + vpb - 1) / vpb;
    const int chunk = local / colblocks, cb = local - chunk * colblocks;
    const int rp = 256 / vpb;
    const int vec = threadIdx.x % vpb, rsub = threadIdx.x / vpb;
    const int v = cb * vpb + vec;
    const float* part = reinterpret_cast<const float*>(base + jb.part_off);
    float* part2 = reinterpret_cast<float*>(base + jb.part2_off);
    const int rpc = (jb.rows + jb.chunks - 1) / jb.chunks;
    const int r0 = chunk * rpc;
    const int r1 = r0 + rpc < jb.rows ? r0 + rpc : jb.rows;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (rsub < rp && v < cv)
        for (int r = r0 + rsub; r < r1; r += rp) {
            const float4 t = *reinterpret_cast<const float4*>(part + (size_t)r * jb.cols + (size_t)v * 4);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
    red[threadIdx.x] = s;
    __syncthreads();
    if (rsub == 0 && v < cv) {
        for (int k = 1; k < rp; ++k) {
            const float4 t = red[k * vpb + vec];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        *reinterpret_cast<float4*>(part2 + (size_t)chunk * jb.cols + (size_t)v * 4) = s;
    }
}

__global__ __launch_bounds__(256) void colsum_f32_finish_kernel(const ColsumJobs js, unsigned char* __restrict__ base) {
    const int t = blockIdx.x * 256 + threadIdx.x;  // column vector in the concatenation of all matrices
    int j = 0, v0 = 0;
    while (j < js.n && t >= v0 + js.job[j].cols / 4) { v0 += js.job[j].cols / 4; ++j; }
    if (j >= js.n) return;
    const ColsumJob& jb = js.job[j];
    const int v = t - v0;
    const float* part2 = reinterpret_cast<const float*>(base + jb.part2_off);
    float4 s = *reinterpret_cast<const float4*>(part2 + (size_t)v * 4);
    for (int k = 1; k < jb.chunks; ++k) {
        const float4 u = *reinterpret_cast<const float4*>(part2 + (size_t)k * jb.cols + (size_t)v * 4);
        s.x += u.x; s.y += u.y; s.z += u.z; s.w += u.w;
    }
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(base + jb.out_off) + (size_t)v * 4) = s;
}

int colsum_f32_chunks(size_t rows) {
    size_t chunks = (rows + 63) / 64;
    if (chunks > 64) chunks = 64;
    return (int)(chunks < 1 ? 1 : chunks);
}

int colsum_jobs_add(ColsumJobs& js, int rows, int cols, size_t part_off, size_t part2_off, size_t out_off) {
    if (js.n >= kMaxColsumJobs || (cols & 3) != 0 || rows < 1) return -1;
    ColsumJob& jb = js.job[js.n];
    jb.rows = rows; jb.cols = cols; jb.chunks = colsum_f32_chunks((size_t)rows);
    jb.part_off = part_off; jb.part2_off = part2_off; jb.out_off = out_off;
    const int cv = cols / 4, vpb = cv < 256 ? cv : 256;
    if (js.n == 0) js.first[0] = 0;
    js.first[js.n + 1] = js.first[js.n] + jb.chunks * ((cv + vpb - 1) / vpb);
    return js.n++;
}

int launch_colsum_f32_multi(const ColsumJobs& js, void* base, hipStream_t st) {
    if (js.n < 1) return WAP_OK;
    hipLaunchKernelGGL(colsum_f32_multi_kernel, dim3(js.first[js.n]), dim3(256), 0, st, js, (unsigned char*)base);
    int rc = check_launch("colsum_f32_multi");
    if (rc != WAP_OK) return rc;
    int vecs = 0;
    for (int j = 0; j < js.n; ++j) vecs += js.job[j].cols / 4;
    hipLaunchKernelGGL(colsum_f32_finish_kernel, dim3((vecs + 255) / 256), dim3(256), 0, st, js, (unsigned char*)base);
    return check_launch("colsum_f32_finish");
}

// Row chunks of the first stage: about 32 loads per thread (a work-group covers min(vectors per row, 256) vectors side
// by side and 256 / that many rows per pass), at most ~8 work-groups per CU over all column blocks.
int bias_grad_chunks(size_t rows, int cols) {
    const int vecw = (cols & 7) == 0 ? 8 : 1;
    const int cv = (cols + vecw - 1) / vecw;
    const int vpb = cv < 256 ? cv : 256;
    const int rp = 256 / vpb;
    const int colblocks = (cv + vpb - 1) / vpb;
    if (rows <= 512) return 1;  // a minibatch of rows (FC layers): one chunk, its sums are the result (no second launch)
    size_t chunks = (rows + (size_t)32 * rp - 1) / ((size_t)32 * rp);
    size_t cap = (size_t)kNumCU * 8 / colblocks;
    if (cap < 1) cap = 1;
    if (chunks > cap) chunks = cap;
    return (int)(chunks < 1 ? 1 : chunks);
}

int launch_bias_grad(size_t rows, int cols, const bf16_t* dy, float* db, float* part, hipStream_t st) {
    const int chunks = bias_grad_chunks(rows, cols);
    const size_t rpc = (rows + chunks - 1) / chunks;
    const int vecw = (cols & 7) == 0 ? 8 : 1;
    const int cv = (cols + vecw - 1) / vecw;
    const int colblocks = (cv + 255) / 256;  // the kernel covers min(cv, 256) vectors per work-group
    float* dst = chunks == 1 ? db : part;  // a single chunk writes the result itself
    if (vecw == 8)
        hipLaunchKernelGGL(bias_grad_kernel<8>, dim3(chunks, colblocks), dim3(256), 0, st, dy, dst, rows, cols, rpc);
    else
        hipLaunchKernelGGL(bias_grad_kernel<1>, dim3(chunks, colblocks), dim3(256), 0, st, dy, dst, rows, cols, rpc);
    int rc = check_launch("bias_grad");
    if (rc != WAP_OK || chunks == 1) return rc;
    return launch_reduce_f32(part, chunks, (size_t)cols, db, st);
}

int launch_relu_bwd(const bf16_t* dy, const bf16_t* y, bf16_t* dx, size_t n, hipStream_t st) {
    hipLaunchKernelGGL(relu_bwd_kernel, dim3(grid_for(n / 8 + 1)), dim3(kThreads), 0, st, dy, y, dx, n);
    return check_launch("relu_bwd");
}

int launch_maxpool_fwd(int N, int H, int W, int C, int win, int stp, const bf16_t* x, bf16_t* y,
                       uint8_t* am, hipStream_t st) {
    int P = (H - win) / stp + 1, Q = (W - win) / stp + 1;
    if ((C & 7) == 0) {
        size_t total = (size_t)N * P * Q * (C / 8);
        hipLaunchKernelGGL(maxpool_fwd_kernel<8>, dim3(grid_for(total)), dim3(kThreads), 0, st, x, y, am, N,
                           H, W, C, P, Q, win, stp);
    } else {
        size_t total = (size_t)N * P * Q * C;
        hipLaunchKernelGGL(maxpool_fwd_kernel<1>, dim3(grid_for(total)), dim3(kThreads), 0, st, x, y, am, N,
                           H, W, C, P, Q, win, stp);
    }
    return check_launch("maxpool_fwd");
}

int launch_maxpool_bwd(int N, int H, int W, int C, int win, int stp, const bf16_t* dy, const uint8_t* am,
                       const bf16_t* ry, bf16_t* dx, hipStream_t st) {
    int P = (H - win) / stp + 1, Q = (W - win) / stp + 1;
    if ((C & 7) == 0) {
        size_t total = (size_t)N * H * W * (C / 8);
        hipLaunchKernelGGL(maxpool_bwd_kernel<8>, dim3(grid_for(total)), dim3(kThreads), 0, st, dy, am, ry,
                           dx, N, H, W, C, P, Q, win, stp);
    } else {
        size_t total = (size_t)N * H * W * C;
        hipLaunchKernelGGL(maxpool_bwd_kernel<1>, dim3(grid_for(total)), dim3(kThreads), 0, st, dy, am, ry,
                           dx, N, H, W, C, P, Q, win, stp);
    }
    return check_launch("maxpool_bwd");
}

int launch_softmax_xent(int B, int classes, const bf16_t* z, const int32_t* labels, float* loss,
                        float* row_loss, bf16_t* dz, hipStream_t st) {
    hipLaunchKernelGGL(softmax_xent_kernel, dim3(B), dim3(256), 0, st, z, labels, B, classes, row_loss, dz);
    int rc = check_launch("softmax_xent");
    if (rc != WAP_OK) return rc;
    hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(256), 0, st, row_loss, B, loss);
    return check_launch("loss_mean");
}

int launch_sgd(size_t n, float* w, const float* dw, float lr, bf16_t* wb, hipStream_t st) {
    hipLaunchKernelGGL(sgd_kernel, dim3(grid_for(n / 4 + 1)), dim3(kThreads), 0, st, n, w, dw, lr, wb);
    return check_launch("sgd");
}

int launch_cast(size_t n, const float* src, bf16_t* dst, hipStream_t st) {
    hipLaunchKernelGGL(cast_kernel, dim3(grid_for(n / 4 + 1)), dim3(kThreads), 0, st, n, src, dst);
    return check_launch("cast");
}

}  // namespace wap
