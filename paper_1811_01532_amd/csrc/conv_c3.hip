// First-layer convolution: 3 input channels, 3x3 filter, stride 1 (gfx950).
//
// With C = 3 the reduction is only 27 long (padded to 32 = two MFMA steps) and the layer moves ~20x more
// bytes of output (forward) or of dy (weight gradient) than of input, so both kernels are bound by that
// one stream; the generic kernels fall back to 2-byte gathers for every operand because C is not a multiple
// of 8 and run far below it.  Here only the tiny x operand is gathered element-wise (it stays in L1/L2):
//   forward : one wavefront per 32 consecutive output pixels; weights sit in registers as MFMA fragments
//             for the whole kernel; the 32 x K result is transposed through a wavefront-private LDS strip so
//             that the output leaves as contiguous 16-byte stores;
//   wgrad   : one wavefront per 16 pixels and step: dy is loaded with 16-byte vectors into a
//             wavefront-private LDS strip and transposed on the way out (ds_read_b64_tr_b16), the x columns
//             are gathered; per-work-group partial sums are added by the fixed-order reduce kernel.
// Reduction index k = (r * 3 + s) * 3 + c; an input row contributes 9 consecutive bf16 (3 pixels x 3
// channels), so k = r * 9 + j addresses element (ow - pad) * 3 + j of input row oh - pad + r.
// Serves the first "primary" convolution node of Section 3.2.2 (forward and weight-gradient halves of
// t_c, Eq. 1); its input gradient is never needed.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int NT = 256;

struct C3Args {
    const bf16_t* x;
    const bf16_t* w;    // forward: weights [K][27]
    const bf16_t* dy;   // wgrad
    const float* bias;
    bf16_t* y;          // forward output
    float* part;        // wgrad partial sums [gridDim.x][K][27]
    int N, H, W, K, OH, OW, pad_h, pad_w, M, relu;
    FastDiv dOHW, dOW;
    // general filter (conv_c3_fwd_general_kernel): R x S taps, strides, reduction length R*S*3 in 16-deep steps
    int R, S, sh, sw, Kred, ksteps;
    FastDiv dS3;  // division by S * 3 (elements of one filter row)
};

__device__ __align__(16) unsigned int g_zero_block_c3[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ unsigned short f2bf(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(unsigned short, b);
}
__device__ __forceinline__ bf16x8 pack8(const unsigned short* h) {
    u32x4 v = {(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16),
               (unsigned)h[4] | ((unsigned)h[5] << 16), (unsigned)h[6] | ((unsigned)h[7] << 16)};
    return __builtin_bit_cast(bf16x8, v);
}

// FB: 32-channel blocks of output channels (K = 32 * FB)
template <int FB>
__global__ __launch_bounds__(NT) void conv_c3_fwd_kernel(const C3Args a) {
    constexpr int K = 32 * FB;
    constexpr int OPITCH = K * 2 + 16;
    __shared__ __align__(16) unsigned char stage[4][32 * OPITCH];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const bf16_t* zero_src = reinterpret_cast<const bf16_t*>(g_zero_block_c3);

    // weight fragments (MFMA A operand): row = output channel, 8 reduction elements per lane and step
    bf16x8 wf[FB][2];
#pragma unroll
    for (int b = 0; b < FB; ++b)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            unsigned short h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = ks * 16 + half * 8 + e;
                h[e] = *(k < 27 ? a.w + (b * 32 + l32) * 27 + k : zero_src);
            }
            wf[b][ks] = pack8(h);
        }

    const int OHW = a.OH * a.OW, W3 = a.W * 3;
    const int ntiles = (a.M + 31) / 32;
    unsigned char* st = stage[wave];
    for (int tile = blockIdx.x * 4 + wave; tile < ntiles; tile += gridDim.x * 4) {
        const int m = tile * 32 + l32;
        const int mm = m < a.M ? m : a.M - 1;  // tail lanes recompute the last pixel; never stored
        const int n = (int)fdiv((uint32_t)mm, a.dOHW);
        const int rem = mm - n * OHW;
        const int oh = (int)fdiv((uint32_t)rem, a.dOW);
        const int ow = rem - oh * a.OW;
        const int ih0 = oh - a.pad_h, iw30 = (ow - a.pad_w) * 3;
        bf16x8 xf[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            unsigned short h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = ks * 16 + half * 8 + e;
                const int r = (k * 57) >> 9, j = k - r * 9;  // k / 9, k % 9 for k < 32
                const int ih = ih0 + r, iw3 = iw30 + j;
                const bool ok = k < 27 && (unsigned)ih < (unsigned)a.H && (unsigned)iw3 < (unsigned)W3;
                h[e] = *(ok ? a.x + ((size_t)(n * a.H + ih) * W3 + iw3) : zero_src);
            }
            xf[ks] = pack8(h);
        }
        f32x16 acc[FB];
#pragma unroll
        for (int b = 0; b < FB; ++b) {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[b][ks], xf[ks], acc[b], 0, 0, 0);
        }
        // accumulator register i of block b: channel b*32 + (i/4)*8 + half*4 + i%4 of pixel l32
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = b * 32 + q * 8 + half * 4;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[b][q * 4 + e];
                if (a.bias) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += a.bias[ch + e];
                }
                if (a.relu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                *reinterpret_cast<uint2*>(st + l32 * OPITCH + ch * 2) =
                    make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                               (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the strip is private to this wavefront
        constexpr int VPR = K / 8;  // 16-byte vectors per pixel
#pragma unroll
        for (int it = 0; it < 32 * VPR / 64; ++it) {
            const int v = it * 64 + lane;
            const int px = v / VPR, vec = v % VPR;
            const int mo = tile * 32 + px;
            u32x4 val = *reinterpret_cast<const u32x4*>(st + px * OPITCH + vec * 16);
            if (mo < a.M) *reinterpret_cast<u32x4*>(a.y + (size_t)mo * K + vec * 8) = val;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // strip reads done before the next tile overwrites it
    }
}

// Any filter size and stride (e.g. 11x11 stride 4): the weights do not fit in registers any more (Kred = R*S*3 up
// to a few hundred), so every work-group packs them once into MFMA fragment order in LDS,
// [reduction step][channel block][lane][8], and its wavefronts walk 32-pixel tiles persistently; the x fragment of a
// step is gathered element-wise exactly as above (k = r * (3 S) + j addresses element (ow*sw - pad)*3 + j of input
// row oh*sh - pad + r).
template <int FB>
__global__ __launch_bounds__(NT) void conv_c3_fwd_general_kernel(const C3Args a) {
    constexpr int K = 32 * FB;
    constexpr int OPITCH = K * 2 + 16;
    extern __shared__ __align__(16) unsigned char dyn[];
    unsigned char* stage_all = dyn;                      // 4 strips of 32 * OPITCH bytes
    u32x4* wfrag = reinterpret_cast<u32x4*>(dyn + 4 * 32 * OPITCH);  // [ksteps][FB][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const bf16_t* zero_src = reinterpret_cast<const bf16_t*>(g_zero_block_c3);

    for (int v = threadIdx.x; v < a.ksteps * FB * 64; v += NT) {
        const int ln = v & 63, b = (v >> 6) % FB, ks = (v >> 6) / FB;
        unsigned short h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = ks * 16 + (ln >> 5) * 8 + e;
            h[e] = *(k < a.Kred ? a.w + (size_t)(b * 32 + (ln & 31)) * a.Kred + k : zero_src);
        }
        wfrag[v] = __builtin_bit_cast(u32x4, pack8(h));
    }
    __syncthreads();

    const int OHW = a.OH * a.OW, W3 = a.W * 3, S3 = a.S * 3;
    const int ntiles = (a.M + 31) / 32;
    unsigned char* st = stage_all + wave * 32 * OPITCH;
    for (int tile = blockIdx.x * 4 + wave; tile < ntiles; tile += gridDim.x * 4) {
        const int m = tile * 32 + l32;
        const int mm = m < a.M ? m : a.M - 1;  // tail lanes recompute the last pixel; never stored
        const int n = (int)fdiv((uint32_t)mm, a.dOHW);
        const int rem = mm - n * OHW;
        const int oh = (int)fdiv((uint32_t)rem, a.dOW);
        const int ow = rem - oh * a.OW;
        const int ih0 = oh * a.sh - a.pad_h, iw30 = (ow * a.sw - a.pad_w) * 3;
        const bf16_t* ximg = a.x + (size_t)n * a.H * W3;
        f32x16 acc[FB];
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;
        for (int ks = 0; ks < a.ksteps; ++ks) {
            unsigned short h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = ks * 16 + half * 8 + e;
                const int r = (int)fdiv((uint32_t)k, a.dS3), j = k - r * S3;
                const int ih = ih0 + r, iw3 = iw30 + j;
                const bool ok = k < a.Kred && (unsigned)ih < (unsigned)a.H && (unsigned)iw3 < (unsigned)W3;
                h[e] = *(ok ? ximg + (size_t)ih * W3 + iw3 : zero_src);
            }
            const bf16x8 xf = pack8(h);
#pragma unroll
            for (int b = 0; b < FB; ++b) {
                const bf16x8 wf = __builtin_bit_cast(bf16x8, wfrag[(ks * FB + b) * 64 + lane]);
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[b], 0, 0, 0);
            }
        }
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = b * 32 + q * 8 + half * 4;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[b][q * 4 + e];
                if (a.bias) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += a.bias[ch + e];
                }
                if (a.relu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                *reinterpret_cast<uint2*>(st + l32 * OPITCH + ch * 2) =
                    make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                               (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the strip is private to this wavefront
        constexpr int VPR = K / 8;
#pragma unroll
        for (int it = 0; it < 32 * VPR / 64; ++it) {
            const int v = it * 64 + lane;
            const int px = v / VPR, vec = v % VPR;
            const int mo = tile * 32 + px;
            u32x4 val = *reinterpret_cast<const u32x4*>(st + px * OPITCH + vec * 16);
            if (mo < a.M) *reinterpret_cast<u32x4*>(a.y + (size_t)mo * K + vec * 8) = val;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // strip reads done before the next tile overwrites it
    }
}

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
__device__ __forceinline__ bf16x8 tr_pair(const unsigned char* p0, const unsigned char* p1) {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p1);
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// dw[ko][k] partial sums; requires OW % 8 == 0 (an 8-pixel run never leaves its image row)
template <int FB>
__global__ __launch_bounds__(NT) void wgrad_c3_kernel(const C3Args a) {
    constexpr int K = 32 * FB;
    constexpr int DPITCH = K * 2 + 64;  // transposing reads: 4 rows x 64 bytes in disjoint bank groups
    constexpr int VPR = K / 8;
    constexpr int DVL = (16 * VPR + 63) / 64;  // dy vectors per lane and step
    __shared__ __align__(16) unsigned char strip[4][16 * DPITCH];
    __shared__ float red[4][32][K + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const bf16_t* zero_src = reinterpret_cast<const bf16_t*>(g_zero_block_c3);
    const int OHW = a.OH * a.OW, W3 = a.W * 3;

    // this lane's x column: k = l32 -> input row offset r and element offset j
    const int k = l32;
    const int r = (k * 57) >> 9, j = k - r * 9;
    const int kl = half * 8 + ((lane & 15) >> 2);
    const int chunk = (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    unsigned char* sD = strip[wave];

    f32x16 acc[FB];
#pragma unroll
    for (int b = 0; b < FB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

    const int nsteps = (a.M + 15) / 16;
    for (int step = blockIdx.x * 4 + wave; step < nsteps; step += gridDim.x * 4) {
        const int m0 = step * 16;
        // dy: 16 pixels x K channels, 16-byte vectors, zero beyond the last pixel
        u32x4 dv[DVL];
#pragma unroll
        for (int i = 0; i < DVL; ++i) {
            const int v = i * 64 + lane;
            const int px = v / VPR, vec = v % VPR;
            const bool ok = v < 16 * VPR && m0 + px < a.M;
            dv[i] = *reinterpret_cast<const u32x4*>(ok ? a.dy + (size_t)(m0 + px) * K + vec * 8 : zero_src);
        }
        // x column fragment (MFMA A operand): row = column k, 8 consecutive pixels of one image row
        const int m8 = m0 + half * 8;
        const int mm = m8 < a.M ? m8 : 0;
        const int n = (int)fdiv((uint32_t)mm, a.dOHW);
        const int rem = mm - n * OHW;
        const int oh = (int)fdiv((uint32_t)rem, a.dOW);
        const int ow = rem - oh * a.OW;
        const int ih = oh - a.pad_h + r;
        const bool rowok = k < 27 && m8 < a.M && (unsigned)ih < (unsigned)a.H;
        const bf16_t* xrow = a.x + (size_t)(n * a.H + (rowok ? ih : 0)) * W3;
        unsigned short h[8];
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int iw3 = (ow + p - a.pad_w) * 3 + j;
            const bool ok = rowok && (unsigned)iw3 < (unsigned)W3;
            h[p] = *(ok ? xrow + iw3 : zero_src);
        }
        const bf16x8 xf = pack8(h);
#pragma unroll
        for (int i = 0; i < DVL; ++i) {
            const int v = i * 64 + lane;
            if (v < 16 * VPR) *reinterpret_cast<u32x4*>(sD + (v / VPR) * DPITCH + (v % VPR) * 16) = dv[i];
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the strip is private to this wavefront
        bf16x8 fd[FB];
#pragma unroll
        for (int b = 0; b < FB; ++b)
            fd[b] = tr_pair(sD + kl * DPITCH + chunk + b * 64, sD + (kl + 4) * DPITCH + chunk + b * 64);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the next step overwrites the strip
#pragma unroll
        for (int b = 0; b < FB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, fd[b], acc[b], 0, 0, 0);
    }

    // accumulator register i of block b: column (i/4)*8 + half*4 + i%4, output channel b*32 + l32.
    // The four wavefronts' sums are added in wavefront order.
#pragma unroll
    for (int b = 0; b < FB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) red[wave][(i >> 2) * 8 + half * 4 + (i & 3)][b * 32 + l32] = acc[b][i];
    __syncthreads();
    float* outp = a.part + (size_t)blockIdx.x * K * 27;
    for (int o = threadIdx.x; o < K * 27; o += NT) {
        const int ko = o / 27, kk = o - ko * 27;
        outp[o] = ((red[0][kk][ko] + red[1][kk][ko]) + red[2][kk][ko]) + red[3][kk][ko];
    }
}

int c3_grid(long units) {
    long blocks = (units + 3) / 4;
    const long cap = (long)kNumCU * 2;
    return (int)(blocks < cap ? (blocks < 1 ? 1 : blocks) : cap);
}

}  // namespace

namespace {
bool c3_special(const GemmGeom& g) { return g.R == 3 && g.S == 3 && g.mul_h == 1 && g.mul_w == 1; }
size_t c3_general_smem(const GemmGeom& g) {
    const size_t ksteps = (size_t)(g.Kred + 15) / 16;
    return 4 * 32 * (size_t)(g.Ncols * 2 + 16) + ksteps * (g.Ncols / 32) * 64 * 16;
}
}  // namespace

bool conv_c3_fwd_supported(const GemmGeom& g) {
    if (g.IC != 3 || g.div_h != 1 || g.div_w != 1 || (g.Ncols != 32 && g.Ncols != 64)) return false;
    return c3_special(g) || c3_general_smem(g) <= 64 * 1024;
}
const char* conv_c3_fwd_kernel_name(const GemmGeom& g) {
    if (c3_special(g)) return g.Ncols == 64 ? "conv_c3_fwd_kernel<2>" : "conv_c3_fwd_kernel<1>";
    return g.Ncols == 64 ? "conv_c3_fwd_general_kernel<2>" : "conv_c3_fwd_general_kernel<1>";
}

int launch_conv_c3_fwd(const GemmGeom& g, const bf16_t* x, const bf16_t* w, const float* bias, bool relu, bf16_t* y,
                       hipStream_t st) {
    if (!conv_c3_fwd_supported(g)) return set_error(WAP_EINVAL, "internal: 3-channel forward kernel not applicable");
    C3Args a = {};
    a.x = x;
    a.w = w;
    a.bias = bias;
    a.y = y;
    a.N = g.M / (g.OH * g.OW);
    a.H = g.IH;
    a.W = g.IW;
    a.K = g.Ncols;
    a.OH = g.OH;
    a.OW = g.OW;
    a.pad_h = g.pad_h;
    a.pad_w = g.pad_w;
    a.M = g.M;
    a.relu = relu ? 1 : 0;
    a.dOHW = make_fastdiv((uint32_t)(g.OH * g.OW));
    a.dOW = make_fastdiv((uint32_t)g.OW);
    long blocks = (((long)g.M + 31) / 32 + 3) / 4;  // 4 wavefronts per work-group, several tiles per wavefront
    if (blocks > (long)kNumCU * 8) blocks = (long)kNumCU * 8;
    const int grid = (int)blocks;
    if (!c3_special(g)) {
        a.R = g.R;
        a.S = g.S;
        a.sh = g.mul_h;
        a.sw = g.mul_w;
        a.Kred = g.Kred;
        a.ksteps = (g.Kred + 15) / 16;
        a.dS3 = make_fastdiv((uint32_t)(g.S * 3));
        const size_t smem = c3_general_smem(g);
        // every work-group packs the weights once: fewer, longer-lived groups than the 3x3 kernel
        const int ggrid = grid < kNumCU * 2 ? grid : kNumCU * 2;
        if (g.Ncols == 64) hipLaunchKernelGGL(conv_c3_fwd_general_kernel<2>, dim3(ggrid), dim3(NT), smem, st, a);
        else hipLaunchKernelGGL(conv_c3_fwd_general_kernel<1>, dim3(ggrid), dim3(NT), smem, st, a);
        return check_launch("conv_c3_fwd_general");
    }
    if (g.Ncols == 64) hipLaunchKernelGGL(conv_c3_fwd_kernel<2>, dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL(conv_c3_fwd_kernel<1>, dim3(grid), dim3(NT), 0, st, a);
    return check_launch("conv_c3_fwd");
}

// (A general-filter variant of the weight gradient was tried and dropped: with lanes indexing the columns k, the
// element-wise gather touches a different cache line per lane, and the generic kernel, which gathers with lanes
// indexing pixels and transposes through LDS, is faster for the 11x11 stride-4 layer.)
bool wgrad_c3_supported(const WgradGeom& g) {
    return g.C == 3 && g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && (g.K == 32 || g.K == 64) && (g.Q % 8) == 0 &&
           (long)g.N * g.P * g.Q >= 4096;
}
const char* wgrad_c3_kernel_name(const WgradGeom& g) { return g.K == 64 ? "wgrad_c3_kernel<2>" : "wgrad_c3_kernel<1>"; }

int wgrad_c3_nsplit(const WgradGeom& g) { return c3_grid(((long)g.N * g.P * g.Q + 15) / 16); }

int launch_wgrad_c3(const WgradGeom& g, int nsplit, const bf16_t* x, const bf16_t* dy, float* part, hipStream_t st) {
    if (!wgrad_c3_supported(g)) return set_error(WAP_EINVAL, "internal: 3-channel weight-gradient kernel not applicable");
    C3Args a = {};
    a.x = x;
    a.dy = dy;
    a.part = part;
    a.N = g.N;
    a.H = g.H;
    a.W = g.W;
    a.K = g.K;
    a.OH = g.P;
    a.OW = g.Q;
    a.pad_h = g.ph;
    a.pad_w = g.pw;
    a.M = g.N * g.P * g.Q;
    a.dOHW = make_fastdiv((uint32_t)(g.P * g.Q));
    a.dOW = make_fastdiv((uint32_t)g.Q);
    if (g.K == 64) hipLaunchKernelGGL(wgrad_c3_kernel<2>, dim3(nsplit), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL(wgrad_c3_kernel<1>, dim3(nsplit), dim3(NT), 0, st, a);
    return check_launch("wgrad_c3");
}

}  // namespace wap
