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
// Larger filters: conv_c3_fwd_general_kernel gathers the same way for any R x S and stride; for a horizontal
// stride that is a multiple of 4 (the 11x11 stride-4 layer) conv_c3_fwd_strided_kernel and wgrad_c3_strided_kernel
// keep the R input rows of one output row in LDS, where the im2col rows of neighbouring pixels are overlapping
// contiguous runs that start 6*stride bytes apart, so no element-wise gather is left.
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
    // rows-in-LDS 3x3 forward (conv_c3_fwd_rows_kernel): 32-pixel tiles per output row, tiles in all
    int tiles_row, ntiles;
    unsigned x_bytes;
    FastDiv dTR, dOH;
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
__global__ __launch_bounds__(NT, 4) void conv_c3_fwd_kernel(const C3Args a) {
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

// The same product on maps whose output rows are whole 32-pixel tiles and whose input rows hold an even number of
// pixels (VGG's 224 x 224): instead of gathering its 16 x-elements one by one (an address computation and a bounds
// check each, ~200 vector instructions per tile, which kept this kernel a third below the rate its output stream
// allows), a wavefront stages the three input rows of its tile -- 36 pixels x 3 channels each, ONE 4-byte load per
// lane and row, starting at an even pixel so that every load is aligned and lies wholly inside or outside the image --
// in a wavefront-private LDS strip, and builds the fragments from there with sixteen 2-byte reads whose addresses
// are computed once per kernel.
template <int FB>
__global__ __launch_bounds__(NT, 4) void conv_c3_fwd_rows_kernel(const C3Args a) {
    constexpr int K = 32 * FB;
    constexpr int OPITCH = K * 2 + 16;
    constexpr int XROW = 256;  // bytes per staged input row: one dword per lane (216 bytes used)
    constexpr unsigned OOB = 0x80000000u;  // x is below 2 GiB (checked on the host)
    __shared__ __align__(16) unsigned char stage[4][32 * OPITCH];
    __shared__ __align__(16) unsigned char xin[4][3 * XROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const bf16_t* zero_src = reinterpret_cast<const bf16_t*>(g_zero_block_c3);
    const __amdgpu_buffer_rsrc_t rsrcX =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.x), 0, (int)a.x_bytes, 0x00020000);

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

    // the staged rows start at pixel ow0 - pad_w - adj, which is even (ow0 is a multiple of 32): element k = r * 9 + j of
    // this lane's pixel l32 sits at byte r * XROW + ((l32 + adj) * 3 + j) * 2 of the strip; k >= 27 (the zero padding of
    // the reduction) reads the tail of a staged row, which lanes 54 .. 63 fill with the zeros of their masked loads
    const int adj = a.pad_w & 1;
    unsigned char* xs = xin[wave];
    const unsigned char* xrd[2][8];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = ks * 16 + half * 8 + e;
            const int r = (k * 57) >> 9, j = k - r * 9;  // k / 9, k % 9 for k < 32
            xrd[ks][e] = k < 27 ? xs + r * XROW + ((l32 + adj) * 3 + j) * 2 : xs + 216;  // bytes 216 .. 255 of a row: always zero
        }
    // the two bf16 elements of this lane's dword belong to the staged pixels (2 lane) / 3 and (2 lane + 1) / 3
    const int dp0 = (2 * lane) / 3, dp1 = (2 * lane + 1) / 3;

    unsigned char* st = stage[wave];
    for (int tile = blockIdx.x * 4 + wave; tile < a.ntiles; tile += gridDim.x * 4) {
        const int rowi = (int)fdiv((uint32_t)tile, a.dTR);        // (image, output row)
        const int ow0 = (tile - rowi * a.tiles_row) * 32;
        const int n = (int)fdiv((uint32_t)rowi, a.dOH);
        const int oh = rowi - n * a.OH;
        const int iws = ow0 - a.pad_w - adj;
        const bool colok = lane < 54 && (unsigned)(iws + dp0) < (unsigned)a.W && (unsigned)(iws + dp1) < (unsigned)a.W;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int ih = oh - a.pad_h + r;
            const bool ok = colok && (unsigned)ih < (unsigned)a.H;
            const unsigned off = (unsigned)((((n * a.H + ih) * a.W + iws) * 3 + 2 * lane) * 2);
            const unsigned v = __builtin_amdgcn_raw_buffer_load_b32(rsrcX, ok ? off : OOB, 0, 0);
            *reinterpret_cast<unsigned*>(xs + r * XROW + lane * 4) = v;
        }
        // the strip is written as dwords and read as halfwords: keep the compiler from moving the reads in front of the
        // writes (the LDS pipe itself executes a wavefront's operations in order, so no wait is needed)
        asm volatile("" ::: "memory");
        bf16x8 xf[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            unsigned short h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                h[e] = *reinterpret_cast<const unsigned short*>(xrd[ks][e]);
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
        // accumulator register i of block b: channel b*32 + (i/4)*8 + half*4 + i%4 of pixel l32; bias and ReLU are
        // decided once per tile (four straight-line variants)
        auto stage_tile = [&](auto bias_tag, auto relu_tag) {
            constexpr bool BIAS = decltype(bias_tag)::value, RELU = decltype(relu_tag)::value;
#pragma unroll
            for (int b = 0; b < FB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int ch = b * 32 + q * 8 + half * 4;
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[b][q * 4 + e];
                    if (BIAS) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += a.bias[ch + e];
                    }
                    if (RELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                    }
                    *reinterpret_cast<uint2*>(st + l32 * OPITCH + ch * 2) =
                        make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                                   (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
                }
        };
        if (a.bias) {
            if (a.relu) stage_tile(std::true_type{}, std::true_type{});
            else stage_tile(std::true_type{}, std::false_type{});
        } else {
            if (a.relu) stage_tile(std::false_type{}, std::true_type{});
            else stage_tile(std::false_type{}, std::false_type{});
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the strips are private to this wavefront
        constexpr int VPR = K / 8;  // 16-byte vectors per pixel
        const size_t m0 = ((size_t)rowi * a.OW + ow0);
#pragma unroll
        for (int it = 0; it < 32 * VPR / 64; ++it) {
            const int v = it * 64 + lane;
            const int px = v / VPR, vec = v % VPR;
            u32x4 val = *reinterpret_cast<const u32x4*>(st + px * OPITCH + vec * 16);
            *reinterpret_cast<u32x4*>(a.y + (m0 + px) * K + vec * 8) = val;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // strip reads done before the next tile overwrites them
    }
}

// Any filter size and stride (e.g. 11x11 stride 4): the weights do not fit in registers any more (Kred = R*S*3 up
// to a few hundred), so every work-group packs them once into MFMA fragment order in LDS,
// [reduction step][channel block][lane][8], and its wavefronts walk 32-pixel tiles persistently; the x fragment of a
// step is gathered element-wise exactly as above (k = r * (3 S) + j addresses element (ow*sw - pad)*3 + j of input
// row oh*sh - pad + r).
template <int FB>
__global__ __launch_bounds__(NT, 2) void conv_c3_fwd_general_kernel(const C3Args a) {
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
__global__ __launch_bounds__(NT, 3) void wgrad_c3_kernel(const C3Args a) {
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

// ---- weight gradient for a LARGE filter at a horizontal stride that is a multiple of 4 (the 11x11 stride-4
// first layer of the AlexNet-style network): dw[ko][(r,s,c)] = sum over pixels of dy[pix][ko] * x[pix @ (r,s)][c].
// For one output row the im2col row of pixel ow and filter row r is a CONTIGUOUS run of S*3 elements of input row
// oh*sh - ph + r starting at element (ow*sw - pw)*3: the runs of neighbouring pixels overlap, start 6*sw bytes
// apart, and need no gather at all once the R input rows sit in LDS: a transposing read whose lanes supply
// "row base + 6*sw*pixel + 2*column" delivers the MFMA operand directly (6*sw is a multiple of 8 bytes, which the
// 8-byte transposing read needs, exactly when sw is a multiple of 4).  Columns are numbered r * SC4 + (s*3 + c)
// with SC4 = S*3 rounded up to a multiple of 4 (a 4-column chunk never straddles two filter rows); the surplus
// columns multiply real neighbouring input elements and are dropped in the epilogue.
// A work-group takes whole output rows (n, oh): R input rows and the dy row go to LDS, then ceil(OW/16) reduction
// steps; wavefront w owns the 32-column blocks w, w+4, ... (at most 4) for all K output channels.  One fp32
// partial per work-group, summed afterwards in a fixed order.
struct C3SArgs {
    const bf16_t* x;
    const bf16_t* dy;
    float* part;
    int N, H, W, OH, OW, R, S, sh, sw, ph, pw;
    int SC4, NB, Kred, xrowb, units, nsteps, nvx;  // columns per filter row (padded), 32-column blocks, LDS bytes per x row,
                                                   // output rows in all, 16-pixel steps per row, 16-byte vectors per x row
    FastDiv dOH, dSC4, dNVX;
};

template <int FB>
__global__ __launch_bounds__(NT, 2) void wgrad_c3_strided_kernel(const C3SArgs a) {
    constexpr int K = 32 * FB;
    constexpr int DPITCH = K * 2 + 64;
    constexpr int VPR = K / 8;
    extern __shared__ __align__(16) unsigned char smem_s[];
    unsigned char* sX = smem_s;                 // [R][xrowb]: element e of an input row at byte 6*pw + 2*e
    unsigned char* sD = smem_s + a.R * a.xrowb;  // [16 * nsteps][DPITCH]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int total16 = (a.R * a.xrowb + 16 * a.nsteps * DPITCH) / 16;
    // the halo left of the row, the run-over right of it and the dy rows past OW are read but never written: zero once
    for (int i = tid; i < total16; i += NT) *reinterpret_cast<u32x4*>(smem_s + i * 16) = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    const int kl = half * 8 + ((lane & 15) >> 2);
    const int ccol = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;  // first of this lane's 4 columns inside a 32-column block
    int xo[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int f = 32 * (wave + 4 * j) + ccol;
        int r = (int)fdiv((uint32_t)f, a.dSC4);
        const int sc = f - r * a.SC4;
        if (r >= a.R) r = a.R - 1;  // columns past the filter: any readable address, the products are dropped
        xo[j] = r * a.xrowb + 2 * sc + 6 * a.sw * kl;
    }
    f32x16 acc[4][FB];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][b][e] = 0.f;

    // Row u+1 is fetched into registers while row u is multiplied out of LDS (one buffer, two barriers per row).
    const int W3 = a.W * 3;
    constexpr int XV = 4, DVL = 2;  // 16-byte vectors per thread: x rows (R * nvx <= 1024), dy row (OW * K / 8 <= 512)
    u32x4 rx[XV], rdv[DVL];
    auto load_row = [&](int u) {
        const int n = (int)fdiv((uint32_t)u, a.dOH), oh = u - n * a.OH;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int v = tid + i * NT;
            const int r = (int)fdiv((uint32_t)v, a.dNVX), j = v - r * a.nvx;
            const int ih = oh * a.sh - a.ph + r;
            const bool ok = v < a.R * a.nvx && (unsigned)ih < (unsigned)a.H;
            rx[i] = *reinterpret_cast<const u32x4*>(
                ok ? a.x + ((size_t)(n * a.H + ih) * W3 + 8 * j) : reinterpret_cast<const bf16_t*>(g_zero_block_c3));
        }
        const bf16_t* dyrow = a.dy + (size_t)u * a.OW * K;
#pragma unroll
        for (int i = 0; i < DVL; ++i) {
            const int v = tid + i * NT;
            rdv[i] = *reinterpret_cast<const u32x4*>(v < a.OW * VPR ? dyrow + (size_t)v * 8
                                                                   : reinterpret_cast<const bf16_t*>(g_zero_block_c3));
        }
    };
    auto store_row = [&]() {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int v = tid + i * NT;
            if (v < a.R * a.nvx) {
                const int r = (int)fdiv((uint32_t)v, a.dNVX), j = v - r * a.nvx;
                unsigned* dst = reinterpret_cast<unsigned*>(sX + r * a.xrowb + 6 * a.pw + 16 * j);  // 4-byte aligned (pw even)
                dst[0] = rx[i][0]; dst[1] = rx[i][1]; dst[2] = rx[i][2]; dst[3] = rx[i][3];
            }
        }
#pragma unroll
        for (int i = 0; i < DVL; ++i) {
            const int v = tid + i * NT;
            if (v < a.OW * VPR) *reinterpret_cast<u32x4*>(sD + (v / VPR) * DPITCH + (v % VPR) * 16) = rdv[i];
        }
    };
    if ((int)blockIdx.x < a.units) load_row(blockIdx.x);
    for (int u = blockIdx.x; u < a.units; u += gridDim.x) {
        store_row();
        __syncthreads();
        if (u + (int)gridDim.x < a.units) load_row(u + gridDim.x);
        for (int step = 0; step < a.nsteps; ++step) {
            const unsigned char* d0 = sD + (step * 16 + kl) * DPITCH + ccol * 2;
            bf16x8 fd[FB];
#pragma unroll
            for (int b = 0; b < FB; ++b) fd[b] = tr_pair(d0 + b * 64, d0 + 4 * DPITCH + b * 64);
            const int xs = 6 * a.sw * 16 * step;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (wave + 4 * j < a.NB) {  // uniform per wavefront
                    const unsigned char* x0 = sX + xo[j] + xs;
                    const bf16x8 fx = tr_pair(x0, x0 + 6 * a.sw * 4);
#pragma unroll
                    for (int b = 0; b < FB; ++b) acc[j][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx, fd[b], acc[j][b], 0, 0, 0);
                }
            }
        }
        __syncthreads();  // every wavefront is done with this row before the next one overwrites it
    }

    // Epilogue.  Accumulator register i holds column (i/4)*8 + half*4 + i%4 of the block for output channel
    // b*32 + l32; a wavefront-private LDS strip turns that around so that 32 consecutive lanes store 32 consecutive
    // columns of one output channel (the LDS rows of the main loop are dead after the last barrier).
    float* outp = a.part + (size_t)blockIdx.x * K * a.Kred;
    float* red = reinterpret_cast<float*>(smem_s) + wave * (K * 33);
    const int S3 = a.S * 3;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (wave + 4 * j >= a.NB) continue;
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) red[(b * 32 + l32) * 33 + (i >> 2) * 8 + half * 4 + (i & 3)] = acc[j][b][i];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the strip is private to this wavefront
        const int f = 32 * (wave + 4 * j) + l32;
        const int r = (int)fdiv((uint32_t)f, a.dSC4), sc = f - r * a.SC4;
        const bool keep = r < a.R && sc < S3;
        for (int k = half; k < K; k += 2) {
            const float v = red[k * 33 + l32];
            if (keep) outp[(size_t)k * a.Kred + r * S3 + sc] = v;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // strip reads done before the next block overwrites it
    }
}

// ---- forward for the same layers (large filter, horizontal stride a multiple of 4): the R input rows of one
// output row sit in LDS exactly as above, and the MFMA operand of pixel ow for 8 consecutive reduction columns of
// filter row r is 16 contiguous, 8-byte aligned bytes at "row base + 6*sw*ow + 2*column": two 8-byte LDS reads
// instead of eight element-wise global loads.  Columns are numbered r * SC8 + (s*3 + c), SC8 = S*3 rounded up to
// a multiple of 8; the surplus columns meet zero weights (inputs are assumed finite).  Wavefront (pt, b) owns
// pixels pt*32.. of the row and the 32-channel block b, with that block's weights in registers as MFMA fragments
// for the whole kernel; the output row leaves through an LDS tile as contiguous 16-byte stores.
struct C3FArgs {
    const bf16_t* x;
    const bf16_t* w;
    const float* bias;
    bf16_t* y;
    int N, H, W, OH, OW, R, S, sh, sw, ph, pw;
    int G8, ksteps, Kred, xrowb, units, nvx, relu;  // 8-column groups per filter row, 16-deep reduction steps
    FastDiv dOH, dNVX, dG8, dKred, dS3;
};
constexpr int C3F_KS = 28;  // most reduction steps (weight fragments held in registers)

template <int FB>
__global__ __launch_bounds__(NT, 2) void conv_c3_fwd_strided_kernel(const C3FArgs a) {
    constexpr int K = 32 * FB;
    constexpr int OPITCH = K * 2 + 16;
    constexpr int VPR = K / 8;
    extern __shared__ __align__(16) unsigned char smem_f[];
    unsigned char* sX = smem_f;                 // [R][xrowb]: element e of an input row at byte 6*pw + 2*e
    unsigned char* sO = smem_f + a.R * a.xrowb;  // [64][OPITCH] output tile
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int pt = wave / FB, b = wave % FB;
    const bool active = pt * 32 < a.OW;
    const int S3 = a.S * 3;
    // Weight fragments: reduction step ks, half h -> column group ks*2 + h -> filter row r, columns sc .. sc + 7.
    // The work-group first lays all weights out in fragment order in LDS (coalesced reads of w, surplus columns
    // zero), then every wavefront takes its block's fragments into registers; the area is reused for the rows.
    {
        const int nfrag16 = FB * a.ksteps * 64;  // 16-byte fragments
        for (int i = tid; i < nfrag16; i += NT) *reinterpret_cast<u32x4*>(smem_f + i * 16) = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();
        unsigned short* wl = reinterpret_cast<unsigned short*>(smem_f);
        for (int idx = tid; idx < K * a.Kred; idx += NT) {
            const int ch = (int)fdiv((uint32_t)idx, a.dKred), k = idx - ch * a.Kred;
            const int r = (int)fdiv((uint32_t)k, a.dS3), sc = k - r * S3;
            const int gi = r * a.G8 + (sc >> 3);
            wl[((((ch >> 5) * a.ksteps + (gi >> 1)) * 64) + (gi & 1) * 32 + (ch & 31)) * 8 + (sc & 7)] = a.w[idx];
        }
        __syncthreads();
    }
    bf16x8 wf[C3F_KS];
#pragma unroll
    for (int ks = 0; ks < C3F_KS; ++ks) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (ks < a.ksteps) v = *reinterpret_cast<const u32x4*>(smem_f + ((b * a.ksteps + ks) * 64 + lane) * 16);
        wf[ks] = __builtin_bit_cast(bf16x8, v);
    }
    __syncthreads();  // every wavefront holds its fragments: the area becomes the row buffer
    for (int i = tid; i < a.R * a.xrowb / 16; i += NT) *reinterpret_cast<u32x4*>(sX + i * 16) = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
    const int pixoff = 6 * a.sw * (pt * 32 + l32);

    const int W3 = a.W * 3;
    constexpr int XV = 4;  // 16-byte x vectors per thread (R * nvx <= 1024)
    u32x4 rx[XV];
    auto load_row = [&](int u) {
        const int n = (int)fdiv((uint32_t)u, a.dOH), oh = u - n * a.OH;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int v = tid + i * NT;
            const int r = (int)fdiv((uint32_t)v, a.dNVX), j = v - r * a.nvx;
            const int ih = oh * a.sh - a.ph + r;
            const bool ok = v < a.R * a.nvx && (unsigned)ih < (unsigned)a.H;
            rx[i] = *reinterpret_cast<const u32x4*>(
                ok ? a.x + ((size_t)(n * a.H + ih) * W3 + 8 * j) : reinterpret_cast<const bf16_t*>(g_zero_block_c3));
        }
    };
    if ((int)blockIdx.x < a.units) load_row(blockIdx.x);
    for (int u = blockIdx.x; u < a.units; u += gridDim.x) {
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            const int v = tid + i * NT;
            if (v < a.R * a.nvx) {
                const int r = (int)fdiv((uint32_t)v, a.dNVX), j = v - r * a.nvx;
                unsigned* dst = reinterpret_cast<unsigned*>(sX + r * a.xrowb + 6 * a.pw + 16 * j);  // 4-byte aligned (pw even)
                dst[0] = rx[i][0]; dst[1] = rx[i][1]; dst[2] = rx[i][2]; dst[3] = rx[i][3];
            }
        }
        __syncthreads();  // the row is complete; the previous row's output tile has been stored
        if (u + (int)gridDim.x < a.units) load_row(u + gridDim.x);
        if (active) {
            f32x16 acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
            int r = 0, g8 = half;  // column group of this half-wavefront, kept incrementally (G8 >= 2)
#pragma unroll
            for (int ks = 0; ks < C3F_KS; ++ks) {
                if (ks < a.ksteps) {  // uniform
                    const int rr = r < a.R ? r : a.R - 1;  // past the filter: any readable row, the weights are zero
                    const unsigned char* xa = sX + rr * a.xrowb + g8 * 16 + pixoff;
                    const uint2 lo = *reinterpret_cast<const uint2*>(xa);
                    const uint2 hi = *reinterpret_cast<const uint2*>(xa + 8);
                    const u32x4 xv = {lo.x, lo.y, hi.x, hi.y};
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks], __builtin_bit_cast(bf16x8, xv), acc, 0, 0, 0);
                    g8 += 2;
                    if (g8 >= a.G8) { g8 -= a.G8; ++r; }
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ch = b * 32 + q * 8 + half * 4;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[q * 4 + e];
                if (a.bias) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += a.bias[ch + e];
                }
                if (a.relu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                *reinterpret_cast<uint2*>(sO + (pt * 32 + l32) * OPITCH + ch * 2) =
                    make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                               (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
            }
        }
        __syncthreads();  // output tile complete, input rows consumed
        bf16_t* yrow = a.y + (size_t)u * a.OW * K;
        for (int v = tid; v < a.OW * VPR; v += NT)
            *reinterpret_cast<u32x4*>(yrow + (size_t)v * 8) =
                *reinterpret_cast<const u32x4*>(sO + (v / VPR) * OPITCH + (v % VPR) * 16);
    }
}

struct C3FPlan {
    int G8, ksteps, xrowb;
    size_t smem;
};
bool c3f_plan(const GemmGeom& g, C3FPlan* out) {
    if (g.IC != 3 || (g.Ncols != 32 && g.Ncols != 64) || g.div_h != 1 || g.div_w != 1) return false;
    if ((g.mul_w % 4) != 0 || (g.pad_w % 2) != 0 || (g.IW % 8) != 0 || g.OW > 64) return false;
    C3FPlan p;
    const int SC8 = (g.S * 3 + 7) / 8 * 8;
    p.G8 = SC8 / 8;
    if (p.G8 < 2) return false;
    p.ksteps = (g.R * p.G8 + 1) / 2;
    if (p.ksteps > C3F_KS) return false;
    if (g.R * (g.IW * 3 / 8) > 4 * NT) return false;  // the kernel stages at most 4 x vectors per thread
    const int data = 6 * g.pad_w + 2 * g.IW * 3;
    const int reach = 6 * g.mul_w * 63 + 2 * SC8;  // pixel 63, last column group of a filter row
    p.xrowb = ((data > reach ? data : reach) + 15) / 16 * 16;
    p.smem = (size_t)g.R * p.xrowb + (size_t)64 * (g.Ncols * 2 + 16);
    const size_t frag = (size_t)(g.Ncols / 32) * p.ksteps * 64 * 16;  // the weight fragments pass through the same area
    if (frag > p.smem) p.smem = frag;
    if (p.smem > 64 * 1024) return false;
    *out = p;
    return true;
}
bool c3_fwd_strided(const GemmGeom& g) {
    C3FPlan p;
    return !(g.R == 3 && g.S == 3 && g.mul_h == 1 && g.mul_w == 1) && c3f_plan(g, &p) && g.M / g.OW >= 64;
}

struct C3SPlan {
    int SC4, NB, xrowb, nsteps;
    size_t smem;
};
bool c3s_plan(const WgradGeom& g, C3SPlan* out) {
    if (g.C != 3 || (g.K != 32 && g.K != 64)) return false;
    if ((g.sw % 4) != 0 || (g.pw % 2) != 0 || (g.W % 8) != 0 || g.Q > 64) return false;
    C3SPlan p;
    p.SC4 = (g.S * 3 + 3) / 4 * 4;
    p.NB = (g.R * p.SC4 + 31) / 32;
    if (p.NB > 16) return false;
    p.nsteps = (g.Q + 15) / 16;
    // bytes of one x row in LDS: the row itself behind its left halo, and the farthest transposing read (pixel
    // 16*nsteps - 1, last chunk of a filter row)
    const int data = 6 * g.pw + 2 * g.W * 3;
    const int reach = 6 * g.sw * (16 * p.nsteps - 1) + 2 * p.SC4;
    p.xrowb = ((data > reach ? data : reach) + 15) / 16 * 16;
    if (g.R * (g.W * 3 / 8) > 4 * NT) return false;  // the kernel stages at most 4 x vectors per thread
    p.smem = (size_t)g.R * p.xrowb + (size_t)16 * p.nsteps * (g.K * 2 + 64);
    const size_t epi = (size_t)4 * g.K * 33 * sizeof(float);  // the epilogue's transposing strips reuse the buffer
    if (epi > p.smem) p.smem = epi;
    if (p.smem > 64 * 1024) return false;
    *out = p;
    return true;
}

int c3_grid(long units) {
    long blocks = (units + 3) / 4;
    const long cap = (long)kNumCU * 2;
    return (int)(blocks < cap ? (blocks < 1 ? 1 : blocks) : cap);
}

}  // namespace

namespace {
bool c3_special(const GemmGeom& g) { return g.R == 3 && g.S == 3 && g.mul_h == 1 && g.mul_w == 1; }
// 3x3 stride 1 with whole 32-pixel tiles per output row and 4-byte-aligned input rows: input rows staged in LDS
bool c3_rows(const GemmGeom& g) {
    return c3_special(g) && (g.OW % 32) == 0 && (g.IW % 2) == 0 &&
           (double)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * 3 * 2.0 < 2147483648.0;
}
size_t c3_general_smem(const GemmGeom& g) {
    const size_t ksteps = (size_t)(g.Kred + 15) / 16;
    return 4 * 32 * (size_t)(g.Ncols * 2 + 16) + ksteps * (g.Ncols / 32) * 64 * 16;
}
}  // namespace

bool conv_c3_fwd_supported(const GemmGeom& g) {
    if (g.IC != 3 || g.div_h != 1 || g.div_w != 1 || (g.Ncols != 32 && g.Ncols != 64)) return false;
    return c3_special(g) || c3_fwd_strided(g) || c3_general_smem(g) <= 64 * 1024;
}
const char* conv_c3_fwd_kernel_name(const GemmGeom& g) {
    if (c3_rows(g)) return g.Ncols == 64 ? "conv_c3_fwd_rows_kernel<2>" : "conv_c3_fwd_rows_kernel<1>";
    if (c3_special(g)) return g.Ncols == 64 ? "conv_c3_fwd_kernel<2>" : "conv_c3_fwd_kernel<1>";
    if (c3_fwd_strided(g)) return g.Ncols == 64 ? "conv_c3_fwd_strided_kernel<2>" : "conv_c3_fwd_strided_kernel<1>";
    return g.Ncols == 64 ? "conv_c3_fwd_general_kernel<2>" : "conv_c3_fwd_general_kernel<1>";
}

int launch_conv_c3_fwd(const GemmGeom& g, const bf16_t* x, const bf16_t* w, const float* bias, bool relu, bf16_t* y,
                       hipStream_t st) {
    if (!conv_c3_fwd_supported(g)) return set_error(WAP_EINVAL, "internal: 3-channel forward kernel not applicable");
    if (!c3_special(g) && c3_fwd_strided(g)) {
        C3FPlan p;
        if (!c3f_plan(g, &p)) return set_error(WAP_EINVAL, "internal: strided 3-channel forward plan");
        C3FArgs fa = {};
        fa.x = x; fa.w = w; fa.bias = bias; fa.y = y;
        fa.N = g.M / (g.OH * g.OW); fa.H = g.IH; fa.W = g.IW; fa.OH = g.OH; fa.OW = g.OW; fa.R = g.R; fa.S = g.S;
        fa.sh = g.mul_h; fa.sw = g.mul_w; fa.ph = g.pad_h; fa.pw = g.pad_w;
        fa.G8 = p.G8; fa.ksteps = p.ksteps; fa.Kred = g.Kred; fa.xrowb = p.xrowb;
        fa.units = fa.N * g.OH; fa.nvx = g.IW * 3 / 8; fa.relu = relu ? 1 : 0;
        fa.dOH = make_fastdiv((uint32_t)g.OH);
        fa.dNVX = make_fastdiv((uint32_t)fa.nvx);
        fa.dG8 = make_fastdiv((uint32_t)p.G8);
        fa.dKred = make_fastdiv((uint32_t)g.Kred);
        fa.dS3 = make_fastdiv((uint32_t)(g.S * 3));
        static std::atomic<bool> attr_done{false};
        if (!attr_done) {
            for (const void* f : {(const void*)conv_c3_fwd_strided_kernel<1>, (const void*)conv_c3_fwd_strided_kernel<2>}) {
                hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
                if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
            }
            attr_done = true;
        }
        // every wavefront gathers its weight fragments once: long-lived groups, at least 4 output rows each
        long want = (long)fa.units / 4;
        const long cap = (long)kNumCU * 2;  // LDS (the fragment staging area) and registers allow two groups per CU
        const int sgrid = (int)(want < 1 ? 1 : want < cap ? want : cap);
        if (g.Ncols == 64) hipLaunchKernelGGL(conv_c3_fwd_strided_kernel<2>, dim3(sgrid), dim3(NT), p.smem, st, fa);
        else hipLaunchKernelGGL(conv_c3_fwd_strided_kernel<1>, dim3(sgrid), dim3(NT), p.smem, st, fa);
        return check_launch("conv_c3_fwd_strided");
    }
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
    if (c3_rows(g)) {
        a.tiles_row = g.OW / 32;
        a.ntiles = (g.M / g.OW) * a.tiles_row;
        a.x_bytes = (unsigned)((size_t)a.N * g.IH * g.IW * 3 * 2);
        a.dTR = make_fastdiv((uint32_t)a.tiles_row);
        a.dOH = make_fastdiv((uint32_t)g.OH);
        if (g.Ncols == 64) hipLaunchKernelGGL(conv_c3_fwd_rows_kernel<2>, dim3(grid), dim3(NT), 0, st, a);
        else hipLaunchKernelGGL(conv_c3_fwd_rows_kernel<1>, dim3(grid), dim3(NT), 0, st, a);
        return check_launch("conv_c3_fwd_rows");
    }
    if (g.Ncols == 64) hipLaunchKernelGGL(conv_c3_fwd_kernel<2>, dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL(conv_c3_fwd_kernel<1>, dim3(grid), dim3(NT), 0, st, a);
    return check_launch("conv_c3_fwd");
}

// (A gather-based general-filter weight gradient, lanes indexing the columns k, was tried and dropped: every lane
// touches a different cache line.  Large filters at horizontal stride 4 use the rows-in-LDS kernel above; all other
// first-layer shapes fall to the generic kernel.)
static bool wgrad_c3_special(const WgradGeom& g) {
    return g.C == 3 && g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && (g.K == 32 || g.K == 64) && (g.Q % 8) == 0 &&
           (long)g.N * g.P * g.Q >= 4096;
}
static bool wgrad_c3_strided(const WgradGeom& g) {
    C3SPlan p;
    return !wgrad_c3_special(g) && c3s_plan(g, &p) && (long)g.N * g.P >= 64;
}
bool wgrad_c3_supported(const WgradGeom& g) { return wgrad_c3_special(g) || wgrad_c3_strided(g); }
const char* wgrad_c3_kernel_name(const WgradGeom& g) {
    if (wgrad_c3_strided(g)) return g.K == 64 ? "wgrad_c3_strided_kernel<2>" : "wgrad_c3_strided_kernel<1>";
    return g.K == 64 ? "wgrad_c3_kernel<2>" : "wgrad_c3_kernel<1>";
}

int wgrad_c3_nsplit(const WgradGeom& g) {
    if (wgrad_c3_strided(g)) {
        // at least 8 output rows per work-group (each leaves a K x R*S*3 fp32 partial), at most two groups per CU
        const long units = (long)g.N * g.P, cap = (long)kNumCU * 2;
        const long want = units / 8;
        return (int)(want < 1 ? 1 : want < cap ? want : cap);
    }
    return c3_grid(((long)g.N * g.P * g.Q + 15) / 16);
}

int launch_wgrad_c3(const WgradGeom& g, int nsplit, const bf16_t* x, const bf16_t* dy, float* part, hipStream_t st) {
    if (!wgrad_c3_supported(g)) return set_error(WAP_EINVAL, "internal: 3-channel weight-gradient kernel not applicable");
    if (wgrad_c3_strided(g)) {
        C3SPlan p;
        if (!c3s_plan(g, &p)) return set_error(WAP_EINVAL, "internal: strided 3-channel weight-gradient plan");
        C3SArgs sa = {};
        sa.x = x; sa.dy = dy; sa.part = part;
        sa.N = g.N; sa.H = g.H; sa.W = g.W; sa.OH = g.P; sa.OW = g.Q; sa.R = g.R; sa.S = g.S;
        sa.sh = g.sh; sa.sw = g.sw; sa.ph = g.ph; sa.pw = g.pw;
        sa.SC4 = p.SC4; sa.NB = p.NB; sa.Kred = g.R * g.S * 3; sa.xrowb = p.xrowb;
        sa.units = g.N * g.P; sa.nsteps = p.nsteps; sa.nvx = g.W * 3 / 8;
        sa.dOH = make_fastdiv((uint32_t)g.P);
        sa.dSC4 = make_fastdiv((uint32_t)p.SC4);
        sa.dNVX = make_fastdiv((uint32_t)sa.nvx);
        static std::atomic<bool> attr_done{false};
        if (!attr_done) {
            for (const void* f : {(const void*)wgrad_c3_strided_kernel<1>, (const void*)wgrad_c3_strided_kernel<2>}) {
                hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
                if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
            }
            attr_done = true;
        }
        if (g.K == 64) hipLaunchKernelGGL(wgrad_c3_strided_kernel<2>, dim3(nsplit), dim3(NT), p.smem, st, sa);
        else hipLaunchKernelGGL(wgrad_c3_strided_kernel<1>, dim3(nsplit), dim3(NT), p.smem, st, sa);
        return check_launch("wgrad_c3_strided");
    }
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
