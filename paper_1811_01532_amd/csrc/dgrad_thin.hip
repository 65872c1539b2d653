// Data gradient of a convolution whose INPUT has very few channels (the 3-channel image of the first layer):
//   dx[n,h,w,c] = sum over (k,r,s) of dy[n,p,q,k] * w[k,r,s,c]   with p*stride_h - pad_h + r = h, q likewise,
// the backward half of t_c (Eq. 1) of the first "primary" node of Section 3.2.2.  As a matrix product it has 3
// (at most 4) output columns, so an MFMA tile would be nine-tenths padding and the pass is bound by reading dy once;
// it runs on the vector ALUs instead:
//   * a wavefront owns 64 pixels of one image row that share their phase (w mod stride_w), so all of them visit the
//     same filter taps, as eight groups of eight neighbouring pixels; lane (pixel i of the group, channel chunk j)
//     fetches 16 bytes = channels 8j..8j+7 of dy at its pixel, so a group's load is one contiguous run of dy
//     (neighbouring pixels of a phase read neighbouring dy pixels) and nothing is fetched twice per tap;
//   * the lane keeps the weights of its eight channels for the current tap in registers (fp32 copy laid out
//     [tap][k][4] by a small packing kernel) and accumulates its partial sums of the <= 4 output channels for
//     each of the eight groups; at the end the eight chunk lanes of a pixel are added with a fixed butterfly
//     (bitwise reproducible) and one lane stores the pixel as bf16;
//   * positions the forward pass never reads come out as exact zeros (no tap is valid there).
// With a stride above one only the taps with (h + pad - r) mod stride = 0 exist for a given row / phase; the loops
// step through exactly those.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int NT = 64;

struct ThinArgs {
    const bf16_t* dy;   // [N][IH][IW][K]
    const float* wp;    // packed weights [R*S][K][4] (column c of tap (r,s), zero beyond Ncols), forward tap order
    bf16_t* dx;         // [N][OH][OW][C]
    int N, IH, IW, K, OH, OW, C, R, S, sh, sw, ph, pw;  // ph / pw: the forward pass's padding
    unsigned dy_bytes, wp_bytes;  // both below 2 GiB (host)
    int cols;           // ceil(OW / sw): pixels of one phase in a row
    int colblocks;      // ceil(cols / 64)
    FastDiv dCB, dSW, dOH;
};

__device__ __forceinline__ unsigned short f2bf(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(unsigned short, b);
}

// fp32 copy of the weights in the order the gradient kernel walks them: wp[(r*S+s)*K + k][c], c < 4
__global__ void dgrad_thin_pack_kernel(const bf16_t* __restrict__ w, float* __restrict__ wp, int K, int RS, int C) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;  // (tap, k)
    if (i >= RS * K) return;
    const int tap = i / K, k = i - tap * K;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    const bf16_t* src = w + ((size_t)k * RS + tap) * C;
    float* f = reinterpret_cast<float*>(&v);
    for (int c = 0; c < C; ++c) f[c] = __uint_as_float((unsigned)src[c] << 16);
    reinterpret_cast<float4*>(wp)[i] = v;
}

__global__ __launch_bounds__(NT) void dgrad_thin_kernel(const ThinArgs a) {
    // block -> (image n, row h, phase of w, block of 64 columns of that phase): all uniform
    int b = blockIdx.x;
    const int cb = b - (int)fdiv((uint32_t)b, a.dCB) * a.colblocks;
    b = (int)fdiv((uint32_t)b, a.dCB);
    const int phase = b - (int)fdiv((uint32_t)b, a.dSW) * a.sw;
    b = (int)fdiv((uint32_t)b, a.dSW);
    const int h = b - (int)fdiv((uint32_t)b, a.dOH) * a.OH;
    const int n = (int)fdiv((uint32_t)b, a.dOH);
    const int lane = threadIdx.x, pi = lane >> 3, kc = lane & 7;  // pixel within a group, channel chunk

    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.dy), 0, (int)a.dy_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.wp), 0, (int)a.wp_bytes, 0x00020000);
    float acc[8][4];
#pragma unroll
    for (int gi = 0; gi < 8; ++gi)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[gi][c] = 0.f;

    // taps with h + ph - r = p * sh: r = r0, r0 + sh, ...
    const int r0 = (h + a.ph) % a.sh, s0 = (phase + a.pw) % a.sw;
    for (int r = r0; r < a.R; r += a.sh) {
        const int p = (h + a.ph - r) / a.sh;
        if (h + a.ph - r < 0 || p >= a.IH) continue;  // uniform
        for (int s = s0; s < a.S; s += a.sw) {
            for (int k0 = 0; k0 < a.K; k0 += 64) {     // 64 channels per pass: chunk kc holds k0 + 8 kc .. + 7
                const int kk = k0 + kc * 8;
                // this lane's weights for the tap (out of range beyond K: zeros)
                f32x4 wv[8];
                const unsigned woff = kk < a.K ? (unsigned)(((r * a.S + s) * a.K + kk) * 16) : 0x80000000u;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    wv[e] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrcW, woff + (unsigned)e * 16u, 0, 0));
#pragma unroll
                for (int gi = 0; gi < 8; ++gi) {
                    const int j = cb * 64 + gi * 8 + pi;   // index within the phase
                    const int wq = phase + j * a.sw;       // the pixel's column
                    const int t = wq + a.pw - s;           // a multiple of sw
                    const int q = t / a.sw;
                    const bool ok = j < a.cols && wq < a.OW && t >= 0 && q < a.IW && kk < a.K;
                    // lanes without a pixel read from beyond the buffer's range: zeros, no branch around the load
                    const unsigned src = ok ? (unsigned)(((n * a.IH + p) * a.IW + q) * a.K + kk) * 2u : 0x80000000u;
                    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, src, 0, 0);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float g = __uint_as_float((e & 1) ? (v[e >> 1] & 0xffff0000u) : (v[e >> 1] << 16));
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[gi][c] = __builtin_fmaf(g, wv[e][c], acc[gi][c]);
                    }
                }
            }
        }
    }
    // add the eight chunk lanes of every pixel (lanes 8 i .. 8 i + 7) in a fixed butterfly; lane 8 i stores
#pragma unroll
    for (int gi = 0; gi < 8; ++gi) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float v = acc[gi][c];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            acc[gi][c] = v;
        }
        const int j = cb * 64 + gi * 8 + pi;
        const int wq = phase + j * a.sw;
        if (kc == 0 && j < a.cols && wq < a.OW) {
            bf16_t* dst = a.dx + ((size_t)(n * a.OH + h) * a.OW + wq) * a.C;
            for (int c = 0; c < a.C; ++c) dst[c] = f2bf(acc[gi][c]);
        }
    }
}

}  // namespace

// g: the data-gradient geometry (rows = input pixels, gathered tensor = dy, Ncols = input channels of the layer)
bool dgrad_thin_supported(const GemmGeom& g) {
    if (g.Ncols > 4 || (g.IC % 8) != 0 || g.mul_h != 1 || g.mul_w != 1) return false;
    if ((double)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * g.IC * 2.0 >= 2147483648.0) return false;  // 32-bit dy offsets
    const long blocks = (long)(g.M / g.OW) * g.div_w * (((g.OW + g.div_w - 1) / g.div_w + NT - 1) / NT);
    return blocks < (1L << 31);
}
size_t dgrad_thin_ws_bytes(const GemmGeom& g) { return (size_t)g.R * g.S * g.IC * 4 * sizeof(float); }

int launch_dgrad_thin(const GemmGeom& g, const bf16_t* dy, const bf16_t* w, bf16_t* dx, void* ws, hipStream_t st) {
    if (!dgrad_thin_supported(g)) return set_error(WAP_EINVAL, "internal: thin data-gradient kernel not applicable");
    const int RS = g.R * g.S, K = g.IC;
    hipLaunchKernelGGL(dgrad_thin_pack_kernel, dim3((RS * K + 255) / 256), dim3(256), 0, st, w, reinterpret_cast<float*>(ws),
                       K, RS, g.Ncols);
    int rc = check_launch("dgrad_thin_pack");
    if (rc != WAP_OK) return rc;
    ThinArgs a;
    a.dy = dy;
    a.wp = reinterpret_cast<const float*>(ws);
    a.dx = dx;
    a.wp_bytes = (unsigned)dgrad_thin_ws_bytes(g);
    a.dy_bytes = (unsigned)((size_t)(g.M / (g.OH * g.OW)) * g.IH * g.IW * g.IC * 2);
    a.N = g.M / (g.OH * g.OW);
    a.IH = g.IH; a.IW = g.IW; a.K = K;
    a.OH = g.OH; a.OW = g.OW; a.C = g.Ncols;
    a.R = g.R; a.S = g.S;
    a.sh = g.div_h; a.sw = g.div_w;
    a.ph = g.R - 1 - g.pad_h; a.pw = g.S - 1 - g.pad_w;  // the geometry carries the flipped-filter padding
    a.cols = (g.OW + a.sw - 1) / a.sw;
    a.colblocks = (a.cols + NT - 1) / NT;
    a.dCB = make_fastdiv((uint32_t)a.colblocks);
    a.dSW = make_fastdiv((uint32_t)a.sw);
    a.dOH = make_fastdiv((uint32_t)a.OH);
    const long blocks = (long)a.N * a.OH * a.sw * a.colblocks;
    hipLaunchKernelGGL(dgrad_thin_kernel, dim3((unsigned)blocks), dim3(NT), 0, st, a);
    return check_launch("dgrad_thin");
}

}  // namespace wap
