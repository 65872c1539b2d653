// Stride-1 convolution (forward, and data gradient with flipped weights) for layers with FEW output
// channels on LARGE feature maps (gfx950): the first VGG blocks, 64 or 128 channels at 224 / 112
// pixels, where a 256-channel tile would idle most of its columns and the layer sits at the ridge
// between the matrix cores and HBM.
//
// Same idea as conv_patch.hip (the zero-padded input patch of one 64-channel slice is written to LDS
// once and every filter tap reads it through a shifted pointer; weights go from their packed copy
// straight into MFMA operand registers), with the pieces re-proportioned for a thin output:
//   * a work-group owns a 2-D tile of 8 x 32 (or 16 x 16) output pixels of ONE image, so the patch is
//     only (8 + R - 1) x (32 + S - 1) padded pixels (49 KB for 3x3) and one 32-pixel fragment is one tile
//     row (two for the square tile): its LDS rows are contiguous at the conflict-free 144-byte pitch;
//   * 4 wavefronts = 2 pixel halves x 2 channel halves, each 128 pixels x 32*FN channels;
//   * the patch is single-buffered and the kernel is written for 2-3 resident work-groups per CU
//     (LDS and registers are sized for that): while one group waits for its patch or drains its
//     epilogue the others keep the matrix cores busy, which suits layers whose 64 input channels give
//     each group a single slice and nothing of its own to overlap with.
// Serves the "primary" convolution nodes of Section 3.2.2 (forward and backward halves of t_c, Eq. 1).
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64, BM = 256, NT = 256, FM = 4;
constexpr int PITCH = (BK + 8) * 2;  // 144 bytes per padded pixel
constexpr int MAX_PATCH = 352;       // padded pixels (>= (tile h + R - 1) * (tile w + S - 1)); also the staging area
constexpr int PV = (MAX_PATCH * 8 + NT - 1) / NT;  // 16-byte patch vectors per thread

struct TArgs {
    const bf16_t* A;
    const bf16_t* Wp;  // packed weights
    const float* bias;
    const bf16_t* mask;  // optional: out = mask > 0 ? out : 0
    bf16_t* out;
    GemmGeom g;
    int tiles_x, tiles_y, tiles_img, tiles_m, tiles_n;
    int PWp, patch_len;  // padded tile width, padded pixels per patch
    int relu;
    unsigned a_bytes, w_bytes;
    FastDiv dTimg, dTx, dPWp;
};

__device__ __forceinline__ int xcd_remap(int bid, int total) {
    int per = total / kNumXCD, rem = total % kNumXCD;
    int xcd = bid % kNumXCD, idx = bid / kNumXCD;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}
__device__ __forceinline__ unsigned short f2bf(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(unsigned short, b);
}

// keeps the bf16 lanes of v whose mask lane is > 0 (the ReLU derivative of the layer that produced the mask)
__device__ __forceinline__ u32x4 relu_mask8(u32x4 v, u32x4 mk) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const unsigned lo = __uint_as_float(mk[k] << 16) > 0.f ? 0xffffu : 0u;
        const unsigned hi = __uint_as_float(mk[k] & 0xffff0000u) > 0.f ? 0xffff0000u : 0u;
        v[k] &= (lo | hi);
    }
    return v;
}

// FN: 32-channel blocks per wavefront (tile = 64 * FN output channels); TW: tile width in pixels (32 or 16)
template <int FN, int TW>
__global__ __launch_bounds__(NT, (FN == 1 ? 3 : 2)) void conv_tile2d_kernel(const TArgs a) {
    constexpr int TH = BM / TW;
    extern __shared__ __align__(16) unsigned char smem[];
    const GemmGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pg = wave & 1, cg = wave >> 1;  // pixel half, channel half
    constexpr int BN = 64 * FN;

    int logical = xcd_remap(blockIdx.x, a.tiles_m * a.tiles_n);
    const int tn = logical % a.tiles_n;
    const int tm = logical / a.tiles_n;
    const int img = (int)fdiv((uint32_t)tm, a.dTimg);
    const int trem = tm - img * a.tiles_img;
    const int tyi = (int)fdiv((uint32_t)trem, a.dTx);
    const int oh0 = tyi * TH, ow0 = (trem - tyi * a.tiles_x) * TW;
    const int n0 = tn * BN;
    const int RS = g.R * g.S;
    const int ncs = g.IC / BK;

    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.A), 0, (int)a.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.Wp), 0, (int)a.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0x80000000u;  // the activation tensor is below 2 GiB (checked on the host)

    // ---- patch vectors of this thread: byte offset of (padded pixel, 8-channel vector) or OOB ----
    unsigned pvoff[PV];
#pragma unroll
    for (int i = 0; i < PV; ++i) {
        int v = tid + i * NT;
        int q = v >> 3;
        unsigned off = OOB;
        if (q < a.patch_len) {
            int py = (int)fdiv((uint32_t)q, a.dPWp);
            int px = q - py * a.PWp;
            int ih = oh0 - g.pad_h + py, iw = ow0 - g.pad_w + px;
            if ((unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW)
                off = (unsigned)(((img * g.IH + ih) * g.IW + iw) * g.IC + (v & 7) * 8) * 2u;
        }
        pvoff[i] = off;
    }

    // ---- fragment rows of this lane: fragment j holds tile pixels (pg * 4 + j) * 32 .. + 31 in raster order ----
    int frow[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int idx = (pg * FM + j) * 32 + (lane & 31);
        frow[j] = ((idx / TW) * a.PWp + (idx % TW)) * PITCH + (lane >> 5) * 16;
    }

    // ---- weights: packed [channel block of 32][reduction step of 16][lane][8] ----
    const unsigned ksteps = (unsigned)g.Kred / 16u;
    unsigned wrow[FN];
#pragma unroll
    for (int i = 0; i < FN; ++i) {
        unsigned blk = (unsigned)(n0 + cg * 32 * FN + i * 32) / 32u;
        wrow[i] = (blk * ksteps * 64u + (unsigned)lane) * 16u;
    }
    auto load_w = [&](int cs, int tap, bf16x8 (&w)[4][FN]) {
        const unsigned koff = ((unsigned)(tap * g.IC + cs * BK) / 16u) * 1024u;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < FN; ++i)
                w[ks][i] = __builtin_bit_cast(
                    bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrcW, wrow[i] + koff + (unsigned)ks * 1024u, 0, 0));
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 wA[4][FN], wB[4][FN];
    load_w(0, 0, wA);

    for (int cs = 0; cs < ncs; ++cs) {
        {
            u32x4 rp[PV];
            const unsigned coff = (unsigned)(cs * BK) * 2u;
#pragma unroll
            for (int i = 0; i < PV; ++i) rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, pvoff[i] + coff, 0, 0);
            if (cs > 0) __syncthreads();  // every wavefront has finished reading the previous slice's patch
#pragma unroll
            for (int i = 0; i < PV; ++i) {
                int v = tid + i * NT;
                if ((v >> 3) < MAX_PATCH) *reinterpret_cast<u32x4*>(smem + (v >> 3) * PITCH + (v & 7) * 16) = rp[i];
            }
        }
        __syncthreads();
        const int cs1 = cs + 1 < ncs ? cs + 1 : cs;
        int r = 0, s = 0;
        for (int tap = 0; tap < RS; ++tap) {
            const bool last = tap + 1 == RS;
            const int tapoff = (r * a.PWp + s) * PITCH;
            load_w(last ? cs1 : cs, last ? 0 : tap + 1, wB);  // one reduction tile ahead (clamped at the very end)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int j = 0; j < FM; ++j) {
                    bf16x8 f = *reinterpret_cast<const bf16x8*>(smem + frow[j] + tapoff + ks * 32);
#pragma unroll
                    for (int i = 0; i < FN; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wA[ks][i], f, acc[i][j], 0, 0, 0);
                }
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < FN; ++i) wA[ks][i] = wB[ks][i];
            if (++s == g.S) { s = 0; ++r; }
        }
    }

    // ---- epilogue: bias / ReLU / bf16, transposed through LDS (the patch is dead) so that every global store
    // is 16 contiguous bytes per lane and a tile row of 32 pixels is one contiguous run ----
    constexpr int OPITCH = BN * 2 + 16;  // bytes per pixel row in the staging buffer
    constexpr int VPR = BN / 8;          // 16-byte vectors per pixel row
    constexpr int RPP = NT / VPR;        // pixel rows stored per pass
    constexpr int HROWS = (FN == 1) ? BM : BM / 2;  // pixel rows staged per pass (fits the patch area)
#pragma unroll
    for (int half = 0; half < BM / HROWS; ++half) {
        __syncthreads();  // previous readers of the staging area (or of the patch) are done
        // FN == 1: all 8 tile rows at once; FN == 2: fragments 0-1 of both pixel halves, then fragments 2-3
        constexpr int JN = (FN == 1) ? FM : FM / 2;
#pragma unroll
        for (int jj = 0; jj < JN; ++jj) {
            const int j = half * JN + jj;
            const int srow = ((FN == 1) ? (pg * FM + j) : (pg * JN + jj)) * 32 + (lane & 31);
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int nl = cg * 32 * FN + i * 32 + q * 8 + (lane >> 5) * 4;  // channel within the tile
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
                    if (a.bias) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += a.bias[n0 + nl + e];
                    }
                    if (a.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                    }
                    uint2 pk = make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                                          (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
                    *reinterpret_cast<uint2*>(smem + srow * OPITCH + nl * 2) = pk;
                }
        }
        __syncthreads();
        for (int row = tid / VPR; row < HROWS; row += RPP) {
            // staged row -> tile pixel: FN == 1: the same; FN == 2: pixel half row / 64, its fragments 2 * half, 2 * half + 1
            const int idx = (FN == 1) ? row : ((row >> 6) * (BM / 2) + half * (BM / 4) + (row & 63));
            const int m = (img * g.OH + oh0 + idx / TW) * g.OW + ow0 + idx % TW;
            u32x4 vv = *reinterpret_cast<const u32x4*>(smem + row * OPITCH + (tid % VPR) * 16);
            const size_t o = (size_t)m * g.Ncols + n0 + (tid % VPR) * 8;
            if (a.mask) vv = relu_mask8(vv, *reinterpret_cast<const u32x4*>(a.mask + o));
            *reinterpret_cast<u32x4*>(a.out + o) = vv;
        }
    }
}

template <int FN, int TW>
int launch_tile2d_t(const TArgs& ta, hipStream_t st) {
    auto kfn = conv_tile2d_kernel<FN, TW>;
    constexpr size_t smem = (size_t)MAX_PATCH * PITCH;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(ta.tiles_m * ta.tiles_n), dim3(NT), smem, st, ta);
    return check_launch("conv_tile2d");
}

}  // namespace

namespace {
// tile width that divides the feature map (and whose patch fits), or 0
int tile_width(const GemmGeom& g) {
    for (int tw : {32, 16, 8}) {
        const int th = BM / tw;
        if ((g.OH % th) == 0 && (g.OW % tw) == 0 && (th + g.R - 1) * (tw + g.S - 1) <= MAX_PATCH) return tw;
    }
    return 0;
}
}  // namespace

// 0 = not applicable, otherwise FN (32-channel blocks per wavefront)
int tile2d_supported(const GemmGeom& g) {
    if ((g.IC % BK) != 0 || g.div_h != 1 || g.div_w != 1 || g.mul_h != 1 || g.mul_w != 1) return 0;
    if (g.R * g.S < 2) return 0;
    if (!tile_width(g)) return 0;
    if (g.Ncols != 64 && (g.Ncols % 128) != 0) return 0;
    long a_elems = (long)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * g.IC;
    if (a_elems * 2 >= (1L << 31)) return 0;
    return g.Ncols == 64 ? 1 : 2;
}

const char* tile2d_kernel_name(const GemmGeom& g) {
    static const char* names[2][3] = {{"conv_tile2d_kernel<1,32>", "conv_tile2d_kernel<1,16>", "conv_tile2d_kernel<1,8>"},
                                      {"conv_tile2d_kernel<2,32>", "conv_tile2d_kernel<2,16>", "conv_tile2d_kernel<2,8>"}};
    const int fn = tile2d_supported(g), tw = tile_width(g);
    return names[fn == 2 ? 1 : 0][tw == 32 ? 0 : tw == 16 ? 1 : 2];
}

int launch_tile2d(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                  hipStream_t st, const bf16_t* mask) {
    TArgs ta;
    ta.mask = mask;
    const int fn = tile2d_supported(g);
    if (!fn) return set_error(WAP_EINVAL, "internal: 2-D tile kernel not applicable");
    ta.A = A;
    ta.Wp = reinterpret_cast<const bf16_t*>(Wp);
    ta.bias = bias;
    ta.out = out;
    ta.g = g;
    const int TW = tile_width(g), TH = BM / TW;
    ta.tiles_x = g.OW / TW;
    ta.tiles_y = g.OH / TH;
    ta.tiles_img = ta.tiles_x * ta.tiles_y;
    ta.tiles_m = ta.tiles_img * (g.M / (g.OH * g.OW));
    ta.tiles_n = g.Ncols / (64 * fn);
    ta.PWp = TW + g.S - 1;
    ta.patch_len = (TH + g.R - 1) * ta.PWp;
    ta.relu = relu ? 1 : 0;
    ta.a_bytes = (unsigned)((size_t)(g.M / (g.OH * g.OW)) * g.IH * g.IW * g.IC * 2);
    ta.w_bytes = (unsigned)wreg_wt_bytes(g);
    ta.dTimg = make_fastdiv((uint32_t)ta.tiles_img);
    ta.dTx = make_fastdiv((uint32_t)ta.tiles_x);
    ta.dPWp = make_fastdiv((uint32_t)ta.PWp);
    if (TW == 32) return fn == 1 ? launch_tile2d_t<1, 32>(ta, st) : launch_tile2d_t<2, 32>(ta, st);
    if (TW == 16) return fn == 1 ? launch_tile2d_t<1, 16>(ta, st) : launch_tile2d_t<2, 16>(ta, st);
    return fn == 1 ? launch_tile2d_t<1, 8>(ta, st) : launch_tile2d_t<2, 8>(ta, st);
}

}  // namespace wap
