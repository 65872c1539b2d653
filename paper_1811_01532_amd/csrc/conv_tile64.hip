// Stride-1 convolution (forward, and data gradient with flipped weights) for layers with 64 OUTPUT channels on
// LARGE feature maps (gfx950): conv1_2 of VGG-16 and the data gradient of conv2_1, where a wider channel tile
// would idle most of its columns and the layer sits at the ridge between the matrix cores and HBM.
//
// Same idea as conv_tile2d.hip (the zero-padded input patch of a channel slice is written to LDS once and every
// filter tap reads it through a shifted pointer; weights go from their packed copy straight into MFMA operand
// registers), with the pieces proportioned for a thin output:
//   * a work-group owns a 2-D tile of 8 x 32 (16 x 16, 32 x 8) output pixels of ONE image and all 64 channels; the
//     patch is (8 + R - 1) x (32 + S - 1) padded pixels of a 64-channel slice (49 KB for 3x3) at a 144-byte pitch;
//   * 4 wavefronts = 2 pixel halves x 2 channel halves, each 128 pixels x 32 channels (64 accumulator registers);
//   * the patch is single-buffered and the kernel is sized for THREE resident work-groups per CU (LDS and
//     registers): a layer with 64 input channels gives each group a single slice and nothing of its own to overlap
//     with, so while one group waits for its patch or drains its epilogue the others keep the matrix cores busy.
//     (The double-buffered 32-channel slices of conv_tile2d.hip fit only two groups per CU and measured 12-15 %
//     slower on these layers.)
// UP variant (data gradient of a layer followed by a 2x2 / stride-2 max-pool): the input operand arrives as
// the gradient of the POOLED output plus the pool's argmax; the patch loader routes each window's value to
// the pixel its argmax names, so the max-pool backward costs no pass over the full-size gradient.
// Serves the "primary" convolution nodes of Section 3.2.2 (forward and backward halves of t_c, Eq. 1).
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64, NT = 256;
constexpr int PITCH = (BK + 8) * 2;  // 144 bytes per padded pixel: 16 consecutive rows fall into 16 distinct bank groups
constexpr int MAX_PATCH = 352;       // padded pixels (>= (tile h + R - 1) * (tile w + S - 1)); also the staging area
constexpr int FM = 4, PG = 2, BM = 32 * FM * PG, BN = 64;  // 256 pixels x 64 channels, 2 x 2 wavefronts

struct T64Args {
    const bf16_t* A;
    const bf16_t* Wp;      // packed weights
    const float* bias;
    const bf16_t* mask;    // optional: out = mask > 0 ? out : 0
    const uint8_t* up_am;  // UP: argmax (r * 2 + s) per pooling window; A is then N x IH/2 x IW/2 x IC
    bf16_t* out;           // may be NULL when only the pooled output is wanted
    bf16_t* pool_y;        // optional: 2x2 / stride-2 max-pool of the output tile ...
    uint8_t* pool_am;      // ... and the position r*2+s of the first maximum of every window
    float* colsum;         // optional: [tiles_m][64] column sums of this tile's stored (masked) rows, for a bias gradient
    GemmGeom g;
    int tiles_x, tiles_img, tiles_m;
    int RW, patch_len;     // patch row width in pixels (tile width + S - 1), patch pixels to load
    int relu;
    unsigned a_bytes, w_bytes;
    FastDiv dTimg, dTx, dRW;
    int UW, units;         // UP: pooling windows per patch row, windows per patch
    FastDiv dUW;
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

// keeps the bf16 lanes of the pooled gradient v whose window's argmax byte equals this pixel's position code
__device__ __forceinline__ u32x4 unpool_select8(u32x4 v, u32x2 am, unsigned code) {
    const unsigned c4 = code * 0x01010101u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const unsigned x = ((k < 2 ? am[0] : am[1]) >> ((k & 1) * 16)) ^ c4;  // a zero byte where argmax == code
        const unsigned lo = (x & 0xffu) == 0u ? 0xffffu : 0u;
        const unsigned hi = (x & 0xff00u) == 0u ? 0xffff0000u : 0u;
        v[k] &= (lo | hi);
    }
    return v;
}

// TW: tile width in pixels (the tile is 256 / TW rows high).  UP: pooled input operand.  T9: 3x3 filter, the nine
// taps of a slice as straight-line code (every fragment address an immediate offset, the two weight register sets
// alternating by tap instead of being copied, no loop bookkeeping: the time of these kernels follows their
// instruction count).
template <int TW, bool UP, bool T9>
__global__ __launch_bounds__(NT, 3) void conv_tile64_kernel(const T64Args a) {
    constexpr int TH = BM / TW;
    constexpr int PV = (MAX_PATCH * 8 + NT - 1) / NT;  // 16-byte patch vectors per thread
    extern __shared__ __align__(16) unsigned char smem[];
    const GemmGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pg = wave % PG, cg = wave / PG;  // pixel half, channel half

    const int tm = xcd_remap(blockIdx.x, a.tiles_m);
    const int img = (int)fdiv((uint32_t)tm, a.dTimg);
    const int trem = tm - img * a.tiles_img;
    const int tyi = (int)fdiv((uint32_t)trem, a.dTx);
    const int oh0 = tyi * TH, ow0 = (trem - tyi * a.tiles_x) * TW;
    const int RS = g.R * g.S;
    const int ncs = g.IC / BK;

    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.A), 0, (int)a.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.Wp), 0, (int)a.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0x80000000u;  // the activation tensor is below 2 GiB (checked on the host)
    const __amdgpu_buffer_rsrc_t rsrcM =  // UP: one argmax byte per pooled element, half the bytes of the pooled tensor
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(UP ? a.up_am : nullptr), 0, UP ? (int)(a.a_bytes / 2) : 0, 0x00020000);
    const int IH2 = g.IH >> 1, IW2 = g.IW >> 1;

    // ---- patch vectors of this thread: byte offset of (padded pixel, 8-channel vector) or OOB ----
    unsigned pvoff[UP ? 1 : PV];
#pragma unroll
    for (int i = 0; i < (UP ? 0 : PV); ++i) {
        int v = tid + i * NT;
        int q = v >> 3;
        unsigned off = OOB;
        if (q < a.patch_len) {
            int py = (int)fdiv((uint32_t)q, a.dRW);
            int px = q - py * a.RW;
            int ih = oh0 - g.pad_h + py, iw = ow0 - g.pad_w + px;
            if ((unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW)
                off = (unsigned)(((img * g.IH + ih) * g.IW + iw) * g.IC + (v & 7) * 8) * 2u;
        }
        pvoff[i] = off;
    }

    // ---- UP: window `unit` = thread index / 8 (+ 32 per round) of the (UH x UW) windows that touch the patch; one
    // 16-byte load of the pooled gradient and one 8-byte load of the argmax serve its four pixels.  uq0 = patch row of
    // the window's top-left pixel (it may lie one row / column outside the patch), uval = which of the four pixels are
    // inside the patch, 4 bits per window ----
    constexpr int UPV = 4;
    unsigned uoff[UP ? UPV : 1];
    int uq0[UP ? UPV : 1];
    unsigned uval = 0;
    if (UP) {
        const int ihf = oh0 - g.pad_h, iwf = ow0 - g.pad_w;  // image coordinates of patch pixel (0, 0)
        const int wy0 = ihf >> 1, wx0 = iwf >> 1;            // its window (floor division also below zero)
        const int PHt = TH + g.R - 1;
#pragma unroll
        for (int i = 0; i < UPV; ++i) {
            const int unit = (tid >> 3) + i * (NT / 8);
            const int uy = (int)fdiv((uint32_t)unit, a.dUW), ux = unit - uy * a.UW;
            const int wy = wy0 + uy, wx = wx0 + ux;
            const int py = 2 * wy - ihf, px = 2 * wx - iwf;
            unsigned off = OOB;
            if (unit < a.units && (unsigned)wy < (unsigned)IH2 && (unsigned)wx < (unsigned)IW2)
                off = (unsigned)(((img * IH2 + wy) * IW2 + wx) * g.IC + (tid & 7) * 8) * 2u;
            uoff[i] = off;
            uq0[i] = py * a.RW + px;
            if (unit < a.units) {
                const unsigned vy0 = py >= 0, vy1 = py + 1 < PHt, vx0 = px >= 0, vx1 = px + 1 < a.RW;
                uval |= ((vy0 & vx0) | ((vy0 & vx1) << 1) | ((vy1 & vx0) << 2) | ((vy1 & vx1) << 3)) << (4 * i);
            }
        }
    }

    // ---- fragment rows of this lane: fragment j holds tile pixels (pg * 4 + j) * 32 .. + 31 in raster order ----
    int frow[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int idx = (pg * FM + j) * 32 + (lane & 31);
        frow[j] = ((idx / TW) * (T9 ? TW + 2 : a.RW) + (idx % TW)) * PITCH + (lane >> 5) * 16;
    }

    // ---- weights: packed [channel block of 32][reduction step of 16][lane][8] ----
    const unsigned ksteps = (unsigned)g.Kred / 16u;
    const unsigned wrow = ((unsigned)cg * ksteps * 64u + (unsigned)lane) * 16u;
    auto load_w = [&](int cs, int tap, bf16x8 (&w)[4]) {
        const unsigned koff = ((unsigned)(tap * g.IC + cs * BK) / 16u) * 1024u;  // uniform: rides in the scalar offset
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            w[ks] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrcW, wrow + (unsigned)ks * 1024u, koff, 0));
    };

    f32x16 acc[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

    bf16x8 wA[4], wB[4];
    load_w(0, 0, wA);

    for (int cs = 0; cs < ncs; ++cs) {
        const unsigned coff = (unsigned)(cs * BK) * 2u;
        if (UP) {
            u32x4 rp[UPV];
            u32x2 ra[UPV];  // the out-of-range offset halves to one that is still past the (half as long) argmax tensor
#pragma unroll
            for (int i = 0; i < UPV; ++i) {
                rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, uoff[i] + coff, 0, 0);
                ra[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrcM, (uoff[i] + coff) >> 1, 0, 0);
            }
            if (cs > 0) __syncthreads();  // every wavefront has finished reading the previous slice's patch
#pragma unroll
            for (int i = 0; i < UPV; ++i)
#pragma unroll
                for (int pos = 0; pos < 4; ++pos)
                    if ((uval >> (4 * i + pos)) & 1u)
                        *reinterpret_cast<u32x4*>(smem + (uq0[i] + (pos >> 1) * a.RW + (pos & 1)) * PITCH + (tid & 7) * 16) =
                            unpool_select8(rp[i], ra[i], (unsigned)pos);
        } else {
            u32x4 rp[PV];
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
        // Fragment reads run one reduction step ahead of the MFMAs that consume them (two register sets), and the
        // issue order is pinned: with three wavefronts per SIMD the compiler's own order (read, wait, MFMA) leaves the
        // LDS latency exposed in front of most MFMAs.
        bf16x8 fa[2][FM];
#pragma unroll
        for (int j = 0; j < FM; ++j) fa[0][j] = *reinterpret_cast<const bf16x8*>(smem + frow[j]);
        __builtin_amdgcn_s_setprio(1);
        // one tap: 4 reduction steps of 16 channels x FM fragments; the weights of the following tap are fetched
        // meanwhile, and the last step's fragment reads already belong to that tap
        auto tap_body = [&](const bf16x8 (&wc)[4], bf16x8 (&wn)[4], int tapoff, int tapoff1, int ncs_, int ntap) {
            __builtin_amdgcn_sched_barrier(0);
            load_w(ncs_, ntap, wn);  // one reduction tile ahead
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int j = 0; j < FM; ++j)
                    fa[(ks + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(
                        smem + frow[j] + (ks < 3 ? tapoff + (ks + 1) * 32 : tapoff1));
#pragma unroll
                for (int j = 0; j < FM; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wc[ks], fa[ks & 1][j], acc[j], 0, 0, 0);
            }
            // issue order: the 4 weight loads ride on the first MFMAs, then one fragment read per MFMA
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
            }
#pragma unroll
            for (int q = 0; q < 4 * FM - 4; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        if constexpr (T9) {
            constexpr int RWc = TW + 2;
            auto off = [](int t) { return ((t / 3) * RWc + (t % 3)) * PITCH; };
            // taps 0, 2, 4, 6, 8 run from wA and fetch into wB, the odd ones the other way round; the weights of the
            // next slice's first tap arrive in wB and are moved once per slice (after the last tap the fragment read
            // is discarded, and past the last slice the weight load is a harmless repeat)
            tap_body(wA, wB, off(0), off(1), cs, 1);
            tap_body(wB, wA, off(1), off(2), cs, 2);
            tap_body(wA, wB, off(2), off(3), cs, 3);
            tap_body(wB, wA, off(3), off(4), cs, 4);
            tap_body(wA, wB, off(4), off(5), cs, 5);
            tap_body(wB, wA, off(5), off(6), cs, 6);
            tap_body(wA, wB, off(6), off(7), cs, 7);
            tap_body(wB, wA, off(7), off(8), cs, 8);
            tap_body(wA, wB, off(8), off(8), cs1, 0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) wA[ks] = wB[ks];
        } else {
            int r = 0, s = 0;
            for (int tap = 0; tap < RS; ++tap) {
                const bool last = tap + 1 == RS;
                int s1 = s + 1, r1 = r;
                if (s1 == g.S) { s1 = 0; r1 = r + 1; }
                const int tapoff = (r * a.RW + s) * PITCH;
                const int tapoff1 = last ? tapoff : (r1 * a.RW + s1) * PITCH;  // after the last tap the read is discarded
                tap_body(wA, wB, tapoff, tapoff1, last ? cs1 : cs, last ? 0 : tap + 1);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) wA[ks] = wB[ks];
                r = r1;
                s = s1;
            }
        }
        __builtin_amdgcn_s_setprio(0);
    }

    // ---- epilogue: bias / ReLU / bf16, transposed through LDS (the patch is dead) so that every global store is 16
    // contiguous bytes per lane; the whole 256 x 64 tile is staged in one pass (staged row = tile pixel index) ----
    constexpr int OPITCH = BN * 2 + 16;  // bytes per pixel row in the staging buffer
    constexpr int VPR = BN / 8;          // 16-byte vectors per pixel row
    constexpr int RPP = NT / VPR;        // pixel rows stored per pass
    static_assert(BM * OPITCH <= MAX_PATCH * PITCH, "the staged tile must fit the patch area");
    __syncthreads();  // the last readers of the patch are done
    // bias and ReLU are decided once for the whole tile (four straight-line variants), not per register group
    auto stage_tile = [&](auto bias_tag, auto relu_tag) {
        constexpr bool BIAS = decltype(bias_tag)::value, RELU = decltype(relu_tag)::value;
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const int srow = (pg * FM + j) * 32 + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int nl = cg * 32 + q * 8 + (lane >> 5) * 4;  // channel
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[j][q * 4 + e];
                if (BIAS) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] += a.bias[nl + e];
                }
                if (RELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                uint2 pk = make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                                      (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
                *reinterpret_cast<uint2*>(smem + srow * OPITCH + nl * 2) = pk;
            }
        }
    };
    if (a.bias) {
        if (a.relu) stage_tile(std::true_type{}, std::true_type{});
        else stage_tile(std::true_type{}, std::false_type{});
    } else {
        if (a.relu) stage_tile(std::false_type{}, std::true_type{});
        else stage_tile(std::false_type{}, std::false_type{});
    }
    __syncthreads();
    float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // column sums over this thread's rows (its 8 channels)
    if (a.out || a.colsum)  // (pooled output only: nothing to store per pixel)
    for (int row = tid / VPR; row < BM; row += RPP) {
        const int m = (img * g.OH + oh0 + row / TW) * g.OW + ow0 + row % TW;
        u32x4 vv = *reinterpret_cast<const u32x4*>(smem + row * OPITCH + (tid % VPR) * 16);
        const size_t o = (size_t)m * BN + (tid % VPR) * 8;
        if (a.mask) vv = relu_mask8(vv, *reinterpret_cast<const u32x4*>(a.mask + o));
        if (a.out) *reinterpret_cast<u32x4*>(a.out + o) = vv;
        if (a.colsum) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                csum[2 * k] += __uint_as_float(vv[k] << 16);
                csum[2 * k + 1] += __uint_as_float(vv[k] & 0xffff0000u);
            }
        }
    }
    // ---- column sums of the stored tile (the bias gradient of the layer whose pre-activation gradient this is): the
    // RPP row groups are added in group order through LDS, one partial row per pixel tile; a second kernel adds the
    // tiles in a fixed order ----
    if (a.colsum) {
        __syncthreads();  // the staged tile has been read
        float* red = reinterpret_cast<float*>(smem);  // [RPP][BN]
#pragma unroll
        for (int e = 0; e < 8; ++e) red[(tid / VPR) * BN + (tid % VPR) * 8 + e] = csum[e];
        __syncthreads();
        if (tid < BN) {
            float t = red[tid];
            for (int k = 1; k < RPP; ++k) t += red[k * BN + tid];
            a.colsum[(size_t)tm * BN + tid] = t;
        }
    }
    // ---- fused 2x2 / stride-2 max-pool of the staged (bias / ReLU applied, bf16) tile: tile origin and size are
    // even, so every window is complete.  Same rule as maxpool_fwd_kernel: first maximum in (r, s) order. ----
    if (a.pool_y) {
        constexpr int PWT = TW / 2;  // pooled pixels per tile row
        for (int item = tid; item < (BM / 4) * VPR; item += NT) {
            const int pp = item / VPR, vec = item % VPR;
            const int py = pp / PWT, px = pp - py * PWT;
            const int idx00 = (2 * py) * TW + 2 * px;
            const int idx4[4] = {idx00, idx00 + 1, idx00 + TW, idx00 + TW + 1};
            unsigned short best[8];
            float bestf[8];
            unsigned char bi[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(smem + idx4[k] * OPITCH + vec * 16);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned short bits = (unsigned short)((e & 1) ? (v[e >> 1] >> 16) : (v[e >> 1] & 0xffffu));
                    const float f = __uint_as_float((unsigned)bits << 16);
                    if (k == 0 || f > bestf[e]) { bestf[e] = f; best[e] = bits; bi[e] = (unsigned char)k; }
                }
            }
            const size_t po = ((size_t)(img * (g.OH / 2) + oh0 / 2 + py) * (g.OW / 2) + ow0 / 2 + px) * BN + vec * 8;
            u32x4 yo = {(unsigned)best[0] | ((unsigned)best[1] << 16), (unsigned)best[2] | ((unsigned)best[3] << 16),
                        (unsigned)best[4] | ((unsigned)best[5] << 16), (unsigned)best[6] | ((unsigned)best[7] << 16)};
            *reinterpret_cast<u32x4*>(a.pool_y + po) = yo;
            uint2 am;
            am.x = bi[0] | (bi[1] << 8) | (bi[2] << 16) | ((unsigned)bi[3] << 24);
            am.y = bi[4] | (bi[5] << 8) | (bi[6] << 16) | ((unsigned)bi[7] << 24);
            *reinterpret_cast<uint2*>(a.pool_am + po) = am;
        }
    }
}

template <int TW, bool UP, bool T9>
int launch_t64(const T64Args& ta, hipStream_t st) {
    auto kfn = conv_tile64_kernel<TW, UP, T9>;
    constexpr size_t smem = (size_t)MAX_PATCH * PITCH;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(ta.tiles_m), dim3(NT), smem, st, ta);
    return check_launch("conv_tile64");
}

}  // namespace

// tile width (32, 16 or 8; the tile is 256 / width rows high) if this kernel serves the geometry, else 0
int tile64_width(const GemmGeom& g) {
    if (g.Ncols != 64 || (g.IC % BK) != 0 || g.div_h != 1 || g.div_w != 1 || g.mul_h != 1 || g.mul_w != 1) return 0;
    if (g.R * g.S < 2) return 0;
    long a_elems = (long)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * g.IC;
    if (a_elems * 2 >= (1L << 31)) return 0;
    for (int tw : {32, 16, 8}) {
        const int th = 256 / tw;
        if ((g.OH % th) == 0 && (g.OW % tw) == 0 && (th + g.R - 1) * (tw + g.S - 1) <= MAX_PATCH) return tw;
    }
    return 0;
}

const char* tile64_kernel_name(const GemmGeom& g, bool unpool) {
    static const char* names[2][2][3] = {
        {{"conv_tile64_kernel<32,false,false>", "conv_tile64_kernel<16,false,false>", "conv_tile64_kernel<8,false,false>"},
         {"conv_tile64_kernel<32,true,false>", "conv_tile64_kernel<16,true,false>", "conv_tile64_kernel<8,true,false>"}},
        {{"conv_tile64_kernel<32,false,true>", "conv_tile64_kernel<16,false,true>", "conv_tile64_kernel<8,false,true>"},
         {"conv_tile64_kernel<32,true,true>", "conv_tile64_kernel<16,true,true>", "conv_tile64_kernel<8,true,true>"}}};
    const int tw = tile64_width(g);
    return names[g.R == 3 && g.S == 3 ? 1 : 0][unpool ? 1 : 0][tw == 32 ? 0 : tw == 16 ? 1 : 2];
}

// can the patch loader take the input operand pooled (2x2 / stride 2, whole windows) plus the argmax?
bool tile64_fuses_unpool(const GemmGeom& g) {
    const int tw = tile64_width(g);
    if (!tw || (g.IH % 2) != 0 || (g.IW % 2) != 0) return false;
    const int th = 256 / tw;
    return ((th + g.R - 1) / 2 + 1) * ((tw + g.S - 1) / 2 + 1) <= 4 * (NT / 8);  // windows per patch: 4 per 8 threads
}

int launch_tile64(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                  hipStream_t st, const bf16_t* mask, bf16_t* pool_y, uint8_t* pool_am, const uint8_t* unpool_am,
                  float* colsum) {
    const int tw = tile64_width(g);
    if (!tw) return set_error(WAP_EINVAL, "internal: 64-channel tile kernel not applicable");
    if (unpool_am && !tile64_fuses_unpool(g))
        return set_error(WAP_EINVAL, "internal: fused max-pool backward not available for this shape");
    if ((pool_y || pool_am) && !(pool_y && pool_am)) return set_error(WAP_EINVAL, "internal: fused pooling needs both outputs");
    if (!out && !pool_y) return set_error(WAP_EINVAL, "internal: no output");
    const int th = 256 / tw;
    T64Args ta = {};
    ta.A = A;
    ta.Wp = reinterpret_cast<const bf16_t*>(Wp);
    ta.bias = bias;
    ta.mask = mask;
    ta.up_am = unpool_am;
    ta.out = out;
    ta.pool_y = pool_y;
    ta.pool_am = pool_am;
    ta.colsum = colsum;
    ta.g = g;
    ta.tiles_x = g.OW / tw;
    ta.tiles_img = ta.tiles_x * (g.OH / th);
    ta.tiles_m = ta.tiles_img * (g.M / (g.OH * g.OW));
    ta.RW = tw + g.S - 1;
    ta.patch_len = (th + g.R - 1) * ta.RW;
    ta.UW = (tw + g.S - 1) / 2 + 1;  // windows that can touch the patch: its first pixel may be the second of its window
    ta.units = ((th + g.R - 1) / 2 + 1) * ta.UW;
    ta.dUW = make_fastdiv((uint32_t)ta.UW);
    ta.relu = relu ? 1 : 0;
    ta.a_bytes = (unsigned)((size_t)(g.M / (g.OH * g.OW)) * g.IH * g.IW * g.IC * 2 / (unpool_am ? 4 : 1));
    ta.w_bytes = (unsigned)wreg_wt_bytes(g);
    ta.dTimg = make_fastdiv((uint32_t)ta.tiles_img);
    ta.dTx = make_fastdiv((uint32_t)ta.tiles_x);
    ta.dRW = make_fastdiv((uint32_t)ta.RW);
    const bool t9 = g.R == 3 && g.S == 3;
    if (unpool_am) {
        if (tw == 32) return t9 ? launch_t64<32, true, true>(ta, st) : launch_t64<32, true, false>(ta, st);
        if (tw == 16) return t9 ? launch_t64<16, true, true>(ta, st) : launch_t64<16, true, false>(ta, st);
        return t9 ? launch_t64<8, true, true>(ta, st) : launch_t64<8, true, false>(ta, st);
    }
    if (tw == 32) return t9 ? launch_t64<32, false, true>(ta, st) : launch_t64<32, false, false>(ta, st);
    if (tw == 16) return t9 ? launch_t64<16, false, true>(ta, st) : launch_t64<16, false, false>(ta, st);
    return t9 ? launch_t64<8, false, true>(ta, st) : launch_t64<8, false, false>(ta, st);
}

}  // namespace wap
