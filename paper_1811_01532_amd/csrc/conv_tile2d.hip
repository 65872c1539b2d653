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
// UP variant (data gradient of a layer followed by a 2x2 / stride-2 max-pool): the input operand arrives as
// the gradient of the POOLED output plus the pool's argmax; the patch loader routes each window's value to
// the pixel its argmax names, so the max-pool backward costs no pass over the full-size gradient.
// Serves the "primary" convolution nodes of Section 3.2.2 (forward and backward halves of t_c, Eq. 1).
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64, NT = 256;
constexpr int PITCH = (BK + 8) * 2;  // 144 bytes per padded pixel
constexpr int MAX_PATCH = 352;       // padded pixels (>= (tile h + R - 1) * (tile w + S - 1)); also the staging area
constexpr int MAX_PATCH_FLAT = 384;  // the same for flat (raster-order) tiles, which may straddle rows and images
constexpr int MAX_PATCH_FLAT64 = 512;  // flat 192-pixel x 64-channel tiles (5x5 filters on 27-wide maps, across images)
// LDS rows.  A 32-pixel fragment whose pixels wrap from one patch row to the next (flat tiles, 28-wide strips) reads
// LDS rows with a gap at the wrap; the 16 lanes a ds_read_b128 serves per cycle then no longer hit 16 distinct
// 16-byte bank groups (row r sits in group 9 r mod 16 at the 144-byte pitch) and the read takes ~7.4 instead of 4
// cycles.  Giving every patch row 16 surplus LDS rows (row stride = width + 16) makes the gap a multiple of 16 rows
// and the reads conflict-free again; the surplus rows are never read or written.  Two work-groups must still fit
// the CU's 160 KB, else the dense layout is used.
constexpr int LDS_ROWS_FLAT = 560;   // 2 x 560 x 144 B = 161280 B
constexpr int LDS_ROWS_STRIP = 448;  // 8 x 28 strips: (8 + R - 1) x (28 + 16)

struct TArgs {
    const bf16_t* A;
    const bf16_t* Wp;  // packed weights
    const float* bias;
    const bf16_t* mask;  // optional: out = mask > 0 ? out : 0
    const uint8_t* up_am;  // UP: argmax (r * 2 + s) per pooling window; A is then N x IH/2 x IW/2 x IC
    bf16_t* out;         // may be NULL when only the pooled output is wanted
    bf16_t* pool_y;      // optional (2-D 256-pixel tiles only): 2x2 / stride-2 max-pool of the output tile ...
    uint8_t* pool_am;    // ... and the position r*2+s of the first maximum of every window
    GemmGeom g;
    int tiles_x, tiles_y, tiles_img, tiles_m, tiles_n;
    int PWp, patch_len;  // LDS row stride of a patch row (>= RW), patch pixels to load (2-D tiles)
    int RW;              // patch row width in pixels: tile (flat tiles: image) width + S - 1
    FastDiv dRW, dRPHW;  // division by RW and (flat tiles) by PH * RW
    FastDiv dOW2;        // flat tiles with the fused pool: division by OW / 2
    int PH;              // flat tiles: padded image height
    int relu;
    unsigned a_bytes, w_bytes;
    FastDiv dTimg, dTx, dPWp;
    FastDiv dOHW, dOW, dPHW;  // flat tiles
    int UW, units;            // UP, 2-D tiles: pooling windows per patch row, windows per patch
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

// FN: 32-channel blocks per wavefront; TW: tile width in pixels; FM: 32-pixel fragments per wavefront;
// PG: wavefronts along the pixels (4 / PG along the channels).  Tile = 32*FM*PG pixels x 32*FN*(4/PG) channels.
// TW = 0: flat tiles, 32*FM*PG consecutive output pixels in raster order (they may straddle rows and images;
// the patch is then a run of the zero-padded image in raster order, as in conv_patch.hip).  UP: pooled input operand.
template <int FN, int TW, int FM, int PG, bool UP>
__global__ __launch_bounds__(NT, (FN * FM <= 4 && TW != 0 ? 3 : 2)) void conv_tile2d_kernel(const TArgs a) {
    constexpr bool FLAT = (TW == 0);
    constexpr int BM = 32 * FM * PG;
    constexpr int CG = 4 / PG;
    constexpr int TWD = FLAT ? 1 : TW;  // divisor that is never zero
    constexpr int TH = BM / TWD;
    static_assert(FLAT || TH * TW == BM, "tile width must divide the tile");
    // PATCH_ROWS: most patch pixels to load (sizes the per-thread vector list); LROWS: LDS rows behind them
    constexpr bool SPREAD = FLAT || TW == 28;  // fragments wrap patch rows: the LDS row stride may exceed the row width
    constexpr int PATCH_ROWS = FLAT ? (PG == 2 ? MAX_PATCH_FLAT64 : MAX_PATCH_FLAT) : MAX_PATCH;
    constexpr int LROWS = FLAT ? LDS_ROWS_FLAT : (TW == 28 ? LDS_ROWS_STRIP : MAX_PATCH);
    constexpr int PV = (PATCH_ROWS * 8 + NT - 1) / NT;  // 16-byte patch vectors per thread
    extern __shared__ __align__(16) unsigned char smem[];
    const GemmGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pg = wave % PG, cg = wave / PG;  // pixel group, channel group
    constexpr int BN = 32 * FN * CG;

    int logical = xcd_remap(blockIdx.x, a.tiles_m * a.tiles_n);
    const int tn = logical % a.tiles_n;
    const int tm = logical / a.tiles_n;
    const int img = (int)fdiv((uint32_t)tm, a.dTimg);
    const int trem = tm - img * a.tiles_img;
    const int tyi = (int)fdiv((uint32_t)trem, a.dTx);
    const int oh0 = tyi * TH, ow0 = (trem - tyi * a.tiles_x) * TW;
    const int n0 = tn * BN;
    // flat tiles: padded-flat index ((n * PH + oh) * PW + ow) of output pixel m at tap (0,0)
    const int OHW = g.OH * g.OW, PHW = a.PH * a.PWp;
    auto pflat = [&](int m) {
        int n = (int)fdiv((uint32_t)m, a.dOHW);
        int rem = m - n * OHW;
        int oh = (int)fdiv((uint32_t)rem, a.dOW);
        return n * PHW + oh * a.PWp + (rem - oh * g.OW);
    };
    const int m0 = tm * BM;
    const int m_last = (m0 + BM <= g.M ? m0 + BM : g.M) - 1;
    const int p_lo = FLAT ? pflat(m0) : 0;
    // the same in units of patch pixels (rows RW wide): what is loaded
    const int RPHW = a.PH * a.RW;
    auto rflat = [&](int m) {
        int n = (int)fdiv((uint32_t)m, a.dOHW);
        int rem = m - n * OHW;
        int oh = (int)fdiv((uint32_t)rem, a.dOW);
        return n * RPHW + oh * a.RW + (rem - oh * g.OW);
    };
    const int r_lo = FLAT ? rflat(m0) : 0;
    const int patch_len = FLAT ? rflat(m_last) + (g.R - 1) * a.RW + (g.S - 1) + 1 - r_lo : a.patch_len;
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

    // ---- patch vectors of this thread: byte offset of (padded pixel, 8-channel vector) or OOB.  UP: the offset is
    // that of the pixel's pooling window in the pooled tensor (the argmax byte sits at half of it), and pvcode holds
    // the pixel's position (ih % 2) * 2 + iw % 2 inside the window, 2 bits per vector ----
    constexpr bool UNITS = UP && !FLAT;  // 2-D tiles: a thread fetches whole pooling windows instead (below)
    unsigned pvoff[UNITS ? 1 : PV];
    int plrow[(SPREAD && !UNITS) ? PV : 1];  // LDS row of each vector's pixel (-1: none); dense layouts use the index itself
    unsigned pvcode = 0;
#pragma unroll
    for (int i = 0; i < (UNITS ? 0 : PV); ++i) {
        int v = tid + i * NT;
        int q = v >> 3;
        unsigned off = OOB;
        if (SPREAD) plrow[i] = -1;
        if (q < patch_len) {
            if (FLAT) {
                int p = r_lo + q;
                int n = (int)fdiv((uint32_t)p, a.dRPHW);
                int rem = p - n * RPHW;
                int vh = (int)fdiv((uint32_t)rem, a.dRW);
                int pxp = rem - vh * a.RW;
                int ih = vh - g.pad_h, iw = pxp - g.pad_w;
                plrow[i] = n * PHW + vh * a.PWp + pxp - p_lo;
                if (n * OHW < g.M && (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW) {
                    if (UP) {
                        off = (unsigned)(((n * IH2 + (ih >> 1)) * IW2 + (iw >> 1)) * g.IC + (v & 7) * 8) * 2u;
                        pvcode |= (unsigned)(((ih & 1) << 1) | (iw & 1)) << (2 * i);
                    } else {
                        off = (unsigned)(((n * g.IH + ih) * g.IW + iw) * g.IC + (v & 7) * 8) * 2u;
                    }
                }
            } else {
                int py = (int)fdiv((uint32_t)q, a.dRW);
                int px = q - py * a.RW;
                int ih = oh0 - g.pad_h + py, iw = ow0 - g.pad_w + px;
                if (SPREAD) plrow[i] = py * a.PWp + px;
                if ((unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW) {
                    if (UP) {
                        off = (unsigned)(((img * IH2 + (ih >> 1)) * IW2 + (iw >> 1)) * g.IC + (v & 7) * 8) * 2u;
                        pvcode |= (unsigned)(((ih & 1) << 1) | (iw & 1)) << (2 * i);
                    } else {
                        off = (unsigned)(((img * g.IH + ih) * g.IW + iw) * g.IC + (v & 7) * 8) * 2u;
                    }
                }
            }
        }
        pvoff[i] = off;
    }

    // ---- UP, 2-D tiles: window `unit` = thread index / 8 (+ 32 per round) of the (UH x UW) windows that touch the
    // patch; one 16-byte load of the pooled gradient and one 8-byte load of the argmax serve its four pixels.
    // uq0 = patch row of the window's top-left pixel (it may lie one row / column outside the patch), uval = which of
    // the four pixels are inside the patch, 4 bits per window ----
    constexpr int UPV = 4;
    unsigned uoff[UNITS ? UPV : 1];
    int uq0[UNITS ? UPV : 1];
    unsigned uval = 0;
    if (UNITS) {
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
            uq0[i] = py * a.PWp + px;
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
        if (FLAT) {
            const int m = m0 + idx <= m_last ? m0 + idx : m_last;  // tile tail: computed on a valid pixel, never stored
            frow[j] = (pflat(m) - p_lo) * PITCH + (lane >> 5) * 16;
        } else {
            frow[j] = ((idx / TWD) * a.PWp + (idx % TWD)) * PITCH + (lane >> 5) * 16;
        }
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
        if (UNITS) {
            u32x4 rp[UPV];
            u32x2 ra[UPV];  // the out-of-range offset halves to one that is still past the (half as long) argmax tensor
            const unsigned coff = (unsigned)(cs * BK) * 2u;
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
                        *reinterpret_cast<u32x4*>(smem + (uq0[i] + (pos >> 1) * a.PWp + (pos & 1)) * PITCH + (tid & 7) * 16) =
                            unpool_select8(rp[i], ra[i], (unsigned)pos);
        } else {
            u32x4 rp[PV];
            const unsigned coff = (unsigned)(cs * BK) * 2u;
#pragma unroll
            for (int i = 0; i < PV; ++i) rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, pvoff[i] + coff, 0, 0);
            if (UP) {
                u32x2 ra[PV];  // the out-of-range offset halves to one that is still past the (half as long) argmax tensor
#pragma unroll
                for (int i = 0; i < PV; ++i) ra[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrcM, (pvoff[i] + coff) >> 1, 0, 0);
#pragma unroll
                for (int i = 0; i < PV; ++i) rp[i] = unpool_select8(rp[i], ra[i], (pvcode >> (2 * i)) & 3u);
            }
            if (cs > 0) __syncthreads();  // every wavefront has finished reading the previous slice's patch
#pragma unroll
            for (int i = 0; i < PV; ++i) {
                int v = tid + i * NT;
                if (SPREAD) {
                    if (plrow[i] >= 0) *reinterpret_cast<u32x4*>(smem + plrow[i] * PITCH + (v & 7) * 16) = rp[i];
                } else if ((v >> 3) < PATCH_ROWS) {
                    *reinterpret_cast<u32x4*>(smem + (v >> 3) * PITCH + (v & 7) * 16) = rp[i];
                }
            }
        }
        __syncthreads();
        const int cs1 = cs + 1 < ncs ? cs + 1 : cs;
        // Fragment reads run one reduction step ahead of the MFMAs that consume them (two register sets), and the
        // issue order is pinned: with two or three wavefronts per SIMD the compiler's own order (read, wait, MFMA)
        // leaves the LDS latency exposed in front of most MFMAs.
        bf16x8 fa[2][FM];
#pragma unroll
        for (int j = 0; j < FM; ++j) fa[0][j] = *reinterpret_cast<const bf16x8*>(smem + frow[j]);
        __builtin_amdgcn_s_setprio(1);
        int r = 0, s = 0;
        for (int tap = 0; tap < RS; ++tap) {
            const bool last = tap + 1 == RS;
            int s1 = s + 1, r1 = r;
            if (s1 == g.S) { s1 = 0; r1 = r + 1; }
            const int tapoff = (r * a.PWp + s) * PITCH;
            const int tapoff1 = last ? tapoff : (r1 * a.PWp + s1) * PITCH;  // after the last tap the read is discarded
            __builtin_amdgcn_sched_barrier(0);
            load_w(last ? cs1 : cs, last ? 0 : tap + 1, wB);  // one reduction tile ahead (clamped at the very end)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int j = 0; j < FM; ++j)
                    fa[(ks + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(
                        smem + frow[j] + (ks < 3 ? tapoff + (ks + 1) * 32 : tapoff1));
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int i = 0; i < FN; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wA[ks][i], fa[ks & 1][j], acc[i][j], 0, 0, 0);
            }
            // issue order: the 4*FN weight loads ride on the first MFMAs, then one fragment read per FN MFMAs
            constexpr int NW = 4 * FN < 4 * FM ? 4 * FN : 4 * FM;
#pragma unroll
            for (int q = 0; q < NW; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
                __builtin_amdgcn_sched_group_barrier(0x008, FN, 0);  // MFMA
            }
#pragma unroll
            for (int q = 0; q < 4 * FM - NW; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, FN, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < FN; ++i) wA[ks][i] = wB[ks][i];
            r = r1;
            s = s1;
        }
        __builtin_amdgcn_s_setprio(0);
    }

    // ---- epilogue: bias / ReLU / bf16, transposed through LDS (the patch is dead) so that every global store
    // is 16 contiguous bytes per lane and a tile row of 32 pixels is one contiguous run ----
    constexpr int OPITCH = BN * 2 + 16;  // bytes per pixel row in the staging buffer
    constexpr int VPR = BN / 8;          // 16-byte vectors per pixel row
    constexpr int RPP = NT / VPR;        // pixel rows stored per pass
    // fragments of every pixel group staged per pass: as many as fit the (dead) patch area
    constexpr int JFIT = (LROWS * PITCH) / (OPITCH * 32 * PG);
    constexpr int JN = JFIT < FM ? JFIT : FM;
    constexpr int HROWS = PG * JN * 32;
    static_assert(JN >= 1, "staging area too small");
    static_assert(TW != 28 || JN == FM, "the strip tile must be staged in one pass (the fused pool relies on it)");
    static_assert(!(FLAT && PG == 1 && FM == 7) || JN == FM, "the flat 224-pixel tile must be staged in one pass");
#pragma unroll
    for (int half = 0; half < (FM + JN - 1) / JN; ++half) {
        __syncthreads();  // previous readers of the staging area (or of the patch) are done
#pragma unroll
        for (int jj = 0; jj < JN; ++jj) {
            const int j = half * JN + jj;
            if (j >= FM) continue;
            const int srow = (pg * JN + jj) * 32 + (lane & 31);
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
            // staged row -> (pixel group, fragment of this pass, pixel) -> tile pixel
            const int j = half * JN + (row % (JN * 32)) / 32;
            if (j >= FM) continue;
            const int idx = ((row / (JN * 32)) * FM + j) * 32 + (row & 31);
            const int m = FLAT ? m0 + idx : (img * g.OH + oh0 + idx / TWD) * g.OW + ow0 + idx % TWD;
            if (FLAT && m > m_last) continue;
            u32x4 vv = *reinterpret_cast<const u32x4*>(smem + row * OPITCH + (tid % VPR) * 16);
            const size_t o = (size_t)m * g.Ncols + n0 + (tid % VPR) * 8;
            if (a.mask) vv = relu_mask8(vv, *reinterpret_cast<const u32x4*>(a.mask + o));
            if (a.out) *reinterpret_cast<u32x4*>(a.out + o) = vv;
        }
        // ---- fused 2x2 / stride-2 max-pool of the staged (bias / ReLU applied, bf16) tile: tile origin and size
        // are even, and both rows of a window are staged in the same pass (a 32-pixel fragment holds whole tile
        // rows and passes hold fragment pairs).  Same rule as maxpool_fwd_kernel: first maximum in (r, s) order. ----
        // The 8 x 28 strips and the flat 224-pixel tiles stage their whole tile in one pass (JN == FM), so every window
        // is complete there as well; a flat tile is then a whole number of row pairs (the host checks 224 % (2 OW) == 0
        // and even map sizes), possibly of two images.
        constexpr bool POOLS = FLAT ? (PG == 1 && JN == FM) : ((PG == 2 && FM == 4) || (TW == 28 && JN == FM));
        if (POOLS && a.pool_y) {
            const int roww = FLAT ? g.OW : TWD;  // pixels per tile row
            const int PWT = roww >> 1;           // pooled pixels per tile row
            auto srow_of = [&](int idx) {
                const int f = idx >> 5;
                return ((f / FM) * JN + (f % FM) - half * JN) * 32 + (idx & 31);
            };
            for (int item = tid; item < (BM / 4) * VPR; item += NT) {
                const int pp = item / VPR, vec = item % VPR;
                const int py = FLAT ? (int)fdiv((uint32_t)pp, a.dOW2) : pp / (TWD / 2);
                const int px = pp - py * PWT;
                const int idx00 = (2 * py) * roww + 2 * px;
                if ((((idx00 >> 5) % FM) / JN) != half) continue;  // window staged in the other pass
                if (FLAT && m0 + idx00 + roww + 1 > m_last) continue;  // beyond the last pixel of the layer
                const int idx4[4] = {idx00, idx00 + 1, idx00 + roww, idx00 + roww + 1};
                unsigned short best[8];
                float bestf[8];
                unsigned char bi[8];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(smem + srow_of(idx4[k]) * OPITCH + vec * 16);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const unsigned short bits = (unsigned short)((e & 1) ? (v[e >> 1] >> 16) : (v[e >> 1] & 0xffffu));
                        const float f = __uint_as_float((unsigned)bits << 16);
                        if (k == 0 || f > bestf[e]) { bestf[e] = f; best[e] = bits; bi[e] = (unsigned char)k; }
                    }
                }
                size_t po;
                if (FLAT) {
                    const int m = m0 + idx00;
                    const int n = (int)fdiv((uint32_t)m, a.dOHW);
                    const int rem = m - n * OHW;
                    const int oh = (int)fdiv((uint32_t)rem, a.dOW), ow = rem - oh * g.OW;
                    po = ((size_t)(n * (g.OH / 2) + oh / 2) * (g.OW / 2) + ow / 2) * g.Ncols + n0 + vec * 8;
                } else {
                    po = ((size_t)(img * (g.OH / 2) + oh0 / 2 + py) * (g.OW / 2) + ow0 / 2 + px) * g.Ncols + n0 + vec * 8;
                }
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
}

template <int FN, int TW, int FM, int PG, bool UP>
int launch_tile2d_u(const TArgs& ta, hipStream_t st) {
    auto kfn = conv_tile2d_kernel<FN, TW, FM, PG, UP>;
    constexpr size_t smem = (size_t)(TW == 0 ? LDS_ROWS_FLAT : (TW == 28 ? LDS_ROWS_STRIP : MAX_PATCH)) * PITCH;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(ta.tiles_m * ta.tiles_n), dim3(NT), smem, st, ta);
    return check_launch("conv_tile2d");
}
template <int FN, int TW, int FM, int PG>
int launch_tile2d_t(const TArgs& ta, hipStream_t st) {
    return ta.up_am ? launch_tile2d_u<FN, TW, FM, PG, true>(ta, st) : launch_tile2d_u<FN, TW, FM, PG, false>(ta, st);
}

}  // namespace

namespace {
struct TileCfg {
    int fn, tw, th, variant;  // variant 0: 256 pixels as 2 x 4 fragments; 1: 224 pixels (8 x 28) as 1 x 7 fragments,
                              // 128 channels; 2: the same with flat tiles (224 consecutive pixels); 3: flat tiles of
                              // 192 pixels x 64 channels (2 x 3 fragments) for thin outputs on maps no 2-D tile divides
};
// largest flat patch (in rows of the given stride; 0: the dense width) any bm-pixel raster-order tile of this geometry needs
int max_flat_patch(const GemmGeom& g, int bm, int stride = 0) {
    const int PH = g.OH + g.R - 1, PW = stride > 0 ? stride : g.OW + g.S - 1;
    const long OHW = (long)g.OH * g.OW;
    auto pflat = [&](long m) {
        long n = m / OHW, rem = m - n * OHW;
        long oh = rem / g.OW, ow = rem - oh * g.OW;
        return n * PH * PW + oh * PW + ow;
    };
    long worst = 0;
    for (long m0 = 0; m0 < g.M; m0 += bm) {
        long ml = (m0 + bm <= g.M ? m0 + bm : g.M) - 1;
        long len = pflat(ml) + (long)(g.R - 1) * PW + (g.S - 1) + 1 - pflat(m0);
        if (len > worst) worst = len;
    }
    return (int)worst;
}
// Wide outputs at a small minibatch: the 128-channel tiles leave most CUs without work and conv_patch.hip does not
// apply, so the alternative is the generic tap-by-tap kernel with a split reduction (measured 270-390 TFLOP/s there,
// plus ~9 us for the launch of its reduction epilogue).  One 192 x 64 tile's serial reduction loop takes 5.4-6.6 us
// per 64-channel slice of a 3x3 filter whatever the minibatch, so the flat tiles win only once the layer holds
// enough work.
bool flat64_wins_small_batch(const GemmGeom& g) {
    if ((g.Ncols % 64) != 0 || g.Ncols <= 64 || g.M >= 224 * 32 || g.M < 192 * 4) return false;
    if ((long)((g.M + 191) / 192) * (g.Ncols / 64) < 64) return false;
    if (max_flat_patch(g, 192) > MAX_PATCH_FLAT64) return false;
    const double flops = 2.0 * g.M * (double)g.Ncols * g.Kred;
    const double t_generic = flops / 330e12 + 9e-6;
    const double floor_s = 5.5e-6 * (g.IC / 64) * (g.R * g.S / 9.0);
    const double t_flat = floor_s > flops / 900e12 ? floor_s : flops / 900e12;
    return t_flat < 0.85 * t_generic;
}
// Tile shape for this geometry (width must divide the map, patch must fit), fn = 0 if none.
TileCfg tile_cfg(const GemmGeom& g) {
    TileCfg c = {0, 0, 0, 0};
    if ((g.Ncols % 64) != 0) return c;
    const bool tiles128 = g.Ncols == 64 || (g.Ncols % 128) == 0;  // 2-D tiles: 64 channels, or 128-channel tiles
    for (int tw : {32, 16, 8}) {
        const int th = 256 / tw;
        if (tiles128 && (g.OH % th) == 0 && (g.OW % tw) == 0 && (th + g.R - 1) * (tw + g.S - 1) <= MAX_PATCH) {
            c = {g.Ncols == 64 ? 1 : 2, tw, th, 0};
            return c;
        }
    }
    // maps of 28k x 8j pixels (56 x 56): 8 x 28 tiles, one 224-pixel strip per wavefront, 128-channel tiles
    if ((g.Ncols % 128) == 0 && (g.OW % 28) == 0 && (g.OH % 8) == 0 && (8 + g.R - 1) * (28 + g.S - 1) <= MAX_PATCH)
        c = {1, 28, 8, 1};
    else if ((g.Ncols % 128) == 0 && g.M >= 224 * 4 && max_flat_patch(g, 224) <= MAX_PATCH_FLAT)
        c = {1, 0, 0, 2};
    // 192-pixel x 64-channel flat tiles where none of the above applies (64 or 192 output channels on maps no 2-D
    // tile divides), and for wide outputs at a small minibatch where they beat the generic kernel
    if (c.fn == 0 && g.M >= 192 * 4 && max_flat_patch(g, 192) <= MAX_PATCH_FLAT64) c = {1, 0, 0, 3};
    if (c.fn != 0 && c.variant >= 1 && c.variant <= 2 &&
        (long)((g.M + 223) / 224) * (g.Ncols / 128) < kNumCU * 3 / 4 && flat64_wins_small_batch(g))
        c = {1, 0, 0, 3};
    return c;
}
}  // namespace

// 0 = not applicable, otherwise FN (32-channel blocks per wavefront)
int tile2d_supported(const GemmGeom& g) {
    if ((g.IC % BK) != 0 || g.div_h != 1 || g.div_w != 1 || g.mul_h != 1 || g.mul_w != 1) return 0;
    if (g.R * g.S < 2) return 0;
    long a_elems = (long)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * g.IC;
    if (a_elems * 2 >= (1L << 31)) return 0;
    return tile_cfg(g).fn;
}

// Shapes on which this kernel measured faster than conv_patch.hip: thin outputs on 256-pixel 2-D tiles, and the
// 224-pixel x 128-channel tiles (8 x 28 strips or flat) at any width once the map is large enough to fill the CUs.
bool tile2d_preferred(const GemmGeom& g) {
    if (!tile2d_supported(g)) return false;
    const TileCfg c = tile_cfg(g);
    if (c.variant == 0) return g.Ncols <= 128;
    if (c.variant == 3) {  // measured against the generic tap-by-tap kernel (64 channels) and conv_patch (wider)
        const long t3 = (long)((g.M + 191) / 192) * (g.Ncols / 64);
        return g.Ncols == 64 ? t3 >= 48 : (t3 >= 200 || flat64_wins_small_batch(g));
    }
    return (long)((g.M + 223) / 224) * (g.Ncols / 128) >= kNumCU * 3 / 4;
}

const char* tile2d_kernel_name(const GemmGeom& g, bool unpool) {
    const TileCfg c = tile_cfg(g);
    const int u = unpool ? 1 : 0;
    static const char* n1[2] = {"conv_tile2d_kernel<1,28,7,1,false>", "conv_tile2d_kernel<1,28,7,1,true>"};
    static const char* n2[2] = {"conv_tile2d_kernel<1,0,7,1,false>", "conv_tile2d_kernel<1,0,7,1,true>"};
    static const char* n3[2] = {"conv_tile2d_kernel<1,0,3,2,false>", "conv_tile2d_kernel<1,0,3,2,true>"};
    if (c.variant == 1) return n1[u];
    if (c.variant == 2) return n2[u];
    if (c.variant == 3) return n3[u];
    static const char* names[2][2][3] = {
        {{"conv_tile2d_kernel<1,32,4,2,false>", "conv_tile2d_kernel<1,16,4,2,false>", "conv_tile2d_kernel<1,8,4,2,false>"},
         {"conv_tile2d_kernel<2,32,4,2,false>", "conv_tile2d_kernel<2,16,4,2,false>", "conv_tile2d_kernel<2,8,4,2,false>"}},
        {{"conv_tile2d_kernel<1,32,4,2,true>", "conv_tile2d_kernel<1,16,4,2,true>", "conv_tile2d_kernel<1,8,4,2,true>"},
         {"conv_tile2d_kernel<2,32,4,2,true>", "conv_tile2d_kernel<2,16,4,2,true>", "conv_tile2d_kernel<2,8,4,2,true>"}}};
    return names[u][c.fn == 2 ? 1 : 0][c.tw == 32 ? 0 : c.tw == 16 ? 1 : 2];
}

// can the patch loader take the input operand pooled (2x2 / stride 2, whole windows) plus the argmax?
bool tile2d_fuses_unpool(const GemmGeom& g) {
    if (!tile2d_supported(g) || (g.IH % 2) != 0 || (g.IW % 2) != 0) return false;
    const TileCfg c = tile_cfg(g);
    if (c.variant >= 2) return true;
    return ((c.th + g.R - 1) / 2 + 1) * ((c.tw + g.S - 1) / 2 + 1) <= 4 * (NT / 8);  // windows per patch: 4 per 8 threads
}

// can the epilogue also emit the 2x2 / stride-2 max-pool of the output?
bool tile2d_fuses_pool(const GemmGeom& g) {
    if (!tile2d_supported(g)) return false;
    const TileCfg c = tile_cfg(g);  // even tile origin and size, whole windows per staging pass
    if (c.variant == 0 || c.variant == 1) return true;  // strips stage the whole 224 x 128 tile in one pass
    // flat 224 x 128 tiles: whole row pairs per tile
    return c.variant == 2 && (g.OH % 2) == 0 && (g.OW % 2) == 0 && (224 % (2 * g.OW)) == 0;
}

int launch_tile2d(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                  hipStream_t st, const bf16_t* mask, bf16_t* pool_y, uint8_t* pool_am, const uint8_t* unpool_am) {
    TArgs ta = {};
    ta.mask = mask;
    if (unpool_am && !tile2d_fuses_unpool(g))
        return set_error(WAP_EINVAL, "internal: fused max-pool backward not available for this shape");
    ta.up_am = unpool_am;
    if ((pool_y || pool_am) && !(pool_y && pool_am && tile2d_fuses_pool(g)))
        return set_error(WAP_EINVAL, "internal: fused pooling not available for this shape");
    if (!out && !pool_y) return set_error(WAP_EINVAL, "internal: no output");
    ta.pool_y = pool_y;
    ta.pool_am = pool_am;
    if (!tile2d_supported(g)) return set_error(WAP_EINVAL, "internal: 2-D tile kernel not applicable");
    const TileCfg c = tile_cfg(g);
    const int fn = c.fn;
    ta.A = A;
    ta.Wp = reinterpret_cast<const bf16_t*>(Wp);
    ta.bias = bias;
    ta.out = out;
    ta.g = g;
    ta.tiles_n = c.variant == 3 ? g.Ncols / 64 : c.variant >= 1 ? g.Ncols / 128 : g.Ncols / (64 * fn);
    if (c.variant >= 2) {
        const int bm = c.variant == 3 ? 192 : 224;
        ta.tiles_x = ta.tiles_y = ta.tiles_img = 1;
        ta.tiles_m = (g.M + bm - 1) / bm;
        ta.PH = g.OH + g.R - 1;
        ta.RW = g.OW + g.S - 1;
        ta.PWp = ta.RW;
        if (g.S - 1 <= 16 && max_flat_patch(g, bm, g.OW + 16) <= LDS_ROWS_FLAT) ta.PWp = g.OW + 16;  // conflict-free stride
        ta.dRPHW = make_fastdiv((uint32_t)(ta.PH * ta.RW));
        ta.patch_len = 0;  // per tile, computed in the kernel
        ta.dOHW = make_fastdiv((uint32_t)(g.OH * g.OW));
        ta.dOW = make_fastdiv((uint32_t)g.OW);
        ta.dOW2 = make_fastdiv((uint32_t)(g.OW / 2 > 0 ? g.OW / 2 : 1));
        ta.dPHW = make_fastdiv((uint32_t)(ta.PH * ta.PWp));
    } else {
        ta.tiles_x = g.OW / c.tw;
        ta.tiles_y = g.OH / c.th;
        ta.tiles_img = ta.tiles_x * ta.tiles_y;
        ta.tiles_m = ta.tiles_img * (g.M / (g.OH * g.OW));
        ta.RW = c.tw + g.S - 1;
        ta.PWp = ta.RW;
        if (c.variant == 1 && g.S - 1 <= 16 && (c.th + g.R - 1) * (c.tw + 16) <= LDS_ROWS_STRIP) ta.PWp = c.tw + 16;
        ta.patch_len = (c.th + g.R - 1) * ta.RW;
        // windows that can touch the patch: its first pixel may be the second of its window
        ta.UW = (c.tw + g.S - 1) / 2 + 1;
        ta.units = ((c.th + g.R - 1) / 2 + 1) * ta.UW;
        ta.dUW = make_fastdiv((uint32_t)ta.UW);
    }
    ta.relu = relu ? 1 : 0;
    ta.a_bytes = (unsigned)((size_t)(g.M / (g.OH * g.OW)) * g.IH * g.IW * g.IC * 2 / (unpool_am ? 4 : 1));
    ta.w_bytes = (unsigned)wreg_wt_bytes(g);
    ta.dTimg = make_fastdiv((uint32_t)ta.tiles_img);
    ta.dTx = make_fastdiv((uint32_t)ta.tiles_x);
    ta.dPWp = make_fastdiv((uint32_t)ta.PWp);
    ta.dRW = make_fastdiv((uint32_t)ta.RW);
    if (c.variant == 1) return launch_tile2d_t<1, 28, 7, 1>(ta, st);
    if (c.variant == 2) return launch_tile2d_t<1, 0, 7, 1>(ta, st);
    if (c.variant == 3) return launch_tile2d_t<1, 0, 3, 2>(ta, st);
    const int TW = c.tw;
    if (TW == 32) return fn == 1 ? launch_tile2d_t<1, 32, 4, 2>(ta, st) : launch_tile2d_t<2, 32, 4, 2>(ta, st);
    if (TW == 16) return fn == 1 ? launch_tile2d_t<1, 16, 4, 2>(ta, st) : launch_tile2d_t<2, 16, 4, 2>(ta, st);
    return fn == 1 ? launch_tile2d_t<1, 8, 4, 2>(ta, st) : launch_tile2d_t<2, 8, 4, 2>(ta, st);
}

}  // namespace wap
