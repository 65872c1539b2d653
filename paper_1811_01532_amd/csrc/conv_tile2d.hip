// Stride-1 convolution (forward, and data gradient with flipped weights) with the input PATCH resident in LDS
// (gfx950): every VGG-16 layer but the first, and the 13 x 13 / 27 x 27 AlexNet-style layers.
//
// The zero-padded input patch of a work-group's pixel tile (tile plus halo) is written to LDS one 32-channel slice
// at a time and every filter tap reads it through a shifted pointer, so activations cross L2 -> LDS once instead of
// R*S times; weights go from their packed copy straight into MFMA operand registers, one tap ahead.
//   * tiles: 8 x 32 / 16 x 16 pixels of one image (4 wavefronts = 2 pixel halves x 2 channel halves, 64 or 128
//     channels), 8 x 28 strips and flat runs of 224 raster-order pixels x 128 channels (4 channel wavefronts; the
//     runs may straddle rows and images), flat 192 x 64 tiles for thin outputs on maps nothing else divides;
//   * the patch is DOUBLE buffered: the global loads of slice c+1 are issued when the MFMA loop of slice c starts,
//     sit in registers for half of the taps and are written to the other buffer in the middle of the loop.  One
//     barrier per slice, placed in front of the last fragment read of the slice (which already targets the other
//     buffer), so no wavefront ever waits for a load or store phase.  (Two resident work-groups per CU that started
//     together reach such phases together: nobody covers them.)
//   * a 32-channel slice keeps a buffer near 30 KB (80-byte pixel rows: 64 bytes of data and 16 of padding, so 16
//     consecutive rows fall into 16 distinct 16-byte bank groups) and the staging registers at 24;
//   * patch rows are laid out with a BYTE stride chosen so that the first pixel of the next patch row lands in the
//     bank group that the pixel after this row's last tile pixel would have had (row stride = tile width x 80 plus a
//     multiple of 256 bytes): fragments that wrap from one patch row to the next still read conflict-free.
// UP variant (data gradient of a layer followed by a 2x2 / stride-2 max-pool): the input operand arrives as
// the gradient of the POOLED output plus the pool's argmax; the patch loader routes each window's value to
// the pixel its argmax names, so the max-pool backward costs no pass over the full-size gradient.
// Serves the "primary" convolution nodes of Section 3.2.2 (forward and backward halves of t_c, Eq. 1).
#include <algorithm>
#include <type_traits>

#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 32, NT = 256;
constexpr int PITCH = 80;            // LDS bytes per padded pixel: 32 channels + 16 bytes
constexpr int VPP = BK / 8;          // 16-byte vectors per patch pixel
constexpr int MAX_PATCH = 352;       // padded pixels per 2-D tile patch (>= (tile h + R - 1) * (tile w + S - 1))
constexpr int MAX_PATCH_FLAT = 384;  // the same for flat (raster-order) 224-pixel tiles, which may straddle rows and images
constexpr int MAX_PATCH_FLAT64 = 512;  // flat 192-pixel x 64-channel tiles (5x5 filters on 27-wide maps, across images)
constexpr size_t LDS_CAP = 160 * 1024;

struct TArgs {
    const bf16_t* A;
    const bf16_t* Wp;  // packed weights
    const float* bias;
    const bf16_t* mask;  // optional: out = mask > 0 ? out : 0
    const uint8_t* up_am;  // UP: argmax (r * 2 + s) per pooling window; A is then N x IH/2 x IW/2 x IC
    bf16_t* out;         // may be NULL when only the pooled output is wanted
    bf16_t* pool_y;      // optional: 2x2 / stride-2 max-pool of the output tile ...
    uint8_t* pool_am;    // ... and the position r*2+s of the first maximum of every window
    float* colsum;       // optional: [tiles_m][Ncols] column sums of this tile's stored (masked) rows, for a bias gradient
    GemmGeom g;
    int tiles_x, tiles_y, tiles_img, tiles_m, tiles_n;
    int RWB, buf_bytes;  // LDS byte stride of a patch row, bytes of one patch buffer
    int patch_len;       // patch pixels to load (2-D tiles)
    int RW;              // patch row width in pixels: tile (flat tiles: image) width + S - 1
    FastDiv dRW, dRPHW;  // division by RW and (flat tiles) by PH * RW
    FastDiv dOW2;        // flat tiles with the fused pool: division by OW / 2
    int PH;              // flat tiles: padded image height
    int relu;
    unsigned a_bytes, w_bytes;
    FastDiv dTimg, dTx;
    FastDiv dOHW, dOW;   // flat tiles
    int UW, units;       // UP, 2-D tiles: pooling windows per patch row, windows per patch
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
// the patch is then a run of the zero-padded image in raster order).  UP: pooled input operand.
template <int FN, int TW, int FM, int PG, bool UP, bool T9>
__global__ __launch_bounds__(NT, 2) void conv_tile2d_kernel(const TArgs a) {
    constexpr bool FLAT = (TW == 0);
    constexpr int BM = 32 * FM * PG;
    constexpr int CG = 4 / PG;
    constexpr int TWD = FLAT ? 1 : TW;  // divisor that is never zero
    constexpr int TH = BM / TWD;
    static_assert(FLAT || TH * TW == BM, "tile width must divide the tile");
    constexpr int PATCH_ROWS = FLAT ? (PG == 2 ? MAX_PATCH_FLAT64 : MAX_PATCH_FLAT) : MAX_PATCH;  // most patch pixels
    constexpr int PV = (PATCH_ROWS * VPP + NT - 1) / NT;  // 16-byte patch vectors per thread
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
    const int OHW = g.OH * g.OW;
    // flat tiles: LDS byte position of output pixel m at tap (0,0) in the (unbounded) padded raster, rows RWB apart
    auto lbyte = [&](int m) {
        int n = (int)fdiv((uint32_t)m, a.dOHW);
        int rem = m - n * OHW;
        int oh = (int)fdiv((uint32_t)rem, a.dOW);
        return (n * a.PH + oh) * a.RWB + (rem - oh * g.OW) * PITCH;
    };
    const int m0 = tm * BM;
    const int m_last = (m0 + BM <= g.M ? m0 + BM : g.M) - 1;
    const int lds_lo = FLAT ? lbyte(m0) : 0;
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

    // ---- patch vectors of this thread: global byte offset of (padded pixel, 8-channel vector) or OOB, and the LDS
    // byte offset it goes to (-1: none, stored to the dump slot).  UP: the global offset is that of the pixel's pooling window in the pooled
    // tensor (the argmax byte sits at half of it), and pvcode holds the pixel's position (ih % 2) * 2 + iw % 2 inside
    // the window, 2 bits per vector ----
    constexpr bool UNITS = UP && !FLAT;  // 2-D tiles: a thread fetches whole pooling windows instead (below)
    unsigned pvoff[UNITS ? 1 : PV];
    int ploff[UNITS ? 1 : PV];
    unsigned pvcode = 0;
    // vectors with no patch pixel are stored unconditionally as well (no branches in the slice body), to a per-lane
    // slot behind the two buffers
    unsigned char* const dump = smem + 2 * a.buf_bytes + lane * 16;
#pragma unroll
    for (int i = 0; i < (UNITS ? 0 : PV); ++i) {
        int v = tid + i * NT;
        int q = v >> 2;
        unsigned off = OOB;
        ploff[i] = -1;
        if (q < patch_len) {
            if (FLAT) {
                int p = r_lo + q;
                int n = (int)fdiv((uint32_t)p, a.dRPHW);
                int rem = p - n * RPHW;
                int vh = (int)fdiv((uint32_t)rem, a.dRW);
                int pxp = rem - vh * a.RW;
                int ih = vh - g.pad_h, iw = pxp - g.pad_w;
                ploff[i] = (n * a.PH + vh) * a.RWB + pxp * PITCH - lds_lo + (v & 3) * 16;
                if (n * OHW < g.M && (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW) {
                    if (UP) {
                        off = (unsigned)(((n * IH2 + (ih >> 1)) * IW2 + (iw >> 1)) * g.IC + (v & 3) * 8) * 2u;
                        pvcode |= (unsigned)(((ih & 1) << 1) | (iw & 1)) << (2 * i);
                    } else {
                        off = (unsigned)(((n * g.IH + ih) * g.IW + iw) * g.IC + (v & 3) * 8) * 2u;
                    }
                }
            } else {
                int py = (int)fdiv((uint32_t)q, a.dRW);
                int px = q - py * a.RW;
                int ih = oh0 - g.pad_h + py, iw = ow0 - g.pad_w + px;
                ploff[i] = py * a.RWB + px * PITCH + (v & 3) * 16;
                if ((unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW)
                    off = (unsigned)(((img * g.IH + ih) * g.IW + iw) * g.IC + (v & 3) * 8) * 2u;
            }
        }
        pvoff[i] = off;
    }

    // ---- UP, 2-D tiles: window `unit` = thread index / 4 (+ 64 per round) of the (UH x UW) windows that touch the
    // patch; one 16-byte load of the pooled gradient and one 8-byte load of the argmax serve its four pixels.
    // uq0 = LDS byte offset of the window's top-left pixel (it may lie one row / column outside the patch), uval =
    // which of the four pixels are inside the patch, 4 bits per window ----
    constexpr int UPV = 2;
    unsigned uoff[UNITS ? UPV : 1];
    int uq0[UNITS ? UPV : 1];
    unsigned uval = 0;
    if (UNITS) {
        const int ihf = oh0 - g.pad_h, iwf = ow0 - g.pad_w;  // image coordinates of patch pixel (0, 0)
        const int wy0 = ihf >> 1, wx0 = iwf >> 1;            // its window (floor division also below zero)
        const int PHt = TH + g.R - 1;
#pragma unroll
        for (int i = 0; i < UPV; ++i) {
            const int unit = (tid >> 2) + i * (NT / 4);
            const int uy = (int)fdiv((uint32_t)unit, a.dUW), ux = unit - uy * a.UW;
            const int wy = wy0 + uy, wx = wx0 + ux;
            const int py = 2 * wy - ihf, px = 2 * wx - iwf;
            unsigned off = OOB;
            if (unit < a.units && (unsigned)wy < (unsigned)IH2 && (unsigned)wx < (unsigned)IW2)
                off = (unsigned)(((img * IH2 + wy) * IW2 + wx) * g.IC + (tid & 3) * 8) * 2u;
            uoff[i] = off;
            uq0[i] = py * a.RWB + px * PITCH + (tid & 3) * 16;
            if (unit < a.units) {
                const unsigned vy0 = py >= 0, vy1 = py + 1 < PHt, vx0 = px >= 0, vx1 = px + 1 < a.RW;
                uval |= ((vy0 & vx0) | ((vy0 & vx1) << 1) | ((vy1 & vx0) << 2) | ((vy1 & vx1) << 3)) << (4 * i);
            }
        }
    }

    // ---- fragment rows of this lane: fragment j holds tile pixels (pg * FM + j) * 32 .. + 31 in raster order ----
    int frow[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int idx = (pg * FM + j) * 32 + (lane & 31);
        if (FLAT) {
            const int m = m0 + idx <= m_last ? m0 + idx : m_last;  // tile tail: computed on a valid pixel, never stored
            frow[j] = lbyte(m) - lds_lo + (lane >> 5) * 16;
        } else {
            frow[j] = (idx / TWD) * a.RWB + (idx % TWD) * PITCH + (lane >> 5) * 16;
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
    auto load_w = [&](int cs, int tap, bf16x8 (&wd)[2][FN]) {
        const unsigned koff = ((unsigned)(tap * g.IC + cs * BK) / 16u) * 1024u;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < FN; ++i)
                wd[ks][i] = __builtin_bit_cast(
                    bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrcW, wrow[i] + koff + (unsigned)ks * 1024u, 0, 0));
    };

    // ---- patch slice: global -> registers (issue), registers -> LDS buffer (store) ----
    constexpr int NRP = UNITS ? UPV : PV;
    u32x4 rp[NRP];
    u32x2 ra[UP ? NRP : 1];  // an out-of-range offset halves to one that is still past the (half as long) argmax tensor
    auto issue_patch = [&](int cs) {
        const unsigned coff = (unsigned)(cs * BK) * 2u;
#pragma unroll
        for (int i = 0; i < NRP; ++i) {
            const unsigned o = (UNITS ? uoff[i] : pvoff[i]) + coff;
            rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, o, 0, 0);
            if (UP) ra[i] = __builtin_amdgcn_raw_buffer_load_b64(rsrcM, o >> 1, 0, 0);
        }
    };
    auto store_patch = [&](unsigned char* buf) {
        if (UNITS) {
#pragma unroll
            for (int i = 0; i < UPV; ++i)
#pragma unroll
                for (int pos = 0; pos < 4; ++pos)
                    *reinterpret_cast<u32x4*>(((uval >> (4 * i + pos)) & 1u)
                                                  ? buf + uq0[i] + (pos >> 1) * a.RWB + (pos & 1) * PITCH
                                                  : dump) = unpool_select8(rp[i], ra[i], (unsigned)pos);
        } else {
#pragma unroll
            for (int i = 0; i < PV; ++i)
                *reinterpret_cast<u32x4*>(ploff[i] >= 0 ? buf + ploff[i] : dump) =
                    UP ? unpool_select8(rp[i], ra[i], (pvcode >> (2 * i)) & 3u) : rp[i];
        }
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Weight fragments: one register set per tap (two reduction steps).  What bounds the weight stream is how long a
    // load may stay in flight before its wavefront needs it, and a wavefront's loads return in order, so the first
    // weight load issued after the patch loads of the next slice drags those along: with sets filled one tap ahead
    // the patch latency (first touch: HBM or the memory-side cache) would be exposed once per slice.
    //   T9 (3x3 filters, one channel block per wavefront): the nine taps of a slice are straight-line code, the sets
    //   a ring of three filled two taps ahead that rotates without copies, the patch loads go out right behind the
    //   weight loads of tap 0 (three taps until a younger weight load is needed) and reach LDS after tap 7.  No branch
    //   in the slice body: the loads / stores / barrier of a slice beyond the last are issued anyway (clamped to the
    //   last slice, written to the idle buffer), so the compiler's counter waits are exact.
    //   otherwise: a tap loop with two sets, the new one copied over the current one at the end of every tap.
    constexpr int NSET = T9 ? 3 : 2;
    bf16x8 w[NSET][2][FN];
    issue_patch(0);
#pragma unroll
    for (int u = 0; u + 1 < NSET; ++u) load_w(0, u, w[u]);
    store_patch(smem);
    __syncthreads();
    // Fragment reads run one reduction step ahead of the MFMAs that consume them, in place: right after the MFMA that
    // consumed fragment j has been issued, the read of fragment j for the next step is issued into the same registers
    // (FM - 1 MFMAs, some 200 cycles, before it is needed), across taps and across slices.  The issue order is pinned:
    // the compiler's own order (read, wait, MFMA) leaves the LDS latency exposed in front of most MFMAs.
    bf16x8 fa[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j) fa[j] = *reinterpret_cast<const bf16x8*>(smem + frow[j]);

    // one reduction step: consume fragment j with weight fragment wk, then fetch fragment j of the step after
    auto step = [&](bf16x8 (&wk)[FN], const unsigned char* next_base, int next_off, bool with_vmem) {
#pragma unroll
        for (int j = 0; j < FM; ++j) {
#pragma unroll
            for (int i = 0; i < FN; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wk[i], fa[j], acc[i][j], 0, 0, 0);
            fa[j] = *reinterpret_cast<const bf16x8*>(next_base + frow[j] + next_off);
        }
    };
    // issue order of a step: one fragment read behind every FN MFMAs; the step's VMEM loads (weights of a later tap,
    // the next patch slice) ride in front of the first MFMA groups, one or more per group (where they sit within the
    // step measured the same: first, third or fifth group)
    auto pin_step = [&](auto vmem_tag) {
        constexpr int NV = decltype(vmem_tag)::value;  // VMEM loads to place
        constexpr int PER = NV > 0 ? (NV + FM - 1) / FM : 0;
#pragma unroll
        for (int q = 0; q < FM; ++q) {
            if (NV > 0 && q * PER < NV) __builtin_amdgcn_sched_group_barrier(0x020, PER, 0);  // VMEM read
            __builtin_amdgcn_sched_group_barrier(0x008, FN, 0);                                // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                 // DS read
        }
    };

    for (int cs = 0; cs < ncs; ++cs) {
        const unsigned char* cur = smem + (cs & 1) * a.buf_bytes;
        unsigned char* nxt = smem + ((cs + 1) & 1) * a.buf_bytes;
        const int csn = cs + 1 < ncs ? cs + 1 : cs;  // the next slice, clamped
        __builtin_amdgcn_s_setprio(1);
        if constexpr (T9) {
            auto tap9 = [&](auto tap_tag) {
                constexpr int T = decltype(tap_tag)::value;
                constexpr int U = T % 3;
                constexpr int PT = (T + 2) % 9;           // the tap whose weights are fetched now
                const int tapoff = (T / 3) * a.RWB + (T % 3) * PITCH;
                const int tapoff1 = ((T + 1) / 3) * a.RWB + ((T + 1) % 3) * PITCH;
                __builtin_amdgcn_sched_barrier(0);
                load_w(T + 2 >= 9 ? csn : cs, PT, w[(U + 2) % 3]);
                if (T == 0) issue_patch(csn);
                step(w[U][0], cur, tapoff + 32, true);
                if (T == 0) pin_step(std::integral_constant<int, 2 * FN + (UP ? 2 : 1) * NRP>{});
                else pin_step(std::integral_constant<int, 2 * FN>{});
                __builtin_amdgcn_sched_barrier(0);
                if (T == 8) {
                    // every wavefront has written its share of the next slice (after tap 7; the LDS pipe executes a
                    // wavefront's operations in order and fragment reads issued after those writes have returned) and
                    // nobody reads the buffer that slice c+2 will overwrite before this point again
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_sched_barrier(0);
                    step(w[U][1], nxt, 0, false);
                } else {
                    step(w[U][1], cur, tapoff1, false);
                }
                pin_step(std::integral_constant<int, 0>{});
                __builtin_amdgcn_sched_barrier(0);
                if (T == 7) {
                    store_patch(nxt);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            tap9(std::integral_constant<int, 0>{});
            tap9(std::integral_constant<int, 1>{});
            tap9(std::integral_constant<int, 2>{});
            tap9(std::integral_constant<int, 3>{});
            tap9(std::integral_constant<int, 4>{});
            tap9(std::integral_constant<int, 5>{});
            tap9(std::integral_constant<int, 6>{});
            tap9(std::integral_constant<int, 7>{});
            tap9(std::integral_constant<int, 8>{});
        } else {
            const bool has_next = cs + 1 < ncs;
            if (has_next) issue_patch(cs + 1);
            const int mid = (RS - 1) >> 1;  // the tap after which the next slice goes to LDS (never the last tap)
            int r = 0, s2 = 0;
            // LAST: the slice's last tap, whose second step prefetches the first fragments of the next slice from the
            // other buffer, behind the slice's only barrier
            auto tap_body = [&](int tap, auto last_tag) {
                constexpr bool LAST = decltype(last_tag)::value;
                int s1 = s2 + 1, r1 = r;
                if (s1 == g.S) { s1 = 0; r1 = r + 1; }
                const int tapoff = r * a.RWB + s2 * PITCH;
                const int tapoff1 = r1 * a.RWB + s1 * PITCH;
                __builtin_amdgcn_sched_barrier(0);
                load_w(LAST ? csn : cs, LAST ? 0 : tap + 1, w[1]);  // (past the end: a harmless reload)
                step(w[0][0], cur, tapoff + 32, true);
                pin_step(std::integral_constant<int, 2 * FN>{});
                __builtin_amdgcn_sched_barrier(0);
                if (LAST) {
                    __builtin_amdgcn_s_barrier();  // see the note in the straight-line variant
                    __builtin_amdgcn_sched_barrier(0);
                    step(w[0][1], nxt, 0, false);
                } else {
                    step(w[0][1], cur, tapoff1, false);
                }
                pin_step(std::integral_constant<int, 0>{});
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int i = 0; i < FN; ++i) w[0][ks][i] = w[1][ks][i];
                r = r1;
                s2 = s1;
                if (!LAST && tap == mid && has_next) {
                    store_patch(nxt);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            for (int tap = 0; tap + 1 < RS; ++tap) tap_body(tap, std::false_type{});
            tap_body(RS - 1, std::true_type{});
        }
        __builtin_amdgcn_s_setprio(0);
    }

    // ---- epilogue: bias / ReLU / bf16, transposed through LDS (the patch buffers are dead) so that every global
    // store is 16 contiguous bytes per lane and a tile row of 32 pixels is one contiguous run.  The whole tile is
    // staged in one pass (the host sizes the LDS allocation for it): staged row = tile pixel index. ----
    constexpr int OPITCH = BN * 2 + 16;  // bytes per pixel row in the staging buffer
    constexpr int VPR = BN / 8;          // 16-byte vectors per pixel row
    constexpr int RPP = NT / VPR;        // pixel rows stored per pass
    __syncthreads();  // the last readers of the patch are done
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int srow = (pg * FM + j) * 32 + (lane & 31);
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
    float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // column sums over this thread's rows (its 8 channels)
    for (int row = tid / VPR; row < BM; row += RPP) {
        const int idx = row;
        const int m = FLAT ? m0 + idx : (img * g.OH + oh0 + idx / TWD) * g.OW + ow0 + idx % TWD;
        if (FLAT && m > m_last) continue;
        u32x4 vv = *reinterpret_cast<const u32x4*>(smem + row * OPITCH + (tid % VPR) * 16);
        const size_t o = (size_t)m * g.Ncols + n0 + (tid % VPR) * 8;
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
            a.colsum[(size_t)tm * g.Ncols + n0 + tid] = t;
        }
    }
    // ---- fused 2x2 / stride-2 max-pool of the staged (bias / ReLU applied, bf16) tile: tile origin and size are
    // even and the whole tile is staged, so every window is complete.  A flat tile is a whole number of row pairs
    // (the host checks 224 % (2 OW) == 0 and even map sizes), possibly of two images.  Same rule as maxpool_fwd_kernel:
    // first maximum in (r, s) order. ----
    constexpr bool POOLS = FLAT ? (PG == 1) : ((PG == 2 && FM == 4) || TW == 28);
    if (POOLS && a.pool_y) {
        const int roww = FLAT ? g.OW : TWD;  // pixels per tile row
        const int PWT = roww >> 1;           // pooled pixels per tile row
        for (int item = tid; item < (BM / 4) * VPR; item += NT) {
            const int pp = item / VPR, vec = item % VPR;
            const int py = FLAT ? (int)fdiv((uint32_t)pp, a.dOW2) : pp / (TWD / 2);
            const int px = pp - py * PWT;
            const int idx00 = (2 * py) * roww + 2 * px;
            if (FLAT && m0 + idx00 + roww + 1 > m_last) continue;  // beyond the last pixel of the layer
            const int idx4[4] = {idx00, idx00 + 1, idx00 + roww, idx00 + roww + 1};
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

template <int FN, int TW, int FM, int PG, bool UP, bool T9>
int launch_tile2d_w(const TArgs& ta, size_t smem, hipStream_t st) {
    auto kfn = conv_tile2d_kernel<FN, TW, FM, PG, UP, T9>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_CAP);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    hipLaunchKernelGGL(kfn, dim3(ta.tiles_m * ta.tiles_n), dim3(NT), smem, st, ta);
    return check_launch("conv_tile2d");
}
// straight-line 3x3 slices with the three-set weight ring for one-block wavefronts, else the tap loop
template <int FN, int TW, int FM, int PG, bool UP>
int launch_tile2d_u(const TArgs& ta, size_t smem, hipStream_t st) {
    constexpr bool CAN9 = true;
    if (CAN9 && ta.g.R == 3 && ta.g.S == 3) return launch_tile2d_w<FN, TW, FM, PG, UP, CAN9>(ta, smem, st);
    return launch_tile2d_w<FN, TW, FM, PG, UP, false>(ta, smem, st);
}
template <int FN, int TW, int FM, int PG>
int launch_tile2d_t(const TArgs& ta, size_t smem, hipStream_t st) {
    return ta.up_am ? launch_tile2d_u<FN, TW, FM, PG, true>(ta, smem, st) : launch_tile2d_u<FN, TW, FM, PG, false>(ta, smem, st);
}

}  // namespace

namespace {
struct TileCfg {
    int fn, tw, th, variant;  // variant 0: 256 pixels as 2 x 4 fragments; 1: 224 pixels (8 x 28) as 1 x 7 fragments,
                              // 128 channels; 2: the same with flat tiles (224 consecutive pixels); 3: flat tiles of
                              // 192 pixels x 64 channels (2 x 3 fragments) for thin outputs on maps no 2-D tile divides
    int RWB, buf_bytes;       // LDS layout: byte stride of a patch row, bytes of one patch buffer
    size_t smem;              // dynamic LDS of the launch: two patch buffers, or the staged output tile if larger
    int fm;                   // variant 2: 32-pixel fragments per wavefront (7 or 2: tiles of 224 or 64 pixels)
};
int tile_pixels(const TileCfg& c) { return c.variant == 3 ? 192 : c.variant == 2 ? 32 * c.fm : c.variant == 1 ? 224 : 256; }
// most patch pixels (rows of OW + S - 1) any bm-pixel raster-order tile of this geometry loads
int max_flat_patch(const GemmGeom& g, int bm) {
    const int PH = g.OH + g.R - 1, PW = g.OW + g.S - 1;
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
// most LDS bytes one patch buffer of such a tile spans when patch rows are rwb bytes apart
long max_flat_bytes(const GemmGeom& g, int bm, int rwb) {
    const int PH = g.OH + g.R - 1;
    const long OHW = (long)g.OH * g.OW;
    auto lbyte = [&](long m) {
        long n = m / OHW, rem = m - n * OHW;
        long oh = rem / g.OW, ow = rem - oh * g.OW;
        return (n * PH + oh) * rwb + ow * PITCH;
    };
    long worst = 0;
    for (long m0 = 0; m0 < g.M; m0 += bm) {
        long ml = (m0 + bm <= g.M ? m0 + bm : g.M) - 1;
        long len = lbyte(ml) + (long)(g.R - 1) * rwb + (long)(g.S - 1) * PITCH + PITCH - lbyte(m0);
        if (len > worst) worst = len;
    }
    return worst;
}
// Row stride that keeps fragments conflict-free across a row wrap: the next row's first pixel must fall into the bank
// group (address mod 256) that pixel `width` of this row would have had.
int conflict_free_stride(int width, int S) { return width * PITCH + ((S - 1) * PITCH + 255) / 256 * 256; }

// LDS layout of a tile shape: the conflict-free row stride if two work-groups per CU still fit, else dense rows.
bool lds_layout(const GemmGeom& g, TileCfg* c) {
    const int bm = tile_pixels(*c);
    const int bn = c->variant == 3 ? 64 : c->variant >= 1 ? 128 : 64 * c->fn;
    const size_t stage = (size_t)bm * (bn * 2 + 16);
    const bool flat = c->variant >= 2;
    const int width = flat ? g.OW : c->tw;
    const int dense = (width + g.S - 1) * PITCH;
    const int cands[2] = {(flat || (c->tw != 32)) ? conflict_free_stride(width, g.S) : dense, dense};
    size_t best = 0;
    for (int pass = 0; pass < 2 && !best; ++pass)            // first two work-groups per CU, then one
        for (int k = 0; k < 2 && !best; ++k) {
            const int rwb = cands[k];
            const long buf = flat ? max_flat_bytes(g, bm, rwb)
                                  : (long)(c->th + g.R - 2) * rwb + (long)(c->tw + g.S - 1) * PITCH;
            const long bufa = (buf + 15) / 16 * 16;
            const size_t smem = std::max((size_t)(2 * bufa) + 1024, stage);  // + the dump slots of stores without a pixel
            if (smem <= (pass == 0 ? LDS_CAP / 2 : LDS_CAP)) {
                c->RWB = rwb;
                c->buf_bytes = (int)bufa;
                c->smem = smem;
                best = smem;
            }
        }
    return best != 0;
}
// Wide outputs at a small minibatch: the 128-channel tiles leave most CUs without work and conv_patch.hip does not
// apply, so the alternative is the generic tap-by-tap kernel with a split reduction (measured 270-390 TFLOP/s there,
// plus ~9 us for the launch of its reduction epilogue).  One 192 x 64 tile's serial reduction loop takes 5.4-6.6 us
// per 64-channel slice of a 3x3 filter whatever the minibatch, so the flat tiles win only once the layer holds
// enough work.
bool flat64_fits(const GemmGeom& g) {
    TileCfg c = {1, 0, 0, 3, 0, 0, 0, 0};
    return g.M >= 192 * 4 && max_flat_patch(g, 192) <= MAX_PATCH_FLAT64 && lds_layout(g, &c);
}
bool flat64_wins_small_batch(const GemmGeom& g) {
    if ((g.Ncols % 64) != 0 || g.Ncols <= 64 || g.M >= 224 * 32 || g.M < 192 * 4) return false;
    if ((long)((g.M + 191) / 192) * (g.Ncols / 64) < 64) return false;
    if (!flat64_fits(g)) return false;
    const double flops = 2.0 * g.M * (double)g.Ncols * g.Kred;
    const double t_generic = flops / 330e12 + 9e-6;
    const double floor_s = 5.5e-6 * (g.IC / 64.0) * (g.R * g.S / 9.0);
    const double t_flat = floor_s > flops / 900e12 ? floor_s : flops / 900e12;
    return t_flat < 0.85 * t_generic;
}
// Tile shape for this geometry (width must divide the map, patch must fit), fn = 0 if none.
TileCfg tile_cfg(const GemmGeom& g) {
    TileCfg none = {0, 0, 0, 0, 0, 0, 0, 0};
    TileCfg c = none;
    if ((g.Ncols % 64) != 0) return none;
    const bool tiles128 = (g.Ncols % 128) == 0;  // 2-D tiles of 128 channels (64 output channels: conv_tile64.hip)
    for (int tw : {32, 16, 8}) {
        const int th = 256 / tw;
        if (tiles128 && (g.OH % th) == 0 && (g.OW % tw) == 0 && (th + g.R - 1) * (tw + g.S - 1) <= MAX_PATCH) {
            c = {2, tw, th, 0, 0, 0, 0, 0};
            if (lds_layout(g, &c)) return c;
            c = none;
        }
    }
    // maps of 28k x 8j pixels (56 x 56): 8 x 28 tiles, one 224-pixel strip per wavefront, 128-channel tiles
    if ((g.Ncols % 128) == 0 && (g.OW % 28) == 0 && (g.OH % 8) == 0 && (8 + g.R - 1) * (28 + g.S - 1) <= MAX_PATCH) {
        c = {1, 28, 8, 1, 0, 0, 0, 0};
        if (!lds_layout(g, &c)) c = none;
    }
    // Flat 128-channel tiles: 224 pixels per tile while that puts a work-group on at least three quarters of the CUs,
    // else 64 pixels (the serial reduction of a tile is what a small layer waits for: a short tile shortens every
    // reduction step four-fold and puts more work-groups on the chip; the weight stream per pixel grows, which a small
    // layer can afford).  Measured: conv4_2 at minibatch 8 55 -> 44 us, conv5_1 at 32 54 -> 44 us, at 16 37 -> 33 us;
    // 128-pixel tiles lost to 224-pixel ones wherever both applied (conv5_1 at 64: 68 vs 64 us).  Short flat tiles
    // also replace the strips where those leave the chip under-filled.
    const long strips = c.fn ? (long)(g.M / 224) * (g.Ncols / 128) : 0;
    if ((c.fn == 0 || strips < kNumCU * 3 / 4) && (g.Ncols % 128) == 0 && g.M >= 64 * 4) {
        for (int fm : {7, 2}) {
            const int bm = 32 * fm;
            const long wgs = (long)((g.M + bm - 1) / bm) * (g.Ncols / 128);
            if (max_flat_patch(g, bm) > MAX_PATCH_FLAT || (fm > 2 && wgs < kNumCU * 3 / 4)) continue;
            if (c.fn != 0 && wgs <= strips) break;  // no better filled than the strips
            TileCfg f = {1, 0, 0, 2, 0, 0, 0, fm};
            if (lds_layout(g, &f)) { c = f; break; }
        }
    }
    // 192-pixel x 64-channel flat tiles where none of the above applies (64 or 192 output channels on maps no 2-D
    // tile divides), and for wide outputs at a small minibatch where they beat the generic kernel
    const bool use64 = (c.fn == 0 && flat64_fits(g)) ||
                       (c.fn != 0 && c.variant >= 1 && c.variant <= 2 &&
                        (long)((g.M + tile_pixels(c) - 1) / tile_pixels(c)) * (g.Ncols / 128) < kNumCU * 3 / 4 &&
                        flat64_wins_small_batch(g));
    if (use64) {
        c = {1, 0, 0, 3, 0, 0, 0, 0};
        if (!lds_layout(g, &c)) c = none;
    }
    return c;
}
}  // namespace

// 0 = not applicable, otherwise FN (32-channel blocks per wavefront)
int tile2d_supported(const GemmGeom& g) {
    if ((g.IC % BK) != 0 || g.div_h != 1 || g.div_w != 1 || g.mul_h != 1 || g.mul_w != 1) return 0;
    if (g.R * g.S < 2) return 0;
    long a_elems = (long)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * g.IC;
    if (a_elems * 2 >= (1L << 31)) return 0;
    if (tile64_width(g)) return 1;  // 64 output channels on a map that 256-pixel tiles divide: conv_tile64.hip
    return tile_cfg(g).fn;
}

// Shapes on which this kernel measured faster than conv_patch.hip: thin outputs on 256-pixel 2-D tiles, and the
// 224-pixel x 128-channel tiles (8 x 28 strips or flat) at any width once the map is large enough to fill the CUs.
bool tile2d_preferred(const GemmGeom& g) {
    if (!tile2d_supported(g)) return false;
    if (tile64_width(g)) return true;
    const TileCfg c = tile_cfg(g);
    if (c.variant == 0) return g.Ncols <= 128;
    if (c.variant == 3) {  // measured against the generic tap-by-tap kernel (64 channels) and conv_patch (wider)
        // 192 output channels on 13 x 13 maps (384 -> 192 data gradient): 27 against 38 us at minibatch 32 (87 tiles), 27
        // against 41 us at 64; at 16 and below (45 tiles and fewer) the generic kernel with a split reduction wins
        const long t3 = (long)((g.M + 191) / 192) * (g.Ncols / 64);
        return g.Ncols == 64 ? t3 >= 48 : (t3 >= 80 || flat64_wins_small_batch(g));
    }
    const long wgs = (long)((g.M + tile_pixels(c) - 1) / tile_pixels(c)) * (g.Ncols / 128);
    // 64-pixel flat tiles keep winning against the generic kernel well below a work-group per CU while the reduction is
    // short (13 x 13 layers of 192 .. 384 input channels at minibatch 8 .. 32: 23 against 36 us, 18 against 26 us, 17
    // against 21 us); with 512 input channels (reduction 4608) the generic kernel's split reduction draws level
    if (c.variant == 2 && c.fm == 2 && wgs >= 64 && g.Kred <= 3456) return true;
    return wgs >= kNumCU * 3 / 4;
}

const char* tile2d_kernel_name(const GemmGeom& g, bool unpool) {
    if (tile64_width(g)) return tile64_kernel_name(g, unpool);
    const TileCfg c = tile_cfg(g);
    const int u = unpool ? 1 : 0, t9 = (g.R == 3 && g.S == 3) ? 1 : 0;
    static const char* n1[2][2] = {{"conv_tile2d_kernel<1,28,7,1,false,false>", "conv_tile2d_kernel<1,28,7,1,false,true>"},
                                   {"conv_tile2d_kernel<1,28,7,1,true,false>", "conv_tile2d_kernel<1,28,7,1,true,true>"}};
    static const char* n2[2][2] = {{"conv_tile2d_kernel<1,0,7,1,false,false>", "conv_tile2d_kernel<1,0,7,1,false,true>"},
                                   {"conv_tile2d_kernel<1,0,7,1,true,false>", "conv_tile2d_kernel<1,0,7,1,true,true>"}};
    static const char* n3[2][2] = {{"conv_tile2d_kernel<1,0,3,2,false,false>", "conv_tile2d_kernel<1,0,3,2,false,true>"},
                                   {"conv_tile2d_kernel<1,0,3,2,true,false>", "conv_tile2d_kernel<1,0,3,2,true,true>"}};
    static const char* n22[2][2] = {{"conv_tile2d_kernel<1,0,2,1,false,false>", "conv_tile2d_kernel<1,0,2,1,false,true>"},
                                    {"conv_tile2d_kernel<1,0,2,1,true,false>", "conv_tile2d_kernel<1,0,2,1,true,true>"}};
    if (c.variant == 1) return n1[u][t9];
    if (c.variant == 2) return c.fm == 7 ? n2[u][t9] : n22[u][t9];
    if (c.variant == 3) return n3[u][t9];
    static const char* names[2][2][3] = {
        {{"conv_tile2d_kernel<2,32,4,2,false,false>", "conv_tile2d_kernel<2,16,4,2,false,false>", "conv_tile2d_kernel<2,8,4,2,false,false>"},
         {"conv_tile2d_kernel<2,32,4,2,false,true>", "conv_tile2d_kernel<2,16,4,2,false,true>", "conv_tile2d_kernel<2,8,4,2,false,true>"}},
        {{"conv_tile2d_kernel<2,32,4,2,true,false>", "conv_tile2d_kernel<2,16,4,2,true,false>", "conv_tile2d_kernel<2,8,4,2,true,false>"},
         {"conv_tile2d_kernel<2,32,4,2,true,true>", "conv_tile2d_kernel<2,16,4,2,true,true>", "conv_tile2d_kernel<2,8,4,2,true,true>"}}};
    return names[u][t9][c.tw == 32 ? 0 : c.tw == 16 ? 1 : 2];
}

// can the patch loader take the input operand pooled (2x2 / stride 2, whole windows) plus the argmax?
bool tile2d_fuses_unpool(const GemmGeom& g) {
    if (tile64_width(g)) return tile64_fuses_unpool(g);
    if (!tile2d_supported(g) || (g.IH % 2) != 0 || (g.IW % 2) != 0) return false;
    const TileCfg c = tile_cfg(g);
    if (c.variant >= 2) return true;
    return ((c.th + g.R - 1) / 2 + 1) * ((c.tw + g.S - 1) / 2 + 1) <= 2 * (NT / 4);  // windows per patch: 2 per 4 threads
}

// partial rows (pixel tiles) the epilogue's column sums come in: [tile2d_colsum_rows][Ncols]
int tile2d_colsum_rows(const GemmGeom& g) {
    if (const int tw = tile64_width(g)) return (g.M / (g.OH * g.OW)) * (g.OW / tw) * (g.OH / (256 / tw));
    const TileCfg c = tile_cfg(g);
    if (c.variant >= 2) return (g.M + tile_pixels(c) - 1) / tile_pixels(c);
    return (g.M / (g.OH * g.OW)) * (g.OW / c.tw) * (g.OH / c.th);
}

// can the epilogue also emit the 2x2 / stride-2 max-pool of the output?
bool tile2d_fuses_pool(const GemmGeom& g) {
    if (!tile2d_supported(g)) return false;
    if (tile64_width(g)) return true;  // even tile origin and size, whole tile staged
    const TileCfg c = tile_cfg(g);  // even tile origin and size, whole windows per staging pass
    if (c.variant == 0 || c.variant == 1) return true;  // strips stage the whole 224 x 128 tile in one pass
    // flat 224 x 128 tiles: whole row pairs per tile
    return c.variant == 2 && (g.OH % 2) == 0 && (g.OW % 2) == 0 && (tile_pixels(c) % (2 * g.OW)) == 0;
}

int launch_tile2d(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                  hipStream_t st, const bf16_t* mask, bf16_t* pool_y, uint8_t* pool_am, const uint8_t* unpool_am,
                  float* colsum) {
    if (colsum && pool_y) return set_error(WAP_EINVAL, "internal: column sums and the fused pool share the staging area");
    if (tile64_width(g)) return launch_tile64(g, A, Wp, bias, relu, out, st, mask, pool_y, pool_am, unpool_am, colsum);
    TArgs ta = {};
    ta.colsum = colsum;
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
    ta.A = A;
    ta.Wp = reinterpret_cast<const bf16_t*>(Wp);
    ta.bias = bias;
    ta.out = out;
    ta.g = g;
    ta.tiles_n = c.variant == 3 ? g.Ncols / 64 : g.Ncols / 128;
    ta.RWB = c.RWB;
    ta.buf_bytes = c.buf_bytes;
    if (c.variant >= 2) {
        const int bm = tile_pixels(c);
        ta.tiles_x = ta.tiles_y = ta.tiles_img = 1;
        ta.tiles_m = (g.M + bm - 1) / bm;
        ta.PH = g.OH + g.R - 1;
        ta.RW = g.OW + g.S - 1;
        ta.dRPHW = make_fastdiv((uint32_t)(ta.PH * ta.RW));
        ta.patch_len = 0;  // per tile, computed in the kernel
        ta.dOHW = make_fastdiv((uint32_t)(g.OH * g.OW));
        ta.dOW = make_fastdiv((uint32_t)g.OW);
        ta.dOW2 = make_fastdiv((uint32_t)(g.OW / 2 > 0 ? g.OW / 2 : 1));
    } else {
        ta.tiles_x = g.OW / c.tw;
        ta.tiles_y = g.OH / c.th;
        ta.tiles_img = ta.tiles_x * ta.tiles_y;
        ta.tiles_m = ta.tiles_img * (g.M / (g.OH * g.OW));
        ta.RW = c.tw + g.S - 1;
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
    ta.dRW = make_fastdiv((uint32_t)ta.RW);
    const size_t smem = c.smem;
    if (c.variant == 1) return launch_tile2d_t<1, 28, 7, 1>(ta, smem, st);
    if (c.variant == 2 && c.fm == 7) return launch_tile2d_t<1, 0, 7, 1>(ta, smem, st);
    if (c.variant == 2) return launch_tile2d_t<1, 0, 2, 1>(ta, smem, st);
    if (c.variant == 3) return launch_tile2d_t<1, 0, 3, 2>(ta, smem, st);
    const int TW = c.tw;  // 2-D tiles: two channel blocks per wavefront, 128-channel tiles
    if (TW == 32) return launch_tile2d_t<2, 32, 4, 2>(ta, smem, st);
    if (TW == 16) return launch_tile2d_t<2, 16, 4, 2>(ta, smem, st);
    return launch_tile2d_t<2, 8, 4, 2>(ta, smem, st);
}

}  // namespace wap
