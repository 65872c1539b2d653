// Weight gradient of a stride-1 3x3 convolution with the input PATCH resident in LDS (gfx950):
//   dw[k][(r,s,c)] = sum over pixels (n,p,q) of dy[n,p,q,k] * x[n, p-ph+r, q-pw+s, c]
// (backward half of t_c in Eq. 1; the output is the weight-sized tensor whose aggregation cost the
// platform model of Section 3.2.3 prices).
//
// The generic kernel in wgrad.hip gathers one x tile per filter tap, i.e. reads (and writes to LDS)
// every input pixel nine times.  Here a work-group owns 64*FD output channels x 64 input channels x
// ALL nine taps and walks a range of small 2-D pixel tiles (up to 128 pixels); per tile it writes the
// zero-padded x patch (tile plus halo, 64 channels) and the dy tile to LDS once, and every tap is the
// same patch read through a pointer shifted by (r * padded_width + s) pixels.  Both operands are stored
// as loaded (channel-contiguous) and transposed on the way to the MFMA with ds_read_b64_tr_b16, so an
// arbitrary pixel -> LDS row map costs nothing: a tile is a TH x TW rectangle, its width rounded up to a
// multiple of 4 (at least 16) columns whose surplus pixels carry dy = 0.
//   * 12 wavefronts, three per SIMD whatever the dispatcher's placement: wavefront (r, cb, kh) owns filter
//     row r, the 32-channel half cb of the x slice and FD 32-channel blocks of dy: 3 taps x FD tiles;
//   * one work-group per CU.  LDS holds two tile buffers: while the wavefronts run the MFMAs of tile i out
//     of one buffer, their global loads of tile i+2 are in flight and tile i+1 (already in registers) is
//     written to the other buffer, so a tile costs one barrier and no exposed load or store phase;
//   * instruction count is what the kernel is built around (measured: the time of a tile is close to the
//     SUM of its MFMA time and the issue time of everything else, not their maximum): the loader works in
//     whole tile rows so that its address arithmetic is scalar, the reduction steps address LDS through
//     immediate offsets from two per-lane registers, and fragment reads are interleaved with the MFMAs one
//     step ahead;
//   * the pixel range is split across work-groups; every split writes an fp32 partial and the reduce
//     kernel adds them in a fixed order (bitwise reproducible).
// UP variant: dy is given as the gradient of a 2x2 / stride-2 max-pool OUTPUT plus the pool's argmax; the
// loader routes each window's value to the pixel the argmax names (the max-pool backward of the auxiliary
// node between two primary nodes, Section 3.2.2) on the way into LDS, so the full-size dy never exists.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int NT = 768;       // 12 wavefronts
constexpr int XPITCH = 192;   // LDS bytes per patch pixel: 64 channels + 64 bytes, so that the 4 rows x 64 bytes a
                              // half-wavefront touches in one transposing read fall into 4 disjoint bank groups
constexpr int DCAP = 128;     // most dy rows (virtual pixels) per tile: 8 reduction steps of 16
constexpr int PVMAX = 3;      // most wavefront loads of the patch per wavefront and tile: 36 per work-group
constexpr unsigned OOB = 0x80000000u;  // both tensors are below 2 GiB (checked on the host)
constexpr size_t LDS_BYTES = 160 * 1024;

// How the 16 pixels of one reduction step lie in the tile.  Every mode keeps the LDS address of a step at a
// compile-time distance from the address of step 0, so the reduction loop holds no address arithmetic at all:
//   MODE 0: virtual tile width 16, a step is one tile row;
//   MODE 1: virtual tile width 32, a step is half a tile row;
//   MODE 2: any virtual width that is a multiple of 4, tile height 4, a step is a block of 4 rows x 4 columns.
template <int MODE> struct StepMap;
template <> struct StepMap<0> { static constexpr int VW = 16, PWP = 18; };
template <> struct StepMap<1> { static constexpr int VW = 32, PWP = 34; };

struct WPArgs {
    const bf16_t* x;
    const bf16_t* dy;
    float* out;
    WgradGeom g;
    int Kred;
    int TH, TWr, VW, PWp;       // tile rows, real / virtual tile columns, padded patch width
    int nk;                     // reduction steps per tile
    int NSEG, NXL;              // 8-pixel segments per patch row, wavefront loads per patch
    int DSEG, NDL;              // segments per dy tile row (UP: per row of pooling windows), wavefront loads per dy tile
    int tiles_x, tiles_img, tiles_total;
    int kgroups, ncombo, nsplit, tiles_per_split;
    int buf_bytes, d_off;       // bytes per LDS tile buffer, offset of the dy tile inside it
    unsigned x_bytes, dy_bytes;
    const uint8_t* am;  // UP: argmax (r * 2 + s) of every pooling window, same shape as the pooled dy
    int P2, Q2;         // UP: pooled map size
    FastDiv dNSEG, dDSEG, dTimg, dTx;
};

__device__ __forceinline__ int xcd_remap(int bid, int total) {
    int per = total / kNumXCD, rem = total % kNumXCD;
    int xcd = bid % kNumXCD, idx = bid / kNumXCD;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
__device__ __forceinline__ bf16x8 tr_pair(const unsigned char* p0, const unsigned char* p1) {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p1);
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
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

// FD: 32-channel dy blocks per wavefront; the work-group covers 64 * FD output channels.  UP: dy arrives pooled.
// NK: reduction steps per tile (tile pixels / 16).
template <int FD, bool UP, int MODE, int NK>
__global__ __launch_bounds__(NT, 3) void wgrad_patch_kernel(const WPArgs a) {
    constexpr int KO = 64 * FD;             // output channels per work-group
    constexpr int DPITCH = KO * 2 + 64;     // same bank argument as XPITCH
    constexpr int DVP = KO / 8;             // 16-byte vectors per dy pixel
    constexpr int PPW = 64 / DVP;           // dy pixels (UP: pooling windows) one wavefront load covers
    // wavefront loads per wavefront and tile: 12 wavefronts share (tile rows + 2) x segments loads of the patch and
    // tile rows x segments loads of dy (pooled dy: one)
    constexpr int TVW = MODE == 0 ? 16 : MODE == 1 ? 32 : 4 * NK, TTH = NK * 16 / TVW;
    constexpr int PV = ((TTH + 2) * ((TVW + 2 + 7) / 8) + 11) / 12;
    constexpr int DV = UP ? 1 : (TTH * ((TVW + PPW - 1) / PPW) + 11) / 12;
    static_assert(PV <= PVMAX && DV <= 3, "tile too large for the loader");
    extern __shared__ __align__(16) unsigned char smem[];
    const WgradGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: everything derived from it stays scalar
    const int r = wave >> 2, cb = (wave >> 1) & 1, kh = wave & 1;

    const int total = a.ncombo * a.nsplit;
    const int logical = xcd_remap(blockIdx.x, total);
    const int combo = logical % a.ncombo, split = logical / a.ncombo;
    const int ko0 = (combo % a.kgroups) * KO, c0 = (combo / a.kgroups) * 64;
    const int t0 = split * a.tiles_per_split;
    int t1 = t0 + a.tiles_per_split;
    if (t1 > a.tiles_total) t1 = a.tiles_total;

    const __amdgpu_buffer_rsrc_t rsrcX =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.x), 0, (int)a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcD =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.dy), 0, (int)a.dy_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcM =  // one argmax byte per pooled element: half the bytes of the pooled dy
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(UP ? a.am : nullptr), 0, UP ? (int)(a.dy_bytes / 2) : 0, 0x00020000);

    // ---- global loads of one tile.  A wavefront load covers a run of pixels of ONE tile row (8 patch pixels x 64
    // channels; 64 / DVP dy pixels or pooling windows x KO channels), so which row, which segment of it, whether the
    // row exists and where it starts in memory are all wavefront-uniform (scalar unit); a lane contributes a
    // constant offset and one comparison of its pixel against the row's valid columns.  The last segment of a row
    // is moved back so that it ends with the row: it then repeats a few pixels of its neighbour (both write the
    // same bytes to the same LDS address), and no lane ever falls outside its row.  Wavefront w takes the loads
    // w, w + 12, w + 24 of the tile. ----
    auto seg_start = [](int seg, int per, int row_len) {  // first pixel of segment seg of a row of row_len >= per pixels
        const int p0 = seg * per;
        return p0 + per > row_len ? row_len - per : p0;
    };
    const int lx = lane >> 3;                                             // patch pixel within the segment
    const unsigned xv = (unsigned)(lx * g.C * 2 + (lane & 7) * 16);      // its bytes from the segment's first pixel
    const unsigned xs = (unsigned)(lx * XPITCH + (lane & 7) * 16);       // the same in LDS
    const int lp = lane / DVP, lc = lane % DVP;                           // dy pixel (window) within the segment, 16-byte chunk
    const unsigned dvv = (unsigned)((lp * g.K + lc * 8) * 2);            // bytes from the segment's first pixel (window)
    const unsigned dsl = (unsigned)((UP ? 2 * lp : lp) * DPITCH + lc * 16);  // the same in LDS (a window is two pixels wide)
    u32x4 rp[PV], rd[DV];
    u32x2 ra[1];
    auto load_tile = [&](int t) {
        const int img = (int)fdiv((uint32_t)t, a.dTimg);
        const int rem = t - img * a.tiles_img;
        const int tyi = (int)fdiv((uint32_t)rem, a.dTx);
        const int oh0 = tyi * a.TH, ow0 = (rem - tyi * a.tiles_x) * a.TWr;
        const int ih0 = oh0 - g.ph, iw0 = ow0 - g.pw;
        const int xbase = (((img * g.H + ih0) * g.W + iw0) * g.C + c0) * 2;  // first patch pixel (may lie before the tensor)
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            const int j = wave + 12 * i;
            const int py = (int)fdiv((uint32_t)j, a.dNSEG), px0 = seg_start(j - py * a.NSEG, 8, a.PWp);
            // columns of the segment that lie inside the image
            const int lo = -(iw0 + px0);
            const int hi = g.W - iw0 - px0;
            const bool rowok = j < a.NXL && (unsigned)(ih0 + py) < (unsigned)g.H;
            const bool ok = rowok && lx >= lo && lx < hi;
            const unsigned off = xv + (unsigned)(xbase + (py * g.W + px0) * g.C * 2);
            rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcX, ok ? off : OOB, 0, 0);
        }
        if (UP) {
            // one load per wavefront: PPW pooling windows of one pooled row (16 bytes of pooled dy, 8 argmax bytes each);
            // the tile has even origin and size, so windows never straddle tiles
            const int j = wave;
            const int uy = (int)fdiv((uint32_t)j, a.dDSEG), ux0 = seg_start(j - uy * a.DSEG, PPW, a.VW / 2);
            const bool ok = j < a.NDL && oh0 + 2 * uy < g.P && 2 * (ux0 + lp) < a.TWr;
            const unsigned el = (unsigned)(((img * a.P2 + (oh0 >> 1) + uy) * a.Q2 + (ow0 >> 1) + ux0) * g.K + ko0);
            rd[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrcD, ok ? dvv : OOB, el * 2u, 0);
            ra[0] = __builtin_amdgcn_raw_buffer_load_b64(rsrcM, ok ? dvv / 2u : OOB, el, 0);
        } else {
            const int dbase = (((img * g.P + oh0) * g.Q + ow0) * g.K + ko0) * 2;
#pragma unroll
            for (int i = 0; i < DV; ++i) {
                const int j = wave + 12 * i;
                const int ty = (int)fdiv((uint32_t)j, a.dDSEG), tx0 = seg_start(j - ty * a.DSEG, PPW, a.VW);
                const bool ok = j < a.NDL && oh0 + ty < g.P && tx0 + lp < a.TWr;
                const unsigned soff = (unsigned)(dbase + (ty * g.Q + tx0) * g.K * 2);
                rd[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcD, ok ? dvv : OOB, soff, 0);
            }
        }
    };
    // every patch pixel and every dy pixel of the tile is written (zeros where the load was masked), so every row
    // the MFMA loop reads holds either data or zeros
    auto store_tile = [&](int buf) {
        unsigned char* sX = smem + buf * a.buf_bytes;
        unsigned char* sD = sX + a.d_off;
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            const int j = wave + 12 * i;
            const int py = (int)fdiv((uint32_t)j, a.dNSEG), px0 = seg_start(j - py * a.NSEG, 8, a.PWp);
            if (j < a.NXL) *reinterpret_cast<u32x4*>(sX + (py * a.PWp + px0) * XPITCH + xs) = rp[i];
        }
        if (UP) {
            const int j = wave;
            const int uy = (int)fdiv((uint32_t)j, a.dDSEG), ux0 = seg_start(j - uy * a.DSEG, PPW, a.VW / 2);
            if (j < a.NDL) {
#pragma unroll
                for (int pos = 0; pos < 4; ++pos) {
                    const int q = (2 * uy + (pos >> 1)) * a.VW + 2 * ux0 + (pos & 1);
                    *reinterpret_cast<u32x4*>(sD + q * DPITCH + dsl) = unpool_select8(rd[0], ra[0], (unsigned)pos);
                    __builtin_amdgcn_sched_barrier(0);  // one pixel at a time: four selected copies at once do not fit
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < DV; ++i) {
                const int j = wave + 12 * i;
                const int ty = (int)fdiv((uint32_t)j, a.dDSEG), tx0 = seg_start(j - ty * a.DSEG, PPW, a.VW);
                if (j < a.NDL) *reinterpret_cast<u32x4*>(sD + (ty * a.VW + tx0) * DPITCH + dsl) = rd[i];
            }
        }
    };

    f32x16 acc[3][FD];  // [tap s of filter row r][32-channel block of dy]
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int kb = 0; kb < FD; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[s][kb][e] = 0.f;

    // transposing read: a lane supplies the address of pixel kl = (lane / 32) * 8 + (lane % 16) / 4 of the step's 16
    // (kl + 4 for the second read) and of the 4-channel chunk ((lane / 16) % 2) * 16 + (lane % 4) * 4 of its block
    const int kl = (lane >> 5) * 8 + ((lane & 15) >> 2);
    const int chunk = (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    // LDS offsets of the lane's first pixel in step 0: patch (tap s = 0 of filter row r) and dy; the second pixel
    // (kl + 4) lies at a compile-time distance (MODE 2: one tile row further, and the tile is 4 * NK columns wide)
    constexpr int XB = MODE == 2 ? (4 * NK + 2) * XPITCH : 4 * XPITCH;
    constexpr int DB = MODE == 2 ? 4 * NK * DPITCH : 4 * DPITCH;
    int xa, da;
    if (MODE == 2) {     // pixel i of a step = row i / 4, column i % 4 of the block
        xa = ((r + (kl >> 2)) * a.PWp + (kl & 3)) * XPITCH + cb * 64 + chunk;
        da = a.d_off + ((kl >> 2) * a.VW + (kl & 3)) * DPITCH + kh * (FD * 64) + chunk;
    } else {             // pixel i of a step = column i of the row (half row)
        xa = (r * a.PWp + kl) * XPITCH + cb * 64 + chunk;
        da = a.d_off + kl * DPITCH + kh * (FD * 64) + chunk;
    }

    // ---- reduction over one tile, NK steps of 16 pixels.  Fragment reads run one step ahead of the MFMAs that
    // use them, inside the same wavefront, and mostly in place: a fragment is re-read for the next step as soon as
    // the last MFMA that uses it in this step has been issued, and the MFMAs are ordered so that every fragment then
    // has at least two of the wavefront's own MFMAs (about six of the SIMD's) between its read and its first use.
    // (The hardware arbitrates the MFMA pipe round-robin between the wavefronts of a SIMD, which keeps them in
    // lockstep: without the overlap inside a wavefront all of them wait for LDS at the same time.)  The tile's only
    // barrier sits in the LAST step, in front of the reads that fetch step 0 of the next tile from the other
    // buffer, so the pipeline never drains. ----
    bf16x8 fd[FD], fx[3];  // dy fragments (one per 32-channel block), patch fragments (one per tap s)
    bf16x8 fdn[1];         // FD == 1 only: the single dy fragment is used by every MFMA of a step, so the next one gets registers of its own
    auto read_d = [&](bf16x8& f, int kb, const unsigned char* sB, int dO) {
        f = tr_pair(sB + da + dO + kb * 64, sB + da + dO + DB + kb * 64);
    };
    auto read_x = [&](int s, const unsigned char* sB, int xo) {
        fx[s] = tr_pair(sB + xa + xo + s * XPITCH, sB + xa + xo + XB + s * XPITCH);
    };
    auto step_x = [](int ks) {  // compile-time distance of step ks from step 0 in the patch
        return MODE == 0 ? ks * StepMap<0>::PWP * XPITCH
             : MODE == 1 ? ((ks >> 1) * StepMap<1>::PWP + (ks & 1) * 16) * XPITCH : ks * 4 * XPITCH;
    };
    auto step_d = [](int ks) { return (MODE == 2 ? ks * 4 : ks * 16) * DPITCH; };  // ... and in the dy tile
    auto tile_barrier = [&]() {
        // every wavefront's reads of this buffer have returned and its share of the next tile is in the other
        // buffer (its LDS counter is at zero) before anyone passes
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mma = [&](int s, int kb, const bf16x8& d) {
        acc[s][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[s], d, acc[s][kb], 0, 0, 0);
    };
    auto tile_steps = [&](const unsigned char* sB, const unsigned char* sN) {
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            const bool last = ks == NK - 1;
            const unsigned char* src = last ? sN : sB;  // where the fragments of the following step live
            const int xo = last ? 0 : step_x(ks + 1), dO = last ? 0 : step_d(ks + 1);
            if constexpr (FD == 2) {
                mma(0, 0, fd[0]); mma(1, 0, fd[0]); mma(2, 0, fd[0]);
                __builtin_amdgcn_sched_barrier(0);
                if (last) tile_barrier();
                read_d(fd[0], 0, src, dO);
                mma(0, 1, fd[1]);
                __builtin_amdgcn_sched_barrier(0);
                read_x(0, src, xo);
                mma(1, 1, fd[1]);
                __builtin_amdgcn_sched_barrier(0);
                read_x(1, src, xo);
                mma(2, 1, fd[1]);
                __builtin_amdgcn_sched_barrier(0);
                read_x(2, src, xo);
                read_d(fd[1], 1, src, dO);
                __builtin_amdgcn_sched_barrier(0);
            } else {
                if (last) tile_barrier();
                read_d((ks & 1) ? fd[0] : fdn[0], 0, src, dO);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    mma(s, 0, (ks & 1) ? fdn[0] : fd[0]);
                    read_x(s, src, xo);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if (FD == 1 && (NK & 1)) fd[0] = fdn[0];  // the next tile's step 0 sits in the second set: make it the current one
    };

    if (t0 < t1) {
        load_tile(t0);
        store_tile(0);
        if (t0 + 1 < t1) load_tile(t0 + 1);
    }
    __syncthreads();
#pragma unroll
    for (int kb = 0; kb < FD; ++kb) read_d(fd[kb], kb, smem, 0);
#pragma unroll
    for (int s = 0; s < 3; ++s) read_x(s, smem, 0);
    for (int t = t0; t < t1; ++t) {
        const int buf = (t - t0) & 1;
        // tile t+1 (in registers since the previous iteration) -> the other buffer, whose last readers finished
        // before the barrier in the previous tile's last step; then tile t+2 goes in flight
        if (t + 1 < t1) store_tile(buf ^ 1);
        if (t + 2 < t1) load_tile(t + 2);
        const unsigned char* sB = smem + buf * a.buf_bytes;
        const unsigned char* sN = smem + (buf ^ 1) * a.buf_bytes;
        tile_steps(sB, sN);
    }

    // ---- epilogue: a lane holds 4 consecutive input channels of one output channel per register quad ----
    float* outp = a.out + (size_t)split * g.K * a.Kred;
#pragma unroll
    for (int kb = 0; kb < FD; ++kb) {
        const int ko = ko0 + kh * (FD * 32) + kb * 32 + (lane & 31);
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = (r * 3 + s) * g.C + c0 + cb * 32 + q * 8 + (lane >> 5) * 4;
                *reinterpret_cast<float4*>(outp + (size_t)ko * a.Kred + col) =
                    make_float4(acc[s][kb][q * 4 + 0], acc[s][kb][q * 4 + 1], acc[s][kb][q * 4 + 2], acc[s][kb][q * 4 + 3]);
            }
    }
}

struct TileShape {
    int TH, TWr, VW, mode;
    int nseg() const { return (VW + 2 + 7) / 8; }        // 8-pixel segments per patch row
    int nk() const { return TH * VW / 16; }
};

bool choose_tile_fd(const WgradGeom& g, int fd, struct TileShape* out);
int fd_for(const WgradGeom& g);
size_t buf_bytes_for(int fd, const TileShape& ts) {
    return (size_t)(ts.TH + 2) * (ts.VW + 2) * XPITCH + (size_t)ts.TH * ts.VW * (fd * 128 + 64);
}

// Most real pixels per tile (the tile height need not divide the map: the last tile row of an image is then partly
// masked) among the tiles the kernel's three step maps cover and whose two LDS buffers fit; then the least padding.
bool choose_tile_fd(const WgradGeom& g, int fd, TileShape* out) {
    long best = 0;
    for (int twr = 1; twr <= g.Q && twr <= 32; ++twr) {
        if (g.Q % twr) continue;
        const int vw = twr <= 16 ? 16 : (twr + 3) / 4 * 4;
        if (vw > 32) continue;
        const int mode = vw == 16 ? 0 : vw == 32 ? 1 : 2;
        for (int th = 1; th <= g.P; ++th) {
            if ((mode == 2 && th != 4) || (mode == 1 && th != 4) || (mode == 0 && th != 7 && th != 8)) continue;
            const TileShape ts{th, twr, vw, mode};
            if (th * vw > DCAP || (th + 2) * ts.nseg() > 12 * PVMAX) break;
            if (2 * buf_bytes_for(fd, ts) > LDS_BYTES) break;
            const int tiles_y = (g.P + th - 1) / th;
            // real pixels per tile first, then the least padding, then even tiles (whole pooling windows)
            long score = ((long)g.P * twr * 1024 / tiles_y + (1023 - th * (vw - twr))) * 2 + ((th % 2) == 0 && (twr % 2) == 0 ? 1 : 0);
            if (score > best) {
                best = score;
                *out = ts;
            }
        }
    }
    return best > 0;
}

// 32-channel dy blocks per wavefront: two where the layer has a multiple of 128 output channels, unless the pixel range
// is short (at most 28 tiles per work-group: small minibatches, the 14 x 14 layers): the fp32 partial tiles that every
// work-group writes and the reduction that reads them then weigh more than the better register tile saves, and
// 64-channel work-groups halve those bytes for the same number of work-groups (conv4_2 at minibatch 8: 75 -> 38 MB).
// Measured on whole steps with the limit at 8 / 16 / 28 tiles: VGG-16 -5.1 / -5.1 / -5.2 % at b = 8, -2.2 / -3.4 / -3.6 %
// at 16, -0.9 / -1.0 / -1.3 % at 32, 0 / 0 / -0.5 % at 64; the AlexNet-style step -2 .. -3 % at b = 8 .. 64.
int fd_for(const WgradGeom& g) {
    if ((g.K % 128) != 0 || g_force_wgrad_cfg == 6) return 1;
    if (g_force_wgrad_cfg == 5) return 2;
    TileShape ts;
    if (!choose_tile_fd(g, 2, &ts)) return 1;
    const long tiles = (long)g.N * ((g.P + ts.TH - 1) / ts.TH) * (g.Q / ts.TWr);
    const long ncombo2 = (long)(g.K / 128) * (g.C / 64);
    return tiles * ncombo2 <= 28L * kNumCU ? 1 : 2;
}
bool choose_tile(const WgradGeom& g, TileShape* out) { return choose_tile_fd(g, fd_for(g), out); }

}  // namespace

bool wgrad_patch_supported(const WgradGeom& g) {
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1) return false;
    if ((g.C % 64) != 0 || (g.K % 64) != 0) return false;
    if ((size_t)g.N * g.H * g.W * g.C * 2 >= (1ull << 31) || (size_t)g.N * g.P * g.Q * g.K * 2 >= (1ull << 31)) return false;
    TileShape ts;
    if (!choose_tile(g, &ts)) return false;
    return ts.TH * ts.TWr >= 64;  // tiny tiles: the generic kernel is no worse
}

namespace {
// the instantiated (step map, steps per tile) pairs
constexpr int kNumVariants = 6;
constexpr int kVariantMode[kNumVariants] = {0, 0, 1, 2, 2, 2};
constexpr int kVariantNK[kNumVariants] = {7, 8, 8, 5, 6, 7};
int variant_of(const TileShape& ts) {
    for (int v = 0; v < kNumVariants; ++v)
        if (kVariantMode[v] == ts.mode && kVariantNK[v] == ts.nk()) return v;
    return -1;
}
}  // namespace

const char* wgrad_patch_kernel_name(const WgradGeom& g, bool unpool) {
    static const char* names[2][2][kNumVariants] = {
        {{"wgrad_patch_kernel<1,false,0,7>", "wgrad_patch_kernel<1,false,0,8>", "wgrad_patch_kernel<1,false,1,8>",
          "wgrad_patch_kernel<1,false,2,5>", "wgrad_patch_kernel<1,false,2,6>", "wgrad_patch_kernel<1,false,2,7>"},
         {"wgrad_patch_kernel<1,true,0,7>", "wgrad_patch_kernel<1,true,0,8>", "wgrad_patch_kernel<1,true,1,8>",
          "wgrad_patch_kernel<1,true,2,5>", "wgrad_patch_kernel<1,true,2,6>", "wgrad_patch_kernel<1,true,2,7>"}},
        {{"wgrad_patch_kernel<2,false,0,7>", "wgrad_patch_kernel<2,false,0,8>", "wgrad_patch_kernel<2,false,1,8>",
          "wgrad_patch_kernel<2,false,2,5>", "wgrad_patch_kernel<2,false,2,6>", "wgrad_patch_kernel<2,false,2,7>"},
         {"wgrad_patch_kernel<2,true,0,7>", "wgrad_patch_kernel<2,true,0,8>", "wgrad_patch_kernel<2,true,1,8>",
          "wgrad_patch_kernel<2,true,2,5>", "wgrad_patch_kernel<2,true,2,6>", "wgrad_patch_kernel<2,true,2,7>"}}};
    TileShape ts;
    if (!choose_tile(g, &ts) || variant_of(ts) < 0) return "wgrad_patch_kernel";
    return names[fd_for(g) - 1][unpool ? 1 : 0][variant_of(ts)];
}

// dy given as the gradient of the 2x2 / stride-2 pooled output plus the argmax: whole windows only, and one
// wavefront load of windows per wavefront
static int unpool_loads(const WgradGeom& g, const TileShape& ts) {
    const int ppw = fd_for(g) == 2 ? 4 : 8;
    return (ts.TH / 2) * ((ts.VW / 2 + ppw - 1) / ppw);
}
bool wgrad_patch_fuses_unpool(const WgradGeom& g) {
    TileShape ts;
    if (!wgrad_patch_supported(g) || (g.P % 2) != 0 || (g.Q % 2) != 0 || !choose_tile(g, &ts)) return false;
    if ((ts.TH % 2) != 0 || (ts.TWr % 2) != 0) return false;  // windows must not straddle tiles
    return unpool_loads(g, ts) <= NT / 64;
}

int wgrad_patch_nsplit(const WgradGeom& g) {
    TileShape ts;
    if (!choose_tile(g, &ts)) return 1;
    const long tiles = (long)g.N * ((g.P + ts.TH - 1) / ts.TH) * (g.Q / ts.TWr);
    const long ncombo = (long)(g.K / (64 * fd_for(g))) * (g.C / 64);
    long want = kNumCU / ncombo;  // one resident work-group per CU, one round (never a second, nearly empty one)
    if (want < 1) want = 1;
    if (want > tiles) want = tiles;
    const long tps = (tiles + want - 1) / want;
    return (int)((tiles + tps - 1) / tps);
}

namespace {
template <int FD, bool UP>
const void* variant_fn(int v) {
    switch (v) {
        case 0: return (const void*)wgrad_patch_kernel<FD, UP, 0, 7>;
        case 1: return (const void*)wgrad_patch_kernel<FD, UP, 0, 8>;
        case 2: return (const void*)wgrad_patch_kernel<FD, UP, 1, 8>;
        case 3: return (const void*)wgrad_patch_kernel<FD, UP, 2, 5>;
        case 4: return (const void*)wgrad_patch_kernel<FD, UP, 2, 6>;
        default: return (const void*)wgrad_patch_kernel<FD, UP, 2, 7>;
    }
}
const void* kernel_fn(int fd, bool up, int v) {
    if (fd == 1) return up ? variant_fn<1, true>(v) : variant_fn<1, false>(v);
    return up ? variant_fn<2, true>(v) : variant_fn<2, false>(v);
}
}  // namespace

int launch_wgrad_patch(const WgradGeom& g, int nsplit, const bf16_t* x, const bf16_t* dy, float* out, hipStream_t st,
                       const uint8_t* unpool_am) {
    WPArgs wa;
    TileShape ts;
    if (!wgrad_patch_supported(g) || !choose_tile(g, &ts))
        return set_error(WAP_EINVAL, "internal: patch weight-gradient kernel not applicable");
    if (unpool_am && !wgrad_patch_fuses_unpool(g))
        return set_error(WAP_EINVAL, "internal: fused max-pool backward not available for this shape");
    const int fd = fd_for(g);
    const int ppw = fd == 2 ? 4 : 8;
    wa.am = unpool_am;
    wa.P2 = g.P / 2;
    wa.Q2 = g.Q / 2;
    wa.x = x;
    wa.dy = dy;
    wa.out = out;
    wa.g = g;
    wa.Kred = g.R * g.S * g.C;
    wa.TH = ts.TH;
    wa.TWr = ts.TWr;
    wa.VW = ts.VW;
    wa.PWp = ts.VW + 2;
    wa.nk = ts.nk();
    wa.NSEG = ts.nseg();
    wa.NXL = (ts.TH + 2) * wa.NSEG;
    if (unpool_am) {
        wa.DSEG = (ts.VW / 2 + ppw - 1) / ppw;
        wa.NDL = unpool_loads(g, ts);
    } else {
        wa.DSEG = (ts.VW + ppw - 1) / ppw;
        wa.NDL = ts.TH * wa.DSEG;
    }
    // what the kernel's fixed loop counts and compile-time step distances assume
    const bool fits = variant_of(ts) >= 0 && wa.nk <= DCAP / 16 && wa.NXL <= 12 * PVMAX && wa.NDL <= (unpool_am ? 12 : 12 * (fd == 2 ? 3 : 2)) &&
                      ts.VW >= 16 && (ts.mode != 0 || ts.VW == StepMap<0>::VW) && (ts.mode != 1 || ts.VW == StepMap<1>::VW) &&
                      (ts.mode != 2 || (ts.TH == 4 && ts.VW == 4 * wa.nk));
    if (!fits) return set_error(WAP_EINVAL, "internal: patch weight-gradient tile outside the kernel's step maps");
    wa.tiles_x = g.Q / ts.TWr;
    wa.tiles_img = wa.tiles_x * ((g.P + ts.TH - 1) / ts.TH);
    wa.tiles_total = wa.tiles_img * g.N;
    wa.kgroups = g.K / (64 * fd);
    wa.ncombo = wa.kgroups * (g.C / 64);
    wa.nsplit = nsplit;
    wa.tiles_per_split = (wa.tiles_total + nsplit - 1) / nsplit;
    wa.d_off = (ts.TH + 2) * wa.PWp * XPITCH;
    wa.buf_bytes = (int)buf_bytes_for(fd, ts);
    wa.x_bytes = (unsigned)((size_t)g.N * g.H * g.W * g.C * 2);
    wa.dy_bytes = (unsigned)((size_t)g.N * g.P * g.Q * g.K * 2 / (unpool_am ? 4 : 1));
    wa.dNSEG = make_fastdiv((uint32_t)wa.NSEG);
    wa.dDSEG = make_fastdiv((uint32_t)wa.DSEG);
    wa.dTimg = make_fastdiv((uint32_t)wa.tiles_img);
    wa.dTx = make_fastdiv((uint32_t)wa.tiles_x);
    const size_t smem = 2 * (size_t)wa.buf_bytes;
    if (smem > LDS_BYTES) return set_error(WAP_EINVAL, "internal: patch weight-gradient tile does not fit LDS");
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        for (int f = 1; f <= 2; ++f)
            for (int u = 0; u < 2; ++u)
                for (int v = 0; v < kNumVariants; ++v) {
                    hipError_t e = hipFuncSetAttribute(kernel_fn(f, u != 0, v), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
                    if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
                }
        attr_done = true;
    }
    void* kargs[] = {(void*)&wa};
    hipError_t le = hipLaunchKernel(kernel_fn(fd, unpool_am != nullptr, variant_of(ts)), dim3(wa.ncombo * nsplit), dim3(NT), kargs, smem, st);
    if (le != hipSuccess) return set_error(WAP_EHIP, "wgrad_patch launch: %s", hipGetErrorString(le));
    return check_launch("wgrad_patch");
}

}  // namespace wap
