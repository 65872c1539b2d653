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
// arbitrary pixel -> LDS row map costs nothing: a tile may be any TH x TW rectangle, its width rounded up
// to a multiple of 4 (at least 16) columns whose surplus pixels carry dy = 0.
//   * 12 wavefronts, three per SIMD whatever the dispatcher's placement: wavefront (r, cb, kh) owns filter
//     row r, the 32-channel half cb of the x slice and FD 32-channel blocks of dy: 3 taps x FD tiles;
//   * one work-group per CU.  LDS holds two tile buffers: while the wavefronts run the MFMAs of tile i out
//     of one buffer, their global loads of tile i+2 are in flight and tile i+1 (already in registers) is
//     written to the other buffer, so a tile costs one barrier and no exposed load or store phase;
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
constexpr int PCAP = 288;     // most patch rows (padded pixels) per tile
constexpr int DCAP = 128;     // most dy rows (virtual pixels) per tile
constexpr int PV = PCAP * 8 / NT;  // 3 patch vectors per thread
constexpr unsigned OOB = 0x80000000u;  // both tensors are below 2 GiB (checked on the host)
constexpr size_t LDS_BYTES = 160 * 1024;

struct WPArgs {
    const bf16_t* x;
    const bf16_t* dy;
    float* out;
    WgradGeom g;
    int Kred;
    int TH, TWr, VW, PWp;       // tile rows, real / virtual tile columns, padded patch width
    int patch_len, npix, nk16;  // padded pixels per patch, virtual pixels per tile, reduction steps per tile
    int tiles_x, tiles_img, tiles_total;
    int kgroups, ncombo, nsplit, tiles_per_split;
    int buf_bytes, d_off;       // bytes per LDS tile buffer, offset of the dy tile inside it
    unsigned x_bytes, dy_bytes;
    const uint8_t* am;  // UP: argmax (r * 2 + s) of every pooling window, same shape as the pooled dy
    int P2, Q2;         // UP: pooled map size
    int VW2, units;     // UP: pooling windows per virtual tile row, windows per dy tile (all 16 * nk16 rows covered)
    FastDiv dVW2;
    FastDiv dVW, dPWp, dTimg, dTx;
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
template <int FD, bool UP>
__global__ __launch_bounds__(NT, 3) void wgrad_patch_kernel(const WPArgs a) {
    constexpr int KO = 64 * FD;             // output channels per work-group
    constexpr int DPITCH = KO * 2 + 64;     // same bank argument as XPITCH
    constexpr int DVP = KO / 8;             // 16-byte vectors per dy pixel
    constexpr int DV = (DCAP * DVP + NT - 1) / NT;
    extern __shared__ __align__(16) unsigned char smem[];
    const WgradGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    // ---- global loads of one tile.  The slot geometry (which padded pixel / dy pixel a thread fetches) is
    // recomputed from the thread index for every tile: hoisted out of the tile loop it would sit in registers
    // the accumulators need, and come back as scratch reloads on the critical path of every tile. ----
    // UP: a thread fetches one whole pooling window (16 bytes of pooled dy, 8 argmax bytes) and writes its four pixels;
    // the tile has even origin and size, so windows never straddle tiles
    u32x4 rp[PV], rd[UP ? 1 : DV];
    u32x2 ra[1];
    auto load_tile = [&](int t) {
        int tv = tid;
        asm volatile("" : "+v"(tv));  // opaque copy: keeps the slot arithmetic inside the loop
        const int img = (int)fdiv((uint32_t)t, a.dTimg);
        const int rem = t - img * a.tiles_img;
        const int tyi = (int)fdiv((uint32_t)rem, a.dTx);
        const int oh0 = tyi * a.TH, ow0 = (rem - tyi * a.tiles_x) * a.TWr;
        const int ih0 = oh0 - g.ph, iw0 = ow0 - g.pw;
        const unsigned xbase = (unsigned)(img * g.H * g.W * g.C + c0 + (tv & 7) * 8);
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            const int q = (tv >> 3) + i * (NT / 8);
            const int py = (int)fdiv((uint32_t)q, a.dPWp), px = q - py * a.PWp;
            const int ih = ih0 + py, iw = iw0 + px;
            const bool ok = q < a.patch_len && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
            const unsigned off = (xbase + (unsigned)((ih * g.W + iw) * g.C)) * 2u;
            rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcX, ok ? off : OOB, 0, 0);
        }
        if (UP) {
            const int unit = tv / DVP;
            const int uy = (int)fdiv((uint32_t)unit, a.dVW2), ux = unit - uy * a.VW2;
            const bool ok = 2 * uy < a.TH && 2 * ux < a.TWr && oh0 + 2 * uy < g.P;
            const unsigned el =  // pooled element
                (unsigned)(((img * a.P2 + (oh0 >> 1) + uy) * a.Q2 + (ow0 >> 1) + ux) * g.K + ko0 + (tv % DVP) * 8);
            rd[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrcD, ok ? el * 2u : OOB, 0, 0);
            ra[0] = __builtin_amdgcn_raw_buffer_load_b64(rsrcM, ok ? el : OOB, 0, 0);
        } else {
            const unsigned dbase = (unsigned)(((img * g.P + oh0) * g.Q + ow0) * g.K + ko0 + (tv % DVP) * 8);
#pragma unroll
            for (int i = 0; i < DV; ++i) {
                const int q = tv / DVP + i * (NT / DVP);
                const int ty = (int)fdiv((uint32_t)q, a.dVW), tx = q - ty * a.VW;
                const bool ok = ty < a.TH && tx < a.TWr && oh0 + ty < g.P;
                const unsigned off = (dbase + (unsigned)((ty * g.Q + tx) * g.K)) * 2u;
                rd[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcD, ok ? off : OOB, 0, 0);
            }
        }
    };
    // rows [0, patch_len) of the patch and [0, 16 * nk16) of the dy tile are (re)written for every tile, so
    // every row the MFMA loop reads holds either data or zeros
    auto store_tile = [&](int buf) {
        unsigned char* sX = smem + buf * a.buf_bytes;
        unsigned char* sD = sX + a.d_off;
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            const int q = (tid >> 3) + i * (NT / 8);
            if (q < a.patch_len) *reinterpret_cast<u32x4*>(sX + q * XPITCH + (tid & 7) * 16) = rp[i];
        }
        if (UP) {
            int tv = tid;
            asm volatile("" : "+v"(tv));  // opaque copy: the window's row addresses are recomputed per tile, not kept
            const int unit = tv / DVP;
            const int uy = (int)fdiv((uint32_t)unit, a.dVW2), ux = unit - uy * a.VW2;
            if (unit < a.units) {
#pragma unroll
                for (int pos = 0; pos < 4; ++pos) {
                    const int q = (2 * uy + (pos >> 1)) * a.VW + 2 * ux + (pos & 1);
                    if (q < a.nk16 * 16)
                        *reinterpret_cast<u32x4*>(sD + q * DPITCH + (tv % DVP) * 16) =
                            unpool_select8(rd[0], ra[0], (unsigned)pos);
                    __builtin_amdgcn_sched_barrier(0);  // one pixel at a time: four selected copies at once do not fit
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < DV; ++i) {
                const int q = tid / DVP + i * (NT / DVP);
                if (q < a.nk16 * 16) *reinterpret_cast<u32x4*>(sD + q * DPITCH + (tid % DVP) * 16) = rd[i];
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

    // transposing read: lane supplies the address of reduction row (lane / 32) * 8 + (lane % 16) / 4 (+ 4 for the
    // second read) and of the 4-channel chunk ((lane / 16) % 2) * 16 + (lane % 4) * 4 of its 32-channel block
    const int kl = (lane >> 5) * 8 + ((lane & 15) >> 2);
    const int chunk = (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    const int xfix = r * a.PWp * XPITCH + cb * 64 + chunk;
    // first reduction step: virtual pixels kl and kl + 4 -> (row, column) -> patch offset
    const int row_a = (int)fdiv((uint32_t)kl, a.dVW), col_a = kl - row_a * a.VW;
    const int row_b = (int)fdiv((uint32_t)(kl + 4), a.dVW), col_b = kl + 4 - row_b * a.VW;
    const int xoff_a = (row_a * a.PWp + col_a) * XPITCH + xfix, xoff_b = (row_b * a.PWp + col_b) * XPITCH + xfix;
    const int xmax = ((a.TH - 1) * a.PWp + a.VW - 1) * XPITCH + xfix;  // last virtual pixel of the tile
    const int dfix = a.d_off + kl * DPITCH + kh * (FD * 64) + chunk;

    if (t0 < t1) {
        load_tile(t0);
        store_tile(0);
        if (t0 + 1 < t1) load_tile(t0 + 1);
    }
    __syncthreads();
    for (int t = t0; t < t1; ++t) {
        const int buf = (t - t0) & 1;
        // tile t+1 (in registers since the previous iteration) -> the other buffer, whose last readers finished
        // before the barrier that ended the previous iteration; then tile t+2 goes in flight
        if (t + 1 < t1) store_tile(buf ^ 1);
        if (t + 2 < t1) load_tile(t + 2);
        const unsigned char* sB = smem + buf * a.buf_bytes;
        // virtual pixel -> patch row, kept incrementally: 16 pixels further per step, at most one row wrap (VW >= 16)
        int cx0 = col_a, cx1 = col_b, xo0 = xoff_a, xo1 = xoff_b, dof = dfix;
#pragma unroll 2
        for (int ks = 0; ks < a.nk16; ++ks) {
            const unsigned char* x0 = sB + xo0;
            const unsigned char* x1 = sB + xo1;
            const unsigned char* d0 = sB + dof;
            const unsigned char* d1 = d0 + 4 * DPITCH;
            cx0 += 16; xo0 += 16 * XPITCH; dof += 16 * DPITCH;
            cx1 += 16; xo1 += 16 * XPITCH;
            if (cx0 >= a.VW) { cx0 -= a.VW; xo0 += 2 * XPITCH; }
            if (cx1 >= a.VW) { cx1 -= a.VW; xo1 += 2 * XPITCH; }
            if (xo0 > xmax) xo0 = xmax;  // zero-dy tail of a tile whose size is not a multiple of 16: stay on written rows
            if (xo1 > xmax) xo1 = xmax;
            bf16x8 fd[FD], fx[3];
#pragma unroll
            for (int kb = 0; kb < FD; ++kb) fd[kb] = tr_pair(d0 + kb * 64, d1 + kb * 64);
#pragma unroll
            for (int s = 0; s < 3; ++s) fx[s] = tr_pair(x0 + s * XPITCH, x1 + s * XPITCH);
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int kb = 0; kb < FD; ++kb)
                    acc[s][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[s], fd[kb], acc[s][kb], 0, 0, 0);
        }
        __syncthreads();  // tile t is consumed and tile t+1 is complete in the other buffer
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
    int TH, TWr, VW;
};

int fd_for(const WgradGeom& g) { return (g.K % 128) == 0 ? 2 : 1; }
size_t buf_bytes_for(int fd, int patch_len, int nk16) {
    return (size_t)patch_len * XPITCH + (size_t)nk16 * 16 * (fd * 128 + 64);
}

// Most real pixels per tile (the tile height need not divide the map: the last tile row of an image is then partly
// masked) among the tiles whose two LDS buffers fit; then the least padding.
bool choose_tile(const WgradGeom& g, TileShape* out) {
    const int fd = fd_for(g);
    long best = 0;
    for (int twr = 1; twr <= g.Q && twr <= 32; ++twr) {
        if (g.Q % twr) continue;
        const int vw = twr <= 16 ? 16 : (twr + 3) / 4 * 4;  // the kernel's row stepping needs at least 16 columns
        for (int th = 1; th <= g.P; ++th) {
            const int tiles_y = (g.P + th - 1) / th;
            const int npix = th * vw, padded = (npix + 15) / 16 * 16, patch = (th + 2) * (vw + 2);
            if (npix > DCAP || patch > PCAP) break;
            if (2 * buf_bytes_for(fd, patch, padded / 16) > LDS_BYTES) break;
            long score = (long)g.P * twr * 1024 / tiles_y + (1023 - (padded - th * twr));
            if (score > best) {
                best = score;
                *out = {th, twr, vw};
            }
        }
    }
    return best > 0;
}

}  // namespace

bool wgrad_patch_supported(const WgradGeom& g) {
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1) return false;
    if ((g.C % 64) != 0 || (g.K % 64) != 0) return false;
    if ((size_t)g.N * g.H * g.W * g.C * 2 >= (1ull << 31) || (size_t)g.N * g.P * g.Q * g.K * 2 >= (1ull << 31)) return false;
    TileShape ts;
    if (!choose_tile(g, &ts)) return false;
    return ts.TH * ts.TWr >= 64;  // tiny tiles: the generic kernel is no worse
}

const char* wgrad_patch_kernel_name(const WgradGeom& g, bool unpool) {
    if (unpool) return fd_for(g) == 2 ? "wgrad_patch_kernel<2,true>" : "wgrad_patch_kernel<1,true>";
    return fd_for(g) == 2 ? "wgrad_patch_kernel<2,false>" : "wgrad_patch_kernel<1,false>";
}

// dy given as the gradient of the 2x2 / stride-2 pooled output plus the argmax: whole windows only
static int unpool_units(const TileShape& ts) {  // windows of (2 rows x 2 columns) covering every row of the padded dy tile
    const int rows16 = (ts.TH * ts.VW + 15) / 16 * 16;
    return (rows16 + 2 * ts.VW - 1) / (2 * ts.VW) * (ts.VW / 2);
}
bool wgrad_patch_fuses_unpool(const WgradGeom& g) {
    TileShape ts;
    if (!wgrad_patch_supported(g) || (g.P % 2) != 0 || (g.Q % 2) != 0 || !choose_tile(g, &ts)) return false;
    if ((ts.TH % 2) != 0 || (ts.TWr % 2) != 0) return false;  // windows must not straddle tiles
    return unpool_units(ts) * (64 * fd_for(g) / 8) <= NT;      // one window vector per thread
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

int launch_wgrad_patch(const WgradGeom& g, int nsplit, const bf16_t* x, const bf16_t* dy, float* out, hipStream_t st,
                       const uint8_t* unpool_am) {
    WPArgs wa;
    TileShape ts;
    if (!wgrad_patch_supported(g) || !choose_tile(g, &ts))
        return set_error(WAP_EINVAL, "internal: patch weight-gradient kernel not applicable");
    if (unpool_am && !wgrad_patch_fuses_unpool(g))
        return set_error(WAP_EINVAL, "internal: fused max-pool backward not available for this shape");
    const int fd = fd_for(g);
    wa.am = unpool_am;
    wa.P2 = g.P / 2;
    wa.Q2 = g.Q / 2;
    wa.VW2 = ts.VW / 2;
    wa.units = unpool_units(ts);
    wa.dVW2 = make_fastdiv((uint32_t)wa.VW2);
    wa.x = x;
    wa.dy = dy;
    wa.out = out;
    wa.g = g;
    wa.Kred = g.R * g.S * g.C;
    wa.TH = ts.TH;
    wa.TWr = ts.TWr;
    wa.VW = ts.VW;
    wa.PWp = ts.VW + 2;
    wa.patch_len = (ts.TH + 2) * wa.PWp;
    wa.npix = ts.TH * ts.VW;
    wa.nk16 = (wa.npix + 15) / 16;
    wa.tiles_x = g.Q / ts.TWr;
    wa.tiles_img = wa.tiles_x * ((g.P + ts.TH - 1) / ts.TH);
    wa.tiles_total = wa.tiles_img * g.N;
    wa.kgroups = g.K / (64 * fd);
    wa.ncombo = wa.kgroups * (g.C / 64);
    wa.nsplit = nsplit;
    wa.tiles_per_split = (wa.tiles_total + nsplit - 1) / nsplit;
    wa.d_off = wa.patch_len * XPITCH;
    wa.buf_bytes = (int)buf_bytes_for(fd, wa.patch_len, wa.nk16);
    wa.x_bytes = (unsigned)((size_t)g.N * g.H * g.W * g.C * 2);
    wa.dy_bytes = (unsigned)((size_t)g.N * g.P * g.Q * g.K * 2 / (unpool_am ? 4 : 1));
    wa.dVW = make_fastdiv((uint32_t)wa.VW);
    wa.dPWp = make_fastdiv((uint32_t)wa.PWp);
    wa.dTimg = make_fastdiv((uint32_t)wa.tiles_img);
    wa.dTx = make_fastdiv((uint32_t)wa.tiles_x);
    const size_t smem = 2 * (size_t)wa.buf_bytes;
    if (smem > LDS_BYTES) return set_error(WAP_EINVAL, "internal: patch weight-gradient tile does not fit LDS");
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        for (const void* f : {(const void*)wgrad_patch_kernel<1, false>, (const void*)wgrad_patch_kernel<2, false>,
                              (const void*)wgrad_patch_kernel<1, true>, (const void*)wgrad_patch_kernel<2, true>}) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
            if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        }
        attr_done = true;
    }
    const dim3 grid(wa.ncombo * nsplit);
    if (unpool_am) {
        if (fd == 1) hipLaunchKernelGGL((wgrad_patch_kernel<1, true>), grid, dim3(NT), smem, st, wa);
        else hipLaunchKernelGGL((wgrad_patch_kernel<2, true>), grid, dim3(NT), smem, st, wa);
    } else {
        if (fd == 1) hipLaunchKernelGGL((wgrad_patch_kernel<1, false>), grid, dim3(NT), smem, st, wa);
        else hipLaunchKernelGGL((wgrad_patch_kernel<2, false>), grid, dim3(NT), smem, st, wa);
    }
    return check_launch("wgrad_patch");
}

}  // namespace wap
