// Forward-type implicit GEMM on bf16 MFMA (gfx950): rows = output pixels (gathered from an NHWC
// tensor), columns = output channels, reduction = filter taps x input channels.
//
// Serves the convolution forward pass, the convolution data gradient (rows = input pixels,
// gathered from dy; the weights are read with flipped taps and transposed through LDS) and both
// FC products that keep the batch as the row dimension (Section 3.2.2 "primary" nodes; the
// forward / backward halves of t_c in Eq. 1).
//
// Design for CDNA4:
//   * block tile BM x BN x 64, 64-wide wavefronts each owning a (BM/WAVES_M) x (BN/WAVES_N)
//     sub-tile built from v_mfma_f32_32x32x16_bf16; the weight fragment is the MFMA "A" operand so
//     that each lane ends up with 4 consecutive output channels of one pixel (8-byte bf16 stores);
//   * operands staged through LDS, two stages; the next tile's global loads are issued before the
//     current tile's MFMAs and written to the other stage afterwards (one barrier per tile);
//   * LDS rows padded (144 B for reduction-contiguous tiles, +64 B for channel-contiguous tiles) so
//     ds_read_b128 / ds_read_b64_tr_b16 fragment reads are bank-conflict free;
//   * channel-contiguous weight tiles (data gradient) are transposed on the way out of LDS with
//     ds_read_b64_tr_b16 instead of a separate transpose pass over the weights;
//   * blockIdx is remapped so that each XCD (own L2) works on a contiguous range of tiles.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64;
constexpr int A_PITCH = (BK + 8) * 2;  // bytes per LDS row of a reduction-contiguous tile

struct KArgs {
    const bf16_t* A;
    const bf16_t* Bw;
    const float* bias;
    void* out;
    GemmGeom g;
    int tiles_m, tiles_n, nsplit, ktiles, ktiles_per_split;
    int relu, partial;
};

__device__ __forceinline__ int xcd_remap(int bid, int total) {
    int per = total / kNumXCD, rem = total % kNumXCD;
    int xcd = bid % kNumXCD, idx = bid / kNumXCD;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

__device__ __forceinline__ u32x4 ld16(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

// Out-of-image taps and tile tails load from this zero block instead of being masked after the load:
// the loaded registers then have no consumer until the LDS store that follows the MFMAs, so the
// global-load latency overlaps the current tile's compute.
__device__ __align__(16) unsigned int g_zero_block[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ unsigned short f2bf(float f) {
    __bf16 b = (__bf16)f;  // round to nearest even
    return __builtin_bit_cast(unsigned short, b);
}

__device__ __forceinline__ u32x4 pack8(const unsigned short* h) {
    u32x4 v = {(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16),
               (unsigned)h[4] | ((unsigned)h[5] << 16), (unsigned)h[6] | ((unsigned)h[7] << 16)};
    return v;
}

// MODE 0: fast  -- channel counts multiples of 64 / 8, unit tap divisor, 16-byte loads, one tap per tile
// MODE 1: vec   -- channel counts multiples of 8, any geometry
// MODE 2: scalar-- anything (2-byte loads)
template <int BM, int BN, int WAVES_M, int WAVES_N, bool B_TR, int MODE>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void igemm_kernel(const KArgs a) {
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int A_RPP = NT / 8, A_PASSES = BM / A_RPP;
    constexpr int B_PITCH = B_TR ? (BN * 2 + 64) : A_PITCH;
    constexpr int B_VPR = B_TR ? BN / 8 : 8;  // 16-byte vectors per LDS row
    constexpr int B_RPP = NT / B_VPR;
    constexpr int B_ROWS = B_TR ? BK : BN;
    constexpr int B_PASSES = B_ROWS / B_RPP;
    constexpr int A_BYTES = BM * A_PITCH;
    constexpr int B_BYTES = B_ROWS * B_PITCH;
    constexpr int STAGE = A_BYTES + B_BYTES;
    static_assert(A_PASSES >= 1 && B_PASSES >= 1, "tile too small for the block");

    extern __shared__ __align__(16) unsigned char smem[];

    const GemmGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;

    const int total = a.tiles_m * a.tiles_n * a.nsplit;
    int logical = xcd_remap(blockIdx.x, total);
    const int tn = logical % a.tiles_n;
    logical /= a.tiles_n;
    const int tm = logical % a.tiles_m;
    const int split = logical / a.tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;
    const int kt_begin = split * a.ktiles_per_split;
    int kt_end = kt_begin + a.ktiles_per_split;
    if (kt_end > a.ktiles) kt_end = a.ktiles;

    // ---- per-thread row state of the gathered operand ----
    const int a_vec = tid & 7, a_row0 = tid >> 3;
    int hb[A_PASSES], wb[A_PASSES], abase[A_PASSES];
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
        int m = m0 + a_row0 + i * A_RPP;
        if (m < g.M) {
            int ow = m % g.OW;
            int t = m / g.OW;
            int oh = t % g.OH;
            int n = t / g.OH;
            hb[i] = oh * g.mul_h - g.pad_h;
            wb[i] = ow * g.mul_w - g.pad_w;
            abase[i] = n * g.IH * g.IW * g.IC;
        } else {
            hb[i] = -(1 << 28);
            wb[i] = -(1 << 28);
            abase[i] = 0;
        }
    }
    const int b_vec = tid % B_VPR, b_row0 = tid / B_VPR;

    u32x4 ra[A_PASSES], rb[B_PASSES];
    const bf16_t* zero_src = reinterpret_cast<const bf16_t*>(g_zero_block);

    auto tap_ok = [&](int th, int tw, int& ih, int& iw) -> bool {
        if (MODE == 0) {
            ih = th;
            iw = tw;
            return (unsigned)th < (unsigned)g.IH && (unsigned)tw < (unsigned)g.IW;
        } else {
            if (th < 0 || tw < 0) return false;
            ih = th / g.div_h;
            iw = tw / g.div_w;
            return (ih * g.div_h == th) && (iw * g.div_w == tw) && ih < g.IH && iw < g.IW;
        }
    };

    auto load_global = [&](int kt) {
        // Fast mode walks the reduction channel-slice-major (all filter taps of one 64-channel slice
        // before the next slice): the 9 (or 25) shifted re-reads of the same input pixels then happen
        // in consecutive tiles and hit in L2 instead of going back to HBM.
        const int RS = g.R * g.S;
        const int kk0 = (MODE == 0) ? ((kt % RS) * g.IC + (kt / RS) * BK) : kt * BK;
        // ---------- gathered operand ----------
        if (MODE <= 1) {
            int kk = (MODE == 0) ? kk0 : kk0 + a_vec * 8;
            int tap = kk / g.IC;
            int c = kk - tap * g.IC + ((MODE == 0) ? a_vec * 8 : 0);
            int r = tap / g.S, s = tap - r * g.S;
            bool kok = (MODE == 0) ? true : (kk < g.Kred);
#pragma unroll
            for (int i = 0; i < A_PASSES; ++i) {
                int ih, iw;
                bool ok = tap_ok(hb[i] + r, wb[i] + s, ih, iw) && kok;
                int off = abase[i] + (ih * g.IW + iw) * g.IC + c;
                ra[i] = ld16(ok ? a.A + off : zero_src);
            }
        } else {
            int rr[8], ss[8], cc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int kk = kk0 + a_vec * 8 + e;
                int tap = kk / g.IC;
                cc[e] = kk - tap * g.IC;
                rr[e] = tap / g.S;
                ss[e] = tap - rr[e] * g.S;
                if (kk >= g.Kred) rr[e] = -(1 << 20);  // forces the row test to fail
            }
#pragma unroll
            for (int i = 0; i < A_PASSES; ++i) {
                unsigned short h16[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    int ih, iw;
                    bool ok = tap_ok(hb[i] + rr[e], wb[i] + ss[e], ih, iw);
                    int off = abase[i] + (ih * g.IW + iw) * g.IC + cc[e];
                    h16[e] = *(ok ? a.A + off : zero_src);
                }
                ra[i] = pack8(h16);
            }
        }
        // ---------- weight operand ----------
        if (!B_TR) {
            // Bw[n][kk]: LDS row = output channel, 8 vectors of 8 reduction elements per row
            int kk = kk0 + b_vec * 8;
#pragma unroll
            for (int i = 0; i < B_PASSES; ++i) {
                int n = n0 + b_row0 + i * B_RPP;
                if (MODE <= 1) {
                    bool ok = n < g.Ncols && kk < g.Kred;
                    rb[i] = ld16(ok ? a.Bw + (n * g.Kred + kk) : zero_src);
                } else {
                    unsigned short h16[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        bool ok = n < g.Ncols && (kk + e) < g.Kred;
                        h16[e] = *(ok ? a.Bw + (n * g.Kred + kk + e) : zero_src);
                    }
                    rb[i] = pack8(h16);
                }
            }
        } else {
            // Bw[k][R-1-r][S-1-s][n]: LDS row = reduction index (r,s,k), BN/8 vectors of 8 channels
            int n = n0 + b_vec * 8;
#pragma unroll
            for (int i = 0; i < B_PASSES; ++i) {
                int kk = kk0 + b_row0 + i * B_RPP;
                int tap = (MODE == 0) ? kk0 / g.IC : kk / g.IC;  // one tap per tile in the fast mode
                int k = kk - tap * g.IC;
                int r = tap / g.S, s = tap - r * g.S;
                int rowoff = ((k * g.R + (g.R - 1 - r)) * g.S + (g.S - 1 - s)) * g.Ncols;
                if (MODE <= 1) {
                    bool ok = kk < g.Kred && n < g.Ncols;
                    rb[i] = ld16(ok ? a.Bw + (rowoff + n) : zero_src);
                } else {
                    unsigned short h16[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        bool ok = kk < g.Kred && (n + e) < g.Ncols;
                        h16[e] = *(ok ? a.Bw + (rowoff + n + e) : zero_src);
                    }
                    rb[i] = pack8(h16);
                }
            }
        }
    };

    auto store_lds = [&](int stage) {
        unsigned char* sA = smem + stage * STAGE;
        unsigned char* sB = sA + A_BYTES;
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i)
            *reinterpret_cast<u32x4*>(sA + (a_row0 + i * A_RPP) * A_PITCH + a_vec * 16) = ra[i];
#pragma unroll
        for (int i = 0; i < B_PASSES; ++i)
            *reinterpret_cast<u32x4*>(sB + (b_row0 + i * B_RPP) * B_PITCH + b_vec * 16) = rb[i];
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    auto compute = [&](int stage) {
        const unsigned char* sA = smem + stage * STAGE;
        const unsigned char* sB = sA + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[FM], fw[FN];
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                int row = wm * WM + j * 32 + (lane & 31);
                fa[j] = *reinterpret_cast<const bf16x8*>(sA + row * A_PITCH + (ks * 2 + (lane >> 5)) * 16);
            }
#pragma unroll
            for (int i = 0; i < FN; ++i) {
                if (!B_TR) {
                    int row = wn * WN + i * 32 + (lane & 31);
                    fw[i] = *reinterpret_cast<const bf16x8*>(sB + row * B_PITCH + (ks * 2 + (lane >> 5)) * 16);
                } else {
                    int col = wn * WN + i * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
                    int krow = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
                    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4_ptr)(sB + krow * B_PITCH + col * 2));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4_ptr)(sB + (krow + 4) * B_PITCH + col * 2));
                    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    fw[i] = __builtin_bit_cast(bf16x8, both);
                }
            }
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int j = 0; j < FM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
    };

    if (kt_begin < kt_end) {
        // Each work-group starts its walk over the reduction tiles at a different offset (and wraps):
        // work-groups running at the same time then read different channel slices and filter taps,
        // which spreads their requests over the L2 channels instead of hammering the same few.
        const int nkt = kt_end - kt_begin;
        int cur = kt_begin + (int)(((unsigned)blockIdx.x / kNumXCD * 5u) % (unsigned)nkt);
        load_global(cur);
        store_lds(0);
        __syncthreads();
        for (int it = 0; it < nkt; ++it) {
            const int stage = it & 1;
            const bool more = (it + 1 < nkt);
            int nxt = cur + 1;
            if (nxt == kt_end) nxt = kt_begin;
            if (more) load_global(nxt);
            compute(stage);
            if (more) store_lds(stage ^ 1);
            __syncthreads();
            cur = nxt;
        }
    }

    // ---- epilogue: lane holds 4 consecutive channels of one pixel per register quad ----
    const bool vec4 = (g.Ncols & 3) == 0;
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int m = m0 + wm * WM + j * 32 + (lane & 31);
        if (m >= g.M) continue;
#pragma unroll
        for (int i = 0; i < FN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + i * 32 + q * 8 + (lane >> 5) * 4;
                if (n >= g.Ncols) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
                if (a.partial) {
                    float* o = reinterpret_cast<float*>(a.out) + ((size_t)split * g.M + m) * g.Ncols + n;
                    if (vec4) {
                        *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < g.Ncols) o[e] = v[e];
                    }
                } else {
                    if (a.bias) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < g.Ncols) v[e] += a.bias[n + e];
                    }
                    if (a.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                    }
                    bf16_t* o = reinterpret_cast<bf16_t*>(a.out) + (size_t)m * g.Ncols + n;
                    unsigned short hb16[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) hb16[e] = f2bf(v[e]);
                    if (vec4) {
                        *reinterpret_cast<uint2*>(o) = make_uint2((unsigned)hb16[0] | ((unsigned)hb16[1] << 16),
                                                                  (unsigned)hb16[2] | ((unsigned)hb16[3] << 16));
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < g.Ncols) o[e] = hb16[e];
                    }
                }
            }
        }
    }
}

// ---- tile configurations ----
struct Cfg {
    int BM, BN, NT;
};
constexpr Cfg kCfgs[] = {
    {256, 256, 512},  // 0: large
    {128, 128, 256},  // 1: medium / general
    {64, 256, 256},   // 2: few rows (small-batch FC)
    {256, 64, 256},   // 3: few output channels
    {256, 256, 256},  // 4: large, 4 wavefronts of 128x128 (less LDS traffic per MFMA)
    {256, 256, 256},  // 5: large, weights in registers (conv_wreg.hip)
    {224, 256, 256},  // 6: stride-1 multi-tap conv, input patch in LDS (conv_patch.hip)
    {256, 64, 256},   // 7: stride-1 multi-tap conv, 8 x 32-pixel tiles, 64 / 128 channels (conv_tile2d.hip)
};

size_t smem_bytes(const Cfg& c, bool b_tr) {
    size_t a = (size_t)c.BM * A_PITCH;
    size_t b = b_tr ? (size_t)BK * (c.BN * 2 + 64) : (size_t)c.BN * A_PITCH;
    return 2 * (a + b);
}

template <int BM, int BN, int WMv, int WNv, bool B_TR, int MODE>
int launch_one(const KArgs& ka, size_t smem, hipStream_t st) {
    auto kfn = igemm_kernel<BM, BN, WMv, WNv, B_TR, MODE>;
    static std::atomic<bool> attr_done{false};  // one attribute call per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    int total = ka.tiles_m * ka.tiles_n * ka.nsplit;
    hipLaunchKernelGGL(kfn, dim3(total), dim3(64 * WMv * WNv), smem, st, ka);
    return check_launch("igemm");
}

int classify_mode(const GemmGeom& g, bool b_tr) {
    bool vec_a = (g.IC % 8) == 0;
    bool vec_b = b_tr ? (g.Ncols % 8) == 0 : (g.Kred % 8) == 0;
    if (!(vec_a && vec_b)) return 2;
    if ((g.IC % BK) == 0 && g.div_h == 1 && g.div_w == 1) return 0;
    return 1;
}

}  // namespace

GemmPlan plan_fwd_like(const GemmGeom& g, bool b_tr) {
    GemmPlan p;
    if (!b_tr && (g_force_fwd_cfg < 0 || g_force_fwd_cfg == 8) && conv_c3_fwd_supported(g)) {
        p.cfg = 8;
        p.nsplit = 1;
        p.ws_bytes = 0;
        return p;
    }
    if (b_tr && (g_force_fwd_cfg < 0 || g_force_fwd_cfg == 9) && dgrad_thin_supported(g)) {
        p.cfg = 9;  // at most four output columns (gradient w.r.t. a 3-channel image): vector-ALU kernel
        p.nsplit = 1;
        p.ws_bytes = dgrad_thin_ws_bytes(g);
        return p;
    }
    int mode = classify_mode(g, b_tr);
    int ktiles = (g.Kred + BK - 1) / BK;
    auto tiles = [&](int c) {
        return (long)((g.M + kCfgs[c].BM - 1) / kCfgs[c].BM) * ((g.Ncols + kCfgs[c].BN - 1) / kCfgs[c].BN);
    };
    int cfg;
    if (mode != 0) {
        cfg = 1;
    } else if (g.Ncols <= 64) {
        cfg = 3;
    } else if (g.M <= 64) {
        cfg = 2;
    } else if (tiles(0) >= 200 && g.Ncols >= 192) {
        cfg = wreg_supported(g) ? 5 : 0;
    } else {
        cfg = 1;
    }
    if (g_force_fwd_cfg >= 0 && g_force_fwd_cfg < 8 && (mode == 0 || g_force_fwd_cfg == 1)) cfg = g_force_fwd_cfg;
    long t = tiles(cfg);
    int nsplit = 1;
    // split the reduction when the tiles alone leave most CUs idle
    if (t < kNumCU * 3 / 4 && ktiles >= 8) {
        // about one work-group per CU in all (measured on the FC head: more splits only add partial-tile traffic and a
        // longer epilogue), at least 4 reduction tiles per split
        long want = kNumCU / t;
        long maxs = ktiles / 4;
        nsplit = (int)(want < maxs ? want : maxs);
        if (nsplit < 1) nsplit = 1;
        if (nsplit > 64) nsplit = 64;
    }
    if (g_force_nsplit >= 1) nsplit = g_force_nsplit < ktiles ? g_force_nsplit : ktiles;
    int kps = (ktiles + nsplit - 1) / nsplit;
    nsplit = (ktiles + kps - 1) / kps;
    if (cfg == 5 && !wreg_supported(g)) cfg = 0;
    if (g_force_fwd_cfg < 0 && patch_supported(g)) cfg = 6;
    if (cfg == 6 && !patch_supported(g)) cfg = 1;
    if (g_force_fwd_cfg < 0 && tile2d_preferred(g)) cfg = 7;
    if (cfg == 7 && !tile2d_supported(g)) cfg = 1;
    if (cfg == 6 || cfg == 7) nsplit = 1;
    p.cfg = cfg;
    p.nsplit = nsplit;
    p.ws_bytes = nsplit > 1 ? (size_t)nsplit * g.M * g.Ncols * sizeof(float) : 0;
    if (cfg >= 5) p.ws_bytes += wreg_wt_bytes(g);  // weights repacked into MFMA fragment order
    return p;
}

int launch_fwd_like(const GemmGeom& g, bool b_tr, const GemmPlan& plan, const bf16_t* A,
                    const bf16_t* Bw, const float* bias, bool relu, bf16_t* out, void* ws,
                    hipStream_t st, hipEvent_t ev_mid, const bf16_t* relu_mask, hipEvent_t ev_packed,
                    const void* prepacked, bf16_t* pool_y, uint8_t* pool_am, const uint8_t* unpool_am, float* colsum) {
    if (colsum && (fwd_like_colsum_rows(g, plan) == 0 || pool_y))
        return set_error(WAP_EINVAL, "internal: fused column sums not available for this plan");
    if ((pool_y || pool_am) && !(pool_y && pool_am && fwd_like_fuses_pool(g, plan)))
        return set_error(WAP_EINVAL, "internal: fused pooling not available for this plan");
    if (unpool_am && !fwd_like_fuses_unpool(g, plan))
        return set_error(WAP_EINVAL, "internal: fused max-pool backward not available for this plan");
    if (relu_mask && !fwd_like_fuses_mask(g, plan)) {
        // no fused epilogue for this tile configuration: plain product, then the element-wise mask
        int rc = launch_fwd_like(g, b_tr, plan, A, Bw, bias, relu, out, ws, st, ev_mid, nullptr, ev_packed, prepacked);
        if (rc != WAP_OK) return rc;
        return launch_relu_bwd(out, relu_mask, out, (size_t)g.M * g.Ncols, st);
    }
    if (plan.cfg == 8) return launch_conv_c3_fwd(g, A, Bw, bias, relu, out, st);
    if (plan.cfg == 9) return launch_dgrad_thin(g, A, Bw, out, ws, st);
    KArgs ka;
    ka.A = A;
    ka.Bw = Bw;
    ka.g = g;
    const Cfg& c = kCfgs[plan.cfg < 5 ? plan.cfg : 0];
    ka.tiles_m = (g.M + c.BM - 1) / c.BM;
    ka.tiles_n = (g.Ncols + c.BN - 1) / c.BN;
    ka.ktiles = (g.Kred + BK - 1) / BK;
    ka.nsplit = plan.nsplit;
    ka.ktiles_per_split = (ka.ktiles + plan.nsplit - 1) / plan.nsplit;
    ka.partial = plan.nsplit > 1;
    ka.bias = ka.partial ? nullptr : bias;
    ka.relu = ka.partial ? 0 : (relu ? 1 : 0);
    ka.out = ka.partial ? ws : (void*)out;
    if (plan.cfg == 6 || plan.cfg == 7) {
        const void* wp = prepacked;
        if (!wp) {
            int rc0 = launch_pack_weights(g, b_tr, Bw, ws, st);
            if (rc0 != WAP_OK) return rc0;
            wp = ws;
        }
        if (ev_packed) (void)hipEventRecord(ev_packed, st);
        return plan.cfg == 6 ? launch_patch(g, A, wp, bias, relu, out, st, relu_mask)
                             : launch_tile2d(g, A, wp, bias, relu, out, st, relu_mask, pool_y, pool_am, unpool_am, colsum);
    }
    if (plan.cfg == 5) {
        // the (small) weight tensor is first repacked into MFMA fragment order (taps flipped and
        // transposed for the data gradient); the partial tiles, if any, follow it in the workspace
        int rc0 = launch_pack_weights(g, b_tr, Bw, ws, st);
        if (rc0 != WAP_OK) return rc0;
        if (ev_packed) (void)hipEventRecord(ev_packed, st);
        void* part = reinterpret_cast<unsigned char*>(ws) + wreg_wt_bytes(g);
        int rc5 = launch_wreg(g, plan.nsplit, A, reinterpret_cast<const bf16_t*>(ws), bias, relu,
                              ka.partial ? part : (void*)out, ka.partial != 0, st);
        if (rc5 != WAP_OK) return rc5;
        if (ev_mid) (void)hipEventRecord(ev_mid, st);
        if (ka.partial)
            return launch_reduce_bf16(reinterpret_cast<const float*>(part), plan.nsplit, (size_t)g.M * g.Ncols,
                                      g.Ncols, bias, relu, out, st);
        return WAP_OK;
    }
    size_t smem = smem_bytes(c, b_tr);
    int mode = classify_mode(g, b_tr);
    int rc;
#define WAP_DISPATCH(BM, BN, WMv, WNv)                                                     \
    (b_tr ? (mode == 0 ? launch_one<BM, BN, WMv, WNv, true, 0>(ka, smem, st)                \
                       : mode == 1 ? launch_one<BM, BN, WMv, WNv, true, 1>(ka, smem, st)    \
                                   : launch_one<BM, BN, WMv, WNv, true, 2>(ka, smem, st))   \
          : (mode == 0 ? launch_one<BM, BN, WMv, WNv, false, 0>(ka, smem, st)               \
                       : mode == 1 ? launch_one<BM, BN, WMv, WNv, false, 1>(ka, smem, st)   \
                                   : launch_one<BM, BN, WMv, WNv, false, 2>(ka, smem, st)))
    if (plan.cfg == 0) {
        if (mode != 0) return set_error(WAP_EINVAL, "internal: large tile needs the fast mode");
        rc = b_tr ? launch_one<256, 256, 2, 4, true, 0>(ka, smem, st)
                  : launch_one<256, 256, 2, 4, false, 0>(ka, smem, st);
    } else if (plan.cfg == 4) {
        if (mode != 0) return set_error(WAP_EINVAL, "internal: large tile needs the fast mode");
        rc = b_tr ? launch_one<256, 256, 2, 2, true, 0>(ka, smem, st)
                  : launch_one<256, 256, 2, 2, false, 0>(ka, smem, st);
    } else if (plan.cfg == 1) {
        rc = WAP_DISPATCH(128, 128, 2, 2);
    } else if (plan.cfg == 2) {
        if (mode != 0) return set_error(WAP_EINVAL, "internal: row-thin tile needs the fast mode");
        rc = b_tr ? launch_one<64, 256, 1, 4, true, 0>(ka, smem, st)
                  : launch_one<64, 256, 1, 4, false, 0>(ka, smem, st);
    } else {
        if (mode != 0) return set_error(WAP_EINVAL, "internal: channel-thin tile needs the fast mode");
        rc = b_tr ? launch_one<256, 64, 4, 1, true, 0>(ka, smem, st)
                  : launch_one<256, 64, 4, 1, false, 0>(ka, smem, st);
    }
#undef WAP_DISPATCH
    if (rc != WAP_OK) return rc;
    if (ev_mid) (void)hipEventRecord(ev_mid, st);
    if (ka.partial)
        return launch_reduce_bf16(reinterpret_cast<const float*>(ws), plan.nsplit,
                                  (size_t)g.M * g.Ncols, g.Ncols, bias, relu, out, st);
    return WAP_OK;
}

}  // namespace wap

namespace wap {
bool fwd_like_packs_weights(const GemmPlan& plan) { return plan.cfg == 5 || plan.cfg == 6 || plan.cfg == 7; }
bool fwd_like_fuses_pool(const GemmGeom& g, const GemmPlan& plan) {
    return plan.cfg == 7 && (g.OH % 2) == 0 && (g.OW % 2) == 0 && tile2d_fuses_pool(g);
}
bool fwd_like_fuses_unpool(const GemmGeom& g, const GemmPlan& plan) { return plan.cfg == 7 && tile2d_fuses_unpool(g); }
int fwd_like_colsum_rows(const GemmGeom& g, const GemmPlan& plan) {
    return plan.cfg == 7 && (g.Ncols % 8) == 0 ? tile2d_colsum_rows(g) : 0;
}
bool fwd_like_fuses_mask(const GemmGeom& g, const GemmPlan& plan) {
    return (plan.cfg == 6 || plan.cfg == 7) && (g.Ncols % 8) == 0;
}
// Label of the kernel instantiation a plan launches (matches the demangled kernel name).
const char* fwd_like_kernel_name(const GemmGeom& g, bool b_tr, const GemmPlan& plan, bool unpool) {
    if (plan.cfg == 5) return "conv_wreg_kernel";
    if (plan.cfg == 6) return patch_kernel_name(g);
    if (plan.cfg == 7) return tile2d_kernel_name(g, unpool);
    if (plan.cfg == 8) return conv_c3_fwd_kernel_name(g);
    if (plan.cfg == 9) return "dgrad_thin_kernel";
    static const char* names[5][2][3] = {
        {{"igemm_kernel<256,256,2,4,false,0>", "", ""}, {"igemm_kernel<256,256,2,4,true,0>", "", ""}},
        {{"igemm_kernel<128,128,2,2,false,0>", "igemm_kernel<128,128,2,2,false,1>", "igemm_kernel<128,128,2,2,false,2>"},
         {"igemm_kernel<128,128,2,2,true,0>", "igemm_kernel<128,128,2,2,true,1>", "igemm_kernel<128,128,2,2,true,2>"}},
        {{"igemm_kernel<64,256,1,4,false,0>", "", ""}, {"igemm_kernel<64,256,1,4,true,0>", "", ""}},
        {{"igemm_kernel<256,64,4,1,false,0>", "", ""}, {"igemm_kernel<256,64,4,1,true,0>", "", ""}},
        {{"igemm_kernel<256,256,2,2,false,0>", "", ""}, {"igemm_kernel<256,256,2,2,true,0>", "", ""}},
    };
    return names[plan.cfg][b_tr ? 1 : 0][classify_mode(g, b_tr)];
}
}  // namespace wap
