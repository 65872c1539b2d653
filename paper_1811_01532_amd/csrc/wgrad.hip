// Weight-gradient implicit GEMM on bf16 MFMA (gfx950):
//   dw[k][(r,s,c)] = sum over pixels (n,p,q) of dy[n,p,q,k] * x[n, p*sh-ph+r, q*sw-pw+s, c]
// (backward half of t_c in Eq. 1; its output is the weight-sized tensor that the gradient
// aggregation of Section 3.2.3 would move).  Also serves the FC weight gradient (R=S=H=W=1).
//
// The reduction index (the pixel) is the slow axis of both operands in memory (NHWC), so both LDS
// tiles are kept channel-contiguous exactly as loaded and are transposed on the way to the MFMA
// with ds_read_b64_tr_b16.  The reduction is split across work-groups (the output is tiny, the
// reduction is N*P*Q long); every split writes an fp32 partial tile and a second kernel adds the
// partials in split order, so results are bitwise reproducible.  The x-column fragment is the MFMA
// "A" operand: each lane then owns 4 consecutive (r,s,c) columns of one output channel; the epilogue
// turns each wavefront's blocks around in LDS so that 16 lanes store one 256-byte run of a row.  With
// a parameter block the epilogue (or the reduction kernel of a split product) applies the SGD update
// with the finished sums instead of storing them.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64;  // pixels per reduction tile

struct WArgs {
    const bf16_t* x;
    const bf16_t* dy;
    float* out;
    WgradGeom g;
    int Kred, Mred;
    int tiles_c, tiles_k, nsplit, ktiles, ktiles_per_split;
    FastDiv dPQ, dQ;
    SgdFuse sgd;  // w32 != NULL (unsplit reduction, Kred % 4 == 0 only): update the parameters instead of storing dW
};

__device__ __forceinline__ int xcd_remap(int bid, int total) {
    int per = total / kNumXCD, rem = total % kNumXCD;
    int xcd = bid % kNumXCD, idx = bid / kNumXCD;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// Masked-out elements load from this zero block (no select after the load, see igemm.hip).
__device__ __align__(16) unsigned int g_zero_block_w[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ u32x4 pack8(const unsigned short* h) {
    u32x4 v = {(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16),
               (unsigned)h[4] | ((unsigned)h[5] << 16), (unsigned)h[6] | ((unsigned)h[7] << 16)};
    return v;
}

__device__ __forceinline__ u32x4 ld16(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

__device__ __forceinline__ bf16x8 tr_frag(const unsigned char* tile, int pitch, int colbase, int ks, int lane) {
    int col = colbase + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    int krow = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + krow * pitch + col * 2));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + (krow + 4) * pitch + col * 2));
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// MODE 0: C % 8 == 0 and K % 8 == 0 (16-byte loads); MODE 1: anything (2-byte loads)
template <int TC, int TK, int WAVES_C, int WAVES_K, int MODE>
__global__ __launch_bounds__(64 * WAVES_C * WAVES_K) void wgrad_kernel(const WArgs a) {
    constexpr int NT = 64 * WAVES_C * WAVES_K;
    constexpr int WC = TC / WAVES_C, WK = TK / WAVES_K;
    constexpr int FC = WC / 32, FK = WK / 32;
    constexpr int X_PITCH = TC * 2 + 64, D_PITCH = TK * 2 + 64;
    constexpr int XV = TC / 8, DV = TK / 8;
    constexpr int X_RPP = NT / XV, D_RPP = NT / DV;
    constexpr int X_PASSES = BK / X_RPP, D_PASSES = BK / D_RPP;
    constexpr int X_BYTES = BK * X_PITCH, D_BYTES = BK * D_PITCH;
    constexpr int STAGE = X_BYTES + D_BYTES;
    static_assert(X_PASSES >= 1 && D_PASSES >= 1, "tile too small for the block");

    extern __shared__ __align__(16) unsigned char smem[];

    const WgradGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WAVES_C, wk = wave / WAVES_C;

    const int total = a.tiles_c * a.tiles_k * a.nsplit;
    int logical = xcd_remap(blockIdx.x, total);
    const int tc = logical % a.tiles_c;
    logical /= a.tiles_c;
    const int tk = logical % a.tiles_k;
    const int split = logical / a.tiles_k;
    const int col0 = tc * TC, ko0 = tk * TK;
    const int kt_begin = split * a.ktiles_per_split;
    int kt_end = kt_begin + a.ktiles_per_split;
    if (kt_end > a.ktiles) kt_end = a.ktiles;

    // ---- fixed per-thread column decode of the x operand ----
    const int x_vec = tid % XV, x_row0 = tid / XV;
    const int d_vec = tid % DV, d_row0 = tid / DV;
    constexpr int NE = (MODE == 0) ? 1 : 8;
    int xr[NE], xs[NE], xc[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        int col = col0 + x_vec * 8 + e;
        if (col < a.Kred) {
            int tap = col / g.C;
            xc[e] = col - tap * g.C;
            xr[e] = tap / g.S;
            xs[e] = tap - xr[e] * g.S;
        } else {
            xc[e] = 0;
            xr[e] = -(1 << 20);  // fails the bounds test for every pixel
            xs[e] = 0;
        }
    }
    const int ko_d = ko0 + d_vec * 8;

    u32x4 rx[X_PASSES], rd[D_PASSES];
    const bf16_t* zero_src = reinterpret_cast<const bf16_t*>(g_zero_block_w);

    auto load_global = [&](int kt) {
        const int pix0 = kt * BK;
#pragma unroll
        for (int i = 0; i < X_PASSES; ++i) {
            int pix = pix0 + x_row0 + i * X_RPP;
            bool pok = pix < a.Mred;
            uint32_t upix = pok ? (uint32_t)pix : 0u;
            int n = (int)fdiv(upix, a.dPQ);
            int rem = (int)upix - n * (g.P * g.Q);
            int p = (int)fdiv((uint32_t)rem, a.dQ);
            int q = rem - p * g.Q;
            int hb = p * g.sh - g.ph, wb = q * g.sw - g.pw;
            int base = n * g.H * g.W * g.C;
            if (MODE == 0) {
                int h = hb + xr[0], w = wb + xs[0];
                bool ok = pok && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                int off = base + (h * g.W + w) * g.C + xc[0];
                rx[i] = ld16(ok ? a.x + off : zero_src);
            } else {
                unsigned short h16[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    int h = hb + xr[e], w = wb + xs[e];
                    bool ok = pok && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
                    int off = base + (h * g.W + w) * g.C + xc[e];
                    h16[e] = *(ok ? a.x + off : zero_src);
                }
                rx[i] = pack8(h16);
            }
        }
#pragma unroll
        for (int i = 0; i < D_PASSES; ++i) {
            int pix = pix0 + d_row0 + i * D_RPP;
            bool pok = pix < a.Mred;
            if (MODE == 0) {
                bool ok = pok && ko_d < g.K;
                rd[i] = ld16(ok ? a.dy + ((size_t)pix * g.K + ko_d) : zero_src);
            } else {
                unsigned short h16[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    bool ok = pok && (ko_d + e) < g.K;
                    h16[e] = *(ok ? a.dy + ((size_t)pix * g.K + ko_d + e) : zero_src);
                }
                rd[i] = pack8(h16);
            }
        }
    };

    auto store_lds = [&](int stage) {
        unsigned char* sX = smem + stage * STAGE;
        unsigned char* sD = sX + X_BYTES;
#pragma unroll
        for (int i = 0; i < X_PASSES; ++i)
            *reinterpret_cast<u32x4*>(sX + (x_row0 + i * X_RPP) * X_PITCH + x_vec * 16) = rx[i];
#pragma unroll
        for (int i = 0; i < D_PASSES; ++i)
            *reinterpret_cast<u32x4*>(sD + (d_row0 + i * D_RPP) * D_PITCH + d_vec * 16) = rd[i];
    };

    f32x16 acc[FC][FK];
#pragma unroll
    for (int i = 0; i < FC; ++i)
#pragma unroll
        for (int j = 0; j < FK; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    auto compute = [&](int stage) {
        const unsigned char* sX = smem + stage * STAGE;
        const unsigned char* sD = sX + X_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fx[FC], fd[FK];
#pragma unroll
            for (int i = 0; i < FC; ++i) fx[i] = tr_frag(sX, X_PITCH, wc * WC + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < FK; ++j) fd[j] = tr_frag(sD, D_PITCH, wk * WK + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < FC; ++i)
#pragma unroll
                for (int j = 0; j < FK; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[i], fd[j], acc[i][j], 0, 0, 0);
        }
    };

    if (kt_begin < kt_end) {
        load_global(kt_begin);
        store_lds(0);
        __syncthreads();
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            const int stage = (kt - kt_begin) & 1;
            const bool more = (kt + 1 < kt_end);
            if (more) load_global(kt + 1);
            compute(stage);
            if (more) store_lds(stage ^ 1);
            __syncthreads();
        }
    }

    const bool vec4 = (a.Kred & 3) == 0;
    float* outp = a.out + (size_t)split * g.K * a.Kred;
    if (vec4) {
        // A lane of the MFMA accumulator holds 16-byte groups of 32 different output rows, so a direct store touches
        // 32 rows per instruction.  Each wave instead turns its 32 x 64 blocks around in a private LDS region (the
        // operand tiles are dead: the main loop ended with a barrier) and moves 256-byte row segments per 16 lanes.
        // With a parameter block the old master weights are fetched before the block goes through LDS.
        static_assert(FC % 2 == 0, "the epilogue stages 64 columns at a time");
        constexpr int EP_PITCH = 64 * 4 + 16;  // rows 16 bytes apart modulo the bank width: both phases conflict-free
        static_assert((NT / 64) * 32 * EP_PITCH <= 2 * STAGE, "epilogue staging does not fit the operand tiles");
        unsigned char* const ep = smem + wave * (32 * EP_PITCH);
        const int r_rd = lane >> 4, c_rd = (lane & 15) * 4;
        const bool fused = a.sgd.w32 != nullptr;
#pragma unroll
        for (int j = 0; j < FK; ++j) {
#pragma unroll
            for (int ih = 0; ih < FC / 2; ++ih) {
                const int col = col0 + wc * WC + ih * 64 + c_rd;
                const int row0 = ko0 + wk * WK + j * 32 + r_rd;
                float4 old[8];
                if (fused) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        const int ko = row0 + t * 4;
                        old[t] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (ko < g.K && col < a.Kred)
                            old[t] = *reinterpret_cast<const float4*>(a.sgd.w32 + (size_t)ko * a.Kred + col);
                    }
                }
#pragma unroll
                for (int ii = 0; ii < 2; ++ii) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int i = ih * 2 + ii;
                        *reinterpret_cast<float4*>(ep + (lane & 31) * EP_PITCH + (ii * 32 + q * 8 + (lane >> 5) * 4) * 4) =
                            make_float4(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2],
                                        acc[i][j][q * 4 + 3]);
                    }
                }
                __builtin_amdgcn_wave_barrier();  // LDS operations of one wave complete in order
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int ko = row0 + t * 4;
                    const float4 v = *reinterpret_cast<const float4*>(ep + (t * 4 + r_rd) * EP_PITCH + c_rd * 4);
                    if (ko >= g.K || col >= a.Kred) continue;
                    const size_t e = (size_t)ko * a.Kred + col;
                    if (fused) sgd_store4(a.sgd.w32 + e, a.sgd.wb + e, old[t], a.sgd.lr, v.x, v.y, v.z, v.w);
                    else *reinterpret_cast<float4*>(outp + e) = v;
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < FK; ++j) {
        const int ko = ko0 + wk * WK + j * 32 + (lane & 31);
        if (ko >= g.K) continue;
#pragma unroll
        for (int i = 0; i < FC; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = col0 + wc * WC + i * 32 + q * 8 + (lane >> 5) * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < a.Kred) outp[(size_t)ko * a.Kred + col + e] = acc[i][j][q * 4 + e];
            }
        }
    }
}

struct Cfg {
    int TC, TK, NT;
};
constexpr Cfg kCfgs[] = {
    {256, 256, 512},  // 0: large
    {128, 128, 256},  // 1: medium / general
    {256, 64, 256},   // 2: few output channels
};

size_t smem_bytes(const Cfg& c) { return 2 * ((size_t)BK * (c.TC * 2 + 64) + (size_t)BK * (c.TK * 2 + 64)); }

template <int TC, int TK, int WCv, int WKv, int MODE>
int launch_one(const WArgs& wa, size_t smem, hipStream_t st) {
    auto kfn = wgrad_kernel<TC, TK, WCv, WKv, MODE>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    int total = wa.tiles_c * wa.tiles_k * wa.nsplit;
    hipLaunchKernelGGL(kfn, dim3(total), dim3(64 * WCv * WKv), smem, st, wa);
    return check_launch("wgrad");
}

int classify_mode(const WgradGeom& g) { return ((g.C % 8) == 0 && (g.K % 8) == 0) ? 0 : 1; }

}  // namespace

WgradPlan plan_wgrad(const WgradGeom& g) {
    WgradPlan p;
    int mode = classify_mode(g);
    int Kred = g.R * g.S * g.C;
    long Mred = (long)g.N * g.P * g.Q;
    int cfg;
    if (mode != 0) cfg = 1;
    else if (g.K <= 64) cfg = 2;
    else if (g.K >= 192 && Kred >= 256) {
        // A short reduction over a large output (the FC layers at training minibatches) is bound by the epilogue's
        // stores: smaller tiles put several work-groups on a CU, whose store phases then overlap.
        const long small_tiles = (long)((Kred + 127) / 128) * ((g.K + 127) / 128);
        cfg = (Mred <= 256 && small_tiles >= kNumCU) ? 1 : 0;
    } else cfg = 1;
    if (g_force_wgrad_cfg >= 0 && g_force_wgrad_cfg < 3 && (mode == 0 || g_force_wgrad_cfg == 1)) cfg = g_force_wgrad_cfg;
    if ((g_force_wgrad_cfg < 0 || g_force_wgrad_cfg == 4) && wgrad_c3_supported(g)) {
        p.cfg = 4;
        p.nsplit = wgrad_c3_nsplit(g);
        p.ws_bytes = (size_t)p.nsplit * g.K * Kred * sizeof(float);  // always reduced from per-work-group partials
        return p;
    }
    // (5 / 6: the patch kernel with two / one dy blocks per wavefront, for the tests)
    if ((g_force_wgrad_cfg < 0 || g_force_wgrad_cfg == 3 || g_force_wgrad_cfg == 5 || g_force_wgrad_cfg == 6) && mode == 0 &&
        wgrad_patch_supported(g)) {
        p.cfg = 3;
        p.nsplit = g_force_nsplit >= 1 ? g_force_nsplit : wgrad_patch_nsplit(g);
        long tiles_total = (long)g.N * g.P * g.Q / 64;  // every tile holds at least 64 pixels
        if (p.nsplit > tiles_total) p.nsplit = (int)tiles_total;
        p.ws_bytes = p.nsplit > 1 ? (size_t)p.nsplit * g.K * Kred * sizeof(float) : 0;
        return p;
    }
    const Cfg& c = kCfgs[cfg];
    long tiles = (long)((Kred + c.TC - 1) / c.TC) * ((g.K + c.TK - 1) / c.TK);
    int ktiles = (int)((Mred + BK - 1) / BK);
    long want = (2L * kNumCU + tiles - 1) / tiles;
    long maxs = ktiles / 4;
    if (maxs < 1) maxs = 1;
    int nsplit = (int)(want < maxs ? want : maxs);
    if (nsplit > 512) nsplit = 512;
    if (tiles >= kNumCU) nsplit = 1;
    if (g_force_nsplit >= 1) nsplit = g_force_nsplit < ktiles ? g_force_nsplit : ktiles;
    int kps = (ktiles + nsplit - 1) / nsplit;
    nsplit = (ktiles + kps - 1) / kps;
    p.cfg = cfg;
    p.nsplit = nsplit;
    p.ws_bytes = nsplit > 1 ? (size_t)nsplit * g.K * Kred * sizeof(float) : 0;
    return p;
}

int launch_wgrad(const WgradGeom& g, const WgradPlan& plan, const bf16_t* x, const bf16_t* dy,
                 float* dw, void* ws, hipStream_t st, hipEvent_t ev_mid, const uint8_t* unpool_am,
                 const SgdFuse* sgd) {
    if (unpool_am && !wgrad_fuses_unpool(g, plan))
        return set_error(WAP_EINVAL, "internal: fused max-pool backward not available for this weight gradient");
    if (sgd && !wgrad_fuses_sgd(g, plan))
        return set_error(WAP_EINVAL, "internal: fused SGD update not available for this weight gradient");
    WArgs wa;
    wa.sgd = SgdFuse{nullptr, nullptr, 0.f};
    if (sgd && plan.nsplit == 1) wa.sgd = *sgd;  // split reductions apply the update in the reduction kernel
    wa.x = x;
    wa.dy = dy;
    wa.g = g;
    wa.Kred = g.R * g.S * g.C;
    wa.Mred = g.N * g.P * g.Q;
    const Cfg& c = kCfgs[plan.cfg < 3 ? plan.cfg : 0];
    wa.tiles_c = (wa.Kred + c.TC - 1) / c.TC;
    wa.tiles_k = (g.K + c.TK - 1) / c.TK;
    wa.ktiles = (wa.Mred + BK - 1) / BK;
    wa.nsplit = plan.nsplit;
    wa.ktiles_per_split = (wa.ktiles + plan.nsplit - 1) / plan.nsplit;
    wa.dPQ = make_fastdiv((uint32_t)(g.P * g.Q));
    wa.dQ = make_fastdiv((uint32_t)g.Q);
    wa.out = plan.nsplit > 1 ? reinterpret_cast<float*>(ws) : dw;
    if (plan.cfg == 4) {
        int rc4 = launch_wgrad_c3(g, plan.nsplit, x, dy, reinterpret_cast<float*>(ws), st);
        if (rc4 != WAP_OK) return rc4;
        if (ev_mid) (void)hipEventRecord(ev_mid, st);
        return launch_reduce_f32(reinterpret_cast<const float*>(ws), plan.nsplit, (size_t)g.K * wa.Kred, dw, st, sgd);
    }
    if (plan.cfg == 3) {
        int rc3 = launch_wgrad_patch(g, plan.nsplit, x, dy, wa.out, st, unpool_am);
        if (rc3 != WAP_OK) return rc3;
        if (ev_mid) (void)hipEventRecord(ev_mid, st);
        if (plan.nsplit > 1)
            return launch_reduce_f32(reinterpret_cast<const float*>(ws), plan.nsplit, (size_t)g.K * wa.Kred, dw, st, sgd);
        return WAP_OK;
    }
    size_t smem = smem_bytes(c);
    int mode = classify_mode(g);
    int rc;
    if (plan.cfg == 0) {
        if (mode != 0) return set_error(WAP_EINVAL, "internal: large wgrad tile needs 16-byte loads");
        rc = launch_one<256, 256, 2, 4, 0>(wa, smem, st);
    } else if (plan.cfg == 1) {
        rc = mode == 0 ? launch_one<128, 128, 2, 2, 0>(wa, smem, st) : launch_one<128, 128, 2, 2, 1>(wa, smem, st);
    } else {
        if (mode != 0) return set_error(WAP_EINVAL, "internal: channel-thin wgrad tile needs 16-byte loads");
        rc = launch_one<256, 64, 4, 1, 0>(wa, smem, st);
    }
    if (rc != WAP_OK) return rc;
    if (ev_mid) (void)hipEventRecord(ev_mid, st);
    if (plan.nsplit > 1)
        return launch_reduce_f32(reinterpret_cast<const float*>(ws), plan.nsplit,
                                 (size_t)g.K * wa.Kred, dw, st, sgd);
    return WAP_OK;
}

}  // namespace wap

namespace wap {
bool wgrad_fuses_unpool(const WgradGeom& g, const WgradPlan& plan) {
    return plan.cfg == 3 && wgrad_patch_fuses_unpool(g);
}
// The update rides on whichever kernel holds the finished sums: the reduction kernel of a split product (the
// first-layer kernels always reduce), or the epilogue of an unsplit generic product whose accumulator rows are
// 16-byte groups of parameters.
bool wgrad_fuses_sgd(const WgradGeom& g, const WgradPlan& plan) {
    if (plan.cfg == 4 || plan.nsplit > 1) return true;
    return plan.cfg < 3 && ((g.R * g.S * g.C) & 3) == 0;
}
const char* wgrad_kernel_name(const WgradGeom& g, const WgradPlan& plan) { return wgrad_kernel_name(g, plan, false); }
const char* wgrad_kernel_name(const WgradGeom& g, const WgradPlan& plan, bool unpool) {
    if (plan.cfg == 3) return wgrad_patch_kernel_name(g, unpool);
    if (plan.cfg == 4) return wgrad_c3_kernel_name(g);
    static const char* names[3][2] = {
        {"wgrad_kernel<256,256,2,4,0>", ""},
        {"wgrad_kernel<128,128,2,2,0>", "wgrad_kernel<128,128,2,2,1>"},
        {"wgrad_kernel<256,64,4,1,0>", ""},
    };
    return names[plan.cfg][classify_mode(g)];
}
}  // namespace wap
