// Stride-1 convolution (forward, and data gradient with flipped weights) as an implicit GEMM whose
// im2col tile lives in LDS ONCE per channel slice (gfx950).
//
// conv_wreg.hip fetches one 224/256-pixel x 64-channel tile per filter tap, i.e. the same input
// pixels nine times per 3x3 layer, and at that point the L2 -> CU path (about 8 TB/s aggregate,
// measured) is what bounds the kernel, not the matrix cores.  Here a work-group owns 224 consecutive
// output pixels (raster order; 224 = 7 * 32 divides every VGG feature map) and, per 64-channel slice,
// loads the zero-padded input PATCH those pixels touch (the pixels plus halo rows / columns, one
// 144-byte LDS row per padded pixel) once; the fragment of filter tap (r, s) is then the same LDS
// rows shifted by (r * padded_width + s) pixels, so all R*S taps run out of one patch:
//   * L2 -> LDS traffic for the activations drops by ~R*S / 1.5, LDS writes likewise, and there is
//     one barrier per channel slice instead of one per tap;
//   * the weights never touch LDS: every wavefront owns 32*FN output channels and loads its packed
//     fragments (see pack_weights_kernel in conv_wreg.hip) straight into MFMA operand registers,
//     one reduction tile ahead;
//   * 4 wavefronts, one per SIMD, each 224 pixels x 32*FN channels of v_mfma_f32_32x32x16_bf16
//     accumulators (AGPRs); the issue order is pinned with sched_group_barrier because a single
//     wavefront per SIMD has nothing else to hide a bubble.
// Serves the "primary" convolution nodes of Section 3.2.2 (forward and backward halves of t_c, Eq. 1).
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64, BM = 224, NT = 256, FM = 7;
constexpr int PITCH = (BK + 8) * 2;  // 144 bytes per padded pixel

struct PArgs {
    const bf16_t* A;
    const bf16_t* Wp;  // packed weights
    const float* bias;
    const bf16_t* mask;  // optional: out = mask > 0 ? out : 0
    void* out;
    GemmGeom g;
    int tiles_m, tiles_n;
    int PH, PW;        // padded (virtual) input size: OH + R - 1, OW + S - 1
    int patch_cap;     // LDS rows per patch buffer
    int relu;
    unsigned a_bytes, w_bytes;
    FastDiv dOHW, dOW, dPHW, dPW;
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

// PV: 16-byte patch vectors per thread (patch rows <= PV * 32); FN: 32-channel blocks per wavefront
template <int PV, int FN>
__global__ __launch_bounds__(NT) void conv_patch_kernel(const PArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const GemmGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int BN = 128 * FN;

    int logical = xcd_remap(blockIdx.x, a.tiles_m * a.tiles_n);
    const int tn = logical % a.tiles_n;
    const int tm = logical / a.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int RS = g.R * g.S;
    const int PW = a.PW, PHW = a.PH * a.PW;
    const int OHW = g.OH * g.OW;
    const int ncs = g.IC / BK;

    const __amdgpu_buffer_rsrc_t rsrcA =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.A), 0, (int)a.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.Wp), 0, (int)a.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0x80000000u;  // the activation tensor is below 2 GiB (checked on the host)

    // padded-flat index of output pixel m (tap (0,0)): ((n * PH + oh) * PW + ow)
    auto pflat = [&](int m) {
        int n = (int)fdiv((uint32_t)m, a.dOHW);
        int rem = m - n * OHW;
        int oh = (int)fdiv((uint32_t)rem, a.dOW);
        int ow = rem - oh * g.OW;
        return n * PHW + oh * PW + ow;
    };
    const int m_last = (m0 + BM <= g.M ? m0 + BM : g.M) - 1;
    const int p_lo = pflat(m0);
    const int patch_len = pflat(m_last) + (g.R - 1) * PW + (g.S - 1) + 1 - p_lo;  // <= patch_cap (host)

    // ---- patch vectors of this thread: byte offset of (padded pixel, 8-channel vector) or OOB ----
    unsigned pvoff[PV];
#pragma unroll
    for (int i = 0; i < PV; ++i) {
        int v = tid + i * NT;
        int q = v >> 3;
        unsigned off = OOB;
        if (q < patch_len) {
            int p = p_lo + q;
            int n = (int)fdiv((uint32_t)p, a.dPHW);
            int rem = p - n * PHW;
            int vh = (int)fdiv((uint32_t)rem, a.dPW);
            int vw = rem - vh * PW;
            int ih = vh - g.pad_h, iw = vw - g.pad_w;
            if (n * OHW < g.M && (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW)
                off = (unsigned)(((n * g.IH + ih) * g.IW + iw) * g.IC + (v & 7) * 8) * 2u;
        }
        pvoff[i] = off;
    }
    u32x4 rp[PV];
    auto load_patch = [&](int cs) {
        const unsigned coff = (unsigned)(cs * BK) * 2u;
#pragma unroll
        for (int i = 0; i < PV; ++i) rp[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, pvoff[i] + coff, 0, 0);
    };
    auto store_patch = [&](int buf) {
        unsigned char* sP = smem + buf * a.patch_cap * PITCH;
#pragma unroll
        for (int i = 0; i < PV; ++i) {
            int v = tid + i * NT;
            if ((v >> 3) < a.patch_cap) *reinterpret_cast<u32x4*>(sP + (v >> 3) * PITCH + (v & 7) * 16) = rp[i];
        }
    };

    // ---- fragment rows of this lane: LDS byte offset of its pixel in fragment j (tap (0,0)) ----
    int frow[FM];
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        int m = m0 + j * 32 + (lane & 31);
        if (m > m_last) m = m_last;  // tile tail: computed on a valid pixel, never stored
        frow[j] = (pflat(m) - p_lo) * PITCH + (lane >> 5) * 16;
    }

    // ---- weights: packed [channel block of 32][reduction step of 16][lane][8] ----
    const unsigned ksteps = (unsigned)g.Kred / 16u;
    unsigned wrow[FN];
#pragma unroll
    for (int i = 0; i < FN; ++i) {
        unsigned blk = (unsigned)(n0 + wave * 32 * FN + i * 32) / 32u;
        wrow[i] = (blk * ksteps * 64u + (unsigned)lane) * 16u;
    }
    // reduction tile (cs, tap) -> first reduction element = tap * IC + cs * 64
    auto load_w = [&](int cs, int tap, bf16x8 (&w)[4][FN]) {
        const unsigned koff = ((unsigned)(tap * g.IC + cs * BK) / 16u) * 1024u;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < FN; ++i)
                w[ks][i] = __builtin_bit_cast(
                    bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrcW, wrow[i] + koff + (unsigned)ks * 1024u, 0, 0));
    };
    auto read_frags = [&](const unsigned char* sP, int tapoff, int ks, bf16x8 (&f)[FM]) {
#pragma unroll
        for (int j = 0; j < FM; ++j) f[j] = *reinterpret_cast<const bf16x8*>(sP + frow[j] + tapoff + ks * 32);
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    bf16x8 wA[4][FN], wB[4][FN];
    bf16x8 fa[2][FM];
    load_patch(0);
    load_w(0, 0, wA);
    store_patch(0);
    __syncthreads();

    for (int cs = 0; cs < ncs; ++cs) {
        const unsigned char* sP = smem + (cs & 1) * a.patch_cap * PITCH;
        const int cs1 = cs + 1 < ncs ? cs + 1 : cs;
        load_patch(cs1);  // next slice's patch: in flight during this slice's taps
        read_frags(sP, 0, 0, fa[0]);
        int r = 0, s = 0;
        for (int tap = 0; tap < RS; ++tap) {
            // next reduction tile: next tap of this slice, or tap 0 of the next slice (clamped at the end)
            int s1 = s + 1, r1 = r;
            if (s1 == g.S) { s1 = 0; r1 = r + 1; }
            const bool last = tap + 1 == RS;
            const int tapoff = (r * PW + s) * PITCH;
            const int tapoff1 = last ? tapoff : (r1 * PW + s1) * PITCH;
            __builtin_amdgcn_sched_barrier(0);
            load_w(last ? cs1 : cs, last ? 0 : tap + 1, wB);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < 3) read_frags(sP, tapoff, ks + 1, fa[(ks + 1) & 1]);
                else read_frags(sP, tapoff1, 0, fa[0]);  // after the last tap this read is discarded
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int i = 0; i < FN; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wA[ks][i], fa[ks & 1][j], acc[i][j], 0, 0, 0);
            }
            // issue order: the 4*FN weight loads ride on the first MFMAs, then one fragment read per FN MFMAs
#pragma unroll
            for (int q = 0; q < 4 * FN; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
                __builtin_amdgcn_sched_group_barrier(0x008, FN, 0);  // MFMA
            }
#pragma unroll
            for (int q = 0; q < 4 * FM - 4 * FN; ++q) {
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
        store_patch((cs + 1) & 1);  // last read of that buffer was before the previous slice's barrier
        __syncthreads();
    }

    // ---- epilogue.  A lane holds 4 consecutive channels of one pixel per register quad; when the channel
    // count allows 16-byte rows the tile is transposed through LDS (free after the last slice) in two
    // pixel halves so that every global store is a full, contiguous 16 bytes per lane. ----
    if ((g.Ncols & 7) == 0) {
        constexpr int OPITCH = BN * 2 + 16;  // bytes per pixel row in the staging buffer
        constexpr int VPR = BN / 8;          // 16-byte vectors per pixel row
        constexpr int RPP = NT / VPR;        // pixel rows stored per pass
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int j0 = half * 4, j1 = half ? FM : 4;
            __syncthreads();  // previous readers of the staging area (or of the patch) are done
#pragma unroll
            for (int j = j0; j < j1; ++j)
#pragma unroll
                for (int i = 0; i < FN; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int nl = wave * 32 * FN + i * 32 + q * 8 + (lane >> 5) * 4;  // channel within the tile
                        float v[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
                        if (a.bias) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (n0 + nl + e < g.Ncols) v[e] += a.bias[n0 + nl + e];
                        }
                        if (a.relu) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                        }
                        uint2 pk = make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16),
                                              (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
                        *reinterpret_cast<uint2*>(smem + ((j - j0) * 32 + (lane & 31)) * OPITCH + nl * 2) = pk;
                    }
            __syncthreads();
            const int rows = (j1 - j0) * 32;
            for (int row = tid / VPR; row < rows; row += RPP) {
                const int m = m0 + j0 * 32 + row;
                const int n = n0 + (tid % VPR) * 8;
                if (m <= m_last && n < g.Ncols) {
                    u32x4 vv = *reinterpret_cast<const u32x4*>(smem + row * OPITCH + (tid % VPR) * 16);
                    if (a.mask) vv = relu_mask8(vv, *reinterpret_cast<const u32x4*>(a.mask + (size_t)m * g.Ncols + n));
                    *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(a.out) + (size_t)m * g.Ncols + n) = vv;
                }
            }
        }
        return;
    }
    const bool vec4 = (g.Ncols & 3) == 0;
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int m = m0 + j * 32 + (lane & 31);
        if (m > m_last) continue;
#pragma unroll
        for (int i = 0; i < FN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wave * 32 * FN + i * 32 + q * 8 + (lane >> 5) * 4;
                if (n >= g.Ncols) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e];
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

// largest patch (in padded pixels) any 224-pixel tile of this geometry needs
int max_patch_len(const GemmGeom& g) {
    const int PH = g.OH + g.R - 1, PW = g.OW + g.S - 1;
    const long OHW = (long)g.OH * g.OW;
    auto pflat = [&](long m) {
        long n = m / OHW, rem = m - n * OHW;
        long oh = rem / g.OW, ow = rem - oh * g.OW;
        return n * PH * PW + oh * PW + ow;
    };
    long worst = 0;
    for (long m0 = 0; m0 < g.M; m0 += BM) {
        long ml = (m0 + BM <= g.M ? m0 + BM : g.M) - 1;
        long len = pflat(ml) + (long)(g.R - 1) * PW + (g.S - 1) + 1 - pflat(m0);
        if (len > worst) worst = len;
    }
    return (int)worst;
}

template <int PV, int FN>
int launch_patch_t(const PArgs& pa, hipStream_t st) {
    auto kfn = conv_patch_kernel<PV, FN>;
    size_t smem = (size_t)2 * pa.patch_cap * PITCH;
    static size_t attr_smem = 0;
    if (attr_smem < smem) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kfn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_smem = smem;
    }
    hipLaunchKernelGGL(kfn, dim3(pa.tiles_m * pa.tiles_n), dim3(NT), smem, st, pa);
    return check_launch("conv_patch");
}

}  // namespace

// 0 = not applicable, otherwise the number of LDS rows per patch buffer
int patch_supported(const GemmGeom& g) {
    if ((g.IC % BK) != 0 || g.div_h != 1 || g.div_w != 1 || g.mul_h != 1 || g.mul_w != 1) return 0;
    if (g.R * g.S < 2) return 0;                       // nothing to reuse for 1x1
    if (g.Ncols < 128 || g.M < BM * 32) return 0;      // thin or tiny shapes stay on the other kernels
    long a_elems = (long)(g.M / ((long)g.OH * g.OW)) * g.IH * g.IW * g.IC;
    if (a_elems * 2 >= (1L << 31)) return 0;
    int len = max_patch_len(g);
    if (len > 560) return 0;
    return len <= 384 ? 384 : 560;
}

namespace {
// 256-channel tiles unless they would leave a third of the CUs without a work-group
bool patch_wide(const GemmGeom& g) {
    const long tiles_m = (g.M + BM - 1) / BM;
    return g.Ncols > 128 && tiles_m * ((g.Ncols + 255) / 256) >= kNumCU * 2 / 3;
}
}  // namespace

const char* patch_kernel_name(const GemmGeom& g) {
    const int cap = patch_supported(g);
    const bool wide = patch_wide(g);
    if (cap == 384) return wide ? "conv_patch_kernel<12,2>" : "conv_patch_kernel<12,1>";
    return wide ? "conv_patch_kernel<18,2>" : "conv_patch_kernel<18,1>";
}

int launch_patch(const GemmGeom& g, const bf16_t* A, const void* Wp, const float* bias, bool relu, bf16_t* out,
                 hipStream_t st, const bf16_t* mask) {
    PArgs pa;
    if (mask && (g.Ncols & 7)) return set_error(WAP_EINVAL, "internal: fused mask needs 16-byte output rows");
    pa.mask = mask;
    pa.A = A;
    pa.Wp = reinterpret_cast<const bf16_t*>(Wp);
    pa.bias = bias;
    pa.out = out;
    pa.g = g;
    pa.PH = g.OH + g.R - 1;
    pa.PW = g.OW + g.S - 1;
    pa.patch_cap = patch_supported(g);
    if (!pa.patch_cap) return set_error(WAP_EINVAL, "internal: patch kernel not applicable");
    pa.relu = relu ? 1 : 0;
    pa.dOHW = make_fastdiv((uint32_t)(g.OH * g.OW));
    pa.dOW = make_fastdiv((uint32_t)g.OW);
    pa.dPHW = make_fastdiv((uint32_t)(pa.PH * pa.PW));
    pa.dPW = make_fastdiv((uint32_t)pa.PW);
    pa.a_bytes = (unsigned)((size_t)(g.M / (g.OH * g.OW)) * g.IH * g.IW * g.IC * 2);
    pa.w_bytes = (unsigned)wreg_wt_bytes(g);
    pa.tiles_m = (g.M + BM - 1) / BM;
    const bool wide = patch_wide(g);
    pa.tiles_n = wide ? (g.Ncols + 255) / 256 : (g.Ncols + 127) / 128;
    if (pa.patch_cap == 384) return wide ? launch_patch_t<12, 2>(pa, st) : launch_patch_t<12, 1>(pa, st);
    return wide ? launch_patch_t<18, 2>(pa, st) : launch_patch_t<18, 1>(pa, st);
}

}  // namespace wap
