// Large-shape forward-type implicit GEMM with the weight operand held in registers (gfx950).
//
// Same product as igemm.hip (rows = output pixels gathered from NHWC, columns = output channels,
// reduction = filter taps x 64-channel slices) for the shapes that dominate the training step
// (conv forward and, with flipped / transposed weights, the conv data gradient: the forward and
// backward halves of t_c in Eq. 1).  What limits a 256x256x64 MFMA tile on CDNA4 is the LDS, not the
// matrix cores: ds_write_b128 sustains only about 64 B/clk per CU and ds_read_b128 about 256 B/clk
// (measured), so staging both operands through LDS keeps the LDS busier than the MFMA pipe.  Here
//   * the block is 4 wavefronts (one per SIMD), each owning ALL 256 pixels x 64 output channels
//     (8 x 2 accumulators of v_mfma_f32_32x32x16_bf16 = 256 accumulator registers);
//   * only the gathered activation tile goes through LDS (shared by the 4 wavefronts, three stages
//     so the barrier is off the critical path and a tile is fetched two tiles ahead);
//   * each wavefront loads the weight fragments of its own 64 channels straight from global memory
//     into MFMA operand layout (the weights are reduction-contiguous, 16 bytes per lane) -- no LDS
//     traffic and no duplication between wavefronts, one tile ahead.
// LDS traffic per tile drops from 64 KB written + 192 KB read to 32 KB written + 128 KB read.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int BK = 64, BM = 256, BN = 256, NT = 256;
constexpr int A_PITCH = (BK + 8) * 2;
constexpr int A_STAGE = BM * A_PITCH;  // 36864
constexpr int NSTAGE = 3;
constexpr int A_PASSES = 8;            // 256 rows x 8 vectors / 256 threads
constexpr int FM = 8, FN = 2;

struct WArgsR {
    const bf16_t* A;
    const bf16_t* Bw;  // packed weights (pack_weights_kernel)
    const float* bias;
    void* out;
    GemmGeom g;
    int tiles_m, tiles_n, nsplit, ktiles, ktiles_per_split;
    int relu, partial;
    unsigned a_bytes, w_bytes;
};

__device__ __forceinline__ int xcd_remap(int bid, int total) {
    int per = total / kNumXCD, rem = total % kNumXCD;
    int xcd = bid % kNumXCD, idx = bid / kNumXCD;
    return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}
__device__ __forceinline__ u32x4 ld16(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ unsigned short f2bf(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(unsigned short, b);
}

__global__ __launch_bounds__(NT) void conv_wreg_kernel(const WArgsR a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const GemmGeom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

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
    const int nkt = kt_end - kt_begin;
    const int RS = g.R * g.S;

    // Both operands are read through raw buffer descriptors: a 32-bit byte offset per lane, and lanes
    // that must contribute zeros (padding taps, tile tails) get an offset beyond the buffer, which the
    // hardware answers with zeros -- no select after the load, no 64-bit address registers.
    const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(a.A), 0, (int)a.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrcW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(a.Bw), 0, (int)a.w_bytes, 0x00020000);
    constexpr unsigned OOB = 0xFFFFFF00u;

    // ---- gathered operand: fixed rows per thread; (h,w) base packed in one register ----
    const int a_vec = tid & 7, a_row0 = tid >> 3;
    int hw[A_PASSES];
    unsigned abase[A_PASSES];  // byte offset of (image n, channel vector a_vec)
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
        int m = m0 + a_row0 + i * 32;
        if (m < g.M) {
            int ow = m % g.OW;
            int t = m / g.OW;
            int oh = t % g.OH;
            int n = t / g.OH;
            int hb = oh * g.mul_h - g.pad_h, wb = ow * g.mul_w - g.pad_w;
            hw[i] = (hb << 16) | (wb & 0xffff);
            abase[i] = (unsigned)(n * g.IH * g.IW * g.IC + a_vec * 8) * 2u;
        } else {
            hw[i] = (int)0x80008000u;  // h = w = -32768: never in range
            abase[i] = 0;
        }
    }
    // ---- weight operand: this wavefront's 64 channels = two 32-channel blocks of the packed weights.
    // Packed layout (pack_weights_kernel): [channel block of 32][16-element reduction step][lane][8],
    // i.e. every fragment load of a wavefront is one contiguous, fully used 1 KB.
    const unsigned ksteps = (unsigned)g.Kred / 16u;
    unsigned wrow[FN];
#pragma unroll
    for (int i = 0; i < FN; ++i) {
        unsigned blk = (unsigned)(n0 + wave * 64 + i * 32) / 32u;
        wrow[i] = (blk * ksteps * 64u + (unsigned)lane) * 16u;
    }

    // reduction tile index -> element offset of its first reduction element (channel-slice-major walk)
    auto kk_of = [&](int kt) { return (kt % RS) * g.IC + (kt / RS) * BK; };

    u32x4 ra[A_PASSES];
    auto load_a = [&](int kt) {
        const int kk0 = kk_of(kt);
        const int tap = kk0 / g.IC;
        const int c0 = kk0 - tap * g.IC;
        const int r = tap / g.S, s = tap - r * g.S;
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i) {
            int th = (hw[i] >> 16) + r, tw = (int)(short)(hw[i] & 0xffff) + s;
            bool ok = (unsigned)th < (unsigned)g.IH && (unsigned)tw < (unsigned)g.IW;
            unsigned off = abase[i] + (unsigned)((th * g.IW + tw) * g.IC + c0) * 2u;
            ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, ok ? off : OOB, 0, 0);
        }
    };
    auto store_a = [&](int stage) {
        unsigned char* sA = smem + stage * A_STAGE;
#pragma unroll
        for (int i = 0; i < A_PASSES; ++i)
            *reinterpret_cast<u32x4*>(sA + (a_row0 + i * 32) * A_PITCH + a_vec * 16) = ra[i];
    };
    // one 16-element reduction step of this wavefront's weight fragments
    auto load_w_step = [&](int kt, int ks, bf16x8 (&w)[FN]) {
        const unsigned koff = ((unsigned)kk_of(kt) / 16u + (unsigned)ks) * 1024u;
#pragma unroll
        for (int i = 0; i < FN; ++i)
            w[i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrcW, wrow[i] + koff, 0, 0));
    };
    const int frag_base = (lane & 31) * A_PITCH + (lane >> 5) * 16;
    auto read_frags = [&](int stage, int ks, bf16x8 (&f)[FM]) {
        const unsigned char* sA = smem + stage * A_STAGE + frag_base + ks * 32;
#pragma unroll
        for (int j = 0; j < FM; ++j) f[j] = *reinterpret_cast<const bf16x8*>(sA + j * 32 * A_PITCH);
    };

    f32x16 acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    if (nkt > 0) {
        bf16x8 wA[4][FN], wB[4][FN];
        bf16x8 fa[2][FM];
        // prologue: tiles 0 and 1 of the gathered operand into LDS, weights of tile 0 into registers
        load_a(kt_begin);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) load_w_step(kt_begin, ks, wA[ks]);
        store_a(0);
        if (nkt > 1) {
            load_a(kt_begin + 1);
            store_a(1);
        }
        __syncthreads();
        read_frags(0, 0, fa[0]);
        int stage = 0;
        // One reduction tile per iteration.  All global loads of the iteration (activation tile it+2 for
        // the LDS, weight fragments of tile it+1 into the spare register set) are issued at its top and
        // consumed after its 64 MFMAs, so the only vmcnt wait sits at the end of the tile.
        // The body is branch-free on purpose (a conditional load inside the loop makes the compiler's
        // wait-count insertion serialise every MFMA group behind the loads): past the end of the
        // reduction range the tile indices are clamped, which only repeats loads of valid addresses into
        // registers / LDS stages that nobody reads any more.
        for (int it = 0; it < nkt; ++it) {
            const int kt1 = kt_begin + (it + 1 < nkt ? it + 1 : nkt - 1);
            const int kt2 = kt_begin + (it + 2 < nkt ? it + 2 : nkt - 1);
            const int stage1 = stage == NSTAGE - 1 ? 0 : stage + 1;
            const int stage2 = stage1 == NSTAGE - 1 ? 0 : stage1 + 1;
            __builtin_amdgcn_sched_barrier(0);
            load_a(kt2);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) load_w_step(kt1, ks, wB[ks]);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < 3) read_frags(stage, ks + 1, fa[(ks + 1) & 1]);
                else read_frags(stage1, 0, fa[0]);
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int i = 0; i < FN; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wA[ks][i], fa[ks & 1][j], acc[i][j], 0, 0, 0);
            }
            store_a(stage2);
            // Issue order within the tile (one wavefront per SIMD: nothing else hides a bubble):
            //   step 0: 8 x { global load (activations), LDS fragment read, 2 MFMA }
            //   step 1: 8 x { global load (weights),     LDS fragment read, 2 MFMA }
            //   step 2: 8 x {                            LDS fragment read, 2 MFMA }
            //   step 3: 8 x { LDS write (tile it+2),     LDS fragment read, 2 MFMA }
            // every fragment read is issued 16 MFMAs (one step) before its first use.
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // MFMA
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // DS write
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < FN; ++i) wA[ks][i] = wB[ks][i];
            __syncthreads();
            stage = stage1;
        }
    }

    // ---- epilogue: lane holds 4 consecutive channels of one pixel per register quad ----
    const bool vec4 = (g.Ncols & 3) == 0;
#pragma unroll
    for (int j = 0; j < FM; ++j) {
        const int m = m0 + j * 32 + (lane & 31);
        if (m >= g.M) continue;
#pragma unroll
        for (int i = 0; i < FN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wave * 64 + i * 32 + q * 8 + (lane >> 5) * 4;
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

// Packs the weights into MFMA fragment order: Wp[channel block of 32][reduction step of 16][lane][8] with
// lane = (channel % 32) + 32 * (reduction half), zero-filled past the last channel.
//   flip == 0: forward weights, element (n, kk) = w[n][kk]                       (w is [Ncols][Kred])
//   flip == 1: data gradient, reduction index kk = (r', s', k): element = w[k][R-1-r'][S-1-s'][n]
__device__ __forceinline__ void pack_one(const bf16_t* __restrict__ w, u32x4* __restrict__ Wp, int Ncols, int Kred,
                                         int IC, int R, int S, int flip, size_t v) {
    const int ksteps = Kred / 16;
    {
        int lane = (int)(v & 63);
        size_t t = v >> 6;
        int kstep = (int)(t % ksteps);
        int blk = (int)(t / ksteps);
        int n = blk * 32 + (lane & 31);
        int kk = kstep * 16 + (lane >> 5) * 8;
        u32x4 out = {0u, 0u, 0u, 0u};
        if (n < Ncols) {
            if (!flip) {
                out = *reinterpret_cast<const u32x4*>(w + (size_t)n * Kred + kk);
            } else {
                int tap = kk / IC, k = kk - tap * IC;  // IC % 64 == 0: the 8 elements share one tap
                int r2 = tap / S, s2 = tap - r2 * S;
                unsigned short h[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    h[e] = w[(((size_t)(k + e) * R + (R - 1 - r2)) * S + (S - 1 - s2)) * Ncols + n];
                out[0] = (unsigned)h[0] | ((unsigned)h[1] << 16);
                out[1] = (unsigned)h[2] | ((unsigned)h[3] << 16);
                out[2] = (unsigned)h[4] | ((unsigned)h[5] << 16);
                out[3] = (unsigned)h[6] | ((unsigned)h[7] << 16);
            }
        }
        Wp[v] = out;
    }
}

__global__ void pack_weights_kernel(const bf16_t* __restrict__ w, u32x4* __restrict__ Wp, int Ncols, int Kred,
                                    int IC, int R, int S, int flip) {
    const int ksteps = Kred / 16;
    const int nblk = (Ncols + 31) / 32;
    size_t total = (size_t)nblk * ksteps * 64;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += stride)
        pack_one(w, Wp, Ncols, Kred, IC, R, S, flip, v);
}

// Every packing job of a training step in one launch: job j owns the 16-byte vectors [first[j], first[j+1]).
__global__ void pack_weights_multi_kernel(const PackJobs js, unsigned char* __restrict__ base) {
    const size_t total = js.first[js.n];
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < total; v += stride) {
        int j = 0;
        while (j + 1 < js.n && v >= js.first[j + 1]) ++j;
        const PackJob& b = js.job[j];
        pack_one(reinterpret_cast<const bf16_t*>(base + b.w_off), reinterpret_cast<u32x4*>(base + b.out_off), b.Ncols,
                 b.Kred, b.IC, b.R, b.S, b.flip, v - js.first[j]);
    }
}

}  // namespace

bool wreg_supported(const GemmGeom& g) {
    // The kernel keeps a pixel's (row, column) base as two signed 16-bit halves of one register and addresses the
    // activations with 32-bit byte offsets whose top value is the out-of-range sentinel: maps whose padded
    // coordinates or byte size exceed those ranges go to the generic tiles.
    const long h_hi = (long)(g.OH - 1) * g.mul_h - g.pad_h + g.R - 1, w_hi = (long)(g.OW - 1) * g.mul_w - g.pad_w + g.S - 1;
    const bool coords_fit = h_hi < 32768 && w_hi < 32768 && g.pad_h < 32768 && g.pad_w < 32768;
    const long imgs = (long)(g.M / ((long)g.OH * g.OW));
    const bool bytes_fit = (double)imgs * g.IH * g.IW * g.IC * 2.0 <= (double)0xFFFFFF00u;
    return (g.IC % BK) == 0 && g.div_h == 1 && g.div_w == 1 && (g.Kred % 8) == 0 && coords_fit && bytes_fit;
}

size_t wreg_smem_bytes() { return (size_t)NSTAGE * A_STAGE; }

void pack_jobs_add(PackJobs& js, const GemmGeom& g, bool flip, size_t w_off, size_t out_off) {
    PackJob& b = js.job[js.n];
    b.w_off = w_off;
    b.out_off = out_off;
    b.Ncols = g.Ncols;
    b.Kred = g.Kred;
    b.IC = g.IC;
    b.R = g.R;
    b.S = g.S;
    b.flip = flip ? 1 : 0;
    if (js.n == 0) js.first[0] = 0;
    js.first[js.n + 1] = js.first[js.n] + (size_t)((g.Ncols + 31) / 32) * (g.Kred / 16) * 64;
    ++js.n;
}

int launch_pack_weights_multi(const PackJobs& js, void* base, hipStream_t st) {
    if (js.n == 0) return WAP_OK;
    size_t blocks = (js.first[js.n] + 255) / 256;
    if (blocks > (size_t)kNumCU * 16) blocks = (size_t)kNumCU * 16;
    hipLaunchKernelGGL(pack_weights_multi_kernel, dim3((unsigned)blocks), dim3(256), 0, st, js,
                       reinterpret_cast<unsigned char*>(base));
    return check_launch("pack_weights_multi");
}

int launch_pack_weights(const GemmGeom& g, bool flip, const bf16_t* w, void* Wp, hipStream_t st) {
    size_t total = (size_t)((g.Ncols + 31) / 32) * (g.Kred / 16) * 64;
    size_t blocks = (total + 255) / 256;
    if (blocks > (size_t)kNumCU * 8) blocks = (size_t)kNumCU * 8;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, st, w,
                       reinterpret_cast<u32x4*>(Wp), g.Ncols, g.Kred, g.IC, g.R, g.S, flip ? 1 : 0);
    return check_launch("pack_weights");
}

int launch_wreg(const GemmGeom& g, int nsplit, const bf16_t* A, const bf16_t* Bw, const float* bias, bool relu,
                void* out, bool partial, hipStream_t st) {
    WArgsR ka;
    ka.A = A;
    ka.Bw = Bw;
    ka.g = g;
    ka.tiles_m = (g.M + BM - 1) / BM;
    ka.tiles_n = (g.Ncols + BN - 1) / BN;
    ka.ktiles = g.Kred / BK;
    ka.nsplit = nsplit;
    ka.ktiles_per_split = (ka.ktiles + nsplit - 1) / nsplit;
    ka.partial = partial ? 1 : 0;
    ka.bias = partial ? nullptr : bias;
    ka.relu = partial ? 0 : (relu ? 1 : 0);
    ka.out = out;
    ka.a_bytes = (unsigned)((size_t)(g.M / (g.OH * g.OW)) * g.IH * g.IW * g.IC * 2);
    ka.w_bytes = (unsigned)wreg_wt_bytes(g);
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_wreg_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)wreg_smem_bytes());
        if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        attr_done = true;
    }
    int total = ka.tiles_m * ka.tiles_n * ka.nsplit;
    hipLaunchKernelGGL(conv_wreg_kernel, dim3(total), dim3(NT), wreg_smem_bytes(), st, ka);
    return check_launch("conv_wreg");
}

}  // namespace wap
