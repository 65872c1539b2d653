// wap_measure_mfma_ceiling: what the bf16 matrix pipe of THIS device sustains, measured, as the yardstick beside
// the published peak that the utilisation figures of Table 1 / Section 3.2.1 (the measured t_c of Eq. 1) are
// quoted against.  The chip lowers its clock under load, and by how much depends on what the operands look like
// and on what else a kernel does per MFMA, so the rate a convolution kernel can reach is well below
// clock_max x units; this routine measures that rate for three situations:
//   feed 0: operands stay in registers (nothing but MFMAs);
//   feed 1: the operand traffic of the forward / data-gradient kernels' main loop: per 7 MFMAs seven 16-byte
//           LDS fragment reads and one 16-byte global (L2-resident) fragment load, two work-groups of four
//           wavefronts per CU;
// each with data 0 (every operand 1.0) or data 1 (pseudo-random bf16 operands: random sign and mantissa, exponents
// 2^-3 .. 2^0).  The kernel also reads the shader clock counter against the constant 100 MHz counter, so the row
// carries the average clock the loop ran at.
#include "wap_internal.h"

namespace wap {

namespace {

constexpr int kBlocks = 2 * kNumCU;   // two resident work-groups per CU
constexpr int kWaves = 4;
constexpr int kFM = 7;                // MFMAs per operand-B fragment, as in the flat forward tiles
constexpr int kTable = 4096;          // 16-byte entries of the global fragment table (64 KB: stays in L2)
constexpr int kLds = 65536;

__device__ __forceinline__ unsigned operand_bits(unsigned h, int data) {
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    // two bf16 values: sign and mantissa from the hash, exponent field 0x7c .. 0x7f
    return data ? ((h & 0x807f807fu) | 0x3e003e00u | ((h >> 3) & 0x01800180u)) : 0x3f803f80u;
}

__global__ void ceiling_fill_kernel(unsigned* tab, int words, int data) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) tab[i] = operand_bits((unsigned)i * 2654435761u + 977u, data);
}

template <int FEED>
__global__ __launch_bounds__(kWaves * 64, 2) void ceiling_kernel(float* out, const u32x4* __restrict__ tab, int iters, int data,
                                                                long long* clk) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kLds / 4; i += blockDim.x)
        reinterpret_cast<unsigned*>(smem)[i] = operand_bits((unsigned)i * 2654435761u + blockIdx.x * 40503u, data);
    __syncthreads();
    // every LDS read below stays inside [0, 8368 + 6 * 4096 + 3072 + 16384 + 16) < 64 KB
    const unsigned char* base = smem + wave * 64 + (lane * 80) % 8192;
    f32x16 acc[kFM];
#pragma unroll
    for (int a = 0; a < kFM; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
    bf16x8 fa[kFM], fb;
#pragma unroll
    for (int a = 0; a < kFM; ++a) fa[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(base + a * 4096));
    fb = __builtin_bit_cast(bf16x8, tab[(lane + wave * 128) & (kTable - 1)]);
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        bf16x8 nb = fb;
        if (FEED) nb = __builtin_bit_cast(bf16x8, tab[(lane + wave * 128 + it * 256) & (kTable - 1)]);
#pragma unroll
        for (int a = 0; a < kFM; ++a) {
            acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb, acc[a], 0, 0, 0);
            if (FEED)
                fa[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(base + a * 4096 + ((it + 1) & 3) * 1024 + (a & 1) * 16384));
        }
        fb = nb;
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clk[0] = c1 - c0;
        clk[1] = w1 - w0;
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < kFM; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[a][e];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;  // keeps the accumulators alive
}

}  // namespace

}  // namespace wap

using namespace wap;

extern "C" {

size_t wap_mfma_ceiling_scratch_bytes(void) { return (size_t)1 << 20; }

int wap_measure_mfma_ceiling(int32_t data, int32_t feed, int32_t iters, void* scratch, size_t scratch_bytes, void* stream,
                             wap_mfma_ceiling_row* out) {
    if (!out || !scratch || (data != 0 && data != 1) || (feed != 0 && feed != 1) || iters < 1 || iters > (1 << 20))
        return set_error(WAP_EINVAL, "mfma ceiling: bad argument");
    if (scratch_bytes < wap_mfma_ceiling_scratch_bytes() || (reinterpret_cast<uintptr_t>(scratch) & 255u))
        return set_error(WAP_EWORKSPACE, "mfma ceiling: scratch must hold %zu bytes, 256-byte aligned", wap_mfma_ceiling_scratch_bytes());
    hipStream_t st = (hipStream_t)stream;
    // scratch: [0, 64 KB) fragment table, [64 KB, 64 KB + 256) clock counters, [128 KB, 128 KB + 512 KB) sink
    unsigned char* sp = reinterpret_cast<unsigned char*>(scratch);
    u32x4* tab = reinterpret_cast<u32x4*>(sp);
    long long* clk = reinterpret_cast<long long*>(sp + 65536);
    float* sink = reinterpret_cast<float*>(sp + 131072);
    static_assert((size_t)kBlocks * kWaves * 64 * sizeof(float) <= ((size_t)1 << 20) - 131072, "sink does not fit the scratch");
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        for (const void* f : {(const void*)ceiling_kernel<0>, (const void*)ceiling_kernel<1>}) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
            if (e != hipSuccess) return set_error(WAP_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
        }
        attr_done = true;
    }
    hipLaunchKernelGGL(ceiling_fill_kernel, dim3(kTable * 4 / 256), dim3(256), 0, st, reinterpret_cast<unsigned*>(tab), kTable * 4, (int)data);
    int rc = check_launch("ceiling_fill");
    if (rc != WAP_OK) return rc;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return set_error(WAP_EHIP, "hipEventCreate failed");
    auto launch = [&](int n) {
        if (feed) hipLaunchKernelGGL(ceiling_kernel<1>, dim3(kBlocks), dim3(kWaves * 64), kLds, st, sink, tab, n, (int)data, clk);
        else hipLaunchKernelGGL(ceiling_kernel<0>, dim3(kBlocks), dim3(kWaves * 64), kLds, st, sink, tab, n, (int)data, clk);
    };
    launch(iters / 8 + 1);  // warm-up: clocks settle
    hipError_t e = hipEventRecord(e0, st);
    launch(iters);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    rc = check_launch("ceiling");
    long long h[2] = {0, 0};
    if (e == hipSuccess) e = hipMemcpyAsync(h, clk, sizeof(h), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != WAP_OK) return rc;
    if (e != hipSuccess) return set_error(WAP_EHIP, "mfma ceiling: %s", hipGetErrorString(e));
    const double flops = (double)kBlocks * kWaves * (double)iters * kFM * 32768.0;  // 2 * 32 * 32 * 16 per MFMA
    out->data = data;
    out->feed = feed;
    out->us = ms * 1e3;
    out->tflops = ms > 0.f ? flops / (ms * 1e-3) / 1e12 : 0.0;
    out->clock_ghz = h[1] > 0 ? (double)h[0] / (double)h[1] * 0.1 : 0.0;  // shader-clock ticks per tick of the 100 MHz counter
    return WAP_OK;
}

}  // extern "C"
