// Calibration probe: the rate at which a compute unit's SIMDs can issue the matrix instruction of the 16-bit kernels
// when nothing has to be moved (operands and accumulators stay in registers).  The benchmark reports the convolution's
// rate against this measured ceiling next to the published peak.
#include "ss_internal.h"
#include "../../include/ss_debug.h"
#include <type_traits>

namespace ss {

typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x16 __attribute__((ext_vector_type(16)));
typedef __bf16 b16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16x16 __attribute__((ext_vector_type(16)));
typedef float acc16 __attribute__((ext_vector_type(16)));

constexpr int kProbeAcc = 4;      // independent accumulators per wave: no instruction waits for the one before it

template <int DT, bool SPARSE>
__global__ __launch_bounds__(512) void issue_probe_kernel(float *sink, int iters)
{
    acc16 c[kProbeAcc];
#pragma unroll
    for (int i = 0; i < kProbeAcc; i++)
#pragma unroll
        for (int v = 0; v < 16; v++) c[i][v] = 0.f;
    // operands: built once, outside the timed loop
    const float seed = (float)(threadIdx.x & 7) * 0.125f;
    typename std::conditional<DT == SS_F16, h16x8, b16x8>::type a;
    typename std::conditional<DT == SS_F16, h16x16, b16x16>::type b;
    typedef typename std::conditional<DT == SS_F16, _Float16, __bf16>::type elem;
#pragma unroll
    for (int e = 0; e < 8; e++) a[e] = (elem)seed;
#pragma unroll
    for (int e = 0; e < 16; e++) b[e] = (elem)(seed + 1.f);
    const auto blo = __builtin_shufflevector(b, b, 0, 1, 2, 3, 4, 5, 6, 7);
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int i4 = 0; i4 < 4 * kProbeAcc; i4++) {
            const int i = i4 % kProbeAcc;
            if constexpr (DT == SS_F16) {
                if constexpr (SPARSE) c[i] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b, c[i], 0x4444, 0, 0);
                else c[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, blo, c[i], 0, 0, 0);
            } else {
                if constexpr (SPARSE) c[i] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, b, c[i], 0x4444, 0, 0);
                else c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, blo, c[i], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeAcc; i++)
#pragma unroll
        for (int v = 0; v < 16; v++) s += c[i][v];
    sink[blockIdx.x * 512 + threadIdx.x] = s;       // keeps the loop alive
}

// LDS bandwidth of a compute unit: every wave issues eight independent 16-byte-per-lane LDS instructions, waits for
// them, and repeats.  MODE 0: reads in the convolution kernels' fragment pattern (lane % 32 = pixel row of `row_bytes`,
// lane / 32 = second half of the step); MODE 1: lane-linear writes (a wave's 1 KiB contiguous); MODE 2 / 3: the same
// bytes as 8-byte / 4-byte writes; MODE 4: even waves read, odd waves write.
typedef uint32_t pu32x4 __attribute__((ext_vector_type(4)));
template <int MODE>
__global__ __launch_bounds__(1024) void lds_probe_kernel(uint32_t *sink, int iters, int row_bytes)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    for (int i = t; i < 65536 / 4; i += blockDim.x) reinterpret_cast<uint32_t *>(lds)[i] = (uint32_t)i;
    __syncthreads();
    // byte offsets stay below 64 KiB: rows 0..63 of at most 592 bytes plus 8 x 64 bytes; 16 KiB + 3 x 16 KiB for the writes
    // (the LDS instructions are written out: the probe must issue exactly these, eight in flight, then one wait)
    const uint32_t base = (uint32_t)(uintptr_t)lds;
    const uint32_t rd = base + (lane & 31) * row_bytes + (lane >> 5) * 32 + (w & 1) * 32 * row_bytes;
    const uint32_t wr = base + lane * 16 + (w & 15) * 1024;
    uint32_t acc = 0;
    for (int it = 0; it < iters; it++) {
        if constexpr (MODE == 0) {
            pu32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[j]) : "v"(rd), "n"(j * 64));
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int j = 0; j < 8; j++) acc ^= v[j][0];
        } else if constexpr (MODE == 4) {            // even waves read, odd waves write (16 bytes per lane each): do the two share the LDS's time?
            if ((w & 1) == 0) {
                pu32x4 v[8];
#pragma unroll
                for (int j = 0; j < 8; j++) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[j]) : "v"(rd), "n"(j * 64));
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int j = 0; j < 8; j++) acc ^= v[j][0];
            } else {
                const pu32x4 d = {acc, (uint32_t)it, 1u, 2u};
                const uint32_t wr2 = wr + 40960;     // (above the rows the readers use)
#pragma unroll
                for (int j = 0; j < 8; j++) asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(wr2), "v"(d), "n"((j & 1) * 8192) : "memory");
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
        } else if constexpr (MODE == 1) {
            const pu32x4 d = {acc, (uint32_t)it, 1u, 2u};
#pragma unroll
            for (int j = 0; j < 8; j++) asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(wr), "v"(d), "n"((j % 3) * 16384) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        } else if constexpr (MODE == 2) {            // the same bytes as 8-byte writes (a wave's 512 bytes contiguous per instruction)
            typedef uint32_t pu32x2 __attribute__((ext_vector_type(2)));
            const pu32x2 d = {acc, (uint32_t)it};
            const uint32_t wr8 = base + lane * 8 + (w & 15) * 1024;
#pragma unroll
            for (int j = 0; j < 16; j++) asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(wr8), "v"(d), "n"((j % 3) * 16384 + (j & 1) * 512) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        } else {                                     // ... and as 4-byte writes (256 bytes contiguous per instruction)
            const uint32_t d = acc + (uint32_t)it;
            const uint32_t wr4 = base + lane * 4 + (w & 15) * 1024;
#pragma unroll
            for (int j = 0; j < 32; j++) asm volatile("ds_write_b32 %0, %1 offset:%2" ::"v"(wr4), "v"(d), "n"((j % 3) * 16384 + (j & 3) * 256) : "memory");
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }
    sink[blockIdx.x * 1024 + t] = acc;
}

}  // namespace ss

using namespace ss;

extern "C" int ss_debug_issue_peak(int32_t dtype, int32_t sparse, void *scratch, size_t scratch_bytes, float *tflops, void *stream)
{
    if (!tflops || !scratch) return SS_ERR_INVALID_ARG;
    if (dtype != SS_F16 && dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    int dev = 0, ncu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0)
        return SS_ERR_HIP;
    const int blocks = ncu;                          // one workgroup of eight waves per compute unit: two waves per SIMD
    if (scratch_bytes < (size_t)blocks * 512 * 4) return SS_ERR_WORKSPACE;
    const int iters = 20000;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return SS_ERR_HIP;
    float *sink = static_cast<float *>(scratch);
    auto launch = [&](int n) {
        if (dtype == SS_F16) {
            if (sparse) issue_probe_kernel<SS_F16, true><<<blocks, 512, 0, s>>>(sink, n);
            else issue_probe_kernel<SS_F16, false><<<blocks, 512, 0, s>>>(sink, n);
        } else {
            if (sparse) issue_probe_kernel<SS_BF16, true><<<blocks, 512, 0, s>>>(sink, n);
            else issue_probe_kernel<SS_BF16, false><<<blocks, 512, 0, s>>>(sink, n);
        }
    };
    launch(100);                                     // warm-up
    (void)hipEventRecord(e0, s);
    launch(iters);
    (void)hipEventRecord(e1, s);
    int st = SS_OK;
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess || ms <= 0.f)
        st = SS_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != SS_OK) return st;
    // dense-equivalent operations: 2 * 32 * 32 * 32 per sparse instruction, 2 * 32 * 32 * 16 per dense one
    const double flop = (double)blocks * 8 * iters * kProbeAcc * (sparse ? 65536.0 : 32768.0);
    *tflops = (float)(flop / (ms * 1e-3) / 1e12);
    return SS_OK;
}

extern "C" int ss_debug_lds_bandwidth(int32_t write, int32_t waves_per_simd, int32_t row_bytes, void *scratch, size_t scratch_bytes,
                                      float *gb_per_s_per_cu, void *stream)
{
    if (!gb_per_s_per_cu || !scratch) return SS_ERR_INVALID_ARG;
    if (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4) return SS_ERR_INVALID_ARG;
    if (row_bytes < 16 || row_bytes > 592 || row_bytes % 16 != 0) return SS_ERR_INVALID_ARG;
    int dev = 0, ncu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0)
        return SS_ERR_HIP;
    if (scratch_bytes < (size_t)ncu * 1024 * 4) return SS_ERR_WORKSPACE;
    const int threads = 256 * waves_per_simd, iters = 2000;
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto kern = write == 0 ? lds_probe_kernel<0> : (write == 1 ? lds_probe_kernel<1> : (write == 2 ? lds_probe_kernel<2> : (write == 3 ? lds_probe_kernel<3> : lds_probe_kernel<4>)));
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess) return SS_ERR_HIP;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return SS_ERR_HIP;
    uint32_t *sink = static_cast<uint32_t *>(scratch);
    kern<<<ncu, threads, 65536, s>>>(sink, 10, row_bytes);
    (void)hipEventRecord(e0, s);
    kern<<<ncu, threads, 65536, s>>>(sink, iters, row_bytes);
    (void)hipEventRecord(e1, s);
    int st = SS_OK;
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess || ms <= 0.f)
        st = SS_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != SS_OK) return st;
    const double bytes_per_cu = (double)iters * 8 * 64 * 16 * (threads / 64);     // per workgroup = per compute unit
    *gb_per_s_per_cu = (float)(bytes_per_cu / (ms * 1e-3) / 1e9);
    return SS_OK;
}
