// Max pooling over NHWC 16-bit activations: the one non-convolution step between the convolutions of a
// ResNet trunk (after the stem), so that a chained stack runs without leaving the library.
#include "ss_internal.h"

namespace ss {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ float widen16(uint32_t bits)
{
    if constexpr (DT == SS_F16)
        return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
    else
        return __builtin_bit_cast(float, bits << 16);
}

// One thread per (output pixel, run of 8 channels): k*k 16-byte loads, element-wise maximum.  The result is
// one of the inputs (its bit pattern is copied); positions outside the image do not take part; a NaN wins.
template <int DT>
__global__ __launch_bounds__(256) void maxpool_kernel(const uint16_t *__restrict__ x, uint16_t *__restrict__ y, int N,
                                                      int H, int W, int C, int k, int s, int pad, int Ho, int Wo)
{
    const int runs = C >> 3;
    const long long total = (long long)N * Ho * Wo * runs;
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    const int run = (int)(gid % runs);
    long long pix = gid / runs;
    const int wo = (int)(pix % Wo);
    pix /= Wo;
    const int ho = (int)(pix % Ho);
    const int n = (int)(pix / Ho);
    uint32_t best[8];
    float bestf[8];
    bool have = false;
    for (int r = 0; r < k; r++) {
        const int ih = ho * s - pad + r;
        if ((unsigned)ih >= (unsigned)H) continue;
        for (int t = 0; t < k; t++) {
            const int iw = wo * s - pad + t;
            if ((unsigned)iw >= (unsigned)W) continue;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(x + (((size_t)n * H + ih) * W + iw) * C + run * 8);
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint32_t b = (v[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                const float f = widen16<DT>(b);
                if (!have || f > bestf[e] || f != f) {
                    if (!(have && bestf[e] != bestf[e])) {      // a NaN already there stays
                        best[e] = b;
                        bestf[e] = f;
                    }
                }
            }
            have = true;
        }
    }
    u32x4 out;
#pragma unroll
    for (int e = 0; e < 4; e++) out[e] = have ? (best[2 * e] | (best[2 * e + 1] << 16)) : 0u;
    *reinterpret_cast<u32x4 *>(y + (((size_t)n * Ho + ho) * Wo + wo) * C + run * 8) = out;
}

}  // namespace ss

using namespace ss;

extern "C" int ss_maxpool2d(const void *x, int32_t N, int32_t H, int32_t Wd, int32_t C, int32_t dtype, int32_t k,
                            int32_t stride, int32_t pad, void *y, void *stream)
{
    if (!x || !y) return SS_ERR_INVALID_ARG;
    if (N <= 0 || H <= 0 || Wd <= 0 || C <= 0 || k <= 0 || stride <= 0 || pad < 0 || 2 * pad > k) return SS_ERR_INVALID_ARG;
    if (dtype != SS_F16 && dtype != SS_BF16) return SS_ERR_INVALID_ARG;
    if (C % 8 != 0) return SS_ERR_UNSUPPORTED;
    if (((uintptr_t)x & 15) || ((uintptr_t)y & 15)) return SS_ERR_INVALID_ARG;
    if (H + 2 * pad < k || Wd + 2 * pad < k) return SS_ERR_INVALID_ARG;
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
    const long long total = (long long)N * Ho * Wo * (C / 8);
    if (total <= 0 || (total + 255) / 256 > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == SS_F16)
        maxpool_kernel<SS_F16><<<grid, block, 0, s>>>(static_cast<const uint16_t *>(x), static_cast<uint16_t *>(y), N, H,
                                                      Wd, C, k, stride, pad, Ho, Wo);
    else
        maxpool_kernel<SS_BF16><<<grid, block, 0, s>>>(static_cast<const uint16_t *>(x), static_cast<uint16_t *>(y), N, H,
                                                       Wd, C, k, stride, pad, Ho, Wo);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}
