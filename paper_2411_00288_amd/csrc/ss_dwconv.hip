// Depthwise convolution (one filter per channel), NHWC 16-bit, stride 1: the grouped convolutions that the paper
// leaves dense (Sec. 4, "Architectures"), e.g. the 7x7 of a ConvNeXt block.  A simple dedicated kernel: it is
// bound by vector ALU work (49 multiply-adds per output), not by a matrix unit.
#include "ss_internal.h"

namespace ss {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ void widen8(const u32x4 &v, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 4; e++) {
        if constexpr (DT == SS_F16) {
            f[2 * e] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[e] & 0xFFFFu));
            f[2 * e + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[e] >> 16));
        } else {
            f[2 * e] = __builtin_bit_cast(float, v[e] << 16);
            f[2 * e + 1] = __builtin_bit_cast(float, v[e] & 0xFFFF0000u);
        }
    }
}

template <int DT>
__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    if constexpr (DT == SS_F16) {
        _Float16 ha = (_Float16)a, hb = (_Float16)b;
        return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
    } else {
        __bf16 ha = (__bf16)a, hb = (__bf16)b;
        return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
    }
}

constexpr int TW = 4;      // adjacent outputs along the image row per thread: a loaded input vector serves up to KW of them

// One thread: TW output pixels x 8 channels.  The filter taps sit in LDS ([kh][KW][C], 16-bit); input vectors come
// through raw buffer loads whose offset is out of range outside the image (the hardware returns zeros).
template <int DT, int KW>
__global__ __launch_bounds__(256) void dwconv_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w,
                                                     const float *__restrict__ bias, uint16_t *__restrict__ y, int N, int H,
                                                     int W, int C, int kh, int ph, int pw, int Ho, int Wo, int act,
                                                     unsigned x_bytes)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t w_s[];
    const int ntap = kh * KW * C;
    for (int i = threadIdx.x * 8; i < ntap; i += 256 * 8)
        *reinterpret_cast<u32x4 *>(w_s + i) = *reinterpret_cast<const u32x4 *>(w + i);
    __syncthreads();
    const int runs = C >> 3, wq = (Wo + TW - 1) / TW;
    const long long total = (long long)N * Ho * wq * runs;
    const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    const int run = (int)(gid % runs);
    long long rest = gid / runs;
    const int wo0 = (int)(rest % wq) * TW;
    rest /= wq;
    const int ho = (int)(rest % Ho);
    const int n = (int)(rest / Ho);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(x), 0, (int)x_bytes, 0x00020000);

    float acc[TW][8];
    {
        float b[8];
#pragma unroll
        for (int e = 0; e < 8; e++) b[e] = bias ? bias[run * 8 + e] : 0.f;
#pragma unroll
        for (int j = 0; j < TW; j++)
#pragma unroll
            for (int e = 0; e < 8; e++) acc[j][e] = b[e];
    }
    for (int r = 0; r < kh; r++) {
        const int ih = ho - ph + r;
        if ((unsigned)ih >= (unsigned)H) continue;
        float xf[KW + TW - 1][8];
#pragma unroll
        for (int j = 0; j < KW + TW - 1; j++) {
            const int iw = wo0 - pw + j;
            const unsigned off = (unsigned)iw < (unsigned)W ? (unsigned)((((size_t)n * H + ih) * W + iw) * C + run * 8) * 2u : 0x80000000u;
            widen8<DT>(__builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0), xf[j]);
        }
#pragma unroll
        for (int t = 0; t < KW; t++) {
            float wf[8];
            widen8<DT>(*reinterpret_cast<const u32x4 *>(w_s + ((size_t)r * KW + t) * C + run * 8), wf);
#pragma unroll
            for (int j = 0; j < TW; j++)
#pragma unroll
                for (int e = 0; e < 8; e++) acc[j][e] = __builtin_fmaf(wf[e], xf[j + t][e], acc[j][e]);
        }
    }
#pragma unroll
    for (int j = 0; j < TW; j++) {
        if (wo0 + j >= Wo) break;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const float z = acc[j][e];
            v[e] = act == SS_ACT_RELU ? (z < 0.f ? 0.f : z) : z;
        }
        u32x4 out = {pack2<DT>(v[0], v[1]), pack2<DT>(v[2], v[3]), pack2<DT>(v[4], v[5]), pack2<DT>(v[6], v[7])};
        *reinterpret_cast<u32x4 *>(y + ((((size_t)n * Ho + ho) * Wo + wo0 + j) * C + run * 8)) = out;
    }
}

template <int DT>
static int launch_dw(const uint16_t *x, const uint16_t *w, const float *bias, uint16_t *y, int N, int H, int W, int C, int kh,
                     int kw, int ph, int pw, int Ho, int Wo, int act, unsigned x_bytes, hipStream_t s)
{
    const long long total = (long long)N * Ho * ((Wo + TW - 1) / TW) * (C / 8);
    if (total <= 0 || (total + 255) / 256 > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    const size_t smem = (size_t)kh * kw * C * 2;
    switch (kw) {
        case 3: dwconv_kernel<DT, 3><<<grid, block, smem, s>>>(x, w, bias, y, N, H, W, C, kh, ph, pw, Ho, Wo, act, x_bytes); break;
        case 5: dwconv_kernel<DT, 5><<<grid, block, smem, s>>>(x, w, bias, y, N, H, W, C, kh, ph, pw, Ho, Wo, act, x_bytes); break;
        case 7: dwconv_kernel<DT, 7><<<grid, block, smem, s>>>(x, w, bias, y, N, H, W, C, kh, ph, pw, Ho, Wo, act, x_bytes); break;
        default: return SS_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

}  // namespace ss

using namespace ss;

extern "C" int ss_dwconv2d_fwd(const void *x, int32_t N, int32_t H, int32_t Wd, int32_t C, int32_t dtype, const void *w,
                               const float *bias, int32_t kh, int32_t kw, int32_t pad_h, int32_t pad_w, int32_t act,
                               void *y, void *stream)
{
    if (!x || !w || !y) return SS_ERR_INVALID_ARG;
    if (N <= 0 || H <= 0 || Wd <= 0 || C <= 0 || kh <= 0 || kw <= 0 || pad_h < 0 || pad_w < 0) return SS_ERR_INVALID_ARG;
    if (dtype != SS_F16 && dtype != SS_BF16) return SS_ERR_INVALID_ARG;
    if (act != SS_ACT_NONE && act != SS_ACT_RELU) return SS_ERR_INVALID_ARG;
    if (((uintptr_t)x & 15) || ((uintptr_t)w & 15) || ((uintptr_t)y & 15) || (bias && ((uintptr_t)bias & 3))) return SS_ERR_INVALID_ARG;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw) return SS_ERR_INVALID_ARG;
    if (C % 8 != 0 || (kw != 3 && kw != 5 && kw != 7) || (long long)kh * kw * C * 2 > 64 * 1024) return SS_ERR_UNSUPPORTED;
    const long long xbytes = (long long)N * H * Wd * C * 2;
    if (xbytes >= (1ll << 31)) return SS_ERR_UNSUPPORTED;
    const int Ho = H + 2 * pad_h - kh + 1, Wo = Wd + 2 * pad_w - kw + 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *xs = static_cast<const uint16_t *>(x), *ws = static_cast<const uint16_t *>(w);
    uint16_t *ys = static_cast<uint16_t *>(y);
    return dtype == SS_F16 ? launch_dw<SS_F16>(xs, ws, bias, ys, N, H, Wd, C, kh, kw, pad_h, pad_w, Ho, Wo, act, (unsigned)xbytes, s)
                           : launch_dw<SS_BF16>(xs, ws, bias, ys, N, H, Wd, C, kh, kw, pad_h, pad_w, Ho, Wo, act, (unsigned)xbytes, s);
}
