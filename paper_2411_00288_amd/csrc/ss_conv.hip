// NHWC implicit-GEMM convolution with a 2:4-sparse (or, for the twin, dense) weight operand.
//
// Sec. 3.3: Y~ = (M (.) W) U(X) (Eq. 6).  The unfold U(X) (Eq. 5) is never materialised: every
// workgroup builds the [pixels x reduction-chunk] slice of it that it needs in LDS, straight from
// the NHWC activations, and multiplies it with weight tiles that are already stored in the
// register layout of the matrix instruction.
//
//   GEMM view:  D[o, p] = sum_k A[o, k] * B[k, p]
//     A = weights, rows o = output channels (the sparse operand of V_SMFMAC must be A),
//     B = unfolded activations, columns p = (n, ho, wo) flattened, k = reduction index in the
//         flattening the descriptor declares (blocks of 4 consecutive k form a 2:4 group).
//   One 32x32x32 sparse MFMA consumes, per lane l: 8 kept weights of row l%32 (+16 index bits)
//   and the 16 activations k = 16*(l/32) + [0,16) of pixel l%32; it leaves rows
//   8*(v/4) + 4*(l/32) + v%4, v = 0..15, of column l%32 in the lane's 16 accumulators, i.e. runs
//   of 4 consecutive output channels of one pixel: an 8-byte NHWC store.
//   The dense twin issues two 32x32x16 dense MFMAs on the same B registers instead.
#include "ss_internal.h"

namespace ss {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct B32 {   // one lane's B fragment for a 32-wide reduction step: 16 x 16-bit
    uint4 lo, hi;
};

struct ConvParams {
    const uint16_t *x;
    const uint8_t *a_vals;    // first value tile (after the header)
    const uint32_t *a_meta;   // first metadata tile (sparse only)
    const float *bias;
    uint16_t *y;
    int N, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw, Ho, Wo, P, K, Ks, Kp, Mt, act, korder;
    int tiles_m;
};

enum { MODE_VEC = 0, MODE_GATHER = 1 };

template <int DT, int ABID>
__device__ __forceinline__ f32x16 mma_sparse(uint4 a, const B32 &b, f32x16 c, uint32_t idx)
{
    if constexpr (DT == SS_F16)
        return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x16, b), c,
                                                         (int)idx, 0, ABID);
    else
        return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x16, b), c,
                                                          (int)idx, 0, ABID);
}

template <int DT>
__device__ __forceinline__ f32x16 mma_dense(uint4 a, uint4 b, f32x16 c)
{
    if constexpr (DT == SS_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int DT>
__device__ __forceinline__ uint32_t cvt_pack2(float a, float b)
{
    if constexpr (DT == SS_F16) {
        _Float16 ha = (_Float16)a, hb = (_Float16)b;   // round-to-nearest-even
        return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
    } else {
        __bf16 ha = (__bf16)a, hb = (__bf16)b;         // round-to-nearest-even
        return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
    }
}

// Weight fragments of one reduction chunk (KSTEPS steps) for the TM row tiles of a wave.
template <bool SPARSE, int KSTEPS, int TM>
struct AFrag {
    uint4 v[KSTEPS][SPARSE ? 1 : 2][TM];
    uint32_t idx[(KSTEPS + 1) / 2][TM];
};

template <int DT, bool SPARSE, int WAVES_M, int WAVES_N, int TM, int TN, int MODE>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void conv_kernel(ConvParams p)
{
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int BM = WAVES_M * TM * 32;
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int KSTEPS = 2;
    constexpr int BK = KSTEPS * 32;
    constexpr int ROW = BK + 8;          // +16 bytes: consecutive pixels land 9 x 16 bytes apart -> conflict-free b128 reads
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *Bs0 = smem;
    uint16_t *Bs1 = smem + BN * ROW;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WAVES_M;
    const int wn = wave / WAVES_M;
    const int tile_m = blockIdx.x % p.tiles_m;
    const int tile_n = blockIdx.x / p.tiles_m;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int HoWo = p.Ho * p.Wo;

    // ------------------------------------------------------------------ activation staging state
    constexpr int UNITS = (MODE == MODE_VEC) ? 8 : 16;     // 16-byte chunks or 4-element blocks per pixel row
    constexpr int ITEMS = BN * UNITS / NT;
    static_assert(BN * UNITS % NT == 0 && NT % UNITS == 0, "tile/threads mismatch");
    const int unit = tid % UNITS;
    int pixoff[ITEMS], ih0[ITEMS], iw0[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; i++) {
        int pr = tid / UNITS + i * (NT / UNITS);
        int pg = n0 + pr;
        if (pg < p.P) {
            int n = pg / HoWo;
            int rem = pg - n * HoWo;
            int ho = rem / p.Wo;
            int wo = rem - ho * p.Wo;
            ih0[i] = ho * p.sh - p.ph;
            iw0[i] = wo * p.sw - p.pw;
            pixoff[i] = ((n * p.H + ih0[i]) * p.W + iw0[i]) * p.Cin;
        } else {
            ih0[i] = -(1 << 28);     // every bounds test fails -> zeros
            iw0[i] = -(1 << 28);
            pixoff[i] = 0;
        }
    }
    // MODE_VEC: position of this thread's 8-element chunk in the (tap, channel) space
    int vk = unit * 8, vc = 0, vr = 0, vt = 0;
    if constexpr (MODE == MODE_VEC) {
        int tap = vk / p.Cin;
        vc = vk - tap * p.Cin;
        vr = tap / p.kw;
        vt = tap - vr * p.kw;
    }

    uint4 stage_v[MODE == MODE_VEC ? ITEMS : 1];
    uint16_t stage_g[MODE == MODE_GATHER ? ITEMS : 1][4];

    auto stage_load = [&](int k0) {
        if constexpr (MODE == MODE_VEC) {
            (void)k0;
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
                int ih = ih0[i] + vr, iw = iw0[i] + vt;
                bool ok = vk < p.K && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (ok) v = *reinterpret_cast<const uint4 *>(p.x + (pixoff[i] + (vr * p.W + vt) * p.Cin + vc));
                stage_v[i] = v;
            }
            vk += BK;
            vc += BK;
            while (vc >= p.Cin) {
                vc -= p.Cin;
                if (++vt == p.kw) { vt = 0; ++vr; }
            }
        } else {
            int off[4], er[4], et[4];
            bool kok[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                int k = k0 + unit * 4 + e;
                kok[e] = k < p.K;
                int c, r, t;
                if (p.korder == SS_K_CRS) {
                    int khw = p.kh * p.kw;
                    c = k / khw;
                    int rem = k - c * khw;
                    r = rem / p.kw;
                    t = rem - r * p.kw;
                } else {
                    int tap = k / p.Cin;
                    c = k - tap * p.Cin;
                    r = tap / p.kw;
                    t = tap - r * p.kw;
                }
                er[e] = r;
                et[e] = t;
                off[e] = (r * p.W + t) * p.Cin + c;
            }
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    int ih = ih0[i] + er[e], iw = iw0[i] + et[e];
                    bool ok = kok[e] && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    stage_g[i][e] = ok ? p.x[pixoff[i] + off[e]] : (uint16_t)0;
                }
            }
        }
    };
    auto stage_store = [&](uint16_t *Bs) {
#pragma unroll
        for (int i = 0; i < ITEMS; i++) {
            int pr = tid / UNITS + i * (NT / UNITS);
            if constexpr (MODE == MODE_VEC) {
                *reinterpret_cast<uint4 *>(Bs + pr * ROW + unit * 8) = stage_v[i];
            } else {
                uint2 v = make_uint2((uint32_t)stage_g[i][0] | ((uint32_t)stage_g[i][1] << 16),
                                     (uint32_t)stage_g[i][2] | ((uint32_t)stage_g[i][3] << 16));
                *reinterpret_cast<uint2 *>(Bs + pr * ROW + unit * 4) = v;
            }
        }
    };

    // ------------------------------------------------------------------ weight fragments
    const int mt0 = (m0 >> 5) + wm * TM;
    auto load_a = [&](AFrag<SPARSE, KSTEPS, TM> &a, int ks0) {
#pragma unroll
        for (int s = 0; s < KSTEPS; s++) {
            int ks = ks0 + s;
#pragma unroll
            for (int tm = 0; tm < TM; tm++) {
                int mt = mt0 + tm;
                bool ok = ks < p.Ks && mt < p.Mt;
                if constexpr (SPARSE) {
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (ok) v = *reinterpret_cast<const uint4 *>(p.a_vals + (((size_t)mt * p.Ks + ks) * 64 + lane) * 16);
                    a.v[s][0][tm] = v;
                } else {
#pragma unroll
                    for (int h = 0; h < 2; h++) {
                        uint4 v = make_uint4(0, 0, 0, 0);
                        if (ok) v = *reinterpret_cast<const uint4 *>(p.a_vals + ((((size_t)mt * p.Ks + ks) * 2 + h) * 64 + lane) * 16);
                        a.v[s][h][tm] = v;
                    }
                }
            }
        }
        if constexpr (SPARSE) {
#pragma unroll
            for (int sp = 0; sp < (KSTEPS + 1) / 2; sp++) {
                int kp = (ks0 >> 1) + sp;
#pragma unroll
                for (int tm = 0; tm < TM; tm++) {
                    int mt = mt0 + tm;
                    uint32_t w = 0x44444444u;
                    if (kp < p.Kp && mt < p.Mt) w = p.a_meta[((size_t)mt * p.Kp + kp) * 64 + lane];
                    a.idx[sp][tm] = w;
                }
            }
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; tm++)
#pragma unroll
        for (int tn = 0; tn < TN; tn++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[tm][tn][v] = 0.f;

    auto compute = [&](const uint16_t *Bs, const AFrag<SPARSE, KSTEPS, TM> &a) {
#pragma unroll
        for (int s = 0; s < KSTEPS; s++) {
            B32 b[TN];
#pragma unroll
            for (int tn = 0; tn < TN; tn++) {
                const uint16_t *src = Bs + ((wn * TN + tn) * 32 + (lane & 31)) * ROW + s * 32 + 16 * (lane >> 5);
                b[tn].lo = *reinterpret_cast<const uint4 *>(src);
                b[tn].hi = *reinterpret_cast<const uint4 *>(src + 8);
            }
#pragma unroll
            for (int tm = 0; tm < TM; tm++)
#pragma unroll
                for (int tn = 0; tn < TN; tn++) {
                    if constexpr (SPARSE) {
                        if (s & 1) acc[tm][tn] = mma_sparse<DT, 1>(a.v[s][0][tm], b[tn], acc[tm][tn], a.idx[s >> 1][tm]);
                        else       acc[tm][tn] = mma_sparse<DT, 0>(a.v[s][0][tm], b[tn], acc[tm][tn], a.idx[s >> 1][tm]);
                    } else {
                        acc[tm][tn] = mma_dense<DT>(a.v[s][0][tm], b[tn].lo, acc[tm][tn]);
                        acc[tm][tn] = mma_dense<DT>(a.v[s][1][tm], b[tn].hi, acc[tm][tn]);
                    }
                }
        }
    };

    // ------------------------------------------------------------------ main loop (double-buffered LDS)
    const int nchunks = (p.Ks + KSTEPS - 1) / KSTEPS;
    AFrag<SPARSE, KSTEPS, TM> a_cur, a_nxt;
    stage_load(0);
    load_a(a_cur, 0);
    stage_store(Bs0);
    __syncthreads();
    for (int ci = 0; ci < nchunks; ci++) {
        uint16_t *cur = (ci & 1) ? Bs1 : Bs0;
        uint16_t *nxt = (ci & 1) ? Bs0 : Bs1;
        const bool more = ci + 1 < nchunks;
        if (more) {
            stage_load((ci + 1) * BK);
            load_a(a_nxt, (ci + 1) * KSTEPS);
        }
        compute(cur, a_cur);
        if (more) {
            stage_store(nxt);
            a_cur = a_nxt;
        }
        __syncthreads();
    }

    // ------------------------------------------------------------------ epilogue: bias, activation, one rounding, NHWC store
    const bool vec_ok = (p.Cout & 3) == 0;
#pragma unroll
    for (int tn = 0; tn < TN; tn++) {
        int pg = n0 + (wn * TN + tn) * 32 + (lane & 31);
        if (pg >= p.P) continue;
#pragma unroll
        for (int tm = 0; tm < TM; tm++) {
#pragma unroll
            for (int q = 0; q < 4; q++) {
                int o = m0 + (wm * TM + tm) * 32 + 8 * q + 4 * (lane >> 5);
                if (o >= p.Cout) continue;
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    float v = acc[tm][tn][4 * q + e];
                    if (p.bias != nullptr && o + e < p.Cout) v += p.bias[o + e];
                    if (p.act == SS_ACT_RELU) v = v > 0.f ? v : (v != v ? v : 0.f);
                    r[e] = v;
                }
                uint16_t *dst = p.y + (size_t)pg * p.Cout + o;
                if (vec_ok) {
                    *reinterpret_cast<uint2 *>(dst) = make_uint2(cvt_pack2<DT>(r[0], r[1]), cvt_pack2<DT>(r[2], r[3]));
                } else {
                    uint32_t lo = cvt_pack2<DT>(r[0], r[1]), hi = cvt_pack2<DT>(r[2], r[3]);
                    dst[0] = (uint16_t)lo;
                    if (o + 1 < p.Cout) dst[1] = (uint16_t)(lo >> 16);
                    if (o + 2 < p.Cout) dst[2] = (uint16_t)hi;
                    if (o + 3 < p.Cout) dst[3] = (uint16_t)(hi >> 16);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
template <int DT, bool SPARSE, int WAVES_M, int WAVES_N, int TM, int TN, int MODE>
static int launch(const ConvParams &p0, hipStream_t s)
{
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int ROW = 2 * 32 + 8;
    constexpr size_t smem = (size_t)2 * BN * ROW * sizeof(uint16_t);
    ConvParams p = p0;
    p.tiles_m = (p.Cout + BM - 1) / BM;
    long long tiles_n = ((long long)p.P + BN - 1) / BN;
    long long blocks = (long long)p.tiles_m * tiles_n;
    if (blocks <= 0 || blocks > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    auto kern = conv_kernel<DT, SPARSE, WAVES_M, WAVES_N, TM, TN, MODE>;
    if (smem > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return SS_ERR_HIP;
    }
    kern<<<dim3((unsigned)blocks), dim3(WAVES_M * WAVES_N * 64), smem, s>>>(p);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

template <int DT, bool SPARSE, int MODE>
static int pick_tile(const ConvParams &p, hipStream_t s)
{
    // Enough workgroups to cover the 256 compute units decides the tile size.
    long long big = (long long)((p.Cout + 127) / 128) * ((p.P + 127) / 128);
    if (p.Cout > 64 && big >= 256) return launch<DT, SPARSE, 2, 2, 2, 2, MODE>(p, s);
    return launch<DT, SPARSE, 2, 2, 1, 1, MODE>(p, s);
}

template <bool SPARSE>
static int conv_entry(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd, const void *wbuf,
                      const float *bias, int32_t sh, int32_t sw, int32_t ph, int32_t pw, int32_t act, void *y,
                      void *workspace, size_t ws_bytes, void *stream)
{
    (void)workspace;
    (void)ws_bytes;
    int st = check_desc(desc, SPARSE);
    if (st != SS_OK) return st;
    if (!x || !wbuf || !y) return SS_ERR_INVALID_ARG;
    if (N <= 0 || H <= 0 || Wd <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return SS_ERR_INVALID_ARG;
    if (act != SS_ACT_NONE && act != SS_ACT_RELU) return SS_ERR_INVALID_ARG;
    if (H + 2 * ph < desc->kh || Wd + 2 * pw < desc->kw) return SS_ERR_INVALID_ARG;
    if (!aligned(x, 16) || !aligned(wbuf, 16) || !aligned(y, 8) || (bias && !aligned(bias, 4))) return SS_ERR_INVALID_ARG;
    int Ho = (H + 2 * ph - desc->kh) / sh + 1;
    int Wo = (Wd + 2 * pw - desc->kw) / sw + 1;
    if (Ho <= 0 || Wo <= 0) return SS_ERR_INVALID_ARG;
    long long P = (long long)N * Ho * Wo;
    long long xelems = (long long)N * H * Wd * desc->cin;
    long long yelems = P * desc->cout;
    // 32-bit element offsets inside the kernel (with head-room for the padded halo arithmetic)
    if (xelems >= (1ll << 31) - (1ll << 24) || yelems >= (1ll << 31) || P >= (1ll << 31) - 256) return SS_ERR_UNSUPPORTED;
    if ((long long)(ph + desc->kh) * Wd * desc->cin >= (1ll << 30)) return SS_ERR_UNSUPPORTED;

    TileDims t = tile_dims(desc);
    ConvParams p;
    p.x = static_cast<const uint16_t *>(x);
    p.a_vals = static_cast<const uint8_t *>(wbuf) + kHeaderBytes;
    p.a_meta = reinterpret_cast<const uint32_t *>(p.a_vals + (size_t)t.Mt * t.Ks * 1024);
    p.bias = bias;
    p.y = static_cast<uint16_t *>(y);
    p.N = N; p.H = H; p.W = Wd; p.Cin = desc->cin; p.Cout = desc->cout; p.kh = desc->kh; p.kw = desc->kw;
    p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.Ho = Ho; p.Wo = Wo; p.P = (int)P;
    p.K = t.K; p.Ks = t.Ks; p.Kp = t.Kp; p.Mt = t.Mt; p.act = act; p.korder = desc->korder;
    p.tiles_m = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // channels contiguous inside every 8-element chunk of the reduction index?
    bool vec = (desc->cin % 8 == 0) && (desc->korder == SS_K_RSC || desc->kh * desc->kw == 1);
    if (desc->dtype == SS_F16) {
        return vec ? pick_tile<SS_F16, SPARSE, MODE_VEC>(p, s) : pick_tile<SS_F16, SPARSE, MODE_GATHER>(p, s);
    } else {
        return vec ? pick_tile<SS_BF16, SPARSE, MODE_VEC>(p, s) : pick_tile<SS_BF16, SPARSE, MODE_GATHER>(p, s);
    }
}

}  // namespace ss

using namespace ss;

extern "C" int ss_conv2d_workspace_bytes(const ss_weight_desc *desc, int32_t N, int32_t H, int32_t Wd, int32_t stride_h,
                                         int32_t stride_w, int32_t pad_h, int32_t pad_w, size_t *bytes)
{
    if (!bytes) return SS_ERR_INVALID_ARG;
    int st = check_desc(desc, false);
    if (st != SS_OK) return st;
    if (N <= 0 || H <= 0 || Wd <= 0 || stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return SS_ERR_INVALID_ARG;
    *bytes = 0;
    return SS_OK;
}

extern "C" int ss_conv2d_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                             const void *packed, const float *bias, int32_t stride_h, int32_t stride_w, int32_t pad_h,
                             int32_t pad_w, int32_t act, void *y, void *workspace, size_t ws_bytes, void *stream)
{
    return conv_entry<true>(desc, x, N, H, Wd, packed, bias, stride_h, stride_w, pad_h, pad_w, act, y, workspace,
                            ws_bytes, stream);
}

extern "C" int ss_conv2d_dense_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                                   const void *dense, const float *bias, int32_t stride_h, int32_t stride_w,
                                   int32_t pad_h, int32_t pad_w, int32_t act, void *y, void *workspace, size_t ws_bytes,
                                   void *stream)
{
    return conv_entry<false>(desc, x, N, H, Wd, dense, bias, stride_h, stride_w, pad_h, pad_w, act, y, workspace,
                             ws_bytes, stream);
}
