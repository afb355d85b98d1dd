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

// How the [pixels x reduction-chunk] slice of the unfolded input is built in LDS:
//   MODE_VEC    channels are contiguous inside every aligned run of 8 reduction indices (1x1
//               kernels, or the channels-last flattening, with cin % 8 == 0): 16-byte loads.
//   MODE_GATHER any flattening / shape: one 16-bit load per element.
//   MODE_TAPS   the paper's flattening (channel slowest) with a KH x KW kernel and cin % 4 == 0:
//               a 2:4 block then holds 4 consecutive (channel, tap) pairs, i.e. activations of
//               different pixels.  A thread loads, for one output pixel and 4 channels, the
//               KH*KW taps as 8-byte channel vectors and transposes them in registers to
//               channel-major order before the LDS write, so the MFMA side still reads 16-byte
//               vectors.  A chunk is 32 channels = KH*KW reduction steps.
enum { MODE_VEC = 0, MODE_GATHER = 1, MODE_TAPS = 2 };

// Weight fragments of one 32-wide reduction step for the TM row tiles of a wave.
template <bool SPARSE, int TM>
struct AStep {
    uint4 v[SPARSE ? 1 : 2][TM];
    uint32_t idx[TM];
};

template <int DT, bool SPARSE, int WAVES_M, int WAVES_N, int TM, int TN, int MODE, int KH, int KW>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void conv_kernel(ConvParams p)
{
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int BM = WAVES_M * TM * 32;
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int TAPS = KH * KW;
    constexpr int KSTEPS = (MODE == MODE_TAPS) ? TAPS : 2;    // 32-wide reduction steps per LDS chunk
    constexpr int RING = (KSTEPS % 3 == 0) ? 3 : ((KSTEPS % 4 == 0) ? 4 : 2);   // weight prefetch ring, divides KSTEPS
    constexpr int PF = RING - 1;
    static_assert(KSTEPS % RING == 0, "ring must divide the chunk");
    constexpr int BK = KSTEPS * 32;
    constexpr int ROW = BK + 8;          // +16 bytes per pixel row: 16-byte LDS reads of 16 consecutive pixels hit distinct banks
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
    constexpr int UNITS = (MODE == MODE_GATHER) ? 16 : 8;   // per pixel row and chunk: 4-element blocks / 16-byte runs / 4-channel bricks
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
    // MODE_VEC: position of this thread's 8-element run in the (tap, channel) space
    int vk = unit * 8, vc = 0, vr = 0, vt = 0;
    if constexpr (MODE == MODE_VEC) {
        int tap = vk / p.Cin;
        vc = vk - tap * p.Cin;
        vr = tap / p.kw;
        vt = tap - vr * p.kw;
    }

    uint4 stage_v[MODE == MODE_VEC ? ITEMS : 1];
    uint16_t stage_g[MODE == MODE_GATHER ? ITEMS : 1][4];
    uint2 stage_t[MODE == MODE_TAPS ? ITEMS : 1][MODE == MODE_TAPS ? TAPS : 1];

    auto stage_load = [&](int ci) {
        if constexpr (MODE == MODE_VEC) {
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
        } else if constexpr (MODE == MODE_GATHER) {
            int off[4], er[4], et[4];
            bool kok[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                int k = ci * BK + unit * 4 + e;
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
        } else {
            const int cb = ci * 32 + unit * 4;          // first of this thread's 4 channels
            const bool cok = cb < p.Cin;
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
#pragma unroll
                for (int tap = 0; tap < TAPS; tap++) {
                    const int r = tap / KW, t = tap % KW;
                    int ih = ih0[i] + r, iw = iw0[i] + t;
                    bool ok = cok && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    uint2 v = make_uint2(0, 0);
                    if (ok) v = *reinterpret_cast<const uint2 *>(p.x + (pixoff[i] + (r * p.W + t) * p.Cin + cb));
                    stage_t[i][tap] = v;
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
            } else if constexpr (MODE == MODE_GATHER) {
                uint2 v = make_uint2((uint32_t)stage_g[i][0] | ((uint32_t)stage_g[i][1] << 16),
                                     (uint32_t)stage_g[i][2] | ((uint32_t)stage_g[i][3] << 16));
                *reinterpret_cast<uint2 *>(Bs + pr * ROW + unit * 4) = v;
            } else {
                // [tap][4 channels] -> [channel][tap]: output element h = c*TAPS + tap, two per dword
                uint32_t o[2 * TAPS];
#pragma unroll
                for (int d = 0; d < 2 * TAPS; d++) {
                    const int ha = 2 * d, hb = 2 * d + 1;
                    const int ca = ha / TAPS, ta = ha % TAPS, cbn = hb / TAPS, tb = hb % TAPS;
                    uint32_t sa = (ca < 2) ? stage_t[i][ta].x : stage_t[i][ta].y;
                    uint32_t sb = (cbn < 2) ? stage_t[i][tb].x : stage_t[i][tb].y;
                    const uint32_t sel = (uint32_t)(2 * (ca & 1)) | ((uint32_t)(2 * (ca & 1) + 1) << 8) |
                                         ((uint32_t)(4 + 2 * (cbn & 1)) << 16) | ((uint32_t)(5 + 2 * (cbn & 1)) << 24);
                    o[d] = __builtin_amdgcn_perm(sb, sa, sel);
                }
                uint2 *dst = reinterpret_cast<uint2 *>(Bs + pr * ROW + unit * (4 * TAPS));
#pragma unroll
                for (int d = 0; d < TAPS; d++) dst[d] = make_uint2(o[2 * d], o[2 * d + 1]);
            }
        }
    };

    // ------------------------------------------------------------------ weight fragments
    const int mt0 = (m0 >> 5) + wm * TM;
    auto load_a = [&](AStep<SPARSE, TM> &a, int ks) {
#pragma unroll
        for (int tm = 0; tm < TM; tm++) {
            int mt = mt0 + tm;
            bool ok = ks < p.Ks && mt < p.Mt;
            if constexpr (SPARSE) {
                uint4 v = make_uint4(0, 0, 0, 0);
                uint32_t w = 0x44444444u;
                if (ok) {
                    v = *reinterpret_cast<const uint4 *>(p.a_vals + (((size_t)mt * p.Ks + ks) * 64 + lane) * 16);
                    w = p.a_meta[((size_t)mt * p.Kp + (ks >> 1)) * 64 + lane];
                }
                a.v[0][tm] = v;
                a.idx[tm] = (ks & 1) ? (w >> 16) : w;    // the instruction reads index bits [15:0]
            } else {
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (ok) v = *reinterpret_cast<const uint4 *>(p.a_vals + ((((size_t)mt * p.Ks + ks) * 2 + h) * 64 + lane) * 16);
                    a.v[h][tm] = v;
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

    // ------------------------------------------------------------------ main loop (double-buffered LDS, ring of weight steps)
    const int nchunks = (p.Ks + KSTEPS - 1) / KSTEPS;
    AStep<SPARSE, TM> a[RING];
    stage_load(0);
#pragma unroll
    for (int s = 0; s < PF; s++) load_a(a[s], s);
    stage_store(Bs0);
    __syncthreads();
    for (int ci = 0; ci < nchunks; ci++) {
        const uint16_t *cur = (ci & 1) ? Bs1 : Bs0;
        uint16_t *nxt = (ci & 1) ? Bs0 : Bs1;
        const bool more = ci + 1 < nchunks;
        if (more) stage_load(ci + 1);
#pragma unroll
        for (int s = 0; s < KSTEPS; s++) {
            load_a(a[(s + PF) % RING], ci * KSTEPS + s + PF);
            B32 b[TN];
#pragma unroll
            for (int tn = 0; tn < TN; tn++) {
                const uint16_t *src = cur + ((wn * TN + tn) * 32 + (lane & 31)) * ROW + s * 32 + 16 * (lane >> 5);
                b[tn].lo = *reinterpret_cast<const uint4 *>(src);
                b[tn].hi = *reinterpret_cast<const uint4 *>(src + 8);
            }
            const AStep<SPARSE, TM> &as = a[s % RING];
#pragma unroll
            for (int tm = 0; tm < TM; tm++)
#pragma unroll
                for (int tn = 0; tn < TN; tn++) {
                    if constexpr (SPARSE) {
                        acc[tm][tn] = mma_sparse<DT, 0>(as.v[0][tm], b[tn], acc[tm][tn], as.idx[tm]);
                    } else {
                        acc[tm][tn] = mma_dense<DT>(as.v[0][tm], b[tn].lo, acc[tm][tn]);
                        acc[tm][tn] = mma_dense<DT>(as.v[1][tm], b[tn].hi, acc[tm][tn]);
                    }
                }
        }
        if (more) stage_store(nxt);
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
template <int DT, bool SPARSE, int WAVES_M, int WAVES_N, int TM, int TN, int MODE, int KH, int KW>
static int launch(const ConvParams &p0, hipStream_t s)
{
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int KSTEPS = (MODE == MODE_TAPS) ? KH * KW : 2;
    constexpr int ROW = KSTEPS * 32 + 8;
    constexpr size_t smem = (size_t)2 * BN * ROW * sizeof(uint16_t);
    static_assert(smem <= 160 * 1024, "LDS tile too large");
    ConvParams p = p0;
    p.tiles_m = (p.Cout + BM - 1) / BM;
    long long tiles_n = ((long long)p.P + BN - 1) / BN;
    long long blocks = (long long)p.tiles_m * tiles_n;
    if (blocks <= 0 || blocks > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    auto kern = conv_kernel<DT, SPARSE, WAVES_M, WAVES_N, TM, TN, MODE, KH, KW>;
    if (smem > 64 * 1024) {
        static bool attr_set = false;    // once per process: raises this kernel's dynamic-LDS limit
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)smem) != hipSuccess)
                return SS_ERR_HIP;
            attr_set = true;
        }
    }
    kern<<<dim3((unsigned)blocks), dim3(WAVES_M * WAVES_N * 64), smem, s>>>(p);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

template <int DT, bool SPARSE, int MODE, int KH, int KW>
static int pick_tile(const ConvParams &p, hipStream_t s)
{
    // Enough workgroups to cover the 256 compute units decides the tile size.
    long long big = (long long)((p.Cout + 127) / 128) * ((p.P + 127) / 128);
    if constexpr (MODE == MODE_TAPS && KH * KW > 4) {
        // a 128-pixel tile of the 3x3 unfold does not fit LDS twice: 128 x 64 is the large shape
        if (p.Cout > 64 && big >= 128) return launch<DT, SPARSE, 2, 2, 2, 1, MODE, KH, KW>(p, s);
    } else {
        if (p.Cout > 64 && big >= 256) return launch<DT, SPARSE, 2, 2, 2, 2, MODE, KH, KW>(p, s);
    }
    return launch<DT, SPARSE, 2, 2, 1, 1, MODE, KH, KW>(p, s);
}

template <int DT, bool SPARSE>
static int pick_mode(const ss_weight_desc *desc, const ConvParams &p, hipStream_t s)
{
    const int taps = desc->kh * desc->kw;
    // channels contiguous inside every aligned run of 8 reduction indices?
    if ((desc->cin % 8 == 0) && (desc->korder == SS_K_RSC || taps == 1)) return pick_tile<DT, SPARSE, MODE_VEC, 1, 1>(p, s);
    if (desc->korder == SS_K_CRS && desc->cin % 4 == 0) {
        if (desc->kh == 3 && desc->kw == 3) return pick_tile<DT, SPARSE, MODE_TAPS, 3, 3>(p, s);
        if (desc->kh == 2 && desc->kw == 2) return pick_tile<DT, SPARSE, MODE_TAPS, 2, 2>(p, s);
    }
    return pick_tile<DT, SPARSE, MODE_GATHER, 1, 1>(p, s);
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
    return desc->dtype == SS_F16 ? pick_mode<SS_F16, SPARSE>(desc, p, s) : pick_mode<SS_BF16, SPARSE>(desc, p, s);
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
