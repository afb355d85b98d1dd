// Pointwise (1x1) convolution with the activation tile stationary: Sec. 3.3 Eq. 6 for kh = kw = 1, where the unfold
// is the identity and a layer is Y = (M (.) W) X with X the [K x pixels] activation matrix.
//
// The channel-expanding 1x1 layers of a bottleneck (K = 64 ... 512, Cout = 4 K) have short reductions: in the
// one-tile-per-workgroup kernels a workgroup lives for a prologue (first loads, LDS fill), two to sixteen reduction
// steps and an epilogue (store drain), and the steps are the smallest part.  Here a workgroup loads its 64 pixels'
// activations (all K channels) into LDS once and then walks down the output channels: each of the four waves takes
// 64 rows of W at a time, multiplies them against the resident tile (a 2 x 2 block of 32 x 32 accumulator tiles per
// step: every activation fragment read from LDS and every weight fragment fetched from memory feeds two matrix
// instructions), writes its 64 x 64 outputs through a private LDS slab and goes on to its next 64 rows with no
// barrier in between.  The weight fragments travel in a register ring that runs ahead across the hand-over from one
// row block to the next, so the only exposed memory latency is the workgroup's first.
// Bias, residual (added in fp32 before the activation), activation and the single rounding are those of the other
// kernels; the bias starts in the accumulators.
#ifndef SS_CONV_ROWS_H_
#define SS_CONV_ROWS_H_
#include "ss_conv_stream.h"

namespace ss {

template <int KS>
struct RowsShape {
    static constexpr int BN = 64;                               // pixels of a workgroup
    static constexpr int K = 32 * KS;
    static constexpr int ROW = K + 8;                           // 16-bit units per pixel row in LDS (+16 bytes: conflict-free 16-byte reads)
    static constexpr int SLAB_ROW = 32 + 4;                     // floats per pixel row of a wave's output slab
    static constexpr size_t b_bytes = (size_t)BN * ROW * 2;
    static constexpr size_t slab_bytes = (size_t)4 * 32 * SLAB_ROW * 4;
};
template <int KS>
static inline size_t rows_smem_bytes(int pairs_per_group)
{
    return RowsShape<KS>::b_bytes + RowsShape<KS>::slab_bytes + (size_t)pairs_per_group * 64 * 4;
}

// mg workgroups share a pixel tile; each takes pairs_per_group blocks of 64 output channels.
template <int DT, bool SPARSE, int KS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv_pw_rows_kernel(ConvParams p, int mg, int pairs_per_group)
{
    using SH = RowsShape<KS>;
    constexpr int BN = SH::BN, ROW = SH::ROW, VPP = SH::K / 8;      // 16-byte vectors per pixel
    constexpr int RMAX = SPARSE ? 8 : 4;                             // (a dense fragment is twice the registers)
    constexpr int R = KS < RMAX ? KS : RMAX;                         // weight ring: reduction steps in flight
    static_assert(KS % R == 0, "the ring nests with the reduction");
    constexpr int ODT = DT;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *const Bs = reinterpret_cast<uint16_t *>(smem_raw);
    float *const slab_all = reinterpret_cast<float *>(smem_raw + SH::b_bytes);
    float *const bias_s = reinterpret_cast<float *>(smem_raw + SH::b_bytes + SH::slab_bytes);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g2 = lane >> 5, c2 = lane & 31;
    const int tile_n = blockIdx.x / mg, grp = blockIdx.x - tile_n * mg;
    const int n0 = tile_n * BN;
    const int pairs_all = (p.Mt + 1) >> 1;
    const int rp0 = grp * pairs_per_group;
    const int rp1 = min(rp0 + pairs_per_group, pairs_all);

    // ---- the activation tile: 64 pixels x K channels, 16-byte loads, one LDS row per pixel
    {
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, (int)p.x_bytes, kRsrcFlags);
        const int HoWo = p.Ho * p.Wo;
        u32x4 v[KS];
#pragma unroll
        for (int i = 0; i < KS; i++) {
            const int idx = tid + 256 * i;
            const int pl = idx / VPP, vec = idx % VPP;
            const int pg = n0 + pl;
            const bool live = pg < p.P;
            const int n = fast_div(live ? pg : 0, p.howo_mul, p.howo_sh);
            const int rem = (live ? pg : 0) - n * HoWo;
            const int ho = fast_div(rem, p.wo_mul, p.wo_sh);
            const int wo = rem - ho * p.Wo;
            const int ih = ho * p.sh - p.ph, iw = wo * p.sw - p.pw;
            const bool ok = live && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            const unsigned off = (unsigned)(((n * p.H + ih) * p.W + iw) * p.Cin * 2) + (unsigned)vec * 16u;
            v[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(ok ? off : kOutOfRange), 0, 0);
        }
        for (int i = tid; i < (rp1 - rp0) * 64; i += 256) {
            const int o = rp0 * 64 + i;
            bias_s[i] = (p.bias != nullptr && o < p.Cout) ? p.bias[o] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < KS; i++) {
            const int idx = tid + 256 * i;
            const int pl = idx / VPP, vec = idx % VPP;
            *reinterpret_cast<u32x4 *>(Bs + pl * ROW + vec * 8) = v[i];
        }
    }
    __syncthreads();                                  // the only barrier

    int rp = rp0 + wave;                              // this wave's first block of 64 rows; the next ones follow at a stride of 4
    if (rp >= rp1) return;

    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a_vals), 0, (int)p.a_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.a_meta), 0, (int)p.meta_bytes, kRsrcFlags);
    const unsigned ybytes = (unsigned)p.P * (unsigned)p.Cout * 2u;
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)ybytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.residual), 0, p.residual ? (int)ybytes : 0, kRsrcFlags);
    const unsigned a_lane = (unsigned)lane * 16u, m_lane = (unsigned)lane * 4u;
    struct AFrag {
        u32x4 v[SPARSE ? 1 : 2];
        uint32_t idx;
    };
    AFrag a[R][2];
    // Weight fragments of reduction step ks for the two row tiles of row block rpb (a block past the last repeats the
    // last one: fetched, never used).
    auto load_a = [&](AFrag (&f)[2], int rpb, int ks) {
#pragma unroll
        for (int tm = 0; tm < 2; tm++) {
            const int mt = min(2 * rpb + tm, p.Mt - 1);
            if constexpr (SPARSE) {
                f[tm].v[0] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_lane, (mt * p.Ks + ks) * 1024, 0);
                f[tm].idx = __builtin_amdgcn_raw_buffer_load_b32(rm, (int)m_lane, (mt * p.Kp + (ks >> 1)) * 256, 0);
            } else {
                f[tm].v[0] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_lane, (mt * p.Ks + ks) * 2048, 0);
                f[tm].v[1] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_lane, (mt * p.Ks + ks) * 2048 + 1024, 0);
            }
        }
    };
    // Activation fragment of step ks for pixel subtile tn: this lane's 16 reduction indices of pixel c2
    const uint16_t *const bsrc = Bs + c2 * ROW + 16 * g2;
    B32 b[2][2];
    auto load_b = [&](B32 (&f)[2], int ks) {
#pragma unroll
        for (int tn = 0; tn < 2; tn++) {
            const uint16_t *src = bsrc + tn * 32 * ROW + 32 * ks;
            f[tn].lo = *reinterpret_cast<const u32x4 *>(src);
            f[tn].hi = *reinterpret_cast<const u32x4 *>(src + 8);
        }
    };
    float *const slab = slab_all + wave * 32 * SH::SLAB_ROW;
    const float relu_floor = p.act == SS_ACT_RELU ? 0.f : -__builtin_inff();
    const bool has_res = p.residual != nullptr;
    // Byte offset of this lane's 16-byte output run number j of tile t = 2 tm + tn of row block rpb: a pixel past the
    // last lies past the buffer's end, a channel past the last is sent there.
    auto out_off = [&](int rpb, int t, int j) {
        const int it = lane + 64 * j;
        const int pg = n0 + (t & 1) * 32 + (it >> 2), o = rpb * 64 + (t >> 1) * 32 + (it & 3) * 8;
        return o < p.Cout ? ((unsigned)pg * (unsigned)p.Cout + (unsigned)o) * 2u : kOutOfRange;
    };
    u32x4 res[2][2];                                  // residual runs of two tiles in flight
    auto load_res = [&](u32x4 (&f)[2], int rpb, int t) {
#pragma unroll
        for (int j = 0; j < 2; j++) f[j] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)out_off(rpb, t, j), 0, 0);
    };

#pragma unroll
    for (int s = 0; s < R; s++) {
        load_a(a[s], rp, s);
        __builtin_amdgcn_sched_barrier(0);
    }
    load_b(b[0], 0);

    for (; rp < rp1; rp += 4) {
        Acc<DT> acc[2][2];
#pragma unroll
        for (int tm = 0; tm < 2; tm++)
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const f32x4 bq = *reinterpret_cast<const f32x4 *>(bias_s + (rp - rp0) * 64 + tm * 32 + 8 * q + 4 * g2);
#pragma unroll
                for (int tn = 0; tn < 2; tn++)
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[tm][tn][4 * q + e] = bq[e];
            }
        const int rpn = rp + 4;
        if (has_res) load_res(res[0], rp, 0);         // its latency hides behind the reduction
#pragma unroll
        for (int s = 0; s < KS; s++) {
            // the next step's activation fragments; after the last step, step 0 again for the next row block, into
            // buffer 0 -- which an odd number of steps is still reading from, so that load then follows the step
            if (s + 1 < KS) load_b(b[(s + 1) & 1], s + 1);
            else if (KS % 2 == 0) load_b(b[0], 0);
#pragma unroll
            for (int tn = 0; tn < 2; tn++)
#pragma unroll
                for (int tm = 0; tm < 2; tm++) {
                    const AFrag &af = a[s % R][tm];
                    if constexpr (SPARSE) {
                        acc[tm][tn] = mma_sparse<DT>(af.v[0], b[s & 1][tn], acc[tm][tn], af.idx >> ((s & 1) * 16));
                    } else {
                        acc[tm][tn] = mma_dense<DT>(af.v[0], b[s & 1][tn].lo, acc[tm][tn]);
                        acc[tm][tn] = mma_dense<DT>(af.v[1], b[s & 1][tn].hi, acc[tm][tn]);
                    }
                }
            if (s + 1 == KS && KS % 2 == 1) load_b(b[0], 0);
            // the slot is free: fetch the step R ahead, which may belong to the next row block
            if (s + R < KS) load_a(a[s % R], rp, s + R);
            else load_a(a[s % R], rpn, s + R - KS);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- epilogue: 2 x 2 tiles of 32 channels x 32 pixels through the slab, fp32; residual, activation, rounding
        // (the residual runs of tile t + 1 are fetched while tile t is written; those of tile 0 were fetched before the
        // reduction, see above)
        // (A wave's LDS operations execute in order: a piece's reads see its writes, and the next piece may be written
        // as soon as this one's reads are issued -- its writes then cover part of the slab's read latency.)
        auto write_out = [&](auto actf) {
            auto put = [&](int t) {
                const int tm = t >> 1, tn = t & 1;
#pragma unroll
                for (int q = 0; q < 4; q++)
                    *reinterpret_cast<f32x4 *>(slab + c2 * SH::SLAB_ROW + 8 * q + 4 * g2) =
                        f32x4{acc[tm][tn][4 * q + 0], acc[tm][tn][4 * q + 1], acc[tm][tn][4 * q + 2], acc[tm][tn][4 * q + 3]};
            };
            put(0);
#pragma unroll
            for (int t = 0; t < 4; t++) {
                if (has_res && t + 1 < 4) load_res(res[(t + 1) & 1], rp, t + 1);
                f32x4 lo[2], hi[2];
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    const int it = lane + 64 * j;
                    const int px = it >> 2, run = it & 3;
                    lo[j] = *reinterpret_cast<const f32x4 *>(slab + px * SH::SLAB_ROW + run * 8);
                    hi[j] = *reinterpret_cast<const f32x4 *>(slab + px * SH::SLAB_ROW + run * 8 + 4);
                }
                if (t + 1 < 4) put(t + 1);
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    float v[8] = {lo[j][0], lo[j][1], lo[j][2], lo[j][3], hi[j][0], hi[j][1], hi[j][2], hi[j][3]};
                    if (has_res) {
                        const u32x4 r4 = res[t & 1][j];
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            v[2 * e] += widen<ODT>((uint16_t)(r4[e] & 0xFFFFu));
                            v[2 * e + 1] += widen<ODT>((uint16_t)(r4[e] >> 16));
                        }
                    }
                    const u32x4 w = {cvt_pack2<ODT>(actf(v[0]), actf(v[1])), cvt_pack2<ODT>(actf(v[2]), actf(v[3])),
                                     cvt_pack2<ODT>(actf(v[4]), actf(v[5])), cvt_pack2<ODT>(actf(v[6]), actf(v[7]))};
                    __builtin_amdgcn_raw_buffer_store_b128(w, ry, (int)out_off(rp, t, j), 0, 0);
                }
            }
        };
        if (p.act == SS_ACT_GELU) write_out([](float v) { return gelu_erfc(v); });
        else write_out([&](float v) { return floor_at(v, relu_floor); });
    }
}

// Can the activation-stationary kernel take this problem?  16-bit operands, 1x1 kernel, a reduction of 64, 96, 128, 256
// or 512 channels, 16-byte output runs, output below 2 GiB (32-bit store offsets, out-of-range mark above every real
// one; the pixel tail relies on the buffer's range check).
static inline bool rows_eligible(const ss_weight_desc *desc, const ConvParams &p)
{
    const int K = desc->cin;
    return !is_byte_type(desc->dtype) && desc->kh == 1 && desc->kw == 1 && (K == 64 || K == 96 || K == 128 || K == 256 || K == 512) &&
           desc->cout % 8 == 0 && p.nsplit <= 1 && (long long)(p.P + 64) * p.Cout * 2 < (1ll << 31) - (1ll << 27);
}

// Output-channel blocks of 64 per workgroup.  Measured on MI355X: the best number of workgroups per pixel tile is the
// one that gives every compute unit about two workgroups (one for the 512-channel reduction, whose LDS tile leaves
// room for one), rounded to the nearest, in multiples of four blocks (one per wave).  forced > 0 (test hook): that
// many workgroups per pixel tile.
static inline int rows_pairs_per_group(const ConvParams &p, int ncu, int forced)
{
    const int pairs_all = ((p.Cout + 31) / 32 + 1) / 2;
    const long long tiles_n = ((long long)p.P + 63) / 64;
    const long long target = (p.K >= 512 ? 1ll : 2ll) * ncu;
    long long mg = forced > 0 ? forced : (target + tiles_n / 2) / tiles_n;
    if (mg < 1) mg = 1;
    long long ppg = (pairs_all + mg - 1) / mg;
    ppg = (ppg + 3) / 4 * 4;
    if (ppg > pairs_all) ppg = pairs_all;
    return (int)ppg;
}

template <int DT, bool SPARSE, int KS>
static int launch_rows_ks(const ConvParams &p, int ncu, hipStream_t s)
{
    const int ppg = rows_pairs_per_group(p, ncu, forced_split());
    const int pairs_all = ((p.Cout + 31) / 32 + 1) / 2;
    const int mg = (pairs_all + ppg - 1) / ppg;
    const long long tiles_n = ((long long)p.P + 63) / 64;
    const long long blocks = tiles_n * mg;
    if (blocks <= 0 || blocks > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    const size_t smem = rows_smem_bytes<KS>(ppg);
    if (smem > 160 * 1024) return SS_ERR_UNSUPPORTED;
    auto kern = conv_pw_rows_kernel<DT, SPARSE, KS>;
    if (smem > 64 * 1024) {
        // (raised to the most this kernel can ask for, once per device)
        static std::atomic<unsigned long long> done_mask{0};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return SS_ERR_HIP;
        const unsigned long long bit = 1ull << (dev & 63);
        if (dev >= 64 || !(done_mask.load(std::memory_order_acquire) & bit)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
                return SS_ERR_HIP;
            if (dev < 64) done_mask.fetch_or(bit, std::memory_order_release);
        }
    }
    kern<<<dim3((unsigned)blocks), dim3(256), smem, s>>>(p, mg, ppg);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

template <int DT, bool SPARSE>
static int launch_rows(const ss_weight_desc *desc, const ConvParams &p, int ncu, hipStream_t s)
{
    switch (desc->cin) {
        case 64: return launch_rows_ks<DT, SPARSE, 2>(p, ncu, s);
        case 96: return launch_rows_ks<DT, SPARSE, 3>(p, ncu, s);
        case 128: return launch_rows_ks<DT, SPARSE, 4>(p, ncu, s);
        case 256: return launch_rows_ks<DT, SPARSE, 8>(p, ncu, s);
        case 512: return launch_rows_ks<DT, SPARSE, 16>(p, ncu, s);
        default: return SS_ERR_UNSUPPORTED;
    }
}

}  // namespace ss

#endif
