// Dense 7x7 stride-2 convolution on an image of 3 or 4 channels: the first layer of a ResNet, which the method leaves
// dense (Sec. 4 "Architectures": its reduction length 3*7*7 = 147 is no multiple of 4; Sec. 3.3 suggests padding the
// image to four channels).  Same contraction as ss_conv_kernel.h (Sec. 3.3 Eq. 5: Y~ = W U(X)), other data movement:
//
//   * The general kernels build the unfolded input from global memory element by element (2-byte or 8-byte loads per
//     2:4 block), 49 loads per input pixel.  Here a workgroup loads the input patch of a 16 x 16 output tile once
//     (37 x 38 pixels, coalesced), parks it in LDS as 8-byte pixels (a three-channel pixel gets a zero fourth
//     channel), and every activation fragment of the matrix instruction is one aligned 16-byte LDS read.
//   * For that the reduction runs in the kernel's own order k' = (r * 8 + t) * 4 + c (kernel row, tap padded from 7
//     to 8, channel padded to 4): the 8 consecutive k' a lane feeds to one 32x32x16 instruction are two neighbouring
//     pixels of one patch row.  The weights are brought into that order once per workgroup, gathered from the dense
//     tile buffer (whatever flattening it was packed in) into LDS and from there into registers, where they stay: the
//     workgroups are resident and walk over the output tiles.  The padded tap and channel carry zero weights; the
//     activations under the padded tap (real pixels that belong to the neighbouring window) are cleared in the
//     fragment, so that a non-finite pixel outside a window cannot reach it through 0 x inf.
//   * Four waves per workgroup; a wave owns all 64 output channels of 4 x 16 output pixels (two 32-pixel column
//     tiles of two rows each), i.e. four independent accumulator tiles per reduction step.  Output tiles leave
//     through a wave-private LDS slab as 128-byte pixel rows (16-byte stores, 1 KiB contiguous per instruction).
//   * The next tile's patch is fetched into registers before the current tile is multiplied.
// Arithmetic: fp32 accumulation starting from the bias, activation, one rounding to nearest even -- as everywhere.
#ifndef SS_CONV_IMAGE_H_
#define SS_CONV_IMAGE_H_
#include "ss_conv_stream.h"

namespace ss {

struct ImageShape {
    static constexpr int KH = 7, KW = 7, S = 2;
    static constexpr int TH = 16, TW = 16;                      // output tile of a workgroup
    static constexpr int PH = (TH - 1) * S + KH;                // 37 patch rows
    static constexpr int PW = (TW - 1) * S + 8;                 // 38 patch columns (taps padded to 8)
    static constexpr int PITCH = 40;                            // pixels per patch row in LDS, 8 bytes each
    static constexpr int NPIX = PH * PW;                        // 1406
    static constexpr int NLOAD = (NPIX + 255) / 256;            // patch pixels per thread
    static constexpr int STEPS = 2 * KH;                        // reduction steps of 16: (kernel row, half of the 8 taps)
    static constexpr int SLAB_ROW = 64 + 8;                     // 16-bit units per pixel row of a wave's output slab
    static constexpr int A_ELEMS = STEPS * 2 * 64 * 8;          // weights of 64 output channels in fragment order
    static constexpr size_t patch_bytes = (size_t)PH * PITCH * 8;
    static constexpr size_t slab_bytes = (size_t)4 * 32 * SLAB_ROW * 2;
    static constexpr size_t a_bytes = (size_t)A_ELEMS * 2;
    static constexpr int KS_MAX = 7;                            // reduction steps of 32 in the weight buffer: K = 49 cin <= 224
    static constexpr int RAW_VECS = 2 * KS_MAX * 128;           // 16-byte vectors of two row tiles' dense tiles
    static constexpr size_t raw_bytes = (size_t)RAW_VECS * 16;
    // at set-up: fragment-ordered weights, then the raw tiles; afterwards: patch, then the slabs
    static constexpr size_t body = a_bytes + raw_bytes > patch_bytes + slab_bytes ? a_bytes + raw_bytes : patch_bytes + slab_bytes;
    static constexpr size_t smem = body + 64 * 4;               // + the bias of the 64 channels
};

template <int DT, int CIN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void conv_image_kernel(ConvParams p, int tiles_h, int tiles_w, int ntiles)
{
    using SH = ImageShape;
    static_assert(CIN == 3 || CIN == 4, "three or four channels");
    static_assert(SH::patch_bytes % 16 == 0 && SH::A_ELEMS % 256 == 0 && SH::RAW_VECS % 256 == 0, "layout");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    unsigned char *const patch = smem_raw;
    uint16_t *const slab_all = reinterpret_cast<uint16_t *>(smem_raw + SH::patch_bytes);
    float *const bias_s = reinterpret_cast<float *>(smem_raw + SH::body);
    unsigned char *const raw_s = smem_raw + SH::a_bytes;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5;                         // half of the wave: which 8 of a step's 16 reduction indices
    const int m0 = blockIdx.y * 64;                  // first output channel of this workgroup
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, (int)p.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a_vals), 0, (int)p.a_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)((unsigned)p.P * (unsigned)p.Cout * 2u), kRsrcFlags);

    // ---- weights: dense tile buffer -> LDS in fragment order [step][row tile][lane][8] -> registers
    // Element e = ((step * 2 + tm) * 64 + l) * 8 + s is the weight of output channel m0 + 32 tm + l % 32 at kernel
    // row step / 2, tap 4 (step % 2) + 2 (l / 32) + s / 4, channel s % 4; in the buffer it sits at reduction index k
    // of the declared flattening: tile ((mt * Ks + k / 32) * 2 + (k % 16) / 8), lane 32 ((k % 32) / 16) + row % 32,
    // slot k % 8, i.e. at byte  mt Ks 2048 + (row % 32) 16 + [k / 32] 2048 + [k bit 3] 1024 + [k bit 4] 512 + (k % 8) 2.
    // Thread tid moves the elements e = tid + 256 i: slot and row are its own, step, row tile and wave half follow
    // from i at compile time, so k is a per-thread term plus a per-i constant.  The tiles are first copied to LDS
    // with wide loads: fetching the elements one by one from global memory (7 million scattered 2-byte loads over
    // the grid) took a tenth of the whole kernel.
    auto gather_weights = [&]() {
        // (1) the two row tiles' dense tiles, as they are, into LDS: contiguous in the buffer, 16-byte loads
        const unsigned tile_stride = (unsigned)p.Ks * 2048u;
        const unsigned first = (unsigned)(m0 >> 5) * tile_stride;
        u32x4 raw[SH::RAW_VECS / 256];
#pragma unroll
        for (int i = 0; i < SH::RAW_VECS / 256; i++) {
            const unsigned v = (unsigned)(tid + 256 * i) * 16u;
            raw[i] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)(v < 2u * tile_stride ? first + v : kOutOfRange), 0, 0);
        }
#pragma unroll
        for (int i = 0; i < SH::RAW_VECS / 256; i++) *reinterpret_cast<u32x4 *>(raw_s + (size_t)(tid + 256 * i) * 16) = raw[i];
        __syncthreads();
        // (2) from there into fragment order
        constexpr int PER = SH::A_ELEMS / 256;
        const bool crs = p.korder == SS_K_CRS;
        const int s = tid & 7, ts = s >> 2, c = s & 3, row = (tid >> 3) & 31;
        const int k_thread = crs ? c * (SH::KH * SH::KW) + ts : ts * CIN + c;
        const unsigned row_off = (unsigned)row * 16u;
        uint16_t val[PER];
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int ge = i & 1, tm = (i >> 1) & 1, step = i >> 2, r = step >> 1, h = step & 1;
            const int t0 = 4 * h + 2 * ge;           // first of the two taps this wave half holds at this step
            const int k = k_thread + (crs ? SH::KW * r + t0 : (SH::KW * r + t0) * CIN);
            const bool valid = (t0 + 1 < SH::KW || ts == 0) && c < CIN;       // (rows past the last channel are zero in the tiles)
            const unsigned off = (unsigned)tm * tile_stride + row_off + (((unsigned)k >> 5) << 11) + (((unsigned)k & 8u) << 7) +
                                 (((unsigned)k & 16u) << 5) + (((unsigned)k & 7u) << 1);
            const uint16_t w = *reinterpret_cast<const uint16_t *>(raw_s + (valid ? off : 0u));
            val[i] = valid ? w : (uint16_t)0;
        }
        // (all reads before the first write: the compiler keeps LDS reads and writes to one array in program order, and
        // element by element every write would wait for its read's full latency)
#pragma unroll
        for (int i = 0; i < PER; i++) reinterpret_cast<uint16_t *>(smem_raw)[tid + 256 * i] = val[i];
    };

    // ---- patch staging
    // A tile index past the last one loads nothing (every offset out of range), so the loop below can prefetch
    // unconditionally.  The loaded words are kept as they arrive and only put together when they are written to LDS:
    // any arithmetic on them right after the loads would make the wave wait for them before it multiplies.
    const int per_image = tiles_h * tiles_w;
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    uint32_t stage_a[SH::NLOAD];
    uint32_t stage_b[CIN == 4 ? SH::NLOAD : 1];     // four channels: second dword of a pixel
    s16x2 stage_h[CIN == 3 ? (SH::NLOAD + 1) / 2 : 1];      // three channels: the pixels' odd halfwords, two per register
    auto load_patch = [&](int t) {
        const int n = t / per_image, rem = t - n * per_image;
        const int th = rem / tiles_w, tw = rem - th * tiles_w;
        const int ih0 = th * (SH::TH * SH::S) - p.ph, iw0 = tw * (SH::TW * SH::S) - p.pw;
        const bool live = t < ntiles;
#pragma unroll
        for (int i = 0; i < SH::NLOAD; i++) {
            const int idx = tid + 256 * i;
            const int pr = idx / SH::PW, pc = idx - pr * SH::PW;
            const int ih = ih0 + pr, iw = iw0 + pc;
            const bool inb = live && idx < SH::NPIX && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            const unsigned pix = (unsigned)((n * p.H + ih) * p.W + iw);
            if constexpr (CIN == 4) {
                const uint2 v = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(inb ? pix * 8u : kOutOfRange), 0, 0));
                stage_a[i] = v.x;
                stage_b[i] = v.y;
            } else {
                // six bytes at offset 6 pix: a dword on its 4-byte boundary and the remaining halfword
                const unsigned byte = pix * 6u;
                const bool odd = pix & 1u;
                stage_a[i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rx, (int)(inb ? (odd ? byte + 2u : byte) : kOutOfRange), 0, 0);
                stage_h[i >> 1][i & 1] = __builtin_amdgcn_raw_buffer_load_b16(rx, (int)(inb ? (odd ? byte : byte + 4u) : kOutOfRange), 0, 0);
            }
        }
    };
    auto store_patch = [&](int t) {                  // t: the tile the staged words belong to
        const int n = t / per_image, rem = t - n * per_image;
        const int th = rem / tiles_w, tw = rem - th * tiles_w;
        const int ih0 = th * (SH::TH * SH::S) - p.ph, iw0 = tw * (SH::TW * SH::S) - p.pw;
#pragma unroll
        for (int i = 0; i < SH::NLOAD; i++) {
            const int idx = tid + 256 * i;
            const int pr = idx / SH::PW, pc = idx - pr * SH::PW;
            uint2 v;
            if constexpr (CIN == 4) v = make_uint2(stage_a[i], stage_b[i]);
            if constexpr (CIN == 3) {
                const uint32_t d = stage_a[i], w = (uint16_t)stage_h[i >> 1][i & 1];
                v = make_uint2(d, w);
                const unsigned pix = (unsigned)((n * p.H + ih0 + pr) * p.W + iw0 + pc);      // as in load_patch: its parity chose the loads
                if (pix & 1u) v = make_uint2(w | (d << 16), d >> 16);
            }
            // (threads past the patch's last pixel write to an unused pad column instead of skipping the store: a branch
            // here would leave their loads "possibly pending" for the compiler, which then waits for everything,
            // the previous tile's output stores included, at the top of the next tile)
            const int slot = idx < SH::NPIX ? pr * SH::PITCH + pc : SH::PW;
            *reinterpret_cast<uint2 *>(patch + (size_t)slot * 8) = v;
        }
    };

    // ---- per-lane constants of the multiply phase
    // Lane (n = lane % 32, g) of column tile c reads, at step (r, h), the two pixels at patch row 2 ho_l + r, column
    // 2 wo_l + 4 h + 2 g, with ho_l = 4 wave + 2 c + n / 16, wo_l = n % 16.
    const int n32 = lane & 31;
    const unsigned char *const bbase = patch + (size_t)(((4 * wave + (n32 >> 4)) * 2) * SH::PITCH + (n32 & 15) * 2 + 2 * g) * 8;
    // taps 4 h + 2 g + {0, 1} that lie past the kernel's width: only h = 1, g = 1, second pixel for a 7-wide kernel
    const uint32_t keep_hi = (4 + 2 * g + 1 < SH::KW) ? 0xFFFFFFFFu : 0u;
    // Output slab of a wave: 32 pixel rows of 128 + 16 bytes, so that every address below is one per-lane base plus a
    // compile-time offset (an XOR swizzle would remove the slab's two-way bank conflicts, but costs twelve more
    // address registers than this kernel has: the reload of a spilled one makes the wave wait for all its stores).
    uint16_t *const slab = slab_all + wave * 32 * SH::SLAB_ROW;
    const float relu_floor = p.act == SS_ACT_RELU ? 0.f : -__builtin_inff();

    // The wait for a prefetched patch sits at the end of the loop body, where the instructions issued since the
    // prefetch are the same on every path: at the head of the loop the compiler has to assume the fewest (none, on
    // entry) and the wait for the patch would also wait for most of the previous tile's output stores.
    int t = blockIdx.x;                              // < ntiles: the grid is no larger than the number of tiles
    load_patch(t);                                   // on its way while the weights are brought in
    // (the bias too: fetched after the weights it would cost a memory round trip of its own)
    const float bias_v = (tid < 64 && p.bias != nullptr && m0 + tid < p.Cout) ? p.bias[m0 + tid] : 0.f;
    __builtin_amdgcn_sched_barrier(0);
    gather_weights();
    if (tid < 64) bias_s[tid] = bias_v;
    __syncthreads();
    u32x4 A[SH::STEPS][2];
#pragma unroll
    for (int st = 0; st < SH::STEPS; st++)
#pragma unroll
        for (int tm = 0; tm < 2; tm++)
            A[st][tm] = *reinterpret_cast<const u32x4 *>(smem_raw + (size_t)((st * 2 + tm) * 64 + lane) * 16);
    __syncthreads();                                 // the fragment area becomes patch and slabs

    store_patch(t);
    lds_barrier();                                   // the first patch is in LDS
    for (;;) {
        const int tnext = t + gridDim.x;
        load_patch(tnext);                           // in flight while this tile is multiplied
        __builtin_amdgcn_sched_barrier(0);           // (the scheduler would sink the loads into the multiply phase)

        const int n = t / per_image, rem = t - n * per_image;
        const int th = rem / tiles_w, tw = rem - th * tiles_w;
        const int ho0 = th * SH::TH + 4 * wave, wo0 = tw * SH::TW;

        f32x16 acc[2][2];                            // [row tile][column tile]
#pragma unroll
        for (int tm = 0; tm < 2; tm++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const f32x4 b4 = *reinterpret_cast<const f32x4 *>(bias_s + 32 * tm + 8 * j + 4 * g);
#pragma unroll
                for (int c = 0; c < 2; c++)
#pragma unroll
                    for (int e = 0; e < 4; e++) acc[tm][c][4 * j + e] = b4[e];
            }
#pragma unroll
        for (int st = 0; st < SH::STEPS; st++) {
            const int r = st >> 1, h = st & 1;
#pragma unroll
            for (int c = 0; c < 2; c++) {
                u32x4 b = *reinterpret_cast<const u32x4 *>(bbase + (size_t)((4 * c + r) * SH::PITCH + 4 * h) * 8);
                if (h == 1) {
                    b[2] &= keep_hi;
                    b[3] &= keep_hi;
                }
#pragma unroll
                for (int tm = 0; tm < 2; tm++) acc[tm][c] = mma_dense<DT>(A[st][tm], b, acc[tm][c]);
            }
        }

        // ---- epilogue: activation, one rounding, slab, 16-byte stores
        // (A wave's LDS operations execute in order: a piece's reads see its writes, and the next piece may be written
        // as soon as this one's reads are issued -- its conversion and writes then cover the slab's read latency.)
        auto write_out = [&](auto actf) {
            auto put = [&](int c) {
#pragma unroll
                for (int tm = 0; tm < 2; tm++)
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        float rr[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) rr[e] = actf(acc[tm][c][4 * j + e]);
                        *reinterpret_cast<uint2 *>(slab + n32 * SH::SLAB_ROW + 32 * tm + 8 * j + 4 * g) =
                            make_uint2(cvt_pack2<DT>(rr[0], rr[1]), cvt_pack2<DT>(rr[2], rr[3]));
                    }
            };
            put(0);
#pragma unroll
            for (int c = 0; c < 2; c++) {
                u32x4 w[4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int q = lane + 64 * i, px = q >> 3, run = q & 7;
                    w[i] = *reinterpret_cast<const u32x4 *>(slab + px * SH::SLAB_ROW + run * 8);
                }
                if (c == 0) put(1);
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int q = lane + 64 * i, px = q >> 3, run = q & 7;
                    const int ho = ho0 + 2 * c + (px >> 4), wo = wo0 + (px & 15), o = m0 + run * 8;
                    const bool ok = ho < p.Ho && wo < p.Wo && o < p.Cout;
                    const unsigned off = ((unsigned)((n * p.Ho + ho) * p.Wo + wo) * (unsigned)p.Cout + (unsigned)o) * 2u;
                    __builtin_amdgcn_raw_buffer_store_b128(w[i], ry, (int)(ok ? off : kOutOfRange), 0, 0);
                }
            }
        };
        if (p.act == SS_ACT_GELU) write_out([](float v) { return gelu_erfc(v); });
        else write_out([&](float v) { return floor_at(v, relu_floor); });      // ReLU, or the identity with a floor of -inf (a NaN passes)
        lds_barrier();                               // every wave is done with the patch
        if (tnext >= ntiles) break;
        store_patch(tnext);
        lds_barrier();                               // the next patch is in LDS
        t = tnext;
    }
}

// Can the image kernel take this problem?  Dense 16-bit 7x7 kernel with stride 2 on three or four channels, 16-byte
// output runs, no residual, output below 2 GiB (32-bit store offsets, out-of-range mark above every real one).
static inline bool image_eligible(const ss_weight_desc *desc, const ConvParams &p)
{
    return !is_byte_type(desc->dtype) && desc->kh == 7 && desc->kw == 7 && (desc->cin == 3 || desc->cin == 4) && p.sh == 2 &&
           p.sw == 2 && desc->cout % 8 == 0 && p.residual == nullptr && p.nsplit <= 1 &&
           (long long)p.P * p.Cout * 2 < (1ll << 31) - (1ll << 27);
}

// Launches the image kernel on a resident grid: at most two workgroups per compute unit (their register budget),
// each walking over output tiles of 16 x 16 pixels x 64 channels.
template <int DT>
static int launch_image(const ss_weight_desc *desc, const ConvParams &p, int ncu, hipStream_t s)
{
    using SH = ImageShape;
    static_assert(SH::smem <= 64 * 1024, "fits the default dynamic LDS limit");
    const long long tiles_h = (p.Ho + SH::TH - 1) / SH::TH, tiles_w = (p.Wo + SH::TW - 1) / SH::TW;
    const long long ntiles = (long long)p.N * tiles_h * tiles_w;
    const int groups = (p.Cout + 63) / 64;
    if (ntiles <= 0 || ntiles > 0x7FFF0000ll || groups > 0xFFFF) return SS_ERR_UNSUPPORTED;      // (the kernel adds the grid size to a tile index)
    long long gx = 2ll * ncu / groups;
    if (gx < 1) gx = 1;
    if (gx > ntiles) gx = ntiles;
    const dim3 grid((unsigned)gx, (unsigned)groups);
    if (desc->cin == 3)
        conv_image_kernel<DT, 3><<<grid, dim3(256), SH::smem, s>>>(p, (int)tiles_h, (int)tiles_w, (int)ntiles);
    else
        conv_image_kernel<DT, 4><<<grid, dim3(256), SH::smem, s>>>(p, (int)tiles_h, (int)tiles_w, (int)ntiles);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

}  // namespace ss

#endif
