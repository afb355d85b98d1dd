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
//   of 4 consecutive output channels of one pixel.
//   The dense twin issues two 32x32x16 dense MFMAs on the same B registers instead.
//
// 8-bit operands (int8, FP8 E4M3) run through the same kernel: activations are staged as 2-byte units (pairs of
// channels), one 32x32x64 instruction then consumes the same 32 B of B and 16 B of A per lane as the 16-bit one
// and does twice the multiply-adds; sums are int32 (exact) or fp32, and the tail multiplies by a per-channel scale.
//
// All global reads of activations and weights are raw buffer loads: a lane whose element lies in
// the zero padding, past the last pixel or past the reduction length presents an offset beyond the
// buffer's size and the hardware returns 0 -- no branches, no selects.
//
// This header holds the kernel templates and their launch / tile-choice code.  It is included by one translation
// unit per (operand type, sparse | dense) pair, each of which instantiates its share (ss_conv_inst.h), so that the
// library's build runs in parallel.
#ifndef SS_CONV_KERNEL_H_
#define SS_CONV_KERNEL_H_
#include "ss_internal.h"
#include "ss_conv_params.h"
#include <atomic>
#include <type_traits>

namespace ss {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

// Accumulators of one 32x32 tile: fp32 for the floats (16-bit and FP8), int32 (exact) for 8-bit integers.
template <int DT> using Acc = typename std::conditional<DT == SS_I8, i32x16, f32x16>::type;
// Type of the 16-bit output (and of a residual): the operands' own, or binary16 for 8-bit operands.
template <int DT> constexpr int out_type() { return is_byte_type(DT) ? SS_F16 : DT; }

struct B32 {   // one lane's B fragment for a reduction step: 32 bytes (16 x 16-bit, or 32 x int8)
    u32x4 lo, hi;
};


// floor(n / d) by multiply + shift with the host-computed constants of fast_div_setup.
__device__ __forceinline__ int fast_div(int n, unsigned mul, unsigned sh)
{
    return (int)(((unsigned long long)(unsigned)n * mul) >> sh);
}

constexpr unsigned kOutOfRange = 0x80000000u;   // >= any buffer size used here: the load returns 0
constexpr int kRsrcFlags = 0x00020000;          // raw buffer, 32-bit data format (gfx9 family)

// The 8-bit instructions (32x32x64, integer and FP8 alike) pair slot s of A lane l (16 kept bytes, index field s of a full index
// word) with bytes 16*(l/32) + 4*((s%8)/2) + idx of the B lane of the same column in lane group s/8; B lane
// l holds the 32 reduction indices 32*(l/32) + [0,32) of pixel l%32.  Accumulators are laid out as above.
template <int DT>
__device__ __forceinline__ Acc<DT> mma_sparse(u32x4 a, const B32 &b, Acc<DT> c, uint32_t idx)
{
    if constexpr (DT == SS_I8)
        return __builtin_amdgcn_smfmac_i32_32x32x64_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x8, b), c, (int)idx, 0, 0);
    else if constexpr (DT == SS_F8)
        return __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x8, b), c, (int)idx, 0, 0);
    else if constexpr (DT == SS_F16)
        return __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x16, b), c,
                                                         (int)idx, 0, 0);
    else
        return __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x16, b), c,
                                                          (int)idx, 0, 0);
}

// Which dense FP8 kernels use the 32x32x64 instruction (the others use pairs of 32x32x16, see mma_dense): the deep
// ones, which have the registers for its 8-register operands, and the short-chunk channels-last staging, whose shallow
// kernels are otherwise bound by the half-rate instruction (measured: 81 vs 69 us on the N=500 benchmark layer).
constexpr bool f8_wide(bool deep, int mode) { return deep || mode == 0 /* MODE_VEC */; }

// Dense FP8: one 32x32x64 instruction of the scaled-format family with both formats E4M3 and both block scales
// 2^0 (exponent byte 127); A and B slots s of lane l are k = 32*(l/32) + s.
__device__ __forceinline__ f32x16 mma_dense_f8(u32x4 a0, u32x4 a1, const B32 &b, f32x16 c)
{
    const i32x8 a = __builtin_shufflevector(__builtin_bit_cast(i32x4, a0), __builtin_bit_cast(i32x4, a1), 0, 1, 2, 3, 4, 5, 6, 7);
    const i32x8 bb = __builtin_shufflevector(__builtin_bit_cast(i32x4, b.lo), __builtin_bit_cast(i32x4, b.hi), 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, bb, c, 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
}

template <int DT>
__device__ __forceinline__ Acc<DT> mma_dense(u32x4 a, u32x4 b, Acc<DT> c)
{
    if constexpr (DT == SS_I8)      // 32x32x32: A lane l slot s <-> k = 16*(l/32) + s, B likewise
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    else if constexpr (DT == SS_F8) {
        // Two 32x32x16 FP8 instructions on the low and high 8 bytes (A and B share the lane -> reduction-index map,
        // and the weight tile was laid out for these very bytes of B).  Half the rate of the 32x32x64 form, but its
        // operands are register pairs: used by the shallow kernels, which need the occupancy more than the rate.
        const unsigned long long a0 = a[0] | ((unsigned long long)a[1] << 32), a1 = a[2] | ((unsigned long long)a[3] << 32);
        const unsigned long long b0 = b[0] | ((unsigned long long)b[1] << 32), b1 = b[2] | ((unsigned long long)b[3] << 32);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8((long)a0, (long)b0, c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8((long)a1, (long)b1, c, 0, 0, 0);
    } else if constexpr (DT == SS_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Two fp32 values to one dword of 16-bit floats, round to nearest even, in one instruction (V_CVT_PK_F16_F32 /
// V_CVT_PK_BF16_F32).
template <int DT>
__device__ __forceinline__ uint32_t cvt_pack2(float a, float b)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {a, b};
    if constexpr (DT == SS_F16)
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    else
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// max(v, floor) that hands a NaN through (the IEEE 754-2019 maximum, one V_MAXIMUM3_F32): ReLU with floor = 0, the
// identity with floor = -inf.  (A sum of exactly -0 comes out as +0.)
__device__ __forceinline__ float floor_at(float v, float floor)
{
    return __builtin_elementwise_maximum(v, floor);
}

// Exact value of a 16-bit pattern as fp32.
template <int DT>
__device__ __forceinline__ float widen(uint16_t bits)
{
    if constexpr (DT == SS_F16)
        return (float)__builtin_bit_cast(_Float16, bits);
    else
        return __builtin_bit_cast(float, (uint32_t)bits << 16);
}

// GELU z * Phi(z) with the exact standard normal CDF Phi(z) = erfc(-z / sqrt 2) / 2.  erfc by the rational
// approximation 7.1.26 of Abramowitz & Stegun (erfc(x) = t (a1 + t (a2 + ... a5 t)) exp(-x^2), t = 1 / (1 + p x),
// x >= 0; absolute error below 1.5e-7, i.e. at fp32 round-off and three orders below the 16-bit output's), which
// costs a third of the library erfc in an epilogue that otherwise only adds and rounds.  With h = Phi(-|z|):
//     z >= 0:  z (1 - h) = z - |z| h        z < 0:  z h = -|z| h        i.e.  gelu(z) = max(z, 0) - |z| h,
// which keeps the lower tail's relative accuracy (no 1 - erf cancellation) and needs no select.  The constants carry
// the 1/sqrt 2 of the argument and the 1/2 of Phi; exp(-z^2 / 2) is one exp2.  (A NaN stays a NaN.)
__device__ __forceinline__ float gelu_erfc(float z)
{
    const float a = fabsf(z);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f * 0.70710678118654752f, a, 1.0f));
    const float poly = t * (0.5f * 0.254829592f + t * (0.5f * -0.284496736f + t * (0.5f * 1.421413741f +
                       t * (0.5f * -1.453152027f + t * (0.5f * 1.061405429f)))));
    const float e = __builtin_amdgcn_exp2f(a * a * (-0.5f * 1.44269504088896341f));      // exp(-z^2 / 2)
    return __builtin_fmaf(-a, poly * e, fmaxf(z, 0.f));
}

// How the [pixels x reduction-chunk] slice of the unfolded input is built in LDS:
//   MODE_VEC    channels are contiguous inside every aligned run of 8 reduction indices (1x1
//               kernels, or the channels-last flattening, with cin % 8 == 0): 16-byte loads,
//               chunks of 64 reduction indices.
//   MODE_VEC8   the same with chunks of 256 reduction indices, for long reductions: a quarter of the barriers.
//   MODE_PW     MODE_VEC specialised for 1x1 kernels: a pixel's offset is fixed for the whole
//               reduction and the chunk's channel offset travels in the load's scalar offset.
//               Chunks of 128 reduction indices (MODE_PW) or 64 (MODE_PW2, for very short reductions).
//   MODE_GATHER any flattening / shape: one 16-bit load per element (slow, general fallback).
//   MODE_GATHER4 channels-last flattening with cin % 4 == 0 (e.g. an image padded from 3 to 4 channels, the
//               column-wise augmentation Sec. 3.3 suggests for reductions that are no multiple of 4): every
//               aligned run of 4 reduction indices is 8 contiguous, 8-byte aligned bytes of one pixel: one 8-byte
//               load per 2:4 block.
//   MODE_TAPS   the paper's flattening (channel slowest) with a KH x KW kernel and cin % 32 == 0:
//               a 2:4 block then holds 4 consecutive (channel, tap) pairs, i.e. activations of
//               different pixels.  A thread loads, for one output pixel and 8 channels, the
//               KH*KW taps as 16-byte channel vectors and transposes them in registers to
//               channel-major order before the LDS write, so the MFMA side still reads 16-byte
//               vectors.  A chunk is 32 channels = KH*KW reduction steps.  (8-bit operands: 16 channels per
//               vector, a byte transpose, chunks of 64 channels.)
enum { MODE_VEC = 0, MODE_GATHER = 1, MODE_TAPS = 2, MODE_PW = 3, MODE_PW2 = 4, MODE_VEC8 = 5, MODE_GATHER4 = 6 };
constexpr bool is_vec(int mode) { return mode == MODE_VEC || mode == MODE_VEC8; }

// Weight fragments of one 32-wide reduction step for the TM row tiles of a wave.
template <bool SPARSE, int TM>
struct AStep {
    u32x4 v[SPARSE ? 1 : 2][TM];
    uint32_t idx[TM];
};

template <int MODE, int KH, int KW, bool DEEP>
struct ChunkShape {
    static constexpr int TAPS = KH * KW;
    static constexpr int KSTEPS = (MODE == MODE_TAPS) ? TAPS : (MODE == MODE_VEC8 ? 8 : (MODE == MODE_PW ? 4 : 2));   // 32-wide reduction steps per LDS chunk
    static constexpr int BK = KSTEPS * 32;
    // Bank-conflict-free layout of a pixel row in LDS.  Default: +16 bytes per row, so that the 16-byte fragment reads
    // of consecutive pixels hit distinct banks.  The 3x3 tap-transposing mode writes 16-byte vectors at a stride of 9
    // vectors (one 8-channel unit) from four threads per pixel, which collides with any such padding; there the row
    // is left unpadded (36 vectors) and the index of a 16-byte vector inside its row is XOR-ed with bits 2..3 of the
    // pixel row (SWZ): the vector stays inside its aligned group of four, and both the transposed writes (4 pixel
    // rows x 4 units per 16 lanes) and the fragment reads (16 consecutive pixel rows) cover all 64 banks exactly once.
    // Only in the deep variants: the swizzled addresses cost the shallow 128 x 64 kernel eight registers, which is the
    // step from four to three waves per SIMD (its fused form ran 35 -> 49 us with it); the deep variants run at one to
    // three waves per SIMD anyway.
    static constexpr bool SWZ = MODE == MODE_TAPS && TAPS == 9 && DEEP;
    static constexpr int ROW = SWZ ? BK : BK + 8;
    // LDS copies of the chunk: double-buffered, so that the next chunk is written while this one is
    // multiplied -- except for the large unfolded 3x3 chunk in the shallow variant, which is kept once
    // (more workgroups per compute unit then hide the store phase instead).
    static constexpr int NBUF = (MODE == MODE_TAPS && TAPS > 4 && !DEEP) ? 1 : 2;
};

constexpr int ring_size(int ksteps, int regs_per_step, int budget)
{
    int depth = budget / regs_per_step + 1;
    if (depth > 12) depth = 12;
    if (depth < 2) depth = 2;
    int best = 1;
    for (int r = 2; r <= depth; r++)
        if (ksteps % r == 0 || r % ksteps == 0) best = r;
    if (best >= 2) return best;
    for (int r = depth + 1;; r++)                    // nothing that shallow nests with the chunk: take the next that does
        if (ksteps % r == 0 || r % ksteps == 0) return r;
}

// LDS of a workgroup: the staging buffers, reused by the epilogue for the output tile (16-bit, or fp32 when a
// residual is added after it), followed by the tile's bias values (fp32).
// Fused second contraction: every wave owns a staging region of 32 pixels x (32 + 4) floats behind the 16-bit tile.
constexpr int kFuseRow = 32 + 4;
constexpr size_t kFuseRegion = 32 * kFuseRow * 4;

template <int BM, int BN, int MODE, int KH, int KW, bool DEEP>
constexpr size_t smem_body(bool with_residual, int fuse_waves = 0)
{
    using CS = ChunkShape<MODE, KH, KW, DEEP>;
    size_t stage = (size_t)CS::NBUF * BN * CS::ROW * 2;
    size_t epi = with_residual ? (size_t)BN * (BM + 4) * 4 : (size_t)BN * (BM * 2 + 8) + (size_t)fuse_waves * kFuseRegion;
    return stage > epi ? stage : epi;
}
template <int BM, int BN, int MODE, int KH, int KW, bool DEEP>
constexpr size_t smem_bytes(bool with_residual, int fuse_waves = 0)
{
    return smem_body<BM, BN, MODE, KH, KW, DEEP>(with_residual, fuse_waves) + (size_t)BM * 4;
}

// Waves per SIMD the register allocator must leave room for: small wave tiles are latency-bound
// and profit from 4 resident waves (128 VGPRs each); large ones need the registers.
constexpr int min_waves_per_simd(int tm, int tn, bool big_stage)
{
    return tm * tn <= 2 ? (big_stage ? 3 : 4) : (tm * tn <= 4 ? 2 : 1);   // the 3x3 transpose needs ~134 VGPRs: 4 waves would spill
}

// DEEP: for grids of at most about one workgroup per compute unit, where no other wave hides
// latency: weight fragments are prefetched 8+ steps ahead and activation fragments 3 steps ahead
// (instead of 1), at the price of registers, i.e. of the occupancy such a grid cannot use anyway.
// SPEC: four extra waves do nothing but build the activation chunks in LDS (loads two chunks ahead,
// transposes, LDS writes); the WAVES_M x WAVES_N waves only fetch weights, read LDS and multiply.
// A wave issues in order, so without this split every wait of the staging code also stalls the
// wave's matrix instructions.
// FUSE: the tile (all output channels of this convolution for BN pixels, bias and activation applied, rounded to
// 16 bit exactly as it would be stored) stays in LDS and is at once the activation operand of a following 1x1
// convolution, whose output (+ bias + residual, activation) is what the kernel writes: the 3x3 -> 1x1 expansion of a
// bottleneck without the intermediate tensor's round trip through memory.
template <int DT, bool SPARSE, int WAVES_M, int WAVES_N, int TM, int TN, int MODE, int KH, int KW, bool DEEP, bool SPEC, bool FUSE = false>
__global__ __launch_bounds__((WAVES_M * WAVES_N + (SPEC ? 4 : 0)) * 64)
__attribute__((amdgpu_waves_per_eu(DEEP ? 1 : (((DT == SS_F8 || FUSE) && !SPARSE && MODE == MODE_VEC && TM * TN == 2) ? 3 : min_waves_per_simd(TM, TN, MODE == MODE_TAPS || MODE == MODE_VEC8)))))
void conv_kernel(ConvParams p)
{
    using CS = ChunkShape<MODE, KH, KW, DEEP>;
    static_assert(!SPEC || DEEP, "producer waves come with the deep variant only");
    constexpr bool Q8 = is_byte_type(DT);                 // 8-bit operands: staged as byte pairs, full index words, scaled tail
    constexpr int ODT = out_type<DT>();
    static_assert(!Q8 || (MODE != MODE_GATHER && MODE != MODE_GATHER4), "8-bit operands travel in 16-byte runs only");
    constexpr int NMATH = WAVES_M * WAVES_N * 64;         // threads that multiply
    constexpr int NT = NMATH + (SPEC ? 256 : 0);
    constexpr int BM = WAVES_M * TM * 32;
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int TAPS = CS::TAPS;
    constexpr int KSTEPS = CS::KSTEPS;
    // Weight fragments are prefetched RING-1 reduction steps ahead into a register ring, as deep as
    // about 24 (48 when DEEP) VGPRs allow (deeper rings cost occupancy, which the bandwidth-bound layers need more); RING divides the chunk or is a multiple of it (then the chunk loop is
    // unrolled RING/KSTEPS times so that every ring slot is a compile-time register).
    constexpr int RING = ring_size(KSTEPS, TM * (SPARSE ? 5 : 8), SPEC ? 96 : (DEEP ? 48 : 24));
    constexpr int BD = DEEP ? 4 : 2;                      // activation-fragment ring depth
    constexpr int PF = RING - 1;
    constexpr int UNROLL = RING > KSTEPS ? RING / KSTEPS : 1;
    static_assert(KSTEPS % RING == 0 || RING % KSTEPS == 0, "ring and chunk must nest");
    constexpr int BK = CS::BK;
    constexpr int ROW = CS::ROW;
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *Bs0 = smem;
    constexpr int NBUF = CS::NBUF;
    uint16_t *Bs1 = smem + (NBUF - 1) * BN * ROW;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = SPEC && wave >= NMATH / 64;     // wave-uniform
    const int wm = wave % WAVES_M;               // (producer waves: unused)
    const int wn = (wave / WAVES_M) % WAVES_N;
    // Workgroups are handed to the 8 XCDs round-robin, and each XCD has its own L2.  Renumber them so
    // that an XCD works on a contiguous run of tiles: both row tiles of a pixel tile, and pixel tiles
    // that share halo rows, then hit the same L2.
    const int nb = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int lidx = xcd * (nb >> 3) + min(xcd, nb & 7) + slot;
    // Split reduction (p.nsplit > 1): nsplit workgroups share an output tile and each takes a contiguous share of the
    // reduction chunks; their fp32 partial sums meet in the workspace (see the epilogue).
    constexpr bool CAN_SPLIT = !FUSE && !is_byte_type(DT);
    const int nsplit = CAN_SPLIT ? p.nsplit : 1;
    // (split-major numbering: neighbouring workgroups, which land on the same XCD, work on neighbouring tiles with the
    // same share of the reduction and so share that share's weights in their L2)
    const int ntiles = nsplit > 1 ? nb / nsplit : nb;
    const int split = nsplit > 1 ? lidx / ntiles : 0;
    const int lid = nsplit > 1 ? lidx - split * ntiles : lidx;
    const int nchunks_all = (p.Ks + ChunkShape<MODE, KH, KW, DEEP>::KSTEPS - 1) / ChunkShape<MODE, KH, KW, DEEP>::KSTEPS;
    const int c_first = split * nchunks_all / nsplit;                  // this workgroup's chunks: [c_first, c_first + nchunks)
    const int nchunks = (split + 1) * nchunks_all / nsplit - c_first;
    const int tile_n = fast_div(lid, p.tm_mul, p.tm_sh);
    const int tile_m = lid - tile_n * p.tiles_m;
    const int m0 = tile_m * BM;
    const int n0 = tile_n * BN;
    const int HoWo = p.Ho * p.Wo;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, (int)p.x_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a_vals), 0, (int)p.a_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.a_meta), 0, (int)p.meta_bytes, kRsrcFlags);

    // The tile's bias values are fetched now and parked in LDS after the first staging store, so the
    // epilogue does not pay a global-memory round trip.
    static_assert(!FUSE || !Q8, "the fused second contraction is built for the 16-bit types");
    const bool with_res = !Q8 && !FUSE && p.residual != nullptr;     // uniform (fused: the residual belongs to the second layer)
    float *bias_s = reinterpret_cast<float *>(reinterpret_cast<char *>(smem) +
                                              (with_res ? smem_body<BM, BN, MODE, KH, KW, DEEP>(true)
                                                        : smem_body<BM, BN, MODE, KH, KW, DEEP>(false, FUSE ? NT / 64 : 0)));
    // (Loaded after the first activation / weight loads are on their way: issued first, its latency would
    // sit in front of everything else.)
    float *scale_s = bias_s + BM;                     // (8-bit operands only)
    float bias_r[(BM + NMATH - 1) / NMATH], scale_r[Q8 ? (BM + NMATH - 1) / NMATH : 1];
    auto load_bias = [&]() {
#pragma unroll
        for (int j = 0; j < (BM + NMATH - 1) / NMATH; j++) {
            const int o = m0 + tid + j * NMATH;
            const bool in = tid + j * NMATH < BM && o < p.Cout;
            bias_r[j] = (p.bias != nullptr && in) ? p.bias[o] : 0.f;
            if constexpr (Q8) scale_r[j] = (p.scale != nullptr && in) ? p.scale[o] : 1.f;
        }
    };

    // ------------------------------------------------------------------ activation staging state
    // per pixel row and chunk: 16-byte runs (VEC: 8, TAPS: 4 channel octets) or 4-element blocks (GATHER: 16)
    constexpr int UNITS = (MODE == MODE_GATHER || MODE == MODE_GATHER4) ? 16 : (MODE == MODE_TAPS ? 4 : (MODE == MODE_VEC8 ? 32 : (MODE == MODE_PW ? 16 : 8)));
    constexpr int ST = SPEC ? (256 < BN * UNITS ? 256 : BN * UNITS) : (NT < BN * UNITS ? NT : BN * UNITS);     // staging threads (whole waves); the rest only multiply
    constexpr int ITEMS = BN * UNITS / ST;
    constexpr int NSET = SPEC ? 2 : 1;                    // producer waves hold two chunks in registers
    static_assert(BN * UNITS % ST == 0 && ST % UNITS == 0 && ST % 64 == 0 && ITEMS >= 1, "tile/threads mismatch");
    const int stid = SPEC ? tid - NMATH : tid;            // index among the staging threads
    static_assert(!SPEC || ST == 256, "every producer thread stages");
    const bool stager = SPEC ? true : ((ST == NT) || tid < ST);     // (producer waves: only they call the staging code)
    // Thread -> (pixel row, unit): unit fastest, so consecutive lanes read consecutive 16-byte pieces of one
    // pixel (coalesced).  (Putting 16 pixel rows of one unit on consecutive lanes makes the transposed LDS
    // writes conflict-free but quadruples the cache lines per load instruction: measured 30-40 % slower.)
    const int unit = (stid & 0xFFFF) % UNITS;
    const int pr0 = ((stid & 0xFFFF) % ST) / UNITS;
    unsigned pixbyte[ITEMS];          // byte offset of x[n, ho*sh-ph, wo*sw-pw, 0] (wraps below 0 for padded pixels)
    int ih0[ITEMS], iw0[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; i++) {
        int pr = pr0 + i * (ST / UNITS);
        int pg = n0 + pr;
        if (pg < p.P) {
            int n = fast_div(pg, p.howo_mul, p.howo_sh);
            int rem = pg - n * HoWo;
            int ho = fast_div(rem, p.wo_mul, p.wo_sh);
            int wo = rem - ho * p.Wo;
            ih0[i] = ho * p.sh - p.ph;
            iw0[i] = wo * p.sw - p.pw;
            pixbyte[i] = (unsigned)(((n * p.H + ih0[i]) * p.W + iw0[i]) * p.Cin * 2);
        } else {
            ih0[i] = -(1 << 28);     // every bounds test fails -> zeros
            iw0[i] = -(1 << 28);
            pixbyte[i] = 0;
        }
    }

    // MODE_VEC: position of this thread's 8-element run in the (tap, channel) space
    int vk = unit * 8 + c_first * ChunkShape<MODE, KH, KW, DEEP>::BK, vc = 0, vr = 0, vt = 0;
    if constexpr (is_vec(MODE)) {
        int tap = vk / p.Cin;
        vc = vk - tap * p.Cin;
        vr = tap / p.kw;
        vt = tap - vr * p.kw;
    }
    // MODE_TAPS: per (pixel, tap) byte offsets, fixed for the whole reduction; the chunk's channel
    // offset travels in the scalar offset of the load.  Out-of-image taps are out of range for good.
    unsigned tapoff[MODE == MODE_TAPS ? ITEMS : 1][MODE == MODE_TAPS ? TAPS : 1];
    if constexpr (MODE == MODE_TAPS) {
#pragma unroll
        for (int i = 0; i < ITEMS; i++)
#pragma unroll
            for (int tap = 0; tap < TAPS; tap++) {
                const int r = tap / KW, t = tap % KW;
                int ih = ih0[i] + r, iw = iw0[i] + t;
                bool ok = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                tapoff[i][tap] = ok ? pixbyte[i] + (unsigned)(((r * p.W + t) * p.Cin + unit * 8) * 2) : kOutOfRange;
            }
    }

    // MODE_PW: per pixel byte offset of this thread's 16-byte run in the first chunk (out of range for pixels
    // past the end or in the padding)
    unsigned pwoff[(MODE == MODE_PW || MODE == MODE_PW2) ? ITEMS : 1];
    if constexpr (MODE == MODE_PW || MODE == MODE_PW2) {
#pragma unroll
        for (int i = 0; i < ITEMS; i++) {
            bool ok = (unsigned)ih0[i] < (unsigned)p.H && (unsigned)iw0[i] < (unsigned)p.W;
            pwoff[i] = ok ? pixbyte[i] + (unsigned)(unit * 16) : kOutOfRange;
        }
    }

    u32x4 stage_v_[NSET][(is_vec(MODE) || MODE == MODE_PW || MODE == MODE_PW2) ? ITEMS : 1];
    uint16_t stage_g_[NSET][MODE == MODE_GATHER ? ITEMS : 1][4];
    uint2 stage_g4_[NSET][MODE == MODE_GATHER4 ? ITEMS : 1];
    u32x4 stage_t_[NSET][MODE == MODE_TAPS ? ITEMS : 1][MODE == MODE_TAPS ? TAPS : 1];

    auto stage_load = [&](int ci_rel, int set = 0) {      // set: compile time at every call site; chunk relative to c_first
        if (!stager) return;
        const int ci = ci_rel + c_first;
        auto &stage_v = stage_v_[set];
        auto &stage_g = stage_g_[set];
        auto &stage_t = stage_t_[set];
        if constexpr (is_vec(MODE)) {
            const unsigned koff = vk < p.K ? (unsigned)(((vr * p.W + vt) * p.Cin + vc) * 2) : kOutOfRange;
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
                int ih = ih0[i] + vr, iw = iw0[i] + vt;
                bool ok = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W && koff != kOutOfRange;
                unsigned off = ok ? pixbyte[i] + koff : kOutOfRange;
                stage_v[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0);
            }
            vk += BK;
            vc += BK;
            while (vc >= p.Cin) {
                vc -= p.Cin;
                if (++vt == p.kw) { vt = 0; ++vr; }
            }
        } else if constexpr (MODE == MODE_PW || MODE == MODE_PW2) {
            const bool kok = ci * BK + unit * 8 < p.K;      // the last chunk may reach past the reduction length
#pragma unroll
            for (int i = 0; i < ITEMS; i++)
                stage_v[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(kok ? pwoff[i] : kOutOfRange), ci * (BK * 2), 0);
        } else if constexpr (MODE == MODE_GATHER4) {
            // this thread's block of 4 reduction indices: one tap, 4 consecutive channels
            auto &stage_g4 = stage_g4_[set];
            const int k0 = ci * BK + unit * 4;
            const int tap = fast_div(k0, p.cin_mul, p.cin_sh);
            const int c = k0 - tap * p.Cin;
            const int r = fast_div(tap, p.kw_mul, p.kw_sh);
            const int t = tap - r * p.kw;
            const unsigned koff = k0 < p.K ? (unsigned)(((r * p.W + t) * p.Cin + c) * 2) : kOutOfRange;
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
                int ih = ih0[i] + r, iw = iw0[i] + t;
                bool ok = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W && koff != kOutOfRange;
                stage_g4[i] = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(ok ? pixbyte[i] + koff : kOutOfRange), 0, 0));
            }
        } else if constexpr (MODE == MODE_GATHER) {
            unsigned off[4];
            int er[4], et[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                int k = ci * BK + unit * 4 + e;
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
                er[e] = k < p.K ? r : (1 << 29);      // past the reduction length: fails the bounds test
                et[e] = t;
                off[e] = (unsigned)(((r * p.W + t) * p.Cin + c) * 2);
            }
#pragma unroll
            for (int i = 0; i < ITEMS; i++) {
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    int ih = ih0[i] + er[e], iw = iw0[i] + et[e];
                    bool ok = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    unsigned o = ok ? pixbyte[i] + off[e] : kOutOfRange;
                    stage_g[i][e] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, (int)o, 0, 0);
                }
            }
        } else {
            const int soff = ci * 64;                   // 32 channels per chunk
#pragma unroll
            for (int i = 0; i < ITEMS; i++)
#pragma unroll
                for (int tap = 0; tap < TAPS; tap++)
                    stage_t[i][tap] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)tapoff[i][tap], soff, 0);
        }
    };
    // Writes slice j of n of the staged chunk to LDS (j, n are compile-time at every call site): a share of the
    // transposed 16-byte vectors (tap mode) or of the items (other modes).  stage_store = all of it.
    auto stage_store_slice = [&](uint16_t *Bs, int j, int n, int set = 0) {
        if (!stager) return;
        auto &stage_v = stage_v_[set];
        auto &stage_g = stage_g_[set];
        auto &stage_t = stage_t_[set];
#pragma unroll
        for (int i = 0; i < ITEMS; i++) {
            int pr = pr0 + i * (ST / UNITS);
            if constexpr (MODE == MODE_TAPS) {
                // [tap][8 channels] -> [channel][tap]: output element h = c*TAPS + tap, two per dword, four dwords per vector
                u32x4 *rowp = reinterpret_cast<u32x4 *>(Bs + pr * ROW);
                const int vec0 = unit * TAPS, swz = CS::SWZ ? (pr >> 2) & 3 : 0;     // first vector of the unit; the row's XOR key
#pragma unroll
                for (int v = 0; v < TAPS; v++) {
                    if (v < j * TAPS / n || v >= (j + 1) * TAPS / n) continue;
                    uint32_t o[4];
                    if constexpr (Q8) {
                        // bytes: [tap][16 channels] -> [channel][tap]; output byte h = c*TAPS + tap, four per dword, each
                        // from its own tap's vector: two byte pairs are picked first, then joined
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            const int d = 4 * v + q;
                            uint32_t src[4], pick[4];
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                const int h = 4 * d + e, c = h / TAPS, t = h % TAPS;
                                src[e] = stage_t[i][t][c >> 2];
                                pick[e] = (uint32_t)(c & 3);
                            }
                            const uint32_t p01 = __builtin_amdgcn_perm(src[1], src[0], pick[0] | ((4u + pick[1]) << 8));
                            const uint32_t p23 = __builtin_amdgcn_perm(src[3], src[2], pick[2] | ((4u + pick[3]) << 8));
                            o[q] = __builtin_amdgcn_perm(p23, p01, 0x05040100u);
                        }
                        u32x4 w = {o[0], o[1], o[2], o[3]};
                        rowp[(vec0 + v) ^ swz] = w;
                        continue;
                    }
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int d = 4 * v + q;
                        const int ha = 2 * d, hb = 2 * d + 1;
                        const int ca = ha / TAPS, ta = ha % TAPS, cb = hb / TAPS, tb = hb % TAPS;
                        uint32_t sa = stage_t[i][ta][ca >> 1];
                        uint32_t sb = stage_t[i][tb][cb >> 1];
                        const uint32_t sel = (uint32_t)(2 * (ca & 1)) | ((uint32_t)(2 * (ca & 1) + 1) << 8) |
                                             ((uint32_t)(4 + 2 * (cb & 1)) << 16) | ((uint32_t)(5 + 2 * (cb & 1)) << 24);
                        o[q] = __builtin_amdgcn_perm(sb, sa, sel);
                    }
                    u32x4 w = {o[0], o[1], o[2], o[3]};
                    rowp[(vec0 + v) ^ swz] = w;
                }
            } else {
                if (i < j * ITEMS / n || i >= (j + 1) * ITEMS / n) continue;
                if constexpr (MODE == MODE_GATHER4) {
                    *reinterpret_cast<uint2 *>(Bs + pr * ROW + unit * 4) = stage_g4_[set][i];
                } else if constexpr (MODE == MODE_GATHER) {
                    uint2 v = make_uint2((uint32_t)stage_g[i][0] | ((uint32_t)stage_g[i][1] << 16),
                                         (uint32_t)stage_g[i][2] | ((uint32_t)stage_g[i][3] << 16));
                    *reinterpret_cast<uint2 *>(Bs + pr * ROW + unit * 4) = v;
                } else {
                    *reinterpret_cast<u32x4 *>(Bs + pr * ROW + unit * 8) = stage_v[i];
                }
            }
        }
    };
    auto stage_store = [&](uint16_t *Bs, int set = 0) { stage_store_slice(Bs, 0, 1, set); };

    // ------------------------------------------------------------------ weight fragments
    // Row tiles past the last one are clamped to it (their rows are never stored); reduction steps
    // past the last one are clamped too: they only ever meet all-zero activations.
    unsigned a_voff[TM], m_voff[TM];
#pragma unroll
    for (int tm = 0; tm < TM; tm++) {
        int mt = min((m0 >> 5) + wm * TM + tm, p.Mt - 1);
        a_voff[tm] = (unsigned)((mt * p.Ks * (SPARSE ? 1 : 2)) * 64 + lane) * 16u;
        m_voff[tm] = (unsigned)(mt * p.Kp * 64 + lane) * 4u;
    }
    const int ks_first = c_first * KSTEPS;
    auto load_a = [&](AStep<SPARSE, TM> &a, int ks_rel) {       // step relative to this workgroup's first
        const int ks = min(ks_rel + ks_first, p.Ks - 1);
#pragma unroll
        for (int tm = 0; tm < TM; tm++) {
            if constexpr (SPARSE) {
                a.v[0][tm] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_voff[tm], ks * 1024, 0);
                // The index word of the step pair; the step's half is shifted down where it is used, steps later (a
                // shift here would have to wait for the load it follows and stall the wave at every step).
                a.idx[tm] = __builtin_amdgcn_raw_buffer_load_b32(rm, (int)m_voff[tm], (Q8 ? ks : (ks >> 1)) * 256, 0);
            } else {
                a.v[0][tm] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_voff[tm], ks * 2048, 0);
                a.v[1][tm] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)a_voff[tm], ks * 2048 + 1024, 0);
            }
        }
    };

    // This lane's two 16-byte vectors of a fragment inside the step's aligned group of four (in 16-bit units): lanes
    // 0..31 take vectors 0, 1 and lanes 32..63 vectors 2, 3, XOR-ed with the pixel row's key in the swizzled layout.
    const int frag_key = CS::SWZ ? (lane >> 2) & 3 : 0;
    const int frag_lo = ((2 * (lane >> 5)) ^ frag_key) * 8, frag_hi = ((2 * (lane >> 5) + 1) ^ frag_key) * 8;

    Acc<DT> acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; tm++)
#pragma unroll
        for (int tn = 0; tn < TN; tn++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[tm][tn][v] = 0;

    // ------------------------------------------------------------------ main loop (double-buffered LDS, ring of weight steps)
    AStep<SPARSE, TM> a[RING];
    if constexpr (SPEC) {
        if (producer) {
            // ---- producer waves: chunk ci+1 is written to LDS while the others multiply chunk ci; its loads were
            // issued one chunk earlier.  One barrier per chunk, exactly as in the multiplying waves' loop below.
            // The steady-state loop issues its loads unconditionally: behind a condition, the compiler's wait before
            // the LDS writes must also cover the path without new loads, and so waits for the new loads as well
            // (a full memory latency per chunk).
            stage_load(0, 0);
            stage_store(Bs0, 0);
            if (nchunks > 1) stage_load(1, 1);
            __syncthreads();
            // the last two chunks: nothing left to load (set, buf: where chunk ci + 1 waits and where it goes)
            auto tail = [&](int ci, int set, uint16_t *buf) {
                if (ci + 1 < nchunks) {
                    stage_store(buf, set);
                    __syncthreads();
                    ci++;
                }
                if (ci < nchunks) __syncthreads();
            };
            for (int ci = 0;;) {
                if (ci + 2 >= nchunks) { tail(ci, 1, Bs1); break; }
                stage_load(ci + 2, 0);                      // set 0 held chunk ci, which is in LDS already
                stage_store(Bs1, 1);
                __syncthreads();
                ci++;
                if (ci + 2 >= nchunks) { tail(ci, 0, Bs0); break; }
                stage_load(ci + 2, 1);
                stage_store(Bs0, 0);
                __syncthreads();
                ci++;
            }
        }
    }
    if (!producer) {
    // With producer waves in the workgroup the multiplying waves set the pace (the producers wait for them at every
    // chunk's barrier): they get the issue slots first (measured 2-4 % on the 3x3 256 -> 256 layer at batch 32).
    if constexpr (SPEC) __builtin_amdgcn_s_setprio(3);
    if constexpr (!SPEC) stage_load(0);
    // (Issue order pinned: the loop's waits count loads in flight, and the compiler takes the weaker of the counts
    // that hold on entry and around the back edge; values and index words must interleave here as they do there.)
#pragma unroll
    for (int s = 0; s < PF; s++) {
        load_a(a[s], s);
        __builtin_amdgcn_sched_barrier(0);
    }
    load_bias();
    if constexpr (!SPEC) stage_store(Bs0);
#pragma unroll
    for (int j = 0; j < (BM + NMATH - 1) / NMATH; j++)
        if (tid + j * NMATH < BM) {
            bias_s[tid + j * NMATH] = bias_r[j];
            if constexpr (Q8) scale_s[tid + j * NMATH] = scale_r[j];
        }
    __syncthreads();
    for (int c0 = 0; c0 < nchunks; c0 += UNROLL) {
#pragma unroll
        for (int u = 0; u < UNROLL; u++) {
            const int ci = c0 + u;
            if (ci >= nchunks) break;                       // uniform
            const uint16_t *cur = (ci & 1) ? Bs1 : Bs0;
            uint16_t *nxt = (ci & 1) ? Bs0 : Bs1;
            const bool more = ci + 1 < nchunks;
            if constexpr (!SPEC)
                if (more) stage_load(ci + 1);
            __builtin_amdgcn_sched_barrier(0);
            B32 b[BD][TN];
            auto load_b = [&](B32 (&bf)[TN], int s) {
#pragma unroll
                for (int tn = 0; tn < TN; tn++) {
                    const uint16_t *src = cur + ((wn * TN + tn) * 32 + (lane & 31)) * ROW + s * 32;
                    bf[tn].lo = *reinterpret_cast<const u32x4 *>(src + frag_lo);
                    bf[tn].hi = *reinterpret_cast<const u32x4 *>(src + frag_hi);
                }
            };
#pragma unroll
            for (int s = 0; s < BD - 1 && s < KSTEPS; s++) load_b(b[s], s);
#pragma unroll
            for (int s = 0; s < KSTEPS; s++) {
                const int g = u * KSTEPS + s;               // position in the ring (compile time)
                load_a(a[(g + PF) % RING], ci * KSTEPS + s + PF);
                if (s + BD - 1 < KSTEPS) load_b(b[(s + BD - 1) % BD], s + BD - 1);   // later steps' activations while this step multiplies
                if constexpr (NBUF == 2 && !SPEC) {          // the next chunk's share of transposes / LDS writes rides along with the later steps
                    constexpr int S0 = KSTEPS / 2;
                    if (more && s >= S0) stage_store_slice(nxt, s - S0, KSTEPS - S0);
                }
                // (steps past the reduction length multiply clamped weights with all-zero activations:
                // cheaper than a branch, which would force copies of every accumulator)
                const AStep<SPARSE, TM> &as = a[g % RING];
                // the 16-bit instruction reads index bits [15:0]; the 8-bit one the whole word
                const int idx_shift = Q8 ? 0 : (min(ks_first + ci * KSTEPS + s, p.Ks - 1) & 1) * 16;
#pragma unroll
                for (int tm = 0; tm < TM; tm++)
#pragma unroll
                    for (int tn = 0; tn < TN; tn++) {
                        if constexpr (SPARSE) {
                            acc[tm][tn] = mma_sparse<DT>(as.v[0][tm], b[s % BD][tn], acc[tm][tn], as.idx[tm] >> idx_shift);
                        } else if constexpr (DT == SS_F8 && f8_wide(DEEP, MODE)) {
                            acc[tm][tn] = mma_dense_f8(as.v[0][tm], as.v[1][tm], b[s % BD][tn], acc[tm][tn]);
                        } else {
                            acc[tm][tn] = mma_dense<DT>(as.v[0][tm], b[s % BD][tn].lo, acc[tm][tn]);
                            acc[tm][tn] = mma_dense<DT>(as.v[1][tm], b[s % BD][tn].hi, acc[tm][tn]);
                        }
                    }
                // Scheduling: left alone, the compiler sinks every load to just before its first use and the
                // prefetch distance collapses to zero.  Pin this step's instructions to the step (barriers at both
                // ends) and interleave the loads for later steps between its matrix instructions.
                constexpr int NMMA = TM * TN * (SPARSE ? 1 : (DT == SS_F8 ? (f8_wide(DEEP, MODE) ? 1 : 4) : 2));
                constexpr int DSR = (2 * TN + NMMA - 1) / NMMA;
                constexpr int VMR = (TM * 2 + NMMA - 1) / NMMA;
#pragma unroll
                for (int i = 0; i < NMMA; i++) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, DSR, 0);    // LDS reads
                    __builtin_amdgcn_sched_group_barrier(0x020, VMR, 0);    // global reads
                    __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);      // transposes of the next chunk (when this step has any)
                    __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);      // and their LDS writes
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (NBUF == 1) {
                __syncthreads();                            // everyone is done reading the only copy
                if (more) stage_store(nxt);
            }
            __syncthreads();
        }
    }
    }   // !producer

    // ------------------------------------------------------------------ epilogue
    // bias (+ residual) + activation in fp32, one rounding to the 16-bit type; the tile goes through LDS so that
    // every pixel's run of BM output channels leaves as 16-byte, fully coalesced NHWC stores.
    constexpr int RUNS = BM / 8;                  // 16-byte runs per pixel row
    const bool vec_ok = (p.Cout & 7) == 0;
    // The thread index again, from the wave number (scalar) and the lane count: keeping the launch-time register
    // alive across the main loop costs a spill in the variants that run at the register limit.
    const int etid = wave * 64 + (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const float relu_floor = p.act == SS_ACT_RELU ? 0.f : -__builtin_inff();
    // ReLU when relu_floor = 0, identity when -inf (a NaN passes through); GELU = z * Phi(z) with the exact normal
    // CDF, written with erfc so that the lower tail keeps its relative accuracy
    auto relu_or_id = [&](float v) { return floor_at(v, relu_floor); };
    auto gelu = [](float v) { return gelu_erfc(v); };
    if constexpr (CAN_SPLIT) {
        if (nsplit > 1) {
            // Every workgroup of the tile leaves its partial sums in the workspace, in register order (one 16-byte
            // vector per thread and accumulator quad: fully coalesced), and takes a ticket.  The last one to arrive adds
            // the partials in the order of the splits -- so the result does not depend on who arrived last --, hands the
            // ticket counter back at zero for the next launch, and runs the usual tail; the others are done.
            // The workgroups of a tile may run on different XCDs, whose L2 caches are not coherent with each other.  The
            // partial sums are therefore stored and loaded with the device-scope cache policy (sc1: written through to,
            // and read from, the level all XCDs share -- what a relaxed device-scope atomic store / load compiles to),
            // every wave waits for the acknowledgement of its stores before the workgroup takes its ticket, and the
            // ticket is a device-scope atomic.  Device-scope fences would do as well, but they write back (release) and
            // invalidate (acquire) the XCD's whole L2 under the workgroups still in their main loops: measured at
            // 3 us per doubling of the split with the release fence alone, 4-8 us per workgroup with both.
            constexpr int kDeviceScope = 16;            // cache-policy bit sc1 of the buffer instructions
            const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(p.ws_part + (size_t)lid * nsplit * (BM * BN), 0,
                                                                               nsplit * (BM * BN) * 4, kRsrcFlags);
            const int mtid = etid;                      // (multiplying threads are 0 .. NMATH-1)
            if (!producer) {
#pragma unroll
                for (int tm = 0; tm < TM; tm++)
#pragma unroll
                    for (int tn = 0; tn < TN; tn++)
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            const f32x4 fw = {(float)acc[tm][tn][4 * q + 0], (float)acc[tm][tn][4 * q + 1], (float)acc[tm][tn][4 * q + 2], (float)acc[tm][tn][4 * q + 3]};
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, fw), rp, (((tm * TN + tn) * 4 + q) * NMATH + mtid) * 16, split * (BM * BN * 4), kDeviceScope);
                        }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's partial sums have been acknowledged
            __syncthreads();
            unsigned *ticket_s = reinterpret_cast<unsigned *>(smem);      // (the staging buffers are free)
            if (etid == 0) *ticket_s = __hip_atomic_fetch_add(p.ws_ctr + lid, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const unsigned ticket = *ticket_s;
            if (ticket != (unsigned)(nsplit - 1)) return;                 // (uniform)
            if (etid == 0) __hip_atomic_store(p.ws_ctr + lid, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (!producer) {
#pragma unroll
                for (int tm = 0; tm < TM; tm++)
#pragma unroll
                    for (int tn = 0; tn < TN; tn++)
#pragma unroll
                        for (int v = 0; v < 16; v++) acc[tm][tn][v] = 0.f;
                for (int j = 0; j < nsplit; j++) {
#pragma unroll
                    for (int tm = 0; tm < TM; tm++)
#pragma unroll
                        for (int tn = 0; tn < TN; tn++)
#pragma unroll
                            for (int q = 0; q < 4; q++) {
                                // (the whole vector is reinterpreted at once: a bit cast of a single vector element reads element 0)
                                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rp, (((tm * TN + tn) * 4 + q) * NMATH + mtid) * 16, j * (BM * BN * 4), kDeviceScope));
                                acc[tm][tn][4 * q + 0] += v[0]; acc[tm][tn][4 * q + 1] += v[1];
                                acc[tm][tn][4 * q + 2] += v[2]; acc[tm][tn][4 * q + 3] += v[3];
                            }
                }
            }
            __syncthreads();                            // the ticket word's LDS is about to hold the output tile
        }
    }
    if (!with_res) {
        constexpr int CROW = BM + 4;     // halfs per pixel row in LDS (+8 bytes: the 8-byte writes of 32 consecutive pixels spread over all banks)
        uint16_t *Cs = smem;             // the staging buffers are free: the loop ended with a barrier (every wave, producers included, ran the same number)
        auto to_lds = [&](auto actf) {
#pragma unroll
            for (int tm = 0; tm < TM; tm++) {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int ol = (wm * TM + tm) * 32 + 8 * q + 4 * (lane >> 5);    // first of 4 consecutive output channels (tile-local)
                    const float4 bq = *reinterpret_cast<const float4 *>(bias_s + ol);
                    const float bv[4] = {bq.x, bq.y, bq.z, bq.w};
                    float sv[4] = {1.f, 1.f, 1.f, 1.f};
                    if constexpr (Q8) {
                        const float4 sq = *reinterpret_cast<const float4 *>(scale_s + ol);
                        sv[0] = sq.x; sv[1] = sq.y; sv[2] = sq.z; sv[3] = sq.w;
                    }
#pragma unroll
                    for (int tn = 0; tn < TN; tn++) {
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            if constexpr (Q8) r[e] = actf((float)acc[tm][tn][4 * q + e] * sv[e] + bv[e]);
                            else r[e] = actf(acc[tm][tn][4 * q + e] + bv[e]);
                        }
                        const int pl = (wn * TN + tn) * 32 + (lane & 31);
                        *reinterpret_cast<uint2 *>(Cs + pl * CROW + ol) = make_uint2(cvt_pack2<ODT>(r[0], r[1]), cvt_pack2<ODT>(r[2], r[3]));
                    }
                }
            }
        };
        if (!producer) {
            if (p.act == SS_ACT_GELU) to_lds(gelu); else to_lds(relu_or_id);
        }
        __syncthreads();
        if constexpr (FUSE) {
            // ---- second contraction: y2[pixel, o2] = act2( sum_c A2[o2, c] * tile[pixel, c] + bias2[o2] + residual[pixel, o2] )
            // Every wave (producers included) takes row tiles of 32 output channels in turn; its weights and bias for
            // the next row tile are fetched while the current one is multiplied.  The fp32 result of 32 pixels x 32
            // channels crosses the wave's own LDS region so that residual loads and stores are 16-byte runs.
            constexpr int NW = NT / 64;
            constexpr int KS2 = BM / 32;                  // upper bound of the second reduction's steps (its length is this convolution's cout)
            constexpr int TN2 = BN / 32;
            float *reg = reinterpret_cast<float *>(reinterpret_cast<char *>(smem) + (size_t)BN * (BM * 2 + 8)) + wave * (32 * kFuseRow);
            const __amdgpu_buffer_rsrc_t ra2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a2_vals), 0, (int)p.a2_bytes, kRsrcFlags);
            const __amdgpu_buffer_rsrc_t rm2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.a2_meta), 0, (int)p.meta2_bytes, kRsrcFlags);
            const int lane2 = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
            const int g2 = lane2 >> 5, c2 = lane2 & 31;
            const float floor2 = p.act2 == SS_ACT_RELU ? 0.f : -__builtin_inff();
            struct Row2 {
                u32x4 v[SPARSE ? 1 : 2][KS2];
                uint32_t idx[KS2];
                float4 b[4];
            };
            auto load_row = [&](Row2 &r, int mt) {
#pragma unroll
                for (int s2 = 0; s2 < KS2; s2++) {
                    if (s2 >= p.Ks2) break;               // uniform
                    if constexpr (SPARSE) {
                        r.v[0][s2] = __builtin_amdgcn_raw_buffer_load_b128(ra2, (int)(((unsigned)(mt * p.Ks2 + s2) * 64 + lane2) * 16u), 0, 0);
                        r.idx[s2] = __builtin_amdgcn_raw_buffer_load_b32(rm2, (int)(((unsigned)(mt * p.Kp2 + (s2 >> 1)) * 64 + lane2) * 4u), 0, 0);
                    } else {
                        const unsigned off = ((unsigned)(mt * p.Ks2 + s2) * 128 + lane2) * 16u;
                        r.v[0][s2] = __builtin_amdgcn_raw_buffer_load_b128(ra2, (int)off, 0, 0);
                        r.v[1][s2] = __builtin_amdgcn_raw_buffer_load_b128(ra2, (int)off, 1024, 0);
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; q++)
                    r.b[q] = p.bias2 ? *reinterpret_cast<const float4 *>(p.bias2 + mt * 32 + 8 * q + 4 * g2) : make_float4(0.f, 0.f, 0.f, 0.f);
            };
            Row2 cur, nxt;
            if (wave < p.Mt2) load_row(cur, wave);
            for (int mt = wave; mt < p.Mt2; mt += NW) {
                if (mt + NW < p.Mt2) load_row(nxt, mt + NW);
#pragma unroll
                for (int tn = 0; tn < TN2; tn++) {
                    f32x16 acc2;
#pragma unroll
                    for (int v = 0; v < 16; v++) acc2[v] = 0.f;
#pragma unroll
                    for (int s2 = 0; s2 < KS2; s2++) {
                        if (s2 >= p.Ks2) break;           // uniform
                        const uint16_t *src = Cs + (tn * 32 + c2) * CROW + 32 * s2 + 16 * g2;     // 8-byte aligned
                        const uint2 u0 = *reinterpret_cast<const uint2 *>(src), u1 = *reinterpret_cast<const uint2 *>(src + 4);
                        const uint2 u2 = *reinterpret_cast<const uint2 *>(src + 8), u3 = *reinterpret_cast<const uint2 *>(src + 12);
                        B32 bf;
                        bf.lo = u32x4{u0.x, u0.y, u1.x, u1.y};
                        bf.hi = u32x4{u2.x, u2.y, u3.x, u3.y};
                        if constexpr (SPARSE) {
                            acc2 = mma_sparse<DT>(cur.v[0][s2], bf, acc2, cur.idx[s2] >> ((s2 & 1) * 16));
                        } else {
                            acc2 = mma_dense<DT>(cur.v[0][s2], bf.lo, acc2);
                            acc2 = mma_dense<DT>(cur.v[1][s2], bf.hi, acc2);
                        }
                    }
#pragma unroll
                    for (int q = 0; q < 4; q++)
                        *reinterpret_cast<float4 *>(reg + c2 * kFuseRow + 8 * q + 4 * g2) =
                            make_float4(acc2[4 * q + 0] + cur.b[q].x, acc2[4 * q + 1] + cur.b[q].y, acc2[4 * q + 2] + cur.b[q].z, acc2[4 * q + 3] + cur.b[q].w);
                    // (a wave's LDS operations execute in order: the reads below see the writes above)
#pragma unroll
                    for (int j = 0; j < 2; j++) {
                        const int it = lane2 + 64 * j;
                        const int px = it >> 2, run = it & 3;
                        const int pg = n0 + tn * 32 + px, o = mt * 32 + run * 8;
                        const float4 lo = *reinterpret_cast<const float4 *>(reg + px * kFuseRow + run * 8);
                        const float4 hi = *reinterpret_cast<const float4 *>(reg + px * kFuseRow + run * 8 + 4);
                        if (pg >= p.P) continue;
                        float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                        if (p.res2 != nullptr) {
                            const u32x4 rr = *reinterpret_cast<const u32x4 *>(p.res2 + (size_t)pg * p.Cout2 + o);
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                v[2 * e] += widen<ODT>((uint16_t)(rr[e] & 0xFFFFu));
                                v[2 * e + 1] += widen<ODT>((uint16_t)(rr[e] >> 16));
                            }
                        }
                        uint32_t w[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            float a = v[2 * e], b = v[2 * e + 1];
                            if (p.act2 == SS_ACT_GELU) { a = gelu(a); b = gelu(b); }
                            else { a = a < floor2 ? 0.f : a; b = b < floor2 ? 0.f : b; }
                            w[e] = cvt_pack2<ODT>(a, b);
                        }
                        *reinterpret_cast<uint4 *>(p.y2 + (size_t)pg * p.Cout2 + o) = make_uint4(w[0], w[1], w[2], w[3]);
                    }
                }
                cur = nxt;
            }
            return;
        }
        for (int it = etid; it < BN * RUNS; it += NT) {
            const int pl = it / RUNS, run = it % RUNS;
            const int pg = n0 + pl, o = m0 + run * 8;
            if (pg >= p.P || o >= p.Cout) continue;
            const uint2 lo = *reinterpret_cast<const uint2 *>(Cs + pl * CROW + run * 8);
            const uint2 hi = *reinterpret_cast<const uint2 *>(Cs + pl * CROW + run * 8 + 4);
            uint16_t *dst = p.y + (size_t)pg * p.Cout + o;
            if (vec_ok) {
                *reinterpret_cast<uint4 *>(dst) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            } else {
                const uint32_t w[4] = {lo.x, lo.y, hi.x, hi.y};
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (o + e < p.Cout) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
    } else if constexpr (!Q8) {
        // With a residual the tile crosses LDS in fp32 (conv + bias); the thread that stores a 16-byte run adds the
        // residual's run (fetched before the tile is written, so its latency hides behind the LDS phase), applies
        // the activation and rounds once.
        constexpr int CROW = BM + 4;     // floats per pixel row (+16 bytes: 16-byte writes of consecutive pixels spread over the banks)
        constexpr int ITERS = (BN * RUNS + NT - 1) / NT;
        float *Cf = reinterpret_cast<float *>(smem);
        u32x4 res[ITERS];
        auto load_res = [&]() {
            if (!vec_ok) return;
#pragma unroll
            for (int j = 0; j < ITERS; j++) {
                const int it = etid + j * NT;
                const int pl = it / RUNS, run = it % RUNS;
                const int pg = n0 + pl, o = m0 + run * 8;
                res[j] = u32x4{0u, 0u, 0u, 0u};
                if (it < BN * RUNS && pg < p.P && o < p.Cout)
                    res[j] = *reinterpret_cast<const u32x4 *>(p.residual + (size_t)pg * p.Cout + o);
            }
        };
        if constexpr (DEEP) load_res();      // (the shallow variants have no registers to spare next to the accumulators)
        if (!producer) {
#pragma unroll
            for (int tm = 0; tm < TM; tm++) {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int ol = (wm * TM + tm) * 32 + 8 * q + 4 * (lane >> 5);
                    const float4 bq = *reinterpret_cast<const float4 *>(bias_s + ol);
#pragma unroll
                    for (int tn = 0; tn < TN; tn++) {
                        const int pl = (wn * TN + tn) * 32 + (lane & 31);
                        *reinterpret_cast<float4 *>(Cf + pl * CROW + ol) =
                            make_float4((float)acc[tm][tn][4 * q + 0] + bq.x, (float)acc[tm][tn][4 * q + 1] + bq.y,
                                        (float)acc[tm][tn][4 * q + 2] + bq.z, (float)acc[tm][tn][4 * q + 3] + bq.w);
                    }
                }
            }
        }
        if constexpr (!DEEP) load_res();
        __syncthreads();
        auto from_lds = [&](auto actf) {
#pragma unroll
            for (int j = 0; j < ITERS; j++) {
                const int it = etid + j * NT;
                const int pl = it / RUNS, run = it % RUNS;
                const int pg = n0 + pl, o = m0 + run * 8;
                if (it >= BN * RUNS || pg >= p.P || o >= p.Cout) continue;
                const float4 lo = *reinterpret_cast<const float4 *>(Cf + pl * CROW + run * 8);
                const float4 hi = *reinterpret_cast<const float4 *>(Cf + pl * CROW + run * 8 + 4);
                const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                uint16_t *dst = p.y + (size_t)pg * p.Cout + o;
                if (vec_ok) {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; e++)
                        w[e] = cvt_pack2<ODT>(actf(v[2 * e] + widen<ODT>((uint16_t)(res[j][e] & 0xFFFFu))),
                                              actf(v[2 * e + 1] + widen<ODT>((uint16_t)(res[j][e] >> 16))));
                    *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
                } else {
                    const uint16_t *rs = p.residual + (size_t)pg * p.Cout + o;
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        if (o + e < p.Cout) dst[e] = (uint16_t)(cvt_pack2<ODT>(actf(v[e] + widen<ODT>(rs[e])), 0.f) & 0xFFFFu);
                }
            }
        };
        if (p.act == SS_ACT_GELU) from_lds(gelu); else from_lds(relu_or_id);
    }
}

// ---------------------------------------------------------------------------------------------
// 1x1 -> activation -> 1x1 (+ residual): the inverted bottleneck of a ConvNeXt block (narrow -> 4x wide -> narrow)
// in one kernel.  A workgroup owns 64 pixels.  Their input rows are staged in LDS once; the wide intermediate is
// produced 128 channels at a time (first contraction, bias, activation, rounding to 16 bit, LDS) and consumed at
// once by the second contraction, whose accumulators stay in registers across the chunks.  The intermediate, four
// times the size of the block's input and output, never reaches memory.
// ---------------------------------------------------------------------------------------------


template <int DT, bool SPARSE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void mlp_kernel(MlpParams p)
{
    constexpr int BN = 64, CH = 128;                      // pixels per workgroup, intermediate channels per chunk
    constexpr int CROW = CH + 4;                          // halfs per pixel row of the intermediate chunk (8-byte aligned rows)
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    const int XROW = p.Cin + 8;                           // halfs per pixel row of the input tile (16-byte aligned rows)
    uint16_t *Xs = smem;
    uint16_t *Cs = smem + BN * XROW;
    float *b1s = reinterpret_cast<float *>(Cs + BN * CROW);       // the first layer's bias, all Cmid values
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, c = lane & 31;
    const int n0 = blockIdx.x * BN;
    const __amdgpu_buffer_rsrc_t r1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a1_vals), 0, (int)p.a1_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t m1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.a1_meta), 0, (int)p.meta1_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t r2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.a2_vals), 0, (int)p.a2_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t m2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(p.a2_meta), 0, (int)p.meta2_bytes, kRsrcFlags);

    struct Row1 {                                         // one 32-row tile of the first layer: all its reduction steps
        u32x4 v[SPARSE ? 1 : 2][kMlpKs1];
        uint32_t idx[kMlpKs1];
    };
    auto load_row1 = [&](Row1 &r, int mt) {
#pragma unroll
        for (int s = 0; s < kMlpKs1; s++) {
            if (s >= p.Ks1) break;                        // uniform
            if constexpr (SPARSE) {
                r.v[0][s] = __builtin_amdgcn_raw_buffer_load_b128(r1, (int)(((unsigned)(mt * p.Ks1 + s) * 64 + lane) * 16u), 0, 0);
                r.idx[s] = __builtin_amdgcn_raw_buffer_load_b32(m1, (int)(((unsigned)(mt * p.Kp1 + (s >> 1)) * 64 + lane) * 4u), 0, 0);
            } else {
                const unsigned off = ((unsigned)(mt * p.Ks1 + s) * 128 + lane) * 16u;
                r.v[0][s] = __builtin_amdgcn_raw_buffer_load_b128(r1, (int)off, 0, 0);
                r.v[1][s] = __builtin_amdgcn_raw_buffer_load_b128(r1, (int)off, 1024, 0);
            }
        }
    };
    // the second layer's weights for this wave's output tiles and the 4 reduction steps of one chunk
    struct Row2 {
        u32x4 v[SPARSE ? 1 : 2][kMlpTiles][4];
        uint32_t idx[kMlpTiles][4];
    };
    const int ntiles2 = p.Mt2 * 2;                        // output tiles of the second layer: (row tile, pixel half)
    auto load_row2 = [&](Row2 &r, int mc) {
#pragma unroll
        for (int ti = 0; ti < kMlpTiles; ti++) {
            const int t = wave + 4 * ti;
            if (t >= ntiles2) break;                      // uniform
            const int rt = t >> 1;
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const int ks = mc * 4 + s;
                if constexpr (SPARSE) {
                    r.v[0][ti][s] = __builtin_amdgcn_raw_buffer_load_b128(r2, (int)(((unsigned)(rt * p.Ks2 + ks) * 64 + lane) * 16u), 0, 0);
                    r.idx[ti][s] = __builtin_amdgcn_raw_buffer_load_b32(m2, (int)(((unsigned)(rt * p.Kp2 + (ks >> 1)) * 64 + lane) * 4u), 0, 0);
                } else {
                    const unsigned off = ((unsigned)(rt * p.Ks2 + ks) * 128 + lane) * 16u;
                    r.v[0][ti][s] = __builtin_amdgcn_raw_buffer_load_b128(r2, (int)off, 0, 0);
                    r.v[1][ti][s] = __builtin_amdgcn_raw_buffer_load_b128(r2, (int)off, 1024, 0);
                }
            }
        }
    };

    Row1 a1;
    Row2 a2;
    load_row1(a1, wave);
    // ---- the input tile: 64 pixel rows of Cin channels, 16-byte vectors, zeros past the last pixel
    {
        const int upr = p.Cin >> 3;                       // 16-byte units per row
        for (int i = tid; i < BN * upr; i += 256) {
            const int px = i / upr, u = i - px * upr;
            const int pg = n0 + px;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (pg < p.P) v = *reinterpret_cast<const u32x4 *>(p.x + (size_t)pg * p.Cin + u * 8);
            *reinterpret_cast<u32x4 *>(Xs + px * XROW + u * 8) = v;
        }
        for (int i = tid; i < p.Cmid; i += 256) b1s[i] = p.bias1 ? p.bias1[i] : 0.f;
    }
    // this workgroup's residual, in the output stage's thread -> (pixel, run) mapping: fetched now, used at the very end
    u32x4 rres[kMlpTiles][2];
#pragma unroll
    for (int ti = 0; ti < kMlpTiles; ti++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int t = wave + 4 * ti, it = lane + 64 * j;
            const int pg = n0 + (t & 1) * 32 + (it >> 2);
            rres[ti][j] = u32x4{0u, 0u, 0u, 0u};
            if (p.res2 != nullptr && t < p.Mt2 * 2 && pg < p.P)
                rres[ti][j] = *reinterpret_cast<const u32x4 *>(p.res2 + (size_t)pg * p.Cout2 + (t >> 1) * 32 + (it & 3) * 8);
        }
    f32x16 acc2[kMlpTiles];
#pragma unroll
    for (int ti = 0; ti < kMlpTiles; ti++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc2[ti][v] = 0.f;
    const float floor1 = p.act1 == SS_ACT_RELU ? 0.f : -__builtin_inff();
    __syncthreads();

    const int nchunks = p.Cmid / CH;
    for (int mc = 0; mc < nchunks; mc++) {
        load_row2(a2, mc);                                // in flight while the first contraction runs
        // ---- first contraction: rows 128*mc + 32*wave + [0,32) of the intermediate, all 64 pixels
        f32x16 acc1[2];
#pragma unroll
        for (int tn = 0; tn < 2; tn++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc1[tn][v] = 0.f;
#pragma unroll
        for (int s = 0; s < kMlpKs1; s++) {
            if (s >= p.Ks1) break;                        // uniform
#pragma unroll
            for (int tn = 0; tn < 2; tn++) {
                const uint16_t *src = Xs + (tn * 32 + c) * XROW + 32 * s + 16 * g;
                B32 bf;
                bf.lo = *reinterpret_cast<const u32x4 *>(src);
                bf.hi = *reinterpret_cast<const u32x4 *>(src + 8);
                if constexpr (SPARSE) {
                    acc1[tn] = mma_sparse<DT>(a1.v[0][s], bf, acc1[tn], a1.idx[s] >> ((s & 1) * 16));
                } else {
                    acc1[tn] = mma_dense<DT>(a1.v[0][s], bf.lo, acc1[tn]);
                    acc1[tn] = mma_dense<DT>(a1.v[1][s], bf.hi, acc1[tn]);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const float4 bq1 = *reinterpret_cast<const float4 *>(b1s + (mc * 4 + wave) * 32 + 8 * q + 4 * g);
            const float bv[4] = {bq1.x, bq1.y, bq1.z, bq1.w};
#pragma unroll
            for (int tn = 0; tn < 2; tn++) {
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const float z = acc1[tn][4 * q + e] + bv[e];
                    r[e] = p.act1 == SS_ACT_GELU ? gelu_erfc(z) : (z < floor1 ? 0.f : z);
                }
                *reinterpret_cast<uint2 *>(Cs + (tn * 32 + c) * CROW + wave * 32 + 8 * q + 4 * g) =
                    make_uint2(cvt_pack2<DT>(r[0], r[1]), cvt_pack2<DT>(r[2], r[3]));
            }
        }
        if (mc + 1 < nchunks) load_row1(a1, (mc + 1) * 4 + wave);       // (its registers are free) in flight while the second contraction runs
        __syncthreads();
        // ---- second contraction: this chunk's 128 intermediate channels into the output accumulators
#pragma unroll
        for (int ti = 0; ti < kMlpTiles; ti++) {
            const int t = wave + 4 * ti;
            if (t >= ntiles2) break;                      // uniform
            const int ct = t & 1;
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const uint16_t *src = Cs + (ct * 32 + c) * CROW + 32 * s + 16 * g;       // 8-byte aligned
                const uint2 u0 = *reinterpret_cast<const uint2 *>(src), u1 = *reinterpret_cast<const uint2 *>(src + 4);
                const uint2 u2 = *reinterpret_cast<const uint2 *>(src + 8), u3 = *reinterpret_cast<const uint2 *>(src + 12);
                B32 bf;
                bf.lo = u32x4{u0.x, u0.y, u1.x, u1.y};
                bf.hi = u32x4{u2.x, u2.y, u3.x, u3.y};
                if constexpr (SPARSE) {
                    acc2[ti] = mma_sparse<DT>(a2.v[0][ti][s], bf, acc2[ti], a2.idx[ti][s] >> ((s & 1) * 16));
                } else {
                    acc2[ti] = mma_dense<DT>(a2.v[0][ti][s], bf.lo, acc2[ti]);
                    acc2[ti] = mma_dense<DT>(a2.v[1][ti][s], bf.hi, acc2[ti]);
                }
            }
        }
        __syncthreads();                                  // the chunk buffer is free again
    }

    // ---- output: bias + residual + activation in fp32, one rounding; each 32 x 32 tile crosses the wave's own LDS region
    // (the input tile and the chunk buffer are dead: the loop ended with a barrier) and leaves as 16-byte runs
    float *reg = reinterpret_cast<float *>(smem) + wave * (32 * kFuseRow);
    const float floor2 = p.act2 == SS_ACT_RELU ? 0.f : -__builtin_inff();
#pragma unroll
    for (int ti = 0; ti < kMlpTiles; ti++) {
        const int t = wave + 4 * ti;
        if (t >= ntiles2) break;                          // uniform
        const int rt = t >> 1, ct = t & 1;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const float4 bq = p.bias2 ? *reinterpret_cast<const float4 *>(p.bias2 + rt * 32 + 8 * q + 4 * g) : make_float4(0.f, 0.f, 0.f, 0.f);
            *reinterpret_cast<float4 *>(reg + c * kFuseRow + 8 * q + 4 * g) =
                make_float4(acc2[ti][4 * q + 0] + bq.x, acc2[ti][4 * q + 1] + bq.y, acc2[ti][4 * q + 2] + bq.z, acc2[ti][4 * q + 3] + bq.w);
        }
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int it = lane + 64 * j;
            const int px = it >> 2, run = it & 3;
            const int pg = n0 + ct * 32 + px, o = rt * 32 + run * 8;
            const float4 lo = *reinterpret_cast<const float4 *>(reg + px * kFuseRow + run * 8);
            const float4 hi = *reinterpret_cast<const float4 *>(reg + px * kFuseRow + run * 8 + 4);
            if (pg >= p.P) continue;
            float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            if (p.res2 != nullptr) {
                const u32x4 rr = rres[ti][j];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    v[2 * e] += widen<DT>((uint16_t)(rr[e] & 0xFFFFu));
                    v[2 * e + 1] += widen<DT>((uint16_t)(rr[e] >> 16));
                }
            }
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float a = v[2 * e], b = v[2 * e + 1];
                if (p.act2 == SS_ACT_GELU) { a = gelu_erfc(a); b = gelu_erfc(b); }
                else { a = a < floor2 ? 0.f : a; b = b < floor2 ? 0.f : b; }
                w[e] = cvt_pack2<DT>(a, b);
            }
            *reinterpret_cast<uint4 *>(p.y2 + (size_t)pg * p.Cout2 + o) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

template <int DT, bool SPARSE>
static int launch_mlp(const MlpParams &p, hipStream_t s)
{
    const long long blocks = ((long long)p.P + 63) / 64;
    if (blocks <= 0 || blocks > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    size_t smem = (size_t)64 * (p.Cin + 8) * 2 + (size_t)64 * (128 + 4) * 2 + (size_t)p.Cmid * 4;
    const size_t epi = 4 * kFuseRegion;
    if (smem < epi) smem = epi;
    mlp_kernel<DT, SPARSE><<<dim3((unsigned)blocks), dim3(256), smem, s>>>(p);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
template <int DT, bool SPARSE, int WAVES_M, int WAVES_N, int TM, int TN, int MODE, int KH, int KW, bool DEEP = false, bool SPEC = false, bool FUSE = false>
static int launch(const ConvParams &p0, hipStream_t s)
{
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int NWAVES = WAVES_M * WAVES_N + (SPEC ? 4 : 0);
    constexpr size_t scale_bytes = is_byte_type(DT) ? (size_t)BM * 4 : 0;      // the per-channel scales sit behind the bias values
    constexpr size_t smem_plain = smem_bytes<BM, BN, MODE, KH, KW, DEEP>(false, FUSE ? NWAVES : 0) + scale_bytes;
    constexpr size_t smem_res = (is_byte_type(DT) || FUSE) ? smem_plain : smem_bytes<BM, BN, MODE, KH, KW, DEEP>(true);
    static_assert(smem_plain <= 160 * 1024 && smem_res <= 160 * 1024, "LDS tile too large");
    const size_t smem = (p0.residual && !FUSE) ? smem_res : smem_plain;
    if (FUSE && (p0.Cout > BM || p0.Cout % 32 != 0)) return SS_ERR_UNSUPPORTED;      // the whole channel range must sit in one tile
    ConvParams p = p0;
    p.tiles_m = (p.Cout + BM - 1) / BM;
    fast_div_setup((unsigned)p.tiles_m, &p.tm_mul, &p.tm_sh);
    long long tiles_n = ((long long)p.P + BN - 1) / BN;
    long long blocks = (long long)p.tiles_m * tiles_n;
    if (FUSE || is_byte_type(DT) || p.nsplit < 1) p.nsplit = 1;
    if (p.nsplit > 1) {
        // the entry point planned the split for this very tile shape (plan_split) and sized the workspace for it
        if (p.ws_part == nullptr || p.ws_ctr == nullptr || p.plan_bm != BM || p.plan_bn != BN) return SS_ERR_WORKSPACE;
        blocks *= p.nsplit;
    }
    if (blocks <= 0 || blocks > 0x7FFFFFFFll) return SS_ERR_UNSUPPORTED;
    auto kern = conv_kernel<DT, SPARSE, WAVES_M, WAVES_N, TM, TN, MODE, KH, KW, DEEP, SPEC, FUSE>;
    if (smem_res > 64 * 1024) {
        // Raises this kernel's dynamic-LDS limit, once per device (the attribute belongs to the device's copy of the
        // kernel).  Two threads racing here both set it: harmless.
        static std::atomic<unsigned long long> done_mask{0};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return SS_ERR_HIP;
        const unsigned long long bit = 1ull << (dev & 63);
        if (dev >= 64 || !(done_mask.load(std::memory_order_acquire) & bit)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)smem_res) != hipSuccess)
                return SS_ERR_HIP;
            if (dev < 64) done_mask.fetch_or(bit, std::memory_order_release);
        }
    }
    kern<<<dim3((unsigned)blocks), dim3((WAVES_M * WAVES_N + (SPEC ? 4 : 0)) * 64), smem, s>>>(p);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

// Tile shapes (WAVES_M x WAVES_N multiplying waves, each TM x TN tiles of 32x32):
//   id 0:  64 x  64 (2x2 waves, 1x1)
//   id 1:  same, deep prefetch
//   id 2: 128 x  64 (4x1 waves, 1x2)
//   id 3: 256 x  64 (4x1 waves, 2x2), deep prefetch
//   id 4: 128 x  64 (4x1 waves, 1x2), deep prefetch, plus four producer waves
//   id 5: 256 x  64 (4x1 waves, 2x2), deep prefetch, plus four producer waves
// Layouts with all four waves along the output channels fetch no weight tile twice inside a workgroup.
// Measured and dropped because they won nowhere: 2x2 layouts of the larger tiles, 128x128 and 256x128 tiles,
// deep 128x64 and shallow 256x64 without producer waves, and splitting a tile's reduction over two wave groups
// (halves the LDS reads per multiply, but the exchange of partial sums and the doubled first chunk cost more), and a
// 128x64 tile of two multiplying waves of 64x64 plus producers (half the LDS reads of id 4, same memory traffic:
// 11.2 vs 9.6 us on the 3x3 256 -> 256 layer at batch 32 -- two waves do not keep four SIMDs' worth of latency hidden).
template <int DT, bool SPARSE, int MODE, int KH, int KW>
static int launch_tile(int id, const ConvParams &p, hipStream_t s)
{
    if constexpr (MODE != MODE_VEC8) {       // (the long-chunk staging is only ever paired with the deep tiles)
        switch (id) {
            case 0: return launch<DT, SPARSE, 2, 2, 1, 1, MODE, KH, KW, false>(p, s);
            case 1: return launch<DT, SPARSE, 2, 2, 1, 1, MODE, KH, KW, true>(p, s);
            case 2: return launch<DT, SPARSE, 4, 1, 1, 2, MODE, KH, KW, false>(p, s);
            default: break;
        }
    }
    if constexpr (MODE != MODE_VEC8 || !is_byte_type(DT)) {
        if (id == 3) return launch<DT, SPARSE, 4, 1, 2, 2, MODE, KH, KW, true>(p, s);
    }
    switch (id) {
        case 4: return launch<DT, SPARSE, 4, 1, 1, 2, MODE, KH, KW, true, true>(p, s);
        case 5: return launch<DT, SPARSE, 4, 1, 2, 2, MODE, KH, KW, true, true>(p, s);
        default: break;
    }
    return SS_ERR_INVALID_ARG;
}

template <int DT, bool SPARSE, int MODE, int KH, int KW>
static int pick_tile(const ConvParams &p, hipStream_t s)
{
    if (p.nsplit > 1) return launch_tile<DT, SPARSE, MODE, KH, KW>(p.plan_tile, p, s);     // planned by the entry point
    const int forced = forced_tile();                  // test hook (ss_debug.h): a tile shape by id, or -1
    if (forced >= 0) {
        int st = launch_tile<DT, SPARSE, MODE, KH, KW>(forced, p, s);
        if (st != SS_ERR_INVALID_ARG) return st;
    }
    constexpr bool pointwise = MODE == MODE_PW || MODE == MODE_PW2;
    constexpr bool bigchunk = (MODE == MODE_TAPS && KH * KW > 4) || MODE == MODE_VEC8;
    int id = choose_tile(p, pointwise, bigchunk);
    // The dense FP8 instruction of the deep kernels wants its 32-byte A operand in eight consecutive registers; the
    // 256x64 four-wave tile then runs at one wave per SIMD (measured 40 % slower than with producer waves).
    if (DT == SS_F8 && !SPARSE && id == 3) id = 5;
    return launch_tile<DT, SPARSE, MODE, KH, KW>(id, p, s);
}

// Channels-last flattening with taps: chunks of 256 reduction indices (a quarter of the barriers, four times the
// LDS) pay where the tile that goes with them is one of the deep ones -- few workgroups per compute unit anyway --
// and cost occupancy on the large grids of the shallow tiles.  (The 8-bit 256x64 tile without producer waves needs
// a few registers more than two waves per SIMD leave, so it keeps the short chunks.)
template <int DT, bool SPARSE>
static int pick_vec(const ConvParams &p, hipStream_t s)
{
    if (p.K >= 512) {
        const int forced = forced_tile();
        const int id = forced >= 0 ? forced : choose_tile(p, false, true);
        if (id == 4 || id == 5 || (id == 3 && !is_byte_type(DT))) return pick_tile<DT, SPARSE, MODE_VEC8, 1, 1>(p, s);
    }
    return pick_tile<DT, SPARSE, MODE_VEC, 1, 1>(p, s);
}

template <int DT, bool SPARSE>
static int pick_mode(const ss_weight_desc *desc, const ConvParams &p, hipStream_t s)
{
    const int taps = desc->kh * desc->kw;
    if constexpr (is_byte_type(DT)) {    // validated by the entry point: byte pairs are contiguous in every 16-byte run
        if (taps == 1) return p.Ks <= 2 ? pick_tile<DT, SPARSE, MODE_PW2, 1, 1>(p, s) : pick_tile<DT, SPARSE, MODE_PW, 1, 1>(p, s);
        if (desc->korder == SS_K_RSC) return pick_vec<DT, SPARSE>(p, s);
        if (desc->kh == 3) return pick_tile<DT, SPARSE, MODE_TAPS, 3, 3>(p, s);
        return pick_tile<DT, SPARSE, MODE_TAPS, 2, 2>(p, s);
    } else {
    // channels contiguous inside every aligned run of 8 reduction indices?
    if (desc->cin % 8 == 0 && taps == 1)
        return p.Ks <= 2 ? pick_tile<DT, SPARSE, MODE_PW2, 1, 1>(p, s) : pick_tile<DT, SPARSE, MODE_PW, 1, 1>(p, s);
    if (desc->cin % 8 == 0 && desc->korder == SS_K_RSC) return pick_vec<DT, SPARSE>(p, s);
    if (desc->korder == SS_K_CRS && desc->cin % 32 == 0) {
        if (desc->kh == 3 && desc->kw == 3) return pick_tile<DT, SPARSE, MODE_TAPS, 3, 3>(p, s);
        if (desc->kh == 2 && desc->kw == 2) return pick_tile<DT, SPARSE, MODE_TAPS, 2, 2>(p, s);
    }
    if (desc->cin % 4 == 0 && desc->korder == SS_K_RSC) return pick_tile<DT, SPARSE, MODE_GATHER4, 1, 1>(p, s);
    return pick_tile<DT, SPARSE, MODE_GATHER, 1, 1>(p, s);
    }
}

// ---------------------------------------------------------------------------------------------
// 3x3 (or any k x k with a fast staging mode) convolution followed by a 1x1 convolution, fused
// ---------------------------------------------------------------------------------------------
template <int DT, bool SPARSE, int MODE, int KH, int KW>
static int launch_fused_tile(int id, const ConvParams &p, hipStream_t s)
{
    switch (id) {
        case 0: return launch<DT, SPARSE, 2, 2, 1, 1, MODE, KH, KW, false, false, true>(p, s);
        case 1: return launch<DT, SPARSE, 2, 2, 1, 1, MODE, KH, KW, true, false, true>(p, s);
        case 2: return launch<DT, SPARSE, 4, 1, 1, 2, MODE, KH, KW, false, false, true>(p, s);
        case 3: return launch<DT, SPARSE, 4, 1, 2, 2, MODE, KH, KW, true, false, true>(p, s);
        case 4: return launch<DT, SPARSE, 4, 1, 1, 2, MODE, KH, KW, true, true, true>(p, s);
        case 5: return launch<DT, SPARSE, 4, 1, 2, 2, MODE, KH, KW, true, true, true>(p, s);
        default: break;
    }
    return SS_ERR_INVALID_ARG;
}

// The tile must hold every output channel of the first convolution: 64, 128 or 256 rows; among the tiles of that
// height the grid size decides as in choose_tile.
static inline int choose_fused_tile(const ConvParams &p)
{
    if (p.Cout <= 64) return n_blocks(p, 64, 64) <= 1024 ? 1 : 0;
    if (p.Cout <= 128) return n_blocks(p, 128, 64) <= 256 ? 4 : 2;
    return n_blocks(p, 256, 64) <= 256 ? 5 : 3;
}

template <int DT, bool SPARSE>
static int fused_mode(const ss_weight_desc *d1, const ConvParams &p, hipStream_t s)
{
    auto run = [&](int id) {
        if (d1->korder == SS_K_CRS && d1->kh == 3 && d1->kw == 3 && d1->cin % 32 == 0)
            return launch_fused_tile<DT, SPARSE, MODE_TAPS, 3, 3>(id, p, s);
        if (d1->korder == SS_K_RSC && d1->cin % 8 == 0) return launch_fused_tile<DT, SPARSE, MODE_VEC, 1, 1>(id, p, s);
        return (int)SS_ERR_UNSUPPORTED;
    };
    const int forced = forced_tile();      // test hook; a tile that cannot hold the first layer's channels falls back
    if (forced >= 0) {
        const int st = run(forced);
        if (st != SS_ERR_UNSUPPORTED && st != SS_ERR_INVALID_ARG) return st;
    }
    return run(choose_fused_tile(p));
}

}  // namespace ss

#endif
