// Parameter blocks of the convolution kernels and the per-type dispatch functions that connect the entry points
// (ss_conv.hip) with the translation units that instantiate the kernels (ss_conv_inst_*.hip).
#ifndef SS_CONV_PARAMS_H_
#define SS_CONV_PARAMS_H_
#include "ss_internal.h"

namespace ss {

struct ConvParams {
    const uint16_t *x;
    const uint8_t *a_vals;    // first value tile (after the header)
    const uint32_t *a_meta;   // first metadata tile (sparse only)
    const float *bias;
    const float *scale;       // 8-bit operands: per-output-channel factor of the sum, or nullptr (= 1)
    const uint16_t *residual; // [P][Cout] like y, or nullptr
    uint16_t *y;
    int N, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw, Ho, Wo, P, K, Ks, Kp, Mt, act, korder;
    int tiles_m;
    unsigned x_bytes, a_bytes, meta_bytes;
    // division by Ho*Wo, Wo and tiles_m as multiply + shift (see fast_div)
    unsigned howo_mul, howo_sh, wo_mul, wo_sh, tm_mul, tm_sh, cin_mul, cin_sh, kw_mul, kw_sh;
    // fused second contraction (a 1x1 convolution on this convolution's output tile)
    const uint8_t *a2_vals;
    const uint32_t *a2_meta;
    const float *bias2;
    const uint16_t *res2;     // [P][Cout2] or nullptr
    uint16_t *y2;             // [P][Cout2]
    int Cout2, Ks2, Kp2, Mt2, act2;
    unsigned a2_bytes, meta2_bytes;
    // split reduction: workgroups per output tile (1 = none), fp32 partial sums [tile][split][BM*BN] and one ticket
    // counter per tile, both in the caller's workspace
    int nsplit, plan_tile, plan_bm, plan_bn;      // plan_*: the tile the split was planned (and the workspace sized) for
    float *ws_part;
    unsigned *ws_ctr;
};

// floor(n / d) for 0 <= n < 2^31 as (n * mul) >> sh with s = ceil(log2 d), sh = 31 + s, mul = ceil(2^sh / d):
// mul * d - 2^sh < d <= 2^s, so the product overshoots n / d by less than 1 / d, never reaching the next integer.
static inline void fast_div_setup(unsigned d, unsigned *mul, unsigned *sh)
{
    unsigned s = 0;
    while ((1ull << s) < d) s++;
    *sh = 31 + s;
    *mul = (unsigned)(((1ull << (31 + s)) + d - 1) / d);
}

struct MlpParams {
    const uint16_t *x;        // [P][Cin]
    const uint8_t *a1_vals, *a2_vals;
    const uint32_t *a1_meta, *a2_meta;
    const float *bias1, *bias2;
    const uint16_t *res2;     // [P][Cout2] or nullptr
    uint16_t *y2;             // [P][Cout2]
    int P, Cin, Cmid, Cout2, Ks1, Kp1, Ks2, Kp2, Mt2, act1, act2;
    unsigned a1_bytes, meta1_bytes, a2_bytes, meta2_bytes;
};

constexpr int kMlpKs1 = 4;        // first reduction: at most 128 input channels
constexpr int kMlpTiles = 2;      // 32x32 output tiles of the second layer per wave: at most 128 output channels x 64 pixels over 4 waves

static inline long long n_blocks(const ConvParams &p, int bm, int bn)
{
    return (long long)((p.Cout + bm - 1) / bm) * (((long long)p.P + bn - 1) / bn);
}


// Tile id for a problem.  Measured on MI355X (tile sweep over the ResNet-50 / ConvNeXt-T layer shapes, 256 compute
// units).  pointwise: 1x1 staging; bigchunk: staging in chunks of 256+ reduction indices (3x3 tap transpose, long
// channels-last reductions).
static inline int choose_tile(const ConvParams &p, bool pointwise, bool bigchunk)
{
    if (p.Cout <= 64) {
        const bool deep = n_blocks(p, 64, 64) <= 1024 || (pointwise && p.K >= 256);
        return deep ? 1 : 0;
    }
    // Grids of at most one workgroup per compute unit: nothing else hides a wave's stalls, so separate producer
    // waves pay.  Larger grids do better with two four-wave workgroups per compute unit.
    const long long b128 = n_blocks(p, 128, 64), b256 = n_blocks(p, 256, 64);
    if (p.Cout > 128 && b256 > 128 && b256 <= 256) return 5;
    if (b128 <= 256) return 4;
    if (p.Cout >= 512 && p.K >= 512) return 3;
    if (bigchunk && p.Cout >= 256 && b256 >= 512) return 3;
    return 2;
}


// Split of a convolution's reduction over several workgroups per output tile (for grids that leave most compute
// units idle: few output pixels, long reductions -- small-batch inference and the last stages of a network).
struct SplitPlan {
    int tile, bm, bn, nsplit;        // tile id and shape; workgroups per output tile (1 = no split, nothing else is used)
    long long tiles;
    size_t ctr_bytes, part_bytes;    // workspace: ticket counters, then fp32 partial sums [tile][split][bm * bn]
};
// Decides tile and split for a 16-bit problem.  Only the two staging modes of the networks' own layers split (1x1
// kernels with more than two 32-wide steps; 3x3 kernels in the channel-slowest flattening with cin % 32 == 0).
// forced_tile / forced_split: test hooks (negative / zero: the library decides).  A split happens by itself when the
// grid would leave at least half of the compute units idle and the reduction is long enough to pay for the hand-over.
inline SplitPlan plan_split(const ss_weight_desc *d, long long P, int Ks, int ncu, int forced_tile, int forced_split)
{
    SplitPlan pl{};
    pl.nsplit = 1;
    if (is_byte_type(d->dtype)) return pl;
    if (forced_tile >= 10) return pl;              // the resident-grid, image and activation-stationary kernels do not split
    const bool pw = d->kh * d->kw == 1 && d->cin % 8 == 0 && Ks > 2;
    const bool taps = d->korder == SS_K_CRS && d->kh == 3 && d->kw == 3 && d->cin % 32 == 0;
    if (!pw && !taps) return pl;
    const int ksteps = taps ? 9 : 4;
    ConvParams q{};
    q.Cout = d->cout; q.P = (int)P; q.K = d->cin * d->kh * d->kw;
    pl.tile = (forced_tile >= 0 && forced_tile <= 5) ? forced_tile : choose_tile(q, pw, taps);
    pl.bm = pl.tile <= 1 ? 64 : ((pl.tile == 2 || pl.tile == 4) ? 128 : 256);
    pl.bn = 64;
    pl.tiles = n_blocks(q, pl.bm, pl.bn);
    const int nchunks = (Ks + ksteps - 1) / ksteps;
    int n = 1;
    if (forced_split > 0) n = forced_split;
    else if (forced_tile < 0 && pl.tiles * 2 <= ncu) {
        // Measured on MI355X: handing the partial sums over costs about as much as four 3x3 chunks (sixteen of the
        // shorter 1x1 chunks), so a share keeps at least that many.  (512 -> 512 3x3 at 7x7: batch 1, 4 tiles, 14.5 us
        // whole, 9.6 us in four shares; batch 8, 28 tiles, 14.8 -> 11.7 us; reductions of 2304 and the 1x1 layers up
        // to 2048 channels gained nothing and stay whole.)
        const int per_share = taps ? 4 : 16;
        n = (int)(ncu / pl.tiles);
        if (n > nchunks / per_share) n = nchunks / per_share;
        if (n > 8) n = 8;
        if (nchunks < 3 * per_share) n = 1;
    }
    if (n > nchunks) n = nchunks;
    if (n < 1) n = 1;
    pl.nsplit = n;
    pl.ctr_bytes = (size_t)((pl.tiles * 4 + 255) / 256 * 256);
    pl.part_bytes = (size_t)pl.tiles * n * pl.bm * pl.bn * 4;
    return pl;
}

// Test hook (ss_debug.h): the tile id forced by ss_debug_force_tile, or -1 when the library chooses.
int forced_tile();
// Test hook (ss_debug.h): upper bound on the workgroups of the resident-grid kernels, or 0 for none.
int block_limit();
// Test hook (ss_debug.h): workgroups per output tile forced by ss_debug_force_split, or 0 when the library decides.
int forced_split();

// Compute units of the current device (cached per device), or -1 when the runtime cannot say.
int compute_units();

// One function per operand type and operand form, each defined in its own translation unit.  conv_dispatch_* picks
// the staging mode and tile for the problem and launches; fused_dispatch_* does so for a k x k convolution followed by
// a 1x1 one; mlp_dispatch_* launches the 1x1 -> 1x1 kernel.  All return an SS_* status.
#define SS_DECLARE_CONV(NAME) \
    int conv_dispatch_##NAME(const ss_weight_desc *desc, const ConvParams &p, hipStream_t s);
#define SS_DECLARE_FUSED(NAME) \
    int fused_dispatch_##NAME(const ss_weight_desc *d1, const ConvParams &p, hipStream_t s); \
    int mlp_dispatch_##NAME(const MlpParams &p, hipStream_t s);
SS_DECLARE_CONV(f16_sparse) SS_DECLARE_CONV(f16_dense) SS_DECLARE_CONV(bf16_sparse) SS_DECLARE_CONV(bf16_dense)
SS_DECLARE_CONV(i8_sparse) SS_DECLARE_CONV(i8_dense) SS_DECLARE_CONV(f8_sparse) SS_DECLARE_CONV(f8_dense)
SS_DECLARE_FUSED(f16_sparse) SS_DECLARE_FUSED(f16_dense) SS_DECLARE_FUSED(bf16_sparse) SS_DECLARE_FUSED(bf16_dense)

}  // namespace ss

#endif
