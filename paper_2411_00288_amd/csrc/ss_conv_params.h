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

// Test hook (ss_debug.h): the tile id forced by ss_debug_force_tile, or -1 when the library chooses.
int forced_tile();
// Test hook (ss_debug.h): upper bound on the workgroups of the resident-grid kernels, or 0 for none.
int block_limit();

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
