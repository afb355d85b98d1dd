// Instantiates the convolution kernels for one operand type and one operand form (2:4-sparse or dense), named by the
// including file through SS_INST_NAME / SS_INST_DT / SS_INST_SPARSE / SS_INST_FUSED.
#include "ss_conv_kernel.h"
#include "ss_conv_stream.h"
#include "ss_conv_image.h"
#include "ss_conv_rows.h"

#define SS_CAT2(a, b) a##b
#define SS_CAT(a, b) SS_CAT2(a, b)

namespace ss {

int SS_CAT(conv_dispatch_, SS_INST_NAME)(const ss_weight_desc *desc, const ConvParams &p, hipStream_t s)
{
    if constexpr (!is_byte_type(SS_INST_DT)) {
        if (p.nsplit <= 1 && stream_eligible(desc, p)) {
            int ncu = compute_units();
            if (ncu <= 0) return SS_ERR_HIP;
            if (block_limit() > 0 && block_limit() < ncu) ncu = block_limit();
            const int forced = forced_tile();
            // The resident-grid kernel pays where every compute unit gets at least two of its 256 x 128 tiles (measured:
            // 16-20 % faster than the one-tile kernels at three tiles per compute unit, slower at one) and the 256-row
            // tile is mostly filled.
            const long long tiles = (long long)((p.Cout + 255) / 256) * (((long long)p.P + 127) / 128);
            const bool pays = p.Cout % 256 == 0 || p.Cout % 256 >= 192;
            if (forced == 10 || (forced < 0 && pays && tiles >= 2ll * ncu))
                return launch_stream<SS_INST_DT, SS_INST_SPARSE, 2, 4>(p, ncu, s);
            if (forced == 11) return launch_stream<SS_INST_DT, SS_INST_SPARSE, 2, 2>(p, ncu, s);
        }
    }
    if constexpr (!is_byte_type(SS_INST_DT)) {
        // 1x1 layers with short reductions and many output channels: activations stationary (tile id 13 when forced)
        const int forced = forced_tile();
        // Measured on the ResNet-50 / ConvNeXt-T layers: it pays for the channel-expanding layers (64 -> 256 ... 512 -> 2048
        // and the 512 -> 1024 projection: 5-13 % faster; 96 -> 384 with GELU: 117 -> 84 us) and loses on the reducing
        // ones, whose few output channels leave nothing to walk over.
        // With a residual tail the gain is smaller (the residual runs are fetched by the same waves that multiply), and
        // at 512 channels, where LDS leaves room for one workgroup per compute unit, it turns into a loss.
        // With few pixel tiles (small batches of the late stages) the long reductions do better in the tiled kernels
        // (7x7 images, 512 -> 2048: 4.4 vs 5.7 us at batch 1, 4.7 vs 6.0 us at batch 8).
        const bool pays = p.Cout >= 2 * desc->cin && p.Cout >= 256 && !(desc->cin >= 512 && p.residual != nullptr) &&
                          (desc->cin <= 128 || (long long)p.P >= 48 * 64);
        if ((forced == 13 || (forced < 0 && pays)) && rows_eligible(desc, p)) {
            int ncu = compute_units();
            if (ncu <= 0) return SS_ERR_HIP;
            if (block_limit() > 0 && block_limit() < ncu) ncu = block_limit();
            return launch_rows<SS_INST_DT, SS_INST_SPARSE>(desc, p, ncu, s);
        }
    }
    if constexpr (!is_byte_type(SS_INST_DT) && !SS_INST_SPARSE) {
        // the dense first layer of an image network (tile id 12 when forced)
        const int forced = forced_tile();
        if ((forced < 0 || forced == 12) && image_eligible(desc, p)) {
            int ncu = compute_units();
            if (ncu <= 0) return SS_ERR_HIP;
            if (block_limit() > 0 && block_limit() < ncu) ncu = block_limit();
            return launch_image<SS_INST_DT>(desc, p, ncu, s);
        }
    }
    return pick_mode<SS_INST_DT, SS_INST_SPARSE>(desc, p, s);
}

#if SS_INST_FUSED
int SS_CAT(fused_dispatch_, SS_INST_NAME)(const ss_weight_desc *d1, const ConvParams &p, hipStream_t s)
{
    return fused_mode<SS_INST_DT, SS_INST_SPARSE>(d1, p, s);
}

int SS_CAT(mlp_dispatch_, SS_INST_NAME)(const MlpParams &p, hipStream_t s)
{
    return launch_mlp<SS_INST_DT, SS_INST_SPARSE>(p, s);
}
#endif

}  // namespace ss
