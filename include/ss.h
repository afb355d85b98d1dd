/*
 * ss.h -- C ABI of the 2:4 semi-structured-sparse convolution library for AMD MI355X (gfx950).
 *
 * The library computes the inference-time masked convolution of
 * "Inducing Semi-Structured Sparsity by Masking for Efficient Model Inference in Convolutional
 * Networks" (Sec. 3.3, Eq. 6):
 *
 *        Y = (M (.) W) * U(X)
 *
 * where W in R^{cout x K}, K = cin*kh*kw, is the weight matrix built from the cout kernels
 * (Eq. 5), M in {0,1}^{cout x K} is a 2:4 mask (Sec. 3.1, Eq. 2: every block of 4 consecutive
 * entries of a row holds exactly two ones), and U is the unfold operator, which is never
 * materialised.  W and M are inputs and are never written: the original weights stay unchanged
 * (abstract; Sec. 3.1, last paragraph).
 *
 * General conventions
 *   - Every function returns an int status: SS_OK (0) or a negative SS_ERR_* code.  Nothing throws.
 *   - Unless a parameter is marked [host], every data pointer is a DEVICE pointer.  The caller
 *     owns every buffer; the library never allocates or frees device memory.  Its only state is a per-device
 *     record of which kernels have had their shared-memory limit raised (set once, at a kernel's first launch).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The convolution
 *     calls only enqueue work on it and return; ss_mask_compress additionally waits for the
 *     stream once, because it reports the mask's validity.
 *   - 16-bit element types: SS_F16 (IEEE binary16) and SS_BF16 (bfloat16).  Activations, weights
 *     and outputs of one call share the type.  Products are accumulated in fp32, the bias is
 *     fp32, and the result is rounded once (round-to-nearest-even) when it is stored.
 *   - 8-bit operands (SS_I8, SS_F8): further precision points beyond the 16-bit floats the paper uses.
 *     SS_I8: weights and activations are signed bytes, products are accumulated exactly in int32.
 *     SS_F8: weights and activations are OCP FP8 E4M3 bytes, products (exact in fp32) are accumulated
 *     in fp32.  Either way the output is the 16-bit float act(scale[o]*sum + bias[o]); see
 *     ss_conv2d_q8_fwd.  The packing functions take such descriptors (layout below, the same for both:
 *     bytes are copied, never interpreted); ss_mask_update_compress and the 16-bit convolution entry
 *     points reject them with SS_ERR_UNSUPPORTED.
 *   - Activations and outputs are NHWC: x[N][H][Wd][cin], y[N][Ho][Wo][cout], with
 *     Ho = floor((H + 2*pad_h - kh)/stride_h) + 1 and likewise Wo.  Zero padding, no dilation,
 *     no groups (grouped convolutions are left dense by the method, Sec. 4 "Architectures").
 *   - The operation is a cross-correlation, as Eq. (4) writes it: input row = ho*stride_h - pad_h + r.
 *   - Flattening of (c, r, t) into the reduction index k, which decides which 4 weights form a
 *     block:  SS_K_CRS  k = (c*kh + r)*kw + t   (channel slowest; the order in which Eq. (5)
 *                                                builds W from the kernels; default)
 *             SS_K_RSC  k = (r*kw + t)*cin + c   (channels-last flattening)
 *     For 1x1 kernels the two coincide.
 *   - K must be a multiple of 4 per row (blocks never straddle rows); otherwise the layer is
 *     rejected with SS_ERR_UNSUPPORTED and stays dense at the caller's side (Sec. 3.3, last
 *     paragraph, leaves the augmentation to the user).
 */
#ifndef SS_H_
#define SS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SS_OK = 0,
    SS_ERR_INVALID_ARG = -1, /* null required pointer, non-positive size, unknown enum, empty output */
    SS_ERR_BAD_MASK    = -2, /* a block of 4 mask entries without exactly two ones (or an entry > 1) */
    SS_ERR_UNSUPPORTED = -3, /* K % 4 != 0, or sizes beyond 32-bit index limits */
    SS_ERR_WORKSPACE   = -4, /* workspace smaller than ss_conv2d_workspace_bytes reports */
    SS_ERR_HIP         = -5  /* a HIP runtime call failed (launch error, no device, ...) */
};

enum { SS_F16 = 0, SS_BF16 = 1, SS_I8 = 2, SS_F8 = 3 /* OCP FP8 E4M3 (no infinities; S.1111.111 = NaN) */ };
enum { SS_K_CRS = 0, SS_K_RSC = 1 };
enum { SS_ACT_NONE = 0, SS_ACT_RELU = 1, SS_ACT_GELU = 2 };

/* Describes one weight matrix W in R^{cout x (cin*kh*kw)} (Eq. 5).  Plain data, passed by pointer [host]. */
typedef struct {
    int32_t cout, cin, kh, kw;
    int32_t dtype;  /* SS_F16 | SS_BF16 | SS_I8 | SS_F8 (weights and activations; see "8-bit operands") */
    int32_t korder; /* SS_K_CRS | SS_K_RSC */
} ss_weight_desc;

/* Human-readable name of a status code.  Never NULL.  [host] */
const char *ss_status_string(int status);

/*
 * Size in bytes of the packed (structured) representation that ss_mask_compress writes and
 * ss_conv2d_fwd reads (Fig. 1: surviving values + a 2-bit position index each).
 *
 * Device layout, with Mt = ceil(cout/32) row tiles and Ks = ceil(K/32) reduction steps:
 *   bytes [0, 256)       header, 64 little-endian uint32:
 *                        [0]=0x34325353 [1]=1 [2]=cout [3]=cin [4]=kh [5]=kw [6]=dtype [7]=korder
 *                        [8]=Mt [9]=Ks [10]=index of the first invalid block (row*K/4+block) or
 *                        0xFFFFFFFF if the mask is valid, rest 0
 *   values               Mt*Ks tiles of 64 lanes x 8 elements (16 bytes per lane, 1 KiB per tile),
 *                        tile (mt, ks) at 256 + (mt*Ks + ks)*1024.  Lane l, slot s holds, for row
 *                        o = 32*mt + l%32 and block g = 8*ks + 4*(s/4) + 2*(l/32) + (s/2)%2 of that
 *                        row, the (s%2)-th kept weight of the block (ascending position).
 *   metadata             Mt*ceil(Ks/2) tiles of 64 uint32, after the values.  Lane l of tile
 *                        (mt, ks/2) holds in its low (ks even) or high (ks odd) 16 bits four
 *                        nibbles, nibble j (bits 4j..4j+3) = i0 | (i1 << 2) for the block held in
 *                        slots 2j, 2j+1 of the same lane of value tile (mt, ks); i0 < i1 are the
 *                        kept positions inside the block.
 *   Rows >= cout and blocks >= K/4 are padding: values +0, nibble 0x4.
 * This is the operand layout of gfx950's V_SMFMAC_F32_32X32X32_{F16,BF16} (sparse A operand and
 * its index register), so the convolution loads it straight into registers.
 *
 * SS_I8 / SS_F8: same header ([6] = dtype) and tile sizes, with Ks = ceil(K/64) reduction steps of 64 indices:
 *   values               tile (mt, ks): 64 lanes x 16 bytes.  Lane l, slot s holds, for row 32*mt + l%32 and
 *                        block g = 16*ks + 8*(s/8) + 4*(l/32) + (s%8)/2, the (s%2)-th kept weight.
 *   metadata             Mt*Ks tiles of 64 uint32, after the values; lane l of tile (mt, ks) holds eight
 *                        nibbles, nibble j = i0 | (i1 << 2) for the block in slots 2j, 2j+1.
 * (the operand layout of V_SMFMAC_I32_32X32X64_I8 and V_SMFMAC_F32_32X32X64_FP8_FP8).
 */
int ss_packed_bytes(const ss_weight_desc *desc, size_t *packed_bytes /*[host] out*/);

/*
 * Size in bytes of the dense tiled copy of M (.) W that ss_dense_pack writes and
 * ss_conv2d_dense_fwd reads: a 256-byte header as above (magic 0x44325353) followed by
 * Mt*Ks*2 tiles of 64 lanes x 8 elements; tile (mt, ks, h) lane l slot s holds
 * (M (.) W)[32*mt + l%32][32*ks + 16*(l/32) + 8*h + s], zero where out of range.
 * SS_I8 / SS_F8: tiles of 64 lanes x 16 bytes, Ks = ceil(K/64); tile (mt, ks, h) lane l slot s holds
 * (M (.) W)[32*mt + l%32][64*ks + 32*(l/32) + 16*h + s].
 */
int ss_dense_bytes(const ss_weight_desc *desc, size_t *dense_bytes /*[host] out*/);

/*
 * Weight compressor (Fig. 1; Sec. 3.1 Eq. 2 for the validity rule).
 *   W       [cout][K] elements of desc->dtype (16-bit, or int8), flattening per desc->korder   (read only)
 *   M       [cout][K] bytes, each 0 or 1                                    (read only)
 *   packed  ss_packed_bytes(desc) bytes, 16-byte aligned                    (written)
 *   bad_row_group [host, optional] two int32: on SS_ERR_BAD_MASK receives the row and the block
 *           index of the first (row-major) invalid block.
 * Values are copied bit for bit: a kept weight that is -0, NaN or subnormal is preserved.
 * Waits for `stream`.  On SS_ERR_BAD_MASK the contents of `packed` must not be used.
 */
int ss_mask_compress(const ss_weight_desc *desc, const void *W, const uint8_t *M,
                     void *packed, int32_t *bad_row_group, void *stream);

/*
 * Re-packing after a weight update (Sec. 3.2, the lemma on masking an updated model: the weights
 * move to V = W + U and the mask learned for W stays).  One pass over the weights:
 *     V = round16( float(W) + float(U) )     element-wise, binary32 sum, one rounding to nearest even,
 *                                            written back over W,
 *     packed = the structured representation of M (.) V, exactly as ss_mask_compress(V, M) writes it.
 *   W  [cout][K] 16-bit, desc->dtype, 8-byte aligned                        (read and written)
 *   U  [cout][K] 16-bit, desc->dtype, 8-byte aligned; must not overlap W    (read only)
 * Every other argument, the synchronisation and the error behaviour as for ss_mask_compress.  W is
 * updated in every block, also in one whose mask is invalid.  The bit pattern of a NaN result is
 * the hardware's.
 */
int ss_mask_update_compress(const ss_weight_desc *desc, void *W, const void *U, const uint8_t *M,
                            void *packed, int32_t *bad_row_group, void *stream);

/*
 * Inverse of the compressor: writes M (.) W as a plain [cout][K] matrix (desc->korder), +0 at
 * the dropped positions.  Test and debugging aid; asynchronous on `stream`.
 */
int ss_mask_decompress(const ss_weight_desc *desc, const void *packed, void *W_masked_out,
                       void *stream);

/*
 * Builds the dense twin's operand: the entry-wise product M (.) W (Eq. 6) in the tiled layout
 * described at ss_dense_bytes.  M == NULL means an all-ones mask (plain dense layer).  The mask
 * is not validated here.  Asynchronous on `stream`.
 */
int ss_dense_pack(const ss_weight_desc *desc, const void *W, const uint8_t *M, void *dense,
                  void *stream);

/*
 * Set-up-time check that a weight buffer belongs to a descriptor.  The convolution calls are asynchronous and
 * trust their weight operand: they read it with the sizes the descriptor implies and never look at its header.
 * This call reads the buffer's 256-byte header back (one stream synchronisation, like ss_mask_compress) and returns
 *   SS_ERR_INVALID_ARG  when the buffer was not written by ss_mask_compress / ss_mask_update_compress (sparse != 0)
 *                       or ss_dense_pack (sparse == 0), or was written for another cout, cin, kh, kw, dtype or
 *                       korder than desc states (e.g. a dense operand offered to ss_conv2d_fwd);
 *   SS_ERR_BAD_MASK     when it was written by a compression call that rejected its mask (Eq. 2 violated);
 *   SS_OK               otherwise.
 * Call it once per weight buffer, after packing and before the first convolution.
 */
int ss_weights_check(const ss_weight_desc *desc, const void *weights, int32_t sparse, void *stream);

/*
 * Scratch the convolution needs for the given problem on the current device: 0 for most problems.  Where the output
 * has so few tiles that most compute units would idle (few output pixels and a long reduction: small-batch inference,
 * the last stages of a network), the 16-bit convolutions split the reduction over several workgroups per output tile;
 * the workspace then holds their fp32 partial sums and one ticket counter per tile.  The partial sums are added in a
 * fixed order and rounded once, so the result does not depend on which workgroup finishes last.  Same value for the
 * sparse and the dense call and for the calls with a residual; 0 for the 8-bit operand types.
 *
 * Contract of a non-empty workspace: 256-byte aligned; zero-filled by the caller once, before the first call that
 * uses it (every call hands the ticket counters back at zero, so one clearing per allocation is enough, also under
 * HIP-graph replay); not shared by calls that may run at the same time.
 */
int ss_conv2d_workspace_bytes(const ss_weight_desc *desc, int32_t N, int32_t H, int32_t Wd,
                              int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                              size_t *bytes /*[host] out*/);

/*
 * Masked convolution, Eq. (6), with the layer model sigma(Wx + b) of Lemma 3.1 fused:
 *     y[n,ho,wo,o] = act( bias[o] + sum_{c,r,t} (M (.) W)[o,k(c,r,t)] * x[n, ho*sh-ph+r, wo*sw-pw+t, c] )
 * Only the two kept products of each block are issued (gfx950 sparse MFMA).
 *   x         [N][H][Wd][cin]    16-bit, desc->dtype                        (read only)
 *   packed    buffer written by ss_mask_compress for the same desc          (read only)
 *   bias      [cout] fp32, or NULL for no bias                              (read only)
 *   act       SS_ACT_NONE | SS_ACT_RELU | SS_ACT_GELU (z * Phi(z), exact normal CDF)
 *   y         [N][Ho][Wo][cout]  16-bit, desc->dtype                        (written)
 *   workspace ws_bytes >= ss_conv2d_workspace_bytes(...) bytes, see there; may be NULL when that size is 0
 *             (SS_ERR_WORKSPACE when it is needed and missing or too small)
 * Asynchronous on `stream`; launch errors are returned as SS_ERR_HIP.
 */
int ss_conv2d_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                  const void *packed, const float *bias,
                  int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                  void *y, void *workspace, size_t ws_bytes, void *stream);

/*
 * ss_conv2d_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP-graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace pair, same kernels, same
 * result bits.  The scratch of a split reduction lives in a device array inside the library's code object instead:
 * 16 MiB + 64 KiB per GPU the library runs on, held until the process ends; that is the largest workspace the library
 * plans by itself (ss_conv2d_workspace_bytes never reports more unless a test hook forces a split), and a problem that
 * would need more is rejected with SS_ERR_WORKSPACE.  The call allocates and frees nothing.  All calls on one GPU
 * share the array: it starts out zero, every call hands its ticket counters back at zero, and calls that may run at
 * the same time on one GPU (different streams, different threads) race on it -- serialise them or use ss_conv2d_fwd
 * with workspaces of their own.
 */
int ss_conv2d_fwd_static_ws(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                            const void *packed, const float *bias,
                            int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                            void *y, void *stream);

/*
 * The same-design dense twin: identical tiling, staging and epilogue, with the dense MFMA
 * instruction on the operand built by ss_dense_pack.  Denominator of the speed-up metric, and
 * the path for layers that stay dense.
 */
int ss_conv2d_dense_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                        const void *dense, const float *bias,
                        int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                        void *y, void *workspace, size_t ws_bytes, void *stream);

/*
 * The masked convolution as the last layer of a residual block: the layer model sigma(Wx + b) of
 * Lemma 3.1 with the block's skip connection added before the activation,
 *     y = act( conv(x) + bias + residual ),
 * computed in fp32 and rounded once at the store.  Saves the separate pass that would read and
 * rewrite the whole activation tensor.
 *   residual  [N][Ho][Wo][cout]  16-bit, desc->dtype, 16-byte aligned, or NULL (then the call is
 *             ss_conv2d_fwd).  Read only; it may be the same buffer as y (every element is read
 *             by the thread that then writes it).
 * Every other argument, and the error behaviour, as for ss_conv2d_fwd.
 */
int ss_conv2d_res_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                      const void *packed, const float *bias, const void *residual,
                      int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                      void *y, void *workspace, size_t ws_bytes, void *stream);

/* The dense twin of ss_conv2d_res_fwd (operand built by ss_dense_pack). */
int ss_conv2d_dense_res_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                            const void *dense, const float *bias, const void *residual,
                            int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                            void *y, void *workspace, size_t ws_bytes, void *stream);

/*
 * Two masked convolutions in one kernel: a convolution whose output tile can be held on chip, followed by a 1x1
 * convolution on its output -- the 3x3 -> 1x1 expansion that closes a ResNet bottleneck, or the two pointwise
 * layers of a ConvNeXt block:
 *     t = act1( conv_kxk(x; W1) + bias1 )          rounded to the 16-bit type, exactly as ss_conv2d_fwd would store it
 *     y = act2( conv_1x1(t; W2) + bias2 + residual ) = what ss_conv2d_res_fwd would compute from t
 * The intermediate t never leaves the compute unit's LDS, which saves its write and read (the results are those
 * of the two separate calls up to the order of the fp32 additions in the second one).
 *   desc1   the first layer, 16-bit dtype.  Either k x k with k > 1: cout % 32 == 0, cout <= 256, and SS_K_CRS with a
 *           3x3 kernel and cin % 32 == 0, or SS_K_RSC with cin % 8 == 0.  Or 1x1 (the inverted bottleneck of a
 *           ConvNeXt block, narrow -> wide -> narrow: the wide intermediate is produced and consumed 128 channels
 *           at a time): stride 1, no padding, cin % 32 == 0, cin <= 128, cout % 128 == 0 and cout <= 8192 (its bias sits in LDS), bias1 16-byte
 *           aligned, and desc2->cout <= 128.  Anything else: SS_ERR_UNSUPPORTED
 *   desc2   the 1x1 layer: same dtype, cin == desc1->cout, cout % 32 == 0
 *   packed1, packed2   written by ss_mask_compress for desc1 / desc2                         (read only)
 *   bias1   [desc1->cout] fp32 or NULL; bias2 [desc2->cout] fp32, 16-byte aligned, or NULL     (read only)
 *   residual [N][Ho][Wo][desc2->cout] 16-bit, 16-byte aligned, or NULL; may alias y            (read only)
 *   y       [N][Ho][Wo][desc2->cout], Ho / Wo from the k x k layer's stride and padding        (written)
 * Asynchronous on `stream`.
 */
int ss_conv2d_pw_fused_fwd(const ss_weight_desc *desc1, const void *x, int32_t N, int32_t H, int32_t Wd,
                           const void *packed1, const float *bias1,
                           int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act1,
                           const ss_weight_desc *desc2, const void *packed2, const float *bias2,
                           const void *residual, int32_t act2, void *y, void *stream);

/*
 * Would ss_conv2d_pw_fused_fwd (sparse != 0) or ss_conv2d_pw_fused_dense_fwd (sparse == 0) take this pair of layers,
 * and does the library expect the fused kernel to be faster than the two separate calls?  Answers from the
 * descriptors and the first layer's stride and padding alone; [host], touches no device.
 *   *supported  1 when the fused entry point accepts the pair (same conditions as listed there), else 0
 *   *pays       1 when, on the library's own measurements, the fused kernel beats the two calls: always for the
 *               1x1 -> 1x1 pair; for a k x k -> 1x1 pair while the first layer is at most 128 channels wide on the
 *               sparse path (64 on the dense twin).  A caller that chains layers fuses where pays is 1.
 * Returns SS_ERR_INVALID_ARG for null pointers, malformed descriptors, or a second layer that is not a 1x1
 * convolution on the first one's output channels.
 */
int ss_conv2d_pw_fused_query(const ss_weight_desc *desc1, int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                             const ss_weight_desc *desc2, int32_t sparse, int32_t *supported /*[host] out*/,
                             int32_t *pays /*[host] out*/);

/* The dense twin of ss_conv2d_pw_fused_fwd (operands built by ss_dense_pack). */
int ss_conv2d_pw_fused_dense_fwd(const ss_weight_desc *desc1, const void *x, int32_t N, int32_t H, int32_t Wd,
                                 const void *dense1, const float *bias1,
                                 int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act1,
                                 const ss_weight_desc *desc2, const void *dense2, const float *bias2,
                                 const void *residual, int32_t act2, void *y, void *stream);

/*
 * The masked convolution on 8-bit operands: Eq. (6) with every product and the running sum exact in
 * int32 (SS_I8), or with exact products summed in fp32 (SS_F8), followed by the dequantising layer tail
 *     y[n,ho,wo,o] = act( scale[o] * sum_k (M (.) W)[o,k] * U(X)[k,p] + bias[o] ),
 * evaluated in fp32 (an int32 sum is converted with round-to-nearest-even) and rounded once to the
 * output type.  The paper stops at 16-bit floats; this is the same method one precision step further,
 * on gfx950's V_SMFMAC_I32_32X32X64_I8 / V_SMFMAC_F32_32X32X64_FP8_FP8, which consume twice the
 * reduction length per instruction.
 *   desc    dtype SS_I8 or SS_F8; cin % 16 == 0; with korder SS_K_CRS and a kernel larger than 1x1 (a
 *           4-block then spans kernel taps, i.e. bytes of different pixels, which are transposed in
 *           registers) only 3x3 and 2x2 kernels with cin % 64 == 0 -- otherwise SS_ERR_UNSUPPORTED
 *   x       [N][H][Wd][cin] bytes of desc->dtype, 16-byte aligned                   (read only)
 *   packed  written by ss_mask_compress for this descriptor                         (read only)
 *   scale   [cout] fp32 or NULL (= 1): weight step * activation step of the quantiser (read only)
 *   bias    [cout] fp32 or NULL (= 0)                                               (read only)
 *   act     SS_ACT_NONE | SS_ACT_RELU | SS_ACT_GELU
 *   out_dtype  SS_F16 (the only one built; anything else SS_ERR_UNSUPPORTED)
 *   y       [N][Ho][Wo][cout] 16-bit, 16-byte aligned                               (written)
 *   SS_I8: |sum| must stay below 2^31: K * 128 * 128 < 2^31, i.e. K <= 131071 (else SS_ERR_UNSUPPORTED).
 *   SS_F8: a NaN byte propagates; sums beyond fp32 range cannot occur (K * 448^2 < 2^128).
 * Everything else (workspace, stream, errors) as for ss_conv2d_fwd.
 */
int ss_conv2d_q8_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                     const void *packed, const float *scale, const float *bias,
                     int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                     int32_t out_dtype, void *y, void *workspace, size_t ws_bytes, void *stream);

/* The dense twin of ss_conv2d_q8_fwd (V_MFMA_I32_32X32X32_I8, or V_MFMA_SCALE_F32_32X32X64_F8F6F4 with unit
 * scales, on the operand built by ss_dense_pack). */
int ss_conv2d_q8_dense_fwd(const ss_weight_desc *desc, const void *x, int32_t N, int32_t H, int32_t Wd,
                           const void *dense, const float *scale, const float *bias,
                           int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t act,
                           int32_t out_dtype, void *y, void *workspace, size_t ws_bytes, void *stream);

/*
 * Max pooling of NHWC 16-bit activations with a k x k window (the pooling between the stem and the
 * first residual block of the ResNet models of Sec. 4), so that a chained convolution stack stays
 * inside the library.  Positions outside the image do not take part (with 2*pad <= k every window
 * holds at least one pixel); the output element is the bit pattern of the largest input (-0 < +0 is
 * not distinguished: whichever comes first in row-major window order stays); a NaN wins.
 *   x  [N][H][Wd][C]    16-bit, dtype, 16-byte aligned, C % 8 == 0 (else SS_ERR_UNSUPPORTED)  (read only)
 *   y  [N][Ho][Wo][C]   Ho = (H + 2*pad - k) / stride + 1, same for Wo                      (written)
 * Asynchronous on `stream`.
 */
int ss_maxpool2d(const void *x, int32_t N, int32_t H, int32_t Wd, int32_t C, int32_t dtype, int32_t k,
                 int32_t stride, int32_t pad, void *y, void *stream);

/*
 * Depthwise convolution (one kh x kw filter per channel), stride 1: the grouped convolutions that
 * the paper leaves dense (Sec. 4, "Architectures"), e.g. the 7x7 of a ConvNeXt block, so that the
 * dense layers of such a block are measured next to its masked ones.
 *     y[n,h,w,c] = act( bias[c] + sum_{r,t} w[r][t][c] * x[n, h - pad_h + r, w - pad_w + t, c] )
 * fp32 accumulation, one rounding to the 16-bit type at the store.
 *   x     [N][H][Wd][C]   16-bit, dtype, 16-byte aligned                          (read only)
 *   w     [kh][kw][C]     16-bit, dtype (channel fastest), 16-byte aligned         (read only)
 *   bias  [C] fp32 or NULL                                                        (read only)
 *   act   SS_ACT_NONE | SS_ACT_RELU
 *   y     [N][Ho][Wo][C], Ho = H + 2*pad_h - kh + 1, Wo = Wd + 2*pad_w - kw + 1    (written)
 * SS_ERR_UNSUPPORTED unless C % 8 == 0, kw in {3, 5, 7} and kh*kw*C*2 <= 65536 bytes.
 * Asynchronous on `stream`.
 */
int ss_dwconv2d_fwd(const void *x, int32_t N, int32_t H, int32_t Wd, int32_t C, int32_t dtype, const void *w,
                    const float *bias, int32_t kh, int32_t kw, int32_t pad_h, int32_t pad_w, int32_t act,
                    void *y, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SS_H_ */
