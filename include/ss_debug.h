/*
 * ss_debug.h -- test hooks of the 2:4 sparse convolution library.  Not part of the product interface: nothing a
 * caller needs for correct results or for speed lives here.  The hooks exist so that tests can reach every kernel
 * variant the library would otherwise choose by problem size.
 */
#ifndef SS_DEBUG_H_
#define SS_DEBUG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Forces the workgroup tile of the convolution entry points (ss_conv2d_*_fwd) to the kernel variant with this id
 * for all later calls of the process; a negative id returns the choice to the library.  Ids: 0-5 the one-tile-per-
 * workgroup shapes (64x64 shallow / deep, 128x64 shallow, 256x64 deep, 128x64 and 256x64 with producer waves);
 * 10 / 11 the resident-grid 3x3 kernel with 256x128 / 256x64 tiles; 12 the dense 7x7 first-layer kernel; 13 the
 * activation-stationary 1x1 kernel.  Ids the problem has no kernel for fall back to the library's choice; with an
 * id of 10 or more no split of the reduction is planned.  Process-wide, read with a relaxed atomic load at every
 * launch; meant for single-threaded tests.  Always returns SS_OK.  [host]
 */
int ss_debug_force_tile(int32_t id);

/*
 * Forces the number of workgroups that share one output tile of the 16-bit convolutions, each taking a share of the
 * reduction (see ss_conv2d_workspace_bytes); the value is clamped to the number of reduction chunks, and layers whose
 * staging mode does not split ignore it.  (With the activation-stationary 1x1 kernel forced, the value is instead the
 * number of workgroups that share a pixel tile, each taking a share of the output channels; no workspace is involved.)
 * 0 or a negative value returns the decision to the library.  The workspace
 * query answers for the forced value, so query after forcing.  Process-wide, as above.  Always returns SS_OK.  [host]
 */
int ss_debug_force_split(int32_t n);

/*
 * Caps the number of workgroups the resident-grid convolution kernels launch (they normally launch one per compute
 * unit and let each walk over several output tiles); 0 or a negative value removes the cap.  With a small cap a small
 * test problem exercises the tile-to-tile hand-over that otherwise only large problems reach.  Process-wide, as
 * above.  Always returns SS_OK.  [host]
 */
int ss_debug_limit_blocks(int32_t n);

/*
 * Calibration probe: measures the rate at which the chip issues the matrix instruction of the 16-bit kernels
 * (sparse != 0: the 2:4-sparse 32x32x32 instruction, else the dense 32x32x16 one; dtype SS_F16 or SS_BF16) with
 * operands and accumulators in registers only, two waves per SIMD on every compute unit, and writes it to *tflops
 * [host] in dense-equivalent TFLOP/s.  `scratch` is device memory of at least 2048 bytes per compute unit (512 KiB
 * on MI355X) that the probe may overwrite.  Waits for the stream.  SS_ERR_WORKSPACE when `scratch` is too small.
 */
int ss_debug_issue_peak(int32_t dtype, int32_t sparse, void *scratch, size_t scratch_bytes, float *tflops, void *stream);

/*
 * Calibration probe: LDS bandwidth of one compute unit in GB/s (divide by the clock in GHz for bytes per clock),
 * with one workgroup per compute unit and `waves_per_simd` (1, 2 or 4) waves per SIMD, each issuing eight independent
 * 16-byte-per-lane instructions between waits.  write == 0: reads in the convolution kernels' fragment pattern over
 * pixel rows of `row_bytes` (a multiple of 16, at most 592); write == 1: lane-linear 16-byte writes; write == 2 / 3:
 * the same bytes as 8-byte / 4-byte writes; write == 4: even waves read, odd waves write 16 bytes per lane (the sum of
 * both is reported).  `scratch` as for
 * ss_debug_issue_peak, 4096 bytes per compute unit.  Waits for the stream.
 */
int ss_debug_lds_bandwidth(int32_t write, int32_t waves_per_simd, int32_t row_bytes, void *scratch, size_t scratch_bytes,
                           float *gb_per_s_per_cu, void *stream);

#ifdef __cplusplus
}
#endif

#endif
