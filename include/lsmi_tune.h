/*
 * lsmi - sweep controls and diagnostics.
 *
 * Not part of the compute boundary (lsmi.h): these calls exist for the tuning script
 * (the three-step sweep of Section 6.3, "Scripted Tuning") and for tests and benchmarks
 * that want to pin or report which kernel ran.  Every override is per calling thread and
 * changes only which kernel computes a call, never its result beyond the summation order.
 */
#ifndef LSMI_TUNE_H
#define LSMI_TUNE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Tuning override for the calling thread, for sweeps: a variant index >= 0 forces that
 * tile configuration (see lsmi_variant_name), -1 restores the built-in choice; split_k
 * >= 1 forces the number of K partitions (1: no tile is partitioned, results are then
 * reproducible from run to run), 0 restores the built-in choice.  Returns
 * LSMI_ERR_DIM for an unknown index.
 */
int lsmi_set_tuning(int sgemm_variant, int split_k);

/*
 * Order in which the workgroups of sgemm and of the direct-to-LDS igemm kernels walk the tiles of C
 * (the loop order of the two outer loops of Fig. 1, the second step of the tuning script of
 * Section 6.3): the tiles are taken down bands of band_rows tile rows, column by column inside a
 * band, so that the tiles in flight at one time share band_rows row panels of A and a few column
 * panels of B.  band_rows >= 1 forces it for the calling thread, 0 restores the built-in choice
 * (sgemm: 8 tile rows, 4 for 256-row tiles; igemm: 8, 2 for 256-row tiles).  Returns LSMI_ERR_DIM for
 * a negative value or one above 65535.
 */
int lsmi_set_tile_walk(int band_rows);

/*
 * The same for igemm_s8s32: kernel index >= 0 (names from lsmi_igemm_variant_name; a
 * direct-to-LDS kernel that does not fit the call's shape or alignment is ignored), -1
 * restores the built-in choice.  The split_k of lsmi_set_tuning applies to igemm_s8s32 as
 * well.  Returns LSMI_ERR_DIM for an unknown index.
 */
int lsmi_set_igemm_tuning(int igemm_variant);

/* Name of igemm_s8s32 kernel `index`, or NULL when index is out of range. */
const char *lsmi_igemm_variant_name(int index);

/*
 * The same for conv2d_nhwc: a tile configuration index >= 0 is forced for the
 * calling thread, -1 restores the built-in choice.  Returns LSMI_ERR_DIM for an unknown index.
 */
int lsmi_set_conv_tuning(int conv_variant);

/*
 * Number of slices the reduction over (r, s, c) of conv2d_nhwc is cut into (direct-to-LDS
 * kernels only): >= 1 forces it for the calling thread, 0 restores the built-in choice,
 * which splits only when the output has too few tiles to fill the GPU.  With more than
 * one slice the partial sums are combined with floating-point atomics, so the summation
 * order, hence the last bits of the result, can differ from run to run.  Returns
 * LSMI_ERR_DIM for a negative value.
 */
int lsmi_set_conv_split(int slices);

/*
 * Number of tile rows at the end of the pixel range of conv2d_nhwc that are computed as
 * quarter-tile pieces (32 x 32 outputs per workgroup, the reduction split over its waves and
 * summed in a fixed order) instead of whole tiles; four-wave direct-to-LDS kernels without a
 * split reduction only.  >= 0 forces it for the calling thread (clamped to the tile rows there
 * are; 0 = none), -1 restores the built-in choice, which hands over the tiles of a last round
 * that would fill at most half of the CUs.  Results stay deterministic.  Returns LSMI_ERR_DIM
 * for a value below -1.
 */
int lsmi_set_conv_tail(int tile_rows);

/* Name of conv2d_nhwc tile configuration `index`, or NULL when index is out of range. */
const char *lsmi_conv_variant_name(int index);

/*
 * The same for dwconv2d_nhwc: kernel index >= 0 (names from lsmi_dwconv_variant_name; an
 * index whose kernel does not fit the call's filter size, stride, channel count or
 * alignment is ignored), -1 restores the built-in choice; strip >= 1 forces the number of
 * output rows a lane (register-window kernels) or a workgroup (LDS-staged kernels) walks,
 * 0 restores the built-in choice.  Returns LSMI_ERR_DIM for an unknown index or a negative
 * strip.
 */
int lsmi_set_dwconv_tuning(int dwconv_variant, int strip);

/*
 * Tile override for the LDS-staged dwconv2d_nhwc kernels, calling thread only: output
 * columns per tile, channels per tile, and how many steps the loads run ahead (1 or 2);
 * 0 leaves a value to the built-in search.  A combination that does not fit the kernel's
 * limits makes the call fall back to another kernel.  Returns LSMI_ERR_DIM for negative
 * values or depth > 2.
 */
int lsmi_set_dwconv_tile(int cols, int channels, int depth);

/* Name of dwconv2d_nhwc kernel `index`, or NULL when index is out of range. */
const char *lsmi_dwconv_variant_name(int index);

/* Number of slices the reduction of the calling thread's last sgemm, sgemm_op, sgemm_ws or
 * sgemm_fused launch was cut into (1: not cut). */
int lsmi_last_split(void);

/* Name of sgemm tile configuration `index`, or NULL when index is out of range. */
const char *lsmi_variant_name(int index);

/*
 * Diagnostic, host only: the tile (row, column) that workgroup `wg` of a launch over a
 * tiles_m x tiles_n grid processes, using the same XCD-aware mapping as the kernels
 * (bands of `group_m` tile rows).  Returns LSMI_ERR_DIM unless 0 <= wg < tiles_m*tiles_n,
 * tiles_m, tiles_n, group_m >= 1 and the outputs are non-NULL.
 */
int lsmi_tile_of_workgroup(int wg, int tiles_m, int tiles_n, int group_m, int *tile_row,
                           int *tile_col);

/*
 * Diagnostic, host only: n / d as the kernels compute it for divisors fixed at launch (a high
 * multiply by the divisor's rounded-up reciprocal, an add and two shifts).  Exact for every
 * 32-bit unsigned n and d >= 1; d == 0 is taken as 1.
 */
uint32_t lsmi_fast_divide(uint32_t n, uint32_t d);

/*
 * Calibration, waits for its own kernels: the rate of a loop of matrix instructions on
 * registers alone (v_mfma_f32_32x32x2_f32, or v_mfma_i32_32x32x32_i8 when int8 != 0), four
 * workgroups of four waves per compute unit on the calling thread's stream, and the shader
 * clock during that loop (cycle counter against the constant 100 MHz counter).  With
 * random_operands != 0 the instructions rotate over eight register sets of pseudo-random
 * values, as a product of random matrices presents them; with 0 every instruction sees the
 * same registers.  This is the rate to hold a kernel's figure against besides the datasheet
 * peak.  device_words: caller-owned device memory of `words` 8-byte words, at least
 * 8 * compute units + 1 (LSMI_ERR_DIM otherwise); its contents are overwritten.  Results in
 * operations per second (2 per multiply-add) and Hz.  Errors: LSMI_ERR_NULL, LSMI_ERR_DIM,
 * LSMI_ERR_NO_DEVICE, LSMI_ERR_LAUNCH.
 */
int lsmi_mfma_rate(int int8, int random_operands, void *device_words, int64_t words,
                   double *ops_per_second, double *shader_clock_hz);

#ifdef __cplusplus
}
#endif
#endif /* LSMI_TUNE_H */
