/*
 * flexiq_test.h -- test and tuning aids of libflexiq.  Not part of the method and not needed by a user of
 * the library: the parity tests use them to force every code path of the GEMM kernel (each tile shape, each
 * weight route, blocks that walk several output tiles) on inputs small enough for the CPU oracle.
 *
 * All of them act on process-wide state that the launch path reads without synchronisation: call them only
 * while no flexiq call is in flight on any thread, and reset them (-1 / 0) afterwards.
 */
#ifndef FLEXIQ_TEST_H
#define FLEXIQ_TEST_H

#ifdef __cplusplus
extern "C" {
#endif

/* Force tile shape `index` of the kernel's shape table for every following GEMM / convolution call;
 * -1 = automatic choice (the default).  Returns the number of shapes in the table, or FLEXIQ_EINVAL. */
int flexiq_debug_force_tile(int index);

/* Where the kernel takes the weights of 4-bit channel groups from: 1 = the packed 4-bit codes (expanded in
 * registers), 0 = the position-expanded int8 copy, -1 = automatic (the default). */
int flexiq_debug_force_packed4(int mode);

/* Blocks launched by a GEMM / convolution call whose tile shape lets a block walk several output tiles:
 * 0 = automatic (one resident wave of blocks; the default), n > 0 = at most n blocks, n < 0 = one block per tile. */
int flexiq_debug_max_blocks(int n);

/* What the last GEMM / convolution launch used.  which = 0: tile shape index, 1: blocks launched,
 * 2: blocks of that kernel resident per compute unit. */
int flexiq_debug_last_launch(int which);

/* The few-row kernels (linear calls with at most 64 rows; last launch: tile shape index -4): 1 = the matrix-core kernel
 * whenever the call qualifies, 2 = the dot-product kernel (at most 4 rows) whenever it qualifies (14: with 4 groups of 8 columns per
 * block where the layer's padding allows), 0 = never, -1 = automatic.
 * Returns which of them the last call they were offered ran on (0: neither; 3: the matrix-core kernel's FP6 build, which
 * flexiq_mixed_gemm_fp6 takes for at most 64 rows unless an FP6 tile shape is forced or mode is 0).  While mode is not -1,
 * calls of at most 64 rows are also kept off the kernel of flexiq_debug_force_tile_splitk (so that 0 means "the tiled kernel"). */
int flexiq_debug_force_few_rows(int mode);

/* The kernel that gives a block one output tile and splits the reduction over its waves (linear calls of more than 64 rows with
 * few tiles and a long reduction; last launch: tile shape index -5): 1 = take it whenever the call qualifies (whatever the
 * tile count and reduction length), 2 / 3 / 4 = the same with tiles of 64 x 64 / 32 x 64 / 32 x 32 (rows x columns), 0 = never,
 * -1 = automatic (more than 32 rows, at most one 64 x 64 tile per compute unit, at least 12 K-steps of 64 channels).  Serves
 * flexiq_mixed_gemm and flexiq_mixed_gemm_fp6 (FP6 build; forced FP6 tile shapes go first; FP6 calls with lower_for at any row
 * count), from 17 rows when forced.
 * Returns the tile the last call it was offered ran on (1 / 2 / 3 in that order; 0: another kernel). */
int flexiq_debug_force_tile_splitk(int mode);

/* The row-streaming kernels for layers with 64, 128 or 256 input channels (last launch: tile shape index -2):
 * 1 / 2 = take the one whose blocks walk tiles of 128 rows / the one whose waves walk groups of 32 rows on their own,
 * whenever the layer form qualifies (whatever the row count), 0 = never, -1 = automatic.  Returns which of them the
 * last GEMM / convolution call ran on (0: neither). */
int flexiq_debug_force_stream(int mode);

/* The 3x3 convolution kernel for 64 or 128 input channels, stride 1, padding 1 (last launch: tile shape index -3):
 * mode 1 = take it whenever the layer form qualifies (whatever the tile count), 0 = never, -1 = automatic;
 * rows_per_tile > 0 forces the output rows of an image tile (0 = automatic).  Returns whether the last convolution call
 * ran on it. */
int flexiq_debug_force_conv3(int mode, int rows_per_tile);

/* Force tile shape `index` of the FP6-variant kernel's table (-1 = automatic).  Returns the table size. */
int flexiq_debug_force_fp6_tile(int index);

#ifdef __cplusplus
}
#endif
#endif /* FLEXIQ_TEST_H */
