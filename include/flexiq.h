/*
 * flexiq.h -- C ABI of the gfx950 (MI355X) FlexiQ hot path: channel-level mixed 4-bit / 8-bit
 * quantized GEMM and implicit-GEMM convolution (arXiv 2510.02822).
 *
 * Conventions
 *   - Every function returns FLEXIQ_OK (0) or a negative flexiq_status; nothing throws or aborts.
 *     flexiq_strerror() names a code; after FLEXIQ_EHIP, flexiq_last_hip_error() gives the HIP text.
 *   - "host" / "dev" in a comment says where a pointer must live.  Device pointers are the caller's
 *     (e.g. torch tensors); the library never frees or reallocates them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device work of the
 *     run-time entry points is asynchronous on it; they never synchronise and never allocate.
 *   - Input channels are handled in "stored order": the permutation chosen offline (small-range
 *     channels first).  Activations are expected already in stored order, as the paper arranges by
 *     reordering the previous layer's output channels (Section 5, steps 1-2);
 *     flexiq_permute_channels() is the run-time reorder operator of Section 5, step 3.
 *   - A layer handle may be used from one stream at a time; flexiq_set_ratio() must not run
 *     concurrently with a launch on the same handle.
 */
#ifndef FLEXIQ_H
#define FLEXIQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FLEXIQ_OK = 0,
    FLEXIQ_EINVAL = -1, /* null pointer, bad shape, ratio outside [0,1], C not a multiple of group_size ... */
    FLEXIQ_EALIGN = -2, /* a device pointer is not 16-byte aligned */
    FLEXIQ_ENOMEM = -3, /* host or device allocation failed (offline entry points only) */
    FLEXIQ_EHIP = -4    /* a HIP runtime call failed; see flexiq_last_hip_error() */
} flexiq_status;

const char *flexiq_strerror(int status);
const char *flexiq_last_hip_error(void);

/* Opaque packed layer.  Owns (device) the permuted int8 weights, the cached packed 4-bit copy of
 * every channel group, the extraction positions and the scales, and (host) copies of the small
 * tables.  One handle serves every low-bit ratio: nothing is repacked when the ratio changes
 * (Section 7, "Low-bitwidth Ratio Adjustment"). */
typedef struct flexiq_layer flexiq_layer;

/* Description of one linear (R = S = 1) or convolution layer to quantise and pack.
 * Problem statement of Section 2.3: C feature channels, a low-bit subset chosen per target ratio. */
typedef struct {
    int32_t N;               /* output channels */
    int32_t C;               /* input (feature) channels; reduction length K = R*S*C */
    int32_t R, S;            /* filter height, width (1,1 for a linear layer) */
    int32_t group_size;      /* channels per same-bitwidth group: 32 or 64 (Sections 4.2, 7); C % group_size == 0 */
    const float *W;          /* host fp32 [N][R][S][C], channels in ORIGINAL order */
    const float *act_absmax; /* host fp32 [C]: calibration max|x| of each input channel, ORIGINAL order (Section 4.2) */
    float x_scale;           /* per-tensor activation scale S of Eq. 1 */
    const int32_t *perm;     /* optional host int32 [C]: stored position -> original channel.  NULL: ascending
                                error-estimation score (Section 4.2), ties by original index */
    const float *bias;       /* optional host fp32 [N] */
    const int32_t *out_perm; /* optional host int32 [N]: output column j of this layer = original output channel
                                out_perm[j].  Set it to the NEXT layer's stored channel order (its `perm`) and this
                                layer writes its outputs directly in the order the next layer reads them: the static
                                reordering of Section 5, steps 1-2 (only residual paths need the run-time
                                flexiq_permute_channels).  Every per-output-channel table of the handle (w_scale,
                                w_shift, dumps) is then indexed by output column.  NULL: original order */
} flexiq_pack_desc;

/* Offline steps (Eq. 1; Sections 4.1, 4.2, 5): per-output-channel symmetric int8 quantisation of W,
 * channel scores and order, channel groups, extraction positions a_shift[g] (from the calibration
 * ranges) and w_shift[n][g] (from the quantised weights, over all filter taps), permuted int8 weight
 * tiles and the packed 4-bit bit-lowered copy.  Runs HIP kernels on the current device and
 * synchronises; allocates device memory owned by the handle (FLEXIQ_ENOMEM when the device has none left).  Also
 * prepares the GEMM kernels for the current device once (dynamic-LDS limits, occupancy), so that the run-time entry
 * points only launch.  *out is set only on success.
 * Limits, refused with FLEXIQ_EINVAL before any device work: more than 159 channel groups (C / group_size); a padded
 * weight matrix (R*S*C rounded up to 64 per tap, times N rounded up to 256) of 1 GiB or more. */
int flexiq_quantize_pack(const flexiq_pack_desc *desc, flexiq_layer **out);

/* Releases the handle and its device memory.  NULL is accepted. */
int flexiq_layer_free(flexiq_layer *layer);

/* Read-only views of the handle's host tables (valid until flexiq_layer_free); any out pointer may be NULL.
 *   perm      int32 [C]        stored position -> original channel
 *   a_shift   uint8 [G]        activation extraction position per group, G = C / group_size
 *   w_shift   uint8 [N][G]     weight extraction position per (output channel, group)
 *   w_scale   fp32  [N]        per-output-channel weight scale
 *   G         number of channel groups;  max_4bit_ch: current count of 4-bit channels (Section 7) */
int flexiq_layer_info(const flexiq_layer *layer, const int32_t **perm, const uint8_t **a_shift,
                      const uint8_t **w_shift, const float **w_scale, int32_t *G, int32_t *max_4bit_ch);

/* Test aid for Section 7, "Low-bitwidth Ratio Adjustment" (one stored copy serves every ratio, nothing is
 * repacked between calls): copies the handle's device buffers back for inspection.
 *   w8 : host int8  [N][R*S][C]    permuted 8-bit weights, decoded from the tiled device layout
 *   w4 : host uint8 [N][R*S][C/2]  4-bit codes of ALL groups, channel c in byte c/2 (low half for even c)
 *   w4x: host int8  [N][R*S][C]    the copy of those codes that the matrix kernel streams for compute-bound
 *                                  shapes: every code put back at its extraction position, code << w_shift
 * Any may be NULL.  Synchronises the device. */
int flexiq_layer_dump(const flexiq_layer *layer, int8_t *w8, uint8_t *w4, int8_t *w4x);

/* Run-time ratio switch (Section 7): sets max_4bit_ch = group_size * ceil(r * G), the number of
 * leading stored channels computed at 4 bits.  Host-only, O(1): one integer in the handle, passed to
 * the next launch as a kernel argument.  r must lie in [0,1].  *max_4bit_ch (optional) gets the value. */
int flexiq_set_ratio(flexiq_layer *layer, float r, int32_t *max_4bit_ch);

/* Eq. 1 on the producer side: q[i] = clip(round_half_even(x[i] / scale), -127, 127).
 * x: dev fp32 [n], q: dev int8 [n]. */
int flexiq_quantize_act(const float *x, int8_t *q, int64_t n, float scale, void *stream);

/* Effective-bit extraction (Section 4.1) as a stand-alone kernel:
 * src dev int8 [rows][C]  ->  dst dev uint8 [rows][C/2]; channel c goes to byte c/2, low half for even c,
 * as a two's-complement 4-bit code clamp((v >> s), -8, 7), s = shifts[row][c/group_size] if per_row
 * else shifts[c/group_size].  shifts: dev uint8, values 0..4.  mode bit 0: 0 = truncate (the method),
 * 1 = round half up before the shift (variant). */
int flexiq_bitlower(const int8_t *src, uint8_t *dst, int64_t rows, int32_t C, int32_t group_size,
                    const uint8_t *shifts, int per_row, int mode, void *stream);

/* Extraction positions of the activations found at run time (Section 4.1, the dynamic option; Section 9
 * "Finding extraction positions at runtime"): for every channel group that is computed at 4 bits under the
 * handle's current ratio, the magnitude bits of all its values in X (ones' complement for negative values) are
 * OR-ed together; with p the highest set bit the position is max(0, p - 2).  Groups beyond the 4-bit range keep
 * their calibrated position.  The result stays on the device, in the handle, and every later
 * flexiq_mixed_gemm / flexiq_mixed_conv_implicit call on the handle uses it until flexiq_static_positions() or
 * the next scan; the scan is ordered on `stream` like any kernel (call it on the stream of the GEMM, with the
 * activations the GEMM will read).  After flexiq_set_ratio() raises the ratio, scan again.
 *   X    : dev int8 [rows][C], channels in stored order (rows = tokens, or B*H*W pixels of an NHWC tensor), 16-byte aligned
 * One kernel, no allocation, no host synchronisation.  rows == 0: every scanned group gets position 0. */
int flexiq_dynamic_positions(flexiq_layer *layer, const int8_t *X, int64_t rows, void *stream);

/* flexiq_dynamic_positions() for callers that cannot allocate or must not depend on allocations made elsewhere
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same scan with the same
 * result, but its scratch (one OR mask per channel group and a block counter) lives in a file-scope device array of
 * the library, 160 32-bit words per GPU, instead of the handle's allocation.  Calls no hipMalloc / hipFree and no
 * allocating routine.  Limit: G + 1 <= 160 channel groups, else FLEXIQ_EINVAL.  All calls on one GPU share that
 * array: two calls of this function that overlap on one GPU (different streams, different handles) race; calls on
 * one stream are ordered and each leaves the array zero for the next.  The handle's device must be current. */
int flexiq_dynamic_positions_static(flexiq_layer *layer, const int8_t *X, int64_t rows, void *stream);

/* Tells the handle that the activations handed to flexiq_mixed_gemm / flexiq_mixed_conv_implicit are bit-lowered
 * already for its current ratio and positions (written by the producing layer with flexiq_out.lower_for): the
 * kernel then copies them like 8-bit activations and only the weights of the 4-bit groups differ.  Host-side
 * switch, O(1); on != 0 enables.  The caller keeps producer and consumer settings consistent. */
int flexiq_input_prelowered(flexiq_layer *layer, int on);

/* Back to the calibrated positions of flexiq_quantize_pack, the static option of Section 4.1 (positions assigned
 * per feature channel group from calibration ranges).  Host-side switch, O(1). */
int flexiq_static_positions(flexiq_layer *layer);

/* Test aid for Section 4.1 (static and dynamic extraction positions): copies the activation positions that the
 * next GEMM / conv call would use to the host.
 *   a_shift : host uint8 [G].  Synchronises the device. */
int flexiq_layer_positions(const flexiq_layer *layer, uint8_t *a_shift);

/* Section 5 step 3, the residual reorder operator: dst[row][j] = src[row][perm[j]] for every row.
 * src, dst: dev int8 [rows][C]; uses the handle's permutation. */
int flexiq_permute_channels(const flexiq_layer *layer, const int8_t *src, int8_t *dst, int64_t rows, void *stream);

/* Outputs of a GEMM / conv call; any subset may be NULL (at least one must be set).
 *   acc : dev int32 [M][N]  raw accumulators (parity / debugging)
 *   y   : dev fp32  [M][N]  y = float(acc) * (x_scale * w_scale[n]) + bias[n]
 *   q   : dev int8  [M][N]  next layer's input, clip(round(y / out_scale), -128, 127), decided in fp32 in offset
 *                           form: clip(round_half_even(fma(float(acc), m[n], b[n])), 0, 255) - 128 with
 *                           m[n] = (x_scale*w_scale[n]) * (1/out_scale), b[n] = bias[n] * (1/out_scale) + 128,
 *                           every operation a correctly rounded fp32 one
 *   out_scale : scale of q (used only when q != NULL; must be > 0)
 *   lower_for : optional.  The layer that will consume q (its C == this layer's N, and this layer was packed
 *               with out_perm = that layer's stored channel order).  The codes of the columns that are 4-bit
 *               channels of the consumer under ITS current ratio are then written bit-lowered at ITS current
 *               positions, L(v, s) << s (Section 4.1), in the same pass: the consumer, switched with
 *               flexiq_input_prelowered(consumer, 1), no longer lowers them itself.  Both settings of the consumer
 *               are read when this call is made.  FLEXIQ_EINVAL unless this layer's out_perm equals the consumer's
 *               stored channel order (compared by hash).  NULL: plain int8 codes
 *   scan_for  : optional, not together with lower_for.  The layer that will consume q (same conditions).  The
 *               run-time scan of flexiq_dynamic_positions (Section 4.1; Section 9 "Finding extraction positions at
 *               runtime") is done on q in the same pass: every block ORs the magnitude bits of the codes it writes
 *               per channel group of the consumer, and the block that finishes last leaves the consumer's run-time
 *               positions for its 4-bit groups (its ratio when this call is made) and switches it to them, exactly
 *               as flexiq_dynamic_positions(consumer, q, M) would, without a second kernel.  Uses the consumer's scan
 *               scratch, which the kernel leaves clean (safe to replay from a captured graph): calls that scan for
 *               the same consumer must not overlap, nor overlap its flexiq_dynamic_positions.  A call with M == 0
 *               launches nothing and leaves the positions as they were.  NULL: no scan
 *   x6        : optional, only with lower_for and only for flexiq_mixed_gemm_fp6 (FLEXIQ_EINVAL elsewhere): the
 *               consumer's FP6 activation buffer (flexiq_fp6_bytes(consumer, M) bytes).  The columns that are FP6
 *               channels of the consumer (flexiq_fp6_channels) are then written there as FP6 codes instead of into q;
 *               q keeps the other columns (those of its remaining 4-bit channels lowered).  Needs N % 64 == 0
 *   x4        : optional, with lower_for on a linear consumer and q (flexiq_mixed_gemm / flexiq_mixed_conv_implicit): dev
 *               pointer to the consumer's packed 4-bit activation buffer (flexiq_packed4_bytes(consumer, M) bytes).  The
 *               columns that are packed channels of the consumer (flexiq_packed4_channels) are then written there as
 *               4-bit codes instead of into q; q keeps the other columns.  Needs N % 32 == 0 */
typedef struct {
    int32_t *acc;
    float *y;
    int8_t *q;
    float out_scale;
    const flexiq_layer *lower_for;
    flexiq_layer *scan_for;
    uint8_t *x6;
    uint8_t *x4;
} flexiq_out;

/* Mixed-precision GEMM (Sections 2.3, 7):
 *   acc[m][n] = sum_{g < G4} 2^(a_shift[g]+w_shift[n][g]) * sum_{k in g} L(X[m][k], a_shift[g]) * L(W[n][k], w_shift[n][g])
 *             + sum_{k >= max_4bit_ch} X[m][k] * W[n][k],          L(v, s) = clamp(v >> s, -8, 7)
 * with G4 = max_4bit_ch / group_size as last set by flexiq_set_ratio (0 after packing).
 * X: dev int8 [M][C] row-major, channels in stored order, 16-byte aligned; M >= 0 (M == 0 is a no-op).
 * The activations are bit-lowered on the fly inside the kernel, at the handle's current positions (calibrated, or
 * those of the last flexiq_dynamic_positions scan); the weights of 4-bit groups are read from the handle's cached
 * lowered copies.  Layer must be linear (R = S = 1).  Which kernel serves the call (tiled, row-streaming for at most 256
 * channels, the few-row kernels for at most 64 rows) follows from the shape; the int32 sums are the same bit for bit.
 * Launches on `stream`; allocates nothing; returns before the kernel has run.  Errors: FLEXIQ_EINVAL (null / inconsistent arguments, M >= 2^31 - 512, more than 159 channel
 * groups, a padded weight matrix of 1 GiB or more, current device is not the handle's), FLEXIQ_EALIGN, FLEXIQ_EHIP. */
int flexiq_mixed_gemm(const flexiq_layer *layer, const int8_t *X, int64_t M, const flexiq_out *out, void *stream);

/* The same sum as an implicit GEMM over (filter tap, channel) for a convolution layer:
 * X: dev int8 NHWC [B][H][W][C], stored channel order, zero padding `pad`, stride `stride`;
 * outputs are [B][Ho][Wo][N] with Ho = (H + 2*pad - R)/stride + 1 (likewise Wo).
 * The channel groups, a_shift and the 4-bit prefix are the same for every tap.
 * Further limit: H*W*C * (320 / (Ho*Wo) + 2) must be below 2^31 bytes (a block reads its images through a 2 GiB window). */
int flexiq_mixed_conv_implicit(const flexiq_layer *layer, const int8_t *X, int32_t B, int32_t H, int32_t W,
                               int32_t stride, int32_t pad, const flexiq_out *out, void *stream);

/* ---- 4-bit activations in packed form (Section 4.1: the bit-lowered activations, stored two codes per byte; Section 7
 * "Resource Consumption" caches extracted 4-bit values for the weights, this does the same for a tensor that one layer
 * writes and the next one reads).  Linear layers.  Where a layer is bound by memory traffic the ratio then saves
 * activation bytes as well: the leading flexiq_packed4_channels() stored channels (the 4-bit channels of the current ratio,
 * cut to whole K-steps of 64) are read from the packed buffer, everything else from X.  Same result, bit for bit, as
 * flexiq_mixed_gemm. */

/* Leading stored channels read in packed form under the handle's current ratio (a multiple of 64; 0 for convolutions and
 * for handles whose input arrives lowered). */
int flexiq_packed4_channels(const flexiq_layer *layer, int32_t *k4p);

/* Bytes of the packed buffer for M rows: M * C / 2 (negative flexiq_status on error).  Row m starts at byte m * C / 2; the
 * sixteen channels 16 p .. 16 p + 15 of a row are the eight bytes at 8 p: in dword e (little endian) byte b holds the code
 * of channel 16 p + 8 e + b in its low half and the code of channel 16 p + 8 e + 4 + b in its high half (two's
 * complement, L(v, s) & 15).  Only the first flexiq_packed4_channels() / 2 bytes of a row are read or written. */
int64_t flexiq_packed4_bytes(const flexiq_layer *layer, int64_t M);

/* Stand-alone producer of that buffer from X (dev int8 [M][C], stored channel order) with the handle's current ratio and
 * positions.  One kernel, no allocation. */
int flexiq_lower_packed4(const flexiq_layer *layer, const int8_t *X, int64_t M, uint8_t *x4, void *stream);

/* flexiq_mixed_gemm with the leading flexiq_packed4_channels() channels taken from x4 (dev, flexiq_packed4_bytes(layer, M)
 * bytes, 16-byte aligned, M * C / 2 < 2^31); those columns of X are not read.  Other 4-bit channels (a trailing group of 32)
 * are lowered on the fly from X as usual.  Launch only; no allocation. */
int flexiq_mixed_gemm_packed4(const flexiq_layer *layer, const int8_t *X, const uint8_t *x4, int64_t M, const flexiq_out *out,
                              void *stream);

/* ---- Variant of the 4-bit phase on the FP6 matrix path (Section 7: the low-bit groups on a faster matrix
 * instruction; on gfx950 that instruction is the FP8/FP6/FP4 MFMA with block scales, since no 4-bit integer MFMA
 * exists).  Same result, bit for bit, as flexiq_mixed_gemm: a 4-bit code L(v, s) in [-8, 7] is the exact FP6 (E2M3)
 * value code / 8, and the block scale 2^(s+3) per 32 channels is the extraction shift.  Linear layers with
 * C % 64 == 0 only.  The leading flexiq_fp6_channels() stored channels run as FP6: the 4-bit channels of the current
 * ratio, cut to a multiple of 64 and to the prefix for which exact fp32 accumulation is certified from the packed
 * weights and the positions in use (every partial sum below 2^24); remaining 4-bit channels run on the int8 path. */

/* Leading stored channels that run as FP6 under the handle's current ratio and positions (a multiple of 64). */
int flexiq_fp6_channels(const flexiq_layer *layer, int32_t *k6);

/* Bytes of the FP6 activation buffer for M rows: ceil(M / 64) * (C / 64) * 3072 (negative flexiq_status on error).
 * Layout [row / 64][K-step of 64 channels][plane 0..2][row % 64][16 bytes]: planes 0 and 1 hold the first 16 bytes of
 * the 24-byte image of the K-step's two 32-channel units, plane 2 the last 8 bytes of both (unit h in half
 * h ^ ((row >> 4) & 1)); element e (6 bits, little-endian bit order) of a unit is the code of its channel
 * 8 * ((e % 16) / 4) + 4 * (e / 16) + e % 4, as sign << 5 | |code|. */
int64_t flexiq_fp6_bytes(const flexiq_layer *layer, int64_t M);

/* Stand-alone producer of that buffer (Section 4.1 bit-lowering of the activations, then the FP6 pattern):
 *   X    : dev int8 [M][C], stored channel order
 *   x6   : dev, flexiq_fp6_bytes(layer, M) bytes; K-steps below flexiq_fp6_channels() / 64 are written (rows of the last
 *          block beyond M are not)
 *   xlow : dev int8 [M][C] or NULL: copy of X whose 4-bit channels outside the FP6 prefix are lowered in place
 *          (L(v, s) << s); required when flexiq_fp6_channels() is smaller than max_4bit_ch, else X itself can be
 *          handed to flexiq_mixed_gemm_fp6
 * Uses the handle's current ratio and positions.  Two kernels at most, no allocation. */
int flexiq_lower_fp6(const flexiq_layer *layer, const int8_t *X, int64_t M, uint8_t *x6, int8_t *xlow, void *stream);

/* The mixed GEMM with the FP6 prefix on v_mfma_scale_f32_32x32x64_f8f6f4 (twice the int8 matrix rate) and everything
 * else on the int8 MFMA, same accumulators: acc, y, q as for flexiq_mixed_gemm (out->scan_for is not supported).
 *   X  : dev int8 [M][C]; columns below flexiq_fp6_channels() are not read; 4-bit columns beyond it must arrive lowered
 *        (flexiq_lower_fp6's xlow, or a producer's lower_for); may be NULL when every channel is FP6
 *   x6 : dev FP6 activations (flexiq_lower_fp6, or a producer's flexiq_out.x6); may be NULL when no channel is FP6
 * Launch only; no allocation.  Further limit: flexiq_fp6_bytes(layer, M) < 2^31. */
int flexiq_mixed_gemm_fp6(const flexiq_layer *layer, const int8_t *X, const uint8_t *x6, int64_t M, const flexiq_out *out,
                          void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXIQ_H */
