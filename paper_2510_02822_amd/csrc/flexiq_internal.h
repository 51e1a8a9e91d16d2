// Internal definitions shared by the translation units of libflexiq (HIP side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "flexiq.h"

namespace flexiq {

// Channels are processed in "units" of 32 (the smallest group size of Section 7); a K-step of the
// matrix pipeline is two units = 64 reduction elements = two v_mfma_i32_32x32x32_i8 per pair of fragments.
constexpr int kUnit = 32;
constexpr int kNPadTo = 256;  // weight tiles are padded in N to the largest block tile

// Record a failed HIP call for flexiq_last_hip_error().
void set_hip_error(hipError_t e, const char *what);

// A failed HIP call ends the entry point: FLEXIQ_ENOMEM when the device is out of memory, FLEXIQ_EHIP otherwise.
#define FLEXIQ_HIP(call)                                                       \
    do {                                                                       \
        hipError_t e__ = (call);                                               \
        if (e__ != hipSuccess) {                                               \
            ::flexiq::set_hip_error(e__, #call);                               \
            return e__ == hipErrorOutOfMemory ? FLEXIQ_ENOMEM : FLEXIQ_EHIP;   \
        }                                                                      \
    } while (0)

// Once per device, when the first layer is packed on it: dynamic-LDS limits and occupancy of every kernel of the
// GEMM shape table, so that a launch is only a launch.
int prepare_kernels(int device);
int prepare_fp6_kernels(int device);
int prepare_stream_kernels(int device);
int prepare_conv3_kernels(int device);
int prepare_tile_splitk_kernels(int device);

// Order hash of a channel permutation (FNV-1a over the 32-bit entries; `n` entries, identity when p == nullptr).
inline uint64_t order_hash(const int32_t *p, int n)
{
    uint64_t h = 1469598103934665603ull;
    for (int i = 0; i < n; ++i) {
        uint32_t v = (uint32_t)(p ? p[i] : i);
        for (int b = 0; b < 4; ++b) {
            h ^= (v >> (8 * b)) & 0xFFu;
            h *= 1099511628211ull;
        }
    }
    return h;
}

// Limits of the GEMM kernel that depend on the layer alone (checked when it is packed, and again at launch).
constexpr int kMaxGroups = 159;                       // the kernel keeps the position table of G + 1 groups in LDS
// Scan words of a layer (run-time positions, d_scan; all zero between calls).  First the area a producing layer's GEMM
// epilogue uses: a ticket (alone in its 64-byte line) and kFusedScanRows rows of G group masks (a block ORs into row
// blockIdx.x % kFusedScanRows, so that the atomics of a launch spread over many addresses); then the area of the
// stand-alone scan kernel: its ticket and one row of partial masks per block.
constexpr int kScanHead = 16;
constexpr int kFusedScanRows = 8;
constexpr int kScanRowBlocks = 128;   // most blocks of the stand-alone scan along the rows (measured: 64 ... 128 is best)
inline size_t fused_scan_words(int G) { return (size_t)kScanHead + (size_t)kFusedScanRows * G; }
inline size_t scan_words_total(int G) { return ((fused_scan_words(G) + 15) & ~(size_t)15) + kScanHead + (size_t)kScanRowBlocks * G; }
inline size_t standalone_scan_offset(int G) { return (fused_scan_words(G) + 15) & ~(size_t)15; }
constexpr int64_t kMaxWeightBytes = 0x7fffffff;       // both int8 weight copies sit behind one buffer descriptor

}  // namespace flexiq

struct flexiq_layer;
namespace flexiq {
// Leading channels of the layer that run on the FP6 matrix path under its current ratio and positions (a multiple of 64).
int fp6_channels(const flexiq_layer *L);
// (smallm.hip) the same for flexiq_mixed_gemm_fp6: the leading K6 channels on the FP6 matrix path
int launch_few_rows_fp6(const flexiq_layer *L, const int8_t *X, const uint8_t *X6, int64_t M, const flexiq_out *out, void *stream, int K6,
                        int num_cu, int *taken);
// The consumer named by flexiq_out.lower_for, checked (gemm.hip): its positions, 4-bit prefix and log2 of its group size;
// ashift == nullptr: the call names none.
struct LowerArgs {
    const int32_t *ashift = nullptr;
    int32_t K4 = 0, gs_log2 = 5;
    // FP6 calls only (flexiq_out.x6, checked in fp6_gemm.hip): the consumer's FP6 activation buffer, its FP6 prefix and C / 64
    uint8_t *x6 = nullptr;
    int32_t K6 = 0, S = 0;
};
int lower_for_args(const flexiq_layer *L, const flexiq_out *out, LowerArgs *la);
// (smallm.hip) linear calls of more than 64 rows with few 64 x 64 tiles and a long reduction: a tile per block, the reduction
// split over its waves; *taken = 0: the call does not qualify
int launch_tile_splitk(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int num_cu, int *taken,
                       const LowerArgs *lower = nullptr);
int launch_tile_splitk_fp6(const flexiq_layer *L, const int8_t *X, const uint8_t *X6, int64_t M, const flexiq_out *out, void *stream, int K6,
                           int num_cu, int *taken, const LowerArgs *lower);
// (smallm.hip) linear calls with at most 64 rows: a block per 16 (or 8) output columns whose waves split the reduction
// and meet in LDS; *taken = 0: the call does not qualify.  X4: a producer's packed activation codes; lower: flexiq_out.lower_for
int launch_few_rows(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int num_cu, int *taken,
                    const uint8_t *X4 = nullptr, const LowerArgs *lower = nullptr);
// (stream.hip) the row-streaming kernels for layers with a short reduction; *taken = 0: the call does not qualify
int launch_stream(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, bool rows_contiguous, int *taken,
                  const uint8_t *X4 = nullptr, const LowerArgs *lower = nullptr);
// (conv3.hip) 3x3 convolutions, stride 1, padding 1, with 64 or 128 input channels: weights of all taps resident in LDS,
// image tiles streamed past them; *taken = 0: the call does not qualify
int launch_conv3(const flexiq_layer *L, const int8_t *X, int B, int H, int W, int stride, int pad, const flexiq_out *out, void *stream, int *taken,
                 const LowerArgs *lower = nullptr);
}  // namespace flexiq

// Device layouts (all offsets in bytes unless noted), T = R*S filter taps, CUp = C/32 rounded up to
// even, U = T * CUp units, unit u = tap * CUp + c32 (tap-major; a pad unit c32 == C/32 is all zero),
// Npad = N rounded up to 256, rows >= N are zero:
//   w8     int8  [U][2][Npad][16]   8-bit weights; plane q2 of unit u holds stored channels
//                                   c32*32 + q2*16 .. +15 of every output channel
//   w4     uint8 [U][Npad][16]      4-bit codes of the same 32 channels: dword e (0..3) of a row
//                                   carries channels 8e..8e+3 in the low halves of its bytes 0..3
//                                   and channels 8e+4..8e+7 in the high halves
//   w4x    int8  [U][2][Npad][16]   the same 4-bit codes, each put back at its extraction position as an
//                                   int8 value (code << wshift), in the layout of w8: the copy the matrix
//                                   kernel streams when the problem is compute-bound, so that no expansion
//                                   work shares the vector ALU with the matrix pipe.  w8 and w4x are the two
//                                   halves of one allocation (d_w4x = d_w8 + U*Npad*32): one buffer
//                                   descriptor reaches both
//   wshift uint8 [G+1][Npad]        weight extraction position per (group, output channel); row G is zero
//                                   (looked up by the pad unit)
//   ashift int32 [G+1]              activation extraction position per group (+1 entry for the pad unit);
//                                   a second table of the same shape holds the positions found at run time
//   scan   uint32 [G+1]             OR masks of the run-time scan per group, then a block counter; all zero
//                                   between calls (the scanning kernel, stand-alone or a producing layer's GEMM,
//                                   cleans up after itself)
//   cs     fp32  [2][Npad]          x_scale * w_scale[n], then the biases (zeros when the layer has none):
//                                   one allocation, d_bias = d_cs + Npad
struct flexiq_layer {
    int32_t N, C, R, S, group_size;
    int32_t G, T, U, Npad;
    int32_t max_4bit_ch;
    float x_scale;
    bool has_bias;
    std::vector<int32_t> perm;
    uint64_t perm_hash;        // of perm: the order in which this layer reads its input channels
    uint64_t out_order_hash;   // of out_perm (identity if none): the order in which it writes its output columns
    std::vector<uint8_t> a_shift, w_shift;
    std::vector<float> w_scale, bias;
    int device;
    int8_t *d_w8;
    uint8_t *d_w4;
    int8_t *d_w4x;
    uint8_t *d_wshift;
    int32_t *d_ashift;
    int32_t *d_ashift_dyn;
    uint32_t *d_scan;
    bool dynamic;   // GEMM / conv calls read d_ashift_dyn (written by the stand-alone scan kernel or by the
                    // epilogue of a producing layer's call) instead of d_ashift
    bool x_prelowered;   // the caller's activations are bit-lowered already (by the producing layer's epilogue)
    float *d_cs;
    float *d_bias;
    int32_t *d_perm;
    // FP6 copy of the 4-bit codes of all groups (linear layers with C a multiple of 64; null otherwise), for the variant
    // whose 4-bit groups run on the FP6 matrix path:
    //   w6   uint8 [C/64][3][Npad][16]  per K-step of 64 channels three 16-byte planes per output channel: planes 0 and
    //                                   1 hold the first 16 bytes of the 24-byte FP6 image of units 0 and 1, plane 2 the
    //                                   last 8 bytes of both (unit h in half h ^ ((n >> 4) & 1)); element e of a unit is
    //                                   the code of its channel 8 * ((e % 16) / 4) + 4 * (e / 16) + e % 4, as the 6-bit
    //                                   pattern sign << 5 | |code| (E2M3 value code / 8)
    //   w6s  uint8 [ceil(C/256)][Npad][2][4]  E8M0 block scales 127 + 3 + w_shift of (output channel, unit 0 / 1 of a K-step)
    //                                   for four consecutive K-steps: one 32-bit load per lane serves four steps
    uint8_t *d_w6;
    uint8_t *d_w6s;
    // Leading channels whose FP6 accumulation is certified exact (every partial sum below 2^24 in magnitude, from the
    // packed weights): with the calibrated activation positions, and with any positions (run-time scan).
    int32_t fp6_limit_static, fp6_limit_dynamic;
};
