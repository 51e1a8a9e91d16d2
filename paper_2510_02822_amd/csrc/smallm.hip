// Few-row calls of the mixed GEMM (at most 64 activation rows): the regime in which the call is a stream of the
// weight matrix and little else, i.e. the one place where the integer path on gfx950 moves fewer bytes as the
// low-bit ratio rises (Section 7: 4-bit groups move half the weight bytes).
//
// The tiled kernel launches one block per 64 x 64 output tile here: 16 to 64 blocks on 256 compute units, each
// walking the whole reduction alone.  The two kernels below give a block a few output columns and split the reduction
// over its waves, which meet in LDS.  Weights never go through LDS: the packed weight layouts hold 16-channel pieces of
// a weight row contiguously, which is both the MFMA fragment order and what a dot-product lane wants, so a lane loads
//   * 8-bit units: 16 bytes from the 8-bit tiles;
//   * 4-bit units: 16 bytes from the position-expanded copy, or 8 bytes of packed 4-bit codes (half the bytes) plus one
//     position byte.
// k_few_rows (3 .. 64 rows) feeds the matrix cores as the tiled kernel does: 4-bit units from the position-expanded int8 copy
// (16 bytes per lane like 8-bit units), their activations bit-lowered (same int8 MFMA, same int32 sums).
// k_few_rows_dot (1 .. 4 rows) multiplies on the vector ALU, 4-bit units as the packed 4-bit codes (Section 7's shifted
// accumulation): the kernel for calls that are bound by weight bytes.
// Both give the tiled kernel's results bit for bit.
#include <algorithm>

#include "flexiq_internal.h"

namespace flexiq {
namespace smallm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef short v2s __attribute__((ext_vector_type(2)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// clamp(v, -(8 << s), (8 << s) - 1) with the low s bits cleared, on the four int8 lanes of a dword: the bit-lowered
// value L(v, s) put back at its position (Section 4.1)
__device__ __forceinline__ uint32_t lower4(uint32_t d, int s)
{
    const short lo = (short)((-(8 << s)) << 8), hi = (short)((((8 << s) - 1) << 8) | 0xFF);
    const v2s lo2 = {lo, lo}, hi2 = {hi, hi};
    v2s o = __builtin_bit_cast(v2s, d);   // odd bytes sit on top of the 16-bit halves
    v2s e = o << (short)8;                // even bytes moved up
    o = __builtin_elementwise_min(__builtin_elementwise_max(o, lo2), hi2);
    e = __builtin_elementwise_min(__builtin_elementwise_max(e, lo2), hi2);
    const uint32_t r = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u);
    return r & (0x01010101u * ((0xFFu << s) & 0xFFu));
}

// ---- A block owns 16 output columns and the whole reduction.
//
// Splitting the reduction across blocks makes the slices meet in memory (store, ticket, re-read: three dependent trips;
// built and measured: ViT-L fc2 with 16 rows took 11 us that way, 4.7 us this way).  Here the slices of a column tile are
// the waves of one block (up to sixteen), which meet in LDS: every wave takes the K-steps (64 channels) wave,
// wave + waves, ... of the block's 16 columns, issues the loads of up to four of them at once
// (weight fragments straight into MFMA operand registers: 16 bytes per lane), multiplies with `v_mfma_i32_16x16x64_i8` (lane: weight row
// n0 + lane % 16 resp. activation row 16 f + lane % 16, channels 16 (lane / 16) ... of the K-step) and leaves its
// accumulators in LDS; waves 0 .. MF-1 add them up and run the epilogue of one 16-row fragment each.  One trip to memory
// for the operands and one for the outputs; nothing to zero, nothing to hand in.
struct RowsParams {
    const int8_t *X;        // int8 [M][C], stored channel order
    const int8_t *W8;       // [U][2][Npad][16]
    int32_t w4x_delta;      // bytes from the 8-bit tiles to the position-expanded copy of every 4-bit group (same layout)
    const uint8_t *W4;      // [U][Npad][16] packed 4-bit codes                  (k_few_rows_dot)
    const uint8_t *wshift;  // [G + 1][Npad] weight positions                    (k_few_rows_dot)
    const int32_t *ashift;  // [G + 1]
    const float *cs;        // [2][Npad]: x_scale * w_scale, then bias
    int32_t *acc;
    float *y;
    int8_t *q;
    float r_out;
    int32_t M, N, Npad, C;
    int32_t units;          // C / 32
    int32_t units4;         // leading units computed at 4 bits
    int32_t x_pre;          // activations of those units arrive lowered
    int32_t gs_shift;
    int32_t steps;          // K-steps of 64 channels (the last one may hold a single unit)
    // FP6 builds of k_few_rows (the variant of the 4-bit phase on the f8f6f4 matrix path, fp6_kernel.h): the leading s6 K-steps
    // come as FP6 codes, 24 bytes per (row, 32-channel unit), in the layouts of that kernel
    const uint8_t *X6;      // activations [ceil(M/64)][C/64][3][64][16]
    const uint8_t *W6;      // weights [C/64][3][Npad][16]
    const uint8_t *W6S;     // weight block scales [ceil(C/256)][Npad][2][4] (E8M0 bytes of four consecutive K-steps)
    int32_t s6;             // K-steps on the FP6 path (K6 / 64)
    // optional: the layer that reads the int8 output (flexiq_out.lower_for): its positions, 4-bit prefix, log2 of its group size;
    // the codes of its 4-bit channels then leave clamped and masked at its positions (Section 4.1 applied at the producer)
    const int32_t *next_ashift;
    int32_t next_K4, next_gs_log2;
    uint8_t *nx6;           // optional (k_tile_splitk, FP6 calls): the consumer's FP6 activation buffer; its leading next_K6 channels
    int32_t next_K6, next_S;   //   leave as FP6 codes as well (next_S = its C / 64)
    const uint8_t *X4;      // optional (k_few_rows_dot): packed activation codes [M][C / 2] of the leading pieces_p pieces of a row
    int32_t pieces_p;       // 16-channel pieces whose codes come from X4 (a multiple of 4: whole K-steps)
};

constexpr int kRowCols = 16;   // output columns per block

// MF: 16-row fragments of activations (M <= 16 MF).  COOP (MF = 1, at most 8 rows, activations not lowered yet): the 4-bit
// channels of the rows are lowered once per block into LDS instead of per lane in fragment layout.  FP6: the leading s6
// K-steps run on the FP6 matrix path first (`v_mfma_scale_f32_16x16x128_f8f6f4`: two K-steps per instruction, a lane holds
// the 32 codes of one unit and its block scale; exact integer sums in fp32, see fp6_kernel.h), every other K-step as usual
// with activations that arrive lowered.
template <int MF, bool COOP, bool FP6 = false>
__global__ __launch_bounds__(1024) void k_few_rows(const RowsParams p)
{
    static_assert(!COOP || MF == 1, "the cooperative pass is for calls of a few rows");
    static_assert(!(COOP && FP6), "FP6 calls bring lowered activations");
    extern __shared__ __align__(16) unsigned char lds[];   // [waves][MF][64 lanes] accumulator quads, then (COOP) the lowered rows
    v4i *const red = reinterpret_cast<v4i *>(lds);
    const int xl_stride = 32 * p.units4 + 16;   // (+16: rows start in different banks)
    unsigned char *const xl = lds + (blockDim.x >> 6) * MF * 1024;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = (int)(blockDim.x >> 6);
    const int c = lane & 15, qd = lane >> 4;   // row of the fragment (weight row / activation row), 16-channel quarter of the K-step
    const int n0 = blockIdx.x * kRowCols;
    const int n = n0 + c;                      // < Npad: the weight tiles are padded

    // the epilogue's scales and biases travel with the first operands (waves 0 .. MF-1: fragment `wave`, rows 16 wave + c,
    // output channels n0 + 4 qd + i)
    float cs4[4] = {0.f, 0.f, 0.f, 0.f}, bi4[4] = {0.f, 0.f, 0.f, 0.f};
    if (wave < MF) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            cs4[i] = p.cs[n0 + 4 * qd + i];
            bi4[i] = p.cs[p.Npad + n0 + 4 * qd + i];
        }
    }
    // ... and so does the consumer's position of these four columns (flexiq_out.lower_for; 4: no 4-bit channels of a consumer)
    const int sn_pre = wave < MF && p.next_ashift != nullptr && n0 + 4 * qd < p.next_K4 ? p.next_ashift[(n0 + 4 * qd) >> p.next_gs_log2] : 4;

    v4i acc[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f) acc[f] = (v4i){0, 0, 0, 0};

    constexpr int UN = MF <= 3 ? 4 : 3;   // K-steps in flight per wave (four with four fragments spill)
    v4i w8[UN], x[UN][MF];
    int sa[UN];
    bool low[UN], valid[UN];
    // weight fragments (and activation positions) of the K-steps ks0, ks0 + nw, ...: loads only.  4-bit units come from the
    // position-expanded copy (code << w_shift as int8, 16 bytes per lane like an 8-bit unit): measured against the packed codes
    // expanded in registers (8 bytes and a position byte per lane, 22 vector-ALU operations per 16 codes) it is faster at every
    // size (ViT-L fc2, 16 rows, r = 1: 5.2 against 6.1 us; 16384 x 4096 weights, 8 rows: 16.1 against 18.7 us): what the packed
    // codes save in bytes the expansion costs in instructions.  One and two rows, where bytes decide, go to k_few_rows_dot.
    auto issue_w = [&](int ks0) {
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int ks = ks0 + k * nw;
            const int u = 2 * ks + (qd >> 1), h = qd & 1;   // this lane's unit and k-half
            valid[k] = ks < p.steps && u < p.units;
            low[k] = valid[k] && u < p.units4;
            w8[k] = (v4i){0, 0, 0, 0};
            sa[k] = 0;
            if (valid[k]) w8[k] = *reinterpret_cast<const v4i *>(p.W8 + (low[k] ? p.w4x_delta : 0) + (((int64_t)u * 2 + h) * p.Npad + n) * 16);
            if (low[k] && !COOP && !p.x_pre) sa[k] = p.ashift[u >> p.gs_shift];
        }
    };
    // activation fragments of the same K-steps: from memory, or (COOP, 4-bit units) lowered already from LDS
    auto issue_x = [&](int ks0) {
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int u = 2 * (ks0 + k * nw) + (qd >> 1), h = qd & 1;
#pragma unroll
            for (int f = 0; f < MF; ++f) {
                const int m = 16 * f + c;
                if (COOP && low[k])
                    x[k][f] = m < p.M ? *reinterpret_cast<const v4i *>(xl + m * xl_stride + u * 32 + 16 * h) : (v4i){0, 0, 0, 0};
                else
                    x[k][f] = valid[k] && m < p.M ? *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + u * 32 + 16 * h) : (v4i){0, 0, 0, 0};
            }
        }
    };
    int ks0 = wave;
    if constexpr (FP6) {
        // chunks of two FP6 K-steps (128 channels), dealt to the waves in turn; the int8 K-steps after them continue the deal
        const int chunks = (p.s6 + 1) >> 1, S = p.C >> 6;
        v4f accf[MF];
#pragma unroll
        for (int f = 0; f < MF; ++f) accf[f] = (v4f){0.f, 0.f, 0.f, 0.f};
        constexpr int U6 = 2;   // chunks in flight
        for (int c0 = wave; c0 < chunks; c0 += nw * U6) {
            v4i wlo[U6], xlo[U6][MF];
            v2i whi[U6], xhi[U6][MF];
            int wsc[U6], asc[U6];
#pragma unroll
            for (int k = 0; k < U6; ++k) {
                const int ks = 2 * (c0 + k * nw) + (qd >> 1), h = qd & 1;   // this lane's K-step and unit
                const bool ok = ks < p.s6;
                wlo[k] = (v4i){0, 0, 0, 0};
                whi[k] = (v2i){0, 0};
                wsc[k] = asc[k] = 127;
                if (ok) {
                    // the first 16 code bytes of unit h in plane h, the last 8 of both units in plane 2 (unit h in half h ^ ((row / 16) % 2))
                    wlo[k] = *reinterpret_cast<const v4i *>(p.W6 + (((int64_t)ks * 3 + h) * p.Npad + n) * 16);
                    whi[k] = *reinterpret_cast<const v2i *>(p.W6 + (((int64_t)ks * 3 + 2) * p.Npad + n) * 16 + 8 * (h ^ ((n >> 4) & 1)));
                    wsc[k] = p.W6S[((int64_t)(ks >> 2) * p.Npad + n) * 8 + 4 * h + (ks & 3)];
                    asc[k] = 130 + p.ashift[(2 * ks + h) >> p.gs_shift];   // 2^(position + 3): the codes are k / 8
                }
#pragma unroll
                for (int f = 0; f < MF; ++f) {
                    const int m = 16 * f + c, blk = m >> 6, r = m & 63;
                    xlo[k][f] = (v4i){0, 0, 0, 0};
                    xhi[k][f] = (v2i){0, 0};
                    if (ok && m < p.M) {
                        xlo[k][f] = *reinterpret_cast<const v4i *>(p.X6 + ((((int64_t)blk * S + ks) * 3 + h) * 64 + r) * 16);
                        xhi[k][f] = *reinterpret_cast<const v2i *>(p.X6 + ((((int64_t)blk * S + ks) * 3 + 2) * 64 + r) * 16 + 8 * (h ^ ((r >> 4) & 1)));
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < U6; ++k)
#pragma unroll
                for (int f = 0; f < MF; ++f)
                    accf[f] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        (v8i){wlo[k].x, wlo[k].y, wlo[k].z, wlo[k].w, whi[k].x, whi[k].y, 0, 0},
                        (v8i){xlo[k][f].x, xlo[k][f].y, xlo[k][f].z, xlo[k][f].w, xhi[k][f].x, xhi[k][f].y, 0, 0}, accf[f], 2, 2, 0, wsc[k], 0, asc[k]);
        }
#pragma unroll
        for (int f = 0; f < MF; ++f)
            acc[f] = (v4i){(int)accf[f].x, (int)accf[f].y, (int)accf[f].z, (int)accf[f].w};   // exact integers below 2^24
        ks0 = p.s6 + (wave + nw - chunks % nw) % nw;
    }
    issue_w(ks0);   // (a wave beyond the last K-step loads nothing)
    if constexpr (COOP) {
        // few rows: in the fragment layout most lanes hold no row, and lowering there would cost every wave the full
        // instruction count for a handful of values.  The block lowers the 4-bit channels of its rows once, every lane a
        // 16-byte piece, into LDS, while the first weight fragments are on their way.
        const int per_row = 2 * p.units4;   // pieces per row
        for (int i = tid; i < p.M * per_row; i += (int)blockDim.x) {
            const int m = i / per_row, j = i - m * per_row;
            const v4i v = *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + 16 * j);
            const int s_ = p.ashift[(j >> 1) >> p.gs_shift];
            *reinterpret_cast<v4i *>(xl + m * xl_stride + 16 * j) =
                (v4i){(int)lower4((uint32_t)v.x, s_), (int)lower4((uint32_t)v.y, s_), (int)lower4((uint32_t)v.z, s_), (int)lower4((uint32_t)v.w, s_)};
        }
        __syncthreads();
    }
    if (ks0 < p.steps) for (;;) {   // (a wave beyond the last K-step has nothing to multiply)
        issue_x(ks0);
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            if (low[k] && !COOP && !p.x_pre) {
#pragma unroll
                for (int f = 0; f < MF; ++f)
                    x[k][f] = (v4i){(int)lower4((uint32_t)x[k][f].x, sa[k]), (int)lower4((uint32_t)x[k][f].y, sa[k]),
                                    (int)lower4((uint32_t)x[k][f].z, sa[k]), (int)lower4((uint32_t)x[k][f].w, sa[k])};
            }
#pragma unroll
            for (int f = 0; f < MF; ++f) acc[f] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w8[k], x[k][f], acc[f], 0, 0, 0);
        }
        ks0 += nw * UN;
        if (ks0 >= p.steps) break;
        issue_w(ks0);
    }

    // ---- the waves' sums meet in LDS
#pragma unroll
    for (int f = 0; f < MF; ++f) red[(wave * MF + f) * 64 + lane] = acc[f];
    __syncthreads();
    if (wave >= MF) return;
    v4i s = {0, 0, 0, 0};
    for (int w = 0; w < nw; ++w) s += red[(w * MF + wave) * 64 + lane];

    // ---- epilogue.  Lane: row m = 16 wave + c; accumulator register i: output channel n0 + 4 qd + i
    const int m = 16 * wave + c;
    if (m >= p.M) return;
    const int nn0 = n0 + 4 * qd;
    if (nn0 >= p.N) return;
    const int64_t o = (int64_t)m * p.N + nn0;
    float yv[4];
    uint32_t qw = 0;
    // the consumer's position for these four columns (one channel group of the consumer: nn0 is a multiple of four)
    const bool lower = p.next_ashift != nullptr && nn0 < p.next_K4;
    const int sn = sn_pre;
    const float lo = 128.0f - (float)(8 << sn), hi = 127.0f + (float)(8 << sn);   // (position 4: the whole int8 range)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        yv[i] = __builtin_fmaf((float)s[i], cs4[i], bi4[i]);
        // offset form, as in the tiled kernel: round to nearest-even, saturate to 0..255, flip the top bit; for a consumer's
        // 4-bit channel the offset code is clamped first (integer bounds: the same as clamping the rounded code)
        qw = __builtin_amdgcn_cvt_pk_u8_f32(
            __builtin_amdgcn_fmed3f(__builtin_fmaf((float)s[i], cs4[i] * p.r_out, bi4[i] * p.r_out + 128.0f), lo, hi), i, qw);
    }
    qw ^= 0x80808080u;
    if (lower) qw &= 0x01010101u * ((0xFFu << sn) & 0xFFu);
    if ((p.N & 3) == 0) {   // four whole columns, aligned rows
        if (p.acc) *reinterpret_cast<v4i *>(p.acc + o) = s;
        if (p.y) *reinterpret_cast<float4 *>(p.y + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
        if (p.q) *reinterpret_cast<uint32_t *>(p.q + o) = qw;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (nn0 + i >= p.N) continue;
            if (p.acc) p.acc[o + i] = s[i];
            if (p.y) p.y[o + i] = yv[i];
            if (p.q) p.q[o + i] = (int8_t)(qw >> (8 * i));
        }
    }
}

// ---- Calls of at most four rows: matrix-vector products on the vector ALU's integer dot instructions.
//
// With so few rows the matrix cores have nothing to reuse a weight fragment for, and their 16-column fragments tie the
// block count to N / 16.  Here a lane multiplies a 16-channel piece of one weight row with the same piece of every
// activation row: 8-bit units with `v_dot4_i32_i8` (four per piece and row), 4-bit units with `v_dot8_i32_i4` on the packed
// codes as they are stored (two per piece and row; the sum of code products is put at its position afterwards,
// sum << (activation position + weight position): Section 7's shifted accumulation, one `v_lshl_add_u32`).  This is the one
// place on this chip where 4-bit groups cost fewer bytes AND fewer operations than 8-bit ones: nothing is expanded.
// The activation codes of the 4-bit channels are produced once per block (clamp at the group's position, Section 4.1,
// then two codes per byte in the order of the packed weights) and kept in LDS.  A block owns 8 output columns (a
// wave load covers 8 columns x 8 pieces: 128-byte runs of the weight tiles) and the whole reduction; lanes of a
// column meet by cross-lane adds, waves in LDS.
constexpr int kVecCols = 8;

// MR: activation rows (1 .. 4).  CG: groups of 8 columns per block (1 or 4; a lane then holds a piece of CG weight rows per
// activation piece: more bytes in flight per wave, activation pieces and the block's set-up shared by more columns; for
// layers with enough columns to still give every compute unit several blocks).
template <int MR, int CG>
__global__ __launch_bounds__(512) void k_few_rows_dot(const RowsParams p)
{
    // LDS: [waves][MR][8 CG] wave sums, then [MR][units4][16] packed activation codes, then [MR][C] the activation rows
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int BC = kVecCols * CG;   // columns per block
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = (int)(blockDim.x >> 6);
    int *const red = reinterpret_cast<int *>(lds);
    unsigned char *const xl = lds + nw * MR * BC * 4;
    const int xl_stride = 16 * p.units4;
    unsigned char *const xr = xl + MR * xl_stride;   // (8-bit channels only are read from here)
    const int col = lane & 7, sub = lane >> 3;   // column of a group, piece of the wave load
    const int n0 = blockIdx.x * BC;
    const int n = n0 + col;                      // + 8 c for column group c; < Npad (checked by the launcher)
    const int pieces = 2 * p.units;              // 16-channel pieces of the reduction
    const int groups = (pieces + 7) >> 3;        // wave loads of 8 pieces

    // the epilogue's scale and bias travel with the first operands (thread BC m + j: row m, column n0 + j)
    float cs_e = 0.f, bi_e = 0.f;
    if (tid < MR * BC) {
        cs_e = p.cs[n0 + tid % BC];
        bi_e = p.cs[p.Npad + n0 + tid % BC];
    }
    // ... and so does the consumer's position of that column (flexiq_out.lower_for; 4: no 4-bit channel of a consumer)
    const int sn_e = tid < MR * BC && p.next_ashift != nullptr && n0 + tid % BC < p.next_K4 ? p.next_ashift[(n0 + tid % BC) >> p.next_gs_log2] : 4;
    constexpr int UN = CG == 4 ? 2 : 4;   // wave loads in flight per wave and column group
    v4i w8[UN][CG];
    v2i w4[UN][CG];
    int sh[UN][CG], sa[UN];
    bool low[UN], valid[UN];
    auto issue = [&](int g0) {
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int j = 8 * (g0 + k * nw) + sub;   // this lane's piece: unit j / 2, half j % 2
            const int u = j >> 1;
            valid[k] = g0 + k * nw < groups && j < pieces;
            low[k] = valid[k] && u < p.units4;
            sa[k] = 0;
#pragma unroll
            for (int c = 0; c < CG; ++c) {
                w8[k][c] = (v4i){0, 0, 0, 0};
                w4[k][c] = (v2i){0, 0};
                sh[k][c] = 0;
            }
            if (low[k]) {
#pragma unroll
                for (int c = 0; c < CG; ++c) {
                    w4[k][c] = *reinterpret_cast<const v2i *>(p.W4 + ((int64_t)u * p.Npad + n + 8 * c) * 16 + 8 * (j & 1));
                    sh[k][c] = p.wshift[(int64_t)(u >> p.gs_shift) * p.Npad + n + 8 * c];
                }
                sa[k] = p.ashift[u >> p.gs_shift];
            } else if (valid[k]) {
#pragma unroll
                for (int c = 0; c < CG; ++c) w8[k][c] = *reinterpret_cast<const v4i *>(p.W8 + ((int64_t)j * p.Npad + n + 8 * c) * 16);
            }
        }
    };
    int g0 = wave;
    issue(g0);   // (a wave beyond the last piece loads nothing)

    // ---- the activation rows go to LDS once per block (the eight columns of a wave load read the same pieces: a broadcast
    // there, a trip through the vector memory path per lane otherwise); every thread one 16-channel piece of one row at a
    // time: 8-bit channels as they are, 4-bit channels as codes
    {
        const int per_row = 2 * p.units4, all_per_row = 2 * p.units;
        for (int i = tid; i < p.M * (all_per_row - per_row); i += (int)blockDim.x) {
            const int m = i / (all_per_row - per_row), j = per_row + i - m * (all_per_row - per_row);
            *reinterpret_cast<v4i *>(xr + m * p.C + 16 * j) = *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + 16 * j);
        }
        for (int i = tid; i < p.M * per_row; i += (int)blockDim.x) {
            const int m = i / per_row, j = i - m * per_row;
            if (j < p.pieces_p) {   // the producer has made the codes (same layout: flexiq_lower_packed4, flexiq_out.x4)
                *reinterpret_cast<v2i *>(xl + m * xl_stride + 8 * j) = *reinterpret_cast<const v2i *>(p.X4 + (int64_t)m * (p.C >> 1) + 8 * j);
                continue;
            }
            const v4i v = *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + 16 * j);
            const int s_ = p.ashift[(j >> 1) >> p.gs_shift];
            // lowered bytes are code << s with the low s bits clear, so a dword-wide shift right leaves the code's two's
            // complement nibble at the bottom of every byte; dword e of a piece: channels 8 e .. 8 e + 3 in the low
            // halves of its bytes, 8 e + 4 .. 8 e + 7 in the high halves (the order of the packed weight codes)
            const uint32_t a = (lower4((uint32_t)v.x, s_) >> s_) & 0x0F0F0F0Fu, b = (lower4((uint32_t)v.y, s_) >> s_) & 0x0F0F0F0Fu;
            const uint32_t c = (lower4((uint32_t)v.z, s_) >> s_) & 0x0F0F0F0Fu, d = (lower4((uint32_t)v.w, s_) >> s_) & 0x0F0F0F0Fu;
            *reinterpret_cast<v2i *>(xl + m * xl_stride + 8 * j) = (v2i){(int)(a | (b << 4)), (int)(c | (d << 4))};
        }
        __syncthreads();
    }

    int acc[MR][CG];
#pragma unroll
    for (int m = 0; m < MR; ++m)
#pragma unroll
        for (int c = 0; c < CG; ++c) acc[m][c] = 0;
    for (;;) {
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int j = 8 * (g0 + k * nw) + sub;
            if (low[k]) {
#pragma unroll
                for (int m = 0; m < MR; ++m) {
                    const v2i xc = m < p.M ? *reinterpret_cast<const v2i *>(xl + m * xl_stride + 8 * j) : (v2i){0, 0};
#pragma unroll
                    for (int c = 0; c < CG; ++c) {
                        int t = __builtin_amdgcn_sdot8(w4[k][c].x, xc.x, 0, false);
                        t = __builtin_amdgcn_sdot8(w4[k][c].y, xc.y, t, false);
                        acc[m][c] += (int)((uint32_t)t << (sh[k][c] + sa[k]));
                    }
                }
            } else if (valid[k]) {
#pragma unroll
                for (int m = 0; m < MR; ++m) {
                    const v4i xv = m < p.M ? *reinterpret_cast<const v4i *>(xr + m * p.C + 16 * j) : (v4i){0, 0, 0, 0};
#pragma unroll
                    for (int c = 0; c < CG; ++c) {
                        int t = __builtin_amdgcn_sdot4(w8[k][c].x, xv.x, acc[m][c], false);
                        t = __builtin_amdgcn_sdot4(w8[k][c].y, xv.y, t, false);
                        t = __builtin_amdgcn_sdot4(w8[k][c].z, xv.z, t, false);
                        acc[m][c] = __builtin_amdgcn_sdot4(w8[k][c].w, xv.w, t, false);
                    }
                }
            }
        }
        g0 += nw * UN;
        if (g0 >= groups) break;
        issue(g0);
    }

    // ---- the eight lanes of a column, then the waves
#pragma unroll
    for (int m = 0; m < MR; ++m)
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            int a = acc[m][c];
            a += __shfl_xor(a, 8);
            a += __shfl_xor(a, 16);
            a += __shfl_xor(a, 32);
            if (sub == 0) red[(wave * MR + m) * BC + 8 * c + col] = a;
        }
    __syncthreads();
    if (tid >= MR * BC) return;
    const int m = tid / BC, jn = tid % BC, nn = n0 + jn;
    if (m >= p.M || nn >= p.N) return;
    int v = 0;
    for (int w = 0; w < nw; ++w) v += red[(w * MR + m) * BC + jn];
    const float c = cs_e, b = bi_e;
    const int64_t o = (int64_t)m * p.N + nn;
    if (p.acc) p.acc[o] = v;
    if (p.y) p.y[o] = __builtin_fmaf((float)v, c, b);
    if (p.q) {
        // offset form, as in the tiled kernel: round to nearest-even, saturate to 0..255, flip the top bit
        // (for a 4-bit channel of the consumer named by lower_for: clamped and masked at its position, as in k_few_rows)
        const bool lower = p.next_ashift != nullptr && nn < p.next_K4;
        const int sn = sn_e;
        const float t = __builtin_amdgcn_fmed3f(__builtin_fmaf((float)v, c * p.r_out, b * p.r_out + 128.0f), 128.0f - (float)(8 << sn),
                                                127.0f + (float)(8 << sn));
        uint32_t code = __builtin_amdgcn_cvt_pk_u8_f32(t, 0, 0u) ^ 0x80u;
        if (lower) code &= (0xFFu << sn) & 0xFFu;
        p.q[o] = (int8_t)code;
    }
}

// ---- Calls of 65 rows to about a thousand on layers with few output tiles: a 64 x 64 tile per block, the reduction split
// over its waves.
//
// The tiled kernel gives such a call a handful of 64 x 64 blocks that each walk the whole reduction, one barrier per
// K-step: bound by the latency of a step (ViT-L fc2 with 197 rows: 64 steps, 14.6 us at r = 0 and 22.1 us at r = 1 for
// 0.3 us of matrix work).  Here the eight waves of a block take the K-steps wave, wave + 8, ... of the tile on their own:
// operands straight from global memory into MFMA registers (every byte of the tile's weights and activations is loaded by
// exactly one lane of the block), sixteen v_mfma_i32_16x16x64_i8 per K-step and wave, no barrier until the waves' sums
// meet in LDS.  4-bit units come from the position-expanded weight copy and their activations are lowered in registers.
// FR x FC: 16 x 16 fragments of the tile (rows x columns), NW: waves.  A smaller tile means more blocks, i.e. more compute
// units pulling operands, at more operand bytes per multiply.
// FP6: the leading s6 K-steps run first on `v_mfma_scale_f32_16x16x128_f8f6f4`, as in the FP6 build of k_few_rows (chunks of
// two K-steps dealt to the waves in turn; a lane holds the 32 codes of one unit and its block scale), every other K-step as
// usual with activations that arrive lowered.
template <int FR, int FC, int NW, int UN, bool FP6 = false>
__global__ __launch_bounds__(64 * NW) void k_tile_splitk(const RowsParams p)
{
    constexpr int kTileRows = 16 * FR, kTileCols = 16 * FC, kTileWaves = NW, NF = FR * FC;
    constexpr int E = (NF + NW - 1) / NW;   // fragments a wave finishes: wave, wave + NW, ...
    extern __shared__ __align__(16) unsigned char lds[];   // [waves][fragments][64 lanes] accumulator quads
    v4i *const red = reinterpret_cast<v4i *>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, qd = lane >> 4;
    const int n0 = blockIdx.x * kTileCols;      // columns n0 + 16 g + c < Npad: the weight tiles are padded
    const int m0 = blockIdx.y * kTileRows;

    // the epilogue's scales and biases travel with the first operands
    // (fragment id = FC f + g: rows m0 + 16 f + c, columns n0 + 16 g + 4 qd + i)
    float cs4[E][4], bi4[E][4];
#pragma unroll
    for (int e = 0; e < E; ++e)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int nn = n0 + 16 * ((wave + NW * e) % FC) + 4 * qd + i;   // < Npad
            cs4[e][i] = p.cs[nn];
            bi4[e][i] = p.cs[p.Npad + nn];
        }
    // ... and so does the consumer's position of the lane's four columns (flexiq_out.lower_for): those of its FP6 prefix leave
    // clamped in q and as FP6 codes in its activation buffer, its other 4-bit channels clamped and masked in q
    int sn_e[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int nn0 = n0 + 16 * ((wave + NW * e) % FC) + 4 * qd;
        const bool to6 = FP6 && p.nx6 != nullptr && nn0 < p.next_K6;
        sn_e[e] = p.next_ashift != nullptr && (to6 || nn0 < p.next_K4) ? p.next_ashift[nn0 >> p.next_gs_log2] : 4;
    }

    v4i acc[FR][FC];
#pragma unroll
    for (int f = 0; f < FR; ++f)
#pragma unroll
        for (int g = 0; g < FC; ++g) acc[f][g] = (v4i){0, 0, 0, 0};

    int first = wave;
    if constexpr (FP6) {
        const int chunks = (p.s6 + 1) >> 1, S = p.C >> 6;
        v4f accf[FR][FC];
#pragma unroll
        for (int f = 0; f < FR; ++f)
#pragma unroll
            for (int g = 0; g < FC; ++g) accf[f][g] = (v4f){0.f, 0.f, 0.f, 0.f};
        constexpr int U6 = UN >= 4 ? 2 : 1;   // chunks in flight
        for (int c0 = wave; c0 < chunks; c0 += NW * U6) {
            v4i wlo[U6][FC], xlo[U6][FR];
            v2i whi[U6][FC], xhi[U6][FR];
            int wsc[U6][FC], asc[U6];
#pragma unroll
            for (int k = 0; k < U6; ++k) {
                const int ks = 2 * (c0 + k * NW) + (qd >> 1), h = qd & 1;   // this lane's K-step and unit
                const bool ok = ks < p.s6;
                asc[k] = ok ? 130 + p.ashift[(2 * ks + h) >> p.gs_shift] : 127;   // 2^(position + 3): the codes are k / 8
#pragma unroll
                for (int g = 0; g < FC; ++g) {
                    const int n = n0 + 16 * g + c;
                    wlo[k][g] = (v4i){0, 0, 0, 0};
                    whi[k][g] = (v2i){0, 0};
                    wsc[k][g] = 127;
                    if (ok) {
                        wlo[k][g] = *reinterpret_cast<const v4i *>(p.W6 + (((int64_t)ks * 3 + h) * p.Npad + n) * 16);
                        whi[k][g] = *reinterpret_cast<const v2i *>(p.W6 + (((int64_t)ks * 3 + 2) * p.Npad + n) * 16 + 8 * (h ^ ((n >> 4) & 1)));
                        wsc[k][g] = p.W6S[((int64_t)(ks >> 2) * p.Npad + n) * 8 + 4 * h + (ks & 3)];
                    }
                }
#pragma unroll
                for (int f = 0; f < FR; ++f) {
                    const int m = m0 + 16 * f + c, blk = m >> 6, r = m & 63;
                    xlo[k][f] = (v4i){0, 0, 0, 0};
                    xhi[k][f] = (v2i){0, 0};
                    if (ok && m < p.M) {
                        xlo[k][f] = *reinterpret_cast<const v4i *>(p.X6 + ((((int64_t)blk * S + ks) * 3 + h) * 64 + r) * 16);
                        xhi[k][f] = *reinterpret_cast<const v2i *>(p.X6 + ((((int64_t)blk * S + ks) * 3 + 2) * 64 + r) * 16 + 8 * (h ^ ((r >> 4) & 1)));
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < U6; ++k)
#pragma unroll
                for (int f = 0; f < FR; ++f)
#pragma unroll
                    for (int g = 0; g < FC; ++g)
                        accf[f][g] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                            (v8i){wlo[k][g].x, wlo[k][g].y, wlo[k][g].z, wlo[k][g].w, whi[k][g].x, whi[k][g].y, 0, 0},
                            (v8i){xlo[k][f].x, xlo[k][f].y, xlo[k][f].z, xlo[k][f].w, xhi[k][f].x, xhi[k][f].y, 0, 0}, accf[f][g], 2, 2, 0,
                            wsc[k][g], 0, asc[k]);
        }
#pragma unroll
        for (int f = 0; f < FR; ++f)
#pragma unroll
            for (int g = 0; g < FC; ++g)
                acc[f][g] = (v4i){(int)accf[f][g].x, (int)accf[f][g].y, (int)accf[f][g].z, (int)accf[f][g].w};   // exact integers below 2^24
        first = p.s6 + (wave + NW - chunks % NW) % NW;   // the int8 K-steps continue the deal
    }
    // UN K-steps in flight per wave
    for (int ks0 = first; ks0 < p.steps; ks0 += kTileWaves * UN) {
        v4i w8[UN][FC], x[UN][FR];
        int sa[UN];
        bool low[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int ks = ks0 + k * kTileWaves;
            const int u = 2 * ks + (qd >> 1), h = qd & 1;   // this lane's unit and k-half
            const bool valid = ks < p.steps && u < p.units;
            low[k] = valid && u < p.units4;
            sa[k] = low[k] && !p.x_pre ? p.ashift[u >> p.gs_shift] : 0;
#pragma unroll
            for (int g = 0; g < FC; ++g)
                w8[k][g] = valid ? *reinterpret_cast<const v4i *>(p.W8 + (low[k] ? p.w4x_delta : 0) + (((int64_t)u * 2 + h) * p.Npad + n0 + 16 * g + c) * 16)
                                 : (v4i){0, 0, 0, 0};
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                const int m = m0 + 16 * f + c;
                x[k][f] = valid && m < p.M ? *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + u * 32 + 16 * h) : (v4i){0, 0, 0, 0};
            }
        }
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            if (low[k] && !p.x_pre) {
#pragma unroll
                for (int f = 0; f < FR; ++f)
                    x[k][f] = (v4i){(int)lower4((uint32_t)x[k][f].x, sa[k]), (int)lower4((uint32_t)x[k][f].y, sa[k]),
                                    (int)lower4((uint32_t)x[k][f].z, sa[k]), (int)lower4((uint32_t)x[k][f].w, sa[k])};
            }
#pragma unroll
            for (int f = 0; f < FR; ++f)
#pragma unroll
                for (int g = 0; g < FC; ++g) acc[f][g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w8[k][g], x[k][f], acc[f][g], 0, 0, 0);
        }
    }

    // ---- the waves' sums meet in LDS; wave w adds up and finishes fragments w, w + NW, ...
#pragma unroll
    for (int f = 0; f < FR; ++f)
#pragma unroll
        for (int g = 0; g < FC; ++g) red[(wave * NF + FC * f + g) * 64 + lane] = acc[f][g];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int id = wave + NW * e, f = id / FC, g = id % FC;
        if (id >= NF) break;
        v4i s = {0, 0, 0, 0};
#pragma unroll
        for (int w = 0; w < kTileWaves; ++w) s += red[(w * NF + id) * 64 + lane];
        const int m = m0 + 16 * f + c, nn0 = n0 + 16 * g + 4 * qd;
        if (m >= p.M || nn0 >= p.N) continue;
        const int64_t o = (int64_t)m * p.N + nn0;
        float yv[4];
        uint32_t qw = 0;
        const bool to6 = FP6 && p.nx6 != nullptr && nn0 < p.next_K6;
        const bool lower = p.next_ashift != nullptr && !to6 && nn0 < p.next_K4;
        const int sn = sn_e[e];
        const float lo = 128.0f - (float)(8 << sn), hi = 127.0f + (float)(8 << sn);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            yv[i] = __builtin_fmaf((float)s[i], cs4[e][i], bi4[e][i]);
            qw = __builtin_amdgcn_cvt_pk_u8_f32(
                __builtin_amdgcn_fmed3f(__builtin_fmaf((float)s[i], cs4[e][i] * p.r_out, bi4[e][i] * p.r_out + 128.0f), lo, hi), i, qw);
        }
        if (to6) {
            // four codes (offset form u = code + 128, clamped above): floor(code / 2^sn) + 8 = (u >> sn) - ((128 >> sn) - 8), 0 .. 15 per
            // byte; E2M3 pattern of L / 8: sign << 5 | |L|.  Element 16 a + 4 b + i of a unit is its channel 8 b + 4 a + i (the order of the
            // packed FP6 weights), so the 24 bits are bytes 3 j .. 3 j + 2 of the unit's 24 with j = 4 a + b:
            // the first 16 bytes of a unit lie in plane (unit % 2) of the consumer's K-step, the last 8 in plane 2
            const uint32_t cb = ((qw >> sn) & (0x01010101u * (0xFFu >> sn))) - 0x01010101u * (uint32_t)((128 >> sn) - 8);
            const uint32_t neg = (~cb >> 3) & 0x01010101u;
            const uint32_t mag = ((cb & 0x07070707u) ^ (neg * 7u)) + neg;
            const uint32_t c6 = mag | (neg << 5);
            const uint32_t w24 = (c6 & 0x3Fu) | ((c6 >> 2) & 0xFC0u) | ((c6 >> 4) & 0x3F000u) | ((c6 >> 6) & 0xFC0000u);
            const int u = nn0 >> 5, hh = u & 1, rr = m & 63, j = 4 * ((nn0 >> 2) & 1) + ((nn0 & 31) >> 3);
            uint8_t *const blk = p.nx6 + ((int64_t)(m >> 6) * p.next_S + (u >> 1)) * 3072;
            // (one 2-byte and one 1-byte store: the even one of 3 j and 3 j + 1 starts the pair, which never straddles bytes 15 | 16)
            auto at = [&](int byte) { return byte < 16 ? blk + hh * 1024 + rr * 16 + byte : blk + 2048 + rr * 16 + 8 * (hh ^ ((rr >> 4) & 1)) + byte - 16; };
            if (j & 1) {
                *at(3 * j) = (uint8_t)w24;
                *reinterpret_cast<uint16_t *>(at(3 * j + 1)) = (uint16_t)(w24 >> 8);
            } else {
                *reinterpret_cast<uint16_t *>(at(3 * j)) = (uint16_t)w24;
                *at(3 * j + 2) = (uint8_t)(w24 >> 16);
            }
        }
        qw ^= 0x80808080u;
        if (lower) qw &= 0x01010101u * ((0xFFu << sn) & 0xFFu);
        if ((p.N & 3) == 0) {
            if (p.acc) *reinterpret_cast<v4i *>(p.acc + o) = s;
            if (p.y) *reinterpret_cast<float4 *>(p.y + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
            if (p.q) *reinterpret_cast<uint32_t *>(p.q + o) = qw;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (nn0 + i >= p.N) continue;
                if (p.acc) p.acc[o + i] = s[i];
                if (p.y) p.y[o + i] = yv[i];
                if (p.q) p.q[o + i] = (int8_t)(qw >> (8 * i));
            }
        }
    }
}

static int g_force_tile_splitk = -1;   // test hook: 1 = take k_tile_splitk whenever the call qualifies, 0 = never, -1 = automatic
static int g_last_tile_splitk = 0;
static bool g_tile_splitk_ready[64] = {};
constexpr int kTileMinRows = 32;   // up to here the few-row kernels measure faster

static int g_force_cg = 0;      // test hook: column groups per block of k_few_rows_dot (0 = automatic)
static int g_force_rows = -1;   // test hook: 1 / 2 = take k_few_rows / k_few_rows_dot whenever the call qualifies, 0 = never, -1 = automatic
static int g_last_rows = 0;

}  // namespace smallm

// Launches k_few_rows (*taken = 1) or k_few_rows_dot (*taken = 2) for a linear call with at most 64 rows; *taken = 0: the call
// was left to the other kernels.
int launch_few_rows(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int num_cu, int *taken,
                    const uint8_t *X4, const LowerArgs *lower)
{
    using namespace smallm;
    *taken = 0;
    g_last_rows = 0;
    if (g_force_rows == 0 || M < 1 || M > 64) return FLEXIQ_OK;
    if (out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
    if (out->lower_for && !lower) return FLEXIQ_OK;   // (the caller has checked the consumer; null positions: nothing to lower)
    if ((reinterpret_cast<uintptr_t>(X) & 15u) || (L->C & 15)) return FLEXIQ_OK;   // 16-byte activation pieces
    // Every block reads all activation rows: with more than 16 rows that traffic (blocks x M x C bytes through the compute
    // units' 64 B/clk path) decides, and beyond about one block per compute unit the tiled kernel's 64 x 64 tiles win
    // (16384 x 4096 weights, 32 / 64 rows: 23 / 38 us here against 18 / 19 us tiled; 4096 x 1024, 64 rows: 4.9 against 6.7 us).
    if (g_force_rows < 0 && M > 16 && (L->N + kRowCols - 1) / kRowCols > num_cu) return FLEXIQ_OK;
    RowsParams p = {};
    p.X = X; p.W8 = L->d_w8; p.W4 = L->d_w4; p.wshift = L->d_wshift;
    p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift;
    p.cs = L->d_cs;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = (int)M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.units = L->C / kUnit;
    p.units4 = L->max_4bit_ch / kUnit;
    p.x_pre = L->x_prelowered ? 1 : 0;
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.steps = (p.units + 1) / 2;
    p.w4x_delta = L->U * 32 * L->Npad;
    if (lower && lower->ashift) { p.next_ashift = lower->ashift; p.next_K4 = lower->K4; p.next_gs_log2 = lower->gs_log2; }
    // packed activation codes of the leading whole K-steps of 4-bit channels (the caller has checked alignment): the dot-product
    // kernel takes them as they are; the matrix-core kernel has no use for them and leaves such a call to the tiled kernel
    p.X4 = X4 && !L->x_prelowered ? X4 : nullptr;
    p.pieces_p = p.X4 ? (L->max_4bit_ch / 64) * 4 : 0;
    // One or two rows: the dot-product kernel.  Three or four rows: where the layer has columns enough for four column groups per
    // block and at least half of the channels run at 4 bits (measured on 16384 x 4096 weights at four rows, r = 0 / 0.5 / 1: 14.7 / 13.1 /
    // 11.6 us against 13.1 / 12.9 / 14.4 us on the matrix-core kernel; from six rows on it is bound by its vector-ALU work, 22 us; at
    // ViT-L sizes the matrix-core kernel is ahead from three rows on).
    const int ncg = (L->N + kVecCols - 1) / kVecCols;
    const bool wide = ncg >= 4 * num_cu && (ncg + 3) / 4 * 4 * kVecCols <= L->Npad;
    if (g_force_rows == 2 || (g_force_rows < 0 && (M <= 2 || (M <= 4 && wide && 2 * L->max_4bit_ch >= L->C)))) {
        const int groups = (2 * p.units + 7) / 8;
        const int nw = groups >= 32 ? 8 : 4;   // (eight waves for shorter reductions measured slower: 3.6 against 3.4 us on 4096 x 1024)
        // column groups per block: four where the layer still gives every compute unit several blocks (measured on 16384 x 4096
        // and 8192 x 8192 weights, one row, r = 0 / 1: 12.0 / 7.9 us and 12.0 / 9.3 us against 12.1 / 14.4 and 12.9 / 13.1 us with one
        // group; ViT-L sizes are faster with one); the last block's columns must stay inside the padded weight tiles
        int cg = g_force_cg > 0 ? g_force_cg : (wide ? 4 : 1);
        if (((ncg + cg - 1) / cg) * cg * kVecCols > L->Npad) cg = 1;
        const size_t lds = (size_t)nw * M * kVecCols * cg * 4 + (size_t)M * 16 * p.units4 + (size_t)M * L->C;
        if (M <= 4 && lds <= 64 * 1024) {
            void (*fn)(const RowsParams) = nullptr;
            switch ((int)M) {
            case 1: fn = cg == 4 ? k_few_rows_dot<1, 4> : k_few_rows_dot<1, 1>; break;
            case 2: fn = cg == 4 ? k_few_rows_dot<2, 4> : k_few_rows_dot<2, 1>; break;
            case 3: fn = cg == 4 ? k_few_rows_dot<3, 4> : k_few_rows_dot<3, 1>; break;
            default: fn = cg == 4 ? k_few_rows_dot<4, 4> : k_few_rows_dot<4, 1>; break;
            }
            hipLaunchKernelGGL(fn, dim3((unsigned)((ncg + cg - 1) / cg)), dim3(64 * nw), lds, (hipStream_t)stream, p);
            FLEXIQ_HIP(hipGetLastError());
            *taken = 2;
            g_last_rows = 2;
            return FLEXIQ_OK;
        }
        if (g_force_rows == 2) return FLEXIQ_OK;
    }
    if (X4) return FLEXIQ_OK;
    const int mf = (int)((M + 15) / 16);
    const unsigned blocks = (unsigned)((L->N + kRowCols - 1) / kRowCols);
    // waves per block: as many as there are K-steps to split while the layer gives a compute unit a block or so (the call is one
    // trip to memory: widest wins); with several blocks per compute unit four waves that each stream batch after batch, so that
    // one block's meeting in LDS and epilogue hide behind the others' loads (16384 x 4096 weights, 8 rows: 13.4 against 17.2 us)
    const int nw = (int)blocks >= 2 * num_cu ? 4 : (p.steps >= 12 ? 16 : (p.steps >= 6 ? 8 : 4));
    size_t lds = (size_t)nw * mf * 64 * 16;
    // few rows whose 4-bit channels the kernel lowers: once per block, through LDS
    const size_t rows_bytes = (size_t)M * (32 * (size_t)p.units4 + 16);
    const bool coop = M <= 8 && !p.x_pre && p.units4 > 0 && lds + rows_bytes <= 64 * 1024;
    if (coop) lds += rows_bytes;
    void (*fn)(const RowsParams) =
        mf == 1 ? (coop ? k_few_rows<1, true> : k_few_rows<1, false>) : (mf == 2 ? k_few_rows<2, false> : (mf == 3 ? k_few_rows<3, false> : k_few_rows<4, false>));
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(64 * nw), lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    *taken = 1;
    g_last_rows = 1;
    return FLEXIQ_OK;
}

// The FP6 variant of a linear call with at most 64 rows (flexiq_mixed_gemm_fp6): k_few_rows with the leading K6 channels on the
// FP6 matrix path; *taken = 0: the call was left to the tiled FP6 kernel.
int launch_few_rows_fp6(const flexiq_layer *L, const int8_t *X, const uint8_t *X6, int64_t M, const flexiq_out *out, void *stream, int K6,
                        int num_cu, int *taken)
{
    using namespace smallm;
    *taken = 0;
    if (g_force_rows == 0 || M < 1 || M > 64) return FLEXIQ_OK;
    if (out->lower_for || out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
    if (g_force_rows < 0 && M > 16 && (L->N + kRowCols - 1) / kRowCols > num_cu) return FLEXIQ_OK;   // (as in launch_few_rows)
    RowsParams p = {};
    p.X = X; p.W8 = L->d_w8; p.X6 = X6; p.W6 = L->d_w6; p.W6S = L->d_w6s;
    p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift;
    p.cs = L->d_cs;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = (int)M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.units = L->C / kUnit;
    p.units4 = L->max_4bit_ch / kUnit;
    p.x_pre = 1;   // the 4-bit channels beyond the FP6 ones arrive lowered
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.steps = (p.units + 1) / 2;
    p.w4x_delta = L->U * 32 * L->Npad;
    p.s6 = K6 / 64;
    const int mf = (int)((M + 15) / 16);
    const unsigned blocks = (unsigned)((L->N + kRowCols - 1) / kRowCols);
    const int items = (p.s6 + 1) / 2 + (p.steps - p.s6);   // FP6 chunks and int8 K-steps to deal out
    const int nw = (int)blocks >= 2 * num_cu ? 4 : (items >= 12 ? 16 : (items >= 6 ? 8 : 4));
    const size_t lds = (size_t)nw * mf * 64 * 16;
    void (*fn)(const RowsParams) = mf == 1 ? k_few_rows<1, false, true> : (mf == 2 ? k_few_rows<2, false, true> : (mf == 3 ? k_few_rows<3, false, true> : k_few_rows<4, false, true>));
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(64 * nw), lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    *taken = 1;
    g_last_rows = 3;
    return FLEXIQ_OK;
}

// Once per device, when the first layer is packed on it: the dynamic-LDS limit of every build of k_tile_splitk, so that a
// launch is only a launch (and safe under stream capture).
int prepare_tile_splitk_kernels(int device)
{
    using namespace smallm;
    if (device < 0 || device >= 64) return FLEXIQ_EINVAL;
    if (g_tile_splitk_ready[device]) return FLEXIQ_OK;
    FLEXIQ_HIP(hipFuncSetAttribute((const void *)k_tile_splitk<4, 4, 8, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    FLEXIQ_HIP(hipFuncSetAttribute((const void *)k_tile_splitk<2, 4, 16, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    FLEXIQ_HIP(hipFuncSetAttribute((const void *)k_tile_splitk<2, 2, 16, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
    FLEXIQ_HIP(hipFuncSetAttribute((const void *)k_tile_splitk<4, 4, 8, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    FLEXIQ_HIP(hipFuncSetAttribute((const void *)k_tile_splitk<2, 4, 8, 4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
    FLEXIQ_HIP(hipFuncSetAttribute((const void *)k_tile_splitk<2, 2, 16, 4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024));
    g_tile_splitk_ready[device] = true;
    return FLEXIQ_OK;
}

static int launch_tile_any(const flexiq_layer *L, const int8_t *X, const uint8_t *X6, int K6, int64_t M, const flexiq_out *out, void *stream,
                           int num_cu, int *taken, const LowerArgs *lower)
{
    using namespace smallm;
    *taken = 0;
    g_last_tile_splitk = 0;
    // FP6 calls that lower for a consumer have no few-row kernel to go to: this one takes them at any row count
    const bool only_here = X6 && out->lower_for;
    if (g_force_tile_splitk == 0 || M < 1 || (M <= 16 && !only_here) || M > 0x7fffffff / 2) return FLEXIQ_OK;
    // (calls of at most 64 rows: the few-row hook, in any forced state, keeps this kernel out of its comparisons)
    if (M <= 64 && (g_force_rows >= 0 || (g_force_tile_splitk < 0 && M <= kTileMinRows && !only_here))) return FLEXIQ_OK;
    if (out->scan_for || out->x4 || (out->lower_for && !lower)) return FLEXIQ_OK;
    if (out->x6 && !(X6 && lower && lower->x6 == out->x6 && (L->N & 63) == 0 && (lower->K6 & 63) == 0)) return FLEXIQ_OK;   // FP6 output: FP6 calls only
    if ((reinterpret_cast<uintptr_t>(X) & 15u) || (L->C & 15) || L->device < 0 || L->device >= 64) return FLEXIQ_OK;
    const int steps = (L->C / kUnit + 1) / 2;
    auto tiles_of = [&](int tr, int tc) { return ((M + tr - 1) / tr) * (int64_t)((L->N + tc - 1) / tc); };
    // Where it measures faster than the tiled kernel: at most about one 64 x 64 tile per compute unit and a reduction of at
    // least 12 K-steps for the waves to split.  The tile shrinks while the blocks would leave half the compute units idle.
    if (g_force_tile_splitk < 0 && (tiles_of(64, 64) > (int64_t)num_cu || steps < 12)) return FLEXIQ_OK;
    int shape = g_force_tile_splitk >= 2 ? g_force_tile_splitk - 2 : tiles_of(64, 64) * 2 > num_cu ? 0 : tiles_of(32, 64) * 2 > num_cu ? 1 : 2;
    if (shape > 2) return FLEXIQ_EINVAL;
    const int tr = shape == 0 ? 64 : 32, tc = shape == 2 ? 32 : 64;
    if (tiles_of(tr, tc) > 0x7fffffff || (M + tr - 1) / tr > 65535) return FLEXIQ_OK;
    const size_t lds = shape == 2 ? 64 * 1024 : 128 * 1024;   // waves x fragments x 1 KB
    if (!g_tile_splitk_ready[L->device]) return FLEXIQ_OK;   // (set up when the first layer is packed on the device)
    RowsParams p = {};
    p.X = X; p.W8 = L->d_w8;
    p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift;
    p.cs = L->d_cs;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = (int)M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.units = L->C / kUnit;
    p.units4 = L->max_4bit_ch / kUnit;
    p.x_pre = L->x_prelowered || X6 ? 1 : 0;   // (FP6 calls: the 4-bit channels beyond the FP6 ones arrive lowered)
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.steps = steps;
    p.w4x_delta = L->U * 32 * L->Npad;
    if (lower && lower->ashift) {
        p.next_ashift = lower->ashift; p.next_K4 = lower->K4; p.next_gs_log2 = lower->gs_log2;
        if (X6 && lower->x6) { p.nx6 = lower->x6; p.next_K6 = lower->K6; p.next_S = lower->S; }
    }
    const dim3 grid((unsigned)((L->N + tc - 1) / tc), (unsigned)((M + tr - 1) / tr));
    if (X6) {
        p.X6 = X6; p.W6 = L->d_w6; p.W6S = L->d_w6s;
        p.s6 = K6 / 64;
        if (shape == 0) hipLaunchKernelGGL((k_tile_splitk<4, 4, 8, 2, true>), grid, dim3(512), lds, (hipStream_t)stream, p);
        else if (shape == 1) hipLaunchKernelGGL((k_tile_splitk<2, 4, 8, 4, true>), grid, dim3(512), lds / 2, (hipStream_t)stream, p);   // (eight waves: registers)
        else hipLaunchKernelGGL((k_tile_splitk<2, 2, 16, 4, true>), grid, dim3(1024), lds, (hipStream_t)stream, p);
    } else if (shape == 0) hipLaunchKernelGGL((k_tile_splitk<4, 4, 8, 2>), grid, dim3(512), lds, (hipStream_t)stream, p);
    else if (shape == 1) hipLaunchKernelGGL((k_tile_splitk<2, 4, 16, 2>), grid, dim3(1024), lds, (hipStream_t)stream, p);
    else hipLaunchKernelGGL((k_tile_splitk<2, 2, 16, 4>), grid, dim3(1024), lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    *taken = 1 + shape;
    g_last_tile_splitk = 1 + shape;
    g_last_rows = 0;
    return FLEXIQ_OK;
}

// Launches k_tile_splitk for a linear call of more than 32 rows whose output tiles leave most compute units idle on a long
// reduction; *taken = 0: the call was left to the other kernels, else 1 / 2 / 3: tiles of 64 x 64 / 32 x 64 / 32 x 32.
int launch_tile_splitk(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int num_cu, int *taken,
                       const LowerArgs *lower)
{
    return launch_tile_any(L, X, nullptr, 0, M, out, stream, num_cu, taken, lower);
}

// The same for the FP6 variant of the 4-bit phase: X holds the lowered activations, X6 the FP6 codes of the leading K6 channels.
int launch_tile_splitk_fp6(const flexiq_layer *L, const int8_t *X, const uint8_t *X6, int64_t M, const flexiq_out *out, void *stream, int K6,
                           int num_cu, int *taken, const LowerArgs *lower)
{
    *taken = 0;
    if (!X6 || K6 < 0 || (K6 & 63)) return FLEXIQ_OK;
    return launch_tile_any(L, X, X6, K6, M, out, stream, num_cu, taken, lower);
}

}  // namespace flexiq

extern "C" int flexiq_debug_force_few_rows(int mode)
{
    // (mode 14: the dot-product kernel with 4 column groups per block where rows and padding allow)
    if (mode == 14) {
        flexiq::smallm::g_force_cg = 4;
        mode = 2;
    } else {
        flexiq::smallm::g_force_cg = 0;
    }
    if (mode < -1 || mode > 2) return FLEXIQ_EINVAL;
    flexiq::smallm::g_force_rows = mode;
    return flexiq::smallm::g_last_rows;
}

extern "C" int flexiq_debug_force_tile_splitk(int mode)
{
    if (mode < -1 || mode > 4) return FLEXIQ_EINVAL;
    flexiq::smallm::g_force_tile_splitk = mode;
    return flexiq::smallm::g_last_tile_splitk;
}
