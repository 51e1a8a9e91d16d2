// Few-row calls of the mixed GEMM (at most 64 activation rows): the regime in which the call is a stream of the
// weight matrix and little else, i.e. the one place where the integer path on gfx950 moves fewer bytes as the
// low-bit ratio rises (Section 7: 4-bit groups move half the weight bytes).
//
// The tiled kernel launches one block per 64 x 64 output tile here: 16 to 64 blocks on 256 compute units, each
// walking the whole reduction alone.  The kernel below gives a block 16 output columns and splits the reduction over
// its waves.  Nothing but the partial sums goes through LDS: the packed weight layouts are already in MFMA fragment
// order, so a wave's weight fragment of a K-step is a coalesced load per 16-channel quarter straight into the operand
// registers:
//   * 8-bit units: 16 bytes per lane from the 8-bit tiles;
//   * 4-bit units: 8 bytes per lane of packed 4-bit codes (half the bytes) plus one position byte, expanded in
//     registers to code << w_shift; the activations of those units are bit-lowered in registers (unless they arrive
//     lowered), exactly as in the tiled kernel: same int8 MFMA, same int32 accumulators, bit-identical results.
#include <algorithm>

#include "flexiq_internal.h"

namespace flexiq {
namespace smallm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef short v2s __attribute__((ext_vector_type(2)));

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

// four 4-bit codes in the high halves of the bytes of p -> four int8 values code << sw
__device__ __forceinline__ uint32_t expand4(uint32_t p, int sw)
{
    const short t = (short)(4 - sw);
    v2s o = __builtin_bit_cast(v2s, p);
    v2s e = o << (short)8;
    o = o >> t;   // arithmetic: sign-extends the code, leaves junk only below bit sw and in the low byte
    e = e >> t;
    const uint32_t r = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u);
    return r & (0x01010101u * ((0xFFu << sw) & 0xFFu));
}

// ---- A block owns 16 output columns and the whole reduction.
//
// Splitting the reduction across blocks makes the slices meet in memory (store, ticket, re-read: three dependent trips;
// built and measured: ViT-L fc2 with 16 rows took 11 us that way, 4.7 us this way).  Here the slices of a column tile
// are the waves of one block (up to sixteen), which meet in LDS: every wave takes the
// K-steps (64 channels) wave, wave + waves, ... of the block's 16 columns, issues the loads of up to four of them at once
// (weight fragments straight into MFMA operand registers: 16 bytes per lane from the 8-bit tiles, or 8 bytes
// of packed codes and a position byte for 4-bit units), multiplies with `v_mfma_i32_16x16x64_i8` (lane: weight row
// n0 + lane % 16 resp. activation row 16 f + lane % 16, channels 16 (lane / 16) ... of the K-step) and leaves its
// accumulators in LDS; waves 0 .. MF-1 add them up and run the epilogue of one 16-row fragment each.  One trip to memory
// for the operands and one for the outputs; nothing to zero, nothing to hand in.
struct RowsParams {
    const int8_t *X;        // int8 [M][C], stored channel order
    const int8_t *W8;       // [U][2][Npad][16]
    const uint8_t *W4;      // [U][Npad][16] packed 4-bit codes
    const uint8_t *wshift;  // [G + 1][Npad]
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
};

constexpr int kRowCols = 16;   // output columns per block

template <int MF>   // 16-row fragments of activations: M <= 16 MF
__global__ __launch_bounds__(1024) void k_few_rows(const RowsParams p)
{
    extern __shared__ __align__(16) unsigned char lds[];   // [waves][MF][64 lanes] accumulator quads
    v4i *const red = reinterpret_cast<v4i *>(lds);
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

    v4i acc[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f) acc[f] = (v4i){0, 0, 0, 0};

    constexpr int UN = MF <= 2 ? 4 : 2;   // K-steps in flight per wave
    for (int ks0 = wave; ks0 < p.steps; ks0 += nw * UN) {
        v4i w8[UN], x[UN][MF];
        v2i w4[UN];
        int sw[UN], sa[UN];
        bool low[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int ks = ks0 + k * nw;
            const int u = 2 * ks + (qd >> 1), h = qd & 1;   // this lane's unit and k-half
            const bool valid = ks < p.steps && u < p.units;
            low[k] = valid && u < p.units4;
            w8[k] = (v4i){0, 0, 0, 0};
            w4[k] = (v2i){0, 0};
            sw[k] = sa[k] = 0;
            if (low[k]) {
                w4[k] = *reinterpret_cast<const v2i *>(p.W4 + ((int64_t)u * p.Npad + n) * 16 + 8 * h);
                sw[k] = p.wshift[(int64_t)(u >> p.gs_shift) * p.Npad + n];
                if (!p.x_pre) sa[k] = p.ashift[u >> p.gs_shift];
            } else if (valid) {
                w8[k] = *reinterpret_cast<const v4i *>(p.W8 + (((int64_t)u * 2 + h) * p.Npad + n) * 16);
            }
#pragma unroll
            for (int f = 0; f < MF; ++f) {
                const int m = 16 * f + c;
                x[k][f] = valid && m < p.M ? *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + u * 32 + 16 * h) : (v4i){0, 0, 0, 0};
            }
        }
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            v4i w = w8[k];
            if (low[k]) {
                // dword e of the unit's 16 code bytes carries channels 8 e .. 8 e + 3 in the low halves of its bytes and
                // 8 e + 4 .. 8 e + 7 in the high halves; this lane holds dwords 2 h and 2 h + 1
                w = (v4i){(int)expand4((uint32_t)w4[k].x << 4, sw[k]), (int)expand4((uint32_t)w4[k].x, sw[k]),
                          (int)expand4((uint32_t)w4[k].y << 4, sw[k]), (int)expand4((uint32_t)w4[k].y, sw[k])};
                if (!p.x_pre) {
#pragma unroll
                    for (int f = 0; f < MF; ++f)
                        x[k][f] = (v4i){(int)lower4((uint32_t)x[k][f].x, sa[k]), (int)lower4((uint32_t)x[k][f].y, sa[k]),
                                        (int)lower4((uint32_t)x[k][f].z, sa[k]), (int)lower4((uint32_t)x[k][f].w, sa[k])};
                }
            }
#pragma unroll
            for (int f = 0; f < MF; ++f) acc[f] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w, x[k][f], acc[f], 0, 0, 0);
        }
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
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        yv[i] = __builtin_fmaf((float)s[i], cs4[i], bi4[i]);
        // offset form, as in the tiled kernel: round to nearest-even, saturate to 0..255, flip the top bit
        qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)s[i], cs4[i] * p.r_out, bi4[i] * p.r_out + 128.0f), i, qw);
    }
    qw ^= 0x80808080u;
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

static int g_force_rows = -1;   // test hook: 1 = take k_few_rows whenever the call qualifies, 0 = never, -1 = automatic
static int g_last_rows = 0;

}  // namespace smallm

// Launches k_few_rows for a linear call with at most 64 rows; *taken = 0: the call was left to the other kernels.
int launch_few_rows(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int num_cu, int *taken)
{
    using namespace smallm;
    *taken = 0;
    g_last_rows = 0;
    if (g_force_rows == 0 || M < 1 || M > 64) return FLEXIQ_OK;
    if (out->lower_for || out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
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
    const int mf = (int)((M + 15) / 16);
    const int nw = p.steps >= 12 ? 16 : (p.steps >= 6 ? 8 : 4);
    const unsigned blocks = (unsigned)((L->N + kRowCols - 1) / kRowCols);
    const size_t lds = (size_t)nw * mf * 64 * 16;
    void (*fn)(const RowsParams) = mf == 1 ? k_few_rows<1> : (mf == 2 ? k_few_rows<2> : (mf == 3 ? k_few_rows<3> : k_few_rows<4>));
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(64 * nw), lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    *taken = 1;
    g_last_rows = 1;
    return FLEXIQ_OK;
}

}  // namespace flexiq

extern "C" int flexiq_debug_force_few_rows(int mode)
{
    if (mode < -1 || mode > 1) return FLEXIQ_EINVAL;
    flexiq::smallm::g_force_rows = mode;
    return flexiq::smallm::g_last_rows;
}
