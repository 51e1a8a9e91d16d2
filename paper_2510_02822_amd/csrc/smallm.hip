// Few-row calls of the mixed GEMM (at most 64 activation rows): the regime in which the call is a stream of the
// weight matrix and nothing else matters, i.e. the one place where the integer path on gfx950 gets cheaper as the
// low-bit ratio rises (Section 7: 4-bit groups move half the weight bytes).
//
// The tiled kernel launches one block per 64 x 64 output tile here: 16 to 64 blocks on 256 compute units, each
// walking the whole reduction.  This kernel splits the reduction across blocks instead (split-K): a block owns 128
// output columns (four waves x 32) and one slice of the channel units, so that every compute unit streams its share of
// the weights; the partial sums of a column tile meet in a caller-provided workspace, and the block that arrives
// last (a ticket per column tile) adds them up and runs the epilogue.  Nothing goes through LDS: the packed weight
// layouts are already in MFMA fragment order, so a wave's weight fragment of a 32-channel unit is one contiguous,
// fully coalesced load per k-plane straight into the operand registers:
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
typedef int v16i __attribute__((ext_vector_type(16)));
typedef short v2s __attribute__((ext_vector_type(2)));

struct Params {
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
    int32_t splits;         // slices of the reduction
    int32_t units_per_split;
    uint32_t *tickets;      // [column tiles] (a 128-byte line each), zero between calls
    int32_t *partial;       // [column tiles][splits][4 waves][MF * 16][64] partial sums
};

constexpr int kCols = 128;   // output columns per block
constexpr int kTicketStride = 32;   // 32-bit words between two tickets: one 128-byte line each (atomics on one line queue up)
constexpr int kTicketBytes = 1024 * kTicketStride * 4;   // up to 1024 column tiles

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

template <int MF>   // 32-row fragments of activations: 1 (M <= 32) or 2 (M <= 64)
__global__ __launch_bounds__(256) void k_small_m(const Params p)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fh = lane >> 5;
    const int tile = blockIdx.x / p.splits, split = blockIdx.x % p.splits;
    const int n = tile * kCols + wave * 32 + fr;          // this lane's weight row (output channel); < Npad
    const int u0 = split * p.units_per_split, u1 = min(p.units, u0 + p.units_per_split);

    v16i acc[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[f][i] = 0;
    // activation positions of this block's units, one per lane (a slice has at most 64 units): read once, so that no
    // unit waits for a table look-up
    const int sa_lane = (u0 + lane < p.units4 && !p.x_pre) ? p.ashift[(u0 + lane) >> p.gs_shift] : 0;

    // one unit: weight fragment (16 channels 16 fh .. of the unit for output channel n), activation fragments (rows
    // 32 f + fr, the same 16 channels), one MFMA per fragment
    auto load_w = [&](int u, v4i &w8, v2i &w4, int &sw) {
        if (u < p.units4) {
            w4 = *reinterpret_cast<const v2i *>(p.W4 + ((int64_t)u * p.Npad + n) * 16 + 8 * fh);
            sw = p.wshift[(int64_t)(u >> p.gs_shift) * p.Npad + n];
        } else {
            w8 = *reinterpret_cast<const v4i *>(p.W8 + (((int64_t)u * 2 + fh) * p.Npad + n) * 16);
        }
    };
    auto load_x = [&](int u, v4i(&x)[MF]) {
#pragma unroll
        for (int f = 0; f < MF; ++f) {
            const int m = 32 * f + fr;
            x[f] = m < p.M ? *reinterpret_cast<const v4i *>(p.X + (int64_t)m * p.C + u * 32 + 16 * fh) : (v4i){0, 0, 0, 0};
        }
    };
    auto compute = [&](int u, v4i w8, v2i w4, int sw, v4i(&x)[MF]) {
        v4i w = w8;
        if (u < p.units4) {
            // dword e of the unit's 16 code bytes carries channels 8 e .. 8 e + 3 in the low halves of its bytes and
            // 8 e + 4 .. 8 e + 7 in the high halves; this lane holds dwords 2 fh and 2 fh + 1
            w = (v4i){(int)expand4((uint32_t)w4.x << 4, sw), (int)expand4((uint32_t)w4.x, sw), (int)expand4((uint32_t)w4.y << 4, sw),
                      (int)expand4((uint32_t)w4.y, sw)};
            if (!p.x_pre) {
                const int sa = __builtin_amdgcn_readlane(sa_lane, u - u0);
#pragma unroll
                for (int f = 0; f < MF; ++f)
                    x[f] = (v4i){(int)lower4((uint32_t)x[f].x, sa), (int)lower4((uint32_t)x[f].y, sa), (int)lower4((uint32_t)x[f].z, sa),
                                 (int)lower4((uint32_t)x[f].w, sa)};
            }
        }
#pragma unroll
        for (int f = 0; f < MF; ++f) acc[f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x[f], acc[f], 0, 0, 0);
    };

    // several units in flight: all loads of a group are issued before the first is used
    constexpr int UN = MF == 1 ? 8 : 4;
    int u = u0;
    for (; u + UN <= u1; u += UN) {
        v4i w8[UN], x[UN][MF];
        v2i w4[UN];
        int sw[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            w8[k] = (v4i){0, 0, 0, 0};
            w4[k] = (v2i){0, 0};
            sw[k] = 0;
            load_w(u + k, w8[k], w4[k], sw[k]);
            load_x(u + k, x[k]);
        }
#pragma unroll
        for (int k = 0; k < UN; ++k) compute(u + k, w8[k], w4[k], sw[k], x[k]);
    }
    for (; u < u1; ++u) {
        v4i w8 = {0, 0, 0, 0}, x[MF];
        v2i w4 = {0, 0};
        int sw = 0;
        load_w(u, w8, w4, sw);
        load_x(u, x);
        compute(u, w8, w4, sw, x);
    }

    // ---- partial sums of the column tile meet in the workspace; the block that arrives last adds them up.
    // No release / acquire fence is used: at device scope a release fence writes back the whole L2 and an acquire
    // fence invalidates it (measured: 4 us per block, one after the other).  Instead the partial sums are written
    // with device-coherent stores (written through to the device's coherence point) and read with device-coherent
    // loads (which bypass the cache levels that are not coherent across the chip); a block waits until its stores
    // have been performed (vmcnt = 0) before it draws its ticket, so whoever draws the last ticket finds them all.
    if (p.splits > 1) {
        __shared__ int last;
        constexpr int kCoherent = 16;   // cache policy of a buffer access: sc1 = device scope
        const int per_block = 4 * MF * 16 * 64;   // dwords
        const __amdgpu_buffer_rsrc_t rp =
            __builtin_amdgcn_make_buffer_rsrc((void *)(p.partial + (int64_t)tile * p.splits * per_block), 0, p.splits * per_block * 4, 0x00020000);
        const int my_off = ((split * 4 + wave) * (MF * 16 * 64) + lane) * 4;
#pragma unroll
        for (int f = 0; f < MF; ++f)
#pragma unroll
            for (int i = 0; i < 16; ++i) __builtin_amdgcn_raw_buffer_store_b32(acc[f][i], rp, my_off + (f * 16 + i) * 256, 0, kCoherent);
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0): this wave's stores have been performed
        __syncthreads();
        if (tid == 0) last = atomicAdd(p.tickets + tile * kTicketStride, 1u) == (unsigned)p.splits - 1u;
        __syncthreads();
        if (!last) return;
        // the other slices' shares (this block's own is still in its registers): the loads of several slices are in
        // flight together, so that the sum costs one or two trips to memory, not one per slice
        constexpr int CH = MF == 1 ? 8 : 4;
        for (int s0 = 0; s0 < p.splits; s0 += CH) {
            int t[CH][MF * 16];
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                const int s = s0 + k;
                // (a slice that does not exist, or this block's own, reads past the window: zeros)
                const int off = (s < p.splits && s != split) ? ((s * 4 + wave) * (MF * 16 * 64) + lane) * 4 : 0x7f000000;
#pragma unroll
                for (int j = 0; j < MF * 16; ++j) t[k][j] = __builtin_amdgcn_raw_buffer_load_b32(rp, off, j * 256, kCoherent);
            }
#pragma unroll
            for (int k = 0; k < CH; ++k)
#pragma unroll
                for (int f = 0; f < MF; ++f)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[f][i] += t[k][f * 16 + i];
        }
        if (tid == 0) __hip_atomic_store(p.tickets + tile * kTicketStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    }

    // ---- epilogue.  Lane: row 32 f + fr; accumulator register 4 g + i: output channel n0 + 8 g + 4 fh + i
    const int n0 = tile * kCols + wave * 32;
#pragma unroll
    for (int f = 0; f < MF; ++f) {
        const int m = 32 * f + fr;
        if (m >= p.M) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int nn = n0 + 8 * g + 4 * fh + i;
                if (nn >= p.N) continue;
                const int v = acc[f][4 * g + i];
                const int64_t o = (int64_t)m * p.N + nn;
                const float c = p.cs[nn], b = p.cs[p.Npad + nn];
                if (p.acc) p.acc[o] = v;
                if (p.y) p.y[o] = __builtin_fmaf((float)v, c, b);
                if (p.q) {
                    // offset form, as in the tiled kernel: round to nearest-even, saturate to 0..255, flip the top bit
                    const float t = __builtin_fmaf((float)v, c * p.r_out, b * p.r_out + 128.0f);
                    p.q[o] = (int8_t)(__builtin_amdgcn_cvt_pk_u8_f32(t, 0, 0u) ^ 0x80u);
                }
            }
    }
}


// ---- Few-row calls without a workspace: a block owns 16 output columns and the whole reduction.
//
// The split-K kernel above pays for the meeting of its slices in memory (store, ticket, re-read: three dependent trips).
// Here the slices of a column tile are the waves of one block (up to sixteen), which meet in LDS: every wave takes the
// K-steps (64 channels) wave, wave + waves, ... of the block's 16 columns, issues the loads of up to four of them at once
// (weight fragments straight into MFMA operand registers as above: 16 bytes per lane from the 8-bit tiles, or 8 bytes
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
                // (code layout as in k_small_m: this lane holds dwords 2 h and 2 h + 1 of the unit's 16 code bytes)
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

int64_t small_m_workspace_bytes(const flexiq_layer *L)
{
    const int64_t tiles = (L->N + smallm::kCols - 1) / smallm::kCols;
    // tickets, then partial sums for as many slices as there are 32-channel units at most 64 rows deep
    return smallm::kTicketBytes + tiles * (int64_t)(L->C / kUnit) * 4 * 2 * 16 * 64 * 4;
}

// Launches the split-K kernel for a linear call with at most 64 rows; `splits_out` gets the number of slices (0: the
// call was not taken, nothing was launched).
int launch_small_m(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int num_cu, int force_splits,
                   int *splits_out)
{
    using namespace smallm;
    Params p = {};
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
    const int tiles = (L->N + kCols - 1) / kCols;
    if (tiles > 1024) return FLEXIQ_EINVAL;   // tickets live in the first 128 KB of the workspace
    // enough slices to give about every fourth compute unit a block (more slices mean more partial sums to exchange:
    // measured, 64 blocks are the best trade on 256 compute units), at least eight units (256 channels) per slice
    int splits = force_splits > 0 ? force_splits : (num_cu / 4 + tiles - 1) / tiles;
    splits = std::max(1, std::min(splits, std::max(1, force_splits > 0 ? p.units / 2 : p.units / 8)));
    splits = std::max(splits, (p.units + 63) / 64);   // a slice holds at most 64 units (one position per lane)
    p.units_per_split = (p.units + splits - 1) / splits;
    splits = (p.units + p.units_per_split - 1) / p.units_per_split;
    if (splits > 1) {
        const int64_t need = kTicketBytes + (int64_t)tiles * splits * 4 * (M > 32 ? 2 : 1) * 16 * 64 * 4;
        if (!out->workspace || out->workspace_bytes < need || (reinterpret_cast<uintptr_t>(out->workspace) & 15u)) splits = 1;
    }
    if (splits == 1) {
        if (p.units > 64) {   // (cannot be served here: the caller runs the tiled kernel)
            if (splits_out) *splits_out = 0;
            return FLEXIQ_OK;
        }
        p.units_per_split = p.units;
    }
    p.splits = splits;
    p.tickets = reinterpret_cast<uint32_t *>(out->workspace);
    p.partial = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(out->workspace) + kTicketBytes);
    if (splits_out) *splits_out = splits;
    if (M > 32)
        hipLaunchKernelGGL(k_small_m<2>, dim3((unsigned)(tiles * splits)), dim3(256), 0, (hipStream_t)stream, p);
    else
        hipLaunchKernelGGL(k_small_m<1>, dim3((unsigned)(tiles * splits)), dim3(256), 0, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}

// Launches k_few_rows for a linear call with at most 64 rows; *taken = 0: the call was left to the other kernels.
int launch_few_rows(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, int *taken)
{
    using namespace smallm;
    *taken = 0;
    g_last_rows = 0;
    if (g_force_rows == 0 || M < 1 || M > 64) return FLEXIQ_OK;
    if (out->lower_for || out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
    if ((reinterpret_cast<uintptr_t>(X) & 15u) || (L->C & 15)) return FLEXIQ_OK;   // 16-byte activation pieces
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
