// Mixed GEMM whose 4-bit channel groups run on the FP6 matrix path of gfx950 (the variant of the 4-bit phase of
// Section 7 that gets a faster matrix instruction on this chip).
//
// gfx950 has no 4-bit integer MFMA, but v_mfma_scale_f32_32x32x64_f8f6f4 multiplies 6-bit floats (E2M3: sign, 2
// exponent bits with bias 1, 3 mantissa bits) at twice the rate of the int8 MFMA and takes one power-of-two scale
// (E8M0) per lane, i.e. per (row, 32-element block).  E2M3 holds k / 8 exactly for every integer |k| <= 15, as the
// bit pattern sign << 5 | |k|, so a bit-lowered 4-bit code L(v, s) in [-8, 7] is an exact FP6 value, a product of
// two of them is exact, and the block scale 2^(s + 3) of each operand puts the product back at
// 2^(sa + sw) * L(x, sa) * L(w, sw): the paper's shifted accumulation, done by the matrix instruction.  A group of
// 32 channels is exactly one scale block.  Measured on MI355X: the fp32 result of the instruction is the exact
// integer sum whenever every partial sum stays below 2^24 in magnitude (cancelling +-14336 pairs plus a lone 1,
// accumulators of +-(2^24 - 1), chains over K = 1024), and the instruction issues in the time of one
// v_mfma_i32_32x32x32_i8 while covering twice the reduction length.  The host certifies the 2^24 bound per layer
// from the packed weights and the extraction positions (see fp6_gemm.hip); channel groups beyond the certified
// prefix run on the int8 path.
//
// The K loop has two phases over the same accumulator registers: the FP6 K-steps of the leading K6 channels
// (fp32 accumulation of exact integers), a conversion fp32 -> int32 in place, then int8 K-steps for all other
// channels (4-bit groups outside the FP6 prefix from the position-expanded copy with activations that arrive
// lowered, 8-bit groups as they are).  Nothing is lowered or expanded in this kernel: every operand tile is a plain
// copy from global memory straight into LDS (buffer loads that write LDS), three K-steps ahead of its use, into a
// ring of four stages.  FP6 operands arrive packed by the producing layer (or by the stand-alone lowering kernel):
//   * a K-step is 64 channels = two units of 32; the 32 codes of a (row, unit) are 24 bytes; the first 16 bytes of
//     unit h form "plane h", the last 8 bytes of both units share "plane 2" (unit h in half h ^ ((row >> 4) & 1),
//     which makes the 8-byte fragment reads of 32 consecutive rows hit 32 different bank pairs);
//   * global layout of both operands: [block of 64 rows][K-step][plane][64 rows][16 bytes], so that one wave
//     instruction copies one plane of 64 rows (1 KB, contiguous) and the LDS image is the same;
//   * element e of a unit holds channel 8 * ((e % 16) / 4) + 4 * (e / 16) + e % 4 of the unit: the order in which
//     a lane of the producing layer's epilogue owns its 16 output channels, so that it packs them without
//     exchanging data with other lanes (any fixed order is fine for a dot product).
// The MFMA "A" operand is the weight fragment and "B" the activation fragment: a lane owns four consecutive
// output channels of one output row.
#pragma once
#include <type_traits>

#include "flexiq_internal.h"

namespace flexiq {
namespace fp6 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
struct Hi2 { int a, b; };   // last 8 bytes of an FP6 fragment (two scalars: keeps the fragment arrays in registers)

struct Params {
    const int8_t *X;       // int8 [M][C], stored channel order; columns [K6, K4) lowered already, columns < K6 unused
    const uint8_t *X6;     // FP6 activations [ceil(M/64)][C/64][3][64][16]; only K-steps < K6/64 are read
    const int8_t *W8;      // 8-bit weights and, behind them, the position-expanded 4-bit copy (as in the int8 kernel)
    const uint8_t *W6;     // FP6 weights [C/64][3][Npad][16]
    const uint8_t *W6S;    // weight block scales [ceil(C/256)][Npad][2][4]: E8M0 bytes (130 + w_shift) of four consecutive K-steps
    const int32_t *ashift; // activation positions [G + 1]
    const float *cs;       // [2][Npad]: x_scale * w_scale, then bias
    int32_t *acc;
    float *y;
    int8_t *q;
    float r_out;
    int64_t M;
    int32_t N, Npad, C;
    int32_t K4, K6;        // 4-bit channels; of those, the leading K6 (multiple of 64) run as FP6
    int32_t gs_shift;      // log2(group_size / 32)
    int32_t U;             // units of the int8 weight layout (C / 32)
    int32_t tiles_m, tiles_n;
    int64_t x6_bytes;      // size of X6 (for the buffer window)
    // optional: write the int8 output for a consuming layer that runs this kernel too
    uint8_t *nx6;              // its FP6 activation buffer (columns < next_K6); null: plain int8 output only
    const int32_t *next_ashift;
    int32_t next_K4, next_K6, next_gs_log2, next_S;   // next_S = its C / 64
};

typedef __attribute__((address_space(3))) void *lds_ptr_t;
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t r, unsigned char *dst, int voff, int soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)dst, 16, voff, soff, 0, 0);
}

__device__ __forceinline__ void dma4(__amdgpu_buffer_rsrc_t r, void *dst, int voff, int soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)dst, 4, voff, soff, 0, 0);
}

#define FQ6_SB() __builtin_amdgcn_sched_barrier(0)
// Keeps a matrix instruction where it is written: its result is pure data flow, and without an anchor the optimiser
// sinks it past the uniform branches of the step (towards its next use, a whole K-step later), which undoes the
// interleaving with the copies and fragment reads.  Emits no instruction.
#define FQ6_PIN(v) asm volatile("" : "+v"(v))
// matrix-instruction slots between two copies of a K-step (FP6 steps, int8 steps)
#define FQ6_SPREAD6 1
#define FQ6_SPREAD8 2

template <int WAVES_M, int WAVES_N, int TM, int TN>
struct Cfg {
    static constexpr int NW = WAVES_M * WAVES_N;
    static_assert(NW == 8, "eight waves per block: two per SIMD");
    static constexpr int NT = 64 * NW;
    static constexpr int BM = WAVES_M * TM * 32;
    static constexpr int BN = WAVES_N * TN * 32;
    static_assert(BM % 64 == 0 && BN % 64 == 0, "operand tiles are whole blocks of 64 rows");
    static constexpr int XP = (BM + 2) * 16;     // bytes per FP6 activation plane (+2 pieces: planes staggered over the banks)
    static constexpr int WP = (BN + 2) * 16;     // bytes per weight plane (FP6 and int8)
    static constexpr int X8 = BM * 64;           // int8 activation tile, row-major
    static constexpr int STAGE8 = X8 + 4 * WP;
    static constexpr int STAGE6 = 3 * XP + 3 * WP;
    static constexpr int STAGE = STAGE8 > STAGE6 ? STAGE8 : STAGE6;
    static constexpr int NSTAGE = 4;
    static constexpr int RING = NSTAGE * STAGE;
    // scales, biases, consumer positions (per column); activation positions (192 entries: three copy instructions);
    // weight block scales: per wave two sets (the current and the next group of four K-steps) of TN x 64 registers' worth
    static constexpr int WSC = NW * 2 * TN * 64 * 4;
    static constexpr int TABLE = 2 * BN * 4 + BN * 4 + 768 + WSC;
    static constexpr int LDS_BYTES = RING + TABLE;
    static_assert(LDS_BYTES <= 160 * 1024, "fits the CU's LDS");
    // copies per K-step (one wave instruction each = 1 KB)
    static constexpr int C6 = 3 * (BM / 64) + 3 * (BN / 64);       // FP6: activation planes, weight planes
    static constexpr int C8 = BM / 16 + 4 * (BN / 64);             // int8: 16 rows of activations; weight planes
    // per wave, at most: waves 0..3 share the activation copies, waves 4..7 the weight copies
    static constexpr int L6 = (3 * (BM / 64) + 3) / 4 > 3 ? (3 * (BM / 64) + 3) / 4 : 3;
    static constexpr int L8 = BM / 64 > 4 ? BM / 64 : 4;
};

template <int WAVES_M, int WAVES_N, int TM, int TN>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 1) void k_fp6(const Params p)
{
    using C_ = Cfg<WAVES_M, WAVES_N, TM, TN>;
    constexpr int NW = C_::NW, BM = C_::BM, BN = C_::BN, XP = C_::XP, WP = C_::WP, X8 = C_::X8, STAGE = C_::STAGE;
    constexpr int NF = TM + TN, NMF = TM * TN;
    constexpr int L6 = C_::L6, L8 = C_::L8;
    extern __shared__ __align__(16) unsigned char lds[];
    float *const cs_tab = reinterpret_cast<float *>(lds + C_::RING);          // [BN] scales, [BN] biases
    int *const nx_tab = reinterpret_cast<int *>(lds + C_::RING + 2 * BN * 4);  // [BN] consumer position of the column
    int *const as_tab = reinterpret_cast<int *>(lds + C_::RING + 3 * BN * 4);  // activation positions per group
    int *const ws_tab = reinterpret_cast<int *>(lds + C_::RING + 3 * BN * 4 + 768);   // weight block scales, see below

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    __builtin_assume(wave >= 0 && wave < NW);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- tile of this block.  Consecutive block ids land on different XCDs (each with its own L2), and inside a band
    // of 8 tile rows the tile column varies slowest: XCD x then computes tile row x of every band in all its columns,
    // so an activation row is fetched into one L2 only (every L2 needs the whole weight matrix in any case).
    int tile_m, tile_n;
    {
        const uint32_t b = blockIdx.x;
        const uint32_t band_sz = 8u * (uint32_t)p.tiles_n;
        const uint32_t band = b / band_sz, r = b - band * band_sz;
        const uint32_t rows_here = min(8u, (uint32_t)p.tiles_m - band * 8u);
        tile_m = (int)(band * 8u + r % rows_here);
        tile_n = (int)(r / rows_here);
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;
    const int rows_valid = (int)min((int64_t)BM, p.M - m0);

    constexpr int kRsrcFlags = 0x00020000;
    const int S = p.C >> 6;        // K-steps in all
    const int S6 = p.K6 >> 6;      // FP6 K-steps (the leading ones)

    // ---- copies of a K-step (one wave instruction each: 64 lanes x 16 bytes = 1 KB).  Waves 0..3 copy the activation
    // tile, waves 4..7 the weight tile: a wave then needs one buffer descriptor, one per-lane offset and a few scalars
    // per phase, and a K-step issues its copies with two scalar additions each.
    // FP6 K-step: 3 planes x BM/64 row blocks of activations (copy i of the tile = wave + 4 j: row block i % (BM/64),
    // plane i / (BM/64)); 3 planes x BN/64 blocks of weights (wave - 4 = block, j = plane).
    // int8 K-step: BM/16 pieces of 16 activation rows (piece wave + 4 j; lane: row lane/4, LDS slot lane%4, holding
    // k-plane slot ^ ((row/4)%4)); 4 planes x BN/64 blocks of weights (wave - 4 = block, j = plane).
    static_assert(BN == 256 && NW == 8, "four weight blocks of 64 rows, one per wave 4..7");
    constexpr int RB = BM / 64;
    constexpr int LMAX = L6 > L8 ? L6 : L8;
    const bool xwave = wave < 4;
    const int w4 = wave & 3;
    const int w4x_delta = p.U * 32 * p.Npad;   // from the 8-bit copy to the expanded 4-bit copy
    const int units4 = p.K4 >> 5;              // units whose weights come from the 4-bit copy
    __amdgpu_buffer_rsrc_t cdesc;      // the active phase: this wave's buffer
    int cvo = 0;                       // per-lane offset of copy 0 (copy j adds a scalar)
    int cso[LMAX], cd[LMAX];           // scalar offset of copy j at K-step 0; its LDS offset inside the stage
    int cstep = 0;                     // growth of the scalar offsets per K-step
    int ncopies = 0;                   // copies per K-step of this wave in the active phase
    bool mode8 = false;
    auto set_fp6_copies = [&]() {
        cdesc = xwave ? __builtin_amdgcn_make_buffer_rsrc((void *)p.X6, 0, (int)p.x6_bytes, kRsrcFlags)
                      : __builtin_amdgcn_make_buffer_rsrc((void *)p.W6, 0, S * 3 * p.Npad * 16, kRsrcFlags);
        cvo = lane * 16;
#pragma unroll
        for (int j = 0; j < LMAX; ++j) {
            const int i = w4 + 4 * j;
            const int rb = i % RB, pl = i / RB;
            cso[j] = xwave ? (int)(((m0 >> 6) + rb) * (int64_t)S * 3072) + pl * 1024 : (j * p.Npad + n0 + w4 * 64) * 16;
            cd[j] = xwave ? pl * XP + rb * 1024 : 3 * XP + j * WP + w4 * 1024;
        }
        cstep = xwave ? 3072 : 3 * p.Npad * 16;
        ncopies = xwave ? (3 * RB - w4 + 3) / 4 : 3;
        mode8 = false;
    };
    auto set_int8_copies = [&]() {
        cdesc = xwave ? __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + m0 * p.C), 0, rows_valid * p.C, kRsrcFlags)
                      : __builtin_amdgcn_make_buffer_rsrc((void *)p.W8, 0, 2 * p.U * 32 * p.Npad, kRsrcFlags);
        const int xq = (lane & 3) ^ ((lane >> 4) & 3);
        cvo = xwave ? (16 * w4 + (lane >> 2)) * p.C + xq * 16 : lane * 16;
#pragma unroll
        for (int j = 0; j < LMAX; ++j) {
            cso[j] = xwave ? j * 64 * p.C : ((j >> 1) * 2 + (j & 1)) * p.Npad * 16 + (n0 + w4 * 64) * 16;
            cd[j] = xwave ? (w4 + 4 * j) * 1024 : X8 + j * WP + w4 * 1024;
        }
        cstep = xwave ? 64 : 4 * p.Npad * 16;
        ncopies = xwave ? BM / 64 : 4;
        mode8 = true;
    };
    // Copies of K-step t into `stage`: issue_begin() says how many this wave has (0 when the K loop is over) and
    // switches the tables at the first int8 step; issue_item() issues copy j.  issue() does all of them at once.
    auto issue_begin = [&](int t) -> int {
        if (t >= S) return 0;
        if (t == S6) set_int8_copies();   // (t only ever grows: from here on every K-step is an int8 step)
        return ncopies;
    };
    auto issue_item = [&](int t, int j, int n, unsigned char *stage) {
        if (j < n) {
            // weights of an int8 K-step: unit j / 2 of the step may still be a 4-bit unit (then from the expanded copy)
            const int extra = mode8 && !xwave && (2 * t + (j >> 1)) < units4 ? w4x_delta : 0;
            dma16(cdesc, stage + cd[j], cvo, cso[j] + t * cstep + extra);
        }
    };
    auto issue = [&](int t, unsigned char *stage) -> int {
        const int n = issue_begin(t);
#pragma unroll
        for (int j = 0; j < LMAX; ++j) issue_item(t, j, n, stage);
        return n;
    };
    // waits until at most n of this wave's loads are outstanding (n: one of a few wave-uniform values)
    auto wait_vm = [&](int n) {
        switch (n) {
            case 0: __builtin_amdgcn_s_waitcnt(0x0070); break;
            case 1: __builtin_amdgcn_s_waitcnt(0x0071); break;
            case 2: __builtin_amdgcn_s_waitcnt(0x0072); break;
            case 3: __builtin_amdgcn_s_waitcnt(0x0073); break;
            case 4: __builtin_amdgcn_s_waitcnt(0x0074); break;
            case 5: __builtin_amdgcn_s_waitcnt(0x0075); break;
            case 6: __builtin_amdgcn_s_waitcnt(0x0076); break;
            case 7: __builtin_amdgcn_s_waitcnt(0x0077); break;
            case 8: __builtin_amdgcn_s_waitcnt(0x0078); break;
            default: __builtin_amdgcn_s_waitcnt(0x0079); break;
        }
    };
    static_assert(L6 + TN <= 9 && L8 + TN <= 9, "wait counts covered by wait_vm");

    // ---- prologue: tables (scales, biases, consumer positions per column, activation positions per group) and K-steps
    // 0, 1, 2 on their way, all straight into LDS
    {
        const __amdgpu_buffer_rsrc_t rcs = __builtin_amdgcn_make_buffer_rsrc((void *)p.cs, 0, 2 * p.Npad * 4, kRsrcFlags);
        const __amdgpu_buffer_rsrc_t ras = __builtin_amdgcn_make_buffer_rsrc((void *)p.ashift, 0, (p.C >> (5 + p.gs_shift)) * 4 + 4, kRsrcFlags);
        const __amdgpu_buffer_rsrc_t rnx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.next_ashift ? p.next_ashift : p.ashift), 0,
                                                                              p.next_ashift ? ((p.N >> p.next_gs_log2) + 1) * 4 : 0, kRsrcFlags);
        static_assert(BN <= 64 * NW, "one copy instruction per wave covers the tile's columns");
        if (wave * 64 < BN) {
            dma4(rcs, cs_tab + wave * 64, (wave * 64 + lane) * 4, n0 * 4);
            dma4(rcs, cs_tab + BN + wave * 64, (wave * 64 + lane) * 4, (p.Npad + n0) * 4);
            dma4(rnx, nx_tab + wave * 64, ((n0 + wave * 64 + lane) >> p.next_gs_log2) * 4, 0);
        }
        if (wave < 3) dma4(ras, as_tab + wave * 64, (wave * 64 + lane) * 4, 0);   // (past the table: zeros)
    }
    if (S6 > 0) set_fp6_copies();
    else set_int8_copies();
    (void)issue(0, lds);
    (void)issue(1, lds + STAGE);
    (void)issue(2, lds + 2 * STAGE);

    // ---- fragments
    const int fr = lane & 31, fh = lane >> 5;
    // FP6: 16 bytes of plane fh, 8 bytes of plane 2 (half fh ^ ((row >> 4) & 1)); row = fragment base + fr
    const int swz = (fr >> 4) & 1;   // fragment bases are multiples of 32: (row >> 4) & 1 = (fr >> 4) & 1
    const int x6_frag = fh * XP + (wm * TM * 32 + fr) * 16;
    const int x6_tail = 2 * XP + (wm * TM * 32 + fr) * 16 + 8 * (fh ^ swz);
    const int w6_frag = 3 * XP + fh * WP + (wn * TN * 32 + fr) * 16;
    const int w6_tail = 3 * XP + 2 * WP + (wn * TN * 32 + fr) * 16 + 8 * (fh ^ swz);
    // int8: row-major activation rows of 64 bytes, piece q of row R in slot q ^ ((R / 4) % 4); weight plane 2 kh + fh
    const int fsw = (fr >> 2) & 3;
    const int x8_frag0 = (wm * TM * 32 + fr) * 64 + ((fh ^ fsw) * 16);
    const int x8_frag1 = (wm * TM * 32 + fr) * 64 + (((2 + fh) ^ fsw) * 16);
    const int w8_frag = X8 + fh * WP + (wn * TN * 32 + fr) * 16;

    // Fragments, 16 + 8 bytes each.  Weights: two register sets used in turn (a weight fragment is needed until the
    // last row of matrix instructions of a step, and again at the very start of the next).  Activations: one set; a
    // fragment is re-read for the next step as soon as its row of matrix instructions has been issued.
    v4i wa_lo[TN], wb_lo[TN], x_lo[TM];
    Hi2 wa_hi[TN], wb_hi[TN], x_hi[TM];
    auto read6w = [&](v4i(&lo)[TN], Hi2(&hi)[TN], int i, const unsigned char *stage) {
        lo[i] = *reinterpret_cast<const v4i *>(stage + w6_frag + i * 512);
        const v2i t = *reinterpret_cast<const v2i *>(stage + w6_tail + i * 512);
        hi[i].a = t.x;
        hi[i].b = t.y;
    };
    auto read6x = [&](int i, const unsigned char *stage) {
        x_lo[i] = *reinterpret_cast<const v4i *>(stage + x6_frag + i * 512);
        const v2i t = *reinterpret_cast<const v2i *>(stage + x6_tail + i * 512);
        x_hi[i].a = t.x;
        x_hi[i].b = t.y;
    };
    auto op8 = [](const v4i &lo, const Hi2 &hi) { return (v8i){lo.x, lo.y, lo.z, lo.w, hi.a, hi.b, 0, 0}; };
    // Block scales (E8M0 bytes).  Weights: per fragment column and lane (output channel, unit) one 32-bit word holds
    // the bytes of four consecutive K-steps; a wave copies the words of its own columns straight into LDS a group of
    // four steps ahead (no register is the target of a memory load inside the K loop, so no wait for such a register
    // can ever drain the copies in flight) and reads the word of the current group at every step.
    // Activations: one word per group of four steps, built from the position table.
    const __amdgpu_buffer_rsrc_t rws = __builtin_amdgcn_make_buffer_rsrc((void *)p.W6S, 0, ((S + 3) >> 2) * p.Npad * 8, kRsrcFlags);
    int *const ws_mine = ws_tab + wave * (2 * TN * 64);
    auto fetch_wscales = [&](int grp) {   // words of group `grp` -> this wave's set grp % 2
#pragma unroll
        for (int a = 0; a < TN; ++a)
            dma4(rws, ws_mine + ((grp & 1) * TN + a) * 64, ((n0 + (wn * TN + a) * 32 + fr) * 2 + fh) * 4, grp * p.Npad * 8);
    };
    if (S6 > 0) fetch_wscales(0);

    v16f accf[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) accf[a][b][i] = 0.0f;

    // K-steps 0 and 1 have landed (and 2, the tables and the first weight scales)
    __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
    // When int8 is the only scaled output, the table's scales and biases become the requantisation multiplier and
    // addend (c * r_out, bias * r_out + 128: the same two roundings as in the general epilogue) once per column;
    // each thread rewrites the entries its own wave copied.
    const bool pre_scaled = p.q != nullptr && p.y == nullptr;
    if (pre_scaled && tid < BN) {
        const float c = cs_tab[tid], bv = cs_tab[BN + tid];
        cs_tab[tid] = c * p.r_out;
        cs_tab[BN + tid] = bv * p.r_out + 128.0f;
    }
    auto as_of = [&](int t) {   // activation block scales of K-steps 4 (t / 4) .. + 3 for this lane's unit
        int r = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) r |= (130 + as_tab[(2 * ((t & ~3) + k) + fh) >> p.gs_shift]) << (8 * k);
        return r;
    };

    // Two waves share a SIMD's matrix pipe, and the instruction arbiter prefers the older one: left alone it issues its
    // whole step back to back and then idles at the barrier while the younger one works through its step alone, too
    // slowly to keep the pipe full (measured: 530 of a step's 1740 cycles).  A wave's priority therefore falls as it
    // advances through the step, so that whichever of the two is behind wins and their matrix instructions alternate.
    auto set_prio = [](int g, int total) {   // g-th of `total` matrix instructions of a step (compile-time after unrolling)
        const int q = total / 4 > 0 ? total / 4 : 1;
        const int level = g / q < 3 ? 3 - g / q : 0;
        const int before = g == 0 ? -1 : ((g - 1) / q < 3 ? 3 - (g - 1) / q : 0);
        if (level != before) {
            if (level == 3) __builtin_amdgcn_s_setprio(3);
            else if (level == 2) __builtin_amdgcn_s_setprio(2);
            else if (level == 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
    };
    int o_cur = 0, o_nx1 = STAGE, o_nx2 = 2 * STAGE, o_nx3 = 3 * STAGE;
    auto rotate = [&]() {
        const int t = o_cur;
        o_cur = o_nx1; o_nx1 = o_nx2; o_nx2 = o_nx3; o_nx3 = t;
    };
    int s = 0;

    // ---- FP6 phase.  Step s multiplies the fragments in register set `cur` (read during the previous step) and
    // reads those of step s + 1 into the other set (after the last FP6 step that read brings bytes nobody uses),
    // while the copies of step s + 3 are issued.  The scale byte of step s is byte s % 4 of the scale registers.
    int as_cur = as_of(0);
    auto step6 = [&](v4i(&cur_lo)[TN], Hi2(&cur_hi)[TN], v4i(&nxt_lo)[TN], Hi2(&nxt_hi)[TN]) {
        const unsigned char *nx1 = lds + o_nx1;
        unsigned char *nx3 = lds + o_nx3;
        // at the first step of a group of four: the scale words of the next group (older than this step's copies, so
        // the wait at the end of the step, which lets only those stay in flight, covers them)
        if ((s & 3) == 0) fetch_wscales((s >> 2) + 1);
        const int ncp = issue_begin(s + 3);
        const int issued = ncp;
        const int sh = 8 * (s & 3);
        int wsc[TN];
#pragma unroll
        for (int a = 0; a < TN; ++a) wsc[a] = ws_mine[(((s >> 2) & 1) * TN + a) * 64 + lane] >> sh;
        const int asc = as_cur >> sh;
        FQ6_SB();
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int a = 0; a < TN; ++a) {
                const int slot = b * TN + a;
#pragma unroll
                for (int j = 0; j < LMAX; ++j)   // the copies of K-step s + 3, spread over the first matrix instructions
                    if ((j * FQ6_SPREAD6 < NMF ? j * FQ6_SPREAD6 : NMF - 1) == slot) {
                        issue_item(s + 3, j, ncp, nx3);
                        FQ6_SB();
                    }
                set_prio(slot, NMF);
                accf[a][b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(op8(cur_lo[a], cur_hi[a]), op8(x_lo[b], x_hi[b]), accf[a][b], 2, 2,
                                                                             0, wsc[a], 0, asc);
                FQ6_PIN(accf[a][b]);
                FQ6_SB();
                if (b == 0) {   // next step's weight fragments, early
                    read6w(nxt_lo, nxt_hi, a, nx1);
                    FQ6_SB();
                }
                if (a == TN - 1) {   // this activation fragment is done for this step
                    read6x(b, nx1);
                    FQ6_SB();
                }
            }
        if ((s & 3) == 3) as_cur = as_of(s + 1);
        // The copies of K-step s + 2 have landed (this step's own may stay in flight); nothing else has to be
        // complete at the barrier: the fragment reads issued above go to the next step's stage, which no copy touches
        // for two more steps, and every register they fill is waited for where it is used.
        wait_vm(issued);
        __builtin_amdgcn_s_barrier();
        FQ6_SB();
        rotate();
        ++s;
    };
    if (S6 > 0) {
#pragma unroll
        for (int k = 0; k < TN; ++k) read6w(wa_lo, wa_hi, k, lds);
#pragma unroll
        for (int k = 0; k < TM; ++k) read6x(k, lds);
        while (s + 1 < S6) {
            step6(wa_lo, wa_hi, wb_lo, wb_hi);
            step6(wb_lo, wb_hi, wa_lo, wa_hi);
        }
        if (s < S6) step6(wa_lo, wa_hi, wb_lo, wb_hi);
    }

    // ---- fp32 -> int32 in place: the sums are exact integers below 2^24
    v16i acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = (int)accf[a][b][i];

    // ---- int8 phase: two k-halves per K-step, register set ga for the first, gb for the second (the read ahead of
    // the last step brings bytes nobody uses)
    v4i ga[NF], gb[NF];
    auto read8 = [&](v4i(&f)[NF], int i, const unsigned char *stage, int kh) {
        if (i < TN) f[i] = *reinterpret_cast<const v4i *>(stage + w8_frag + kh * 2 * WP + i * 512);
        else f[i] = *reinterpret_cast<const v4i *>(stage + (kh ? x8_frag1 : x8_frag0) + (i - TN) * 2048);
    };
    if (s < S) {
#pragma unroll
        for (int k = 0; k < NF; ++k) read8(ga, k, lds + o_cur, 0);
        while (s < S) {
            const unsigned char *cur = lds + o_cur;
            const unsigned char *nx1 = lds + o_nx1;
            unsigned char *nx3 = lds + o_nx3;
            const int issued = issue_begin(s + 3);
            FQ6_SB();
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int b = 0; b < TM; ++b)
#pragma unroll
                    for (int a = 0; a < TN; ++a) {
                        const int slot = b * TN + a;
#pragma unroll
                        for (int j = 0; j < LMAX; ++j)
                            if ((j * FQ6_SPREAD8 < 2 * NMF ? j * FQ6_SPREAD8 : 2 * NMF - 1) == kh * NMF + slot) {
                                issue_item(s + 3, j, issued, nx3);
                                FQ6_SB();
                            }
                        set_prio(kh * NMF + slot, 2 * NMF);
                        if (kh == 0) acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ga[a], ga[TN + b], acc[a][b], 0, 0, 0);
                        else acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gb[a], gb[TN + b], acc[a][b], 0, 0, 0);
                        FQ6_PIN(acc[a][b]);
                        FQ6_SB();
#pragma unroll
                        for (int k = 0; k < NF; ++k)
                            if (k * NMF / NF == slot) {
                                if (kh == 0) read8(gb, k, cur, 1);
                                else read8(ga, k, nx1, 0);
                                FQ6_SB();
                            }
                    }
            wait_vm(issued);
            __builtin_amdgcn_s_barrier();
            FQ6_SB();
            rotate();
            ++s;
        }
    }

    // ---- epilogue.  Lane: output row m = tile row 32 b + fr of its wave; per accumulator quad g the four
    // consecutive output channels 32 a + 8 g + 4 fh + i.  The int8 code is formed in offset form: one fused
    // multiply-add, then one instruction rounds to nearest-even, saturates to 0..255 and inserts the byte; flipping the
    // top bits gives the two's-complement code.
    const bool want_q = p.q != nullptr, want_y = p.y != nullptr, want_acc = p.acc != nullptr;
    const bool n_vec = (p.N & 3) == 0;
    const bool q_rows = want_q && (p.N & 15) == 0;
    const bool chain = p.nx6 != nullptr;     // FP6 codes for the consumer's leading channels
    if (q_rows && !want_y && !want_acc && p.next_ashift == nullptr) {
        // the common case: int8 only, plain codes, rows of 16-byte pieces
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            const int nl0 = (wn * TN + a) * 32 + 4 * fh;
            uint32_t qrow[TM][4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 mu = *reinterpret_cast<const float4 *>(cs_tab + nl0 + 8 * g);
                const float4 ad = *reinterpret_cast<const float4 *>(cs_tab + BN + nl0 + 8 * g);
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    uint32_t qw = 0;
                    qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[a][b][4 * g], mu.x, ad.x), 0, qw);
                    qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[a][b][4 * g + 1], mu.y, ad.y), 1, qw);
                    qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[a][b][4 * g + 2], mu.z, ad.z), 2, qw);
                    qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[a][b][4 * g + 3], mu.w, ad.w), 3, qw);
                    qrow[b][g] = qw ^ 0x80808080u;
                }
            }
            // The two halves of the wave hold alternating 4-byte pieces of a row: exchanging quads 0 <-> 2 and 1 <-> 3
            // between them leaves lanes 0..31 with channels 0..15 of the fragment's 32 and lanes 32..63 with 16..31.
#pragma unroll
            for (int b = 0; b < TM; ++b) {
                const auto s02 = __builtin_amdgcn_permlane32_swap(qrow[b][0], qrow[b][2], false, false);
                const auto s13 = __builtin_amdgcn_permlane32_swap(qrow[b][1], qrow[b][3], false, false);
                const v4i piece = (v4i){(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
                const int64_t m = m0 + (wm * TM + b) * 32 + fr;
                const int n = n0 + (wn * TN + a) * 32 + 16 * fh;
                if (m < p.M && n < p.N) *reinterpret_cast<v4i *>(p.q + m * p.N + n) = piece;
            }
        }
        return;
    }
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int nl0 = (wn * TN + a) * 32 + 4 * fh;
        const int ncol = n0 + (wn * TN + a) * 32;        // first column of the fragment column: one unit of the consumer
        const bool to6 = chain && ncol < p.next_K6;      // this unit goes out as FP6 codes
        const bool low8 = p.next_ashift != nullptr && !to6 && ncol < p.next_K4;   // int8, lowered for the consumer
        const int sp = nx_tab[(wn * TN + a) * 32];        // consumer's position of this unit's group
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int64_t m = m0 + (wm * TM + b) * 32 + fr;
            const bool m_ok = m < p.M;
            uint32_t qrow[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int nl = nl0 + 8 * g;
                const int n = n0 + nl;
                const float4 cs = *reinterpret_cast<const float4 *>(cs_tab + nl);
                const float4 bi = *reinterpret_cast<const float4 *>(cs_tab + BN + nl);
                const float csv[4] = {cs.x, cs.y, cs.z, cs.w}, biv[4] = {bi.x, bi.y, bi.z, bi.w};
                const int iv[4] = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                uint32_t qw = 0;
                if (want_q) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float mul = pre_scaled ? csv[i] : csv[i] * p.r_out, add = pre_scaled ? biv[i] : biv[i] * p.r_out + 128.0f;
                        float t = __builtin_fmaf((float)iv[i], mul, add);
                        // for the consumer's 4-bit channels: clamp to its 4-bit range at its position
                        if (to6 || low8) t = __builtin_amdgcn_fmed3f(t, (float)(128 - (8 << sp)), (float)(127 + (8 << sp)));
                        qw = __builtin_amdgcn_cvt_pk_u8_f32(t, i, qw);
                    }
                    qw ^= 0x80808080u;
                    if (low8) qw &= 0x01010101u * ((0xFFu << sp) & 0xFFu);
                    qrow[g] = qw;
                }
                if (!(want_y || want_acc || (want_q && !q_rows))) continue;
                if (!m_ok || n >= p.N) continue;
                const int64_t o = m * p.N + n;
                if (n_vec) {
                    if (want_acc) *reinterpret_cast<v4i *>(p.acc + o) = (v4i){iv[0], iv[1], iv[2], iv[3]};
                    if (want_y) {
                        float4 y;
                        y.x = __builtin_fmaf((float)iv[0], csv[0], biv[0]);
                        y.y = __builtin_fmaf((float)iv[1], csv[1], biv[1]);
                        y.z = __builtin_fmaf((float)iv[2], csv[2], biv[2]);
                        y.w = __builtin_fmaf((float)iv[3], csv[3], biv[3]);
                        *reinterpret_cast<float4 *>(p.y + o) = y;
                    }
                    if (want_q && !q_rows) *reinterpret_cast<uint32_t *>(p.q + o) = qw;
                } else {
                    for (int i = 0; i < 4 && n + i < p.N; ++i) {
                        if (want_acc) p.acc[o + i] = iv[i];
                        if (want_y) p.y[o + i] = __builtin_fmaf((float)iv[i], csv[i], biv[i]);
                        if (want_q) p.q[o + i] = (int8_t)((qw >> (8 * i)) & 0xFF);
                    }
                }
            }
            if (want_q && to6) {
                // The lane's 16 codes (clamped above to the consumer's 4-bit range at its position sp) -> 16 FP6
                // elements of the consumer's unit, in the lane's own order: sign << 5 | |L(code, sp)|.
                // With u = code + 128 (the offset form): floor(code / 2^sp) + 8 = (u >> sp) - ((128 >> sp) - 8), a
                // value 0..15 per byte, no borrows.
                uint32_t w24[4];
                const uint32_t kbias = 0x01010101u * (uint32_t)((128 >> sp) - 8);
                const uint32_t kmask = 0x01010101u * (0xFFu >> sp);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t cb = (((qrow[g] ^ 0x80808080u) >> sp) & kmask) - kbias;   // 4-bit code + 8 per byte
                    const uint32_t neg = (~cb >> 3) & 0x01010101u;                           // code < 0
                    const uint32_t mag = ((cb & 0x07070707u) ^ (neg * 7u)) + neg;            // |code|: cb - 8, or 8 - cb
                    const uint32_t c6 = mag | (neg << 5);                                    // E2M3 pattern of code / 8
                    w24[g] = (c6 & 0x3Fu) | ((c6 >> 2) & 0xFC0u) | ((c6 >> 4) & 0x3F000u) | ((c6 >> 6) & 0xFC0000u);
                }
                const uint32_t d0 = w24[0] | (w24[1] << 24), d1 = (w24[1] >> 8) | (w24[2] << 16), d2 = (w24[2] >> 16) | (w24[3] << 8);
                if (m_ok) {
                    const int u = ncol >> 5, t6 = u >> 1, hh = u & 1;
                    const int rr = (int)(m & 63);
                    uint8_t *blk = p.nx6 + ((m >> 6) * (int64_t)p.next_S + t6) * 3072;
                    if (fh == 0) {
                        uint32_t *d = reinterpret_cast<uint32_t *>(blk + hh * 1024 + rr * 16);
                        d[0] = d0; d[1] = d1; d[2] = d2;
                    } else {
                        *reinterpret_cast<uint32_t *>(blk + hh * 1024 + rr * 16 + 12) = d0;
                        uint32_t *d = reinterpret_cast<uint32_t *>(blk + 2 * 1024 + rr * 16 + 8 * (hh ^ ((rr >> 4) & 1)));
                        d[0] = d1; d[1] = d2;
                    }
                }
            } else if (q_rows) {
                const auto s02 = __builtin_amdgcn_permlane32_swap(qrow[0], qrow[2], false, false);
                const auto s13 = __builtin_amdgcn_permlane32_swap(qrow[1], qrow[3], false, false);
                const v4i piece = (v4i){(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
                const int n = n0 + (wn * TN + a) * 32 + 16 * fh;
                if (m_ok && n < p.N) *reinterpret_cast<v4i *>(p.q + m * p.N + n) = piece;
            }
        }
    }
}

typedef void (*kernel_fn)(const Params);
struct Shape {
    int BM, BN, threads, lds;
    kernel_fn fn;
};
template <int WAVES_M, int WAVES_N, int TM, int TN>
inline Shape make_shape()
{
    using C_ = Cfg<WAVES_M, WAVES_N, TM, TN>;
    return Shape{C_::BM, C_::BN, C_::NT, C_::LDS_BYTES, k_fp6<WAVES_M, WAVES_N, TM, TN>};
}

}  // namespace fp6
}  // namespace flexiq
