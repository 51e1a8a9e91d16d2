// Mixed 4-bit / 8-bit GEMM and implicit-GEMM convolution for gfx950 (Section 7 of the paper,
// re-designed for CDNA4).
//
// gfx950 has no 4-bit integer matrix instruction, so a 4-bit channel group cannot run on a faster
// matrix path than an 8-bit one.  The group's contribution
//     2^(sa+sw) * sum_k L(x,sa) * L(w,sw)   =   sum_k (L(x,sa) << sa) * (L(w,sw) << sw)
// is instead formed by putting each bit-lowered operand back at its extraction position as an int8
// value (both factors fit: |L << s| <= 128) and feeding the same int8 MFMA and the same int32
// accumulator as the 8-bit groups: bit-exact by distributivity, and the separate shift-and-accumulate
// stage of the paper's CUDA kernel disappears.  A 4-bit group therefore costs the same matrix cycles as
// an 8-bit one; its weights can be streamed from the packed 4-bit copy (half the bytes) or, by default,
// from a copy that is already expanded (no vector-ALU work beside the matrix pipe).
//
// Work decomposition: a block of four waves (one per SIMD) or eight waves (two per SIMD: the second
// wave's MFMAs fill the issue slots the first one spends on copies, address updates and the epilogue)
// owns a BM x BN output tile; the reduction
// runs in K-steps of 64 elements (two 32-channel units, each independently 4-bit or 8-bit), each
// K-step being two k-halves of v_mfma_i32_32x32x32_i8 (a single wave per SIMD keeps the matrix pipe
// full with this instruction shape; the 16x16x64 shape needs two).  Operand tiles live in an LDS ring of
// four stages and arrive there, three K-steps ahead of their use, by one of two routes:
//   * straight from global memory (buffer loads that write LDS, no register hop): every weight tile that
//     needs no arithmetic (8-bit units; 4-bit units from the position-expanded copy) and the activation tile
//     of an all-8-bit K-step;
//   * through registers, where the vector ALU bit-lowers the activations of 4-bit units (and, for few-row
//     calls, expands packed 4-bit weight codes) before an ordinary LDS store.
// A weight tile is stored as four 16-byte "k-planes" of BN rows (the global layout is the same, so a wave
// copies 64 rows of a plane with one instruction); an activation tile is stored row-major, 64 bytes per row,
// with the four 16-byte pieces of a row permuted by (row / 4) % 4, which makes both the 64-byte-coalesced
// global reads and the 16-byte-per-lane MFMA fragment reads free of bank conflicts.
// The loop is software-pipelined by hand: every MFMA is followed by at most a few memory or VALU
// instructions (fragment reads for the next k-half into a second register set, loads of the tile three steps
// ahead, lowering and LDS stores of the register-routed pieces), pinned in place with scheduling fences.
// The MFMA "A" operand is the weight fragment and "B" the activation fragment, so a lane ends up with
// four consecutive output channels of one output row.
//
// This header holds the kernel template; every tile shape is instantiated in a translation unit of its own
// (mixed_tile.hip compiled once per shape) so that the shapes build in parallel.
#pragma once
#include <type_traits>

#include "flexiq_internal.h"

namespace flexiq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef short v2s __attribute__((ext_vector_type(2)));

struct GemmParams {
    const int8_t *X;
    const uint8_t *X4;   // XP kernels: the 4-bit codes of the leading floor64(K4) channels, packed (see flexiq_packed4_bytes)
    const int8_t *W8;    // 8-bit weights, and right behind them (U * 32 * Npad bytes further) the 4-bit codes expanded
                         // to int8 at their position, in the same layout
    const uint8_t *W4;
    const uint8_t *wshift;
    const int32_t *ashift;
    const float *cs;
    const float *bias;
    int32_t *acc;
    float *y;
    int8_t *q;
    float r_out;     // 1 / out_scale
    int64_t M;       // output rows (tokens, or B*Ho*Wo output pixels)
    int32_t N, Npad, C;
    int32_t K4;      // max_4bit_ch: leading stored channels computed at 4 bits
    int32_t x_pre;   // nonzero: the activations of those channels arrive lowered already (the kernel copies them like
                     // 8-bit ones; the weights are the 4-bit copies all the same)
    // optional: lower the int8 output for the layer that consumes it (its positions, its 4-bit channel count)
    const int32_t *next_ashift;
    int32_t next_K4, next_G, next_gs_log2;
    uint8_t *next_x4;     // optional with next_ashift: the consumer's packed 4-bit buffer (row stride N / 2) ...
    int32_t next_K4P;     // ... which takes the codes of its leading next_K4P channels (a multiple of 64) instead of q
    // optional: scan the int8 output for the consumer's run-time positions (OR of the magnitude bits per channel
    // group of the consumer, merged into its scan words; the block that finishes last turns them into positions)
    uint32_t *next_scan;          // consumer's scan words (ticket, then kFusedScanRows rows of next_G masks; all zero
                                  // between calls); null: no scan
    const int32_t *next_static;   // consumer's calibrated positions (kept for its 8-bit groups)
    int32_t *next_dyn;            // consumer's run-time position table
    int32_t next_g4;              // consumer's 4-bit groups
    int32_t gs_shift;  // log2(group_size / 32): unit c32 belongs to group c32 >> gs_shift
    int32_t G;       // channel groups
    int32_t U;       // units in the reduction (even per tap), CU = C/32 per tap
    int32_t CU;
    int32_t T;       // filter taps
    int32_t tiles_m, tiles_n;
    // division of a tile index by 8 * tiles_n and by tiles_m % 8 (the two run-time divisors of the tile mapping) by
    // multiplication: mag = floor(2^32 / d); d = 1 where the divisor would be 0
    uint32_t band_div, band_mag, tail_div, tail_mag;
    // convolution geometry (unused for the linear form)
    int32_t H, Wd, Ho, Wo, S, stride, pad;
};

// clamp(v, -(8<<s), (8<<s)-1) & (0xFF << s) on the four int8 lanes of a dword: the bit-lowered value
// put back at its position.  lo2/hi2 hold the bounds in the high byte of each 16-bit half.
__device__ __forceinline__ uint32_t lower4(uint32_t d, v2s lo2, v2s hi2, uint32_t mask)
{
    v2s o = __builtin_bit_cast(v2s, d);           // odd bytes are the high bytes of the halves
    v2s e = o << (short)8;                        // even bytes moved up
    o = __builtin_elementwise_min(__builtin_elementwise_max(o, lo2), hi2);
    e = __builtin_elementwise_min(__builtin_elementwise_max(e, lo2), hi2);
    uint32_t r = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u);
    return r & mask;
}

__device__ __forceinline__ v4i lower16(v4i x, int s)
{
    short lo = (short)((-(8 << s)) << 8);
    short hi = (short)(((((8 << s) - 1) << 8) | 0xFF));
    v2s lo2 = {lo, lo}, hi2 = {hi, hi};
    uint32_t mask = 0x01010101u * ((0xFFu << s) & 0xFFu);
    v4i r;
    r.x = (int)lower4((uint32_t)x.x, lo2, hi2, mask);
    r.y = (int)lower4((uint32_t)x.y, lo2, hi2, mask);
    r.z = (int)lower4((uint32_t)x.z, lo2, hi2, mask);
    r.w = (int)lower4((uint32_t)x.w, lo2, hi2, mask);
    return r;
}

// Four 4-bit codes sitting in the HIGH halves of the bytes of p -> four int8 values code << sw.
// Each 16-bit half is shifted right arithmetically by t = 4 - sw with the wanted byte on top, which
// sign-extends the code and leaves junk only in the low sw bits (cleared by mask) and the low byte.
__device__ __forceinline__ uint32_t expand_hi(uint32_t p, short t, uint32_t mask)
{
    v2s o = __builtin_bit_cast(v2s, p);
    v2s e = o << (short)8;
    o = o >> t;
    e = e >> t;
    uint32_t r = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u);
    return r & mask;
}

// 16 bytes of 4-bit codes (32 channels of one output channel) -> 32 int8 values at position sw.
__device__ __forceinline__ void expand32(v4i p, int sw, v4i &first16, v4i &second16)
{
    short t = (short)(4 - sw);
    uint32_t mask = 0x01010101u * ((0xFFu << sw) & 0xFFu);
    uint32_t w[4] = {(uint32_t)p.x, (uint32_t)p.y, (uint32_t)p.z, (uint32_t)p.w};
    uint32_t o[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        o[2 * e] = expand_hi(w[e] << 4, t, mask);  // low halves: channels 8e .. 8e+3
        o[2 * e + 1] = expand_hi(w[e], t, mask);   // high halves: channels 8e+4 .. 8e+7
    }
    first16 = (v4i){(int)o[0], (int)o[1], (int)o[2], (int)o[3]};
    second16 = (v4i){(int)o[4], (int)o[5], (int)o[6], (int)o[7]};
}


// clamp + mask with a per-lane position (the two units of a K-step may have different positions)
__device__ __forceinline__ v4i lower16v(v4i x, v2s lo2, v2s hi2, uint32_t mask)
{
    v4i r;
    r.x = (int)lower4((uint32_t)x.x, lo2, hi2, mask);
    r.y = (int)lower4((uint32_t)x.y, lo2, hi2, mask);
    r.z = (int)lower4((uint32_t)x.z, lo2, hi2, mask);
    r.w = (int)lower4((uint32_t)x.w, lo2, hi2, mask);
    return r;
}

// 16 bytes per lane from a buffer straight into LDS: lane l of the wave writes dst + 16 l (dst wave-uniform).
typedef __attribute__((address_space(3))) void *lds_ptr_t;
__device__ __forceinline__ void lds_load16(__amdgpu_buffer_rsrc_t r, unsigned char *dst, int voff, int soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)dst, 16, voff, soff, 0, 0);
}

// 4 bytes per lane: lane l writes dst + 4 l.
__device__ __forceinline__ void lds_load4(__amdgpu_buffer_rsrc_t r, void *dst, int voff, int soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)dst, 4, voff, soff, 0, 0);
}

template <int WAVES_M, int WAVES_N, int TM, int TN>
struct Cfg {
    static constexpr int NW = WAVES_M * WAVES_N;        // waves per block: 4 (one per SIMD) or 8 (two per SIMD)
    static_assert(NW == 4 || NW == 8, "four or eight waves per block");
    static constexpr int NT = 64 * NW;
    static constexpr int BM = WAVES_M * TM * 32;
    static constexpr int BN = WAVES_N * TN * 32;
    static_assert(BN % 64 == 0, "a wave copies 64 weight rows per instruction");
    static constexpr int XI = (BM + 16 * NW - 1) / (16 * NW);   // activation pieces per thread per K-step (a wave instruction covers 16 rows)
    static constexpr int XROWS = XI * 16 * NW;          // rows staged per K-step (>= BM; the excess reads as zero)
    static_assert((4 * (BN / 64)) % NW == 0, "weight copies divide evenly over the waves");
    static constexpr int WI = 4 * (BN / 64) / NW;       // direct weight loads per wave per K-step (4 planes x BN rows / 64 rows per copy)
    static constexpr int WL4 = (BN + NT - 1) / NT;      // packed-code pieces per thread per 4-bit unit
    // The last round of activation pieces may reach past the tile's BM rows.  Where the stage ring only fits into
    // LDS without that excess, the stage holds exactly BM rows and the waves whose piece would lie beyond them
    // skip it (TIGHT); everywhere else the excess rows are staged as zeros, which keeps every wave's loads alike.
    static constexpr int kLooseLds = 4 * (XROWS * 64 + 4 * (BN + 2) * 16) + 640 + 2 * (3 * BN * 4) + 640;
    static constexpr int kTightLds = 4 * (BM * 64 + 4 * (BN + 2) * 16) + 640 + 2 * (3 * BN * 4) + 640;
    static constexpr bool TIGHT = kLooseLds > 160 * 1024 && kTightLds <= 160 * 1024;
    static constexpr int XBYTES = (TIGHT ? BM : XROWS) * 64;   // activation tile, row-major
    static constexpr int WPS = (BN + 2) * 16;           // bytes per weight k-plane (+2 pieces staggers the planes over the banks)
    static constexpr int STAGE = XBYTES + 4 * WPS;
    static constexpr int NSTAGE = 4;
    // activation positions of up to 160 groups; scale, bias and the consumer's extraction position of the columns
    // of two consecutive tiles
    // ... and the block's share of the masks it collects for a consuming layer (up to 160 groups)
    static constexpr int TABLE = 640 + 2 * (3 * BN * 4) + 640;
    static constexpr int RING = NSTAGE * STAGE;
    // A block may walk several output tiles.  Not for the largest tiles: their accumulators fill the register
    // file, and the values that would have to stay live across an epilogue do not fit beside them.
    static constexpr bool MULTI = TM * TN <= 10 && !(NW == 8 && TM * TN > 8);
    static constexpr int LDS_BYTES = RING + TABLE;
    static_assert(LDS_BYTES == (TIGHT ? kTightLds : kLooseLds), "the size formulas agree");
    static_assert(LDS_BYTES <= 160 * 1024, "fits the CU's LDS");
};

// How the two 32-channel units of a K-step are staged.
enum StepMode { kMode88 = 0, kMode44 = 1, kMode48 = 2, kModeNone = 3 };

#define FQ_SB() __builtin_amdgcn_sched_barrier(0)

// Tiles with at most 128 accumulator registers per lane are compiled for two blocks per CU where LDS allows:
// one block's prologue and epilogue then overlap the other's matrix work.
//
// PACKED4 selects where the weights of a 4-bit unit come from: the packed codes (half the bytes, expanded in
// registers with vector-ALU work: for memory-bound shapes) or the copy that is already expanded (copied
// exactly like an 8-bit unit: for compute-bound shapes).
//
// XP (linear form only): the activations of the all-4-bit K-steps arrive as packed 4-bit codes (half the bytes, written
// by the producing layer or by the stand-alone packer) and are expanded to int8 at their position while the tile is
// staged, in place of the bit-lowering: the HBM-bound regime, where r then saves activation bytes.
template <int WAVES_M, int WAVES_N, int TM, int TN, bool CONV, bool PACKED4, bool XP = false>
// (two blocks per CU only where two copies of the block's LDS fit: otherwise the register budget of a lone block)
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, (WAVES_M * WAVES_N == 4 && TM * TN <= 8 && 2 * Cfg<WAVES_M, WAVES_N, TM, TN>::LDS_BYTES <= 160 * 1024 ? 2 : 1)) void k_mixed(const GemmParams p)
{
    using C_ = Cfg<WAVES_M, WAVES_N, TM, TN>;
    constexpr int NW = C_::NW, NT = C_::NT, BM = C_::BM, BN = C_::BN, XBYTES = C_::XBYTES, WPS = C_::WPS, STAGE = C_::STAGE;
    constexpr int XI = C_::XI, WI = C_::WI, WL4 = C_::WL4;
    constexpr int NP = PACKED4 ? 2 * WL4 : 0;   // packed-code pieces per thread per K-step
    constexpr int NSR = XI + NP;                // staging registers (x4 dwords) per thread
    constexpr int NI = XI + WI + NP;            // staging items per K-step: activation pieces, direct weight loads, packed pieces
    constexpr int NF = TM + TN;   // fragments per k-half
    constexpr int NMF = TM * TN;  // MFMAs per k-half
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *const sa_tab = lds + C_::RING;
    float *const cs_tab = reinterpret_cast<float *>(sa_tab + 640);  // two copies (tile parity) of [BN] scales, [BN] biases, [BN] positions
    uint32_t *const mask_tab = reinterpret_cast<uint32_t *>(sa_tab + 640 + 2 * (3 * BN * 4));   // scan for a consumer: OR masks per group

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: lives in a scalar register
    __builtin_assume(wave >= 0 && wave < NW);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- tile index -> tile.  A block computes the tiles blockIdx.x, blockIdx.x + gridDim.x, ... one after
    // the other with the load pipeline running on across the tile boundary.  Consecutive block ids land on
    // different XCDs (8 of them, each with its own L2); tile indices are renumbered so that the blocks sharing
    // an XCD walk neighbouring tiles, then sweep bands of 8 tile rows with the tile column varying slowest
    // inside a band (weights stay L2-resident).
    const int total_tiles = p.tiles_m * p.tiles_n;
    // n / d for n < 2^31 with mag = floor(2^32 / d): the product's high word is the quotient or one less
    auto udiv = [](uint32_t n, uint32_t d, uint32_t mag, uint32_t &rem) {
        uint32_t q = __umulhi(n, mag);
        uint32_t r = n - q * d;
        const bool more = r >= d;
        q = more ? q + 1 : q;
        rem = more ? r - d : r;
        return q;
    };
    auto map_tile = [&](int t, int &tile_m, int &tile_n) {
        uint32_t b = (uint32_t)t;
        if (total_tiles % 8 == 0) b = (b % 8) * (uint32_t)(total_tiles / 8) + b / 8;
        constexpr int GMB = 8;
        uint32_t r;
        const int band = (int)udiv(b, p.band_div, p.band_mag, r);   // r: index inside the band
        const bool full = p.tiles_m - band * GMB >= GMB;            // a band of 8 tile rows, or the shorter last one
        uint32_t rt;
        const uint32_t qt = udiv(r, p.tail_div, p.tail_mag, rt);
        tile_m = band * GMB + (int)(full ? (r & 7u) : rt);
        tile_n = (int)(full ? (r >> 3) : qt);
    };
    int ctile = blockIdx.x;   // tile being computed
    int64_t m0;               // its origin
    int n0;
    {
        int tile_m, tile_n;
        map_tile(ctile, tile_m, tile_n);
        m0 = (int64_t)tile_m * BM;
        n0 = tile_n * BN;
    }

    // ---- buffer windows.  Weights: the whole arrays (every access is in range by construction: tiles are
    // padded to Npad columns and to whole units), the tile's column offset travels in the scalar offset.
    // Activations: a window per tile; reads past it return zero, which is what rows beyond M, padded pixels
    // and dummy staging rows need.
    constexpr int kRsrcFlags = 0x00020000;
    const __amdgpu_buffer_rsrc_t rw8 = __builtin_amdgcn_make_buffer_rsrc((void *)p.W8, 0, 2 * p.U * 32 * p.Npad, kRsrcFlags);   // both int8 copies
    const __amdgpu_buffer_rsrc_t rw4 = __builtin_amdgcn_make_buffer_rsrc((void *)p.W4, 0, p.U * 16 * p.Npad, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rws = __builtin_amdgcn_make_buffer_rsrc((void *)p.wshift, 0, (p.G + 1) * p.Npad, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rcs = __builtin_amdgcn_make_buffer_rsrc((void *)p.cs, 0, 2 * p.Npad * 4, kRsrcFlags);   // scales, then biases
    const __amdgpu_buffer_rsrc_t rnx =
        __builtin_amdgcn_make_buffer_rsrc((void *)(p.next_ashift ? p.next_ashift : p.ashift), 0, p.next_ashift ? (p.next_G + 1) * 4 : 0, kRsrcFlags);
    // ---- the tile being LOADED (it runs ahead of the tile being computed by three K-steps, which may be
    // several tiles when K is short): its index, activation window and first column
    int ltile = ctile;
    const int8_t *xbase;
    int xwin;
    int ld_n0;
    // Activation piece j of a thread: row 16 (wave + NW j) + lane / 4 of the tile, LDS slot lane % 4 of that row,
    // which holds k-plane xq = slot ^ ((row / 4) % 4); (row / 4) % 4 = (lane / 16) % 4 for every j.
    const int xrow = lane >> 2;
    const int xq = (lane & 3) ^ ((lane >> 4) & 3);   // k-plane of this thread's activation pieces; unit xq >> 1
    int xvoff4[XI];                   // XP: byte offset of the piece's packed codes inside the window of X4
    const uint8_t *x4base = nullptr;
    int x4win = 0;
    int xvoff[XI];                    // linear: byte offset inside the window; conv: xq * 16
    int xh0[XI], xw0[XI], xpix[XI];   // conv: top-left input coordinate, pixel index of the image origin (-1: no row)
#pragma unroll
    for (int j = 0; j < XI; ++j) {
        xvoff[j] = CONV ? xq * 16 : (16 * (wave + NW * j) + xrow) * p.C + xq * 16;  // linear: rows past the window read zeros
        xvoff4[j] = (16 * (wave + NW * j) + xrow) * (p.C >> 1) + xq * 8;
        xh0[j] = xw0[j] = xpix[j] = 0;
    }
    auto load_tile_context = [&](int64_t lm0, int ln0) {
        const int rows_valid = (int)min((int64_t)BM, p.M - lm0);
        ld_n0 = ln0;
        if (CONV) {
            // 32-bit row arithmetic (the launcher refuses M >= 2^31): 64-bit divisions would cost thousands of
            // cycles per tile
            const uint32_t hw_out = (uint32_t)(p.Ho * p.Wo), m32 = (uint32_t)lm0;
            const uint32_t img0 = m32 / hw_out;
            const int64_t img_bytes = (int64_t)p.H * p.Wd * p.C;
            const int64_t imgs_left = (int64_t)((uint32_t)p.M / hw_out) - img0;
            const int64_t win = min(imgs_left * img_bytes, (int64_t)0x7fffffff);
            xbase = p.X + (int64_t)img0 * img_bytes;
            xwin = (int)win;
#pragma unroll
            for (int j = 0; j < XI; ++j) {
                const int row = 16 * (wave + NW * j) + xrow;
                const bool ok = row < rows_valid;
                const uint32_t mm = ok ? m32 + (uint32_t)row : m32;
                const uint32_t t = mm / (uint32_t)p.Wo;
                const int wo = (int)(mm - t * (uint32_t)p.Wo);
                const uint32_t b = t / (uint32_t)p.Ho;
                const int ho = (int)(t - b * (uint32_t)p.Ho);
                xpix[j] = ok ? (int)(b - img0) * p.H * p.Wd : -1;
                xh0[j] = ho * p.stride - p.pad;
                xw0[j] = wo * p.stride - p.pad;
            }
        } else {
            xbase = p.X + lm0 * p.C;
            xwin = rows_valid * p.C;
            if (XP) {
                x4base = p.X4 + lm0 * (p.C >> 1);
                x4win = rows_valid * (p.C >> 1);
            }
        }
    };
    load_tile_context(m0, n0);
    const int x_lds = (16 * wave) * 64 + lane * 16;   // piece j adds 16 NW rows: j * NW * 1024
    int wvoff[WI];   // per-lane offset of direct weight load j: k-plane parity, 64-row block, row = lane
#pragma unroll
    for (int j = 0; j < WI; ++j) {
        const int idx = wave + NW * j;
        const int pl = idx / (BN / 64), blk = idx % (BN / 64);
        wvoff[j] = ((pl & 1) * p.Npad + blk * 64 + lane) * 16;
    }
    // Direct weight load j of this wave: index wave + NW j over (k-plane, block of 64 rows); scalar values.
    // Packed pieces: row tid + j * NT of the tile (one thread per row).
    int w4voff[WL4], w4lds[WL4];
#pragma unroll
    for (int j = 0; j < WL4; ++j) {
        const int row = tid + j * NT;
        w4voff[j] = row * 16;
        w4lds[j] = XBYTES + row * 16;
    }
    // activation positions of all groups: loaded into a register here, written to LDS after the prologue's tile
    // loads have been issued (one memory latency for all)
    static_assert(BN <= NT && 160 <= NT, "one table element per thread");
    const bool need_tab = p.K4 > 0 && !p.x_pre;   // some K-step lowers activations in this kernel
    const int sa_v = need_tab && tid <= p.G ? p.ashift[tid] : 0;
    int parity = 0;   // which copy of the scale / bias table belongs to the tile being computed
    // Scales and biases of the BN columns from column c0 on, straight into table copy `par` (no register hop, so
    // nothing has to wait for them here; the end-of-step waits of the K loop cover them before the epilogue).
    // cs/bias are padded to Npad >= c0 + BN.
    // Shapes whose blocks compute a single tile turn the table entries into the requantisation multiplier and addend
    // (c * r_out, bias * r_out + 128) once per column when int8 is the only scaled output, instead of once per lane
    // and quad in the epilogue: each thread rewrites the entries its own wave loaded, after the prologue's wait.
    constexpr bool kScaleOnce = !C_::MULTI;
    const bool pre_scaled = kScaleOnce && p.q != nullptr && p.y == nullptr;
    auto fetch_scales = [&](int c0, int par) {
        if (wave * 64 < BN) {
            float *dst = cs_tab + par * (3 * BN) + wave * 64;
            lds_load4(rcs, dst, (wave * 64 + lane) * 4, c0 * 4);
            lds_load4(rcs, dst + BN, (wave * 64 + lane) * 4, (p.Npad + c0) * 4);
            // position of the consumer's channel group that output column c0 + c falls into (an empty descriptor,
            // hence zeros, when there is no consumer to lower for)
            lds_load4(rnx, dst + 2 * BN, ((c0 + wave * 64 + lane) >> p.next_gs_log2) * 4, 0);
        }
    };
    fetch_scales(n0, 0);

    // ---- K-step enumeration, phase-major: all-4-bit steps, then mixed steps, then all-8-bit steps;
    // the iterator points at the next K-step to LOAD.  Scalar state only.
    const int SP = (p.CU + 1) >> 1;           // steps per tap
    const int n4 = p.K4 >> 6;                 // full 4-bit steps per tap
    const int mixed = (p.K4 & 63) ? 1 : 0;    // one step per tap with a 4-bit and an 8-bit unit
    const int steps = p.T * SP;
    const int ustride = 32 * p.Npad;          // bytes between the units of the 8-bit weight layout
    const int w4x_delta = p.U * ustride;      // from the 8-bit copy to the expanded 4-bit copy
    // Phase ph covers c64 in [pb(ph), pe(ph)) of every tap; pn(ph) is the next non-empty phase (3 = done).
    // The three small tables are packed into scalars and indexed with shifts (no scalar-memory waits).
    const int ne0 = n4 > 0, ne1 = mixed > 0, ne2 = n4 + mixed < SP;
    const int first_phase = ne0 ? 0 : (ne1 ? 1 : (ne2 ? 2 : 3));
    const int next1 = ne1 ? 1 : (ne2 ? 2 : 3), next2 = ne2 ? 2 : 3;
    const uint64_t pb_tab = ((uint64_t)n4 << 16) | ((uint64_t)(n4 + mixed) << 32);                       // 16 bits per phase
    const uint64_t pe_tab = (uint64_t)n4 | ((uint64_t)(n4 + mixed) << 16) | ((uint64_t)SP << 32);
    const uint32_t pn_tab = (uint32_t)next1 | ((uint32_t)next2 << 4) | (3u << 8) | (3u << 12);             // 4 bits per phase
    // A block that walks several tiles takes the phases of every other tile in reverse (8-bit steps first): a tile then
    // begins with the kind of step the previous one ended with, and the change from plain steps to lowering steps, which
    // costs a wait for every copy in flight (see the step ladder), happens once per two tiles instead of once per tile.
    // Integer sums do not depend on the order.
    const int last_phase = ne2 ? 2 : (ne1 ? 1 : (ne0 ? 0 : 3));
    const int prev1 = ne0 ? 0 : 3, prev2 = ne1 ? 1 : (ne0 ? 0 : 3);
    const uint32_t pp_tab = 3u | ((uint32_t)prev1 << 4) | ((uint32_t)prev2 << 8) | (3u << 12);            // phase before ph (3 = done)
    bool it_rev = false;
    // how the activations of a phase's steps are staged: by the phase, unless they arrive lowered already (then
    // every step copies them like an 8-bit step, while the weights still follow the phase)
    const uint32_t pm_tab = p.x_pre ? ((uint32_t)kMode88 | (kMode88 << 4) | (kMode88 << 8) | (kModeNone << 12))
                                    : ((uint32_t)kMode44 | (kMode48 << 4) | (kMode88 << 8) | (kModeNone << 12));
    auto pb = [&](int ph) { return (int)((pb_tab >> (16 * ph)) & 0xFFFFu); };
    auto pe = [&](int ph) { return (int)((pe_tab >> (16 * ph)) & 0xFFFFu); };
    auto pn = [&](int ph) { return (int)((pn_tab >> (4 * ph)) & 15u); };
    int it_phase = first_phase, it_tap = 0, it_dy = 0, it_dx = 0;
    int it_c64 = pb(first_phase);
    // derived state, refreshed whenever phase, tap or tile change: end of the phase's range, staging mode of its
    // steps, and the scalar offsets of the step's two weight units (tile column, tap, c64 and the choice between
    // the 8-bit copy and the expanded 4-bit copy all folded in)
    int it_pe, it_mode, it_w0, it_w1;
    auto refresh_iterator = [&]() {
        it_pe = pe(it_phase);
        it_mode = (int)((pm_tab >> (4 * it_phase)) & 15u);
        const int base = (it_tap * (2 * SP) + 2 * it_c64) * ustride + ld_n0 * 16;
        it_w0 = base + (it_phase <= 1 ? w4x_delta : 0);
        it_w1 = base + ustride + (it_phase == 0 ? w4x_delta : 0);
    };
    refresh_iterator();
    // Within a phase and tap the update is three scalar additions; everything else (next tap, next phase, next
    // output tile of the block: tile mapping and, for a convolution, the per-row gather state) sits behind one
    // uniform branch.
    auto advance = [&]() {
        const int c = it_c64 + 1;
        if (__builtin_expect(c != it_pe, 1)) {
            it_c64 = c;
            it_w0 += 2 * ustride;
            it_w1 += 2 * ustride;
        } else {
            const int tap1 = it_tap + 1;
            if (tap1 != p.T) {   // same phase, next filter tap
                const int first = pb(it_phase);
                const int dw = 2 * (SP + 1 + first - it_pe) * ustride;
                it_tap = tap1;
                it_c64 = first;
                it_w0 += dw;
                it_w1 += dw;
                if (CONV) {
                    const int dx1 = it_dx + 1;
                    const bool wrap_x = dx1 == p.S;
                    it_dy = wrap_x ? it_dy + 1 : it_dy;
                    it_dx = wrap_x ? 0 : dx1;
                }
            } else {             // the phase is finished
                int ph = it_rev ? (int)((pp_tab >> (4 * it_phase)) & 15u) : pn(it_phase);
                // ... and with it the tile: move on to the block's next tile if there is one
                if (C_::MULTI && ph == 3) {
                    const int nt = ltile + (int)gridDim.x;
                    if (nt < total_tiles) {
                        ltile = nt;
                        int tile_m, tile_n;
                        map_tile(nt, tile_m, tile_n);
                        load_tile_context((int64_t)tile_m * BM, tile_n * BN);
                        it_rev = !it_rev;
                        ph = it_rev ? last_phase : first_phase;
                    }
                }
                it_dy = 0;
                it_dx = 0;
                it_tap = 0;
                it_phase = ph;
                it_c64 = pb(ph);
                refresh_iterator();
            }
        }
    };

    // ---- staging registers (register-routed pieces only) and the descriptor of the tile they hold
    v4i sr[NSR > 0 ? NSR : 1];
    int wsh[2][WL4];
    int st_c64 = 0;   // c64 of the tile in the staging registers

    // Item i of the K-step the iterator points at: load it, either straight into `stage` or into registers.
    // (The K offset of an activation piece goes into the per-lane offset, which the buffer range check covers:
    // what the pad unit of an odd unit count would read past the end of the window's last row comes back as zero.)
    constexpr int kTailRows = BM - (XI - 1) * 16 * NW;          // rows of the last round that belong to the tile
    constexpr int kFullWaves = (kTailRows + 15) / 16;           // waves 0 .. kFullWaves-1 own a piece of the last round
    static_assert(kTailRows > 0 && kTailRows % 16 == 0, "whole pieces");
    auto has_piece = [&](int i) { return !C_::TIGHT || i < XI - 1 || kFullWaves >= NW || wave < kFullWaves; };
    auto gload = [&](v4i(&sr)[NSR > 0 ? NSR : 1], int(&wsh)[2][WL4], int i, int mode, unsigned char *stage) {
        const int c64 = it_c64;
        if (i < XI) {
            if (!has_piece(i)) return;
            const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)xbase, 0, xwin, kRsrcFlags);
            int off;
            if (CONV) {
                const int hi = xh0[i] + it_dy, wi = xw0[i] + it_dx;
                const bool ok = hi >= 0 && hi < p.H && wi >= 0 && wi < p.Wd && xpix[i] >= 0;
                off = ok ? (xpix[i] + hi * p.Wd + wi) * p.C + xvoff[i] + c64 * 64 : (int)0x80000000;
            } else {
                off = xvoff[i] + c64 * 64;
            }
            if (mode == kMode88) {
                lds_load16(rx, stage + (16 * (wave + NW * i)) * 64, off, 0);
            } else if (XP && mode == kMode44) {   // eight bytes of packed codes: the piece's sixteen channels
                const __amdgpu_buffer_rsrc_t rx4 = __builtin_amdgcn_make_buffer_rsrc((void *)x4base, 0, x4win, kRsrcFlags);
                const auto v = __builtin_amdgcn_raw_buffer_load_b64(rx4, xvoff4[i] + c64 * 32, 0, 0);
                sr[i].x = (int)v[0];
                sr[i].y = (int)v[1];
            } else {
                sr[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0);
            }
        } else if (i < XI + WI) {
            const int j = i - XI;
            const int idx = wave + NW * j;                      // (k-plane, 64-row block) of this copy
            const int pl = idx / (BN / 64), blk = idx % (BN / 64);
            const int h = pl >> 1;                              // unit of the K-step
            // (which copy of the weights a unit reads is part of the iterator's offsets; only the packed-code
            // variant needs to know here, to leave its 4-bit units to the register route)
            const bool four_mode = mode == kMode44 || (mode == kMode48 && h == 0);
            if (!(PACKED4 && four_mode)) lds_load16(rw8, stage + XBYTES + pl * WPS + blk * 1024, wvoff[j], h ? it_w1 : it_w0);
        } else if (PACKED4) {
            const int h = (i - XI - WI) / WL4, j = (i - XI - WI) % WL4;
            const bool four = mode == kMode44 || (mode == kMode48 && h == 0);
            if (four && (BN % NT == 0 || tid + j * NT < BN)) {
                const int u = it_tap * (2 * SP) + 2 * c64 + h;
                const int g = (2 * c64 + h) >> p.gs_shift;
                sr[XI + h * WL4 + j] = __builtin_amdgcn_raw_buffer_load_b128(rw4, w4voff[j], u * 16 * p.Npad + ld_n0 * 16, 0);
                wsh[h][j] = __builtin_amdgcn_raw_buffer_load_b8(rws, w4voff[j] >> 4, g * p.Npad + ld_n0, 0);
            }
        }
    };
    // per-step constants of the activation bit-lowering for this thread's unit.  The position comes from the
    // LDS table; sa_fetch() is called a step ahead of lower_setup() so that no step starts by waiting for LDS.
    v2s lo2, hi2;
    uint32_t amask;
    short xp_t = 0;   // XP: right shift that puts a code sitting in the high half of a byte at its position
    int sa_next = 0;
    auto sa_fetch = [&](int c64) { sa_next = reinterpret_cast<const int *>(sa_tab)[(2 * c64 + (xq >> 1)) >> p.gs_shift]; };
    auto lower_setup = [&]() {
        const int sa = sa_next;
        const short lo = (short)((-(8 << sa)) << 8);
        const short hi = (short)((((8 << sa) - 1) << 8) | 0xFF);
        lo2 = (v2s){lo, lo};
        hi2 = (v2s){hi, hi};
        amask = 0x01010101u * ((0xFFu << sa) & 0xFFu);
        xp_t = (short)(4 - sa);
    };
    // Register-routed pieces of the staged K-step -> LDS.  The VALU work of the 4-bit units (bit-lowering
    // of activations, expansion of packed weight codes) is cut into four pieces per item, lmicro(i, 0..3),
    // so that it can be spread over the MFMA stream and co-issue with it; lstore(i) then writes the item.
    uint32_t wexp[8];   // expanded weights of the packed piece in progress
    auto lmicro = [&](v4i(&sr)[NSR > 0 ? NSR : 1], int(&wsh)[2][WL4], int i, int k, int mode) {
        if (i < XI) {
            if (!has_piece(i)) return;
            if (XP && mode == kMode44) {
                // dword e of the packed piece holds channels 8e .. 8e+3 in the low halves of its bytes and 8e+4 .. 8e+7
                // in the high halves; expanded in place from the top so that no source is overwritten early
                if (k == 0) sr[i][3] = (int)expand_hi((uint32_t)sr[i][1], xp_t, amask);
                else if (k == 1) sr[i][2] = (int)expand_hi((uint32_t)sr[i][1] << 4, xp_t, amask);
                else if (k == 2) sr[i][1] = (int)expand_hi((uint32_t)sr[i][0], xp_t, amask);
                else sr[i][0] = (int)expand_hi((uint32_t)sr[i][0] << 4, xp_t, amask);
            } else if (mode == kMode44) {
                sr[i][k] = (int)lower4((uint32_t)sr[i][k], lo2, hi2, amask);
            } else if (mode == kMode48) {
                const int l = (int)lower4((uint32_t)sr[i][k], lo2, hi2, amask);
                sr[i][k] = (xq >> 1) == 0 ? l : sr[i][k];
            }
        } else if (PACKED4 && i >= XI + WI) {
            const int h = (i - XI - WI) / WL4, j = (i - XI - WI) % WL4;
            const bool four = mode == kMode44 || (mode == kMode48 && h == 0);
            if (four) {
                const int sw = wsh[h][j];
                const short t = (short)(4 - sw);
                const uint32_t mask = 0x01010101u * ((0xFFu << sw) & 0xFFu);
                const uint32_t w = (uint32_t)sr[XI + h * WL4 + j][k];
                wexp[2 * k] = expand_hi(w << 4, t, mask);  // low halves: channels 8k .. 8k+3
                wexp[2 * k + 1] = expand_hi(w, t, mask);   // high halves: channels 8k+4 .. 8k+7
            }
        }
    };
    auto lstore = [&](v4i(&sr)[NSR > 0 ? NSR : 1], int i, int mode, unsigned char *stage) {
        if (i < XI) {
            if (!has_piece(i)) return;
            if (mode == kMode44 || mode == kMode48) *reinterpret_cast<v4i *>(stage + x_lds + i * (NW * 1024)) = sr[i];
        } else if (PACKED4 && i >= XI + WI) {
            const int h = (i - XI - WI) / WL4, j = (i - XI - WI) % WL4;
            const bool four = mode == kMode44 || (mode == kMode48 && h == 0);
            if (four && (BN % NT == 0 || tid + j * NT < BN)) {
                *reinterpret_cast<v4i *>(stage + (2 * h) * WPS + w4lds[j]) = (v4i){(int)wexp[0], (int)wexp[1], (int)wexp[2], (int)wexp[3]};
                *reinterpret_cast<v4i *>(stage + (2 * h + 1) * WPS + w4lds[j]) = (v4i){(int)wexp[4], (int)wexp[5], (int)wexp[6], (int)wexp[7]};
            }
        }
    };

    const int frag_half = lane >> 5, frag_row = lane & 31;
    const int fsw = (frag_row >> 2) & 3;
    const int xs_frag0 = (wm * TM * 32 + frag_row) * 64 + ((frag_half ^ fsw) * 16);          // k-half 0
    const int xs_frag1 = (wm * TM * 32 + frag_row) * 64 + (((2 + frag_half) ^ fsw) * 16);    // k-half 1
    const int ws_frag = XBYTES + frag_half * WPS + (wn * TN * 32 + frag_row) * 16;
    // fragments in order of need: w0, x0, w1..w(TN-1), x1..x(TM-1); f[0..TN) weights, f[TN..NF) activations
    auto forder = [](int i) { return i == 0 ? 0 : (i == 1 ? TN : (i <= TN ? i - 1 : i)); };
    auto fread = [&](v4i(&f)[NF], int i, const unsigned char *stage, int kh) {
        if (i < TN) f[i] = *reinterpret_cast<const v4i *>(stage + ws_frag + kh * 2 * WPS + i * 512);
        else f[i] = *reinterpret_cast<const v4i *>(stage + (kh ? xs_frag1 : xs_frag0) + (i - TN) * 2048);
    };
    v4i fA[NF], fB[NF];

    // ---- prologue: the loads of K-steps 0, 1 and 2 are all issued before anything waits (straight into
    // stages 0, 1, 2; the register-routed pieces of steps 0 and 1 into registers of their own, those of
    // step 2 into the staging registers of the main loop); then the tables and the register-routed pieces of
    // steps 0 and 1 go to LDS.
    int mode_staged = kModeNone;   // mode of K-step s+2, whose register-routed pieces sit in the staging registers
    bool plain_prologue;           // K-steps 0, 1 and 2 all exist and are plain copies into LDS
    // K-steps 0, 1 and 2 all exist and all lower their activations: same code with the mode known at compile time,
    // so that the waits for the staging registers are exact and the pieces of step 0 are lowered while the loads
    // of steps 1 and 2 are still in flight (with a run-time mode those waits cover every load issued so far)
    const bool lowering_prologue = !PACKED4 && it_mode == kMode44 && it_c64 + 2 < it_pe;
    {
        v4i sp[2][NSR > 0 ? NSR : 1];
        int wp[2][2][WL4];
        int pmode[2] = {kModeNone, kModeNone}, pc64[2] = {0, 0};
        auto publish_tables = [&]() {
            if (p.next_scan && tid < 160) mask_tab[tid] = 0;   // (first used in an epilogue, many barriers from here)
            if (need_tab) {
                if (tid <= p.G) reinterpret_cast<int *>(sa_tab)[tid] = sa_v;
                __builtin_amdgcn_s_waitcnt(0xc07f);
                __builtin_amdgcn_s_barrier();   // position table visible
            }
        };
        if (lowering_prologue) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                pc64[t] = it_c64;
#pragma unroll
                for (int i = 0; i < NI; ++i) gload(sp[t], wp[t], i, kMode44, lds + t * STAGE);
                advance();
            }
            mode_staged = kMode44;
            st_c64 = it_c64;
#pragma unroll
            for (int i = 0; i < NI; ++i) gload(sr, wsh, i, kMode44, lds + 2 * STAGE);
            advance();
            plain_prologue = false;
            publish_tables();
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                sa_fetch(pc64[t]);
                lower_setup();
#pragma unroll
                for (int i = 0; i < NI; ++i) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) lmicro(sp[t], wp[t], i, k, kMode44);
                    lstore(sp[t], i, kMode44, lds + t * STAGE);
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if (it_mode != kModeNone) {   // the block has a K-step t (of its first tile, or of a following one when K is short)
                    pmode[t] = it_mode;
                    pc64[t] = it_c64;
#pragma unroll
                    for (int i = 0; i < NI; ++i) gload(sp[t], wp[t], i, pmode[t], lds + t * STAGE);
                    advance();
                }
            }
            if (it_mode != kModeNone) {
                mode_staged = it_mode;
                st_c64 = it_c64;
#pragma unroll
                for (int i = 0; i < NI; ++i) gload(sr, wsh, i, mode_staged, lds + 2 * STAGE);
                advance();
            }
            plain_prologue = !PACKED4 && pmode[0] == kMode88 && pmode[1] == kMode88 && mode_staged == kMode88;
            publish_tables();
            // (nothing to do when all three steps are plain copies; the branch also keeps the wait for the staging
            // registers, which covers every load issued so far, out of that path)
            if (!plain_prologue) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    if (pmode[t] != kModeNone) {
                        if (pmode[t] != kMode88) {
                            sa_fetch(pc64[t]);
                            lower_setup();
                        }
#pragma unroll
                        for (int i = 0; i < NI; ++i) {
#pragma unroll
                            for (int k = 0; k < 4; ++k) lmicro(sp[t], wp[t], i, k, pmode[t]);
                            lstore(sp[t], i, pmode[t], lds + t * STAGE);
                        }
                    }
                }
            }
        }
    }
    if (mode_staged == kMode44 || mode_staged == kMode48) sa_fetch(st_c64);
    v16i acc[TN][TM];
    auto zero_acc = [&]() {
#pragma unroll
        for (int a = 0; a < TN; ++a)
#pragma unroll
            for (int b = 0; b < TM; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0;
    };
    // (see the K loop: a tile that begins with lowering steps clears no accumulators)
    constexpr bool kZeroStep = TM * TN <= 10;   // (the 16-fragment shape has no registers to spare for the extra variant)
    bool zero_step = kZeroStep && mode_staged == kMode44 && it_mode == kMode44;
    if (!zero_step) zero_acc();

    // K-steps 0 and 1 have landed (step 0 reads the first fragments of step 1 ahead).  Step 2 may stay in flight
    // when all three are plain copies: every wave then has the same number of loads outstanding, and the wait at
    // the end of step 0 covers it.
    if ((plain_prologue || lowering_prologue) && has_piece(XI - 1))
        __builtin_amdgcn_s_waitcnt(0x0070 | ((XI + WI) & 15) | (((XI + WI) >> 4) << 14));
    else if (plain_prologue || lowering_prologue)   // this wave issues one load less per K-step
        __builtin_amdgcn_s_waitcnt(0x0070 | ((XI - 1 + WI) & 15) | (((XI - 1 + WI) >> 4) << 14));
    else
        __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < NF; ++i) fread(fA, i, lds, 0);
    // (the scale loads were issued before every tile load, so they have landed too; the table is first read in the
    // epilogue, at least one barrier from here)
    if (pre_scaled && wave * 64 < BN) {
        float *own = cs_tab + wave * 64 + lane;
        const float c = own[0], b = own[BN];
        own[0] = c * p.r_out;
        own[BN] = b * p.r_out + 128.0f;
    }

    // ---- main loop.  Step s computes K-step s from stage s % 4 while K-step s+3 is loaded (straight into stage
    // (s+3) % 4, or into the staging registers) and the register-routed pieces of K-step s+2 (loaded during step
    // s-1) are lowered / expanded and stored into stage (s+2) % 4.  `ma` is the mode of K-step s+2 (kModeNone:
    // there is none), `mb` the mode of K-step s+3 (kModeNone: nothing left to load); both are compile-time
    // constants in the steady-state loops and run-time values elsewhere.
    // The K-steps of the block's successive output tiles form one sequence: while the last steps of an
    // output tile are computed, the first K-steps of the next one are already being loaded and staged.
    int o_cur = 0, o_nx1 = STAGE, o_nx2 = 2 * STAGE, o_nx3 = 3 * STAGE;   // byte offsets of the stages of K-steps s .. s+3
    int s = 0;    // K-step within the output tile being computed
    constexpr int kStageSlots = 2 * NMF > 2 ? 2 * NMF - 2 : 1;    // slots that carry staging work
    constexpr int kAdvanceSlot = 2 * NMF > 2 ? 2 * NMF - 2 : 0;   // slot after which the load iterator moves on
    // fragment reads of the second k-half that are issued after the last slot with staging work
    constexpr int kLateReads = [] {
        int n = 0;
        for (int k = 0; k < NF; ++k)
            if (NMF + k * NMF / NF > kStageSlots - 1) ++n;
        return n < 15 ? n : 15;
    }();
    auto step = [&](auto ma_, auto mb_, auto h1_, auto z_) {
        const int ma = ma_, mb = mb_;
        const bool h1 = h1_;
        const bool z = z_;   // first K-step of an output tile: the MFMAs of its first k-half start from zero
        const unsigned char *cur = lds + o_cur;
        const unsigned char *nx1 = lds + o_nx1;
        unsigned char *nx2 = lds + o_nx2;
        unsigned char *nx3 = lds + o_nx3;
        if (ma == kMode44 || ma == kMode48) lower_setup();   // from the position fetched during the previous step
        if (mb == kMode44 || mb == kMode48) st_c64 = it_c64;
        FQ_SB();
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int b = 0; b < TM; ++b)
#pragma unroll
                for (int a = 0; a < TN; ++a) {
                    const int slot = b * TN + a, g = kh * NMF + slot;
                    // Two waves share a SIMD's matrix pipe in the eight-wave shapes, and the arbiter prefers the
                    // older one: it would run ahead and then idle at the barrier (measured: 600 of a step's 1800
                    // cycles) while the younger one finishes alone, too slow to keep the pipe full.  A wave's
                    // priority therefore falls as it advances (one level per quarter of the step, up again for the
                    // last MFMAs and the step boundary), so whichever is behind wins.  Measured: 3-5 % at r = 1 and
                    // 1 % at r = 0 with twenty MFMAs per wave and step, nothing with ten to fourteen; several other
                    // patterns (a level per eighth, wrapping) measured the same within 0.5 %.
                    if constexpr (NW == 8 && NMF >= 10) {
                        constexpr int kEighth = 2 * NMF / 8;
                        auto level_at = [](int x) { return x < 8 * kEighth ? 3 - x / (2 * kEighth) : (x < 9 * kEighth ? 0 : 2); };
                        const int level = level_at(g);
                        if (g == 0 || level != level_at(g - 1)) {
                            if (level == 3) __builtin_amdgcn_s_setprio(3);
                            else if (level == 2) __builtin_amdgcn_s_setprio(2);
                            else if (level == 1) __builtin_amdgcn_s_setprio(1);
                            else __builtin_amdgcn_s_setprio(0);
                        }
                    }
                    if (kh == 0) acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fA[a], fA[TN + b], z ? v16i{} : acc[a][b], 0, 0, 0);
                    else acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fB[a], fB[TN + b], acc[a][b], 0, 0, 0);
                    FQ_SB();
                    // fragment read k of the other register set at slot k*NMF/NF of this k-half
#pragma unroll
                    for (int k = 0; k < NF; ++k)
                        if (k * NMF / NF == slot) {
                            if (kh == 0) fread(fB, forder(k), cur, 1);
                            else if (h1) fread(fA, forder(k), nx1, 0);
                            FQ_SB();
                        }
                    // Staging work, spread over the step's slots but the last two (where the scalar iterator update
                    // runs in the shadow of the MFMAs).  An activation piece or packed-code piece i has six events:
                    // four pieces of VALU work and the LDS store of K-step s+2's copy, then the load of K-step s+3's
                    // into the same registers (or straight into LDS).  Each of the three item groups is spread evenly
                    // over the slots on its own, so VALU-heavy and load-only events alternate.
#pragma unroll
                    for (int t = 0; t < 6 * XI; ++t)
                        if (t * kStageSlots / (6 * XI) == g) {
                            const int i = t / 6, k = t % 6;
                            if (k < 4) {
                                if (ma == kMode44 || ma == kMode48) lmicro(sr, wsh, i, k, ma);
                            } else if (k == 4) {
                                if (ma == kMode44 || ma == kMode48) lstore(sr, i, ma, nx2);
                            } else {
                                if (mb != kModeNone) gload(sr, wsh, i, mb, nx3);
                            }
                            FQ_SB();
                        }
#pragma unroll
                    for (int j = 0; j < WI; ++j)
                        if ((2 * j + 1) * kStageSlots / (2 * WI) == g) {
                            if (mb != kModeNone) gload(sr, wsh, XI + j, mb, nx3);
                            FQ_SB();
                        }
#pragma unroll
                    for (int t = 0; t < 6 * NP; ++t)
                        if (t * kStageSlots / (6 * (NP > 0 ? NP : 1)) == g) {
                            const int i = XI + WI + t / 6, k = t % 6;
                            if (k < 4) {
                                if (ma == kMode44 || ma == kMode48) lmicro(sr, wsh, i, k, ma);
                            } else if (k == 4) {
                                if (ma == kMode44 || ma == kMode48) lstore(sr, i, ma, nx2);
                            } else {
                                if (mb != kModeNone) gload(sr, wsh, i, mb, nx3);
                            }
                            FQ_SB();
                        }
                    if (g == kAdvanceSlot && mb != kModeNone) {
                        if (mb == kMode44 || mb == kMode48) sa_fetch(st_c64);   // position for the next step's lowering
                        advance();
                        FQ_SB();
                    }
                }
        // The direct loads of the previous step (K-step s+2) must have landed before the barrier publishes them;
        // this step's own loads may stay in flight.  Their number is known at compile time where every wave
        // issues the same loads; otherwise wait for everything.
        if (!PACKED4 && (mb == kMode88 || mb == kMode44 || mb == kMode48)) {
            if (has_piece(XI - 1))
                __builtin_amdgcn_s_waitcnt(0x0070 | ((XI + WI) & 15) | (((XI + WI) >> 4) << 14));
            else   // this wave issues one load less per K-step
                __builtin_amdgcn_s_waitcnt(0x0070 | ((XI - 1 + WI) & 15) | (((XI - 1 + WI) >> 4) << 14));
        } else {
            __builtin_amdgcn_s_waitcnt(0x0070);
        }
        // This wave's LDS stores and its reads of the stage that is refilled next are complete.  The fragment reads
        // issued after the last staging slot (they read the next step's stage, which nobody overwrites yet) may
        // stay in flight across the barrier: LDS operations complete in order, so allowing that many outstanding
        // ones still covers every store.
        if (h1)
            __builtin_amdgcn_s_waitcnt(0xc07f | (kLateReads << 8));
        else
            __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
        FQ_SB();
        {
            const int t = o_cur;
            o_cur = o_nx1;
            o_nx1 = o_nx2;
            o_nx2 = o_nx3;
            o_nx3 = t;
        }
        ++s;
        mode_staged = mb;
    };

    // ---- epilogue of one output tile.  Lane holds output row m = 32 b + (lane & 31) and, per accumulator
    // quad g, the four consecutive output channels n = 32 a + 8 g + 4 (lane >> 5) + i.  The body is
    // instantiated with compile-time output flags for the common cases (int8 only; fp32 or int32 only) and
    // once with run-time flags for everything else (ragged N, several outputs at once).
    const bool want_q = p.q != nullptr, want_y = p.y != nullptr, want_acc = p.acc != nullptr;
    const bool n_vec = (p.N & 3) == 0;
    const bool lower_out = p.next_ashift != nullptr;   // int8 output lowered for the consuming layer
    const bool scan_out = p.next_scan != nullptr;      // int8 output scanned for the consuming layer's positions
    const bool q_rows = want_q && (p.N & 15) == 0;   // int8 output as 16-byte row-contiguous pieces
    const int frag_half_e = lane >> 5, frag_row_e = lane & 31;
    // (one call handles fragment column a; the variant is chosen per column, which keeps the live ranges of the
    // accumulators short where the variants branch apart)
    // Sixteen consecutive int8 codes of output row m from column n on.  When the consumer takes its leading channels as
    // packed 4-bit codes, the pieces of those columns (already clamped and masked: L(v, s) << s) are packed instead: two
    // codes per byte in the consumer's order (see flexiq_packed4_bytes) into its buffer, and q is left alone there.
    auto store_row_piece = [&](int64_t m, int n, v4i piece, const float *tab) {
        if (p.next_x4 != nullptr && n < p.next_K4P) {
            const int sp = reinterpret_cast<const int *>(tab + 2 * BN)[n - n0];
            const uint32_t d0 = ((uint32_t)piece.x >> sp) & 0x0F0F0F0Fu, d1 = ((uint32_t)piece.y >> sp) & 0x0F0F0F0Fu;
            const uint32_t d2 = ((uint32_t)piece.z >> sp) & 0x0F0F0F0Fu, d3 = ((uint32_t)piece.w >> sp) & 0x0F0F0F0Fu;
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            *reinterpret_cast<v2u *>(p.next_x4 + m * (p.N >> 1) + (n >> 1)) = (v2u){d0 | (d1 << 4), d2 | (d3 << 4)};
        } else {
            *reinterpret_cast<v4i *>(p.q + m * p.N + n) = piece;
        }
    };
    v4i qout[TN][TM];   // int8 output pieces of a tile (row-contiguous form), stored after the last fragment column
    auto epilogue = [&](auto a_, auto wq_, auto wy_, auto wa_, auto nv_, auto qr_, auto lw_, auto sc_) {
        const bool wq = wq_, wy = wy_, wa = wa_, nv = nv_, qr = qr_, lw = lw_, sc = sc_;
        // the table holds multiplier and addend already: known at compile time in the int8-only variants
        const bool pre = (std::is_same<decltype(wq_), std::true_type>::value && std::is_same<decltype(wy_), std::false_type>::value)
                             ? kScaleOnce : pre_scaled;
        constexpr int a = decltype(a_)::value;
        const float *tab = cs_tab + parity * (3 * BN);
        {
            uint32_t qrow[TM][4];   // int8 codes of the four quads of fragment (a, b)
            uint32_t seen = 0;      // scan: OR of v ^ (v << 1) over this lane's valid codes, per byte (bits 1..7 are used)
            // scale and bias of a quad's four columns are read from the LDS table one quad ahead
            const int nl0 = (wn * TN + a) * 32 + 4 * frag_half_e;
            float4 cs_nx = *reinterpret_cast<const float4 *>(tab + nl0);
            float4 bi_nx = *reinterpret_cast<const float4 *>(tab + BN + nl0);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                FQ_SB();   // keep the accumulator reads of later quads from being hoisted (register pressure)
                const int nl = nl0 + 8 * g;
                const int n = n0 + nl;
                const bool n_ok = n < p.N;
                float csv[4], biv[4], mul[4], add[4];
                {
                    const float4 cs = cs_nx, bi = bi_nx;
                    if (g < 3) {
                        cs_nx = *reinterpret_cast<const float4 *>(tab + nl + 8);
                        bi_nx = *reinterpret_cast<const float4 *>(tab + BN + nl + 8);
                    }
                    csv[0] = cs.x; csv[1] = cs.y; csv[2] = cs.z; csv[3] = cs.w;
                    biv[0] = bi.x; biv[1] = bi.y; biv[2] = bi.z; biv[3] = bi.w;
                }
                // The int8 code is formed in offset form: t = acc * mul + (add + 128) in one fused operation, then
                // one instruction rounds t to nearest-even, saturates it to 0..255 and puts it into its byte; flipping
                // the top bit of every byte gives the two's-complement code clamp(round(.), -128, 127).
                float qlo = 0.0f, qhi = 255.0f;   // clamp of the offset code when the output is lowered as well
                uint32_t qmask = 0xFFFFFFFFu;
                if (wq) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        mul[i] = pre ? csv[i] : csv[i] * p.r_out;
                        add[i] = pre ? biv[i] : biv[i] * p.r_out + 128.0f;
                    }
                    // Output lowered for the consumer (its 4-bit channels only): L(v, s) << s = clamp(v, -(8<<s),
                    // (8<<s)-1) with the low s bits cleared; the four columns of a quad share a channel group.
                    if (lw) {
                        const bool lowered = n < p.next_K4;
                        const int sp = reinterpret_cast<const int *>(tab + 2 * BN)[nl];
                        qhi = (float)((8 << (lowered ? sp : 4)) + 127);
                        qlo = 255.0f - qhi;
                        qmask = lowered ? 0x01010101u * ((0xFFu << sp) & 0xFFu) : 0xFFFFFFFFu;
                    }
                }
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    const int ml = (wm * TM + b) * 32 + frag_row_e;
                    const int64_t m = m0 + ml;
                    const int iv[4] = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                    uint32_t qw = 0;
                    if (wq) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            float t = __builtin_fmaf((float)iv[i], mul[i], add[i]);
                            if (lw) t = __builtin_amdgcn_fmed3f(t, qlo, qhi);
                            qw = __builtin_amdgcn_cvt_pk_u8_f32(t, i, qw);
                        }
                        qw ^= 0x80808080u;
                        if (lw) qw &= qmask;
                        qrow[b][g] = qw;
                        // Bit j + 1 of v ^ (v << 1) says that bits j + 1 and j of v differ; the highest such j is the highest
                        // set bit of the magnitude (v, or ~v when negative) whatever the sign, so no sign handling is
                        // needed.  (The shift carries bit 7 of a byte into bit 0 of the next one, which is not used.)
                        if (sc) seen |= (m < p.M && n_ok) ? (qw ^ (qw << 1)) : 0u;
                    }
                    if (!(wy || wa || (wq && !qr))) continue;   // nothing is stored quad by quad
                    if (m >= p.M || !n_ok) continue;
                    const int64_t o = m * p.N + n;
                    if (nv) {
                        if (wa) *reinterpret_cast<v4i *>(p.acc + o) = (v4i){iv[0], iv[1], iv[2], iv[3]};
                        if (wy) {
                            float4 y;
                            y.x = __builtin_fmaf((float)iv[0], csv[0], biv[0]);
                            y.y = __builtin_fmaf((float)iv[1], csv[1], biv[1]);
                            y.z = __builtin_fmaf((float)iv[2], csv[2], biv[2]);
                            y.w = __builtin_fmaf((float)iv[3], csv[3], biv[3]);
                            *reinterpret_cast<float4 *>(p.y + o) = y;
                        }
                        if (wq && !qr) *reinterpret_cast<uint32_t *>(p.q + o) = qw;
                    } else {
                        for (int i = 0; i < 4 && n + i < p.N; ++i) {
                            if (wa) p.acc[o + i] = iv[i];
                            if (wy) p.y[o + i] = __builtin_fmaf((float)iv[i], csv[i], biv[i]);
                            if (wq) p.q[o + i] = (int8_t)((qw >> (8 * i)) & 0xFF);
                        }
                    }
                }
            }
            FQ_SB();
            if (wq && sc) {
                // The 32 columns of a fragment column lie in one channel group of the consumer (its groups are 32 or 64
                // channels, tiles start at multiples of 32).  Fold the four bytes, OR over the wave one bit at a
                // time (wave-uniform result), and merge.
                seen |= seen >> 16;
                seen |= seen >> 8;
                uint32_t w = 0;
#pragma unroll
                for (int bit = 1; bit < 8; ++bit)
                    if (__builtin_amdgcn_ballot_w64(((seen >> bit) & 1u) != 0u) != 0) w |= 1u << bit;
                const int ncol = n0 + (wn * TN + a) * 32;
                // (into the block's LDS copy; the device-wide merge happens once, when the block has finished its
                // tiles: a global atomic per tile would hold up the loads queued behind it)
                if (lane == 0 && w != 0 && ncol < p.N) __hip_atomic_fetch_or(mask_tab + (ncol >> p.next_gs_log2), w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            if (wq && qr) {
                // The two halves of the wave hold alternating 4-byte pieces of a row.  Exchanging quads 0 <-> 2
                // and 1 <-> 3 between the halves leaves lanes 0..31 with channels 0..15 of the fragment's 32 and
                // lanes 32..63 with channels 16..31: one 16-byte store per lane.  With several fragment columns per
                // wave the pieces are kept until all columns are done, so that the 32-byte halves of a row's
                // contiguous run leave together (stored column by column, a third of the lines left L2 half written).
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    const auto s02 = __builtin_amdgcn_permlane32_swap(qrow[b][0], qrow[b][2], false, false);
                    const auto s13 = __builtin_amdgcn_permlane32_swap(qrow[b][1], qrow[b][3], false, false);
                    const v4i piece = (v4i){(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
                    if (TN > 1) {
                        qout[a][b] = piece;
                    } else {
                        const int64_t m = m0 + (wm * TM + b) * 32 + frag_row_e;
                        const int n = n0 + (wn * TN + a) * 32 + 16 * frag_half_e;
                        if (m < p.M && n < p.N) {
                            if (lw) store_row_piece(m, n, piece, tab);
                            else *reinterpret_cast<v4i *>(p.q + m * p.N + n) = piece;
                        }
                    }
                }
            }
        }
    };
    using M44 = std::integral_constant<int, kMode44>;
    using M88 = std::integral_constant<int, kMode88>;
    using MNone = std::integral_constant<int, kModeNone>;
    using T_ = std::true_type;
    using F_ = std::false_type;
    // Every variant of the step body is straight-line code inside a loop of its own, and the loops follow each
    // other in the order the cases occur (each may run zero times), so that the accumulators never pass
    // through a run-time selection between code paths:
    //   steady 4-bit | transitions (generic, run-time modes) | steady 8-bit | drain: store the last staged
    //   tile without loading | last steps with nothing left to stage
    // The sequence is repeated until the output tile is complete (s == steps); then its epilogue runs and the
    // next output tile of the block, whose first K-steps are already staged, takes over.
    // (Entering a steady-state loop with no load or store in flight lets the compiler count the loads of the
    // loop itself exactly, instead of waiting for all of them before the first LDS store of every step.)
    for (;;) {
        const bool more_tiles = C_::MULTI && ctile + (int)gridDim.x < total_tiles;
        // Nothing in flight (in particular none of the previous epilogue's stores) when the K loop starts: the
        // compiler can then count the register-routed loads of the 4-bit loops exactly.
        if ((n4 + mixed > 0 && !p.x_pre) || PACKED4) __builtin_amdgcn_s_waitcnt(0x0070);
        // When the tile begins with steps that lower their activations, the first K-step starts its accumulators
        // from a zero operand: clearing 16 registers per fragment with the vector ALU would compete with the
        // prologue's lowering work (with plain copies the clearing hides behind the wait for the first loads).
        if (zero_step) step(M44{}, M44{}, T_{}, T_{});
        while (s < steps) {
            if (mode_staged == kMode44 && it_mode == kMode44)
                do step(M44{}, M44{}, T_{}, F_{}); while (s < steps && it_mode == kMode44);
            if (s < steps && mode_staged == kMode44 && it_mode == kMode88) step(M44{}, M88{}, T_{}, F_{});
            if (s < steps && mode_staged == kMode88 && it_mode == kMode88)
                do step(M88{}, M88{}, T_{}, F_{}); while (s < steps && it_mode == kMode88);
            if (s < steps && mode_staged == kMode88 && it_mode == kMode44) step(M88{}, M44{}, T_{}, F_{});   // next tile begins
            while (s < steps && mode_staged != kModeNone && it_mode != kModeNone && (mode_staged == kMode48 || it_mode == kMode48))
                step(mode_staged, it_mode, true, F_{});                                                      // mixed steps
            if (s < steps && mode_staged == kMode88 && it_mode == kModeNone) step(M88{}, MNone{}, T_{}, F_{});
            if (s < steps && mode_staged == kMode44 && it_mode == kModeNone) step(M44{}, MNone{}, T_{}, F_{});
            if (s < steps && mode_staged == kMode48 && it_mode == kModeNone) step(mode_staged, (int)kModeNone, true, F_{});
            // nothing left to stage; the block's very last step reads no fragments ahead
            while (s < steps && mode_staged == kModeNone && (more_tiles || s + 1 < steps)) step(MNone{}, MNone{}, T_{}, F_{});
            if (s < steps && mode_staged == kModeNone && !more_tiles && s + 1 >= steps) step(MNone{}, MNone{}, F_{}, F_{});
        }

        auto epilogue_col = [&](auto a_) {
            if (q_rows && !want_y && !want_acc && !lower_out && !scan_out) epilogue(a_, T_{}, F_{}, F_{}, T_{}, T_{}, F_{}, F_{});
            else if (q_rows && !want_y && !want_acc && !scan_out) epilogue(a_, T_{}, F_{}, F_{}, T_{}, T_{}, T_{}, F_{});
            else if (q_rows && !want_y && !want_acc && !lower_out) epilogue(a_, T_{}, F_{}, F_{}, T_{}, T_{}, F_{}, T_{});
            else if (n_vec && !want_q && want_y && !want_acc) epilogue(a_, F_{}, T_{}, F_{}, T_{}, F_{}, F_{}, F_{});
            else if (n_vec && !want_q && !want_y && want_acc) epilogue(a_, F_{}, F_{}, T_{}, T_{}, F_{}, F_{}, F_{});
            else epilogue(a_, want_q, want_y, want_acc, n_vec, q_rows, lower_out, scan_out);
            FQ_SB();
        };
        epilogue_col(std::integral_constant<int, 0>{});
        if constexpr (TN > 1) epilogue_col(std::integral_constant<int, 1>{});
        if constexpr (TN > 2) epilogue_col(std::integral_constant<int, 2>{});
        if constexpr (TN > 3) epilogue_col(std::integral_constant<int, 3>{});
        static_assert(TN <= 4, "epilogue handles up to four fragment columns");
        if (TN > 1 && q_rows) {
#pragma unroll
            for (int b = 0; b < TM; ++b)
#pragma unroll
                for (int a = 0; a < TN; ++a) {
                    const int64_t m = m0 + (wm * TM + b) * 32 + frag_row_e;
                    const int n = n0 + (wn * TN + a) * 32 + 16 * frag_half_e;
                    if (m < p.M && n < p.N) {
                        if (lower_out) store_row_piece(m, n, qout[a][b], cs_tab + parity * (3 * BN));
                        else *reinterpret_cast<v4i *>(p.q + m * p.N + n) = qout[a][b];
                    }
                }
        }
        if (!more_tiles) break;

        // ---- next output tile of this block
        ctile += (int)gridDim.x;
        {
            int tile_m, tile_n;
            map_tile(ctile, tile_m, tile_n);
            m0 = (int64_t)tile_m * BM;
            n0 = tile_n * BN;
        }
        parity ^= 1;                           // the other table copy was last read two epilogues ago
        fetch_scales(n0, parity);
        zero_step = kZeroStep && mode_staged == kMode44 && it_mode == kMode44;
        if (!zero_step) zero_acc();
        s = 0;
    }
    // ---- scan for the consumer: merge the block's masks into the consumer's scan words (device-scope atomics);
    // the block that finishes last turns the merged masks into positions (highest magnitude bit p of a 4-bit
    // group -> max(0, p - 2); calibrated value for the others) and clears the scan words for the next call.  It is
    // enough that this block's atomics have been performed before its ticket is drawn (no release fence: that
    // would also write back the output tile from L2).
    if (scan_out) {
        // The block's masks go into row blockIdx.x % kFusedScanRows of the consumer's scan words (device-scope atomics that
        // spread over many addresses: on one row they queue up for microseconds); the block that draws the last ticket
        // ORs the rows, writes the positions and leaves every word zero for the next call.
        __syncthreads();
        uint32_t *rows = p.next_scan + kScanHead;
        if (tid < p.next_G) {
            const uint32_t m = mask_tab[tid];
            if (m) atomicOr(rows + (int)(blockIdx.x % kFusedScanRows) * p.next_G + tid, m);
        }
        __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        int *flag = reinterpret_cast<int *>(lds);
        if (tid == 0) *flag = atomicAdd(p.next_scan, 1u) == gridDim.x - 1 ? 1 : 0;
        if (tid < 160) mask_tab[tid] = 0;
        __syncthreads();
        if (*flag) {
            const int used = (int)min(gridDim.x, (unsigned)kFusedScanRows) * p.next_G;
            for (int i = tid; i < used; i += NT) {
                const uint32_t v = __hip_atomic_load(rows + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v) {
                    __hip_atomic_fetch_or(mask_tab + i % p.next_G, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    rows[i] = 0;
                }
            }
            __syncthreads();
            for (int g = tid; g <= p.next_G; g += NT) {
                if (g < p.next_g4) {
                    const uint32_t mask = mask_tab[g] & 0xFEu;   // bit j + 1: some code has its highest magnitude bit at j
                    const int hb = mask ? 31 - __builtin_clz(mask) : 0;
                    p.next_dyn[g] = hb - 3 > 0 ? hb - 3 : 0;
                } else {
                    p.next_dyn[g] = p.next_static[g];
                }
            }
            if (tid == 0) p.next_scan[0] = 0;
        }
    }
}

typedef void (*kernel_fn)(const GemmParams);
struct TileShape {
    int BM, BN, threads, lds;
    bool multi;          // a block of this shape may walk several output tiles (linear form)
    // Measured on MI355X (ViT-B / ViT-L MLP shapes, 8-bit steps), in shader cycles; used by the shape choice:
    double step_alone;   // one K-step of a block that has its CU to itself
    double share;        // relative growth of that time per further block resident on the same CU
    double epilogue;     // epilogue of one output tile
    double lower;        // growth of a K-step whose activations are bit-lowered in the kernel
    kernel_fn fn[2][2];  // [convolution][4-bit weights from the packed codes]
    kernel_fn fn_xp;     // linear form, 4-bit activations from packed codes
};

template <int WAVES_M, int WAVES_N, int TM, int TN>
inline TileShape make_shape(double step_alone, double share, double epilogue, double lower)
{
    using C_ = Cfg<WAVES_M, WAVES_N, TM, TN>;
    return TileShape{C_::BM, C_::BN, C_::NT, C_::LDS_BYTES, C_::MULTI, step_alone, share, epilogue, lower,
                     {{k_mixed<WAVES_M, WAVES_N, TM, TN, false, false>, k_mixed<WAVES_M, WAVES_N, TM, TN, false, true>},
                      {k_mixed<WAVES_M, WAVES_N, TM, TN, true, false>, k_mixed<WAVES_M, WAVES_N, TM, TN, true, true>}},
                     k_mixed<WAVES_M, WAVES_N, TM, TN, false, false, true>};
}

// Shape i of the table, defined in mixed_tile.hip built with -DFQ_TILE=i.
constexpr int kNumTileShapes = 15;
TileShape tile_shape_0();
TileShape tile_shape_1();
TileShape tile_shape_2();
TileShape tile_shape_3();
TileShape tile_shape_4();
TileShape tile_shape_5();
TileShape tile_shape_6();
TileShape tile_shape_7();
TileShape tile_shape_8();
TileShape tile_shape_9();
TileShape tile_shape_10();
TileShape tile_shape_11();
TileShape tile_shape_12();
TileShape tile_shape_13();
TileShape tile_shape_14();

}  // namespace flexiq
