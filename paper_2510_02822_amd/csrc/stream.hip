// Row-streaming form of the mixed GEMM for layers with a short reduction (C = 64, 128 or 256 input channels: the 1x1
// convolutions of the early ResNet stages, Section 8's HBM-bound end of the workloads).  Such a layer is a stream of
// activation rows in and output rows out; the tiled kernel pays a K-step pipeline, a tile switch and an epilogue per
// 4 K-steps there, and its register-routed (bit-lowered) activation pieces get one K-step of latency slack, which
// an HBM-bound layer cannot hide: its latency rises with the low-bit ratio.
//
// Here a block keeps the weights of its (up to 256) output columns in LDS for its whole life, position-expanded copies
// for the 4-bit channel groups and 8-bit tiles for the others (Section 7: cached 4-bit parameters), and walks row tiles
// of 128 rows: the whole tile (all channels) is copied from global memory straight into an LDS ring, several tiles ahead
// of its use, whatever the ratio; the bit-lowering of the activations of 4-bit groups (Section 4.1) is one pass of the
// whole block over the landed tile, in place in LDS, before any fragment is read.  Same int8 MFMA, same int32
// accumulators and the same epilogue arithmetic as the tiled kernel: bit-identical outputs.
//
// Lane roles as in the tiled kernel: the MFMA "A" operand is the weight fragment (32 output channels x 32 channels of
// a unit), "B" the activation fragment (32 rows), so that a lane ends up with four consecutive output channels of one
// row per accumulator quad.
#include <algorithm>

#include "flexiq_internal.h"
#include "flexiq_test.h"
#include "stream_common.h"

namespace flexiq {
namespace stream {

using namespace resident;

struct Params {
    const int8_t *X;        // int8 [M][C], stored channel order
    const uint8_t *X4;      // k_rows, XP builds: packed 4-bit codes [M][C / 2] of the leading 32 * units_p channels (those columns of X are not read)
    const int8_t *W8;       // [U][2][Npad][16], and the position-expanded 4-bit copy w4x_delta bytes further
    const int32_t *ashift;  // [G + 1]
    const float *cs;        // [2][Npad]: x_scale * w_scale, then bias
    int32_t *acc;
    float *y;
    int8_t *q;
    float r_out;
    int64_t M;
    int32_t N, Npad, C;
    int32_t w4x_delta;
    int32_t units, units4;  // C / 32; leading units computed at 4 bits
    int32_t units_p;        // XP builds: leading units that arrive as packed codes (even, <= units4)
    int32_t x_pre;          // activations of those units arrive lowered
    int32_t gs_shift;
    int32_t tiles;          // row tiles of 128
    int32_t slots;          // stages of the activation ring
    int32_t groups;         // k_rows: groups of 32 rows
    // LOWER builds: the layer that reads the int8 rows (its positions, 4-bit prefix and log2 of its group size)
    const int32_t *next_ashift;
    int32_t next_K4, next_gs_log2;
};

constexpr int kRows = 128;        // rows per tile: four waves x 32
constexpr int kMaxCols = 256;     // output columns per block (grid.y walks wider layers)

// Copies row tile t (all channels of its 128 rows) into a ring slot: copy j of a wave moves the 1 KB that holds LDS pieces
// 64 (wave + NW j) .. + 63; voff[j] is the lane's source offset inside the tile (piece order permuted, see swizzle).
template <int C, int COPIES, int NW>
__device__ __forceinline__ void issue_tile(const Params &p, unsigned char *dst, const int *voff, int t, int wave)
{
    const int64_t m0 = (int64_t)t * kRows;
    const int64_t left = p.M - m0;
    const int win = (int)(left < kRows ? left : kRows) * C;    // rows beyond M read as zeros
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + m0 * C), 0, win, kRsrcFlags);
#pragma unroll
    for (int j = 0; j < COPIES; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(dst + 1024 * (wave + NW * j)), 16, voff[j], 0, 0, 0);
}

// Waits until at most n of the wave's copies are outstanding (n <= 48: three tiles of sixteen copies), LDS reads and scalar
// loads all done.
__device__ __forceinline__ void wait_exact(int n)
{
#define FQ_W(k) case k: __builtin_amdgcn_s_waitcnt(0x0070 | ((k) & 15) | (((k) >> 4) << 14)); break;
    switch (n) {
        FQ_W(1) FQ_W(2) FQ_W(3) FQ_W(4) FQ_W(5) FQ_W(6) FQ_W(7) FQ_W(8) FQ_W(9) FQ_W(10) FQ_W(11) FQ_W(12) FQ_W(13) FQ_W(14) FQ_W(15) FQ_W(16)
        FQ_W(17) FQ_W(18) FQ_W(19) FQ_W(20) FQ_W(21) FQ_W(22) FQ_W(23) FQ_W(24) FQ_W(25) FQ_W(26) FQ_W(27) FQ_W(28) FQ_W(29) FQ_W(30) FQ_W(31) FQ_W(32)
        FQ_W(33) FQ_W(34) FQ_W(35) FQ_W(36) FQ_W(37) FQ_W(38) FQ_W(39) FQ_W(40) FQ_W(41) FQ_W(42) FQ_W(43) FQ_W(44) FQ_W(45) FQ_W(46) FQ_W(47) FQ_W(48)
    default: __builtin_amdgcn_s_waitcnt(0x0070); break;
    }
#undef FQ_W
}

// Blocks per compute unit and ring depth for a block of 32 * nt columns and 32 * units channels: the pair that keeps most
// tiles in flight per compute unit (a slot is a whole tile; two to four slots per block; at most two blocks when a wave
// would otherwise hold eight fragment columns of accumulators).  per_cu == 0: does not fit.
struct Plan {
    int per_cu, slots;
};
constexpr Plan plan(int nt, int units)
{
    const int bn = 32 * nt, wbytes = units * 2 * (bn + 2) * 16, slot = kRows * 32 * units;
    Plan best = {0, 0};
    int score = -1;
    for (int b = nt == 8 ? 2 : 4; b >= 1; --b) {
        int s = ((160 * 1024) / b - wbytes - 3 * bn * 4 - 128) / slot;
        if (s > 4) s = 4;
        if (s >= 2 && b * (s - 1) > score) {
            score = b * (s - 1);
            best = {b, s};
        }
    }
    return best;
}

// NT: 32-column fragments of the block (its columns are 32 * NT); UNITS: 32-channel units (C = 32 * UNITS); CW: waves that
// share a group of 32 rows and split the block's columns between them (1: four waves, 2: eight waves per block, two per SIMD);
// QONLY: the call writes int8 rows and nothing else (the usual case between layers): a build without the other outputs'
// address arithmetic, whose registers would otherwise spill, and a reload from scratch waits for every copy in flight
template <int NT, int UNITS, int CW, bool QONLY, bool LOWER = false>
__global__ __launch_bounds__(256 * CW, plan(NT, UNITS).per_cu * CW) void k_stream(const Params p)   // (second figure: waves per SIMD)
{
    static_assert(CW == (plan(NT, UNITS).per_cu <= 2 ? 2 : 1), "eight waves where at most two blocks share a compute unit");
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fh = lane >> 5;
    const int rg = wave & 3, ch = wave >> 2;      // row group of the wave, and which share of the columns it computes
    constexpr int NW = 4 * CW, NTW = NT / CW;     // waves per block, fragment columns per wave
    static_assert(NT % CW == 0, "the columns split evenly");
    constexpr int C = 32 * UNITS, P = 2 * UNITS;   // channels and 16-byte pieces per row
    const int n_blk = blockIdx.y * kMaxCols;       // first output column of this block
    constexpr int BN = 32 * NT;
    constexpr int NS = BN + 2;                     // rows per weight k-plane in LDS (+2: the two planes of a fragment read hit different banks)
    constexpr int wbytes = UNITS * 2 * NS * 16;
    float *const tab = reinterpret_cast<float *>(lds + wbytes);          // [BN] multipliers, [BN] addends
    unsigned char *const ring = lds + wbytes + 3 * BN * 4 + 128;   // (two float tables and the consumer's lowering table; the ring starts on a 128-byte boundary of its own)
    constexpr int slot_bytes = kRows * C;

    // ---- scales and biases (pre-multiplied for the int8 output when it is the only scaled one), positions
    const bool pre_scaled = QONLY || (p.q != nullptr && p.y == nullptr);
    for (int c = tid; c < BN; c += 64 * NW) {
        const int n = n_blk + c;
        const float cs = n < p.Npad ? p.cs[n] : 0.0f, bi = n < p.Npad ? p.cs[p.Npad + n] : 0.0f;
        tab[c] = pre_scaled ? cs * p.r_out : cs;
        tab[BN + c] = pre_scaled ? bi * p.r_out + 128.0f : bi;
    }
    if constexpr (LOWER) fill_lower_table(lds + wbytes + 2 * BN * 4, BN / 4, n_blk, p.next_ashift, p.next_K4, p.next_gs_log2, tid, 64 * NW);
    // positions of up to 8 groups (C <= 256), four bits each, in one scalar
    const int n_low = p.x_pre ? 0 : p.units4;
    uint32_t sa_packed = 0;
    for (int g = 0; g < (n_low > 0 ? ((n_low - 1) >> p.gs_shift) + 1 : 0); ++g) sa_packed |= (uint32_t)p.ashift[g] << (4 * g);
    // ---- copies of a row tile into a ring slot: LDS piece index q = 64 (wave + 4 j) + lane holds row q / P, logical
    // piece (q % P) ^ swizzle(row)
    constexpr int copies_x = (kRows * P) / (64 * NW);   // per wave: 2 (C = 64), 4, 8 (C = 256) with four waves, half with eight
    int voff[copies_x];
#pragma unroll
    for (int j = 0; j < copies_x; ++j) {
        const int qi = 64 * (wave + NW * j) + lane;
        const int row = qi / P, pp = qi % P;
        voff[j] = row * C + ((pp ^ swizzle(row, P)) << 4);
    }

    // ---- weights of the block's columns: unit u, k-plane pl, 64 rows per copy instruction
    {
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.W8, 0, 2 * p.w4x_delta, kRsrcFlags);
        constexpr int copies = UNITS * 2 * (BN / 64 > 0 ? BN / 64 : 1);
        for (int i = wave; i < copies; i += NW) {
            const int per_plane = BN / 64 > 0 ? BN / 64 : 1;
            const int plane = i / per_plane, blk = i % per_plane;      // plane = 2 u + pl
            const int u = plane >> 1;
            const int soff = (u < p.units4 ? p.w4x_delta : 0) + (plane * p.Npad + n_blk + blk * 64) * 16;
            if (BN >= 64 || lane < BN)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(lds + (plane * NS + blk * 64) * 16), 16, lane * 16, soff, 0, 0);
        }
    }
    // ---- prologue: the first slots - 1 tiles of this block are put in flight, right behind the weights
    const int D = p.slots - 1;   // tiles in flight ahead of the one being computed
    int t_load = blockIdx.x, slot_load = 0;
    int mine = 0;   // tiles whose copies this wave has issued
    for (int k = 0; k < D; ++k) {
        if (t_load < p.tiles) issue_tile<C, copies_x, NW>(p, ring + slot_load * slot_bytes, voff, t_load, wave), ++mine;
        t_load += gridDim.x;
        slot_load = slot_load + 1 == p.slots ? 0 : slot_load + 1;
    }

    // the weights (issued before the tiles) and the tables are in place: at most the tile copies are outstanding
    {
        constexpr int w1 = copies_x, w2 = 2 * copies_x, w3 = 3 * copies_x;
        if (mine >= 3) __builtin_amdgcn_s_waitcnt(0x0070 | (w3 & 15) | ((w3 >> 4) << 14));
        else if (mine == 2) __builtin_amdgcn_s_waitcnt(0x0070 | (w2 & 15) | ((w2 >> 4) << 14));
        else if (mine == 1) __builtin_amdgcn_s_waitcnt(0x0070 | (w1 & 15) | ((w1 >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0070);
    }
    block_barrier();

    const int xrow = (32 * rg + fr) * C;
    const bool q_rows = p.q != nullptr && (p.N & 15) == 0;   // int8 rows are stored in 16-byte pieces
    const FragOut fo = {p.acc, p.y, p.q, p.r_out, p.N};
    const int xswz = swizzle(32 * rg + fr, P);
    int slot = 0;
    for (int t = blockIdx.x; t < p.tiles; t += gridDim.x) {
        // the slot that receives tile t + D was read during the previous iteration: every wave is past it
        block_barrier();
        if (t_load < p.tiles) issue_tile<C, copies_x, NW>(p, ring + slot_load * slot_bytes, voff, t_load, wave);
        const bool issued = t_load < p.tiles;
        t_load += gridDim.x;
        slot_load = slot_load + 1 == p.slots ? 0 : slot_load + 1;
        // tile t has landed once at most the copies of the tiles after it are outstanding (and, the first time, the
        // weights: they were issued before everything else)
        {
            int newer = 0;   // tiles issued after tile t
            for (int k = 1, tt = t + (int)gridDim.x; k <= D; ++k, tt += gridDim.x)
                if (tt < p.tiles) ++newer;
            (void)issued;
            // the immediate is the number of copies issued after tile t: vmcnt in bits 3:0 and 15:14, lgkmcnt 0
            constexpr int w1 = copies_x, w2 = 2 * copies_x, w3 = 3 * copies_x;
            static_assert(w3 <= 63, "the counter has six bits");
            if (newer >= 3) __builtin_amdgcn_s_waitcnt(0x0070 | (w3 & 15) | ((w3 >> 4) << 14));
            else if (newer == 2) __builtin_amdgcn_s_waitcnt(0x0070 | (w2 & 15) | ((w2 >> 4) << 14));
            else if (newer == 1) __builtin_amdgcn_s_waitcnt(0x0070 | (w1 & 15) | ((w1 >> 4) << 14));
            else __builtin_amdgcn_s_waitcnt(0x0070);
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        block_barrier();

        // ---- bit-lowering (Section 4.1) of the tile's 4-bit channels, in place: every 16-byte piece of those channels
        // once, by all threads of the block (a wave takes 64 consecutive rows of one piece column, so the position is
        // uniform and the accesses spread over the banks like the fragment reads), before any fragment is read
        if (n_low > 0) {
            unsigned char *xt = ring + slot * slot_bytes;
            uint32_t sap = sa_packed;   // (opaque per tile: the constants derived from it stay out of long-lived scalar registers)
            asm volatile("" : "+s"(sap));
            constexpr int kPasses = (kRows * 2 * UNITS) / (64 * NW);   // pieces per thread when every unit is a 4-bit one
            v4i piece[kPasses];
            v4i *where[kPasses];
#pragma unroll
            for (int k = 0; k < kPasses; ++k) {   // all reads first: their latencies overlap
                const int idx = tid + k * 64 * NW;
                const int row = idx & (kRows - 1), l = idx >> 7;
                where[k] = reinterpret_cast<v4i *>(xt + row * C + ((l ^ swizzle(row, P)) << 4));
                if (idx < kRows * 2 * n_low) {
                    piece[k] = *where[k];
                    // (the ring is only ever written by the copy instructions, which the compiler does not see as stores
                    // to it: it may take what it reads from there for undefined and fold arithmetic on it away)
                    asm volatile("" : "+v"(piece[k]));
                }
            }
#pragma unroll
            for (int k = 0; k < kPasses; ++k) {
                const int idx = tid + k * 64 * NW;
                if (idx >= kRows * 2 * n_low) continue;
                const int l = idx >> 7;
                const int sa = (int)((sap >> (4 * ((l >> 1) >> p.gs_shift))) & 15u);
                const v4i b = lower16_checked(piece[k], sa);
                *where[k] = b;
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            block_barrier();
        }
        const unsigned char *xs = ring + slot * slot_bytes + xrow;
        // all activation fragments of the tile first (UNITS x 16 bytes per lane); then fragment column by fragment column:
        // its weight fragments and matrix instructions, then its epilogue, whose vector-ALU work the scheduler (and the
        // other wave of the SIMD) overlaps with the matrix instructions of the next column
        v4i bfrag[UNITS];
#pragma unroll
        for (int u = 0; u < UNITS; ++u) bfrag[u] = *reinterpret_cast<const v4i *>(xs + (((2 * u + fh) ^ xswz) << 4));

        // Lane: row m; accumulator register 4 g + i of fragment column a: output column 32 a + 8 g + 4 fh + i
        const int64_t m = (int64_t)t * kRows + 32 * rg + fr;
        const bool row_ok = m < p.M;
        // columns left from this lane's first one; made opaque per tile, or the compiler keeps one hoisted lane mask per
        // (fragment, quad, element) in scalar registers and spills them by the hundred
        int lim = p.N - n_blk - 4 * fh;
        asm volatile("" : "+v"(lim));
#pragma unroll
        for (int a = 0; a < NTW; ++a) {
            const int ca = ch * NTW + a;   // fragment column within the block
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0;
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const v4i w = *reinterpret_cast<const v4i *>(lds + ((2 * u + fh) * NS + 32 * ca + fr) * 16);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, bfrag[u], acc, 0, 0, 0);
            }
            store_fragment<QONLY, BN, LOWER>(acc, fo, lds + wbytes, ca, n_blk, m, row_ok, lim, fh, pre_scaled, q_rows);
        }
        slot = slot + 1 == p.slots ? 0 : slot + 1;
    }
    __builtin_amdgcn_s_waitcnt(0x0070);   // nothing of this block's copies is in flight when its LDS is released
}

// ---- The same layer with every wave on its own: a wave owns groups of 32 rows, copies them into a ring of its own (no
// other wave reads them), waits for its own copies only and computes all of the block's columns for them.  No barrier
// after the weights are in place, so the waves of a compute unit drift apart and one wave's waits, bit-lowering and
// epilogue overlap the others' matrix instructions.  And since a 16-byte activation piece is read by exactly one lane,
// once, the bit-lowering (or the expansion of packed codes) happens in registers after the fragment read: no pass over
// the tile in LDS.
constexpr int kGroup = 32;      // rows per group: one MFMA fragment

// Blocks per compute unit, ring slots per wave and waves per block for 32 * nt columns and 32 * units channels: eight waves
// (two blocks per compute unit where LDS allows), fewer where the weights leave no room for eight rings of two slots.
struct RowPlan {
    int per_cu, slots, waves;
};
constexpr RowPlan row_plan(int nt, int units)
{
    const int bn = 32 * nt, wbytes = units * 2 * (bn + 2) * 16, sub = kGroup * 32 * units;
    const int tries[4][2] = {{2, 8}, {1, 8}, {1, 6}, {1, 4}};
    for (int i = 0; i < 4; ++i) {
        const int b = tries[i][0], w = tries[i][1];
        int sl = ((160 * 1024) / b - wbytes - 3 * bn * 4 - 128) / (w * sub);
        if (sl > 4) sl = 4;
        if (sl >= 2) return {b, sl, w};
    }
    return {0, 0, 0};
}

// Ring slot of a row group when the leading `up` units arrive as packed codes (XP builds), in 16-byte pieces:
//   X area, 32 x 2 (UNITS - up) pieces: the int8 channels behind the packed ones, in strips of four pieces (64 bytes of a
//     row): piece lx of row r sits at 128 (lx / 4) + 4 r + ((lx % 4) ^ ((r / 4) % 4)); a copy instruction fills half a
//     strip (sixteen rows), four consecutive lanes fetch 64 contiguous bytes, and the sixteen rows of a fragment read fall
//     into sixteen different 16-byte bank groups;
//   P area behind it, 32 x up pieces: the sixteen bytes of codes of unit u of row r at 64 (u / 2) + 2 r + ((u % 2) ^ ((r / 8) % 2)).
// UNITS - up / 2 copy instructions per group instead of UNITS, every lane of every instruction busy.
//
// Activation fragments of one row group for a lane (row fr, channel half fh of every unit): eight bytes of codes per
// packed unit, expanded here; sixteen int8 values for the others, of which unit UP may still be a 4-bit one (a trailing
// group of 32 channels).
template <int UNITS, int UP>
__device__ __forceinline__ void load_frags_xp(const unsigned char *slot, int fr, int fh, uint32_t sa_packed, int gs_shift, int n_low, v4i *bfrag)
{
    if constexpr (UP <= UNITS) {
        typedef int v2i __attribute__((ext_vector_type(2)));
        v2i codes[UP > 0 ? UP : 1];
        const unsigned char *parea = slot + 1024 * (UNITS - UP);
#pragma unroll
        for (int u = 0; u < UP; ++u)
            codes[u] = *reinterpret_cast<const v2i *>(parea + ((64 * (u >> 1) + 2 * fr + ((u & 1) ^ ((fr >> 3) & 1))) << 4) + 8 * fh);
#pragma unroll
        for (int u = UP; u < UNITS; ++u) {
            const int q = 2 * ((u - UP) & 1) + fh;
            bfrag[u] = *reinterpret_cast<const v4i *>(slot + ((128 * ((u - UP) >> 1) + 4 * fr + (q ^ ((fr >> 2) & 3))) << 4));
        }
#pragma unroll
        for (int u = 0; u < UP; ++u) {
            asm volatile("" : "+v"(codes[u]));
            const int sa = (int)((sa_packed >> (4 * (u >> gs_shift))) & 15u);
            const short t = (short)(4 - sa);
            const uint32_t mask = 0x01010101u * ((0xFFu << sa) & 0xFFu);
            bfrag[u] = (v4i){(int)expand4((uint32_t)codes[u].x << 4, t, mask), (int)expand4((uint32_t)codes[u].x, t, mask),
                             (int)expand4((uint32_t)codes[u].y << 4, t, mask), (int)expand4((uint32_t)codes[u].y, t, mask)};
        }
#pragma unroll
        for (int u = UP; u < UNITS; ++u) asm volatile("" : "+v"(bfrag[u]));
        if constexpr (UP < UNITS) {
            if (UP < n_low) bfrag[UP] = lower16_checked(bfrag[UP], (int)((sa_packed >> (4 * (UP >> gs_shift))) & 15u));
        }
    }
}

// Copies group g (32 rows) to dst.  Plain builds: all channels, COPIES instructions.  XP builds: nxi instructions for the X
// area, npi for the P area (see above).
template <int C, int COPIES, bool XP>
__device__ __forceinline__ void issue_group(const Params &p, unsigned char *dst, const int *voff, const int *voffp, int g, int nxi, int npi)
{
    const int64_t m0 = (int64_t)g * kGroup;
    const int64_t left = p.M - m0;
    const int rows = (int)(left < kGroup ? left : kGroup);       // rows beyond M read as zeros
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + m0 * C), 0, rows * C, kRsrcFlags);
    if constexpr (XP) {
        const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X4 + m0 * (C / 2)), 0, rows * (C / 2), kRsrcFlags);
#pragma unroll
        for (int j = 0; j < COPIES; ++j)
            if (j < nxi) __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(dst + 1024 * j), 16, voff[j], 0, 0, 0);
        unsigned char *parea = dst + 1024 * nxi;
#pragma unroll
        for (int j = 0; j < COPIES / 2; ++j)
            if (j < npi) __builtin_amdgcn_raw_ptr_buffer_load_lds(rp, (lds_ptr_t)(parea + 1024 * j), 16, voffp[j], 0, 0, 0);
    } else {
#pragma unroll
        for (int j = 0; j < COPIES; ++j) __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(dst + 1024 * j), 16, voff[j], 0, 0, 0);
    }
}

template <int NT, int UNITS, bool QONLY, bool XP, bool LOWER = false>
__global__ __launch_bounds__(64 * row_plan(NT, UNITS).waves, (row_plan(NT, UNITS).waves * row_plan(NT, UNITS).per_cu + 3) / 4) void k_rows(const Params p)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;
    constexpr int NW = row_plan(NT, UNITS).waves;
    static_assert(NW > 0, "a block of this shape fits a compute unit");
    constexpr int C = 32 * UNITS, P = 2 * UNITS;
    const int n_blk = blockIdx.y * kMaxCols;
    constexpr int BN = 32 * NT;
    constexpr int NS = BN + 2;
    constexpr int wbytes = UNITS * 2 * NS * 16;
    float *const tab = reinterpret_cast<float *>(lds + wbytes);
    constexpr int sub = kGroup * C;   // bytes of a group of rows
    unsigned char *const ring = lds + wbytes + 3 * BN * 4 + 128 + wave * p.slots * sub;

    const bool pre_scaled = QONLY || (p.q != nullptr && p.y == nullptr);
    for (int c = tid; c < BN; c += 64 * NW) {
        const int n = n_blk + c;
        const float cs = n < p.Npad ? p.cs[n] : 0.0f, bi = n < p.Npad ? p.cs[p.Npad + n] : 0.0f;
        tab[c] = pre_scaled ? cs * p.r_out : cs;
        tab[BN + c] = pre_scaled ? bi * p.r_out + 128.0f : bi;
    }
    if constexpr (LOWER) fill_lower_table(lds + wbytes + 2 * BN * 4, BN / 4, n_blk, p.next_ashift, p.next_K4, p.next_gs_log2, tid, 64 * NW);
    const int n_low = p.x_pre ? 0 : p.units4;
    uint32_t sa_packed = 0;
    for (int g = 0; g < (n_low > 0 ? ((n_low - 1) >> p.gs_shift) + 1 : 0); ++g) sa_packed |= (uint32_t)p.ashift[g] << (4 * g);
    // copies of a group: instruction j moves LDS pieces 64 j .. 64 j + 63 (rows 64 j / P ...), logical piece (q % P) ^ swizzle(row)
    constexpr int copies = (kGroup * P) / 64;   // 2 (C = 64), 4, 8 (C = 256)
    int voff[copies];
    int voffp[XP ? copies / 2 : 1];
    const int up = XP ? p.units_p : 0;
    const int nxi = UNITS - up, npi = up >> 1;          // XP: copy instructions per group for the X area and the P area
    const int cpt = XP ? nxi + npi : copies;            // copy instructions per group
    if constexpr (XP) {
        static_assert(copies == UNITS, "a copy instruction moves 64 pieces");
#pragma unroll
        for (int j = 0; j < copies; ++j) {
            const int row = 16 * (j & 1) + (lane >> 2);
            const int lx = 4 * (j >> 1) + ((lane & 3) ^ ((row >> 2) & 3));
            voff[j] = row * C + ((2 * up + lx) << 4);
        }
#pragma unroll
        for (int j = 0; j < copies / 2; ++j) {
            const int row = lane >> 1;
            const int u = 2 * j + ((lane & 1) ^ ((row >> 3) & 1));
            voffp[j] = row * (C / 2) + (u << 4);
        }
    } else {
#pragma unroll
        for (int j = 0; j < copies; ++j) {
            const int qi = 64 * j + lane;
            const int row = qi / P, pp = qi % P;
            voff[j] = row * C + ((pp ^ swizzle(row, P)) << 4);
        }
    }
    // weights of the block's columns (all waves share the copies)
    {
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.W8, 0, 2 * p.w4x_delta, kRsrcFlags);
        constexpr int per_plane = BN / 64 > 0 ? BN / 64 : 1;
        constexpr int wcopies = UNITS * 2 * per_plane;
        for (int i = wave; i < wcopies; i += NW) {
            const int plane = i / per_plane, blk = i % per_plane;
            const int u = plane >> 1;
            const int soff = (u < p.units4 ? p.w4x_delta : 0) + (plane * p.Npad + n_blk + blk * 64) * 16;
            if (BN >= 64 || lane < BN)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(lds + (plane * NS + blk * 64) * 16), 16, lane * 16, soff, 0, 0);
        }
    }
    // this wave's groups: g0, g0 + stride, ...
    const int stride = (int)gridDim.x * NW;
    const int g0 = (int)blockIdx.x * NW + wave;
    const int D = p.slots - 1;
    int g_load = g0, slot_load = 0, mine = 0;
    for (int k = 0; k < D; ++k) {
        if (g_load < p.groups) issue_group<C, copies, XP>(p, ring + slot_load * sub, voff, voffp, g_load, nxi, npi), ++mine;
        g_load += stride;
        slot_load = slot_load + 1 == p.slots ? 0 : slot_load + 1;
    }
    // weights and tables in place for everybody (this wave's own group copies may stay in flight)
    wait_exact(mine * cpt);
    block_barrier();

    const FragOut fo = {p.acc, p.y, p.q, p.r_out, p.N};
    const bool q_rows = p.q != nullptr && (p.N & 15) == 0;
    const int xswz = swizzle(fr, P);
    int slot = 0;
    for (int g = g0; g < p.groups; g += stride) {
        // the slot that receives group g + D stride held the previous group of this wave: its fragments are in registers
        asm volatile("" ::: "memory");
        if (g_load < p.groups) issue_group<C, copies, XP>(p, ring + slot_load * sub, voff, voffp, g_load, nxi, npi);
        g_load += stride;
        slot_load = slot_load + 1 == p.slots ? 0 : slot_load + 1;
        {
            int newer = 0;   // groups of this wave whose copies were issued after those of group g
            for (int k = 1, gg = g + stride; k <= D; ++k, gg += stride)
                if (gg < p.groups) ++newer;
            wait_exact(newer * cpt);
        }
        asm volatile("" ::: "memory");
        const unsigned char *xs = ring + slot * sub + fr * C;
        // lane (fr, fh) holds the channels 16 fh .. 16 fh + 15 of every unit of row fr
        v4i bfrag[UNITS];
        if constexpr (XP) {
            // (one straight-line body per number of packed units: with a run-time bound every unit would carry both paths)
            switch (up >> 1) {
            case 0: load_frags_xp<UNITS, 0>(ring + slot * sub, fr, fh, sa_packed, p.gs_shift, n_low, bfrag); break;
            case 1: load_frags_xp<UNITS, 2>(ring + slot * sub, fr, fh, sa_packed, p.gs_shift, n_low, bfrag); break;
            case 2: load_frags_xp<UNITS, 4>(ring + slot * sub, fr, fh, sa_packed, p.gs_shift, n_low, bfrag); break;
            case 3: load_frags_xp<UNITS, 6>(ring + slot * sub, fr, fh, sa_packed, p.gs_shift, n_low, bfrag); break;
            default: load_frags_xp<UNITS, 8>(ring + slot * sub, fr, fh, sa_packed, p.gs_shift, n_low, bfrag); break;
            }
        } else {
#pragma unroll
            for (int u = 0; u < UNITS; ++u) bfrag[u] = *reinterpret_cast<const v4i *>(xs + (((2 * u + fh) ^ xswz) << 4));
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                // (the ring is only ever written by the copy instructions, which the compiler does not see as stores)
                asm volatile("" : "+v"(bfrag[u]));
                if (u < n_low) bfrag[u] = lower16_checked(bfrag[u], (int)((sa_packed >> (4 * (u >> p.gs_shift))) & 15u));
            }
        }
        const int64_t m = (int64_t)g * kGroup + fr;
        const bool row_ok = m < p.M;
        int lim = p.N - n_blk - 4 * fh;
        asm volatile("" : "+v"(lim));
#pragma unroll
        for (int a = 0; a < NT; ++a) {
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0;
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const v4i w = *reinterpret_cast<const v4i *>(lds + ((2 * u + fh) * NS + 32 * a + fr) * 16);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, bfrag[u], acc, 0, 0, 0);
            }
            store_fragment<QONLY, BN, LOWER>(acc, fo, lds + wbytes, a, n_blk, m, row_ok, lim, fh, pre_scaled, q_rows);
        }
        slot = slot + 1 == p.slots ? 0 : slot + 1;
    }
    __builtin_amdgcn_s_waitcnt(0x0070);   // nothing of this wave's copies is in flight when the block's LDS is released
}

struct DeviceState {
    bool ready = false;
    int num_cu = 0;
};
static DeviceState g_dev[64];
static int g_force = -1;   // test hook: 1 / 2 = take k_stream / k_rows whenever the layer qualifies, 0 = never, -1 = automatic
static int g_last = 0;

}  // namespace stream

int prepare_stream_kernels(int device)
{
    using namespace stream;
    if (device < 0 || device >= 64) return FLEXIQ_EINVAL;
    if (g_dev[device].ready) return FLEXIQ_OK;
    hipDeviceProp_t prop;
    FLEXIQ_HIP(hipGetDeviceProperties(&prop, device));
    g_dev[device].num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
#define FQ_BOTH(NT_, U_, CW_) (const void *)k_stream<NT_, U_, CW_, false>, (const void *)k_stream<NT_, U_, CW_, true>, (const void *)k_stream<NT_, U_, CW_, true, true>
    const void *fns[] = {FQ_BOTH(2, 2, 1), FQ_BOTH(4, 2, 1), FQ_BOTH(8, 2, 2), FQ_BOTH(2, 4, 2), FQ_BOTH(4, 4, 2), FQ_BOTH(8, 4, 2),
                         FQ_BOTH(2, 8, 2), FQ_BOTH(4, 8, 2), FQ_BOTH(8, 8, 2)};
#undef FQ_BOTH
#define FQ_R(NT_, U_) (const void *)k_rows<NT_, U_, false, false>, (const void *)k_rows<NT_, U_, true, false>, (const void *)k_rows<NT_, U_, true, true>, \
                      (const void *)k_rows<NT_, U_, true, false, true>
    const void *fns_rows[] = {FQ_R(2, 2), FQ_R(4, 2), FQ_R(8, 2), FQ_R(2, 4), FQ_R(4, 4), FQ_R(8, 4), FQ_R(2, 8), FQ_R(4, 8), FQ_R(8, 8)};
#undef FQ_R
    for (const void *fn : fns_rows) FLEXIQ_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    for (const void *fn : fns) FLEXIQ_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    g_dev[device].ready = true;
    return FLEXIQ_OK;
}

// Launches the row-streaming kernel when the call qualifies; *taken says whether it did (0: nothing was launched).
// Qualifying: rows are contiguous [M][C] (linear layers; 1x1 convolutions with stride 1 and no padding), C is 64, 128
// or 256, plain outputs or int8 rows lowered for a consumer (`lower`: flexiq_out.lower_for, checked by the caller; no
// consumer to scan for), and enough rows to give every compute unit several tiles.
// X4 (optional): the packed 4-bit codes of the layer's leading (max_4bit_ch / 64) * 64 channels; taken only when int8 rows
// are the call's only output (the caller has checked alignment and that M * C / 2 fits 31 bits).
int launch_stream(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream_, bool rows_contiguous, int *taken,
                  const uint8_t *X4, const LowerArgs *lower)
{
    using namespace stream;
    *taken = 0;
    g_last = 0;
    if (g_force == 0 || !rows_contiguous) return FLEXIQ_OK;
    if (L->R != 1 || L->S != 1 || (L->C != 64 && L->C != 128 && L->C != 256)) return FLEXIQ_OK;
    if (out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
    const DeviceState &ds = g_dev[L->device];
    if (!ds.ready) return FLEXIQ_OK;
    const int64_t tiles = (M + kRows - 1) / kRows;
    if (tiles > 0x7fffffff) return FLEXIQ_OK;
    const bool q_only = out->q && !out->acc && !out->y && (L->N & 15) == 0;
    const int units_p = X4 && !L->x_prelowered ? (L->max_4bit_ch / 64) * 2 : 0;
    if (units_p > 0 && !q_only) return FLEXIQ_OK;   // (the packed-input builds write int8 rows only)
    // a consumer to lower for: the builds that write int8 rows only, from int8 input
    const bool lowering = lower && lower->ashift;   // (null positions: the consumer has no 4-bit channels at its ratio)
    if (lowering && !(q_only && units_p == 0)) return FLEXIQ_OK;
    // k_rows (every wave on its own) instead of k_stream where it measures faster: whenever packed codes come in (k_stream
    // has no build for them), and where the kernel lowers activations of a layer with 256 channels and at most 64 columns
    // (any share) or 128 columns (half of the channels or more), or 64 channels and at most 64 columns: its bit-lowering
    // runs in registers and overlaps other waves' work, so its time barely grows with the ratio.
    const int lowered = L->x_prelowered ? 0 : L->max_4bit_ch;
    const bool want_rows = units_p > 0 || (lowered > 0 && ((L->C == 256 && (L->N <= 64 || (L->N <= 128 && 2 * lowered >= L->C))) ||
                                                          (L->C == 64 && L->N <= 64)));
    if (g_force < 0) {
        // Taken where it measures faster than the tiled kernel (ResNet-50 stage 1 - 3 shapes at batch 128 and their
        // neighbours).  Always: enough row tiles to give every compute unit a few.  64 channels: up to 256 output columns.
        // 128 channels: up to 512.  256 channels: k_stream (one block per compute unit, which cannot hide the vector-ALU pass
        // of the lowering behind its copies) with at most half of the channels lowered in the kernel unless there are 128
        // columns or more; beyond 256 columns only with at most half lowered.
        if (L->C == 64 && (L->N > 256 || tiles < 2 * (int64_t)ds.num_cu)) return FLEXIQ_OK;
        if (L->C == 128 && (L->N > 512 || tiles < 2 * (int64_t)ds.num_cu)) return FLEXIQ_OK;
        if (L->C == 256) {
            if (L->N <= 256 && (tiles < 8 * (int64_t)ds.num_cu || L->N > 128)) return FLEXIQ_OK;
            if (L->N > 256 && (L->N > 1024 || tiles * ((L->N + kMaxCols - 1) / kMaxCols) < 2 * (int64_t)ds.num_cu)) return FLEXIQ_OK;
            if (!want_rows && 2 * lowered > L->C && (L->N < 128 || L->N > 256)) return FLEXIQ_OK;
        }
    }
    Params p = {};
    p.X = X; p.W8 = L->d_w8; p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift; p.cs = L->d_cs;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.w4x_delta = L->U * 32 * L->Npad;
    p.units = L->C / kUnit;
    p.units4 = L->max_4bit_ch / kUnit;
    p.X4 = units_p > 0 ? X4 : nullptr;
    p.units_p = units_p;
    p.x_pre = L->x_prelowered ? 1 : 0;
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.tiles = (int)tiles;
    if (lowering) { p.next_ashift = lower->ashift; p.next_K4 = lower->K4; p.next_gs_log2 = lower->gs_log2; }
    const int cols = std::min(L->N, kMaxCols);
    const int nt = cols <= 64 ? 2 : (cols <= 128 ? 4 : 8);
    const int bn = 32 * nt;
    const unsigned gy = (unsigned)((L->N + kMaxCols - 1) / kMaxCols);
    // Which of the two kernels
    const RowPlan rp = row_plan(nt, p.units);
    const bool rows_kernel = rp.per_cu > 0 && (g_force == 2 || (g_force < 0 && want_rows));
    if ((g_force == 2 || units_p > 0) && !rows_kernel) return FLEXIQ_OK;   // (packed codes: that kernel only)
    if (rows_kernel) {
        const int64_t groups = (M + kGroup - 1) / kGroup;
        if (groups > 0x7fffffff) return FLEXIQ_OK;
        p.groups = (int)groups;
        p.slots = rp.slots;
        const size_t lds = (size_t)p.units * 2 * (bn + 2) * 16 + 3 * bn * 4 + 128 + (size_t)rp.waves * rp.slots * kGroup * L->C;
        int64_t gx64 = std::max<int64_t>(1, std::min<int64_t>((groups + rp.waves - 1) / rp.waves, (int64_t)ds.num_cu * rp.per_cu / gy));
        if (gy > 1 && gx64 >= 8) gx64 &= ~(int64_t)7;
        void (*fn)(const Params) = nullptr;
#define FQ_R(NT_, U_) (lowering ? k_rows<NT_, U_, true, false, true> : (units_p > 0 ? k_rows<NT_, U_, true, true> : (q_only ? k_rows<NT_, U_, true, false> : k_rows<NT_, U_, false, false>)))
        if (p.units == 2) fn = nt == 2 ? FQ_R(2, 2) : (nt == 4 ? FQ_R(4, 2) : FQ_R(8, 2));
        else if (p.units == 4) fn = nt == 2 ? FQ_R(2, 4) : (nt == 4 ? FQ_R(4, 4) : FQ_R(8, 4));
        else fn = nt == 2 ? FQ_R(2, 8) : (nt == 4 ? FQ_R(4, 8) : FQ_R(8, 8));
#undef FQ_R
        hipLaunchKernelGGL(fn, dim3((unsigned)gx64, gy), dim3(64 * rp.waves), lds, (hipStream_t)stream_, p);
        FLEXIQ_HIP(hipGetLastError());
        *taken = 1;
        g_last = 2;
        return FLEXIQ_OK;
    }
    const int wbytes = p.units * 2 * (bn + 2) * 16, slot = kRows * L->C;
    const Plan pl = plan(nt, p.units);
    if (pl.per_cu == 0) return FLEXIQ_OK;
    const int per_cu = pl.per_cu, slots = pl.slots;
    p.slots = slots;
    const size_t lds = (size_t)wbytes + 3 * bn * 4 + 128 + (size_t)slots * slot;
    // One resident wave of blocks in all: every block loads its weights once and walks tiles / gx row tiles.  With several
    // column blocks (grid.y) the blocks of one row share gx = 0 mod 8, i.e. one XCD and its L2, which then fetches the
    // activation rows from memory once.
    int64_t gx64 = std::max<int64_t>(1, std::min<int64_t>(tiles, (int64_t)ds.num_cu * per_cu / gy));
    if (gy > 1 && gx64 >= 8) gx64 &= ~(int64_t)7;
    const unsigned gx = (unsigned)gx64;
    // eight waves per block (two per SIMD, each pair sharing its rows and splitting the columns) where LDS leaves room
    // for one or two blocks only: the second wave of a SIMD then fills the gaps of the first.  That is every shape but
    // 64 channels with at most 128 columns.
    const int cw = per_cu <= 2 ? 2 : 1;
    if (cw == 1 && !(p.units == 2 && nt <= 4)) return FLEXIQ_EINVAL;   // (no such build: cannot happen with the sizes above)
    void (*fn)(const Params) = nullptr;
#define FQ_Q(NT_, U_, CW_) (lowering ? k_stream<NT_, U_, CW_, true, true> : (q_only ? k_stream<NT_, U_, CW_, true> : k_stream<NT_, U_, CW_, false>))
    if (cw == 1) fn = nt == 2 ? FQ_Q(2, 2, 1) : FQ_Q(4, 2, 1);
    else if (p.units == 2) fn = FQ_Q(8, 2, 2);
    else if (p.units == 4) fn = nt == 2 ? FQ_Q(2, 4, 2) : (nt == 4 ? FQ_Q(4, 4, 2) : FQ_Q(8, 4, 2));
    else fn = nt == 2 ? FQ_Q(2, 8, 2) : (nt == 4 ? FQ_Q(4, 8, 2) : FQ_Q(8, 8, 2));
#undef FQ_Q
    hipLaunchKernelGGL(fn, dim3(gx, gy), dim3(256 * cw), lds, (hipStream_t)stream_, p);
    FLEXIQ_HIP(hipGetLastError());
    *taken = 1;
    g_last = 1;
    return FLEXIQ_OK;
}

}  // namespace flexiq

extern "C" int flexiq_debug_force_stream(int mode)
{
    if (mode < -1 || mode > 2) return FLEXIQ_EINVAL;
    flexiq::stream::g_force = mode;
    return flexiq::stream::g_last;
}
