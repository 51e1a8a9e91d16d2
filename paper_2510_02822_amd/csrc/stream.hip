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
    int32_t x_pre;          // activations of those units arrive lowered
    int32_t gs_shift;
    int32_t tiles;          // row tiles of 128
    int32_t slots;          // stages of the activation ring
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
        int s = ((160 * 1024) / b - wbytes - 2 * bn * 4 - 128) / slot;
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
template <int NT, int UNITS, int CW, bool QONLY>
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
    unsigned char *const ring = lds + wbytes + 2 * BN * 4 + 128;   // (the ring starts on a 128-byte boundary of its own)
    constexpr int slot_bytes = kRows * C;

    // ---- scales and biases (pre-multiplied for the int8 output when it is the only scaled one), positions
    const bool pre_scaled = QONLY || (p.q != nullptr && p.y == nullptr);
    for (int c = tid; c < BN; c += 64 * NW) {
        const int n = n_blk + c;
        const float cs = n < p.Npad ? p.cs[n] : 0.0f, bi = n < p.Npad ? p.cs[p.Npad + n] : 0.0f;
        tab[c] = pre_scaled ? cs * p.r_out : cs;
        tab[BN + c] = pre_scaled ? bi * p.r_out + 128.0f : bi;
    }
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
            store_fragment<QONLY, BN>(acc, fo, lds + wbytes, ca, n_blk, m, row_ok, lim, fh, pre_scaled, q_rows);
        }
        slot = slot + 1 == p.slots ? 0 : slot + 1;
    }
    __builtin_amdgcn_s_waitcnt(0x0070);   // nothing of this block's copies is in flight when its LDS is released
}

struct DeviceState {
    bool ready = false;
    int num_cu = 0;
};
static DeviceState g_dev[64];
static int g_force = -1;   // test hook: 1 = take this kernel whenever the layer qualifies, 0 = never, -1 = automatic
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
#define FQ_BOTH(NT_, U_, CW_) (const void *)k_stream<NT_, U_, CW_, false>, (const void *)k_stream<NT_, U_, CW_, true>
    const void *fns[] = {FQ_BOTH(2, 2, 1), FQ_BOTH(4, 2, 1), FQ_BOTH(8, 2, 2), FQ_BOTH(2, 4, 2), FQ_BOTH(4, 4, 2), FQ_BOTH(8, 4, 2),
                         FQ_BOTH(2, 8, 2), FQ_BOTH(4, 8, 2), FQ_BOTH(8, 8, 2)};
#undef FQ_BOTH
    for (const void *fn : fns) FLEXIQ_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    g_dev[device].ready = true;
    return FLEXIQ_OK;
}

// Launches the row-streaming kernel when the call qualifies; *taken says whether it did (0: nothing was launched).
// Qualifying: rows are contiguous [M][C] (linear layers; 1x1 convolutions with stride 1 and no padding), C is 64, 128
// or 256, plain outputs (no consumer to lower or scan for), and enough rows to give every compute unit several tiles.
int launch_stream(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream_, bool rows_contiguous, int *taken)
{
    using namespace stream;
    *taken = 0;
    g_last = 0;
    if (g_force == 0 || !rows_contiguous) return FLEXIQ_OK;
    if (L->R != 1 || L->S != 1 || (L->C != 64 && L->C != 128 && L->C != 256)) return FLEXIQ_OK;
    if (out->lower_for || out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
    const DeviceState &ds = g_dev[L->device];
    if (!ds.ready) return FLEXIQ_OK;
    const int64_t tiles = (M + kRows - 1) / kRows;
    if (tiles > 0x7fffffff) return FLEXIQ_OK;
    if (g_force < 0) {
        // Taken where it measures faster than the tiled kernel (ResNet-50 stage 1 - 3 shapes at batch 128 and their
        // neighbours).  Always: enough row tiles to give every compute unit a few.  64 channels: up to 256 output columns.
        // 128 channels: up to 512.  256 channels (one block per compute unit, which cannot hide the vector-ALU pass of the
        // lowering behind its copies): at most half of the channels lowered in the kernel unless there are 128 columns
        // or more; beyond 256 columns only with at most half lowered.
        const int lowered = L->x_prelowered ? 0 : L->max_4bit_ch;
        if (L->C == 64 && (L->N > 256 || tiles < 2 * (int64_t)ds.num_cu)) return FLEXIQ_OK;
        if (L->C == 128 && (L->N > 512 || tiles < 2 * (int64_t)ds.num_cu)) return FLEXIQ_OK;
        if (L->C == 256) {
            if (L->N <= 256 && (tiles < 8 * (int64_t)ds.num_cu || L->N > 128)) return FLEXIQ_OK;
            if (L->N > 256 && (L->N > 1024 || tiles * ((L->N + kMaxCols - 1) / kMaxCols) < 2 * (int64_t)ds.num_cu)) return FLEXIQ_OK;
            if (2 * lowered > L->C && (L->N < 128 || L->N > 256)) return FLEXIQ_OK;
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
    p.x_pre = L->x_prelowered ? 1 : 0;
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.tiles = (int)tiles;
    const int cols = std::min(L->N, kMaxCols);
    const int nt = cols <= 64 ? 2 : (cols <= 128 ? 4 : 8);
    const int bn = 32 * nt;
    const int wbytes = p.units * 2 * (bn + 2) * 16, slot = kRows * L->C;
    const Plan pl = plan(nt, p.units);
    if (pl.per_cu == 0) return FLEXIQ_OK;
    const int per_cu = pl.per_cu, slots = pl.slots;
    p.slots = slots;
    const size_t lds = (size_t)wbytes + 2 * bn * 4 + 128 + (size_t)slots * slot;
    // One resident wave of blocks in all: every block loads its weights once and walks tiles / gx row tiles.  With several
    // column blocks (grid.y) the blocks of one row share gx = 0 mod 8, i.e. one XCD and its L2, which then fetches the
    // activation rows from memory once.
    const unsigned gy = (unsigned)((L->N + kMaxCols - 1) / kMaxCols);
    int64_t gx64 = std::max<int64_t>(1, std::min<int64_t>(tiles, (int64_t)ds.num_cu * per_cu / gy));
    if (gy > 1 && gx64 >= 8) gx64 &= ~(int64_t)7;
    const unsigned gx = (unsigned)gx64;
    // eight waves per block (two per SIMD, each pair sharing its rows and splitting the columns) where LDS leaves room
    // for one or two blocks only: the second wave of a SIMD then fills the gaps of the first.  That is every shape but
    // 64 channels with at most 128 columns.
    const int cw = per_cu <= 2 ? 2 : 1;
    if (cw == 1 && !(p.units == 2 && nt <= 4)) return FLEXIQ_EINVAL;   // (no such build: cannot happen with the sizes above)
    const bool q_only = out->q && !out->acc && !out->y && (L->N & 15) == 0;
    void (*fn)(const Params) = nullptr;
#define FQ_Q(NT_, U_, CW_) (q_only ? k_stream<NT_, U_, CW_, true> : k_stream<NT_, U_, CW_, false>)
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
    if (mode < -1 || mode > 1) return FLEXIQ_EINVAL;
    flexiq::stream::g_force = mode;
    return flexiq::stream::g_last;
}
