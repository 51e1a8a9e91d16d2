// 3x3 convolution (stride 1, padding 1) for layers with 64 or 128 input channels: the early ResNet stages, where the
// tiled implicit-GEMM kernel re-reads (and, for 4-bit groups, re-lowers) every activation once per filter tap through the
// 64 B/clk path into LDS.  Here a block keeps the weights of all nine taps of its 64 output columns in LDS for its whole
// life (position-expanded copies for the 4-bit channel groups, 8-bit tiles for the others: Section 7's cached 4-bit
// parameters) and walks image tiles of TR output rows: the TR + 2 input rows of a tile, with one zero pixel to the left
// and right, are copied from global memory straight into one of two or three LDS buffers, one or two tiles ahead; the
// bit-lowering of the 4-bit groups (Section 4.1) is one pass over the landed tile, in place, once per activation
// instead of once per tap; the nine taps are nine shifted reads of the same LDS image.  Same int8 MFMA, int32
// accumulators and epilogue arithmetic as the tiled kernel: bit-identical outputs.
//
// Block: eight computing waves and one loading wave.  Computing wave w owns the output pixels 32 w .. 32 w + 31 and
// 32 (w + 8) .. of the tile (row-major over its rows) and both 32-column fragments; the loading wave issues every copy
// and is the only one that waits for them, so the stores of the computing waves never stand between a wave and its
// operands (stores and loads share one counter).
#include <algorithm>

#include "flexiq_internal.h"
#include "flexiq_test.h"
#include "stream_common.h"

namespace flexiq {
namespace conv3 {

using namespace resident;

struct Params {
    const int8_t *X;        // int8 NHWC [B][H][W][C], stored channel order
    const int8_t *W8;       // [9 * C/32][2][Npad][16], and the position-expanded 4-bit copy w4x_delta bytes further
    const int32_t *ashift;  // [G + 1]
    const float *cs;        // [2][Npad]
    int32_t *acc;
    float *y;
    int8_t *q;
    float r_out;
    int32_t B, H, W, N, Npad;
    int32_t w4x_delta;
    int32_t units4;         // leading 32-channel units computed at 4 bits
    int32_t x_pre;          // activations of those units arrive lowered
    int32_t gs_shift;
    int32_t TR;             // output rows per tile
    int32_t tiles_per_img, tiles;
    int32_t npix;           // LDS pixels per tile: (TR + 2) * (W + 2)
    int32_t copies;         // 1 KB copy instructions per tile
    int32_t nbuf;           // tile buffers (2 to 4)
    // LOWER builds: the layer that reads the int8 output (its positions, 4-bit prefix and log2 of its group size)
    const int32_t *next_ashift;
    int32_t next_K4, next_gs_log2;
};

constexpr int kCols = 64;           // output columns per block
constexpr int kWaves = 8;           // computing waves
constexpr int kMaxCopies = 40;      // per tile: at most 40 KB
constexpr int kFar = 0x40000000;    // source offset of a pixel that reads as zero (beyond every window)

// Copies the TR + 2 input rows of tile t (with their zero columns) into a tile buffer: copy j moves the 1 KB of LDS pieces
// 64 j .. 64 j + 63; voff[j]: the lane's source offset relative to the first pixel of the tile's first output row.
template <int C>
__device__ __forceinline__ void issue_tile(const Params &p, unsigned char *dst, const int *voff, int t)
{
    const int img = t / p.tiles_per_img, y0 = (t - img * p.tiles_per_img) * p.TR;
    const int img_bytes = p.H * p.W * C;
    // window = the image: rows above and below it are out of range and read as zeros
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + (int64_t)img * img_bytes), 0, img_bytes, kRsrcFlags);
    const int row0 = y0 * p.W * C;
#pragma unroll
    for (int j = 0; j < kMaxCopies; ++j)
        if (j < p.copies) __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(dst + 1024 * j), 16, voff[j] + row0, 0, 0, 0);
}

// The 9 * UNITS steps (tap, 32-channel unit) of R fragments of 32 pixels times both 32-column fragments.  The operands of
// step s + 1 (one activation piece per pixel fragment, two weight pieces) are read from LDS before the matrix instructions
// of step s are issued; the scheduling fences pin that order (left alone, the compiler hoists every read and spills).
// base[9 r + tap]: LDS offset of the lane's pixel of fragment r under that tap, k-half folded in.
template <int UNITS, int R>
__device__ __forceinline__ void tile_mma(const unsigned char *xt, const unsigned char *wbase, const int *base, v16i *acc)
{
    constexpr int C = 32 * UNITS, P = 2 * UNITS, NS = kCols + 2, kSteps = 9 * UNITS;
    v4i b[2][R], w[2][2];
    auto operands = [&](int s, int k) {
        const int tap = s / UNITS, u = s % UNITS;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            // unit u sits at piece pair u ^ (swizzle of the pixel >> 1); the pixel index is base / C
            int o = base[9 * r + tap];
            asm volatile("" : "+v"(o));   // (pins the address arithmetic to this step: hoisted, it costs a register per read)
            const int sh = swizzle((int)((unsigned)o / C), P) >> 1;
            b[k][r] = *reinterpret_cast<const v4i *>(xt + o + ((u ^ sh) << 5));
        }
        const unsigned char *ws = wbase + (s * 2) * NS * 16;
        w[k][0] = *reinterpret_cast<const v4i *>(ws);
        w[k][1] = *reinterpret_cast<const v4i *>(ws + 512);
    };
#pragma unroll
    for (int i = 0; i < 2 * R; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0;
    operands(0, 0);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
        const int k = s & 1;
        if (s + 1 < kSteps) operands(s + 1, k ^ 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[2 * r] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[k][0], b[k][r], acc[2 * r], 0, 0, 0);
            acc[2 * r + 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[k][1], b[k][r], acc[2 * r + 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Waits until at most n of this wave's vector-memory operations are outstanding (n rounded down to a multiple of four
// below 64; the count sits in bits 3:0 and 15:14 of the immediate), and for its LDS operations.
__device__ __forceinline__ void wait_outstanding(int n)
{
#define FQ_W(k) case k: __builtin_amdgcn_s_waitcnt(0x0070 | ((4 * k) & 15) | (((4 * k) >> 4) << 14)); break;
    switch (n >= 60 ? 15 : n >> 2) {
        FQ_W(0) FQ_W(1) FQ_W(2) FQ_W(3) FQ_W(4) FQ_W(5) FQ_W(6) FQ_W(7) FQ_W(8) FQ_W(9) FQ_W(10) FQ_W(11) FQ_W(12) FQ_W(13) FQ_W(14) FQ_W(15)
    }
#undef FQ_W
}

template <int UNITS, bool QONLY, bool LOWER = false>
__global__ __launch_bounds__(64 * (kWaves + 1), 3) void k_conv3(const Params p)   // (nine waves: three on one SIMD)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int C = 32 * UNITS, P = 2 * UNITS;
    constexpr int NS = kCols + 2;                       // rows per weight plane in LDS
    constexpr int planes = 9 * UNITS * 2;               // (tap, unit, k-half)
    constexpr int wbytes = planes * NS * 16;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;
    const int n_blk = blockIdx.y * kCols;
    float *const tab = reinterpret_cast<float *>(lds + wbytes);   // [64] multipliers, [64] addends, then the consumer's lowering table
    unsigned char *const bufs = lds + wbytes + 3 * kCols * 4;
    const int tile_bytes = p.copies * 1024;
    const int Wp = p.W + 2;

    const int n_low = p.x_pre ? 0 : p.units4;
    uint32_t sa_packed = 0;   // positions of up to 4 groups, four bits each
    for (int g = 0; g < (n_low > 0 ? ((n_low - 1) >> p.gs_shift) + 1 : 0); ++g) sa_packed |= (uint32_t)p.ashift[g] << (4 * g);
    // a block walks a run of consecutive tiles: the input rows two neighbouring tiles share are then fetched from memory
    // once (by this block's XCD) instead of once per L2
    const int t_first = (int)((int64_t)blockIdx.x * p.tiles / gridDim.x), t_end = (int)((int64_t)(blockIdx.x + 1) * p.tiles / gridDim.x);
    if (wave == kWaves) {
        // ================= the loading wave =================
        // LDS piece q = 64 j + lane of a tile buffer holds pixel q / P (row-major over TR + 2 rows of W + 2 pixels),
        // logical piece (q % P) ^ swizzle(pixel).  voff[j]: its source offset relative to the first pixel of the tile's
        // first output row; pixels of the zero columns get an offset beyond every window.
        int voff[kMaxCopies];
        int t_load = t_first, b_load = 0;
        const int ahead = p.nbuf - 1;
        {
            // (one division; from copy to copy the pixel advances by 64 / P).  The copies
            // of the block's first tile are issued as their offsets become known.
            const int pp = lane % P;
            int lp = lane / P;
            int ry = lp / Wp, px = lp - ry * Wp;
            const bool first = t_first < t_end;
            const int img = first ? t_first / p.tiles_per_img : 0, y0 = first ? (t_first - img * p.tiles_per_img) * p.TR : 0;
            const int img_bytes = p.H * p.W * C;
            const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + (int64_t)img * img_bytes), 0, img_bytes, kRsrcFlags);
            const int row0 = y0 * p.W * C;
            const bool narrow = Wp < 64 / P;   // (an image row shorter than a copy's pixels: the general form, one division per copy)
#pragma unroll
            for (int j = 0; j < kMaxCopies; ++j) {
                voff[j] = kFar;
                if (j < p.copies) {   // (the whole block waits for this loop: nothing is computed for copies that do not exist)
                    const bool real = lp < p.npix && px >= 1 && px <= p.W;
                    voff[j] = real ? ((ry - 1) * p.W + (px - 1)) * C + ((pp ^ swizzle(lp, P)) << 4) : kFar;
                    if (first) __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_ptr_t)(bufs + 1024 * j), 16, voff[j] + row0, 0, 0, 0);
                    lp += 64 / P;
                    if (narrow) {
                        ry = lp / Wp;
                        px = lp - ry * Wp;
                    } else {
                        px += 64 / P;
                        const bool wrap = px >= Wp;
                        px -= wrap ? Wp : 0;
                        ry += wrap ? 1 : 0;
                    }
                }
            }
            ++t_load;
            b_load = 1 == p.nbuf ? 0 : 1;
        }
        // the next tiles are on their way as well while the other waves fetch the weights
        for (int k = 1; k < ahead; ++k) {
            if (t_load < t_end) issue_tile<C>(p, bufs + b_load * tile_bytes, voff, t_load);
            ++t_load;
            b_load = b_load + 1 == p.nbuf ? 0 : b_load + 1;
        }
        block_barrier();   // (the computing waves' weights and tables are in place)
        for (int t = t_first; t < t_end; ++t) {
            // tile t has landed once at most the copies of the tiles issued after it are outstanding
            int newer = 0;
            for (int k = 1; k < ahead; ++k) newer += t + k < t_end ? 1 : 0;
            wait_outstanding(newer * p.copies);
            block_barrier();     // A: tile t may be read; the buffer of tile t - 1 is free
            if (t_load < t_end) issue_tile<C>(p, bufs + b_load * tile_bytes, voff, t_load);
            ++t_load;
            b_load = b_load + 1 == p.nbuf ? 0 : b_load + 1;
            if (n_low > 0) block_barrier();   // L: the computing waves have lowered tile t
        }
        __builtin_amdgcn_s_waitcnt(0x0070);
        return;
    }

    // ---- weights of the block's columns: global plane (tap * UNITS + u) * 2 + k-half, 64 rows of 16 bytes per copy
    {
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.W8, 0, 2 * p.w4x_delta, kRsrcFlags);
        for (int i = wave; i < planes; i += kWaves) {   // (the eight computing waves: the loading wave's counter is for tiles only)
            const int u = (i >> 1) % UNITS;
            const int soff = (u < p.units4 ? p.w4x_delta : 0) + (i * p.Npad + n_blk) * 16;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(lds + i * NS * 16), 16, lane * 16, soff, 0, 0);
        }
    }
    const bool pre_scaled = QONLY || (p.q != nullptr && p.y == nullptr);
    if (tid < kCols) {
        const int n = n_blk + tid;
        const float cs = n < p.Npad ? p.cs[n] : 0.0f, bi = n < p.Npad ? p.cs[p.Npad + n] : 0.0f;
        tab[tid] = pre_scaled ? cs * p.r_out : cs;
        tab[kCols + tid] = pre_scaled ? bi * p.r_out + 128.0f : bi;
    }
    if constexpr (LOWER) fill_lower_table(lds + wbytes + 2 * kCols * 4, kCols / 4, n_blk, p.next_ashift, p.next_K4, p.next_gs_log2, tid, 64 * (kWaves + 1));
    __builtin_amdgcn_s_waitcnt(0x0070);   // weights and tables
    block_barrier();

    // ================= the computing waves =================
    // fragment f of the tile: output pixels 32 f .. 32 f + 31 (row-major); this wave: f = wave and wave + 8
    const int tp_all = p.TR * p.W;
    const int F = (tp_all + 31) >> 5;
    const bool two = F > kWaves;   // every wave runs two pixel fragments per tile (else one)
    int base[2][9];   // per fragment and tap: LDS offset of the lane's pixel, k-half folded in
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        int tp = 32 * (wave + kWaves * r) + fr;
        if (tp >= tp_all) tp = 0;   // (lanes beyond the tile compute pixel 0 again and store nothing)
        const int ty = tp / p.W, tx = tp - ty * p.W;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int lp = (ty + tap / 3) * Wp + tx + tap % 3;
            const int s = swizzle(lp, P);
            base[r][tap] = lp * C + ((fh ^ (s & 1)) << 4);
        }
    }
    const unsigned char *wbase = lds + (fh * NS + fr) * 16;
    const bool q_rows = p.q != nullptr && (p.N & 15) == 0;
    const FragOut fo = {p.acc, p.y, p.q, p.r_out, p.N};
    const int CPP = (p.npix + 63) >> 6;   // 64-pixel chunks of a tile buffer

    int b_cur = 0;
    for (int t = t_first; t < t_end; ++t) {
        block_barrier();   // A
        unsigned char *xt = bufs + b_cur * tile_bytes;
        if (n_low > 0) {
            // ---- bit-lowering of the tile's 4-bit channels, in place: a wave takes 64 consecutive pixels of one logical
            // piece at a time, so the position is uniform
            uint32_t sap = sa_packed;
            asm volatile("" : "+s"(sap));
            const int total = 2 * n_low * CPP;
            for (int c = wave; c < total; c += kWaves) {
                const int l = c / CPP, j = c - l * CPP;
                const int pix = 64 * j + lane;
                const int sa = (int)((sap >> (4 * ((l >> 1) >> p.gs_shift))) & 15u);
                if (pix < p.npix) {
                    v4i *where = reinterpret_cast<v4i *>(xt + pix * C + ((l ^ swizzle(pix, P)) << 4));
                    v4i piece = *where;
                    asm volatile("" : "+v"(piece));   // (the buffers are only written by copy instructions the compiler does not see as stores)
                    *where = lower16_checked(piece, sa);
                }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);
            block_barrier();   // L
        }

        const int img = t / p.tiles_per_img, y0 = (t - img * p.tiles_per_img) * p.TR;
        const int rows_ok = min(p.TR, p.H - y0);
        const int64_t m0 = ((int64_t)img * p.H + y0) * p.W;   // output row index of the tile's first pixel
        int lim = p.N - n_blk - 4 * fh;
        asm volatile("" : "+v"(lim));
        const int tp0 = 32 * wave + fr;
        if (two) {
            // (a wave without a second fragment computes pixel 0 again in its place and stores nothing)
            v16i acc[4];
            tile_mma<UNITS, 2>(xt, wbase, &base[0][0], acc);
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int tp = tp0 + 32 * kWaves * r;
                const bool row_ok = tp < rows_ok * p.W;
                store_fragment<QONLY, kCols, LOWER>(acc[2 * r], fo, lds + wbytes, 0, n_blk, m0 + tp, row_ok, lim, fh, pre_scaled, q_rows);
                __builtin_amdgcn_sched_barrier(0);   // (one fragment at a time: interleaved, their temporaries spill)
                store_fragment<QONLY, kCols, LOWER>(acc[2 * r + 1], fo, lds + wbytes, 1, n_blk, m0 + tp, row_ok, lim, fh, pre_scaled, q_rows);
                __builtin_amdgcn_sched_barrier(0);   // (one fragment at a time: interleaved, their temporaries spill)
            }
        } else {
            v16i acc[2];
            tile_mma<UNITS, 1>(xt, wbase, &base[0][0], acc);
            const bool row_ok = tp0 < rows_ok * p.W;
            store_fragment<QONLY, kCols, LOWER>(acc[0], fo, lds + wbytes, 0, n_blk, m0 + tp0, row_ok, lim, fh, pre_scaled, q_rows);
            __builtin_amdgcn_sched_barrier(0);   // (one fragment at a time: interleaved, their temporaries spill)
            store_fragment<QONLY, kCols, LOWER>(acc[1], fo, lds + wbytes, 1, n_blk, m0 + tp0, row_ok, lim, fh, pre_scaled, q_rows);
            __builtin_amdgcn_sched_barrier(0);   // (one fragment at a time: interleaved, their temporaries spill)
        }
        b_cur = b_cur + 1 == p.nbuf ? 0 : b_cur + 1;
    }
}

struct DeviceState {
    bool ready = false;
    int num_cu = 0;
};
static DeviceState g_dev[64];
static int g_force = -1;   // test hook: 1 = take this kernel whenever the layer qualifies, 0 = never, -1 = automatic
static int g_rows = 0;     // test hook: output rows per tile (0 = automatic)
static int g_last = 0;

}  // namespace conv3

int prepare_conv3_kernels(int device)
{
    using namespace conv3;
    if (device < 0 || device >= 64) return FLEXIQ_EINVAL;
    if (g_dev[device].ready) return FLEXIQ_OK;
    hipDeviceProp_t prop;
    FLEXIQ_HIP(hipGetDeviceProperties(&prop, device));
    g_dev[device].num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const void *fns[] = {(const void *)k_conv3<2, false>, (const void *)k_conv3<2, true>, (const void *)k_conv3<4, false>,
                         (const void *)k_conv3<4, true>, (const void *)k_conv3<2, true, true>, (const void *)k_conv3<4, true, true>};
    for (const void *fn : fns) FLEXIQ_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    g_dev[device].ready = true;
    return FLEXIQ_OK;
}

// Launches the 3x3 kernel when the call qualifies; *taken says whether it did (0: nothing was launched).  Qualifying: a 3x3
// filter, stride 1, padding 1, 64 or 128 input channels, plain outputs or int8 output lowered for a consumer (`lower`:
// flexiq_out.lower_for, checked by the caller; no consumer to scan for), an image whose
// tile of at least one output row fits a 40 KB buffer, and enough tiles to occupy the chip.
int launch_conv3(const flexiq_layer *L, const int8_t *X, int B, int H, int W, int stride, int pad, const flexiq_out *out, void *stream_,
                 int *taken, const LowerArgs *lower)
{
    using namespace conv3;
    *taken = 0;
    g_last = 0;
    if (g_force == 0) return FLEXIQ_OK;
    if (L->R != 3 || L->S != 3 || stride != 1 || pad != 1 || (L->C != 64 && L->C != 128)) return FLEXIQ_OK;
    if (out->scan_for || out->x4 || out->x6) return FLEXIQ_OK;
    const bool q_only = out->q && !out->acc && !out->y && (L->N & 15) == 0;
    const bool lowering = lower && lower->ashift;   // (null positions: the consumer has no 4-bit channels at its ratio)
    if (lowering && !q_only) return FLEXIQ_OK;   // (the lowering build writes int8 only)
    const DeviceState &ds = g_dev[L->device];
    if (!ds.ready) return FLEXIQ_OK;
    if ((int64_t)H * W * L->C >= (1 << 29) || W > 1024) return FLEXIQ_OK;
    const int units = L->C / kUnit;
    const int wbytes = 9 * units * 2 * (kCols + 2) * 16 + 3 * kCols * 4;
    const int gy = (L->N + kCols - 1) / kCols;
    // output rows per tile: every choice whose buffer fits 40 KB, whose pixels fit sixteen fragments and of which two
    // buffers fit next to the weights; the one with the least estimated time of the busiest compute unit (matrix
    // instructions of its fragments per SIMD, plus a fixed cost per tile)
    int best_tr = 0, best_nbuf = 0;
    double best_cost = 0;
    const int blocks = std::max(1, ds.num_cu / gy);
    for (int tr = 1; tr <= H; ++tr) {
        if (g_rows > 0 && tr != g_rows) continue;
        const int npix = (tr + 2) * (W + 2);
        const int copies = (npix * L->C + 1023) / 1024;
        const int frags = (tr * W + 31) / 32;
        if (copies > kMaxCopies || frags > 2 * kWaves) break;
        const int nbuf = std::min(4, (160 * 1024 - wbytes) / (copies * 1024));
        if (nbuf < 2) break;
        const int64_t tiles = (int64_t)B * ((H + tr - 1) / tr);
        const int64_t rounds = (tiles + blocks - 1) / blocks;
        const double cost = (double)rounds * ((frags > kWaves ? 2 : 1) * 2.0 * units * 18 * 32 + 700.0);
        if (best_tr == 0 || cost < best_cost) {
            best_tr = tr;
            best_nbuf = nbuf;
            best_cost = cost;
        }
    }
    if (best_tr == 0) return FLEXIQ_OK;
    const int64_t tiles = (int64_t)B * ((H + best_tr - 1) / best_tr);
    if (tiles > 0x7fffffff) return FLEXIQ_OK;
    if (g_force < 0 && (int64_t)B * H * W < 256 * (int64_t)ds.num_cu) return FLEXIQ_OK;   // too little work to amortise the weight load
    Params p = {};
    p.X = X; p.W8 = L->d_w8; p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift; p.cs = L->d_cs;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.B = B; p.H = H; p.W = W; p.N = L->N; p.Npad = L->Npad;
    p.w4x_delta = L->U * 32 * L->Npad;
    p.units4 = L->max_4bit_ch / kUnit;
    p.x_pre = L->x_prelowered ? 1 : 0;
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.TR = best_tr;
    p.tiles_per_img = (H + best_tr - 1) / best_tr;
    p.tiles = (int)tiles;
    p.npix = (best_tr + 2) * (W + 2);
    p.copies = (p.npix * L->C + 1023) / 1024;
    p.nbuf = best_nbuf;
    const size_t lds = (size_t)wbytes + (size_t)p.nbuf * p.copies * 1024;
    int64_t gx64 = std::max<int64_t>(1, std::min<int64_t>(tiles, ds.num_cu / gy));
    if (gy > 1 && gx64 >= 8) gx64 &= ~(int64_t)7;   // the column blocks of a tile share an XCD and its L2
    if (lowering) { p.next_ashift = lower->ashift; p.next_K4 = lower->K4; p.next_gs_log2 = lower->gs_log2; }
    void (*fn)(const Params) = units == 2 ? (q_only ? k_conv3<2, true> : k_conv3<2, false>) : (q_only ? k_conv3<4, true> : k_conv3<4, false>);
    if (lowering) fn = units == 2 ? k_conv3<2, true, true> : k_conv3<4, true, true>;
    hipLaunchKernelGGL(fn, dim3((unsigned)gx64, (unsigned)gy), dim3(64 * (kWaves + 1)), lds, (hipStream_t)stream_, p);
    FLEXIQ_HIP(hipGetLastError());
    *taken = 1;
    g_last = 1;
    return FLEXIQ_OK;
}

}  // namespace flexiq

extern "C" int flexiq_debug_force_conv3(int mode, int rows_per_tile)
{
    if (mode < -1 || mode > 1 || rows_per_tile < 0) return FLEXIQ_EINVAL;
    flexiq::conv3::g_force = mode;
    flexiq::conv3::g_rows = rows_per_tile;
    return flexiq::conv3::g_last;
}
