// Host side of the mixed GEMM / implicit-GEMM convolution (Section 7 of the paper): tile-shape choice,
// launch, and the C entry points.  The kernel itself is in mixed_kernel.h.
#include <algorithm>
#include <mutex>
#include <utility>
#include <vector>

#include "flexiq_test.h"
#include "mixed_kernel.h"

namespace flexiq {

// ---------------------------------------------------------------------------------------------
// Host side: tile-shape choice and launch
// ---------------------------------------------------------------------------------------------

static const TileShape *shapes(int *count)
{
    static const TileShape tab[kNumTileShapes] = {tile_shape_0(), tile_shape_1(), tile_shape_2(), tile_shape_3(),
                                                  tile_shape_4(), tile_shape_5(), tile_shape_6(), tile_shape_7(),
                                                  tile_shape_8(), tile_shape_9(), tile_shape_10(), tile_shape_11(),
                                                  tile_shape_12(), tile_shape_13(), tile_shape_14()};
    *count = kNumTileShapes;
    return tab;
}

// Test / tuning switches of include/flexiq_test.h: process-wide, not synchronised (set them while no call is in
// flight).  The product never changes them.
static int g_force_shape = -1;
static int g_force_packed = -1;
static int g_max_blocks = 0;
static int g_last_shape = -1, g_last_blocks = 0, g_last_resident = 0;

// Calls with at most this many output rows stream the 4-bit units as packed codes (half the weight bytes, expanded
// in registers); larger ones use the expanded copy.  Measured on MI355X the packed route never wins with this
// kernel: a call with few rows has too few blocks to be limited by memory bandwidth, and pays for the expansion
// in its (latency-bound) K loop.  It therefore stays off by default (-1) and is kept, parity-tested, behind
// flexiq_debug_force_packed4(1); few-row calls are served by the split-K kernel instead.
constexpr int64_t kPackedMaxRows = -1;

// Per-device launch table, filled once per device by prepare_kernels() (called when a layer is packed, so never
// inside a launch): compute units, and for every kernel of the shape table the blocks that fit on one CU.
struct DeviceKernels {
    bool ready = false;
    int num_cu = 0;
    int resident[kNumTileShapes][2][2] = {};
    int resident_xp[kNumTileShapes] = {};   // the variant that reads packed 4-bit activations
};
constexpr int kMaxDevices = 64;
static DeviceKernels g_dev[kMaxDevices];
static std::mutex g_dev_mu;

int prepare_kernels(int device)
{
    if (device < 0 || device >= kMaxDevices) return FLEXIQ_EINVAL;
    std::lock_guard<std::mutex> lk(g_dev_mu);
    DeviceKernels &d = g_dev[device];
    if (d.ready) return FLEXIQ_OK;
    hipDeviceProp_t prop;
    FLEXIQ_HIP(hipGetDeviceProperties(&prop, device));
    d.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    int cnt;
    const TileShape *tab = shapes(&cnt);
    for (int i = 0; i < cnt; ++i)
        for (int c = 0; c < 2; ++c)
            for (int k = 0; k < 2; ++k) {
                const void *fn = (const void *)tab[i].fn[c][k];
                int resident = 0;
                // (raises the dynamic-LDS limit of the kernel; both calls are host-side bookkeeping)
                FLEXIQ_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, tab[i].lds));
                FLEXIQ_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, fn, tab[i].threads, tab[i].lds));
                d.resident[i][c][k] = resident < 1 ? 1 : resident;
            }
    for (int i = 0; i < cnt; ++i) {
        const void *fn = (const void *)tab[i].fn_xp;
        int resident = 0;
        FLEXIQ_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, tab[i].lds));
        FLEXIQ_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, fn, tab[i].threads, tab[i].lds));
        d.resident_xp[i] = resident < 1 ? 1 : resident;
    }
    d.ready = true;
    return FLEXIQ_OK;
}

// Pick the tile shape with the smallest modelled time on the busiest CU: the tiles that CU has to compute, how
// many of them run side by side, and per tile the K-steps (slower when the CU is shared) plus the epilogue.
static int choose_shape(const DeviceKernels &dk, int64_t M, int N, int steps, bool conv, bool packed, double lowered_frac)
{
    int cnt;
    const TileShape *tab = shapes(&cnt);
    if (g_force_shape >= 0 && g_force_shape < cnt) return g_force_shape;
    const int ncu = dk.num_cu;
    // Layers with at most 64 output channels and many rows (ResNet-50 stage 1 at batch 128): every wider shape computes
    // padding columns, and the 128 x 64 shape at three blocks per CU measured 15-20 % faster than the model's pick
    // on all three such layer kinds (1x1 and 3x3, K = 64 ... 576).
    constexpr int kNarrowShape = 14;
    if (N <= 64 && !packed && M >= (int64_t)3 * tab[kNarrowShape].BM * ncu) return kNarrowShape;
    double best = 1e300;
    int bi = 0;
    for (int i = 0; i < cnt; ++i) {
        // (the 160 x 256 four-wave shape keeps part of its accumulators in scratch memory in the convolution form:
        // measured five times slower than its neighbours there, so it only serves linear layers)
        if (conv && i == 3) continue;
        const int occ = dk.resident[i][conv ? 1 : 0][packed ? 1 : 0];
        const double tiles = (double)((M + tab[i].BM - 1) / tab[i].BM) * (double)((N + tab[i].BN - 1) / tab[i].BN);
        const double tiles_cu = __builtin_ceil(tiles / ncu);
        const double conc = tiles_cu < occ ? tiles_cu : occ;
        const double seq = __builtin_ceil(tiles_cu / conc);
        const double step = (tab[i].step_alone + lowered_frac * tab[i].lower) * (1.0 + tab[i].share * (conc - 1.0));
        const double prologue = 7000.0;
        const bool walks = tab[i].multi;   // prologue paid once per block
        // A block that walks several tiles whose K-steps change between lowering and plain copies waits for the copies in
        // flight when it goes from plain steps to lowering steps (the tiles of a block take their phases in alternating
        // order, so that happens once per two tiles).  Priced per tile at what makes the choice match the fastest forced
        // shape on ViT-L fc1 at r = 0.25 ... 0.75 on two boxes (shapes with many short tiles per block lose more than
        // the wait alone: 160 x 256 reads 58.6 ... 64 us there, 320 x 256 58.5 on both).
        const double phase_stall = walks && seq > 1 && lowered_frac > 0.0 && lowered_frac < 1.0 ? 3000.0 : 0.0;
        const double tile_switch = 1200.0;   // next-tile mapping and window, scale fetch, clearing the accumulators
        const double cost = walks ? prologue + seq * (steps * step + tab[i].epilogue + phase_stall) + (seq - 1.0) * tile_switch
                                  : seq * (prologue + steps * step + tab[i].epilogue);
        if (cost < best) {
            best = cost;
            bi = i;
        }
    }
    return bi;
}

// The producer of a fused chain must write its columns in the order the consumer reads its channels.
static bool orders_match(const flexiq_layer *producer, const flexiq_layer *consumer)
{
    return producer->out_order_hash == consumer->perm_hash;
}

// flexiq_out.lower_for as the kernels take it (the same checks whichever kernel serves the call).
int lower_for_args(const flexiq_layer *L, const flexiq_out *out, LowerArgs *la)
{
    *la = LowerArgs();
    const flexiq_layer *nx = out->lower_for;
    if (!nx) return FLEXIQ_OK;
    if (out->scan_for) return FLEXIQ_EINVAL;   // lowering needs positions the scan has yet to find
    if (!out->q || nx->C != L->N || nx->device != L->device) return FLEXIQ_EINVAL;
    if (nx->G > kMaxGroups || !orders_match(L, nx)) return FLEXIQ_EINVAL;
    if (nx->max_4bit_ch == 0) return FLEXIQ_OK;   // the consumer reads every channel at 8 bits: nothing to lower
    la->ashift = nx->dynamic ? nx->d_ashift_dyn : nx->d_ashift;
    la->K4 = nx->max_4bit_ch;
    la->gs_log2 = nx->group_size == 64 ? 6 : 5;
    return FLEXIQ_OK;
}

static int launch(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, bool conv,
                  int H, int Wd, int Ho, int Wo, int stride, int pad, const uint8_t *X4 = nullptr)
{
    GemmParams p = {};   // every field starts as zero / null
    // packed 4-bit activations only matter while some K-step is all 4-bit and the kernel stages activations itself
    const bool xp = X4 != nullptr && !conv && !L->x_prelowered && L->max_4bit_ch >= 64;
    p.X4 = xp ? X4 : nullptr;
    p.X = X; p.W8 = L->d_w8; p.W4 = L->d_w4; p.wshift = L->d_wshift;
    p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift;
    p.cs = L->d_cs; p.bias = L->d_bias;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.K4 = L->max_4bit_ch;
    p.x_pre = L->x_prelowered ? 1 : 0;
    p.next_ashift = nullptr; p.next_K4 = 0; p.next_G = 0; p.next_gs_log2 = 5;
    p.next_scan = nullptr; p.next_static = nullptr; p.next_dyn = nullptr; p.next_g4 = 0;
    if (out->x6) return FLEXIQ_EINVAL;   // FP6 output is written by the FP6-variant kernel only
    if (out->lower_for && out->scan_for) return FLEXIQ_EINVAL;   // lowering needs positions the scan has yet to find
    if (out->lower_for) {
        const flexiq_layer *nx = out->lower_for;
        if (!out->q || nx->C != L->N || nx->device != L->device) return FLEXIQ_EINVAL;
        if (nx->G > kMaxGroups || !orders_match(L, nx)) return FLEXIQ_EINVAL;   // consumer's table lives in LDS; column order
        // (a consumer that reads every channel at 8 bits has nothing lowered: the plain epilogue serves the call)
        if (nx->max_4bit_ch > 0 || out->x4) p.next_ashift = nx->dynamic ? nx->d_ashift_dyn : nx->d_ashift;
        p.next_K4 = nx->max_4bit_ch;
        p.next_G = nx->G;
        p.next_gs_log2 = nx->group_size == 64 ? 6 : 5;
        if (out->x4) {   // the consumer's leading channels leave as packed 4-bit codes
            if (nx->R != 1 || nx->S != 1 || (L->N & 31) || (reinterpret_cast<uintptr_t>(out->x4) & 15u)) return FLEXIQ_EINVAL;
            if (M * (int64_t)(L->N / 2) > 0x7fffffff) return FLEXIQ_EINVAL;
            p.next_x4 = out->x4;
            p.next_K4P = nx->x_prelowered ? 0 : (nx->max_4bit_ch / 64) * 64;
        }
    } else if (out->x4) {
        return FLEXIQ_EINVAL;   // packed output needs the consumer's positions
    }
    if (out->scan_for) {
        flexiq_layer *nx = out->scan_for;
        if (!out->q || nx->C != L->N || nx->device != L->device || nx == L) return FLEXIQ_EINVAL;
        if (nx->G > kMaxGroups || !orders_match(L, nx)) return FLEXIQ_EINVAL;   // the block's mask table holds 160 groups
        p.next_scan = nx->d_scan;
        p.next_static = nx->d_ashift;
        p.next_dyn = nx->d_ashift_dyn;
        p.next_g4 = nx->max_4bit_ch / nx->group_size;
        p.next_G = nx->G;
        p.next_gs_log2 = nx->group_size == 64 ? 6 : 5;
    }
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.U = L->U; p.CU = L->C / kUnit; p.T = L->T; p.G = L->G;
    {   // the handle's buffers live on the device it was packed on
        int dev = -1;
        FLEXIQ_HIP(hipGetDevice(&dev));
        if (dev != L->device || dev < 0 || dev >= kMaxDevices) return FLEXIQ_EINVAL;
    }
    const DeviceKernels &dk = g_dev[L->device];
    if (!dk.ready) return FLEXIQ_EINVAL;   // (set up when the handle was packed)
    if (L->G > kMaxGroups) return FLEXIQ_EINVAL;  // position table kept in LDS
    if (M > 0x7fffffff - 512) return FLEXIQ_EINVAL;  // row indices are 32-bit in the kernel
    if (L->C / kUnit >= 2 * 65535) return FLEXIQ_EINVAL;  // K-step indices are kept in 16-bit fields
    if ((int64_t)L->U * 32 * L->Npad * 2 > kMaxWeightBytes) return FLEXIQ_EINVAL;  // both int8 weight copies must fit one buffer descriptor
    p.H = H; p.Wd = Wd; p.Ho = Ho; p.Wo = Wo; p.S = L->S; p.stride = stride; p.pad = pad;
    // Layers with a short reduction and many contiguous rows: the row-streaming kernel (weights resident in LDS, whole
    // row tiles copied several tiles ahead).
    {
        int taken = 0;
        const bool ok = (!conv || (stride == 1 && pad == 0)) && g_force_shape < 0 && g_force_packed < 0 && g_max_blocks == 0;
        LowerArgs la;
        la.ashift = p.next_ashift; la.K4 = p.next_K4; la.gs_log2 = p.next_gs_log2;   // (checked above)
        const int rc = launch_stream(L, X, M, out, stream, ok, &taken, xp ? X4 : nullptr, &la);
        if (rc != FLEXIQ_OK) return rc;
        if (taken) {
            g_last_shape = -2;
            g_last_blocks = 0;
            g_last_resident = 0;
            return FLEXIQ_OK;
        }
    }
    // More rows, few output tiles, a long reduction: a tile per block whose waves split the reduction (smallm.hip).
    if (!conv && !xp && M > 16 && g_force_shape < 0 && g_force_packed < 0 && g_max_blocks == 0) {
        int taken = 0;
        LowerArgs la;
        la.ashift = p.next_ashift; la.K4 = p.next_K4; la.gs_log2 = p.next_gs_log2;   // (checked above)
        const int rc = launch_tile_splitk(L, X, M, out, stream, dk.num_cu, &taken, &la);
        if (rc != FLEXIQ_OK) return rc;
        if (taken) {
            g_last_shape = -5;
            g_last_blocks = (int)(((M + (taken == 1 ? 63 : 31)) / (taken == 1 ? 64 : 32)) * ((L->N + (taken == 3 ? 31 : 63)) / (taken == 3 ? 32 : 64)));
            g_last_resident = 0;
            return FLEXIQ_OK;
        }
    }
    // Few-row linear calls: a block per 16 output columns, the reduction split over its waves (smallm.hip).  Measured against
    // the tiled kernel, which launches 16-64 blocks of 64 x 64 here: faster for every call of at most 16 rows, and up to 64
    // rows as long as there is at most one block per compute unit or so (every block reads all activation rows).
    if (!conv && M <= 64 && g_force_shape < 0 && g_force_packed < 0 && g_max_blocks == 0) {
        int taken = 0;
        LowerArgs la;
        la.ashift = p.next_ashift; la.K4 = p.next_K4; la.gs_log2 = p.next_gs_log2;   // (checked above)
        const int rc = launch_few_rows(L, X, M, out, stream, dk.num_cu, &taken, xp ? X4 : nullptr, &la);
        if (rc != FLEXIQ_OK) return rc;
        if (taken) {
            g_last_shape = -4;
            g_last_blocks = taken == 2 ? (L->N + 7) / 8 : (L->N + 15) / 16;
            g_last_resident = 0;
            return FLEXIQ_OK;
        }
    }
    const int steps = L->T * ((p.CU + 1) / 2);
    // (activations that arrive lowered always pair with the expanded weight copy)
    const bool packed = !xp && !L->x_prelowered && (g_force_packed >= 0 ? g_force_packed != 0 : M <= kPackedMaxRows);
    int cnt;
    // share of the K-steps whose activations the kernel lowers (none when they arrive lowered)
    const double lowered_frac = L->x_prelowered ? 0.0 : (double)L->max_4bit_ch / (double)L->C;
    g_last_shape = choose_shape(dk, M, L->N, steps, conv, packed, lowered_frac);
    const TileShape &ts = shapes(&cnt)[g_last_shape];
    p.tiles_m = (int)((M + ts.BM - 1) / ts.BM);
    p.tiles_n = (L->N + ts.BN - 1) / ts.BN;
    {   // constants of the kernel's tile-index divisions
        const uint32_t d1 = 8u * (uint32_t)p.tiles_n, d2 = (uint32_t)(p.tiles_m % 8);
        p.band_div = d1;
        p.band_mag = (uint32_t)((1ull << 32) / d1);
        p.tail_div = d2 ? d2 : 1u;
        p.tail_mag = d2 > 1 ? (uint32_t)((1ull << 32) / d2) : 0xffffffffu;
    }
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    if (tiles > 0x7fffffff) return FLEXIQ_EINVAL;
    kernel_fn fn = xp ? ts.fn_xp : ts.fn[conv ? 1 : 0][packed ? 1 : 0];
    const int resident = xp ? dk.resident_xp[g_last_shape] : dk.resident[g_last_shape][conv ? 1 : 0][packed ? 1 : 0];   // blocks of this kernel that fit on one CU
    // Shapes whose blocks can walk several output tiles are launched as one resident wave of blocks (the kernel's
    // load pipeline then runs on across tile boundaries); the others with one block per tile.
    int64_t blocks = tiles;
    if (ts.multi && g_max_blocks >= 0)
        blocks = std::min<int64_t>(tiles, g_max_blocks > 0 ? (int64_t)g_max_blocks : (int64_t)dk.num_cu * resident);
    g_last_blocks = (int)blocks;
    g_last_resident = resident;
    hipLaunchKernelGGL(fn, dim3((unsigned)blocks), dim3(ts.threads), ts.lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    if (out->scan_for) out->scan_for->dynamic = true;   // its next calls read the positions this launch leaves
    return FLEXIQ_OK;
}

static int check_out(const flexiq_out *out)
{
    if (!out || (!out->acc && !out->y && !out->q)) return FLEXIQ_EINVAL;
    if (out->q && !(out->out_scale > 0.0f)) return FLEXIQ_EINVAL;
    const void *ps[] = {out->acc, out->y, out->q};
    for (const void *q : ps)
        if (q && (reinterpret_cast<uintptr_t>(q) & 15u)) return FLEXIQ_EALIGN;
    return FLEXIQ_OK;
}

}  // namespace flexiq

using namespace flexiq;

// Test / tuning hooks (include/flexiq_test.h).
extern "C" int flexiq_debug_force_tile(int index)
{
    int cnt;
    (void)shapes(&cnt);
    if (index < -1 || index >= cnt) return FLEXIQ_EINVAL;
    g_force_shape = index;
    return cnt;
}

// Test / tuning hook: what the last launch used.  which = 0: tile shape index, 1: blocks launched,
// 2: blocks of that kernel resident per CU.
extern "C" int flexiq_debug_last_launch(int which)
{
    return which == 0 ? g_last_shape : (which == 1 ? g_last_blocks : g_last_resident);
}

// Test / tuning hook for the number of blocks of a linear call: 0 = automatic (one resident wave of blocks,
// each walking several output tiles), n > 0 = at most n blocks, n < 0 = one block per output tile.
extern "C" int flexiq_debug_max_blocks(int n)
{
    g_max_blocks = n;
    return FLEXIQ_OK;
}

// Test / tuning hook: 1 = 4-bit units always from the packed codes, 0 = always from the expanded copy,
// -1 = automatic (by the number of output rows).
extern "C" int flexiq_debug_force_packed4(int mode)
{
    if (mode < -1 || mode > 1) return FLEXIQ_EINVAL;
    g_force_packed = mode;
    return FLEXIQ_OK;
}

extern "C" int flexiq_mixed_gemm(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream)
{
    if (!L || M < 0 || L->R != 1 || L->S != 1) return FLEXIQ_EINVAL;
    if (M == 0) return FLEXIQ_OK;  // empty input: nothing to write, output pointers are not looked at
    int rc = check_out(out);
    if (rc) return rc;
    if (!X) return FLEXIQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(X) & 15u) return FLEXIQ_EALIGN;
    return launch(L, X, M, out, stream, false, 1, 1, 1, 1, 1, 0);
}

extern "C" int flexiq_packed4_channels(const flexiq_layer *L, int32_t *k4p)
{
    if (!L || !k4p) return FLEXIQ_EINVAL;
    *k4p = L->R == 1 && L->S == 1 && !L->x_prelowered ? (L->max_4bit_ch / 64) * 64 : 0;
    return FLEXIQ_OK;
}

extern "C" int64_t flexiq_packed4_bytes(const flexiq_layer *L, int64_t M)
{
    if (!L || M < 0 || L->R != 1 || L->S != 1) return FLEXIQ_EINVAL;
    return M * (int64_t)(L->C / 2);
}

extern "C" int flexiq_mixed_gemm_packed4(const flexiq_layer *L, const int8_t *X, const uint8_t *X4, int64_t M, const flexiq_out *out,
                                         void *stream)
{
    if (!L || M < 0 || L->R != 1 || L->S != 1) return FLEXIQ_EINVAL;
    if (M == 0) return FLEXIQ_OK;
    int rc = check_out(out);
    if (rc) return rc;
    if (!X || !X4) return FLEXIQ_EINVAL;
    if ((reinterpret_cast<uintptr_t>(X) & 15u) || (reinterpret_cast<uintptr_t>(X4) & 15u)) return FLEXIQ_EALIGN;
    if (M * (int64_t)(L->C / 2) > 0x7fffffff) return FLEXIQ_EINVAL;   // a tile's window of X4 is addressed with 32 bits
    return launch(L, X, M, out, stream, false, 1, 1, 1, 1, 1, 0, X4);
}

extern "C" int flexiq_mixed_conv_implicit(const flexiq_layer *L, const int8_t *X, int32_t B, int32_t H, int32_t W,
                                          int32_t stride, int32_t pad, const flexiq_out *out, void *stream)
{
    if (!L || B < 0 || H <= 0 || W <= 0 || stride <= 0 || pad < 0) return FLEXIQ_EINVAL;
    if (H + 2 * pad < L->R || W + 2 * pad < L->S) return FLEXIQ_EINVAL;
    const int Ho = (H + 2 * pad - L->R) / stride + 1, Wo = (W + 2 * pad - L->S) / stride + 1;
    const int64_t M = (int64_t)B * Ho * Wo;
    if (M == 0) return FLEXIQ_OK;  // empty batch
    // A block addresses its input through a 2 GiB window that starts at the first image it touches; the images
    // of the tallest tile (320 output rows) must fit in it.
    if ((int64_t)H * W * L->C * (320 / ((int64_t)Ho * Wo) + 2) > 0x7fffffff) return FLEXIQ_EINVAL;
    int rc = check_out(out);
    if (rc) return rc;
    if (!X) return FLEXIQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(X) & 15u) return FLEXIQ_EALIGN;
    {   // 3x3, stride 1, padding 1, 64 or 128 channels: the kernel that keeps all taps' weights resident (conv3.hip)
        int taken = 0;
        if (g_force_shape < 0 && g_force_packed < 0 && g_max_blocks == 0) {
            LowerArgs la;
            rc = lower_for_args(L, out, &la);
            if (rc != FLEXIQ_OK) return rc;
            {   // (as in launch(): the handle's buffers live on the device it was packed on)
                int dev = -1;
                FLEXIQ_HIP(hipGetDevice(&dev));
                if (dev != L->device) return FLEXIQ_EINVAL;
            }
            rc = launch_conv3(L, X, B, H, W, stride, pad, out, stream, &taken, &la);
            if (rc != FLEXIQ_OK) return rc;
        }
        if (taken) {
            g_last_shape = -3;
            g_last_blocks = 0;
            g_last_resident = 0;
            return FLEXIQ_OK;
        }
    }
    // a 1x1 convolution with stride 1 and no padding is the linear form over the pixels: no per-tap address arithmetic
    if (L->R == 1 && L->S == 1 && stride == 1 && pad == 0) return launch(L, X, M, out, stream, false, 1, 1, 1, 1, 1, 0);
    return launch(L, X, M, out, stream, true, H, W, Ho, Wo, stride, pad);
}
