// Host side of the FP6 variant of the mixed GEMM (kernel in fp6_kernel.h): which leading channels run as FP6,
// tile-shape choice, launch, and the C entry points.
#include <algorithm>
#include <mutex>

#include "flexiq_test.h"
#include "fp6_kernel.h"

namespace flexiq {
namespace fp6 {

constexpr int kNumShapes = 4;
static const Shape *shapes()
{
    // (a 320 x 256 tile does not fit the register file next to the FP6 fragments)
    static const Shape tab[kNumShapes] = {make_shape<2, 4, 4, 2>(),    // 256 x 256
                                          make_shape<2, 4, 3, 2>(),    // 192 x 256
                                          make_shape<2, 4, 2, 2>(),    // 128 x 256
                                          make_shape<2, 4, 1, 2>()};   //  64 x 256
    return tab;
}

struct DeviceState {
    bool ready = false;
    int num_cu = 0;
};
static DeviceState g_dev[64];
static std::mutex g_mu;
static int g_force_shape = -1;
static int g_last_shape = -1;

}  // namespace fp6

int prepare_fp6_kernels(int device)
{
    using namespace fp6;
    if (device < 0 || device >= 64) return FLEXIQ_EINVAL;
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceState &d = g_dev[device];
    if (d.ready) return FLEXIQ_OK;
    hipDeviceProp_t prop;
    FLEXIQ_HIP(hipGetDeviceProperties(&prop, device));
    d.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const Shape *tab = shapes();
    for (int i = 0; i < kNumShapes; ++i)
        FLEXIQ_HIP(hipFuncSetAttribute((const void *)tab[i].fn, hipFuncAttributeMaxDynamicSharedMemorySize, tab[i].lds));
    d.ready = true;
    return FLEXIQ_OK;
}

// Leading channels that run as FP6: the 4-bit channels under the current ratio, cut to whole K-steps of 64 and to the
// prefix whose fp32 accumulation is certified exact for the positions in use.
int fp6_channels(const flexiq_layer *L)
{
    if (!L->d_w6) return 0;
    const int limit = L->dynamic ? L->fp6_limit_dynamic : L->fp6_limit_static;
    return (std::min(L->max_4bit_ch, limit) / 64) * 64;
}

}  // namespace flexiq

using namespace flexiq;

extern "C" int flexiq_fp6_channels(const flexiq_layer *L, int32_t *k6)
{
    if (!L || !k6) return FLEXIQ_EINVAL;
    *k6 = fp6_channels(L);
    return FLEXIQ_OK;
}

extern "C" int64_t flexiq_fp6_bytes(const flexiq_layer *L, int64_t M)
{
    if (!L || M < 0 || !L->d_w6) return FLEXIQ_EINVAL;
    return ((M + 63) / 64) * (int64_t)(L->C / 64) * 3072;
}

extern "C" int flexiq_debug_force_fp6_tile(int index)
{
    if (index < -1 || index >= fp6::kNumShapes) return FLEXIQ_EINVAL;
    fp6::g_force_shape = index;
    return fp6::kNumShapes;
}

extern "C" int flexiq_mixed_gemm_fp6(const flexiq_layer *L, const int8_t *X, const uint8_t *X6, int64_t M, const flexiq_out *out,
                                     void *stream)
{
    using namespace fp6;
    if (!L || M < 0 || L->R != 1 || L->S != 1 || !L->d_w6) return FLEXIQ_EINVAL;   // linear layers with C a multiple of 64
    if (M == 0) return FLEXIQ_OK;
    if (!out || (!out->acc && !out->y && !out->q)) return FLEXIQ_EINVAL;
    if (out->q && !(out->out_scale > 0.0f)) return FLEXIQ_EINVAL;
    if (out->scan_for) return FLEXIQ_EINVAL;   // the run-time scan rides in the int8 kernel's epilogue only
    if (out->x4) return FLEXIQ_EINVAL;         // packed 4-bit output is written by the int8 kernel only
    const int K6 = fp6_channels(L);
    if ((K6 > 0 && !X6) || (K6 < L->C && !X)) return FLEXIQ_EINVAL;
    const void *ps[] = {out->acc, out->y, out->q, X, X6, out->x6};
    for (const void *q : ps)
        if (q && (reinterpret_cast<uintptr_t>(q) & 15u)) return FLEXIQ_EALIGN;
    int dev = -1;
    FLEXIQ_HIP(hipGetDevice(&dev));
    if (dev != L->device || dev < 0 || dev >= 64 || !g_dev[dev].ready) return FLEXIQ_EINVAL;
    if (M > 0x7fffffff - 512) return FLEXIQ_EINVAL;
    const int64_t x6_bytes = ((M + 63) / 64) * (int64_t)(L->C / 64) * 3072;
    if (x6_bytes > 0x7fffffff || (int64_t)L->U * 32 * L->Npad * 2 > kMaxWeightBytes) return FLEXIQ_EINVAL;

    // No 4-bit channel at the current ratio: nothing runs as FP6 and nothing arrives lowered, so the call is an ordinary int8
    // call, and the int8 kernels (more tile shapes, blocks that walk tiles) serve it faster than this kernel's int8 phase
    // (ViT-L fc2 at r = 0: 41 against 50 us).  Not when the caller wants FP6 output for a consumer, which only this kernel writes.
    if (L->max_4bit_ch == 0 && !out->x6 && g_force_shape < 0) return flexiq_mixed_gemm(L, X, M, out, stream);
    Params p = {};
    p.X = X; p.X6 = X6; p.W8 = L->d_w8; p.W6 = L->d_w6; p.W6S = L->d_w6s;
    p.ashift = L->dynamic ? L->d_ashift_dyn : L->d_ashift;
    p.cs = L->d_cs;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.K4 = L->max_4bit_ch; p.K6 = K6;
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.U = L->U;
    p.x6_bytes = x6_bytes;
    p.next_gs_log2 = 5;
    if (out->lower_for) {
        const flexiq_layer *nx = out->lower_for;
        if (!out->q || nx->C != L->N || nx->device != L->device || nx->G > kMaxGroups) return FLEXIQ_EINVAL;
        if (L->out_order_hash != nx->perm_hash) return FLEXIQ_EINVAL;
        p.next_ashift = nx->dynamic ? nx->d_ashift_dyn : nx->d_ashift;
        p.next_K4 = nx->max_4bit_ch;
        p.next_gs_log2 = nx->group_size == 64 ? 6 : 5;
        if (out->x6) {   // the consumer's leading channels leave as FP6 codes
            if (!nx->d_w6 || (L->N & 63)) return FLEXIQ_EINVAL;
            p.nx6 = out->x6;
            p.next_K6 = fp6_channels(nx);
            p.next_S = nx->C / 64;
        }
    } else if (out->x6) {
        return FLEXIQ_EINVAL;   // FP6 output needs the consumer's positions
    }

    if ((M > 16 || out->lower_for) && g_force_shape < 0) {   // few output tiles, a long reduction: a tile per block whose waves split the reduction (smallm.hip)
        int taken = 0;
        LowerArgs la;
        la.ashift = p.next_ashift; la.K4 = p.next_K4; la.gs_log2 = p.next_gs_log2;   // (checked above; null: the call names no consumer)
        la.x6 = p.nx6; la.K6 = p.next_K6; la.S = p.next_S;
        const int rc = launch_tile_splitk_fp6(L, X, X6, M, out, stream, K6, g_dev[dev].num_cu, &taken, &la);
        if (rc != FLEXIQ_OK) return rc;
        if (taken) {
            g_last_shape = -5;
            return FLEXIQ_OK;
        }
    }
    if (M <= 64 && g_force_shape < 0) {   // few rows: a block per 16 columns whose waves split the reduction (smallm.hip)
        int taken = 0;
        const int rc = launch_few_rows_fp6(L, X, X6, M, out, stream, K6, g_dev[dev].num_cu, &taken);
        if (rc != FLEXIQ_OK) return rc;
        if (taken) {
            g_last_shape = -4;
            return FLEXIQ_OK;
        }
    }

    const DeviceState &ds = g_dev[dev];
    const Shape *tab = shapes();
    int best = 0;
    if (g_force_shape >= 0) {
        best = g_force_shape;
    } else {
        double best_cost = 1e300;
        const int S = L->C / 64, S6 = K6 / 64;
        for (int i = 0; i < kNumShapes; ++i) {
            const double tiles = (double)((M + tab[i].BM - 1) / tab[i].BM) * (double)((L->N + tab[i].BN - 1) / tab[i].BN);
            const double rounds = __builtin_ceil(tiles / ds.num_cu);
            const double mf = tab[i].BM / 64.0;   // MFMAs per wave and k-half (two waves per SIMD): 2 x BM / 64 ... relative
            const double step8 = 140.0 + 128.0 * mf, step6 = 140.0 + 64.0 * mf;
            const double cost = rounds * (3500.0 + S6 * step6 + (S - S6) * step8 + 1400.0 * mf);
            if (cost < best_cost) {
                best_cost = cost;
                best = i;
            }
        }
    }
    g_last_shape = best;
    const Shape &sh = tab[best];
    p.tiles_m = (int)((M + sh.BM - 1) / sh.BM);
    p.tiles_n = (L->N + sh.BN - 1) / sh.BN;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    if (tiles > 0x7fffffff) return FLEXIQ_EINVAL;
    hipLaunchKernelGGL(sh.fn, dim3((unsigned)tiles), dim3(sh.threads), sh.lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}
