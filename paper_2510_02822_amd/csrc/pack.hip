// Offline steps of the method as HIP kernels: per-output-channel weight quantisation (Eq. 1),
// channel scores and order (Section 4.2), extraction positions (Section 4.1), layout in stored
// order with same-bitwidth channels contiguous (Section 5), and the packed 8-bit / 4-bit weight
// tiles the GEMM kernels stream.  Also the layer handle, the ratio switch (Section 7) and the
// small element-wise run-time kernels (activation quantiser, stand-alone bit-lowering, channel
// reorder operator).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <string>

#include "flexiq_internal.h"

namespace flexiq {

static std::mutex g_err_mu;
static std::string g_err = "";

void set_hip_error(hipError_t e, const char *what)
{
    std::lock_guard<std::mutex> lk(g_err_mu);
    g_err = std::string(hipGetErrorName(e)) + ": " + hipGetErrorString(e) + " in " + what;
    (void)hipGetLastError();  // clear the sticky "last error"
}

// ---------------------------------------------------------------------------------------------
// Weight quantisation, Eq. 1 with one scale per output channel
// ---------------------------------------------------------------------------------------------

// One block per output channel n: scale[n] = max|W[n][:]| / 127 (1 if the row is all zero).
__global__ void k_row_scale(const float *__restrict__ W, int64_t Kt, float *__restrict__ scale)
{
    __shared__ float red[256];
    const float *row = W + (int64_t)blockIdx.x * Kt;
    float m = 0.0f;
    for (int64_t i = threadIdx.x; i < Kt; i += blockDim.x) m = fmaxf(m, fabsf(row[i]));
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) scale[blockIdx.x] = red[0] == 0.0f ? 1.0f : __fdiv_rn(red[0], 127.0f);
}

__device__ __forceinline__ int quant_code(float x, float S, float lo, float hi)
{
    float t = rintf(__fdiv_rn(x, S));  // round to nearest, ties to even
    t = fminf(fmaxf(t, lo), hi);
    return (int)t;
}

// q[n][i] = clip(round(W[n][i] / scale[n]), -127, 127), natural channel order.
__global__ void k_quantize_rows(const float *__restrict__ W, const float *__restrict__ scale, int64_t Kt,
                                int64_t total, int8_t *__restrict__ q)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    q[i] = (int8_t)quant_code(W[i], scale[i / Kt], -127.0f, 127.0f);
}

// wmax[c] = max over output channels and taps of |Wq[n][t][c]|  (the weight range of Section 4.2).
__global__ void k_chan_wmax(const int8_t *__restrict__ q, int N, int T, int C, int *__restrict__ wmax)
{
    int n = blockIdx.x;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        int m = 0;
        for (int t = 0; t < T; ++t) {
            int w = q[((int64_t)n * T + t) * C + c];
            m = max(m, w < 0 ? -w : w);
        }
        atomicMax(&wmax[c], m);
    }
}

// Extraction position of the weights of (output channel n, group g): OR the magnitude bits of the
// group's values over all taps (ones' complement for negatives), take the highest set bit p, keep
// the three bits below it: s = max(0, p - 2)  (Section 4.1).
__global__ void k_weight_shift(const int8_t *__restrict__ q, const int32_t *__restrict__ perm, int N, int T, int C,
                               int gs, int Npad, uint8_t *__restrict__ ws_ng, uint8_t *__restrict__ ws_gn)
{
    int G = C / gs;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)N * G) return;
    int n = (int)(i / G), g = (int)(i % G);
    unsigned m = 0;
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < gs; ++j) {
            int w = q[((int64_t)n * T + t) * C + perm[g * gs + j]];
            m |= (unsigned)(w >= 0 ? w : ~w) & 0x7Fu;
        }
    int p = m ? 31 - __clz(m) : -1;
    int s = max(0, p - 2);
    ws_ng[(int64_t)n * G + g] = (uint8_t)s;
    ws_gn[(int64_t)g * Npad + n] = (uint8_t)s;
}

// One thread per (unit u, padded output channel n): gathers the 32 stored channels of the unit and
// writes the two 16-byte planes of the 8-bit tile and the 16 bytes of 4-bit codes.
__global__ void k_pack_tiles(const int8_t *__restrict__ q, const int32_t *__restrict__ perm,
                             const uint8_t *__restrict__ ws_ng, int N, int T, int C, int gs, int Npad, int U,
                             int8_t *__restrict__ w8, uint8_t *__restrict__ w4, int8_t *__restrict__ w4x)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)U * Npad) return;
    int u = (int)(i / Npad), n = (int)(i % Npad);
    int CU = C / kUnit, CUp = (CU + 1) & ~1;  // every tap is padded to an even number of units
    int tap = u / CUp, c32 = u % CUp;
    int v[32];
    int s = 0;
    if (n < N && c32 < CU) {
        for (int j = 0; j < 32; ++j) v[j] = q[((int64_t)n * T + tap) * C + perm[c32 * 32 + j]];
        s = ws_ng[(int64_t)n * (C / gs) + (c32 * 32) / gs];
    } else {
        for (int j = 0; j < 32; ++j) v[j] = 0;
    }
    uint32_t d8[8], dx[8], d4[4];
    for (int d = 0; d < 8; ++d) {
        d8[d] = (uint32_t)(v[4 * d] & 0xFF) | ((uint32_t)(v[4 * d + 1] & 0xFF) << 8) |
                ((uint32_t)(v[4 * d + 2] & 0xFF) << 16) | ((uint32_t)(v[4 * d + 3] & 0xFF) << 24);
        uint32_t w = 0;
        for (int b = 0; b < 4; ++b) w |= (uint32_t)((min(7, max(-8, v[4 * d + b] >> s)) * (1 << s)) & 0xFF) << (8 * b);
        dx[d] = w;
    }
    for (int e = 0; e < 4; ++e) {
        uint32_t w = 0;
        for (int b = 0; b < 4; ++b) {
            int lo = min(7, max(-8, v[8 * e + b] >> s)) & 0xF;
            int hi = min(7, max(-8, v[8 * e + 4 + b] >> s)) & 0xF;
            w |= (uint32_t)(lo | (hi << 4)) << (8 * b);
        }
        d4[e] = w;
    }
    uint4 *p8 = reinterpret_cast<uint4 *>(w8);
    p8[((int64_t)u * 2 + 0) * Npad + n] = make_uint4(d8[0], d8[1], d8[2], d8[3]);
    p8[((int64_t)u * 2 + 1) * Npad + n] = make_uint4(d8[4], d8[5], d8[6], d8[7]);
    reinterpret_cast<uint4 *>(w4)[(int64_t)u * Npad + n] = make_uint4(d4[0], d4[1], d4[2], d4[3]);
    uint4 *px = reinterpret_cast<uint4 *>(w4x);
    px[((int64_t)u * 2 + 0) * Npad + n] = make_uint4(dx[0], dx[1], dx[2], dx[3]);
    px[((int64_t)u * 2 + 1) * Npad + n] = make_uint4(dx[4], dx[5], dx[6], dx[7]);
}

// FP6 image of the 4-bit codes (linear layers): one thread per (K-step t of 64 channels, padded output channel n)
// writes the three 16-byte planes and the two block-scale bytes; also sabs[n][g32] = sum over the unit's channels of
// |code << w_shift|, from which the host certifies exact fp32 accumulation.
__device__ __forceinline__ uint32_t fp6_pattern(int code) { return (uint32_t)((code < 0 ? 32 : 0) | (code < 0 ? -code : code)); }
__device__ __forceinline__ int fp6_channel_of_element(int e) { return 8 * ((e % 16) / 4) + 4 * (e / 16) + e % 4; }

__global__ void k_pack_w6(const int8_t *__restrict__ q, const int32_t *__restrict__ perm, const uint8_t *__restrict__ ws_ng,
                          int N, int C, int gs, int Npad, uint8_t *__restrict__ w6, uint8_t *__restrict__ w6s,
                          int32_t *__restrict__ sabs)
{
    const int S = C / 64;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)S * Npad) return;
    const int t = (int)(i / Npad), n = (int)(i % Npad);
    uint32_t tail[4] = {0, 0, 0, 0};
    for (int h = 0; h < 2; ++h) {
        const int u = 2 * t + h;
        uint32_t d[6] = {0, 0, 0, 0, 0, 0};
        int s = 0, sum = 0;
        if (n < N) {
            s = ws_ng[(int64_t)n * (C / gs) + (u * 32) / gs];
            for (int e = 0; e < 32; ++e) {
                const int v = q[(int64_t)n * C + perm[u * 32 + fp6_channel_of_element(e)]];
                const int code = min(7, max(-8, v >> s));
                sum += (code < 0 ? -code : code) << s;
                const uint32_t pat = fp6_pattern(code);
                const int bit = 6 * e;
                d[bit / 32] |= pat << (bit % 32);
                if (bit % 32 > 26) d[bit / 32 + 1] |= pat >> (32 - bit % 32);
            }
            sabs[(int64_t)n * (C / 32) + u] = sum;
        }
        reinterpret_cast<uint4 *>(w6)[((int64_t)t * 3 + h) * Npad + n] = make_uint4(d[0], d[1], d[2], d[3]);
        const int half = h ^ ((n >> 4) & 1);
        tail[2 * half] = d[4];
        tail[2 * half + 1] = d[5];
        w6s[((((int64_t)(t >> 2) * Npad + n) * 2 + h) << 2) + (t & 3)] = (uint8_t)(127 + 3 + s);
    }
    reinterpret_cast<uint4 *>(w6)[((int64_t)t * 3 + 2) * Npad + n] = make_uint4(tail[0], tail[1], tail[2], tail[3]);
}

// ---------------------------------------------------------------------------------------------
// Run-time element-wise kernels
// ---------------------------------------------------------------------------------------------

// Activations for the FP6 variant (Section 4.1 bit-lowering, then the 6-bit pattern of code / 8): one thread per
// (row, unit of 32 channels) of the leading k6 channels.  Layout of x6: [row / 64][K-step][plane][row % 64][16].
__global__ void k_lower_fp6(const int8_t *__restrict__ X, int64_t rows, int C, int k6, int gs_shift,
                            const int32_t *__restrict__ ashift, uint8_t *__restrict__ x6)
{
    const int units = k6 / 32, S = C / 64;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * units) return;
    const int64_t m = i / units;
    const int u = (int)(i % units), t = u >> 1, h = u & 1;
    const int s = ashift[u >> gs_shift];
    const uint4 lo = *reinterpret_cast<const uint4 *>(X + m * C + u * 32), hi = *reinterpret_cast<const uint4 *>(X + m * C + u * 32 + 16);
    const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    uint32_t d[6] = {0, 0, 0, 0, 0, 0};
    for (int e = 0; e < 32; ++e) {
        const int c = fp6_channel_of_element(e);
        const int v = (int)(int8_t)((w[c >> 2] >> (8 * (c & 3))) & 0xFF);
        const uint32_t pat = fp6_pattern(min(7, max(-8, v >> s)));
        const int bit = 6 * e;
        d[bit / 32] |= pat << (bit % 32);
        if (bit % 32 > 26) d[bit / 32 + 1] |= pat >> (32 - bit % 32);
    }
    const int rr = (int)(m & 63);
    uint8_t *blk = x6 + ((m >> 6) * (int64_t)S + t) * 3072;
    *reinterpret_cast<uint4 *>(blk + h * 1024 + rr * 16) = make_uint4(d[0], d[1], d[2], d[3]);
    *reinterpret_cast<uint2 *>(blk + 2048 + rr * 16 + 8 * (h ^ ((rr >> 4) & 1))) = make_uint2(d[4], d[5]);
}

// Copy of X in which the channels [c_lo, c_hi) are bit-lowered at their position (L(v, s) << s) and all others are
// unchanged: 16 channels per thread.
__global__ void k_lower_int8_range(const int8_t *__restrict__ X, int8_t *__restrict__ Y, int64_t rows, int C, int c_lo,
                                   int c_hi, int gs_shift, const int32_t *__restrict__ ashift)
{
    const int P = C / 16;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * P) return;
    const int c0 = (int)(i % P) * 16;
    uint4 v = *reinterpret_cast<const uint4 *>(X + i * 16);
    if (c0 >= c_lo && c0 < c_hi) {
        const int s = ashift[(c0 >> 5) >> gs_shift];
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
        for (int k = 0; k < 4; ++k) {
            uint32_t o = 0;
            for (int b = 0; b < 4; ++b) {
                const int x = (int)(int8_t)((w[k] >> (8 * b)) & 0xFF);
                o |= (uint32_t)((min(7, max(-8, x >> s)) * (1 << s)) & 0xFF) << (8 * b);
            }
            w[k] = o;
        }
        v = make_uint4(w[0], w[1], w[2], w[3]);
    }
    *reinterpret_cast<uint4 *>(Y + i * 16) = v;
}

// Packed 4-bit activations (Section 4.1 bit-lowering, two codes per byte): one thread per (row, 16-channel piece) of the
// leading k4p channels writes the piece's eight bytes: dword e holds the codes of channels 8e .. 8e+3 in the low halves of
// its bytes and those of channels 8e+4 .. 8e+7 in the high halves (the order the GEMM kernel expands cheapest).
__global__ void k_lower_packed4(const int8_t *__restrict__ X, uint8_t *__restrict__ X4, int64_t rows, int C, int k4p,
                                int gs_shift, const int32_t *__restrict__ ashift)
{
    const int P = k4p / 16;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * P) return;
    const int64_t row = i / P;
    const int piece = (int)(i % P);
    const uint4 v = *reinterpret_cast<const uint4 *>(X + row * C + piece * 16);
    const int s = ashift[(piece >> 1) >> gs_shift];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t nib[4];   // the four codes of dword k in the low halves of its bytes
    for (int k = 0; k < 4; ++k) {
        uint32_t o = 0;
        for (int b = 0; b < 4; ++b) {
            const int x = (int)(int8_t)((w[k] >> (8 * b)) & 0xFF);
            o |= (uint32_t)(min(7, max(-8, x >> s)) & 0xF) << (8 * b);
        }
        nib[k] = o;
    }
    *reinterpret_cast<uint2 *>(X4 + row * (C / 2) + piece * 8) = make_uint2(nib[0] | (nib[1] << 4), nib[2] | (nib[3] << 4));
}

// Extraction positions found at run time (Section 4.1, dynamic option; Section 9 "Finding extraction positions
// at runtime"): per channel group the highest magnitude bit p of all values (ones' complement for negative ones) is
// found by OR-ing v ^ (v << 1) over the group; three more bits below the sign can be kept: s = max(0, p - 2).
// Thread (tx, ty) of a block of 1024 ORs the 16 channels at column piece blockIdx.y*TX + tx over the rows
// blockIdx.x*TY + ty, + gridDim.x*TY, ...; the block combines its rows in LDS.  PARTIAL: the block then leaves the
// masks of its groups in a row of its own (no atomics on shared words: with a hundred blocks those queue up for tens
// of microseconds) and the block that finishes last ORs the rows.  Otherwise (the variant that lives in G + 1 scan
// words) it adds what is new to the group's mask (an atomic only if a coherent read shows bits missing).  Either way
// the last block turns the masks of the scanned groups (the first g4) into positions, copies the calibrated
// positions of the other groups, and leaves what must be zero for the next call zero.  No block waits for another.
constexpr int kScanThreads = 1024;
template <bool PARTIAL>
__global__ __launch_bounds__(kScanThreads) void k_dyn_positions(const int8_t *__restrict__ X, int64_t rows, int C,
                                                                int pieces, int tx_log2, int gs, int G, int g4,
                                                                uint32_t *scan, const int32_t *__restrict__ ashift_static,
                                                                int32_t *__restrict__ ashift_dyn)
{
    __shared__ uint32_t sh[kScanThreads];
    __shared__ int last;
    const int tid = threadIdx.x;
    const int TX = 1 << tx_log2, TY = kScanThreads >> tx_log2;
    const int tx = tid & (TX - 1), ty = tid >> tx_log2;
    const int piece = blockIdx.y * TX + tx;
    const bool active = piece < pieces;
    uint32_t m = 0;
    if (active) {
        uint32_t acc = 0;
        const int64_t step = (int64_t)gridDim.x * TY;
        const int8_t *src = X + (int64_t)piece * 16;
        // per byte v ^ (v << 1): bit j + 1 is set when bits j + 1 and j of v differ, and the highest such j is the highest
        // set bit of the magnitude (v, or ~v when negative), so the sign needs no handling (the shift carries bit 7 of a
        // byte into bit 0 of the next, which is not used); then the four dwords together
        auto fold = [](const uint4 v) { return (v.x ^ (v.x << 1)) | (v.y ^ (v.y << 1)) | (v.z ^ (v.z << 1)) | (v.w ^ (v.w << 1)); };
        int64_t r = (int64_t)blockIdx.x * TY + ty;
        for (; r + 7 * step < rows; r += 8 * step) {   // eight independent loads in flight
            uint4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = *reinterpret_cast<const uint4 *>(src + (r + k * step) * C);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc |= fold(v[k]);
        }
        for (; r + 1 * step < rows; r += 2 * step) {
            const uint4 v0 = *reinterpret_cast<const uint4 *>(src + r * C);
            const uint4 v1 = *reinterpret_cast<const uint4 *>(src + (r + step) * C);
            acc |= fold(v0) | fold(v1);
        }
        for (; r < rows; r += step) acc |= fold(*reinterpret_cast<const uint4 *>(src + r * C));
        acc |= acc >> 16;
        acc |= acc >> 8;
        m = acc & 0xFEu;
    }
    sh[tid] = m;
    __syncthreads();
    if (PARTIAL) {
        // Every block leaves the masks of its groups in a row of its own (device-coherent stores, no atomics on shared
        // words: with a block per compute unit those queue up for tens of microseconds), draws a ticket once the
        // stores have completed, and the block that draws the last one ORs the rows together.
        __shared__ uint32_t gmask[kMaxGroups + 1];
        const int ppg = gs >> 4;   // pieces per group
        if (ty == 0) {
            for (int y = 1; y < TY; ++y) m |= sh[y * TX + tx];
        }
        __syncthreads();
        if (ty == 0) sh[tx] = m;
        for (int g = tid; g <= kMaxGroups; g += kScanThreads) gmask[g] = 0;
        __syncthreads();
        uint32_t *part = scan + kScanHead;
        if (ty == 0 && active && (tx & (ppg - 1)) == 0) {
            uint32_t gm = 0;
            for (int k = 0; k < ppg; ++k) gm |= sh[tx + k];
            __hip_atomic_store(&part[(int64_t)blockIdx.x * g4 + (piece * 16) / gs], gm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        if (tid == 0) last = atomicAdd(&scan[0], 1u) == gridDim.x * gridDim.y - 1;
        __syncthreads();
        if (!last) return;
        const int total = (int)gridDim.x * g4;
        for (int i = tid; i < total; i += kScanThreads) {
            const uint32_t v = __hip_atomic_load(&part[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v) atomicOr(&gmask[i % g4], v);
        }
        __syncthreads();
        for (int g = tid; g <= G; g += kScanThreads) {
            if (g < g4) {
                const uint32_t mask = gmask[g];
                const int p = mask ? 31 - __clz((int)mask) : 0;   // bit p of the mask: highest magnitude bit p - 1
                ashift_dyn[g] = p - 3 > 0 ? p - 3 : 0;
            } else {
                ashift_dyn[g] = ashift_static[g];
            }
        }
        if (tid == 0) scan[0] = 0;
        return;
    }
    if (ty == 0 && active) {
        for (int y = 1; y < TY; ++y) m |= sh[y * TX + tx];
        uint32_t *dst = &scan[(piece * 16) / gs];
        const uint32_t seen = __hip_atomic_load(dst, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (m & ~seen) atomicOr(dst, m);
    }
    // The only results other blocks need are those of the atomics above, which are performed at the device's
    // coherence point: it is enough that they have completed before this block's ticket is drawn (a full
    // release fence would also write back the L2, i.e. the whole output of the kernel before this one).
    __builtin_amdgcn_s_waitcnt(0x0070);
    __syncthreads();
    if (tid == 0) last = atomicAdd(&scan[G], 1u) == gridDim.x * gridDim.y - 1;
    __syncthreads();
    if (!last) return;
    for (int g = tid; g <= G; g += kScanThreads) {
        if (g < g4) {
            const uint32_t mask = atomicOr(&scan[g], 0u);   // device-scope read of what all blocks added
            const int p = mask ? 31 - __clz((int)mask) : 0;   // bit p of the mask: highest magnitude bit p - 1
            ashift_dyn[g] = p - 3 > 0 ? p - 3 : 0;
            scan[g] = 0;
        } else {
            ashift_dyn[g] = ashift_static[g];
        }
    }
    if (tid == 0) scan[G] = 0;
}

// Eq. 1 for activations: four values per thread, one packed dword out.
__global__ void k_quantize_act(const float *__restrict__ x, int8_t *__restrict__ q, int64_t n, float S)
{
    int64_t i4 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i4 >= n) return;
    if (i4 + 4 <= n) {
        float4 v = *reinterpret_cast<const float4 *>(x + i4);
        uint32_t w = (uint32_t)(quant_code(v.x, S, -127.f, 127.f) & 0xFF) |
                     ((uint32_t)(quant_code(v.y, S, -127.f, 127.f) & 0xFF) << 8) |
                     ((uint32_t)(quant_code(v.z, S, -127.f, 127.f) & 0xFF) << 16) |
                     ((uint32_t)(quant_code(v.w, S, -127.f, 127.f) & 0xFF) << 24);
        *reinterpret_cast<uint32_t *>(q + i4) = w;
    } else {
        for (int64_t i = i4; i < n; ++i) q[i] = (int8_t)quant_code(x[i], S, -127.f, 127.f);
    }
}

// Stand-alone effective-bit extraction (Section 4.1): eight channels per thread.
__global__ void k_bitlower(const int8_t *__restrict__ src, uint8_t *__restrict__ dst, int64_t rows, int C, int gs,
                           const uint8_t *__restrict__ shifts, int per_row, int mode)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int C8 = C / 8;
    if (i >= rows * C8) return;
    int64_t row = i / C8;
    int c0 = (int)(i % C8) * 8;
    int G = C / gs;
    int s = per_row ? shifts[row * G + c0 / gs] : shifts[c0 / gs];  // 8 | group size: one position for all eight
    uint2 in = *reinterpret_cast<const uint2 *>(src + row * C + c0);
    uint32_t w[2] = {in.x, in.y};
    int half = (mode & 1) && s > 0 ? 1 << (s - 1) : 0;
    uint32_t out = 0;
    for (int j = 0; j < 8; ++j) {
        int v = (int)(int8_t)((w[j >> 2] >> (8 * (j & 3))) & 0xFF);
        int l = min(7, max(-8, (v + half) >> s)) & 0xF;
        out |= (uint32_t)l << (4 * j);
    }
    *reinterpret_cast<uint32_t *>(dst + row * (C / 2) + c0 / 2) = out;
}

// Residual reorder operator (Section 5, step 3): dst[row][j] = src[row][perm[j]].  Rows are a multiple of 32 bytes and
// at most 159 groups long (checked when the layer is packed).  A block copies a run of whole rows into LDS with
// coalesced 16-byte loads and gathers from there, so that every input byte leaves HBM once; a
// thread owns the same 16-byte output piece(s) of every row and keeps their sixteen source indices in registers
// (packed in pairs).  NP = pieces per thread: 1 for rows of up to 4096 bytes (several rows per pass then), else the
// row's pieces are dealt out over the 256 threads.
template <int NP>
__global__ __launch_bounds__(256) void k_permute_rows(const int8_t *__restrict__ src, int8_t *__restrict__ dst,
                                                      const int32_t *__restrict__ perm, int64_t rows, int C)
{
    extern __shared__ __align__(16) uint8_t stage[];
    const int P = C >> 4;                              // 16-byte pieces per row
    const int t = threadIdx.x;
    const int RP = NP == 1 ? 256 / P : 1;              // rows per pass over the staged run
    const int RB = 4 * RP;                             // rows per run
    const int slot_row = NP == 1 ? t / P : 0;
    const bool active = NP > 1 || slot_row < RP;
    uint32_t pp[NP][8];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int piece = NP == 1 ? t % P : t + 256 * k;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            pp[k][i] = piece < P ? ((uint32_t)perm[16 * piece + 2 * i] | ((uint32_t)perm[16 * piece + 2 * i + 1] << 16)) : 0u;
    }
    const int64_t runs = (rows + RB - 1) / RB;
    for (int64_t c = blockIdx.x; c < runs; c += gridDim.x) {
        const int64_t r0 = c * RB;
        const int64_t left = rows - r0;
        const int span = (int)(left < RB ? left : RB) * C;   // bytes of this run (rows are contiguous)
        const int8_t *run = src + r0 * C;
        for (int o = t * 16; o < span; o += 256 * 16)
            *reinterpret_cast<uint4 *>(stage + o) = *reinterpret_cast<const uint4 *>(run + o);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row_l = q * RP + slot_row;
            if (!active || row_l >= left) continue;
            const uint8_t *rowp = stage + row_l * C;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                const int piece = NP == 1 ? t % P : t + 256 * k;
                if (piece >= P) continue;
                uint32_t w[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t a = pp[k][2 * i], b = pp[k][2 * i + 1];
                    w[i] = (uint32_t)rowp[a & 0xFFFFu] | ((uint32_t)rowp[a >> 16] << 8) | ((uint32_t)rowp[b & 0xFFFFu] << 16) |
                           ((uint32_t)rowp[b >> 16] << 24);
                }
                *reinterpret_cast<uint4 *>(dst + (r0 + row_l) * C + 16 * piece) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        __syncthreads();
    }
}

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace flexiq

using namespace flexiq;

extern "C" const char *flexiq_strerror(int status)
{
    switch (status) {
        case FLEXIQ_OK: return "ok";
        case FLEXIQ_EINVAL: return "invalid argument";
        case FLEXIQ_EALIGN: return "device pointer not 16-byte aligned";
        case FLEXIQ_ENOMEM: return "out of memory";
        case FLEXIQ_EHIP: return "HIP runtime error";
        default: return "unknown flexiq status";
    }
}

extern "C" const char *flexiq_last_hip_error(void)
{
    static thread_local std::string copy;
    std::lock_guard<std::mutex> lk(g_err_mu);
    copy = g_err;
    return copy.c_str();
}

namespace {
struct DevBuf {  // frees on scope exit unless released
    void *p = nullptr;
    ~DevBuf()
    {
        if (p) (void)hipFree(p);
    }
    void *release()
    {
        void *r = p;
        p = nullptr;
        return r;
    }
};
}  // namespace

extern "C" int flexiq_layer_free(flexiq_layer *L)
{
    if (!L) return FLEXIQ_OK;
    void *bufs[] = {L->d_w8, L->d_w4, L->d_wshift, L->d_ashift, L->d_ashift_dyn, L->d_scan, L->d_cs, L->d_perm, L->d_w6, L->d_w6s};   // d_w4x is the second half of d_w8, d_bias of d_cs
    int rc = FLEXIQ_OK;
    for (void *b : bufs)
        if (b && hipFree(b) != hipSuccess) rc = FLEXIQ_EHIP;
    delete L;
    return rc;
}

extern "C" int flexiq_quantize_pack(const flexiq_pack_desc *d, flexiq_layer **out)
{
    if (!d || !out || !d->W || !d->act_absmax) return FLEXIQ_EINVAL;
    if (d->N <= 0 || d->C <= 0 || d->R <= 0 || d->S <= 0) return FLEXIQ_EINVAL;
    if (d->group_size != 32 && d->group_size != 64) return FLEXIQ_EINVAL;
    if (d->C % d->group_size != 0) return FLEXIQ_EINVAL;
    if (!(d->x_scale > 0.0f) || !std::isfinite(d->x_scale)) return FLEXIQ_EINVAL;
    const int N = d->N, C = d->C, T = d->R * d->S, gs = d->group_size, G = C / gs;
    {   // what the GEMM kernel could never launch is refused here, before any device work
        const int64_t units = (int64_t)T * (((C / kUnit) + 1) & ~1), npad = cdiv(N, kNPadTo) * kNPadTo;
        if (G > kMaxGroups || units * 32 * npad * 2 > kMaxWeightBytes) return FLEXIQ_EINVAL;
    }
    if (d->perm) {  // must be a permutation of 0..C-1
        std::vector<char> seen(C, 0);
        for (int j = 0; j < C; ++j) {
            int v = d->perm[j];
            if (v < 0 || v >= C || seen[v]) return FLEXIQ_EINVAL;
            seen[v] = 1;
        }
    }
    // Output order: the rows of W (and the biases) are taken in the order out_perm names; everything after
    // this point sees an ordinary layer whose channel n is the caller's channel out_perm[n].
    std::vector<float> Wrows, bias_rows;
    const float *Wsrc = d->W, *bias_src = d->bias;
    if (d->out_perm) {
        std::vector<char> seen(N, 0);
        for (int n = 0; n < N; ++n) {
            int v = d->out_perm[n];
            if (v < 0 || v >= N || seen[v]) return FLEXIQ_EINVAL;
            seen[v] = 1;
        }
        const size_t row = (size_t)T * C;
        Wrows.resize((size_t)N * row);
        for (int n = 0; n < N; ++n) std::memcpy(&Wrows[(size_t)n * row], d->W + (size_t)d->out_perm[n] * row, row * sizeof(float));
        Wsrc = Wrows.data();
        if (d->bias) {
            bias_rows.resize(N);
            for (int n = 0; n < N; ++n) bias_rows[n] = d->bias[d->out_perm[n]];
            bias_src = bias_rows.data();
        }
    }
    flexiq_layer *L = new (std::nothrow) flexiq_layer();
    if (!L) return FLEXIQ_ENOMEM;
    struct Guard {
        flexiq_layer *l;
        ~Guard()
        {
            if (l) flexiq_layer_free(l);
        }
    } guard{L};
    L->N = N; L->C = C; L->R = d->R; L->S = d->S; L->group_size = gs; L->G = G; L->T = T;
    const int CU = C / kUnit;
    const int CUp = (CU + 1) & ~1;
    const int U = T * CUp;  // every tap holds an even number of units (a K-step is two of them); the pad unit is zero
    L->U = U;
    L->Npad = (int)(cdiv(N, kNPadTo) * kNPadTo);
    L->max_4bit_ch = 0;
    L->x_scale = d->x_scale;
    L->has_bias = d->bias != nullptr;
    L->d_w8 = nullptr; L->d_w4 = nullptr; L->d_w4x = nullptr; L->d_wshift = nullptr; L->d_ashift = nullptr; L->d_ashift_dyn = nullptr; L->d_scan = nullptr; L->dynamic = false; L->x_prelowered = false;
    L->d_cs = nullptr; L->d_bias = nullptr; L->d_perm = nullptr;
    L->d_w6 = nullptr; L->d_w6s = nullptr; L->fp6_limit_static = 0; L->fp6_limit_dynamic = 0;
    FLEXIQ_HIP(hipGetDevice(&L->device));
    {
        int rc = prepare_kernels(L->device);
        if (rc == FLEXIQ_OK) rc = prepare_fp6_kernels(L->device);
        if (rc == FLEXIQ_OK) rc = prepare_stream_kernels(L->device);
        if (rc == FLEXIQ_OK) rc = prepare_conv3_kernels(L->device);
        if (rc == FLEXIQ_OK) rc = prepare_tile_splitk_kernels(L->device);
        if (rc != FLEXIQ_OK) return rc;
    }
    L->out_order_hash = order_hash(d->out_perm, N);
    const int Npad = L->Npad;
    const int64_t Kt = (int64_t)T * C, total = (int64_t)N * Kt;

    DevBuf dW, dScale, dQ, dWmax, dWsNG;
    FLEXIQ_HIP(hipMalloc(&dW.p, total * sizeof(float)));
    FLEXIQ_HIP(hipMalloc(&dScale.p, N * sizeof(float)));
    FLEXIQ_HIP(hipMalloc(&dQ.p, total));
    FLEXIQ_HIP(hipMalloc(&dWmax.p, C * sizeof(int)));
    FLEXIQ_HIP(hipMalloc(&dWsNG.p, (size_t)N * G));
    FLEXIQ_HIP(hipMemcpy(dW.p, Wsrc, total * sizeof(float), hipMemcpyHostToDevice));
    FLEXIQ_HIP(hipMemset(dWmax.p, 0, C * sizeof(int)));

    k_row_scale<<<N, 256>>>((const float *)dW.p, Kt, (float *)dScale.p);
    k_quantize_rows<<<(unsigned)cdiv(total, 256), 256>>>((const float *)dW.p, (const float *)dScale.p, Kt, total,
                                                         (int8_t *)dQ.p);
    k_chan_wmax<<<N, 256>>>((const int8_t *)dQ.p, N, T, C, (int *)dWmax.p);
    FLEXIQ_HIP(hipGetLastError());

    L->w_scale.resize(N);
    std::vector<int> wmax(C);
    FLEXIQ_HIP(hipMemcpy(L->w_scale.data(), dScale.p, N * sizeof(float), hipMemcpyDeviceToHost));
    FLEXIQ_HIP(hipMemcpy(wmax.data(), dWmax.p, C * sizeof(int), hipMemcpyDeviceToHost));

    // Calibration range of each channel as an 8-bit code, error-estimation score, stored order.
    std::vector<int> rq(C);
    for (int c = 0; c < C; ++c) {
        float t = nearbyintf(d->act_absmax[c] / d->x_scale);
        rq[c] = (int)std::min(127.0f, std::max(0.0f, t));
    }
    L->perm.resize(C);
    if (d->perm) {
        std::memcpy(L->perm.data(), d->perm, C * sizeof(int32_t));
    } else {
        std::vector<int64_t> score(C);
        for (int c = 0; c < C; ++c) score[c] = (int64_t)wmax[c] * rq[c];
        std::iota(L->perm.begin(), L->perm.end(), 0);
        std::stable_sort(L->perm.begin(), L->perm.end(), [&](int a, int b) { return score[a] < score[b]; });
    }
    L->perm_hash = order_hash(L->perm.data(), C);
    // Activation position of a group: the smallest that fits [-a, a], a = widest calibrated range in the group.
    L->a_shift.resize(G);
    for (int g = 0; g < G; ++g) {
        int a = 0;
        for (int j = 0; j < gs; ++j) a = std::max(a, rq[L->perm[g * gs + j]]);
        int s = 0;
        while (s < 4 && a > (8 << s) - 1) ++s;
        L->a_shift[g] = (uint8_t)s;
    }

    FLEXIQ_HIP(hipMalloc((void **)&L->d_perm, C * sizeof(int32_t)));
    FLEXIQ_HIP(hipMemcpy(L->d_perm, L->perm.data(), C * sizeof(int32_t), hipMemcpyHostToDevice));
    {
        std::vector<int32_t> a32(L->a_shift.begin(), L->a_shift.end());
        a32.push_back(0);  // the pad unit of an odd unit count reads one past the last group
        FLEXIQ_HIP(hipMalloc((void **)&L->d_ashift, a32.size() * sizeof(int32_t)));
        FLEXIQ_HIP(hipMemcpy(L->d_ashift, a32.data(), a32.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        FLEXIQ_HIP(hipMalloc((void **)&L->d_ashift_dyn, a32.size() * sizeof(int32_t)));
        FLEXIQ_HIP(hipMemcpy(L->d_ashift_dyn, a32.data(), a32.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        const size_t scan_words = scan_words_total(G);
        FLEXIQ_HIP(hipMalloc((void **)&L->d_scan, scan_words * sizeof(uint32_t)));
        FLEXIQ_HIP(hipMemset(L->d_scan, 0, scan_words * sizeof(uint32_t)));
    }
    // one more (zero) row than groups: the pad unit of an odd unit count looks up group G
    FLEXIQ_HIP(hipMalloc((void **)&L->d_wshift, (size_t)(G + 1) * Npad));
    FLEXIQ_HIP(hipMemset(L->d_wshift, 0, (size_t)(G + 1) * Npad));
    // the 8-bit copy and the expanded 4-bit copy share one allocation: the kernel reaches both through one
    // buffer descriptor and picks the copy with a scalar offset
    FLEXIQ_HIP(hipMalloc((void **)&L->d_w8, (size_t)U * Npad * 32 * 2));
    L->d_w4x = L->d_w8 + (size_t)U * Npad * 32;
    FLEXIQ_HIP(hipMalloc((void **)&L->d_w4, (size_t)U * Npad * 16));

    k_weight_shift<<<(unsigned)cdiv((int64_t)N * G, 256), 256>>>((const int8_t *)dQ.p, L->d_perm, N, T, C, gs, Npad,
                                                                 (uint8_t *)dWsNG.p, L->d_wshift);
    k_pack_tiles<<<(unsigned)cdiv((int64_t)U * Npad, 256), 256>>>((const int8_t *)dQ.p, L->d_perm,
                                                                  (const uint8_t *)dWsNG.p, N, T, C, gs, Npad, U,
                                                                  L->d_w8, L->d_w4, L->d_w4x);
    FLEXIQ_HIP(hipGetLastError());
    L->w_shift.resize((size_t)N * G);
    FLEXIQ_HIP(hipMemcpy(L->w_shift.data(), dWsNG.p, (size_t)N * G, hipMemcpyDeviceToHost));

    // FP6 image for the variant whose 4-bit groups run on the FP6 matrix path (linear layers, whole K-steps), and the
    // certificate of exact fp32 accumulation: with a' = L(x, sa) << sa (|a'| <= 8 << sa) and w' = L(w, sw) << sw, every
    // partial sum of the leading groups is bounded by sum_g (8 << sa_g) * sum_{k in g} |w'[n][k]|; the FP6 prefix ends
    // where that bound would reach 2^24 for some output channel (fp32 holds integers exactly below it).
    if (T == 1 && C % 64 == 0) {
        const int S = C / 64, U32 = C / 32;
        DevBuf dSabs;
        FLEXIQ_HIP(hipMalloc((void **)&L->d_w6, (size_t)S * 3 * Npad * 16));
        FLEXIQ_HIP(hipMalloc((void **)&L->d_w6s, (size_t)((S + 3) / 4) * Npad * 8));
        FLEXIQ_HIP(hipMemset(L->d_w6s, 127, (size_t)((S + 3) / 4) * Npad * 8));
        FLEXIQ_HIP(hipMalloc(&dSabs.p, (size_t)N * U32 * sizeof(int32_t)));
        k_pack_w6<<<(unsigned)cdiv((int64_t)S * Npad, 256), 256>>>((const int8_t *)dQ.p, L->d_perm, (const uint8_t *)dWsNG.p, N, C, gs,
                                                                  Npad, L->d_w6, L->d_w6s, (int32_t *)dSabs.p);
        FLEXIQ_HIP(hipGetLastError());
        std::vector<int32_t> sabs((size_t)N * U32);
        FLEXIQ_HIP(hipMemcpy(sabs.data(), dSabs.p, sabs.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
        const int64_t kExact = (int64_t)1 << 24;
        for (int pass = 0; pass < 2; ++pass) {   // calibrated positions; any positions
            std::vector<int64_t> run(N, 0);
            int limit = 0;
            for (int u = 0; u < U32; ++u) {
                const int amax = 8 << (pass == 0 ? (int)L->a_shift[(u * 32) / gs] : 4);
                bool ok = true;
                for (int n = 0; n < N; ++n) {
                    run[n] += (int64_t)amax * sabs[(size_t)n * U32 + u];
                    ok = ok && run[n] < kExact;
                }
                if (!ok) break;
                limit = (u + 1) * 32;
            }
            (pass == 0 ? L->fp6_limit_static : L->fp6_limit_dynamic) = limit;
        }
    }

    std::vector<float> cs(Npad, 0.0f), bias(Npad, 0.0f);
    for (int n = 0; n < N; ++n) cs[n] = d->x_scale * L->w_scale[n];
    if (bias_src) {
        L->bias.assign(bias_src, bias_src + N);
        std::copy(bias_src, bias_src + N, bias.begin());
    }
    FLEXIQ_HIP(hipMalloc((void **)&L->d_cs, 2 * (size_t)Npad * sizeof(float)));   // scales, then biases
    L->d_bias = L->d_cs + Npad;
    FLEXIQ_HIP(hipMemcpy(L->d_cs, cs.data(), Npad * sizeof(float), hipMemcpyHostToDevice));
    FLEXIQ_HIP(hipMemcpy(L->d_bias, bias.data(), Npad * sizeof(float), hipMemcpyHostToDevice));
    FLEXIQ_HIP(hipDeviceSynchronize());
    guard.l = nullptr;
    *out = L;
    return FLEXIQ_OK;
}

extern "C" int flexiq_layer_info(const flexiq_layer *L, const int32_t **perm, const uint8_t **a_shift,
                                 const uint8_t **w_shift, const float **w_scale, int32_t *G, int32_t *max_4bit_ch)
{
    if (!L) return FLEXIQ_EINVAL;
    if (perm) *perm = L->perm.data();
    if (a_shift) *a_shift = L->a_shift.data();
    if (w_shift) *w_shift = L->w_shift.data();
    if (w_scale) *w_scale = L->w_scale.data();
    if (G) *G = L->G;
    if (max_4bit_ch) *max_4bit_ch = L->max_4bit_ch;
    return FLEXIQ_OK;
}

extern "C" int flexiq_layer_dump(const flexiq_layer *L, int8_t *w8, uint8_t *w4, int8_t *w4x)
{
    if (!L) return FLEXIQ_EINVAL;
    const int N = L->N, C = L->C, T = L->T, Npad = L->Npad, U = L->U, CU = ((C / kUnit) + 1) & ~1;
    FLEXIQ_HIP(hipDeviceSynchronize());
    int8_t *const dst8[2] = {w8, w4x};
    const int8_t *const src8[2] = {L->d_w8, L->d_w4x};
    for (int k = 0; k < 2; ++k) {
        if (!dst8[k]) continue;
        std::vector<int8_t> raw((size_t)U * 2 * Npad * 16);
        FLEXIQ_HIP(hipMemcpy(raw.data(), src8[k], raw.size(), hipMemcpyDeviceToHost));
        for (int n = 0; n < N; ++n)
            for (int t = 0; t < T; ++t)
                for (int c = 0; c < C; ++c) {
                    int u = t * CU + c / 32, q2 = (c % 32) / 16, j = c % 16;
                    dst8[k][((size_t)n * T + t) * C + c] = raw[(((size_t)u * 2 + q2) * Npad + n) * 16 + j];
                }
    }
    if (w4) {
        std::vector<uint8_t> raw((size_t)U * Npad * 16);
        FLEXIQ_HIP(hipMemcpy(raw.data(), L->d_w4, raw.size(), hipMemcpyDeviceToHost));
        std::memset(w4, 0, (size_t)N * T * (C / 2));
        for (int n = 0; n < N; ++n)
            for (int t = 0; t < T; ++t)
                for (int c = 0; c < C; ++c) {
                    int u = t * CU + c / 32, j = c % 32;
                    int e = j / 8, r = j % 8, b = r % 4, hi = r / 4;
                    int code = (raw[((size_t)u * Npad + n) * 16 + e * 4 + b] >> (4 * hi)) & 0xF;
                    w4[((size_t)n * T + t) * (C / 2) + c / 2] |= (uint8_t)(code << (4 * (c & 1)));
                }
    }
    return FLEXIQ_OK;
}

extern "C" int flexiq_set_ratio(flexiq_layer *L, float r, int32_t *max_4bit_ch)
{
    if (!L || !(r >= 0.0f) || !(r <= 1.0f)) return FLEXIQ_EINVAL;
    int g4 = (int)std::ceil((double)r * L->G - 1e-6);
    g4 = std::min(std::max(g4, 0), (int)L->G);
    L->max_4bit_ch = g4 * L->group_size;
    if (max_4bit_ch) *max_4bit_ch = L->max_4bit_ch;
    return FLEXIQ_OK;
}

extern "C" int flexiq_quantize_act(const float *x, int8_t *q, int64_t n, float scale, void *stream)
{
    if (n < 0 || !(scale > 0.0f)) return FLEXIQ_EINVAL;
    if (n == 0) return FLEXIQ_OK;
    if (!x || !q) return FLEXIQ_EINVAL;
    if (!aligned16(x) || !aligned16(q)) return FLEXIQ_EALIGN;
    int64_t threads = cdiv(n, 4);
    k_quantize_act<<<(unsigned)cdiv(threads, 256), 256, 0, (hipStream_t)stream>>>(x, q, n, scale);
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}

extern "C" int flexiq_bitlower(const int8_t *src, uint8_t *dst, int64_t rows, int32_t C, int32_t group_size,
                               const uint8_t *shifts, int per_row, int mode, void *stream)
{
    if (rows < 0 || C <= 0 || group_size <= 0 || C % group_size != 0 || group_size % 8 != 0) return FLEXIQ_EINVAL;
    if (mode != 0 && mode != 1) return FLEXIQ_EINVAL;
    if (rows == 0) return FLEXIQ_OK;
    if (!src || !dst || !shifts) return FLEXIQ_EINVAL;
    if (!aligned16(src) || !aligned16(dst)) return FLEXIQ_EALIGN;
    int64_t threads = rows * (C / 8);
    k_bitlower<<<(unsigned)cdiv(threads, 256), 256, 0, (hipStream_t)stream>>>(src, dst, rows, C, group_size, shifts,
                                                                             per_row ? 1 : 0, mode);
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}

namespace {
// Launch shape of the scan kernel for `rows` rows of the handle's 4-bit channel range.
struct ScanLaunch {
    int g4, pieces, tx_log2;
    unsigned gx, gy;
};
ScanLaunch scan_launch(const flexiq_layer *L, int64_t rows, int max_blocks)
{
    ScanLaunch sl;
    sl.g4 = L->max_4bit_ch / L->group_size;
    sl.pieces = L->max_4bit_ch / 16;             // 16-channel pieces per row to scan
    sl.tx_log2 = 0;
    while ((1 << sl.tx_log2) < sl.pieces && sl.tx_log2 < 8) ++sl.tx_log2;
    const int TX = 1 << sl.tx_log2, TY = kScanThreads >> sl.tx_log2;
    sl.gx = 1;
    sl.gy = 1;
    if (sl.pieces > 0 && rows > 0) {
        sl.gy = (unsigned)cdiv(sl.pieces, TX);
        // at least four rows per thread, and a bounded number of blocks: every block ends with one atomic on a shared
        // counter (and, in the variant without partial rows, with atomics on the group masks)
        sl.gx = (unsigned)std::min<int64_t>(cdiv(rows, (int64_t)TY * 4), std::max<int64_t>(1, max_blocks / sl.gy));
        if (sl.gx < 1) sl.gx = 1;
    }
    return sl;
}
}  // namespace

extern "C" int flexiq_dynamic_positions(flexiq_layer *L, const int8_t *X, int64_t rows, void *stream)
{
    if (!L || rows < 0) return FLEXIQ_EINVAL;
    if (rows > 0 && !X) return FLEXIQ_EINVAL;
    if (rows > 0 && !aligned16(X)) return FLEXIQ_EALIGN;
    const ScanLaunch sl = scan_launch(L, rows, kScanRowBlocks);
    k_dyn_positions<true><<<dim3(sl.gx, sl.gy), kScanThreads, 0, (hipStream_t)stream>>>(
        X, sl.pieces > 0 ? rows : 0, L->C, sl.pieces, sl.tx_log2, L->group_size, L->G, sl.g4, L->d_scan + standalone_scan_offset(L->G), L->d_ashift,
        L->d_ashift_dyn);
    FLEXIQ_HIP(hipGetLastError());
    L->dynamic = true;
    return FLEXIQ_OK;
}

// ---- the same scan for callers that cannot allocate: the scan words live in a file-scope device array ----------
// (each GPU the library runs on holds its own copy of the array, at its own address, until the process ends)
constexpr int kStaticScanWords = 160;   // G + 1 <= 160 words: one OR mask per channel group, then the block counter
static __device__ __align__(256) uint32_t scratch[kStaticScanWords];
namespace {
std::mutex g_scratch_mu;
uint32_t *g_scratch_ptr[64];   // per device: the array's device address (the name `scratch` is only a host-side stand-in)
}  // namespace

extern "C" int flexiq_dynamic_positions_static(flexiq_layer *L, const int8_t *X, int64_t rows, void *stream)
{
    if (!L || rows < 0) return FLEXIQ_EINVAL;
    if (rows > 0 && !X) return FLEXIQ_EINVAL;
    if (rows > 0 && !aligned16(X)) return FLEXIQ_EALIGN;
    if (L->G + 1 > kStaticScanWords) return FLEXIQ_EINVAL;   // more channel groups than the static scan words hold
    int dev = -1;
    FLEXIQ_HIP(hipGetDevice(&dev));
    if (dev != L->device || dev < 0 || dev >= 64) return FLEXIQ_EINVAL;
    uint32_t *words;
    {
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        if (!g_scratch_ptr[dev]) {   // first call on this device (which is current)
            uint32_t *ptr = nullptr;
            FLEXIQ_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
            g_scratch_ptr[dev] = ptr;
        }
        words = g_scratch_ptr[dev];
    }
    // The array is zero when the library is loaded and every scan leaves the words it touched at zero again (its
    // last block clears masks and counter), so nothing is cleared here.
    const ScanLaunch sl = scan_launch(L, rows, 128);
    k_dyn_positions<false><<<dim3(sl.gx, sl.gy), kScanThreads, 0, (hipStream_t)stream>>>(X, sl.pieces > 0 ? rows : 0, L->C, sl.pieces,
                                                                                           sl.tx_log2, L->group_size, L->G, sl.g4, words,
                                                                                           L->d_ashift, L->d_ashift_dyn);
    FLEXIQ_HIP(hipGetLastError());
    L->dynamic = true;
    return FLEXIQ_OK;
}

extern "C" int flexiq_lower_fp6(const flexiq_layer *L, const int8_t *X, int64_t M, uint8_t *x6, int8_t *xlow, void *stream)
{
    if (!L || M < 0 || !L->d_w6) return FLEXIQ_EINVAL;
    if (M == 0) return FLEXIQ_OK;
    const int k6 = fp6_channels(L), k4 = L->max_4bit_ch;
    if (!X || (k6 > 0 && !x6) || (k6 < k4 && !xlow) || xlow == X) return FLEXIQ_EINVAL;
    if (!aligned16(X) || !aligned16(x6) || !aligned16(xlow)) return FLEXIQ_EALIGN;
    const int32_t *pos = L->dynamic ? L->d_ashift_dyn : L->d_ashift;
    const int gs_shift = L->group_size == 64 ? 1 : 0;
    if (k6 > 0) {
        const int64_t threads = M * (k6 / 32);
        k_lower_fp6<<<(unsigned)cdiv(threads, 256), 256, 0, (hipStream_t)stream>>>(X, M, L->C, k6, gs_shift, pos, x6);
    }
    if (xlow) {
        const int64_t threads = M * (L->C / 16);
        k_lower_int8_range<<<(unsigned)cdiv(threads, 256), 256, 0, (hipStream_t)stream>>>(X, xlow, M, L->C, k6, k4, gs_shift, pos);
    }
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}

extern "C" int flexiq_lower_packed4(const flexiq_layer *L, const int8_t *X, int64_t M, uint8_t *x4, void *stream)
{
    if (!L || M < 0 || L->R != 1 || L->S != 1) return FLEXIQ_EINVAL;
    if (M == 0) return FLEXIQ_OK;
    if (!X || !x4) return FLEXIQ_EINVAL;
    if (!aligned16(X) || !aligned16(x4)) return FLEXIQ_EALIGN;
    const int k4p = (L->max_4bit_ch / 64) * 64;
    if (k4p == 0) return FLEXIQ_OK;
    const int64_t threads = M * (k4p / 16);
    if (cdiv(threads, 256) > 0x7fffffff) return FLEXIQ_EINVAL;
    k_lower_packed4<<<(unsigned)cdiv(threads, 256), 256, 0, (hipStream_t)stream>>>(X, x4, M, L->C, k4p, L->group_size == 64 ? 1 : 0,
                                                                                     L->dynamic ? L->d_ashift_dyn : L->d_ashift);
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}

extern "C" int flexiq_input_prelowered(flexiq_layer *L, int on)
{
    if (!L) return FLEXIQ_EINVAL;
    L->x_prelowered = on != 0;
    return FLEXIQ_OK;
}

extern "C" int flexiq_static_positions(flexiq_layer *L)
{
    if (!L) return FLEXIQ_EINVAL;
    L->dynamic = false;
    return FLEXIQ_OK;
}

extern "C" int flexiq_layer_positions(const flexiq_layer *L, uint8_t *a_shift)
{
    if (!L || !a_shift) return FLEXIQ_EINVAL;
    std::vector<int32_t> a32(L->G);
    FLEXIQ_HIP(hipDeviceSynchronize());
    FLEXIQ_HIP(hipMemcpy(a32.data(), L->dynamic ? L->d_ashift_dyn : L->d_ashift, a32.size() * sizeof(int32_t),
                         hipMemcpyDeviceToHost));
    for (int g = 0; g < L->G; ++g) a_shift[g] = (uint8_t)a32[g];
    return FLEXIQ_OK;
}

extern "C" int flexiq_permute_channels(const flexiq_layer *L, const int8_t *src, int8_t *dst, int64_t rows,
                                       void *stream)
{
    if (!L || rows < 0) return FLEXIQ_EINVAL;
    if (rows == 0) return FLEXIQ_OK;
    if (!src || !dst || src == dst) return FLEXIQ_EINVAL;
    if (!aligned16(src) || !aligned16(dst)) return FLEXIQ_EALIGN;
    const int C = L->C;
    if (C % 16 != 0 || C > 16384) return FLEXIQ_EINVAL;   // (no packed layer has such rows)
    const int P = C / 16;
    const int np = P <= 256 ? 1 : P <= 512 ? 2 : 4;
    const int rb = np == 1 ? 4 * (256 / P) : 4;          // rows per staged run: at most 16 KB (64 KB for the long rows)
    const int64_t runs = cdiv(rows, rb);
    const unsigned grid = (unsigned)std::min<int64_t>(runs, 2048);
    const size_t lds = (size_t)rb * C;
    hipStream_t st = (hipStream_t)stream;
    if (np == 1) k_permute_rows<1><<<grid, 256, lds, st>>>(src, dst, L->d_perm, rows, C);
    else if (np == 2) k_permute_rows<2><<<grid, 256, lds, st>>>(src, dst, L->d_perm, rows, C);
    else k_permute_rows<4><<<grid, 256, lds, st>>>(src, dst, L->d_perm, rows, C);
    FLEXIQ_HIP(hipGetLastError());
    return FLEXIQ_OK;
}
