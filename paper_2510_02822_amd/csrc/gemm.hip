// Mixed 4-bit / 8-bit GEMM and implicit-GEMM convolution for gfx950 (Section 7 of the paper,
// re-designed for CDNA4).
//
// gfx950 has no 4-bit integer matrix instruction, so a 4-bit channel group cannot run on a faster
// matrix path than an 8-bit one.  The group's contribution
//     2^(sa+sw) * sum_k L(x,sa) * L(w,sw)   =   sum_k (L(x,sa) << sa) * (L(w,sw) << sw)
// is instead formed by putting each bit-lowered operand back at its extraction position as an int8
// value (both factors fit: |L << s| <= 128) and feeding the same v_mfma_i32_16x16x64_i8 and the same
// int32 accumulator as the 8-bit groups: bit-exact by distributivity, and the separate
// shift-and-accumulate stage of the paper's CUDA kernel disappears.  What the 4-bit groups save
// here is weight bytes (they are streamed from the packed 4-bit copy), not matrix cycles.
//
// Work decomposition: a block owns a BM x BN output tile; the reduction runs in K-steps of 64
// elements (two 32-channel units, each independently 4-bit or 8-bit).  Per K-step the block
// stages the activation tile (bit-lowered on the way: clamp + mask, packed 16-bit VALU ops) and the
// weight tile (8-bit planes copied, 4-bit codes expanded with the per-row position) into LDS as
// four 16-byte "k-planes", so that an MFMA fragment read is 16 lanes x 16 contiguous bytes.
// The MFMA "A" operand is the weight fragment and "B" the activation fragment, so a lane ends up
// with four consecutive output channels of one output row: 16-byte fp32 / 4-byte int8 stores.
#include <mutex>

#include "flexiq_internal.h"

namespace flexiq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef short v2s __attribute__((ext_vector_type(2)));

struct GemmParams {
    const int8_t *X;
    const int8_t *W8;
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
    int32_t gs_shift;  // log2(group_size / 32): unit c32 belongs to group c32 >> gs_shift
    int32_t U;       // units in the reduction (even), CU = C/32 per tap
    int32_t CU;
    int32_t T;       // filter taps
    int32_t tiles_m, tiles_n;
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

template <int WAVES_M, int WAVES_N, int TM, int TN>
struct Cfg {
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int BM = WAVES_M * TM * 16;
    static constexpr int BN = WAVES_N * TN * 16;
    static constexpr int XL = (BM * 4 + NT - 1) / NT;   // 16-byte activation chunks per thread per K-step
    static constexpr int WL8 = (BN * 2 + NT - 1) / NT;  // 16-byte chunks per thread per 8-bit unit
    static constexpr int WL4 = (BN + NT - 1) / NT;      // 16-byte chunks per thread per 4-bit unit
    static constexpr int XROWS = XL * (NT / 4);         // rows staged per K-step (>= BM; the excess reads as zero)
    static constexpr int XPS = (XROWS + 4) * 16;        // bytes per activation k-plane (+4 chunks staggers the planes over the banks)
    static constexpr int WPS = (BN + 4) * 16;
    static constexpr int STAGE = 4 * XPS + 4 * WPS;
    static constexpr int LDS_BYTES = 2 * STAGE;
};

// How the two 32-channel units of the NEXT K-step are staged.
enum StepMode { kMode88 = 0, kMode44 = 1, kMode48 = 2, kModeNone = 3 };

template <int WAVES_M, int WAVES_N, int TM, int TN, bool CONV, int OCC>
struct Kern {
    using C_ = Cfg<WAVES_M, WAVES_N, TM, TN>;
    static constexpr int NT = C_::NT, BM = C_::BM, BN = C_::BN, XPS = C_::XPS, WPS = C_::WPS, STAGE = C_::STAGE;
    static constexpr int XL = C_::XL, WL8 = C_::WL8, WL4 = C_::WL4;

    const GemmParams &p;
    unsigned char *lds;
    int tid;
    __amdgpu_buffer_rsrc_t rx, rw8, rw4, rws;
    // per-thread staging addresses
    int xvoff[XL];            // byte offset of each activation chunk inside the block's buffer window
    int xh0[XL], xw0[XL], xpix[XL];  // conv: top-left input coordinate and pixel index of the image origin
    int x_lds;                // LDS byte offset of chunk 0 inside a stage (chunk j adds j * (NT/4) * 16)
    int w8voff[WL8], w8lds[WL8];
    int w4voff[WL4], w4lds[WL4];
    // staging registers
    v4i xr[XL];
    v4i wr[2][WL8];
    int wsh[2][WL4];
    // scalar K-step iteration state (phase-major: all 4-bit steps, then mixed, then 8-bit)
    int n4, mixed, SP;  // per tap: full 4-bit steps, 0/1 mixed step, steps in total
    int it_phase, it_tap, it_c64;

    __device__ __forceinline__ Kern(const GemmParams &pp, unsigned char *l) : p(pp), lds(l) {}

    __device__ __forceinline__ int phase_begin(int ph) const { return ph == 0 ? 0 : (ph == 1 ? n4 : n4 + mixed); }
    __device__ __forceinline__ int phase_end(int ph) const { return ph == 0 ? n4 : (ph == 1 ? n4 + mixed : SP); }

    // first non-empty phase at or after ph (3 = done)
    __device__ __forceinline__ void seek_phase(int ph)
    {
        while (ph < 3 && phase_begin(ph) == phase_end(ph)) ++ph;
        it_phase = ph;
        it_tap = 0;
        it_c64 = ph < 3 ? phase_begin(ph) : 0;
    }
    __device__ __forceinline__ void advance()
    {
        if (++it_c64 == phase_end(it_phase)) {
            it_c64 = phase_begin(it_phase);
            if (++it_tap == p.T) seek_phase(it_phase + 1);
        }
    }
    __device__ __forceinline__ int cur_mode() const
    {
        return it_phase == 0 ? kMode44 : (it_phase == 1 ? kMode48 : (it_phase == 2 ? kMode88 : kModeNone));
    }

    // ---- global -> registers for the K-step the iterator points at
    template <int MODE>
    __device__ __forceinline__ void load_step()
    {
        const int tap = it_tap, c64 = it_c64;
        if (CONV) {
            const int dy = tap / p.S, dx = tap - dy * p.S;
#pragma unroll
            for (int j = 0; j < XL; ++j) {
                const int hi = xh0[j] + dy, wi = xw0[j] + dx;
                const bool ok = hi >= 0 && hi < p.H && wi >= 0 && wi < p.Wd && xpix[j] >= 0;
                const int off = ok ? (xpix[j] + hi * p.Wd + wi) * p.C + xvoff[j] : (int)0x80000000;
                xr[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, c64 * 64, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < XL; ++j) xr[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, xvoff[j], c64 * 64, 0);
        }
        const int u0 = tap * (2 * SP) + 2 * c64;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int u = u0 + h;
            const bool four = MODE == kMode44 || (MODE == kMode48 && h == 0);
            if (four) {
                const int g = (2 * c64 + h) >> p.gs_shift;
#pragma unroll
                for (int j = 0; j < WL4; ++j) {
                    wr[h][j] = __builtin_amdgcn_raw_buffer_load_b128(rw4, w4voff[j], u * 16 * p.Npad, 0);
                    wsh[h][j] = __builtin_amdgcn_raw_buffer_load_b8(rws, w4voff[j] >> 4, g * p.Npad, 0);
                }
            } else {
#pragma unroll
                for (int j = 0; j < WL8; ++j)
                    wr[h][j] = __builtin_amdgcn_raw_buffer_load_b128(rw8, w8voff[j], u * 32 * p.Npad, 0);
            }
        }
    }

    // ---- registers -> LDS stage, bit-lowering the activations / expanding the 4-bit weights of 4-bit units.
    // (tap, c64) are those the registers were loaded for.
    template <int MODE>
    __device__ __forceinline__ void store_step(unsigned char *stage, int c64)
    {
        unsigned char *xs = stage, *ws = stage + 4 * XPS;
        const int q = tid & 3;
        // this thread's chunks all lie in unit q>>1 of the step
        const bool x_four = MODE == kMode44 || (MODE == kMode48 && (q >> 1) == 0);
        if (MODE == kMode88) {
#pragma unroll
            for (int j = 0; j < XL; ++j) *reinterpret_cast<v4i *>(xs + x_lds + j * (NT / 4) * 16) = xr[j];
        } else {
            // positions of the two units (uniform); a thread uses the one of its own unit
            const int sa0 = p.ashift[(2 * c64) >> p.gs_shift], sa1 = p.ashift[(2 * c64 + 1) >> p.gs_shift];
            const int sa = (q >> 1) ? sa1 : sa0;
#pragma unroll
            for (int j = 0; j < XL; ++j) {
                v4i v = xr[j];
                if (MODE == kMode44) {
                    v = lower16(v, sa);
                } else {
                    const v4i l = lower16(v, sa);
                    v = x_four ? l : v;
                }
                *reinterpret_cast<v4i *>(xs + x_lds + j * (NT / 4) * 16) = v;
            }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const bool four = MODE == kMode44 || (MODE == kMode48 && h == 0);
            if (four) {
#pragma unroll
                for (int j = 0; j < WL4; ++j) {
                    if (BN % NT == 0 || tid + j * NT < BN) {
                        v4i a, b;
                        expand32(wr[h][j], wsh[h][j], a, b);
                        *reinterpret_cast<v4i *>(ws + (2 * h) * WPS + w4lds[j]) = a;
                        *reinterpret_cast<v4i *>(ws + (2 * h + 1) * WPS + w4lds[j]) = b;
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < WL8; ++j)
                    if ((2 * BN) % NT == 0 || tid + j * NT < 2 * BN)
                        *reinterpret_cast<v4i *>(ws + (2 * h) * WPS + w8lds[j]) = wr[h][j];
            }
        }
    }
};

template <int WAVES_M, int WAVES_N, int TM, int TN, bool CONV, int OCC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void k_mixed(const GemmParams p)
{
    using K_ = Kern<WAVES_M, WAVES_N, TM, TN, CONV, OCC>;
    constexpr int NT = K_::NT, BM = K_::BM, BN = K_::BN, XPS = K_::XPS, WPS = K_::WPS, STAGE = K_::STAGE;
    constexpr int XL = K_::XL, WL8 = K_::WL8, WL4 = K_::WL4;
    extern __shared__ __align__(16) unsigned char lds[];

    K_ k(p, lds);
    const int tid = threadIdx.x;
    k.tid = tid;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- block -> tile.  Consecutive block ids land on different XCDs (8 of them, each with its own
    // L2); renumber so that the blocks sharing an XCD walk neighbouring tiles, then sweep bands of 8
    // tile rows with the tile column varying slowest inside a band (weights stay L2-resident).
    int tile_m, tile_n;
    {
        const int nb = gridDim.x;
        int b = blockIdx.x;
        if (nb % 8 == 0) b = (b % 8) * (nb / 8) + b / 8;
        constexpr int GMB = 8;
        const int band = b / (GMB * p.tiles_n);
        const int rows_in_band = min(GMB, p.tiles_m - band * GMB);
        const int r = b - band * GMB * p.tiles_n;
        tile_m = band * GMB + r % rows_in_band;
        tile_n = r / rows_in_band;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;
    const int rows_valid = (int)min((int64_t)BM, p.M - m0);

    // ---- buffer windows: reads past a window return zero, which is what rows beyond M, padded
    // pixels and dummy staging rows need
    constexpr int kRsrcFlags = 0x00020000;
    k.rw8 = __builtin_amdgcn_make_buffer_rsrc((void *)(p.W8 + (int64_t)n0 * 16), 0, p.U * 32 * p.Npad - n0 * 16, kRsrcFlags);
    k.rw4 = __builtin_amdgcn_make_buffer_rsrc((void *)(p.W4 + (int64_t)n0 * 16), 0, p.U * 16 * p.Npad - n0 * 16, kRsrcFlags);
    k.rws = __builtin_amdgcn_make_buffer_rsrc((void *)(p.wshift + n0), 0, (p.C >> (5 + p.gs_shift)) * p.Npad - n0, kRsrcFlags);
    const int xq = tid & 3;
    if (CONV) {
        const int64_t hw_out = (int64_t)p.Ho * p.Wo;
        const int64_t img0 = m0 / hw_out;
        const int64_t img_bytes = (int64_t)p.H * p.Wd * p.C;
        const int64_t imgs_left = (p.M / hw_out) - img0;  // images from img0 to the end of the batch
        const int64_t win = min(imgs_left * img_bytes, (int64_t)0x7fffffff);
        k.rx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + img0 * img_bytes), 0, (int)win, kRsrcFlags);
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int row = (tid >> 2) + j * (NT / 4);
            const int64_t m = m0 + row;
            const bool ok = row < rows_valid;
            const int64_t mm = ok ? m : m0;
            const int wo = (int)(mm % p.Wo);
            const int ho = (int)((mm / p.Wo) % p.Ho);
            const int b = (int)(mm / hw_out - img0);
            k.xpix[j] = ok ? b * p.H * p.Wd : -1;
            k.xh0[j] = ho * p.stride - p.pad;
            k.xw0[j] = wo * p.stride - p.pad;
            k.xvoff[j] = xq * 16;
        }
    } else {
        k.rx = __builtin_amdgcn_make_buffer_rsrc((void *)(p.X + m0 * p.C), 0, rows_valid * p.C, kRsrcFlags);
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int row = (tid >> 2) + j * (NT / 4);
            k.xvoff[j] = row * p.C + xq * 16;  // rows >= rows_valid fall outside the window: zeros
            k.xh0[j] = k.xw0[j] = k.xpix[j] = 0;
        }
    }
    k.x_lds = xq * XPS + (tid >> 2) * 16;
#pragma unroll
    for (int j = 0; j < WL8; ++j) {
        const int i = tid + j * NT;
        const int q2 = i / BN, row = i - q2 * BN;
        k.w8voff[j] = (q2 * p.Npad + row) * 16;
        k.w8lds[j] = q2 * WPS + row * 16;
    }
#pragma unroll
    for (int j = 0; j < WL4; ++j) {
        const int row = tid + j * NT;
        k.w4voff[j] = row * 16;
        k.w4lds[j] = row * 16;
    }

    // ---- K-step enumeration
    k.SP = (p.CU + 1) >> 1;
    k.n4 = p.K4 >> 6;
    k.mixed = (p.K4 & 63) ? 1 : 0;
    const int steps = p.T * k.SP;
    k.seek_phase(0);

    v4i acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) acc[a][b] = (v4i){0, 0, 0, 0};

    const int frag_plane = lane >> 4, frag_row = lane & 15;
    const int xs_frag = frag_plane * XPS + (wm * TM * 16 + frag_row) * 16;
    const int ws_frag = 4 * XPS + frag_plane * WPS + (wn * TN * 16 + frag_row) * 16;
    auto compute = [&](const unsigned char *stage) {
        v4i wf[TN];
#pragma unroll
        for (int a = 0; a < TN; ++a) wf[a] = *reinterpret_cast<const v4i *>(stage + ws_frag + a * 256);
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            v4i xf = *reinterpret_cast<const v4i *>(stage + xs_frag + b * 256);
#pragma unroll
            for (int a = 0; a < TN; ++a)
                acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[a], xf, acc[a][b], 0, 0, 0);
        }
    };

    // ---- prologue: stage K-step 0
    {
        const int mode = k.cur_mode(), c64 = k.it_c64;
        if (mode == kMode44) { k.template load_step<kMode44>(); k.template store_step<kMode44>(lds, c64); }
        else if (mode == kMode48) { k.template load_step<kMode48>(); k.template store_step<kMode48>(lds, c64); }
        else { k.template load_step<kMode88>(); k.template store_step<kMode88>(lds, c64); }
        k.advance();
    }
    __syncthreads();

    // ---- main loop: two LDS stages, one barrier per K-step.  The iterator `k` always points at the
    // NEXT step to stage.  Steps are enumerated phase by phase (all-4-bit, mixed, all-8-bit); while the
    // next step stays in the current phase the body is straight-line code specialised on that phase
    // (hot loops below); the one step per phase whose successor lies in another phase (or nowhere) runs
    // the generic body.  The accumulators are only ever touched in `compute`, in straight-line code.
    int s = 0;  // K-step being computed
    auto generic_step = [&]() {
        unsigned char *cur = lds + (s & 1) * STAGE;
        unsigned char *nxt = lds + ((s + 1) & 1) * STAGE;
        const int mode = k.cur_mode();
        const int c64 = k.it_c64;
        if (mode == kMode44) k.template load_step<kMode44>();
        else if (mode == kMode48) k.template load_step<kMode48>();
        else if (mode == kMode88) k.template load_step<kMode88>();
        __builtin_amdgcn_sched_barrier(0x38F);
        compute(cur);
        if (mode == kMode44) k.template store_step<kMode44>(nxt, c64);
        else if (mode == kMode48) k.template store_step<kMode48>(nxt, c64);
        else if (mode == kMode88) k.template store_step<kMode88>(nxt, c64);
        if (mode != kModeNone) k.advance();
        ++s;
        __syncthreads();
    };
#define FLEXIQ_HOT_LOOP(MODE, PHASE)                                                         \
    while (s + 1 < steps && k.it_phase == (PHASE)) {                                         \
        unsigned char *cur = lds + (s & 1) * STAGE;                                          \
        unsigned char *nxt = lds + ((s + 1) & 1) * STAGE;                                    \
        const int c64 = k.it_c64;                                                            \
        k.template load_step<MODE>();                                                        \
        __builtin_amdgcn_sched_barrier(0x38F); /* global loads stay ahead of the matrix work */ \
        compute(cur);                                                                        \
        k.template store_step<MODE>(nxt, c64);                                               \
        k.advance();                                                                         \
        ++s;                                                                                 \
        __syncthreads();                                                                     \
    }
    FLEXIQ_HOT_LOOP(kMode44, 0)
    if (s < steps && k.it_phase != 2) generic_step();
    FLEXIQ_HOT_LOOP(kMode48, 1)
    if (s < steps && k.it_phase != 2) generic_step();
    FLEXIQ_HOT_LOOP(kMode88, 2)
    while (s < steps) generic_step();
#undef FLEXIQ_HOT_LOOP

    // ---- epilogue: lane holds output row m (lane & 15) and four consecutive output channels
    const bool want_q = p.q != nullptr, want_y = p.y != nullptr, want_acc = p.acc != nullptr;
    const bool n_vec = (p.N & 3) == 0;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        const int n = n0 + (wn * TN + a) * 16 + 4 * frag_plane;
        if (n >= p.N) continue;
        const float4 cs = *reinterpret_cast<const float4 *>(p.cs + n);  // cs/bias are padded to Npad
        const float4 bi = *reinterpret_cast<const float4 *>(p.bias + n);
        const float csv[4] = {cs.x, cs.y, cs.z, cs.w}, biv[4] = {bi.x, bi.y, bi.z, bi.w};
        float mul[4], add[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            mul[i] = csv[i] * p.r_out;
            add[i] = biv[i] * p.r_out;
        }
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int64_t m = m0 + (wm * TM + b) * 16 + frag_row;
            if (m >= p.M) continue;
            const v4i v = acc[a][b];
            const int iv[4] = {v.x, v.y, v.z, v.w};
            const int64_t o = m * p.N + n;
            if (n_vec) {
                if (want_acc) *reinterpret_cast<v4i *>(p.acc + o) = v;
                if (want_y) {
                    float4 y;
                    y.x = __builtin_fmaf((float)iv[0], csv[0], biv[0]);
                    y.y = __builtin_fmaf((float)iv[1], csv[1], biv[1]);
                    y.z = __builtin_fmaf((float)iv[2], csv[2], biv[2]);
                    y.w = __builtin_fmaf((float)iv[3], csv[3], biv[3]);
                    *reinterpret_cast<float4 *>(p.y + o) = y;
                }
                if (want_q) {
                    uint32_t u[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float t = __builtin_fmaf((float)iv[i], mul[i], add[i]);
                        t = __builtin_amdgcn_fmed3f(t, -128.0f, 127.0f);
                        u[i] = __builtin_bit_cast(uint32_t, t + 12582912.0f);  // 1.5 * 2^23: integer lands in the low bits
                    }
                    uint32_t w01 = __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u);
                    uint32_t w23 = __builtin_amdgcn_perm(u[3], u[2], 0x04000c0cu);
                    *reinterpret_cast<uint32_t *>(p.q + o) = w01 | w23;
                }
            } else {
                for (int i = 0; i < 4 && n + i < p.N; ++i) {
                    if (want_acc) p.acc[o + i] = iv[i];
                    if (want_y) p.y[o + i] = __builtin_fmaf((float)iv[i], csv[i], biv[i]);
                    if (want_q) {
                        float t = __builtin_fmaf((float)iv[i], mul[i], add[i]);
                        t = __builtin_amdgcn_fmed3f(t, -128.0f, 127.0f);
                        p.q[o + i] = (int8_t)(__builtin_bit_cast(uint32_t, t + 12582912.0f) & 0xFF);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Host side: tile-shape choice and launch
// ---------------------------------------------------------------------------------------------

typedef void (*kernel_fn)(const GemmParams);
struct TileShape {
    int BM, BN, lds;
    kernel_fn lin, conv;
};

template <int WAVES_M, int WAVES_N, int TM, int TN, int OCC>
static TileShape make_shape()
{
    using C_ = Cfg<WAVES_M, WAVES_N, TM, TN>;
    static_assert(C_::NT == 256, "the launcher uses 256 threads");
    return TileShape{C_::BM, C_::BN, C_::LDS_BYTES, k_mixed<WAVES_M, WAVES_N, TM, TN, false, OCC>,
                     k_mixed<WAVES_M, WAVES_N, TM, TN, true, OCC>};
}

static const TileShape *shapes(int *count)
{
    static const TileShape tab[] = {
        make_shape<2, 2, 8, 8, 1>(),   // 256 x 256
        make_shape<1, 4, 13, 4, 1>(),  // 208 x 256
        make_shape<1, 4, 10, 4, 1>(),  // 160 x 256
        make_shape<2, 2, 4, 8, 2>(),   // 128 x 256, two blocks per CU
        make_shape<2, 2, 8, 4, 2>(),   // 256 x 128, two blocks per CU
        make_shape<2, 2, 4, 4, 2>(),   // 128 x 128
        make_shape<2, 2, 2, 4, 2>(),   //  64 x 128
        make_shape<2, 2, 2, 2, 2>(),   //  64 x  64
    };
    *count = (int)(sizeof(tab) / sizeof(tab[0]));
    return tab;
}

static int g_num_cu = 0;
static int g_force_shape = -1;

// Pick the tile shape with the smallest modelled time: waves of blocks over the CUs times the cost
// of one tile (matrix work plus a per-K-step overhead that penalises small tiles).
static const TileShape &choose_shape(int64_t M, int N)
{
    int cnt;
    const TileShape *tab = shapes(&cnt);
    if (g_force_shape >= 0 && g_force_shape < cnt) return tab[g_force_shape];
    if (g_num_cu <= 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            g_num_cu = prop.multiProcessorCount;
        if (g_num_cu <= 0) g_num_cu = 256;
    }
    double best = 1e300;
    int bi = 0;
    for (int i = 0; i < cnt; ++i) {
        const double tm = (double)((M + tab[i].BM - 1) / tab[i].BM), tn = (double)((N + tab[i].BN - 1) / tab[i].BN);
        const double rounds = __builtin_ceil(tm * tn / g_num_cu);
        // per K-step: BM*BN/256 MFMA issue slots of 16 cycles per SIMD + staging cost ~ (BM + BN) * 0.6
        const double tile = (double)tab[i].BM * tab[i].BN / 256.0 * 4.0 + 0.6 * (tab[i].BM + tab[i].BN) + 40.0;
        const double cost = rounds * tile;
        if (cost < best) {
            best = cost;
            bi = i;
        }
    }
    return tab[bi];
}

static int launch(const flexiq_layer *L, const int8_t *X, int64_t M, const flexiq_out *out, void *stream, bool conv,
                  int H, int Wd, int Ho, int Wo, int stride, int pad)
{
    GemmParams p;
    p.X = X; p.W8 = L->d_w8; p.W4 = L->d_w4; p.wshift = L->d_wshift; p.ashift = L->d_ashift;
    p.cs = L->d_cs; p.bias = L->d_bias;
    p.acc = out->acc; p.y = out->y; p.q = out->q;
    p.r_out = out->q ? 1.0f / out->out_scale : 1.0f;
    p.M = M; p.N = L->N; p.Npad = L->Npad; p.C = L->C;
    p.K4 = L->max_4bit_ch;
    p.gs_shift = L->group_size == 64 ? 1 : 0;
    p.U = L->U; p.CU = L->C / kUnit; p.T = L->T;
    if ((int64_t)L->U * 32 * L->Npad > 0x7fffffff) return FLEXIQ_EINVAL;  // weight window must fit a buffer descriptor
    p.H = H; p.Wd = Wd; p.Ho = Ho; p.Wo = Wo; p.S = L->S; p.stride = stride; p.pad = pad;
    const TileShape &ts = choose_shape(M, L->N);
    p.tiles_m = (int)((M + ts.BM - 1) / ts.BM);
    p.tiles_n = (L->N + ts.BN - 1) / ts.BN;
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n;
    if (blocks > 0x7fffffff) return FLEXIQ_EINVAL;
    kernel_fn fn = conv ? ts.conv : ts.lin;
    {  // raise the dynamic-LDS limit once per kernel
        static std::mutex mu;
        static std::vector<const void *> attr_done;
        std::lock_guard<std::mutex> lk(mu);
        bool seen = false;
        for (const void *f : attr_done) seen = seen || f == (const void *)fn;
        if (!seen) {
            FLEXIQ_HIP(hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, ts.lds));
            attr_done.push_back((const void *)fn);
        }
    }
    const int nt = 256;
    hipLaunchKernelGGL(fn, dim3((unsigned)blocks), dim3(nt), ts.lds, (hipStream_t)stream, p);
    FLEXIQ_HIP(hipGetLastError());
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

// Test / tuning hook: force tile shape `index` of the internal table (-1 = automatic choice).
extern "C" int flexiq_debug_force_tile(int index)
{
    int cnt;
    (void)shapes(&cnt);
    if (index < -1 || index >= cnt) return FLEXIQ_EINVAL;
    g_force_shape = index;
    return cnt;
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

extern "C" int flexiq_mixed_conv_implicit(const flexiq_layer *L, const int8_t *X, int32_t B, int32_t H, int32_t W,
                                          int32_t stride, int32_t pad, const flexiq_out *out, void *stream)
{
    if (!L || B < 0 || H <= 0 || W <= 0 || stride <= 0 || pad < 0) return FLEXIQ_EINVAL;
    if (H + 2 * pad < L->R || W + 2 * pad < L->S) return FLEXIQ_EINVAL;
    const int Ho = (H + 2 * pad - L->R) / stride + 1, Wo = (W + 2 * pad - L->S) / stride + 1;
    const int64_t M = (int64_t)B * Ho * Wo;
    if (M == 0) return FLEXIQ_OK;  // empty batch
    int rc = check_out(out);
    if (rc) return rc;
    if (!X) return FLEXIQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(X) & 15u) return FLEXIQ_EALIGN;
    return launch(L, X, M, out, stream, true, H, W, Ho, Wo, stride, pad);
}
