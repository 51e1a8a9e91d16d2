// Pieces shared by the kernels that keep a block's weights resident in LDS and stream activations past them
// (stream.hip: rows of a linear layer; conv3.hip: image rows of a 3x3 convolution): vector types, the bit-lowering of
// four activation bytes (Section 4.1), the LDS piece permutation, and the epilogue of one 32 x 32 accumulator fragment.
#pragma once
#include "flexiq_internal.h"

namespace flexiq {
namespace resident {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef short v2s __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;

constexpr int kRsrcFlags = 0x00020000;

// Block barrier without the counter waits of __syncthreads() (the caller has waited for what it needs).  The barrier
// builtin is no memory operation to the compiler: the clobbers keep LDS accesses on their side of it.
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// clamp(v >> s, -8, 7) << s for the four int8 values of a dword: lo2 / hi2 hold the bounds in the upper byte of both
// 16-bit halves, mask clears the s low bits of every byte
__device__ __forceinline__ uint32_t lower4(uint32_t d, v2s lo2, v2s hi2, uint32_t mask)
{
    v2s o = __builtin_bit_cast(v2s, d);   // odd bytes sit on top of the 16-bit halves
    v2s e = o << (short)8;                // even bytes moved up
    o = __builtin_elementwise_min(__builtin_elementwise_max(o, lo2), hi2);
    e = __builtin_elementwise_min(__builtin_elementwise_max(e, lo2), hi2);
    const uint32_t r = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u);
    return r & mask;
}

// all sixteen bytes of a piece, position sa
__device__ __forceinline__ v4i lower16(v4i b, int sa)
{
    const short lo = (short)((-(8 << sa)) << 8), hi = (short)((((8 << sa) - 1) << 8) | 0xFF);
    const v2s lo2 = {lo, lo}, hi2 = {hi, hi};
    const uint32_t mask = 0x01010101u * ((0xFFu << sa) & 0xFFu);
    b.x = (int)lower4((uint32_t)b.x, lo2, hi2, mask);
    b.y = (int)lower4((uint32_t)b.y, lo2, hi2, mask);
    b.z = (int)lower4((uint32_t)b.z, lo2, hi2, mask);
    b.w = (int)lower4((uint32_t)b.w, lo2, hi2, mask);
    return b;
}

// The same result as lower16 for less work in the usual case: when, in every lane of the wave, the squares of a dword's
// four bytes sum to less than (8 << sa)^2, no byte can reach the clamp and clearing the low sa bits is all there is to do
// (5 vector-ALU operations per piece for the test and 4 for the masks against 28).
__device__ __forceinline__ v4i lower16_checked(v4i b, int sa)
{
    const int L = 8 << sa;
    const int s0 = __builtin_amdgcn_sdot4(b.x, b.x, 0, false), s1 = __builtin_amdgcn_sdot4(b.y, b.y, 0, false);
    const int s2 = __builtin_amdgcn_sdot4(b.z, b.z, 0, false), s3 = __builtin_amdgcn_sdot4(b.w, b.w, 0, false);
    const int m = max(max(s0, s1), max(s2, s3));
    if (__builtin_amdgcn_ballot_w64(m >= L * L) == 0) {
        const int mask = (int)(0x01010101u * ((0xFFu << sa) & 0xFFu));
        return (v4i){b.x & mask, b.y & mask, b.z & mask, b.w & mask};
    }
    return lower16(b, sa);
}

// Sixteen bytes of packed 4-bit activation codes (one 32-channel unit of a row; dword e: channels 8e .. 8e+3 in the low
// halves of its bytes, 8e+4 .. 8e+7 in the high halves) -> the two 16-byte pieces of int8 values code << sa, i.e. the
// bit-lowered activations put back at their position (Section 4.1).  Per dword and half: each 16-bit half is shifted right
// arithmetically by 4 - sa with the wanted byte on top (that sign-extends the code), the two results are merged bytewise and
// the low sa bits cleared.
__device__ __forceinline__ uint32_t expand4(uint32_t codes_hi, short t, uint32_t mask)
{
    v2s o = __builtin_bit_cast(v2s, codes_hi);
    v2s e = o << (short)8;
    o = o >> t;
    e = e >> t;
    return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u) & mask;
}
__device__ __forceinline__ void expand_unit(v4i pk, int sa, v4i &first16, v4i &second16)
{
    const short t = (short)(4 - sa);
    const uint32_t mask = 0x01010101u * ((0xFFu << sa) & 0xFFu);
    first16 = (v4i){(int)expand4((uint32_t)pk.x << 4, t, mask), (int)expand4((uint32_t)pk.x, t, mask),
                    (int)expand4((uint32_t)pk.y << 4, t, mask), (int)expand4((uint32_t)pk.y, t, mask)};
    second16 = (v4i){(int)expand4((uint32_t)pk.z << 4, t, mask), (int)expand4((uint32_t)pk.z, t, mask),
                     (int)expand4((uint32_t)pk.w << 4, t, mask), (int)expand4((uint32_t)pk.w, t, mask)};
}

// LDS image of activation rows (pixels): row-major, P = 4, 8 or 16 16-byte pieces per row, the pieces of a row permuted so
// that the fragment reads of sixteen consecutive rows (same logical piece) fall into the sixteen different 16-byte groups
// of the 64 banks: 16 / P consecutive rows already differ in their position modulo 256 bytes and share a permutation.
__device__ __forceinline__ int swizzle(int row, int P) { return P == 4 ? (row >> 2) & 3 : (P == 8 ? (row >> 1) & 7 : row & 15); }

struct FragOut {     // the outputs of a call (any may be null) and the requantisation factor 1 / S_out
    int32_t *acc;
    float *y;
    int8_t *q;
    float r_out;
    int32_t N;
};

// What the consumer of the int8 rows does to its input, done here instead (Section 4.1 applied where the tensor is produced):
// per quad of output columns (four consecutive channels of the consumer, which share a channel group) the clamp bounds of
// the offset code, 128 - (8 << s) and 127 + (8 << s) as floats, and the mask that clears the s low bits of four bytes;
// 0, 255 and all ones where the consumer reads the columns at 8 bits.  `quads` entries of 16 bytes from `ltab` on.
__device__ __forceinline__ void fill_lower_table(unsigned char *ltab, int quads, int n_blk, const int32_t *next_ashift, int next_K4,
                                                 int next_gs_log2, int tid, int nthreads)
{
    for (int qd = tid; qd < quads; qd += nthreads) {
        const int n = n_blk + 4 * qd;
        const bool low = n < next_K4;
        const int s = low ? next_ashift[n >> next_gs_log2] : 0;
        const int L = low ? (8 << s) : 128;
        const uint32_t mask = 0x01010101u * ((0xFFu << s) & 0xFFu);
        *reinterpret_cast<v4i *>(ltab + 16 * qd) = (v4i){__float_as_int(128.0f - (float)L), __float_as_int(127.0f + (float)L), (int)mask, 0};
    }
}

// Epilogue of one accumulator fragment (32 rows x 32 columns; lane: row m, register 4 g + i: column 32 ca + 8 g + 4 fh + i
// of the block, n_blk + that of the layer).  tabb: the block's table in LDS, BN multipliers then BN addends (fp32;
// pre-multiplied by 1 / S_out, with 128 added, when pre_scaled).  lim: columns left from the lane's first one
// (N - n_blk - 4 fh).  QONLY: int8 rows and nothing else, N a multiple of 16.  LOWER (with QONLY): the codes leave bit-lowered
// for the consumer, by the table of fill_lower_table behind the two float tables: the offset code is clamped before it is
// rounded (the bounds are integers, so that equals clamping the rounded code) and its low bits are cleared afterwards.
template <bool QONLY, int BN, bool LOWER = false>
__device__ __forceinline__ void store_fragment(const v16i &acc, const FragOut &o, const unsigned char *tabb, int ca, int n_blk, int64_t m,
                                               bool row_ok, int lim, int fh, bool pre_scaled, bool q_rows)
{
    uint32_t qrow[4];
    if constexpr (QONLY) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = 32 * ca + 8 * g + 4 * fh;
            // (read as integer vectors: a float-typed read of LDS makes the compiler wait for every copy in flight;
            // made opaque: what the compiler cannot trace to a store it may take for undefined)
            v4i mi = *reinterpret_cast<const v4i *>(tabb + 4 * c), ai = *reinterpret_cast<const v4i *>(tabb + 4 * (BN + c));
            asm volatile("" : "+v"(mi), "+v"(ai));
            uint32_t qw = 0;
            if constexpr (LOWER) {
                static_assert(QONLY, "the lowering epilogue writes int8 rows only");
                v4i lt = *reinterpret_cast<const v4i *>(tabb + 4 * (2 * BN) + 4 * c);   // entry c / 4
                asm volatile("" : "+v"(lt));
                const float lo = __int_as_float(lt.x), hi = __int_as_float(lt.y);
                qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(__builtin_fmaf((float)acc[4 * g + 0], __int_as_float(mi.x), __int_as_float(ai.x)), lo, hi), 0, qw);
                qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(__builtin_fmaf((float)acc[4 * g + 1], __int_as_float(mi.y), __int_as_float(ai.y)), lo, hi), 1, qw);
                qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(__builtin_fmaf((float)acc[4 * g + 2], __int_as_float(mi.z), __int_as_float(ai.z)), lo, hi), 2, qw);
                qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(__builtin_fmaf((float)acc[4 * g + 3], __int_as_float(mi.w), __int_as_float(ai.w)), lo, hi), 3, qw);
                qrow[g] = (qw ^ 0x80808080u) & (uint32_t)lt.z;
                continue;
            }
            qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[4 * g + 0], __int_as_float(mi.x), __int_as_float(ai.x)), 0, qw);
            qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[4 * g + 1], __int_as_float(mi.y), __int_as_float(ai.y)), 1, qw);
            qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[4 * g + 2], __int_as_float(mi.z), __int_as_float(ai.z)), 2, qw);
            qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[4 * g + 3], __int_as_float(mi.w), __int_as_float(ai.w)), 3, qw);
            qrow[g] = qw ^ 0x80808080u;
        }
    } else {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = 32 * ca + 8 * g + 4 * fh;
            const int n = n_blk + c;
            v4i mi = *reinterpret_cast<const v4i *>(tabb + 4 * c), ai = *reinterpret_cast<const v4i *>(tabb + 4 * (BN + c));
            asm volatile("" : "+v"(mi), "+v"(ai));
            const float mulv[4] = {__int_as_float(mi.x), __int_as_float(mi.y), __int_as_float(mi.z), __int_as_float(mi.w)};
            const float addv[4] = {__int_as_float(ai.x), __int_as_float(ai.y), __int_as_float(ai.z), __int_as_float(ai.w)};
            uint32_t qw = 0;
            if (o.q) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float mu = pre_scaled ? mulv[i] : mulv[i] * o.r_out;
                    const float ad = pre_scaled ? addv[i] : addv[i] * o.r_out + 128.0f;
                    qw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fmaf((float)acc[4 * g + i], mu, ad), i, qw);
                }
                qw ^= 0x80808080u;
            }
            qrow[g] = qw;
            if (row_ok && (o.acc || o.y || (o.q && !q_rows))) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (c - 4 * fh + i >= lim) continue;
                    const int64_t at = m * o.N + n + i;
                    if (o.acc) o.acc[at] = acc[4 * g + i];
                    if (o.y) o.y[at] = __builtin_fmaf((float)acc[4 * g + i], mulv[i], addv[i]);
                    if (o.q && !q_rows) o.q[at] = (int8_t)((qw >> (8 * i)) & 0xFF);
                }
            }
        }
    }
    if (QONLY || q_rows) {
        // the two halves of the wave hold alternating 4-byte pieces of a row: after exchanging quads 0 <-> 2
        // and 1 <-> 3 lanes 0..31 own columns 0..15 of the fragment and lanes 32..63 columns 16..31
        const auto s02 = __builtin_amdgcn_permlane32_swap(qrow[0], qrow[2], false, false);
        const auto s13 = __builtin_amdgcn_permlane32_swap(qrow[1], qrow[3], false, false);
        const int n = n_blk + 32 * ca + 16 * fh;
        if (row_ok && 32 * ca + 12 * fh < lim) *reinterpret_cast<v4i *>(o.q + m * o.N + n) = (v4i){(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
    }
}

}  // namespace resident
}  // namespace flexiq
