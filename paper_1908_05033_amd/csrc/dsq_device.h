// Device-side helpers shared by the libdsqconv kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Container width in bits for a given code width: 3-bit codes travel in
// 4-bit containers, 1-bit codes (the binary case) in 2-bit containers.
__host__ __device__ constexpr int dsq_container(int bits) { return bits <= 2 ? 2 : 4; }
__host__ __device__ constexpr int dsq_round_up(int x, int m) { return (x + m - 1) / m * m; }

// Uniform quantizer of the paper's Sec. 3.1 with clip range [l,u]; a value at
// an interval midpoint goes to the upper level (sgn(0)=+1 applied at m_i,
// Sec. 3.2 / Algorithm 1 step 3).  Every operation is one IEEE binary32
// operation; '/' is the correctly rounded division (hipcc's default for HIP).
__device__ __forceinline__ float dsq_delta(float l, float u, int top)
{
    return (u - l) / (float)top;
}

__device__ __forceinline__ int dsq_code(float x, float l, float u, float delta, int top)
{
    float v = fminf(fmaxf(x, l), u);   // NaN -> l
    float t = (v - l) / delta;
    int c = (int)floorf(t + 0.5f);
    return min(max(c, 0), top);
}

// The quantizer as a step function.  Every operation of dsq_code (clip,
// subtract, divide by Delta > 0, add 1/2, floor) is monotone non-decreasing in x,
// so code(x) = #{j : x >= thr[j]} where thr[j] is the smallest binary32 value
// whose code is >= j; the host finds these thresholds by bisection over the
// ordered floats with the same recipe.  Written without branches.  LINEAR (at most three thresholds): a chain of
// compares.  Otherwise: a first guess from one multiply-add, corrected against
// the two thresholds around it, which `thr_pairs` holds as (thr[c], thr[c+1]) for
// c = 0..15 (-inf below the first, NaN above the last: nothing, not even +inf,
// compares >= NaN).
template <bool LINEAR>
__device__ __forceinline__ int dsq_code_thr(float z, float l_n, float u_n, float inv_delta, int top_n,
                                            float t1, float t2, float t3, const float2 *thr_pairs)
{
    if (LINEAR) return (z >= t1) + (z >= t2) + (z >= t3);
    const float v = fminf(fmaxf(z, l_n), u_n);                       // NaN -> l, as in dsq_code
    const int c0 = min((int)((v - l_n) * inv_delta + 0.5f), top_n);  // >= 0: v >= l
    const float2 t = thr_pairs[c0];
    return c0 + (z >= t.y) - (z < t.x);
}

// Four codes -> one word with one code per byte.
__device__ __forceinline__ uint32_t dsq_bytes4(int c0, int c1, int c2, int c3)
{
    return (uint32_t)c0 | ((uint32_t)c1 << 8) | ((uint32_t)c2 << 16) | ((uint32_t)c3 << 24);
}

// 4-bit container: 8 consecutive channels per word, byte j = c[j] | c[j+4]<<4.
__device__ __forceinline__ uint32_t dsq_pack8x4(uint32_t lo_bytes, uint32_t hi_bytes)
{
    return lo_bytes | (hi_bytes << 4);
}

// Unpack one 4-bit word into channels 0..3 (lo) and 4..7 (hi), one per byte.
__device__ __forceinline__ void dsq_unpack4(uint32_t w, uint32_t &lo, uint32_t &hi)
{
    lo = w & 0x0F0F0F0Fu;
    hi = (w >> 4) & 0x0F0F0F0Fu;
}

// Unpack one 2-bit word (16 channels) into four words of four int8 each.
__device__ __forceinline__ v4i dsq_unpack2(uint32_t w)
{
    v4i r;
    r.x = (int)(w & 0x03030303u);
    r.y = (int)((w >> 2) & 0x03030303u);
    r.z = (int)((w >> 4) & 0x03030303u);
    r.w = (int)((w >> 6) & 0x03030303u);
    return r;
}

// 16 consecutive channels of one lane's MFMA operand from their packed form:
// two words at 4-bit, one word at 2-bit.
__device__ __forceinline__ v4i dsq_unpack16_c4(v2i p)
{
    v4i r;
    uint32_t a, b;
    dsq_unpack4((uint32_t)p.x, a, b);
    r.x = (int)a; r.y = (int)b;
    dsq_unpack4((uint32_t)p.y, a, b);
    r.z = (int)a; r.w = (int)b;
    return r;
}

// ---- dense 3-bit activation codes ---------------------------------------------
//
// 32 consecutive channels c0..c31 of a pixel occupy 12 bytes: word 0 / word 1 hold
// the low two bits of channels 0..15 / 16..31 in the 2-bit container format
// (byte j = lo(c[j]) | lo(c[j+4]) << 2 | lo(c[j+8]) << 4 | lo(c[j+12]) << 6), word 2
// the high bits: bit 8j + g = bit 2 of channel 4g + j (j = 0..3, g = 0..7).
// Group g (channels 4g..4g+3, one code per byte) is therefore
//   ((low_word >> 2(g%4)) & 0x03030303) | (((high_word >> g) & 0x01010101) << 2).

// The eight groups of one 12-byte unit as int8 words, in channel order.
__device__ __forceinline__ void dsq_unpack32_d3(uint32_t l0, uint32_t l1, uint32_t hi, uint32_t (&d)[8])
{
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const uint32_t low = ((g < 4 ? l0 : l1) >> (2 * (g & 3))) & 0x03030303u;
        const uint32_t high = (g >= 2 ? hi >> (g - 2) : hi << (2 - g)) & 0x04040404u;
        d[g] = low | high;
    }
}

// The inverse: eight groups (codes < 8, one per byte) -> the three words of a unit.
__device__ __forceinline__ void dsq_pack32_d3(const uint32_t (&d)[8], uint32_t &l0, uint32_t &l1, uint32_t &hi)
{
    l0 = (d[0] & 0x03030303u) | (d[1] & 0x03030303u) << 2 | (d[2] & 0x03030303u) << 4 | (d[3] & 0x03030303u) << 6;
    l1 = (d[4] & 0x03030303u) | (d[5] & 0x03030303u) << 2 | (d[6] & 0x03030303u) << 4 | (d[7] & 0x03030303u) << 6;
    hi = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) hi |= ((d[g] >> 2) & 0x01010101u) << g;
}

// Sum of the four bytes of a word whose bytes are all < 64.
__device__ __forceinline__ int dsq_bytesum(uint32_t w)
{
    uint32_t s = (w & 0x00FF00FFu) + ((w >> 8) & 0x00FF00FFu);
    return (int)((s + (s >> 16)) & 0xFFFFu);
}

// ---- 2-bit layers on the FP4 matrix instruction ------------------------------
//
// A 2-bit code c in {0,1,2,3}, zero-extended to four bits, is the FP4 (e2m1)
// encoding of c/2 (0, 0.5, 1.0, 1.5).  v_mfma_f32_32x32x64_f8f6f4 on such
// operands therefore returns sum(ca*cw)/4 -- exactly: every product is a multiple
// of 1/4 below 2.25 and the sums stay far below 2^24 quarter units -- at twice the
// K per instruction of the int8 form and without any unpacking of the weights.
// Lane L supplies row/column L%32 and the 32 K values of K group L/32 as 32
// nibbles (16 bytes); results come back in the int8 instruction's layout.

// 32 two-bit codes in the packed activation format (two words, channels 0..15 and
// 16..31 of a K group) -> the lane's 128-bit FP4 operand.  Word d nibble n of the
// result holds channel 16*(d/2) + 4*(d%2) + 8*(n%2) + n/2; dsq_pack_weights lays
// 2-bit weights out in the same order.
__device__ __forceinline__ v4i dsq_fp4_from_c2(uint32_t w0, uint32_t w1)
{
    v4i r;
    r.x = (int)(w0 & 0x33333333u);
    r.y = (int)((w0 >> 2) & 0x33333333u);
    r.z = (int)(w1 & 0x33333333u);
    r.w = (int)((w1 >> 2) & 0x33333333u);
    return r;
}

// acc + (a . b) / 4 over the 64 K values the two 128-bit FP4 operands hold.
__device__ __forceinline__ v16f dsq_mfma_fp4(v4i a, v4i b, v16f acc)
{
    const v8i a8 = {a.x, a.y, a.z, a.w, 0, 0, 0, 0}, b8 = {b.x, b.y, b.z, b.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc, 4, 4, 0, 0, 0, 0);
}

// The integer sums behind a quarter-unit accumulator.
__device__ __forceinline__ v16i dsq_fp4_acc_to_int(v16f acc)
{
    v16i r;
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = (int)(acc[i] * 4.0f);
    return r;
}
