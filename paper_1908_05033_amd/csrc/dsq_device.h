// Device-side helpers shared by the libdsqconv kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Container width in bits for a given code width: 3-bit codes travel in
// 4-bit containers.
__host__ __device__ constexpr int dsq_container(int bits) { return bits == 2 ? 2 : 4; }
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

// Sum of the four bytes of a word whose bytes are all < 64.
__device__ __forceinline__ int dsq_bytesum(uint32_t w)
{
    uint32_t s = (w & 0x00FF00FFu) + ((w >> 8) & 0x00FF00FFu);
    return (int)((s + (s >> 16)) & 0xFFFFu);
}
