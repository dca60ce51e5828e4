// Fused dequantizing epilogue shared by the convolution kernels.
//
// Algorithm 1 steps 4-5 of the paper convolve the dequantized tensors
// a_hat = l_a + Da*ca and w_hat = l_w + Dw*cw with zero padding.  Expanding
// the product over the taps that lie inside the image gives
//   out = Da*Dw*ACC + l_a*Dw*SW + l_w*Da*SA + KV*l_a*l_w
// with ACC = sum ca*cw (the integer GEMM), SA = sum ca, SW = sum cw and KV the
// number of (tap, channel) pairs, all over in-image taps only.  The four terms
// are combined in binary64 (terms 1 and 3 nearly cancel for symmetric weight
// ranges) and the sum is rounded once to binary32.  Every kernel evaluates
//   fma(Da*Dw, ACC, (Da*l_w)*SA)  [+ (l_a*Dw)*SW + KV*(l_a*l_w)]
// in this order, so all store paths give identical bits.
#pragma once
#include "dsq_device.h"
#include "dsq_kernels.h"

struct DsqPixel {
    int n, oy, ox;
    int sa;        // sum of activation codes over in-image taps, all channels
    int tapmask;   // bit t set: tap t lies inside the image
    int ntaps;     // popcount(tapmask)
    bool valid;    // m < M
};

__device__ __forceinline__ DsqPixel dsq_pixel_info(const DsqConvArgs &a, int m, int M)
{
    DsqPixel p;
    p.valid = m < M;
    p.sa = 0; p.tapmask = 0; p.ntaps = 0;
    int mm = p.valid ? m : 0;
    p.ox = mm % a.Wo;
    int t = mm / a.Wo;
    p.oy = t % a.Ho;
    p.n = t / a.Ho;
    if (p.valid) {
        for (int r = 0; r < a.R; ++r)
            for (int s = 0; s < a.R; ++s) {
                int iy = p.oy * a.stride - a.pad + r, ix = p.ox * a.stride - a.pad + s;
                if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) {
                    p.sa += a.pix_sum[((size_t)p.n * a.H + iy) * a.W + ix];
                    p.tapmask |= 1 << (r * a.R + s);
                    ++p.ntaps;
                }
            }
    }
    return p;
}

// The binary32 results of one lane: one pixel, four consecutive output channels
// o0..o0+3 (o0 % 4 == 0, o0 + 3 < Cop).
__device__ __forceinline__ void dsq_out4(const DsqConvArgs &a, const DsqPixel &p, int o0, v4i acc,
                                         float delta_a, float (&res)[4])
{
    const float4 dw = *reinterpret_cast<const float4 *>(a.delta_w + o0);
    const float4 lw = *reinterpret_cast<const float4 *>(a.l_w + o0);
    const float dwv[4] = {dw.x, dw.y, dw.z, dw.w};
    const float lwv[4] = {lw.x, lw.y, lw.z, lw.w};
    const int accv[4] = {acc.x, acc.y, acc.z, acc.w};
    const int T = a.R * a.R;
    const bool full = p.ntaps == T;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double da = (double)delta_a, dwj = (double)dwv[j], lwj = (double)lwv[j];
        double v = __builtin_fma(da * dwj, (double)accv[j], (da * lwj) * (double)p.sa);
        if (a.l_a != 0.0f) {
            int sw;
            if (full) sw = a.sw_total[o0 + j];
            else {
                sw = 0;
                for (int t = 0; t < T; ++t)
                    if (p.tapmask >> t & 1) sw += a.sw_tap[(size_t)(o0 + j) * T + t];
            }
            const double la = (double)a.l_a;
            v += (la * dwj) * (double)sw + (double)(a.C_in * p.ntaps) * (la * lwj);
        }
        res[j] = (float)v;
    }
}

// Stores the results of one lane: one pixel, four consecutive output channels
// o0..o0+3 (o0 % 4 == 0, o0 + 3 < Cop).
__device__ __forceinline__ void dsq_store4(const DsqConvArgs &a, const DsqPixel &p, int m, int o0,
                                           v4i acc, float delta_a)
{
    if (!p.valid || o0 >= a.C_out) return;
    const int accv[4] = {acc.x, acc.y, acc.z, acc.w};
    float res[4];
    dsq_out4(a, p, o0, acc, delta_a, res);
    if (!a.out_nchw) {
        const size_t base = (size_t)m * a.C_out + o0;
        if ((a.C_out & 3) == 0) {
            *reinterpret_cast<float4 *>(a.out + base) = make_float4(res[0], res[1], res[2], res[3]);
            if (a.acc) *reinterpret_cast<v4i *>(a.acc + base) = acc;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (o0 + j < a.C_out) {
                    a.out[base + j] = res[j];
                    if (a.acc) a.acc[base + j] = accv[j];
                }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (o0 + j < a.C_out) {
                const size_t idx = (((size_t)p.n * a.C_out + o0 + j) * a.Ho + p.oy) * a.Wo + p.ox;
                a.out[idx] = res[j];
                if (a.acc) a.acc[idx] = accv[j];
            }
    }
}

// ---- chained mode: the next layer's codes instead of the fp32 tensor --------
//
// The next layer's Algorithm 1 steps 1 and 3 applied to this layer's output:
// z = y*scale[o] + shift[o] (two binary32 roundings), optional ReLU, then the
// uniform quantizer with the next layer's range.

// Codes of four consecutive channels o0..o0+3 from their fp32 results y and the
// channels' scale / shift, one code per byte; channels >= C_out give code 0.
// Adds the codes to `sum`.
__device__ __forceinline__ uint32_t dsq_requant4(const DsqConvArgs &a, int o0, const float (&y)[4],
                                                 const float (&sc)[4], const float (&sh)[4],
                                                 float delta_n, int top_n, int &sum)
{
    int c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float z = y[j] * sc[j];
        z = z + sh[j];
        if (a.rq_relu) z = fmaxf(z, 0.0f);
        c[j] = o0 + j < a.C_out ? dsq_code(z, a.rq_l, a.rq_u, delta_n, top_n) : 0;
        sum += c[j];
    }
    return dsq_bytes4(c[0], c[1], c[2], c[3]);
}

// Codes of four consecutive channels from their fp32 results, one per byte.
// relu_floor is 0 with ReLU and -inf without (max(z, -inf) = z; a NaN becomes
// -inf, which has code 0 like the NaN itself); byte_mask blanks the bytes of
// channels >= C_out.
__device__ __forceinline__ uint32_t dsq_requant4_thr(const float (&y)[4], const float (&sc)[4],
                                                     const float (&sh)[4], float relu_floor, float l_n,
                                                     float u_n, float inv_delta, int top_n,
                                                     const float2 *thr_pairs, uint32_t byte_mask)
{
    int c[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float z = y[j] * sc[j];
        z = z + sh[j];
        z = fmaxf(z, relu_floor);
        c[j] = dsq_code_thr<false>(z, l_n, u_n, inv_delta, top_n, 0.f, 0.f, 0.f, thr_pairs);
    }
    return dsq_bytes4(c[0], c[1], c[2], c[3]) & byte_mask;
}

// Packs and stores one pixel's 32 channels [o_tile, o_tile + 32) of the next
// layer's input.  In the accumulator layout of the 32x32x32 matrix instruction
// lane L (pixel L%32, h = L/32) holds channels o_tile + 8q + 4h + 0..3 for
// q = 0..3; bytes[q] carries their codes one per byte.  Lanes L and L^32 hold
// the two halves of every 8-channel word and swap them; the h = 0 lane then
// stores the 16 (4-bit containers), 12 (dense 3-bit) or 8 (2-bit) bytes of the pixel.  Must be
// called by all 64 lanes; `m` < 0 marks a lane without a pixel.  Returns, in
// the h = 0 lane, the pixel's code sum over these 32 channels.
__device__ __forceinline__ int dsq_requant_store32(const DsqConvArgs &a, int m, int o_tile, int h,
                                                   const uint32_t (&bytes)[4], int sum)
{
    // (v_permlane32_swap exchanges the upper half of its first operand with the lower
    // half of its second: element 1 of the result holds, in lanes 0..31, the values
    // of lanes 32..63)
    uint32_t other[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) other[q] = __builtin_amdgcn_permlane32_swap(bytes[q], bytes[q], false, false)[1];
    const int total = sum + (int)__builtin_amdgcn_permlane32_swap((uint32_t)sum, (uint32_t)sum, false, false)[1];
    if (h == 0 && m >= 0 && o_tile < a.rq_Cp) {
        char *dst = (char *)a.rq_codes;
        if (a.rq_dense) {
            // dense 3-bit: the pixel's 32 channels are one 12-byte unit; group 2q is this
            // lane's bytes[q], group 2q+1 its partner's
            const uint32_t d[8] = {bytes[0], other[0], bytes[1], other[1], bytes[2], other[2], bytes[3], other[3]};
            uint32_t l0, l1, hi;
            dsq_pack32_d3(d, l0, l1, hi);
            uint32_t *w = reinterpret_cast<uint32_t *>(dst + ((size_t)m * a.rq_Cp + o_tile) / 32 * 12);
            w[0] = l0; w[1] = l1; w[2] = hi;
        } else if (dsq_container(a.rq_bits) == 4) {
            // word q = channels 8q..8q+7: byte j = c[j] | c[j+4] << 4
            const v4i w = {(int)(bytes[0] | other[0] << 4), (int)(bytes[1] | other[1] << 4),
                           (int)(bytes[2] | other[2] << 4), (int)(bytes[3] | other[3] << 4)};
            *reinterpret_cast<v4i *>(dst + ((size_t)m * a.rq_Cp + o_tile) / 2) = w;
        } else {
            // word = 16 channels: byte j = c[j] | c[j+4] << 2 | c[j+8] << 4 | c[j+12] << 6
            const v2i w = {(int)(bytes[0] | other[0] << 2 | bytes[1] << 4 | other[1] << 6),
                           (int)(bytes[2] | other[2] << 2 | bytes[3] << 4 | other[3] << 6)};
            *reinterpret_cast<v2i *>(dst + ((size_t)m * a.rq_Cp + o_tile) / 4) = w;
        }
    }
    return total;
}

// Four consecutive channels o0..o0+3 of one pixel through the general formulas
// (any l_a, any border): accumulators -> fp32 results -> the next layer's
// codes, one per byte; adds the codes to `sum`.  o0 < Cop: the side tables cover it.
__device__ __forceinline__ uint32_t dsq_requant_quarter(const DsqConvArgs &a, const DsqPixel &px, int o0, v4i acc,
                                                        float delta_a, float delta_n, int top_n, int &sum)
{
    float y[4], sc[4], sh[4];
    dsq_out4(a, px, o0, acc, delta_a, y);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool in = o0 + j < a.C_out;
        sc[j] = in && a.rq_scale ? a.rq_scale[o0 + j] : 1.0f;
        sh[j] = in && a.rq_shift ? a.rq_shift[o0 + j] : 0.0f;
    }
    return dsq_requant4(a, o0, y, sc, sh, delta_n, top_n, sum);
}

// One whole 32-channel tile of one pixel.  All 64 lanes must call it.
__device__ __forceinline__ int dsq_requant_tile(const DsqConvArgs &a, const DsqPixel &px, int m, int o_tile,
                                                int h, const v16i &acc, float delta_a)
{
    const int top_n = (1 << a.rq_bits) - 1;
    const float delta_n = dsq_delta(a.rq_l, a.rq_u, top_n);
    uint32_t bytes[4];
    int sum = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        bytes[q] = dsq_requant_quarter(a, px, o_tile + 8 * q + 4 * h,
                                       (v4i){acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]}, delta_a,
                                       delta_n, top_n, sum);
    return dsq_requant_store32(a, px.valid ? m : -1, o_tile, h, bytes, sum);
}
