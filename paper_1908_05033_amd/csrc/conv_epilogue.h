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

// Stores the results of one lane: one pixel, four consecutive output channels
// o0..o0+3 (o0 % 4 == 0, o0 + 3 < Cop).
__device__ __forceinline__ void dsq_store4(const DsqConvArgs &a, const DsqPixel &p, int m, int o0,
                                           v4i acc, float delta_a)
{
    if (!p.valid || o0 >= a.C_out) return;
    const float4 dw = *reinterpret_cast<const float4 *>(a.delta_w + o0);
    const float4 lw = *reinterpret_cast<const float4 *>(a.l_w + o0);
    const float dwv[4] = {dw.x, dw.y, dw.z, dw.w};
    const float lwv[4] = {lw.x, lw.y, lw.z, lw.w};
    const int accv[4] = {acc.x, acc.y, acc.z, acc.w};
    const int T = a.R * a.R;
    const bool full = p.ntaps == T;
    float res[4];
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
