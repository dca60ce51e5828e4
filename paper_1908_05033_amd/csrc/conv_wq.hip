// dsq_conv2d_wq: a layer whose weights are quantized and whose activations are not
// (the "b/32" rows of the paper's Tables 3, 6 and 7: b-bit weights, 32-bit
// activations).  Algorithm 1 steps 4 and 5 with a_hat = a: the weight codes are
// turned back into their levels l_w + Dw*code, one binary32 rounding each, and
// convolved with the binary32 activations on the fp32 matrix instruction
// (v_mfma_f32_32x32x2_f32: products are not rounded, sums are accumulated in
// binary32).  There is no integer path here: the inner product is a
// floating-point contraction, which is why this is a kernel of its own.
//
// One wave per tile of 32 output pixels x 32 output channels, operands straight
// from global memory: rows of the first operand are output channels (the packed
// 4-bit weight layout of dsq_pack_weights_for(.., bits_w, 4, ..): a lane holds
// the 16 channels 64cb + 32kh + 16h + 0..15 of its row), columns of the second
// are pixels, and a lane walks its 16 channels one matrix instruction (K = 2:
// one channel per lane half) at a time.
#include "dsq_device.h"
#include "dsq_kernels.h"

namespace {

typedef float v16f_t __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void conv_wq_kernel(DsqConvArgs a, const float *__restrict__ x, int x_nchw)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, h = lane >> 5;
    const int M = a.N * a.Ho * a.Wo;
    const int m = blockIdx.x * 32 + col;
    const int ct = blockIdx.y * 4 + wave;
    if (ct * 32 >= a.C_out) return;                     // (uniform per wave)
    const int T = a.R * a.R;
    const int NCB = a.Cp / 64;
    const bool valid = m < M;
    const int mm = valid ? m : 0;
    const int ox = mm % a.Wo, oy = (mm / a.Wo) % a.Ho, n = mm / (a.Wo * a.Ho);
    const int o_row = ct * 32 + col;                    // this lane's weight row (< Cop: the side table covers it)
    const float dw = a.delta_w[o_row], lw = a.l_w[o_row];
    const uint32_t *wq = (const uint32_t *)a.wq;
    const bool vec = !x_nchw && (a.C_in & 3) == 0;

    v16f_t acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    for (int cb = 0; cb < NCB; ++cb) {
        for (int tap = 0; tap < T; ++tap) {
            const int r = tap / a.R, s = tap % a.R;
            const int iy = oy * a.stride - a.pad + r, ix = ox * a.stride - a.pad + s;
            const bool inside = valid && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
            const uint32_t *wp = wq + ((((size_t)ct * NCB + cb) * T + tap) * 64 + lane) * 4;
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                const int c0 = 64 * cb + 32 * kh + 16 * h;      // this lane's 16 channels
                float av[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) av[j] = 0.f;       // padding and channels >= C_in: the real number 0
                if (inside) {
                    if (vec) {
                        const float *p = x + (((size_t)n * a.H + iy) * a.W + ix) * a.C_in + c0;
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (c0 + 4 * q < a.C_in) {
                                const float4 t = *reinterpret_cast<const float4 *>(p + 4 * q);
                                av[4 * q] = t.x; av[4 * q + 1] = t.y; av[4 * q + 2] = t.z; av[4 * q + 3] = t.w;
                            }
                    } else {
#pragma unroll
                        for (int j = 0; j < 16; ++j)
                            if (c0 + j < a.C_in)
                                av[j] = x_nchw ? x[(((size_t)n * a.C_in + c0 + j) * a.H + iy) * a.W + ix]
                                               : x[(((size_t)n * a.H + iy) * a.W + ix) * a.C_in + c0 + j];
                    }
                }
                // the 16 weight codes of this half: two words of the 4-bit container format
                uint32_t b[4];
                dsq_unpack4(wp[2 * kh], b[0], b[1]);
                dsq_unpack4(wp[2 * kh + 1], b[2], b[3]);
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const float code = (float)((b[j >> 2] >> (8 * (j & 3))) & 0xFFu);
                    const float level = __builtin_fmaf(dw, code, lw);          // l_w + Dw*code, rounded once
                    if (j & 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(level, av[j], acc1, 0, 0, 0);
                    else acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(level, av[j], acc0, 0, 0, 0);
                }
            }
        }
    }
    if (!valid) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int o = ct * 32 + 8 * q + 4 * h + j;
            if (o < a.C_out) {
                const float v = acc0[4 * q + j] + acc1[4 * q + j];
                if (a.out_nchw) a.out[(((size_t)n * a.C_out + o) * a.Ho + oy) * a.Wo + ox] = v;
                else a.out[(size_t)m * a.C_out + o] = v;
            }
        }
}

}  // namespace

hipError_t dsq_launch_conv_wq(const DsqConvArgs &a, const float *x, int x_nchw, hipStream_t stream)
{
    const int M = a.N * a.Ho * a.Wo;
    dim3 grid((M + 31) / 32, (a.C_out + 127) / 128);
    conv_wq_kernel<<<grid, 256, 0, stream>>>(a, x, x_nchw);
    return hipGetLastError();
}
