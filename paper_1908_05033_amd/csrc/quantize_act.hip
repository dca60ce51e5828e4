// dsq_quantize_act kernels: clip + round activations to b-bit codes (paper
// Algorithm 1 steps 1 and 3, i.e. the uniform quantizer of Sec. 3.1), pack
// them sub-byte and emit the per-pixel code sums the convolution epilogue
// needs for the l_w zero-point term.
//
// The kernel is bound by HBM traffic (4 B read and container/8 B written per
// element); the only arithmetic of note is the IEEE division of the recipe.
#include "dsq_device.h"
#include "dsq_kernels.h"

namespace {

template <int DPP_CTRL>
__device__ __forceinline__ int dpp_add(int v)
{
    return v + __builtin_amdgcn_update_dpp(0, v, DPP_CTRL, 0xF, 0xF, true);
}

// Codes of up to four consecutive channels starting at c0 -> one byte each.
// VEC: the pixel's channel count is a multiple of 4 and x is 16-B aligned, so
// a group of four is either wholly inside [0,C) or wholly outside.
template <bool VEC>
__device__ __forceinline__ uint32_t quant4(const float *px, int c0, int C, float l, float u,
                                           float delta, int top)
{
    float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
    bool in0, in1, in2, in3;
    if (VEC) {
        in0 = in1 = in2 = in3 = c0 < C;
        if (in0) {
            float4 f = *reinterpret_cast<const float4 *>(px + c0);
            v0 = f.x; v1 = f.y; v2 = f.z; v3 = f.w;
        }
    } else {
        in0 = c0 < C; in1 = c0 + 1 < C; in2 = c0 + 2 < C; in3 = c0 + 3 < C;
        if (in0) v0 = px[c0];
        if (in1) v1 = px[c0 + 1];
        if (in2) v2 = px[c0 + 2];
        if (in3) v3 = px[c0 + 3];
    }
    int q0 = in0 ? dsq_code(v0, l, u, delta, top) : 0;
    int q1 = in1 ? dsq_code(v1, l, u, delta, top) : 0;
    int q2 = in2 ? dsq_code(v2, l, u, delta, top) : 0;
    int q3 = in3 ? dsq_code(v3, l, u, delta, top) : 0;
    return dsq_bytes4(q0, q1, q2, q3);
}

// NHWC input.  One thread produces one packed word (8 channels at 4-bit, 16 at
// 2-bit).  A block owns PB whole pixels, so pixel sums never straddle blocks.
// Because a pixel is a multiple of 8 (4-bit) or 4 (2-bit) words long and the
// block starts on a pixel, every aligned group of 8 (4) lanes works on one
// pixel: their code sums are combined with DPP adds before one lane either
// stores the pixel sum (one group per pixel) or adds it into LDS.
template <int CONT, bool VEC>
__global__ __launch_bounds__(256) void quantize_act_nhwc_kernel(
    const float *__restrict__ x, uint32_t *__restrict__ codes, int32_t *__restrict__ pix_sum,
    int total_pixels, int C, int DP, int dp_shift, int PB, float l, float u, int top)
{
    constexpr int CPD = 32 / CONT;           // channels per packed word
    constexpr int GROUP = CPD == 8 ? 8 : 4;  // lanes that surely share a pixel
    __shared__ int spix[DSQ_QUANT_MAX_PB];

    const int tid = threadIdx.x;
    const int pixel0 = blockIdx.x * PB;
    const int npix = min(PB, total_pixels - pixel0);
    const bool multi_group = DP != GROUP;
    if (multi_group) {
        for (int i = tid; i < npix; i += 256) spix[i] = 0;
        __syncthreads();
    }
    const float delta = dsq_delta(l, u, top);
    const int ndw = npix * DP;
    const int ndw_up = (ndw + 255) & ~255;   // all lanes take part in the DPP adds

    for (int i = tid; i < ndw_up; i += 256) {
        const bool active = i < ndw;
        const int p = dp_shift >= 0 ? (i >> dp_shift) : (i / DP);
        const int d = i - p * DP;
        const int c0 = d * CPD;
        uint32_t word = 0;
        int s = 0;
        if (active) {
            const float *px = x + (size_t)(pixel0 + p) * C;
            if (CONT == 4) {
                uint32_t lo = quant4<VEC>(px, c0, C, l, u, delta, top);
                uint32_t hi = quant4<VEC>(px, c0 + 4, C, l, u, delta, top);
                word = dsq_pack8x4(lo, hi);
                s = dsq_bytesum(lo) + dsq_bytesum(hi);
            } else {
                uint32_t b0 = quant4<VEC>(px, c0, C, l, u, delta, top);
                uint32_t b1 = quant4<VEC>(px, c0 + 4, C, l, u, delta, top);
                uint32_t b2 = quant4<VEC>(px, c0 + 8, C, l, u, delta, top);
                uint32_t b3 = quant4<VEC>(px, c0 + 12, C, l, u, delta, top);
                word = b0 | (b1 << 2) | (b2 << 4) | (b3 << 6);
                s = dsq_bytesum(b0) + dsq_bytesum(b1) + dsq_bytesum(b2) + dsq_bytesum(b3);
            }
            codes[(size_t)(pixel0 + p) * DP + d] = word;
        }
        s = dpp_add<0xB1>(s);                    // lanes ^1   (quad_perm 1,0,3,2)
        s = dpp_add<0x4E>(s);                    // lanes ^2   (quad_perm 2,3,0,1)
        if (GROUP == 8) s = dpp_add<0x141>(s);   // other quad (row_half_mirror)
        if (active && (tid & (GROUP - 1)) == 0) {
            if (multi_group) atomicAdd(&spix[p], s);
            else pix_sum[pixel0 + p] = s;
        }
    }
    if (multi_group) {
        __syncthreads();
        for (int i = tid; i < npix; i += 256) pix_sum[pixel0 + i] = spix[i];
    }
}

// NCHW input.  Lanes run along the pixels of one image plane (contiguous in
// memory for a fixed channel), the four waves of a block take every fourth
// packed word of those pixels.
template <int CONT>
__global__ __launch_bounds__(256) void quantize_act_nchw_kernel(
    const float *__restrict__ x, uint32_t *__restrict__ codes, int32_t *__restrict__ pix_sum,
    int C, int HW, int DP, float l, float u, int top)
{
    constexpr int CPD = 32 / CONT;
    __shared__ int ssum[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hw = blockIdx.x * 64 + lane;
    const int n = blockIdx.y;
    const bool active = hw < HW;
    const float delta = dsq_delta(l, u, top);
    int s = 0;
    if (active) {
        const float *xn = x + (size_t)n * C * HW + hw;
        uint32_t *crow = codes + ((size_t)n * HW + hw) * DP;
        for (int d = wave; d < DP; d += 4) {
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < CPD; ++j) {
                int c = d * CPD + j;
                int q = 0;
                if (c < C) q = dsq_code(xn[(size_t)c * HW], l, u, delta, top);
                s += q;
                // channel j of the word sits in byte j%4 at bit offset CONT*(j/4)
                word |= (uint32_t)q << (8 * (j & 3) + CONT * (j >> 2));
            }
            crow[d] = word;
        }
    }
    ssum[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && active)
        pix_sum[(size_t)n * HW + hw] = ssum[0][lane] + ssum[1][lane] + ssum[2][lane] + ssum[3][lane];
}

}  // namespace

hipError_t dsq_launch_quantize_act(const float *x, int layout_nchw, int N, int C, int H, int W,
                                   float l, float u, int bits, void *codes, int32_t *pix_sum,
                                   hipStream_t stream)
{
    const int cont = dsq_container(bits);
    const int top = (1 << bits) - 1;
    const int Cp = dsq_round_up(C, 64);
    const int DP = Cp * cont / 32;
    const int total_pixels = N * H * W;
    if (layout_nchw) {
        dim3 grid((H * W + 63) / 64, N);
        if (cont == 4)
            quantize_act_nchw_kernel<4><<<grid, 256, 0, stream>>>(x, (uint32_t *)codes, pix_sum, C,
                                                                  H * W, DP, l, u, top);
        else
            quantize_act_nchw_kernel<2><<<grid, 256, 0, stream>>>(x, (uint32_t *)codes, pix_sum, C,
                                                                  H * W, DP, l, u, top);
        return hipGetLastError();
    }
    // Words per thread: few for small tensors (enough blocks to cover the
    // chip), more for large ones (more loads in flight per thread).
    const long long total_dw = (long long)total_pixels * DP;
    int iters = 8;
    while (iters > 1 && total_dw / (256LL * iters) < 2048) iters >>= 1;
    int PB = (256 * iters) / DP;
    if (PB < 1) PB = 1;
    if (PB > DSQ_QUANT_MAX_PB) PB = DSQ_QUANT_MAX_PB;
    int dp_shift = -1;
    if ((DP & (DP - 1)) == 0) { dp_shift = 0; while ((1 << dp_shift) < DP) ++dp_shift; }
    const bool vec = (C % 4 == 0) && (((uintptr_t)x & 15) == 0);
    dim3 grid((total_pixels + PB - 1) / PB);
#define DSQ_Q_LAUNCH(CONT, VEC)                                                              \
    quantize_act_nhwc_kernel<CONT, VEC><<<grid, 256, 0, stream>>>(                           \
        x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, dp_shift, PB, l, u, top)
    if (cont == 4) { if (vec) DSQ_Q_LAUNCH(4, true); else DSQ_Q_LAUNCH(4, false); }
    else           { if (vec) DSQ_Q_LAUNCH(2, true); else DSQ_Q_LAUNCH(2, false); }
#undef DSQ_Q_LAUNCH
    return hipGetLastError();
}
