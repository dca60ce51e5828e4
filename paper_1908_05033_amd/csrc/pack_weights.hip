// dsq_pack_weights kernel: quantize OIHW float weights per output channel
// (paper Algorithm 1 steps 1 and 3 on the weight side; the uniform quantizer
// of Sec. 3.1) and lay the codes out in the order in which the convolution
// kernels feed them to the matrix cores.  Runs once per layer; not tuned.
#include "dsq_device.h"
#include "dsq_kernels.h"

namespace {

// One block per (padded) output channel o.  Output words of that channel:
// (cb, tap, kh, h, dd) -> 8 (4-bit) or 16 (2-bit) consecutive input channels
// starting at 64*cb + 32*kh + 16*h + 8*dd.  In memory the words of one
// (32-channel tile, cb, tap) block are ordered [lane = 32*h + o%32][kh][dd], so
// that a lane of the 32x32x32 MFMA finds its two K halves in 16 adjacent bytes.
//
// 2-bit layers (CONT == 2) feed the FP4 matrix instruction instead: one code per
// 4-bit field, per lane the 32 channels 64*cb + 32*h + .. of its K group in 16
// bytes, ordered [lane = 32*h + o%32][word d]; word d nibble n holds channel
// offset 16*(d/2) + 4*(d%2) + 8*(n%2) + n/2 -- the order in which the kernels
// spread packed 2-bit activation words into nibbles (dsq_fp4_from_c2).
template <int CONT>
__global__ __launch_bounds__(256) void pack_weights_kernel(
    const float *__restrict__ w, const float *__restrict__ l_w, const float *__restrict__ u_w,
    const uint8_t *__restrict__ codes, int C_out, int C_in, int T, int Cop, int top,
    uint32_t *__restrict__ wq, float *__restrict__ aux_delta, float *__restrict__ aux_l,
    int32_t *__restrict__ aux_total, int32_t *__restrict__ aux_tap)
{
    constexpr int CPD = 32 / CONT;      // channels per word
    constexpr int WPL = 16 / CPD;       // words per lane per K half: 2 or 1
    __shared__ int stap[16];
    const int o = blockIdx.x;
    const int tid = threadIdx.x;
    const int NCB = dsq_round_up(C_in, 64) / 64;
    const bool real = o < C_out;
    if (tid < 16) stap[tid] = 0;
    __syncthreads();

    float l = 0.f, u = 0.f, delta = 0.f;
    if (real) {
        l = l_w[o];
        u = u_w[o];
        // A range that is not finite or not l<u has no levels: mark it.
        const bool ok = (l < u) && (fabsf(l) <= 3.4028234e38f) && (fabsf(u) <= 3.4028234e38f);
        delta = ok ? dsq_delta(l, u, top) : __builtin_nanf("");
    }
    const int ct = o >> 5, row = o & 31;
    if (CONT == 2) {
        const int nw = NCB * T * 8;
        for (int i = tid; i < nw; i += 256) {
            const int d = i & 3, h = (i >> 2) & 1;
            const int tap = (i >> 3) % T, cb = (i >> 3) / T;
            uint32_t word = 0;
            int s = 0;
            if (real) {
#pragma unroll
                for (int n = 0; n < 8; ++n) {
                    const int c = 64 * cb + 32 * h + 16 * (d >> 1) + 4 * (d & 1) + 8 * (n & 1) + (n >> 1);
                    int q = 0;
                    if (c < C_in) {
                        const size_t src = ((size_t)o * C_in + c) * T + tap;
                        q = codes ? min((int)codes[src], top) : dsq_code(w[src], l, u, delta, top);
                    }
                    s += q;
                    word |= (uint32_t)q << (4 * n);
                }
                if (s) atomicAdd(&stap[tap], s);
            }
            wq[((((size_t)ct * NCB + cb) * T + tap) * 64 + (32 * h + row)) * 4 + d] = word;
        }
    }
    const int nwords = CONT == 2 ? 0 : NCB * T * 4 * WPL;
    for (int i = tid; i < nwords; i += 256) {
        int dd = i % WPL;
        int rest = i / WPL;
        int h = rest & 1; rest >>= 1;
        int kh = rest & 1; rest >>= 1;
        int tap = rest % T;
        int cb = rest / T;
        int c0 = 64 * cb + 32 * kh + 16 * h + CPD * dd;
        uint32_t word = 0;
        int s = 0;
        if (real) {
#pragma unroll
            for (int j = 0; j < CPD; ++j) {
                int c = c0 + j;
                int q = 0;
                if (c < C_in) {
                    size_t src = ((size_t)o * C_in + c) * T + tap;
                    q = codes ? min((int)codes[src], top) : dsq_code(w[src], l, u, delta, top);
                }
                s += q;
                word |= (uint32_t)q << (8 * (j & 3) + CONT * (j >> 2));
            }
            if (s) atomicAdd(&stap[tap], s);
        }
        size_t dst = (((((size_t)ct * NCB + cb) * T + tap) * 64 + (32 * h + row)) * 2 + kh) * WPL + dd;
        wq[dst] = word;
    }
    __syncthreads();
    if (tid < T) aux_tap[(size_t)o * T + tid] = stap[tid];
    if (tid == 0) {
        int tot = 0;
        for (int t = 0; t < T; ++t) tot += stap[t];
        aux_total[o] = tot;
        aux_delta[o] = delta;
        aux_l[o] = l;
    }
}

}  // namespace

hipError_t dsq_launch_pack_weights(const float *w, const float *l_w, const float *u_w,
                                   const uint8_t *codes, int C_out, int C_in, int R, int bits, int cont,
                                   void *w_packed, void *w_aux, hipStream_t stream)
{
    const int top = (1 << bits) - 1;
    const int T = R * R;
    const int Cop = dsq_round_up(C_out, 256);
    float *aux_delta = (float *)w_aux;
    float *aux_l = aux_delta + Cop;
    int32_t *aux_total = (int32_t *)(aux_l + Cop);
    int32_t *aux_tap = aux_total + Cop;
    if (cont == 4)
        pack_weights_kernel<4><<<Cop, 256, 0, stream>>>(w, l_w, u_w, codes, C_out, C_in, T, Cop, top,
                                                        (uint32_t *)w_packed, aux_delta, aux_l,
                                                        aux_total, aux_tap);
    else
        pack_weights_kernel<2><<<Cop, 256, 0, stream>>>(w, l_w, u_w, codes, C_out, C_in, T, Cop, top,
                                                        (uint32_t *)w_packed, aux_delta, aux_l,
                                                        aux_total, aux_tap);
    return hipGetLastError();
}
