// dsq_quantize_act kernels: clip + round activations to b-bit codes (paper
// Algorithm 1 steps 1 and 3, i.e. the uniform quantizer of Sec. 3.1), pack
// them sub-byte and emit the per-pixel code sums the convolution epilogue
// needs for the l_w zero-point term.
//
// The kernels are bound by HBM traffic (4 B read and container/8 B written per
// element).  The NHWC kernels evaluate the recipe in its step-function form
// (thresholds found on the host with the recipe itself: exactly the same codes,
// without the IEEE division, which costs more than the memory time per element);
// the NCHW kernel divides.
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
// The codes come from the step-function form of the quantizer (dsq_code_thr):
// LINEAR for 1- and 2-bit codes, the guess-and-correct form with the (lower,
// upper) threshold pairs `tp` in LDS for 3- and 4-bit codes.
struct QuantParams {
    float l, u, delta, inv_delta, t1, t2, t3;
    int top;
};

// MODE 0: the recipe itself (dsq_code, with its division); 1: compare chain;
// 2: guess and correct against the threshold pairs in LDS.
template <int MODE>
__device__ __forceinline__ int qcode(float x, const QuantParams &q, const float2 *tp)
{
    if (MODE == 0) return dsq_code(x, q.l, q.u, q.delta, q.top);
    return dsq_code_thr<MODE == 1>(x, q.l, q.u, q.inv_delta, q.top, q.t1, q.t2, q.t3, tp);
}

// Threshold pairs of this block: pair c = (thr[c], thr[c+1]), -inf below the first
// threshold, NaN above the last.  Needs a barrier before use.
__device__ __forceinline__ void fill_threshold_pairs(float2 *tp, const DsqThresholds &th)
{
    if (threadIdx.x < 16) {
        float lo = -__builtin_inff(), hi = __builtin_nanf("");
#pragma unroll
        for (int j = 1; j < 16; ++j) {
            lo = (int)threadIdx.x == j ? th.thr[j] : lo;
            hi = (int)threadIdx.x + 1 == j ? th.thr[j] : hi;
        }
        tp[threadIdx.x] = make_float2(lo, hi);
    }
}

template <bool VEC, int MODE>
__device__ __forceinline__ uint32_t quant4(const float *px, int c0, int C, const QuantParams &qp,
                                           const float2 *tp)
{
    if (VEC) {
        // C is a multiple of 4 here.  Branch-free: a group past the last channel
        // reads the pixel's first four values instead and is blanked afterwards,
        // so that all loads of a thread are in flight together.
        const bool in = c0 < C;
        const float4 f = *reinterpret_cast<const float4 *>(px + (in ? c0 : 0));
        const uint32_t b = dsq_bytes4(qcode<MODE>(f.x, qp, tp), qcode<MODE>(f.y, qp, tp),
                                      qcode<MODE>(f.z, qp, tp), qcode<MODE>(f.w, qp, tp));
        return in ? b : 0u;
    }
    const bool in0 = c0 < C, in1 = c0 + 1 < C, in2 = c0 + 2 < C, in3 = c0 + 3 < C;
    float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
    if (in0) v0 = px[c0];
    if (in1) v1 = px[c0 + 1];
    if (in2) v2 = px[c0 + 2];
    if (in3) v3 = px[c0 + 3];
    const int q0 = in0 ? qcode<MODE>(v0, qp, tp) : 0;
    const int q1 = in1 ? qcode<MODE>(v1, qp, tp) : 0;
    const int q2 = in2 ? qcode<MODE>(v2, qp, tp) : 0;
    const int q3 = in3 ? qcode<MODE>(v3, qp, tp) : 0;
    return dsq_bytes4(q0, q1, q2, q3);
}

// NHWC input.  One thread produces one packed word (8 channels at 4-bit, 16 at
// 2-bit).  A block owns PB whole pixels, so pixel sums never straddle blocks.
// Because a pixel is a multiple of 8 (4-bit) or 4 (2-bit) words long and the
// block starts on a pixel, every aligned group of 8 (4) lanes works on one
// pixel: their code sums are combined with DPP adds before one lane either
// stores the pixel sum (one group per pixel) or adds it into LDS.
// THR: use the step-function form of the quantizer (large tensors, where the
// division would cost more than the memory time); small, latency-bound tensors
// keep the recipe itself and save the table set-up.
template <int CONT, bool VEC, bool THR>
__global__ __launch_bounds__(256) void quantize_act_nhwc_kernel(
    const float *__restrict__ x, uint32_t *__restrict__ codes, int32_t *__restrict__ pix_sum,
    int total_pixels, int C, int DP, int dp_shift, int PB, float l, float u, int top, DsqThresholds th)
{
    constexpr int CPD = 32 / CONT;           // channels per packed word
    constexpr int GROUP = CPD == 8 ? 8 : 4;  // lanes that surely share a pixel
    constexpr int MODE = !THR ? 0 : CONT == 2 ? 1 : 2;   // 1- and 2-bit codes: at most three thresholds
    __shared__ int spix[DSQ_QUANT_MAX_PB];
    __shared__ float2 tpairs[16];
    const QuantParams qp = {l, u, dsq_delta(l, u, top), th.inv_delta, th.thr[1], th.thr[2], th.thr[3], top};
    if (MODE == 2) fill_threshold_pairs(tpairs, th);

    const int tid = threadIdx.x;
    const int pixel0 = blockIdx.x * PB;
    const int npix = min(PB, total_pixels - pixel0);
    const bool multi_group = DP != GROUP;
    if (multi_group) {
        for (int i = tid; i < npix; i += 256) spix[i] = 0;
    }
    if (multi_group || MODE == 2) __syncthreads();
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
                uint32_t lo = quant4<VEC, MODE>(px, c0, C, qp, tpairs);
                uint32_t hi = quant4<VEC, MODE>(px, c0 + 4, C, qp, tpairs);
                word = dsq_pack8x4(lo, hi);
                s = dsq_bytesum(lo) + dsq_bytesum(hi);
            } else {
                uint32_t b0 = quant4<VEC, MODE>(px, c0, C, qp, tpairs);
                uint32_t b1 = quant4<VEC, MODE>(px, c0 + 4, C, qp, tpairs);
                uint32_t b2 = quant4<VEC, MODE>(px, c0 + 8, C, qp, tpairs);
                uint32_t b3 = quant4<VEC, MODE>(px, c0 + 12, C, qp, tpairs);
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

// NHWC input whose channel count is a multiple of one packed word (8 channels at
// 4-bit containers, 16 at 2-bit) and whose base is 16-byte aligned -- the common
// case.  Lane-contiguous version: consecutive lanes read consecutive float4
// (every load instruction of a wave covers 1 KB of contiguous memory, where the
// kernel above has each lane walk its own 32- or 64-byte segment), each lane
// turns its four values into four code bytes, and the 2 (4) neighbouring lanes
// that share a packed word combine their bytes with DPP moves.  A block owns PB
// whole pixels; code sums are reduced over aligned lane groups inside a pixel
// with DPP adds, then added into LDS counters.
template <int CONT, bool NT = false>
__global__ __launch_bounds__(256) void quantize_act_nhwc_coalesced_kernel(
    const float *__restrict__ x, uint32_t *__restrict__ codes, int32_t *__restrict__ pix_sum,
    int total_pixels, int C, int DP, int PB, float inv_qp, float l, float u, int top, DsqThresholds th)
{
    // CONT = 3: dense 3-bit output, eight lanes per 12-byte unit of 32 channels (C % 32 == 0)
    constexpr bool D3 = CONT == 3;
    constexpr int CPD = D3 ? 32 : 32 / CONT; // channels per packed word (dense: per unit)
    constexpr int LPW = CPD / 4;             // lanes per packed word: 2 or 4 (dense: 8 per unit)
    constexpr int WPU = D3 ? 3 : 1;          // words per packed word / unit
    constexpr int MODE = CONT == 2 ? 1 : 2;  // 1- and 2-bit codes: at most three thresholds
    __shared__ int spix[DSQ_QUANT_MAX_PB];
    __shared__ float2 tpairs[16];
    const QuantParams qp = {l, u, 0.f, th.inv_delta, th.thr[1], th.thr[2], th.thr[3], top};
    if (MODE == 2) fill_threshold_pairs(tpairs, th);

    const int tid = threadIdx.x;
    const int pixel0 = blockIdx.x * PB;
    const int npix = min(PB, total_pixels - pixel0);
    const int QP = C / 4;                    // float4 units per pixel (a multiple of LPW)
    const int real_words = C / CPD * WPU;    // packed words per pixel that carry channels
    for (int i = tid; i < npix; i += 256) spix[i] = 0;
    __syncthreads();

    const int nunits = npix * QP;
    const int nunits_up = (nunits + 255) & ~255;     // all lanes take part in the DPP moves
    const float4 *xb = reinterpret_cast<const float4 *>(x + (size_t)pixel0 * C);
    // lanes of an aligned group of `group` lanes belong to one pixel
    const int group = (QP & 15) == 0 ? 16 : (QP & 7) == 0 ? 8 : (QP & 3) == 0 ? 4 : 2;

    for (int i = tid; i < nunits_up; i += 256) {
        const bool active = i < nunits;
        uint32_t b = 0;
        if (active) {
            float4 f;
            if (NT) {
                // a tensor larger than the last-level cache is read once and never again
                typedef float v4f __attribute__((ext_vector_type(4)));
                const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(xb) + i);
                f = make_float4(t.x, t.y, t.z, t.w);
            } else {
                f = xb[i];
            }
            b = dsq_bytes4(qcode<MODE>(f.x, qp, tpairs), qcode<MODE>(f.y, qp, tpairs),
                           qcode<MODE>(f.z, qp, tpairs), qcode<MODE>(f.w, qp, tpairs));
        }
        int p = (int)((float)i * inv_qp);            // i / QP with a float reciprocal and a fix-up (i < 2^22)
        int q = i - p * QP;
        if (q < 0) { --p; q += QP; }
        if (q >= QP) { ++p; q -= QP; }
        int s = dsq_bytesum(b);
        uint32_t word;
        if (D3) {
            // lane g of a unit holds group g: its low bits go to word g / 4 at bit 2 (g % 4) of
            // every byte, its high bits to word 2 at bit g of every byte; the eight lanes OR
            // their shares together and lanes 0..2 store one word each
            const int g = tid & 7;
            const uint32_t low = (b & 0x03030303u) << (2 * (g & 3));
            uint32_t w0 = g < 4 ? low : 0u, w1 = g < 4 ? 0u : low, w2 = ((b >> 2) & 0x01010101u) << g;
            w0 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w0, 0xB1, 0xF, 0xF, true);
            w1 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w1, 0xB1, 0xF, 0xF, true);
            w2 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w2, 0xB1, 0xF, 0xF, true);
            w0 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w0, 0x4E, 0xF, 0xF, true);
            w1 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w1, 0x4E, 0xF, 0xF, true);
            w2 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w2, 0x4E, 0xF, 0xF, true);
            w0 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w0, 0x141, 0xF, 0xF, true);
            w1 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w1, 0x141, 0xF, 0xF, true);
            w2 |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w2, 0x141, 0xF, 0xF, true);
            word = g == 0 ? w0 : g == 1 ? w1 : w2;
        } else if (CONT == 4) {
            // word = channels 8w..8w+7: byte j = c[j] | c[j+4] << 4; the odd lane holds c[4..7]
            const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)b, 0xB1, 0xF, 0xF, true);
            word = b | (other << 4);
        } else {
            // word = 16 channels: byte j = c[j] | c[j+4] << 2 | c[j+8] << 4 | c[j+12] << 6
            uint32_t v = b << (2 * (tid & 3));
            v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
            v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);
            word = v;
        }
        if (D3) {
            if (active && (tid & 7) < 3) codes[(size_t)(pixel0 + p) * DP + (q >> 3) * 3 + (tid & 7)] = word;
        } else if (active && (tid & (LPW - 1)) == 0) {
            codes[(size_t)(pixel0 + p) * DP + q / LPW] = word;
        }
        s = dpp_add<0xB1>(s);                                   // lanes ^1
        if (group >= 4) s = dpp_add<0x4E>(s);                   // lanes ^2
        if (group >= 8) s = dpp_add<0x141>(s);                  // other quad (row_half_mirror)
        if (group >= 16) s = dpp_add<0x140>(s);                 // other half row (row_mirror)
        if (active && (tid & (group - 1)) == 0) atomicAdd(&spix[p], s);
    }
    __syncthreads();
    for (int i = tid; i < npix; i += 256) pix_sum[pixel0 + i] = spix[i];
    // channels C..Cp-1 of every pixel hold code 0
    const int pad_words = DP - real_words;
    for (int i = tid; i < npix * pad_words; i += 256) {
        const int p = i / pad_words, d = real_words + i - p * pad_words;
        codes[(size_t)(pixel0 + p) * DP + d] = 0;
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

// ---- dense 3-bit output ---------------------------------------------------------
// 32 channels of a pixel become one 12-byte unit (format: dsq_device.h).  The recipe
// itself (dsq_code, IEEE division) runs per element.
//
// NHWC: one thread per unit, the units of a pixel in neighbouring lanes; a block owns
// whole pixels (PB of them, UPX units each) and adds up their code sums in LDS.
__global__ __launch_bounds__(256) void quantize_act_dense3_nhwc_kernel(const float *__restrict__ x, uint32_t *__restrict__ codes,
                                                                       int *__restrict__ pix_sum, int pixels, int C, int UPX,
                                                                       int PB, float l, float u)
{
    __shared__ int psum[256];
    const int tid = threadIdx.x;
    psum[tid] = 0;
    __syncthreads();
    const float delta = dsq_delta(l, u, 7);
    const int pl = tid / UPX, k = tid - pl * UPX;
    const long long p = (long long)blockIdx.x * PB + pl;
    if (pl < PB && p < pixels) {
        const float *row = x + (size_t)p * C;
        const bool vec = (C & 3) == 0 && (((uintptr_t)x & 15) == 0);
        uint32_t d[8];
        int sum = 0;
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            const int c = 32 * k + 4 * g;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (vec && c + 3 < C) {
                const float4 t = *reinterpret_cast<const float4 *>(row + c);
                v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (c + j < C) v[j] = row[c + j];
            }
            int q[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                q[j] = c + j < C ? dsq_code(v[j], l, u, delta, 7) : 0;       // padding channels: code 0
                sum += q[j];
            }
            d[g] = dsq_bytes4(q[0], q[1], q[2], q[3]);
        }
        uint32_t l0, l1, hi;
        dsq_pack32_d3(d, l0, l1, hi);
        uint32_t *w = codes + ((size_t)p * UPX + k) * 3;
        w[0] = l0; w[1] = l1; w[2] = hi;
        atomicAdd(&psum[pl], sum);
    }
    __syncthreads();
    if (tid < PB && (long long)blockIdx.x * PB + tid < pixels) pix_sum[(long long)blockIdx.x * PB + tid] = psum[tid];
}

// NCHW: one thread per pixel (neighbouring lanes = neighbouring pixels of a row, so the
// reads of a channel are contiguous); the thread walks the pixel's units.
__global__ __launch_bounds__(256) void quantize_act_dense3_nchw_kernel(const float *__restrict__ x, uint32_t *__restrict__ codes,
                                                                       int *__restrict__ pix_sum, int C, int HW, int UPX,
                                                                       float l, float u)
{
    const int hw = blockIdx.x * 256 + threadIdx.x;
    const int n = blockIdx.y;
    if (hw >= HW) return;
    const float delta = dsq_delta(l, u, 7);
    const float *img = x + (size_t)n * C * HW + hw;
    const size_t p = (size_t)n * HW + hw;
    int sum = 0;
    for (int k = 0; k < UPX; ++k) {
        uint32_t d[8];
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            int q[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = 32 * k + 4 * g + j;
                q[j] = c < C ? dsq_code(img[(size_t)c * HW], l, u, delta, 7) : 0;
                sum += q[j];
            }
            d[g] = dsq_bytes4(q[0], q[1], q[2], q[3]);
        }
        uint32_t l0, l1, hi;
        dsq_pack32_d3(d, l0, l1, hi);
        uint32_t *w = codes + (p * UPX + k) * 3;
        w[0] = l0; w[1] = l1; w[2] = hi;
    }
    pix_sum[p] = sum;
}

}  // namespace

hipError_t dsq_launch_quantize_act(const float *x, int layout_nchw, int N, int C, int H, int W,
                                   float l, float u, int bits, const DsqThresholds &th, void *codes,
                                   int32_t *pix_sum, hipStream_t stream)
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
    // The lane-contiguous kernel wins on tensors large enough to be bandwidth bound
    // (measured: 4.0 -> 5.0 TB/s at 2 bits); small ones are latency bound and do
    // better with the kernel below, which has less per-block set-up.
    if (vec && C % (32 / cont) == 0 && (long long)total_pixels * (C / 4) >= 512 * 1024) {
        const int QP = C / 4;
        const long long total_units = (long long)total_pixels * QP;
        int it = 8;
        while (it > 2 && total_units / (256LL * it) < 2048) it >>= 1;
        // (pixels that are not a multiple of 16 float4 long reduce their code sums in
        // small lane groups; measured, such tensors do better with few pixels per block)
        if ((QP & 15) != 0) it = 2;
        int pb = (256 * it) / QP;
        if (pb < 1) pb = 1;
        if (pb > DSQ_QUANT_MAX_PB) pb = DSQ_QUANT_MAX_PB;
        dim3 g((total_pixels + pb - 1) / pb);
        // Tensors of 192 MB and more (three quarters of the last-level cache) are read with
        // non-temporal loads: measured 5.2 -> 5.5 TB/s at 411 MB and 4.6 -> 5.1 at 206 MB, while
        // tensors of 50-100 MB lose 5-10 % with them.
        const bool nt = total_units >= 12LL * 1024 * 1024;
        if (cont == 4 && nt)
            quantize_act_nhwc_coalesced_kernel<4, true><<<g, 256, 0, stream>>>(
                x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, pb, 1.0f / (float)QP, l, u, top, th);
        else if (cont == 4)
            quantize_act_nhwc_coalesced_kernel<4><<<g, 256, 0, stream>>>(
                x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, pb, 1.0f / (float)QP, l, u, top, th);
        else if (nt)
            quantize_act_nhwc_coalesced_kernel<2, true><<<g, 256, 0, stream>>>(
                x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, pb, 1.0f / (float)QP, l, u, top, th);
        else
            quantize_act_nhwc_coalesced_kernel<2><<<g, 256, 0, stream>>>(
                x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, pb, 1.0f / (float)QP, l, u, top, th);
        return hipGetLastError();
    }
    dim3 grid((total_pixels + PB - 1) / PB);
    const bool thr = total_dw >= 256 * 1024;       // large enough to be bandwidth bound
#define DSQ_Q_LAUNCH(CONT, VEC)                                                              \
    do {                                                                                     \
        if (thr) quantize_act_nhwc_kernel<CONT, VEC, true><<<grid, 256, 0, stream>>>(        \
            x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, dp_shift, PB, l, u, top, th); \
        else quantize_act_nhwc_kernel<CONT, VEC, false><<<grid, 256, 0, stream>>>(           \
            x, (uint32_t *)codes, pix_sum, total_pixels, C, DP, dp_shift, PB, l, u, top, th); \
    } while (0)
    if (cont == 4) { if (vec) DSQ_Q_LAUNCH(4, true); else DSQ_Q_LAUNCH(4, false); }
    else           { if (vec) DSQ_Q_LAUNCH(2, true); else DSQ_Q_LAUNCH(2, false); }
#undef DSQ_Q_LAUNCH
    return hipGetLastError();
}

hipError_t dsq_launch_quantize_act_dense3(const float *x, int layout_nchw, int N, int C, int H, int W,
                                          float l, float u, const DsqThresholds &th, void *codes, int32_t *pix_sum,
                                          hipStream_t stream)
{
    const int UPX = dsq_round_up(C, 64) / 32;        // units per pixel (<= 256: checked by the caller)
    const int pixels = N * H * W;
    if (layout_nchw) {
        dim3 grid((H * W + 255) / 256, N);
        quantize_act_dense3_nchw_kernel<<<grid, 256, 0, stream>>>(x, (uint32_t *)codes, pix_sum, C, H * W, UPX, l, u);
    } else if (C % 32 == 0 && (((uintptr_t)x & 15) == 0)) {
        // whole units of real channels: the lane-contiguous kernel (step-function form of the recipe)
        const int QP = C / 4;
        const long long total_units = (long long)pixels * QP;
        int it = 8;
        while (it > 2 && total_units / (256LL * it) < 2048) it >>= 1;
        int pb = (256 * it) / QP;
        if (pb < 1) pb = 1;
        if (pb > DSQ_QUANT_MAX_PB) pb = DSQ_QUANT_MAX_PB;
        quantize_act_nhwc_coalesced_kernel<3><<<(pixels + pb - 1) / pb, 256, 0, stream>>>(
            x, (uint32_t *)codes, pix_sum, pixels, C, UPX * 3, pb, 1.0f / (float)QP, l, u, 7, th);
    } else {
        const int PB = 256 / UPX;
        quantize_act_dense3_nhwc_kernel<<<(pixels + PB - 1) / PB, 256, 0, stream>>>(x, (uint32_t *)codes, pix_sum,
                                                                                    pixels, C, UPX, PB, l, u);
    }
    return hipGetLastError();
}
