// Internal launch interface between the C ABI (api.hip) and the kernels.
// Arguments have already been validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DSQ_QUANT_MAX_PB 512   // most pixels one quantizer block may own

struct DsqConvArgs {
    int N, C_in, H, W, C_out, R, stride, pad, bits;
    int Ho, Wo;
    int cont;      // format of the packed activation codes: 2 or 4 = container width in bits,
                   // 3 = dense 3-bit units (weights are then in the 4-bit layout)
    int Cp;        // C_in rounded up to 64
    int Cop;       // C_out rounded up to 256
    const void *act;          // packed activation codes
    const int32_t *pix_sum;   // [N*H*W]
    float l_a, u_a;
    float delta_a;            // (u_a - l_a) / (2^bits - 1) in binary32, computed by the host
    int kernel;               // host only: DSQ_CONV_KERNEL value of the call (0 = automatic)
    int many_in_flight;       // host only: the caller keeps several calls in flight (DSQ_CONV_MANY_IN_FLIGHT)
    const void *wq;           // packed weights
    const float *delta_w;     // [Cop]
    const float *l_w;         // [Cop]
    const int32_t *sw_total;  // [Cop]
    const int32_t *sw_tap;    // [Cop][R*R]
    float *out;
    int32_t *acc;             // may be null
    int out_nchw;
    // chained mode (dsq_conv2d_requant): instead of out / acc the kernels write
    // the next layer's packed codes and add to its pixel code sums
    int rq;                   // 0 = plain fp32 output
    const float *rq_scale;    // [C_out] or null (= 1)
    const float *rq_shift;    // [C_out] or null (= 0)
    int rq_relu;
    float rq_l, rq_u;         // next layer's clip range
    int rq_bits;
    int rq_dense;             // next layer's codes in the dense 3-bit format (rq_bits == 3)
    // The next layer's quantizer as a step function: rq_thr[j] (j = 1..2^bits-1)
    // is the smallest binary32 value whose code is >= j, found on the host with
    // the very recipe of dsq_code (every step of it is monotone, so
    // code(z) = #{j : z >= rq_thr[j]} exactly); unused entries are NaN, which
    // no value compares >= to.  rq_inv_delta gives a first guess
    // (int)((v - l) * rq_inv_delta + rq_bias) of floor((v - l)/Delta + 0.5) that
    // is off by at most one.
    float rq_thr[16];
    float rq_inv_delta, rq_bias;
    // The LDS-patch kernel first decides a code in "code units":
    //   t = ((y*scale + shift) - l)/Delta + 1/2,  code = floor(clamp(t, rq_t_lo, rq_t_hi)),
    // evaluated in binary32 from per-channel constants (conv_patch_kernel.h), and keeps
    // that code when t is farther from every integer than the error bound of the
    // evaluation; otherwise it falls back on the exact sequence above.  The host part
    // of that bound: rq_t_margin = 1/2 - max_j |t(rq_thr[j]) - j| - 2^-20 (how far the
    // true thresholds sit from the integers of the ideal staircase, plus slack for
    // absolute rounding errors); rq_t_lo = 1/2, or code(0) + 1/2 under the ReLU;
    // rq_t_hi = 2^bits - 1/2; rq_inv_dn = 1/Delta and rq_c0 = 1/2 - l/Delta in binary64;
    // rq_sa_max bounds the sum of activation codes under one output, rq_w_max the
    // weight codes.  rq_fast = 0 (deep layers whose accumulators pass 2^24, extreme
    // ranges) sends every output through the exact sequence.
    int rq_fast;
    float rq_t_lo, rq_t_hi, rq_t_margin, rq_sa_max, rq_w_max;
    double rq_inv_dn, rq_c0;
    int rq_Cp;                // C_out rounded up to 64
    void *rq_codes;           // packed codes of the next layer's input
    int32_t *rq_pix;          // [N*Ho*Wo]; the kernels add to it (cleared before the launch) unless rq_store
    int rq_zeroed;            // the caller cleared rq_pix (DSQ_CONV_NEXT_SUMS_ZERO): launch no fill kernel
    int rq_share;             // set by a launcher: the waves of a workgroup add up their pixel sums in LDS first
    int rq_store;             // set by a launcher whose workgroups each hold all channels of their
                              // pixels: plain stores to rq_pix, nothing to clear
};

// The quantizer of one tensor as a step function (see dsq_code_thr): thr[j],
// j = 1..2^bits-1, is the smallest binary32 value whose code is >= j (NaN in
// unused entries), found by the host with the recipe of dsq_code.
struct DsqThresholds {
    float thr[16];
    float inv_delta;
};

hipError_t dsq_launch_quantize_act(const float *x, int layout_nchw, int N, int C, int H, int W,
                                   float l, float u, int bits, const DsqThresholds &th, void *codes,
                                   int32_t *pix_sum, hipStream_t stream);
// The same into the dense 3-bit format (bits == 3, C rounded up to 64 at most 8192).
hipError_t dsq_launch_quantize_act_dense3(const float *x, int layout_nchw, int N, int C, int H, int W,
                                          float l, float u, const DsqThresholds &th, void *codes,
                                          int32_t *pix_sum, hipStream_t stream);

// `cont`: the container (2 or 4 bits) of the layer the weights are for; codes of
// `bits` <= cont bits are stored in it.
hipError_t dsq_launch_pack_weights(const float *w, const float *l_w, const float *u_w,
                                   const uint8_t *codes, int C_out, int C_in, int R, int bits, int cont,
                                   void *w_packed, void *w_aux, hipStream_t stream);

// Constants of the training-mode DSQ function for one tensor, computed on the
// host in binary64 and rounded once.
struct DsqSoftArgs {
    float l, u, delta, inv_delta;
    float last_interval;      // 2^b - 2
    float inv_levels;         // 1 / (2^b - 1)
    float k, s;
    float k_a, k_l, k_u;      // how k moves with alpha, l, u (0 when k is capped)
    float s_a, s_l, s_u;      // how s moves with alpha, l, u
};

hipError_t dsq_launch_soft_fwd(const float *x, float *y, size_t n, const DsqSoftArgs &p, hipStream_t stream);
hipError_t dsq_launch_soft_bwd(const float *x, const float *gy, float *gx, size_t n, const DsqSoftArgs &p,
                               double *sums, hipStream_t stream);

// Sets n int32 words to zero with a kernel (safe inside graph capture).
hipError_t dsq_launch_fill_zero(int32_t *p, size_t n, hipStream_t stream);

hipError_t dsq_launch_conv_simple(const DsqConvArgs &a, hipStream_t stream);
// force_tile: -1 = choose by problem size; 0 / 1 / 2 / 3 = the 128x64 / 128x128 /
// 256x128 / 256x64 (pixels x channels) workgroup tile.
hipError_t dsq_launch_conv_patch(const DsqConvArgs &a, int force_tile, hipStream_t stream);
// Whether the LDS-patch kernel supports this geometry with that tile.
bool dsq_conv_patch_supported(const DsqConvArgs &a, int force_tile);
// The launch configuration it would use, as text; returns 0 if it does not take the geometry.
int dsq_conv_patch_describe(const DsqConvArgs &a, int force_tile, char *text, size_t n);

// Split-K kernel for 1x1 layers with few output pixels (fully connected layers).
bool dsq_conv_fc_supported(const DsqConvArgs &a);   // the kernel takes this layer
bool dsq_conv_fc_preferred(const DsqConvArgs &a);   // ... and is the faster choice for it
hipError_t dsq_launch_conv_fc(const DsqConvArgs &a, hipStream_t stream);

// Weight-only quantized layer: binary32 activations x (NHWC or NCHW), weights in the
// packed 4-bit layout; uses the geometry, wq, delta_w, l_w, out and out_nchw of `a`.
hipError_t dsq_launch_conv_wq(const DsqConvArgs &a, const float *x, int x_nchw, hipStream_t stream);
