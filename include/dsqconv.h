/*
 * dsqconv.h -- C ABI of libdsqconv: b-bit (1..4) uniformly quantized conv2d
 * executed as integer arithmetic on codes, for AMD MI355X (gfx950).
 *
 * The three calls are the deployment form of one DSQ-quantized convolution
 * layer (paper: Algorithm 1, feed-forward, after the soft quantizer has been
 * hardened by the sign function -- Sec. 3.2 -- so that it is the uniform
 * quantizer of Sec. 3.1; Sec. 3.5 "Training and Deploying" and Sec. 4.5 run
 * such layers with integer GEMM kernels):
 *
 *   dsq_pack_weights   once per layer   w -> codes (Alg. 1 steps 1,3 for w),
 *                                       laid out for the matrix cores
 *   dsq_quantize_act   per activation   a -> codes (Alg. 1 steps 1,3 for a)
 *   dsq_conv2d         per layer        o = Convolution(w_hat, a_hat)
 *                                       (Alg. 1 steps 4,5) as an integer GEMM
 *                                       on the codes plus zero-point terms
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE memory owned by the caller; scalars and
 *     the descriptor struct are host values.  The library allocates nothing
 *     and never synchronises: work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = default stream) and the call
 *     returns at once.
 *   - Arguments are validated on the host before anything is launched; on any
 *     error nothing has been enqueued.  Errors are return codes only.
 *   - The library holds no mutable state: every call is a function of its
 *     arguments and may run concurrently with any other call.
 *   - Device pointers must be 16-byte aligned.
 *   - bits is 1, 2, 3 or 4.  The descriptor's bits is the activations' width; the
 *     weights may have another one (dsq_pack_weights_for; their step travels in
 *     w_aux), except 3- or 4-bit weights under 1- or 2-bit activations.
 *     bits = 1 is the binary case of Sec. 3.1: with (l, u) = (-1, +1) the two
 *     levels are sgn(x) (code 1 for x >= 0), and any other (l, u) gives the
 *     two-level quantizer with levels l and u.
 *
 * Quantizer (Sec. 3.1 uniform quantizer with range [l,u]; tie rule from
 * sgn(0)=+1 applied at the interval midpoints m_i of Sec. 3.2), evaluated in
 * IEEE binary32 in exactly this order:
 *     Delta = (u - l) / (2^b - 1)            (true division)
 *     v     = min(max(x, l), u)              (NaN -> l)
 *     t     = (v - l) / Delta                (true division)
 *     code  = clamp((int)floor(t + 0.5), 0, 2^b - 1)
 * The level a code stands for is l + Delta*code (Alg. 1 step 4).
 *
 * Packed code format ("container" = 4 bits for b in {3,4}, 2 bits for b in {1,2})
 *   A 32-bit word holds 8 (4-bit) or 16 (2-bit) consecutive channels
 *   c0, c1, ...; byte j (j=0..3) of the word is
 *       4-bit:  c[j] | c[j+4] << 4
 *       2-bit:  c[j] | c[j+4] << 2 | c[j+8] << 4 | c[j+12] << 6
 *   so (word >> k*container) & 0x0F0F0F0F (or 0x03030303) yields four
 *   consecutive channels as four int8.
 *   Activations: [N][H][W][Cp] with Cp = C rounded up to a multiple of 64,
 *   channels >= C hold code 0; one pixel is Cp*container/8 bytes.
 *   Weights: blocks of 32 output channels x 64 input channels of one filter
 *   tap, ordered [Cop/32][Cp/64][R*S][64 lanes][16 bytes], lane = 32*h + (o % 32).
 *   Cop = C_out rounded up to a multiple of 256; rows >= C_out and channels
 *   >= C_in hold code 0.  One code per 4-bit field at every width:
 *     bits 3, 4: the lane's 16 bytes are its two K halves kh = 0, 1, each the
 *       channels 64*cb + 32*kh + 16*h + 0..15 of output channel o as two words of
 *       the format above -- the operand order of the 32x32x32 int8 matrix
 *       instruction;
 *     bits 1, 2: the lane's 16 bytes are the 32 channels 64*cb + 32*h + 0..31, word d
 *       (0..3) nibble n (0..7, from the low end) holding channel offset
 *       16*(d/2) + 4*(d%2) + 8*(n%2) + n/2.  A 2-bit code zero-extended to four
 *       bits is the FP4 (e2m1) encoding of code/2, so these words are operands
 *       of the 32x32x64 FP4 matrix instruction as they stand; the nibble order
 *       is the one in which a packed 2-bit activation word w spreads into
 *       w & 0x33333333 and (w >> 2) & 0x33333333.
 *
 * Dense 3-bit activation codes (DSQ_PACK_DENSE3; Sec. 3.1 gives every quantizer
 *   its own b, and b = 3 is one of the widths the paper deploys, Sec. 4.5): 3 bits
 *   per code instead of a 4-bit container.  [N][H][W][Cp/32] units of 12 bytes,
 *   Cp = C rounded up to 64 (channels >= C hold code 0).  A unit holds channels
 *   c0..c31 as three words: word 0 / word 1 = the low two bits of channels 0..15 /
 *   16..31 in the 2-bit container format above, word 2 = the high bits, bit
 *   8j + g = bit 2 of channel 4g + j (j = 0..3, g = 0..7).  Written by
 *   dsq_quantize_act_ex and by dsq_conv2d_requant with DSQ_CONV_NEXT_DENSE3, read
 *   by the convolution calls with DSQ_CONV_ACT_DENSE3; the weights of such a layer
 *   are packed as for any 3-bit layer (dsq_pack_weights with bits = 3).
 */
#ifndef DSQCONV_H
#define DSQCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DSQ_OK = 0,
    DSQ_ERR_NULL = 1,        /* a required pointer is NULL */
    DSQ_ERR_BITS = 2,        /* bits not in {1,2,3,4} */
    DSQ_ERR_RANGE = 3,       /* !(l < u), a bound is not finite, or the width
                                u - l of an activation range is outside
                                [1e-30, 1e30] */
    DSQ_ERR_SHAPE = 4,       /* a dimension <= 0, or Ho/Wo <= 0 */
    DSQ_ERR_UNSUPPORTED = 5, /* R != S, R not in {1,3}, stride not in {1,2},
                                pad > R-1, a tensor of 2^31 or more elements,
                                R*S*C_in (C_in rounded up to 64) above 2^22 / 9,
                                unknown layout */
    DSQ_ERR_ALIGN = 6,       /* device pointer not 16-byte aligned */
    DSQ_ERR_SIZE = 7,        /* a caller buffer is smaller than required */
    DSQ_ERR_HIP = 8          /* the HIP runtime refused a launch */
} dsq_status;

typedef enum { DSQ_NHWC = 0, DSQ_NCHW = 1 } dsq_layout;

/* How activation codes are packed: in 2- or 4-bit containers (every width), or
 * 3-bit codes densely (bits = 3 only). */
typedef enum { DSQ_PACK_CONTAINER = 0, DSQ_PACK_DENSE3 = 1 } dsq_packing;

/* Per-call choices of the convolution entry points, OR-ed into
 * dsq_conv_desc.flags.  0 is the normal value: the library picks the kernel
 * and optimises for the shortest time of a single call on an otherwise idle
 * GPU.  The library keeps no state between calls: everything a call depends
 * on is in its arguments, so calls from several threads or streams do not
 * interfere.
 *
 * DSQ_CONV_KERNEL(k), k = 0..7, selects the kernel (for tests and
 *   benchmarking): 0 = automatic, 1 = the simple one-wave-per-tile kernel,
 *   2 = the LDS-patch kernel with its tile chosen by problem size, 3 / 4 / 5 / 6
 *   = the LDS-patch kernel with the 128x64 / 128x128 / 256x128 / 256x64
 *   (pixels x channels) tile, 7 = the split-K kernel for 1x1 layers with few
 *   output pixels and at least 512 input channels (fully connected layers;
 *   taken automatically for those).  With 2..7 the call returns
 *   DSQ_ERR_UNSUPPORTED instead of falling back when the chosen kernel cannot
 *   take the geometry (the 256x128 tile has a dsq_conv2d_requant variant for 1- and
 *   2-bit layers only and reports the same for the others).
 * DSQ_CONV_MANY_IN_FLIGHT tells the automatic choice that the caller keeps
 *   several calls in flight on different streams (a server with several
 *   requests, independent branches of a network): layers that yield only about
 *   one workgroup per compute unit then run with one wave group per workgroup
 *   instead of two, so that workgroups of different calls share the compute
 *   units.  Results are identical bit for bit either way.
 * DSQ_CONV_ACT_DENSE3: act_packed is in the dense 3-bit format (bits must be 3).
 *   The split-K kernel does not read that format: fully connected layers then run
 *   on the implicit-GEMM kernels, and DSQ_CONV_KERNEL(7) gives DSQ_ERR_UNSUPPORTED.
 * DSQ_CONV_NEXT_DENSE3 (dsq_conv2d_requant only): codes_next is written in the
 *   dense 3-bit format (bits_next must be 3).
 * DSQ_CONV_NEXT_SUMS_ZERO (dsq_conv2d_requant only): the caller has set
 *   pix_code_sum_next to zero (by work enqueued earlier on the same stream), so the
 *   call launches no clearing kernel of its own.  A network runner that keeps the
 *   pixel sums of all its layers in one buffer clears them with a single fill per
 *   forward pass instead of one small launch per layer.  If the buffer is not zero
 *   the sums of layers wider than a workgroup's tile come out too large by what it
 *   held.
 * Any other bit set gives DSQ_ERR_UNSUPPORTED.
 */
#define DSQ_CONV_KERNEL(k) ((k) & 15)
#define DSQ_CONV_MANY_IN_FLIGHT 0x10
#define DSQ_CONV_ACT_DENSE3 0x20
#define DSQ_CONV_NEXT_DENSE3 0x40
#define DSQ_CONV_NEXT_SUMS_ZERO 0x80

typedef struct {
    int N, C_in, H, W;   /* input activation */
    int C_out, R, S;     /* filter bank (R = S) */
    int stride, pad;
    int bits;
    int flags;           /* 0, or DSQ_CONV_* values OR-ed together */
} dsq_conv_desc;

/* ---- sizes (pure host functions; 0 on invalid arguments) ---------------- */

/* Bytes of the packed activation tensor for an N x H x W x C input. */
size_t dsq_act_packed_bytes(int N, int H, int W, int C, int bits);
/* The same for a given packing (DSQ_PACK_DENSE3: bits must be 3; 0 otherwise). */
size_t dsq_act_packed_bytes_ex(int N, int H, int W, int C, int bits,
                               dsq_packing packing);
/* Bytes of the packed weight tensor. */
size_t dsq_wgt_packed_bytes(int C_out, int C_in, int R, int S, int bits);
/* Bytes of the per-output-channel side table written by dsq_pack_weights:
 * float delta_w[Cop], float l_w[Cop], int32 sw_total[Cop],
 * int32 sw_tap[Cop][R*S]  (sums of weight codes over C_in). */
size_t dsq_wgt_aux_bytes(int C_out, int R, int S);

/* ---- dsq_quantize_act: Alg. 1 steps 1 and 3 for the activation ---------
 * x            device, float32, N*C*H*W elements in `layout`
 * l, u         the learned clip range of this activation (host scalars)
 * codes_packed device, out, dsq_act_packed_bytes() bytes (codes_bytes is the
 *              caller's buffer size and is checked)
 * pix_code_sum device, out, int32[N*H*W]: sum over channels of the codes of
 *              each pixel (the conv epilogue needs it for the l_w term)
 */
dsq_status dsq_quantize_act(const float *x, dsq_layout layout, int N, int C,
                            int H, int W, float l, float u, int bits,
                            void *codes_packed, size_t codes_bytes,
                            int32_t *pix_code_sum, void *hip_stream);

/* ---- dsq_quantize_act_ex: the same with a choice of packing ---------------
 * packing = DSQ_PACK_CONTAINER is dsq_quantize_act.  DSQ_PACK_DENSE3 (bits = 3,
 * C rounded up to 64 at most 8192, else DSQ_ERR_UNSUPPORTED) writes the dense
 * 3-bit format described at the top of this file; codes and pixel sums are the
 * same numbers in either packing.
 */
dsq_status dsq_quantize_act_ex(const float *x, dsq_layout layout, int N, int C,
                               int H, int W, float l, float u, int bits,
                               dsq_packing packing, void *codes_packed,
                               size_t codes_bytes, int32_t *pix_code_sum,
                               void *hip_stream);

/* ---- dsq_pack_weights: Alg. 1 steps 1 and 3 for the weights ------------
 * w_oihw       device, float32 [C_out][C_in][R][S]; may be NULL if
 *              codes_oihw is given
 * l_w, u_w     device, float32 [C_out]: clip range per output channel (a
 *              per-tensor range is the case of equal entries).  Always
 *              required (they define the levels).  A channel whose range is
 *              not finite or not l<u gets delta_w = NaN, which makes that
 *              channel's outputs NaN; validate ranges on the host if needed.
 * codes_oihw   device, uint8 [C_out][C_in][R][S] or NULL.  If non-NULL the
 *              quantizer is skipped and these codes are packed as they are;
 *              a code above 2^bits - 1 is stored as 2^bits - 1 (saturated, as
 *              the quantizer saturates a value above u).
 * w_packed     device, out, dsq_wgt_packed_bytes() bytes
 * w_aux        device, out, dsq_wgt_aux_bytes() bytes
 */
dsq_status dsq_pack_weights(const float *w_oihw, const float *l_w,
                            const float *u_w, const uint8_t *codes_oihw,
                            int C_out, int C_in, int R, int S, int bits,
                            void *w_packed, size_t w_bytes, void *w_aux,
                            size_t aux_bytes, void *hip_stream);

/* ---- dsq_pack_weights_for: weights and activations of different widths ---
 * Sec. 3.1 gives every quantizer its own b.  The same as dsq_pack_weights,
 * for a layer whose activations have bits_act bits (the descriptor's bits,
 * the width given to dsq_quantize_act) while the weights have bits_w: the
 * weight codes are stored in the fields of that layer's container, so any
 * bits_w goes with 3- or 4-bit activations and 1- or 2-bit weights go with
 * 1- or 2-bit activations; 3- or 4-bit weights under 1- or 2-bit activations
 * give DSQ_ERR_UNSUPPORTED.  dsq_pack_weights(.., bits, ..) is the case
 * bits_w = bits_act = bits.
 */
dsq_status dsq_pack_weights_for(const float *w_oihw, const float *l_w,
                                const float *u_w, const uint8_t *codes_oihw,
                                int C_out, int C_in, int R, int S, int bits_w,
                                int bits_act, void *w_packed, size_t w_bytes,
                                void *w_aux, size_t aux_bytes,
                                void *hip_stream);

/* ---- dsq_conv2d: Alg. 1 steps 4 and 5 ----------------------------------
 * Computes, for every output pixel m = (n, oy, ox) and output channel o,
 *     ACC   = sum over taps (r,s) inside the image, channels c of
 *             code_a[n, oy*stride-pad+r, ox*stride-pad+s, c] * code_w[o,c,r,s]
 *     out   = Da*Dw[o]*ACC + l_a*Dw[o]*SW + l_w[o]*Da*SA + KV*l_a*l_w[o]
 * with SA / SW the sums of activation / weight codes over the same in-image
 * taps and KV = C_in * (number of in-image taps): exactly the convolution of
 * the dequantized tensors with zero padding.  ACC is exact int32; the four
 * terms are combined in binary64 and rounded once to binary32.
 *
 * d            geometry and bits (host struct)
 * act_packed, pix_code_sum   outputs of dsq_quantize_act for this input
 * l_a, u_a     the same range that was given to dsq_quantize_act
 * w_packed, w_aux            outputs of dsq_pack_weights for this layer
 * out          device, float32, N*Ho*Wo*C_out elements in `out_layout`
 * acc_or_null  device, int32, same shape and layout as out, or NULL: raw ACC
 */
dsq_status dsq_conv2d(const dsq_conv_desc *d, const void *act_packed,
                      const int32_t *pix_code_sum, float l_a, float u_a,
                      const void *w_packed, const void *w_aux, float *out,
                      dsq_layout out_layout, int32_t *acc_or_null,
                      void *hip_stream);

/* ---- dsq_conv2d_requant: one layer chained onto the next -----------------
 * Alg. 1 steps 4 and 5 of this layer followed by steps 1 and 3 of the layer that
 * consumes its output (Sec. 3.5 "Training and Deploying": at inference the
 * network runs on the integer codes from layer to layer).  For every output
 * element the call evaluates, without writing the float tensor to memory,
 *     y    = the binary32 value dsq_conv2d would store
 *     z    = y * scale[o]            (binary32, rounded)
 *     z    = z + shift[o]            (binary32, rounded)   folded batch norm
 *     z    = max(z, 0)               if relu != 0
 *     code = the quantizer at the top of this file applied to z with
 *            (l_next, u_next, bits_next)
 * and writes the codes in the packed activation format for C_out channels
 * ([N][Ho][Wo][C_out rounded up to 64], padding channels hold code 0) plus the
 * per-pixel code sums: exactly what dsq_quantize_act would have produced from
 * the NHWC tensor z, ready to be the act_packed / pix_code_sum of the next
 * dsq_conv2d or dsq_conv2d_requant.
 *
 * d .. w_aux        as for dsq_conv2d
 * scale, shift      device, float32 [C_out], or NULL for 1 and 0
 * l_next, u_next, bits_next   clip range and width of the next layer's
 *                   activation quantizer (bits_next may differ from d->bits)
 * codes_next        device, out, dsq_act_packed_bytes(N, Ho, Wo, C_out,
 *                   bits_next) bytes (dsq_act_packed_bytes_ex(.., DSQ_PACK_DENSE3)
 *                   with DSQ_CONV_NEXT_DENSE3); codes_bytes is the caller's buffer size
 * pix_code_sum_next device, out, int32[N*Ho*Wo]; the call clears it with a fill
 *                   kernel on the same stream (no memset node, so the call can
 *                   be captured into a HIP graph; DSQ_CONV_NEXT_SUMS_ZERO says the
 *                   caller already did) and accumulates with integer
 *                   atomics, which are exact in any order (layers narrow enough
 *                   that a pixel's sum is complete within one workgroup have
 *                   it stored directly)
 */
dsq_status dsq_conv2d_requant(const dsq_conv_desc *d, const void *act_packed,
                              const int32_t *pix_code_sum, float l_a, float u_a,
                              const void *w_packed, const void *w_aux,
                              const float *scale, const float *shift, int relu,
                              float l_next, float u_next, int bits_next,
                              void *codes_next, size_t codes_bytes,
                              int32_t *pix_code_sum_next, void *hip_stream);

/* ---- dsq_conv2d_wq: quantized weights, full-precision activations -----------
 * The "b/32" rows of the paper's Tables 3, 6 and 7 (e.g. 1-bit weights and
 * 32-bit activations): Algorithm 1 with the activation quantizer left out, so
 * that step 5 convolves the dequantized weights w_hat = l_w + Dw*code (step 4)
 * with the activations themselves.  There is no integer path: levels and
 * activations are binary32, products are exact inside the fp32 matrix
 * instruction and sums are accumulated in binary32, so an output differs from
 * the real-valued convolution by at most about (K + 2) * 2^-24 of the sum of
 * the absolute values of its K = R*S*C_in products (typically far less).
 *
 * d            geometry; bits is the weights' width (1..4); flags must be 0
 * x            device, float32, N*C_in*H*W elements in x_layout; padding is
 *              the real number 0
 * w_packed, w_aux   outputs of dsq_pack_weights_for(.., bits_w = d->bits,
 *              bits_act = 4, ..): the weight codes in 4-bit fields
 * out          device, float32, N*Ho*Wo*C_out elements in out_layout
 */
dsq_status dsq_conv2d_wq(const dsq_conv_desc *d, const float *x,
                         dsq_layout x_layout, const void *w_packed,
                         const void *w_aux, float *out, dsq_layout out_layout,
                         void *hip_stream);

/* ---- training mode: the differentiable soft quantization function ---------
 * Sec. 3.2: inside interval P_i = [l + i*Delta, l + (i+1)*Delta)
 *     phi(x) = s * tanh(k * (x - m_i)),  m_i = l + (i + 0.5)*Delta
 *     Q_S(x) = l + Delta * (i + (phi(x) + 1)/2);   Q_S = l for x < l, u for x > u
 * Sec. 3.3: k = log(2/alpha - 1)/Delta and s = 1/(1 - alpha); Sec. 4.3 keeps
 * alpha in (0, 0.5) (otherwise DSQ_ERR_RANGE) and k <= 1000 (when the cap is
 * active, s = 1/tanh(0.5*k*Delta) so that the intervals still join).
 * Elementwise binary32 arithmetic on constants the host derives in binary64;
 * NaN inputs give NaN.  n <= 2^31 - 1 elements of any shape, contiguous.
 *
 * dsq_soft_quantize_fwd   y[j] = Q_S(x[j])
 * dsq_soft_quantize_bwd   Algorithm 1, back-propagation, for one tensor:
 *     grad_x[j]         = grad_y[j] * dQ_S/dx
 *     grad_alpha_l_u[0] = sum_j grad_y[j] * dQ_S/dalpha     (Sec. 3.3)
 *     grad_alpha_l_u[1] = sum_j grad_y[j] * dQ_S/dl         (Sec. 3.4)
 *     grad_alpha_l_u[2] = sum_j grad_y[j] * dQ_S/du         (Sec. 3.4)
 *   with the interval index held fixed; outside [l, u] only the clipped bound
 *   receives gradient.  grad_alpha_l_u is device memory, 3 doubles, 16-byte
 *   aligned, overwritten (cleared by a fill kernel on the stream, then
 *   accumulated in binary64, so the order of the partial sums moves the result
 *   by about 1e-16 relative).
 */
dsq_status dsq_soft_quantize_fwd(const float *x, size_t n, float l, float u,
                                 float alpha, int bits, float *y,
                                 void *hip_stream);
dsq_status dsq_soft_quantize_bwd(const float *x, const float *grad_y, size_t n,
                                 float l, float u, float alpha, int bits,
                                 float *grad_x, double *grad_alpha_l_u,
                                 void *hip_stream);

/* ---- dsq_conv2d_plan: which kernel a call would run ------------------------
 * Writes into `text` (host memory, text_bytes bytes, NUL-terminated, truncated
 * if need be) a one-line description of the kernel and launch configuration
 * that dsq_conv2d (chained = 0) or dsq_conv2d_requant (chained != 0) would use
 * for this descriptor (geometry, bits, flags) and this l_a (a non-zero l_a sends
 * chained layers to the simple kernel).  Nothing is launched.  For benchmark
 * reports and tests; returns the status the call itself would return for the
 * descriptor (DSQ_ERR_UNSUPPORTED if a forced kernel cannot take it).
 */
dsq_status dsq_conv2d_plan(const dsq_conv_desc *d, int chained, float l_a,
                           char *text, size_t text_bytes);

/* Static, NUL-terminated description of a status code. */
const char *dsq_status_string(dsq_status s);

#ifdef __cplusplus
}
#endif
#endif /* DSQCONV_H */
