// C ABI of libdsqconv (see include/dsqconv.h): host-side validation and
// dispatch only; every step of the path runs in the HIP kernels.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "../../include/dsqconv.h"
#include "dsq_device.h"
#include "dsq_kernels.h"

namespace {

bool bits_ok(int bits) { return bits >= 1 && bits <= 4; }
bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
// A clip range must be finite, ordered, and of a width whose step Delta = (u - l) / (2^b - 1)
// and the reciprocal of it are normal binary32 numbers with room to spare: the
// step-function kernels start from the guess (v - l) * (1 / Delta).
bool range_ok(float l, float u)
{
    if (!(isfinite(l) && isfinite(u) && l < u)) return false;
    const float width = u - l;
    return width >= 1e-30f && width <= 1e30f;
}
const long long kMaxElems = (1LL << 31) - 1;

void quantizer_thresholds(float l, float u, int bits, float thr[16]);

}  // namespace

extern "C" {

size_t dsq_act_packed_bytes(int N, int H, int W, int C, int bits)
{
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || !bits_ok(bits)) return 0;
    return (size_t)N * H * W * (size_t)(dsq_round_up(C, 64) * dsq_container(bits) / 8);
}

size_t dsq_act_packed_bytes_ex(int N, int H, int W, int C, int bits, dsq_packing packing)
{
    if (packing == DSQ_PACK_CONTAINER) return dsq_act_packed_bytes(N, H, W, C, bits);
    if (packing != DSQ_PACK_DENSE3 || bits != 3 || N <= 0 || H <= 0 || W <= 0 || C <= 0) return 0;
    return (size_t)N * H * W * (size_t)(dsq_round_up(C, 64) / 32 * 12);
}

size_t dsq_wgt_packed_bytes(int C_out, int C_in, int R, int S, int bits)
{
    if (C_out <= 0 || C_in <= 0 || R <= 0 || S <= 0 || !bits_ok(bits)) return 0;
    // one code per 4-bit field at every width (2-bit layers feed the FP4 matrix instruction)
    return (size_t)dsq_round_up(C_out, 256) * R * S * (size_t)(dsq_round_up(C_in, 64) / 2);
}

size_t dsq_wgt_aux_bytes(int C_out, int R, int S)
{
    if (C_out <= 0 || R <= 0 || S <= 0) return 0;
    return (size_t)dsq_round_up(C_out, 256) * (3 + (size_t)R * S) * 4;
}

dsq_status dsq_quantize_act(const float *x, dsq_layout layout, int N, int C, int H, int W, float l,
                            float u, int bits, void *codes_packed, size_t codes_bytes,
                            int32_t *pix_code_sum, void *hip_stream)
{
    if (!x || !codes_packed || !pix_code_sum) return DSQ_ERR_NULL;
    if (!bits_ok(bits)) return DSQ_ERR_BITS;
    if (!range_ok(l, u)) return DSQ_ERR_RANGE;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return DSQ_ERR_SHAPE;
    if (layout != DSQ_NHWC && layout != DSQ_NCHW) return DSQ_ERR_UNSUPPORTED;
    if ((long long)N * H * W * dsq_round_up(C, 64) > kMaxElems) return DSQ_ERR_UNSUPPORTED;
    if (layout == DSQ_NCHW && N > 65535) return DSQ_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(codes_packed) || !aligned16(pix_code_sum)) return DSQ_ERR_ALIGN;
    if (codes_bytes < dsq_act_packed_bytes(N, H, W, C, bits)) return DSQ_ERR_SIZE;
    DsqThresholds th;
    quantizer_thresholds(l, u, bits, th.thr);
    th.inv_delta = 1.0f / ((u - l) / (float)((1 << bits) - 1));
    hipError_t e = dsq_launch_quantize_act(x, layout == DSQ_NCHW, N, C, H, W, l, u, bits, th,
                                           codes_packed, pix_code_sum, (hipStream_t)hip_stream);
    return e == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
}

dsq_status dsq_quantize_act_ex(const float *x, dsq_layout layout, int N, int C, int H, int W, float l, float u,
                               int bits, dsq_packing packing, void *codes_packed, size_t codes_bytes,
                               int32_t *pix_code_sum, void *hip_stream)
{
    if (packing == DSQ_PACK_CONTAINER)
        return dsq_quantize_act(x, layout, N, C, H, W, l, u, bits, codes_packed, codes_bytes, pix_code_sum, hip_stream);
    if (!x || !codes_packed || !pix_code_sum) return DSQ_ERR_NULL;
    if (!bits_ok(bits)) return DSQ_ERR_BITS;
    if (packing != DSQ_PACK_DENSE3 || bits != 3) return DSQ_ERR_UNSUPPORTED;
    if (!range_ok(l, u)) return DSQ_ERR_RANGE;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return DSQ_ERR_SHAPE;
    if (layout != DSQ_NHWC && layout != DSQ_NCHW) return DSQ_ERR_UNSUPPORTED;
    if ((long long)N * H * W * dsq_round_up(C, 64) > kMaxElems) return DSQ_ERR_UNSUPPORTED;
    if (dsq_round_up(C, 64) > 8192) return DSQ_ERR_UNSUPPORTED;       // (one thread per 32-channel unit of a pixel)
    if (layout == DSQ_NCHW && N > 65535) return DSQ_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(codes_packed) || !aligned16(pix_code_sum)) return DSQ_ERR_ALIGN;
    if (codes_bytes < dsq_act_packed_bytes_ex(N, H, W, C, bits, packing)) return DSQ_ERR_SIZE;
    DsqThresholds th;
    quantizer_thresholds(l, u, bits, th.thr);
    th.inv_delta = 1.0f / ((u - l) / 7.0f);
    hipError_t e = dsq_launch_quantize_act_dense3(x, layout == DSQ_NCHW, N, C, H, W, l, u, th, codes_packed,
                                                  pix_code_sum, (hipStream_t)hip_stream);
    return e == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
}

dsq_status dsq_pack_weights_for(const float *w_oihw, const float *l_w, const float *u_w,
                                const uint8_t *codes_oihw, int C_out, int C_in, int R, int S,
                                int bits_w, int bits_act, void *w_packed, size_t w_bytes, void *w_aux,
                                size_t aux_bytes, void *hip_stream)
{
    if ((!w_oihw && !codes_oihw) || !l_w || !u_w || !w_packed || !w_aux) return DSQ_ERR_NULL;
    if (!bits_ok(bits_w) || !bits_ok(bits_act)) return DSQ_ERR_BITS;
    if (C_out <= 0 || C_in <= 0 || R <= 0 || S <= 0) return DSQ_ERR_SHAPE;
    if (R != S || (R != 1 && R != 3)) return DSQ_ERR_UNSUPPORTED;
    // 3/4-bit weight codes do not fit the fields of a layer with 1/2-bit activations
    if (dsq_container(bits_w) > dsq_container(bits_act)) return DSQ_ERR_UNSUPPORTED;
    if ((long long)dsq_round_up(C_out, 256) * dsq_round_up(C_in, 64) * R * S > kMaxElems)
        return DSQ_ERR_UNSUPPORTED;
    if (!aligned16(w_packed) || !aligned16(w_aux)) return DSQ_ERR_ALIGN;
    if (w_bytes < dsq_wgt_packed_bytes(C_out, C_in, R, S, bits_act)) return DSQ_ERR_SIZE;
    if (aux_bytes < dsq_wgt_aux_bytes(C_out, R, S)) return DSQ_ERR_SIZE;
    hipError_t e = dsq_launch_pack_weights(w_oihw, l_w, u_w, codes_oihw, C_out, C_in, R, bits_w,
                                           dsq_container(bits_act), w_packed, w_aux,
                                           (hipStream_t)hip_stream);
    return e == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
}

dsq_status dsq_pack_weights(const float *w_oihw, const float *l_w, const float *u_w,
                            const uint8_t *codes_oihw, int C_out, int C_in, int R, int S, int bits,
                            void *w_packed, size_t w_bytes, void *w_aux, size_t aux_bytes,
                            void *hip_stream)
{
    return dsq_pack_weights_for(w_oihw, l_w, u_w, codes_oihw, C_out, C_in, R, S, bits, bits, w_packed,
                                w_bytes, w_aux, aux_bytes, hip_stream);
}

namespace {

// Geometry checks shared by the convolution entry points; fills the part of the
// kernel arguments that does not depend on where the results go.
dsq_status conv_args(const dsq_conv_desc *d, const void *act_packed, const int32_t *pix_code_sum,
                     float l_a, float u_a, const void *w_packed, const void *w_aux, DsqConvArgs &a)
{
    if (!d || !act_packed || !pix_code_sum || !w_packed || !w_aux) return DSQ_ERR_NULL;
    if (!bits_ok(d->bits)) return DSQ_ERR_BITS;
    if (!range_ok(l_a, u_a)) return DSQ_ERR_RANGE;
    if (d->N <= 0 || d->C_in <= 0 || d->H <= 0 || d->W <= 0 || d->C_out <= 0 || d->R <= 0 ||
        d->S <= 0 || d->stride <= 0 || d->pad < 0)
        return DSQ_ERR_SHAPE;
    if (d->R != d->S || (d->R != 1 && d->R != 3) || (d->stride != 1 && d->stride != 2) ||
        d->pad > d->R - 1)
        return DSQ_ERR_UNSUPPORTED;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return DSQ_ERR_SHAPE;
    const int Ho = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    const int Wo = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    if (Ho <= 0 || Wo <= 0) return DSQ_ERR_SHAPE;
    const int Cp = dsq_round_up(d->C_in, 64), Cop = dsq_round_up(d->C_out, 256);
    if ((long long)d->N * d->H * d->W * Cp > kMaxElems) return DSQ_ERR_UNSUPPORTED;
    // depth of the dot products: 9 * K <= 2^22 keeps the fp32 accumulation of the
    // 1/2-bit path exact (sums of quarter units below 2^24) and the int32 sums of the
    // 3/4-bit path (at most 225 * K) far from overflow
    if (9LL * d->R * d->S * Cp > (1LL << 22)) return DSQ_ERR_UNSUPPORTED;
    if ((long long)d->N * Ho * Wo * dsq_round_up(d->C_out, 64) > kMaxElems) return DSQ_ERR_UNSUPPORTED;
    if ((long long)d->N * Ho * Wo + 1024 > kMaxElems) return DSQ_ERR_UNSUPPORTED;
    if ((d->flags & ~(15 | DSQ_CONV_MANY_IN_FLIGHT | DSQ_CONV_ACT_DENSE3 | DSQ_CONV_NEXT_DENSE3 | DSQ_CONV_NEXT_SUMS_ZERO)) != 0 ||
        (d->flags & 15) > 7)
        return DSQ_ERR_UNSUPPORTED;
    if ((d->flags & DSQ_CONV_ACT_DENSE3) && d->bits != 3) return DSQ_ERR_UNSUPPORTED;
    if (!aligned16(act_packed) || !aligned16(pix_code_sum) || !aligned16(w_packed) || !aligned16(w_aux))
        return DSQ_ERR_ALIGN;

    a.N = d->N; a.C_in = d->C_in; a.H = d->H; a.W = d->W; a.C_out = d->C_out; a.R = d->R;
    a.stride = d->stride; a.pad = d->pad; a.bits = d->bits;
    a.Ho = Ho; a.Wo = Wo; a.Cp = Cp; a.Cop = Cop;
    a.cont = (d->flags & DSQ_CONV_ACT_DENSE3) ? 3 : dsq_container(d->bits);
    a.act = act_packed; a.pix_sum = pix_code_sum; a.l_a = l_a; a.u_a = u_a;
    a.kernel = d->flags & 15;
    a.many_in_flight = (d->flags & DSQ_CONV_MANY_IN_FLIGHT) != 0;
    // (one IEEE binary32 subtraction and division: the value dsq_delta gives on the device)
    a.delta_a = (u_a - l_a) / (float)((1 << d->bits) - 1);
    a.wq = w_packed;
    a.delta_w = (const float *)w_aux;
    a.l_w = a.delta_w + Cop;
    a.sw_total = (const int32_t *)(a.l_w + Cop);
    a.sw_tap = a.sw_total + Cop;
    a.out = nullptr; a.acc = nullptr; a.out_nchw = 0;
    a.rq = 0; a.rq_scale = nullptr; a.rq_shift = nullptr; a.rq_relu = 0;
    a.rq_l = 0.f; a.rq_u = 1.f; a.rq_bits = 4; a.rq_dense = 0; a.rq_Cp = 0; a.rq_codes = nullptr; a.rq_pix = nullptr; a.rq_store = 0; a.rq_share = 0; a.rq_zeroed = 0;
    for (int j = 0; j < 16; ++j) a.rq_thr[j] = 0.f;
    a.rq_inv_delta = 0.f; a.rq_bias = 0.f;
    a.rq_fast = 0; a.rq_t_lo = 0.5f; a.rq_t_hi = 0.5f; a.rq_t_margin = -1.f; a.rq_sa_max = 0.f; a.rq_w_max = 0.f;
    a.rq_inv_dn = 0.0; a.rq_c0 = 0.0;
    return DSQ_OK;
}

// ---- the quantizer as a step function (host side) ---------------------------
// The same binary32 recipe as the device function dsq_code, operation for
// operation (this file is compiled without contraction of a*b+c).
int host_code(float x, float l, float u, float delta, int top)
{
    const float v = fminf(fmaxf(x, l), u);
    const float t = (v - l) / delta;
    int c = (int)floorf(t + 0.5f);
    return c < 0 ? 0 : c > top ? top : c;
}

// Finite floats in increasing order <-> unsigned keys in increasing order.
uint32_t key_of(float x)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
float float_of(uint32_t k)
{
    const uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    float x;
    memcpy(&x, &b, 4);
    return x;
}

// thr[j], j = 1..top: the smallest finite float whose code is >= j (bisection over
// the ordered floats; code() is monotone non-decreasing).
void quantizer_thresholds(float l, float u, int bits, float thr[16])
{
    const int top = (1 << bits) - 1;
    const float delta = (u - l) / (float)top;
    for (int j = 0; j < 16; ++j) thr[j] = NAN;          // unused: no value compares >= NaN
    for (int j = 1; j <= top; ++j) {
        uint32_t lo = key_of(-3.4028234e38f), hi = key_of(3.4028234e38f);   // code(lo) = 0 < j <= code(hi) = top
        while (hi - lo > 1) {
            const uint32_t mid = lo + (hi - lo) / 2;
            if (host_code(float_of(mid), l, u, delta, top) >= j) hi = mid; else lo = mid;
        }
        thr[j] = float_of(hi);
    }
}

// Every launcher checks its plan and kernel attributes first and only then
// enqueues (in chained mode: the clearing of the next layer's pixel sums where
// workgroups add to them, then the kernel), so that an error leaves the stream
// untouched.
dsq_status launch_conv(const DsqConvArgs &a, hipStream_t stream)
{
    // 0 auto, 1 simple, 2 patch (auto tile), 3..6 patch with a fixed tile, 7 split-K 1x1
    const int kernel = a.kernel;
    hipError_t e;
    if (kernel == 7 || kernel == 0) {
        const bool fc_ok = kernel == 7 ? dsq_conv_fc_supported(a) : dsq_conv_fc_preferred(a);
        if (kernel == 7 && !fc_ok) return DSQ_ERR_UNSUPPORTED;
        if (fc_ok) {
            e = dsq_launch_conv_fc(a, stream);
            return e == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
        }
    }
    const int force_tile = kernel >= 3 ? kernel - 3 : -1;
    const bool patch_ok = kernel != 1 && dsq_conv_patch_supported(a, force_tile);
    if (kernel >= 2 && !patch_ok) return DSQ_ERR_UNSUPPORTED;
    e = patch_ok ? dsq_launch_conv_patch(a, force_tile, stream) : dsq_launch_conv_simple(a, stream);
    return e == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
}

// The kernel launch_conv would pick, as text.
dsq_status describe_conv(const DsqConvArgs &a, char *text, size_t n)
{
    const int kernel = a.kernel;
    if (kernel == 7 || kernel == 0) {
        const bool fc_ok = kernel == 7 ? dsq_conv_fc_supported(a) : dsq_conv_fc_preferred(a);
        if (kernel == 7 && !fc_ok) return DSQ_ERR_UNSUPPORTED;
        if (fc_ok) {
            snprintf(text, n, "split-K kernel for 1x1 layers with few pixels: container %d%s", a.cont,
                     a.rq ? ", chained epilogue" : "");
            return DSQ_OK;
        }
    }
    const int force_tile = kernel >= 3 ? kernel - 3 : -1;
    if (kernel != 1 && dsq_conv_patch_describe(a, force_tile, text, n)) return DSQ_OK;
    if (kernel >= 2) return DSQ_ERR_UNSUPPORTED;
    snprintf(text, n, "simple kernel (one wave per 32x32 tile): container %d%s", a.cont,
             a.rq ? ", chained epilogue" : "");
    return DSQ_OK;
}

}  // namespace

dsq_status dsq_conv2d_plan(const dsq_conv_desc *d, int chained, float l_a, char *text, size_t text_bytes)
{
    if (!text || text_bytes == 0) return DSQ_ERR_NULL;
    text[0] = 0;
    DsqConvArgs a;
    // (the pointers only have to pass the checks: nothing is launched)
    alignas(16) static const char dummy[16] = {0};
    const dsq_status st = conv_args(d, dummy, (const int32_t *)dummy, l_a, l_a + 1.0f, dummy, dummy, a);
    if (st != DSQ_OK) return st;
    a.rq = chained != 0;
    a.rq_Cp = dsq_round_up(a.C_out, 64);
    return describe_conv(a, text, text_bytes);
}

dsq_status dsq_conv2d(const dsq_conv_desc *d, const void *act_packed, const int32_t *pix_code_sum,
                      float l_a, float u_a, const void *w_packed, const void *w_aux, float *out,
                      dsq_layout out_layout, int32_t *acc_or_null, void *hip_stream)
{
    if (!out) return DSQ_ERR_NULL;
    DsqConvArgs a;
    const dsq_status st = conv_args(d, act_packed, pix_code_sum, l_a, u_a, w_packed, w_aux, a);
    if (st != DSQ_OK) return st;
    if (d->flags & (DSQ_CONV_NEXT_DENSE3 | DSQ_CONV_NEXT_SUMS_ZERO)) return DSQ_ERR_UNSUPPORTED;   // (only dsq_conv2d_requant writes codes)
    if (out_layout != DSQ_NHWC && out_layout != DSQ_NCHW) return DSQ_ERR_UNSUPPORTED;
    if (!aligned16(out) || (acc_or_null && !aligned16(acc_or_null))) return DSQ_ERR_ALIGN;
    a.out = out; a.acc = acc_or_null; a.out_nchw = out_layout == DSQ_NCHW;
    return launch_conv(a, (hipStream_t)hip_stream);
}

dsq_status dsq_conv2d_wq(const dsq_conv_desc *d, const float *x, dsq_layout x_layout, const void *w_packed,
                         const void *w_aux, float *out, dsq_layout out_layout, void *hip_stream)
{
    if (!x || !out) return DSQ_ERR_NULL;
    if (d && d->flags != 0) return DSQ_ERR_UNSUPPORTED;
    DsqConvArgs a;
    // (geometry and pointer checks shared with the other convolution calls: x stands in
    // for the two activation-side pointers, the clip range is not used)
    const dsq_status st = conv_args(d, x, (const int32_t *)x, 0.0f, 1.0f, w_packed, w_aux, a);
    if (st != DSQ_OK) return st;
    if ((x_layout != DSQ_NHWC && x_layout != DSQ_NCHW) || (out_layout != DSQ_NHWC && out_layout != DSQ_NCHW))
        return DSQ_ERR_UNSUPPORTED;
    if ((long long)d->N * d->H * d->W * d->C_in > kMaxElems) return DSQ_ERR_UNSUPPORTED;
    if (!aligned16(out)) return DSQ_ERR_ALIGN;
    a.out = out; a.out_nchw = out_layout == DSQ_NCHW;
    const hipError_t e = dsq_launch_conv_wq(a, x, x_layout == DSQ_NCHW, (hipStream_t)hip_stream);
    return e == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
}

dsq_status dsq_conv2d_requant(const dsq_conv_desc *d, const void *act_packed,
                              const int32_t *pix_code_sum, float l_a, float u_a,
                              const void *w_packed, const void *w_aux, const float *scale,
                              const float *shift, int relu, float l_next, float u_next,
                              int bits_next, void *codes_next, size_t codes_bytes,
                              int32_t *pix_code_sum_next, void *hip_stream)
{
    if (!codes_next || !pix_code_sum_next) return DSQ_ERR_NULL;
    DsqConvArgs a;
    const dsq_status st = conv_args(d, act_packed, pix_code_sum, l_a, u_a, w_packed, w_aux, a);
    if (st != DSQ_OK) return st;
    if (!bits_ok(bits_next)) return DSQ_ERR_BITS;
    if (!range_ok(l_next, u_next)) return DSQ_ERR_RANGE;
    if (!aligned16(codes_next) || !aligned16(pix_code_sum_next) || (scale && !aligned16(scale)) ||
        (shift && !aligned16(shift)))
        return DSQ_ERR_ALIGN;
    const bool dense_next = (d->flags & DSQ_CONV_NEXT_DENSE3) != 0;
    if (dense_next && bits_next != 3) return DSQ_ERR_UNSUPPORTED;
    if (codes_bytes < dsq_act_packed_bytes_ex(a.N, a.Ho, a.Wo, a.C_out, bits_next,
                                              dense_next ? DSQ_PACK_DENSE3 : DSQ_PACK_CONTAINER))
        return DSQ_ERR_SIZE;
    a.rq_dense = dense_next;
    a.rq_zeroed = (d->flags & DSQ_CONV_NEXT_SUMS_ZERO) != 0;
    a.rq = 1; a.rq_scale = scale; a.rq_shift = shift; a.rq_relu = relu != 0;
    a.rq_l = l_next; a.rq_u = u_next; a.rq_bits = bits_next;
    a.rq_Cp = dsq_round_up(a.C_out, 64);
    a.rq_codes = codes_next; a.rq_pix = pix_code_sum_next;
    quantizer_thresholds(l_next, u_next, bits_next, a.rq_thr);
    {
        const float delta_n = (u_next - l_next) / (float)((1 << bits_next) - 1);
        a.rq_inv_delta = 1.0f / delta_n;
        a.rq_bias = 0.5f;
        // constants of the code-unit form (see DsqConvArgs)
        const int top_n = (1 << bits_next) - 1;
        const double inv_dn = 1.0 / (double)delta_n, c0 = 0.5 - (double)l_next * inv_dn;
        double e_thr = 0.0;
        for (int j = 1; j <= top_n; ++j) e_thr = fmax(e_thr, fabs((double)a.rq_thr[j] * inv_dn + c0 - (double)j));
        const int code0 = host_code(0.0f, l_next, u_next, delta_n, top_n);
        const double c_max = a.cont == 2 ? 3.0 : 15.0;                   // largest code a container field holds
        const double depth = (double)a.R * a.R * a.C_in;
        a.rq_inv_dn = inv_dn; a.rq_c0 = c0;
        a.rq_t_lo = relu ? (float)code0 + 0.5f : 0.5f;
        a.rq_t_hi = (float)top_n + 0.5f;
        a.rq_t_margin = (float)(0.5 - e_thr - 0x1p-20);
        a.rq_sa_max = (float)(c_max * depth);
        a.rq_w_max = (float)c_max;
        a.rq_fast = c_max * c_max * depth < 0x1p24 && delta_n >= 0x1p-60f && delta_n <= 0x1p60f &&
                    fabsf(l_next) <= 0x1p60f && a.rq_t_margin > 0.0f;
    }
    return launch_conv(a, (hipStream_t)hip_stream);
}

namespace {

// Shape of the DSQ function from (l, u, alpha, bits): Sec. 3.3 of the paper,
// with the cap k <= 1000 of Sec. 4.3; when the cap is active s comes from its
// definition 1/tanh(0.5*k*Delta) so that neighbouring intervals still join.
dsq_status soft_args(float l, float u, float alpha, int bits, DsqSoftArgs &p)
{
    if (!bits_ok(bits)) return DSQ_ERR_BITS;
    if (!range_ok(l, u)) return DSQ_ERR_RANGE;
    if (!(alpha > 0.0f && alpha < 0.5f)) return DSQ_ERR_RANGE;
    const double levels = (double)((1 << bits) - 1);
    const double delta = ((double)u - (double)l) / levels;
    if (!(delta > 0.0)) return DSQ_ERR_RANGE;
    const double a = (double)alpha;
    const double c = log(2.0 / a - 1.0);
    double k = c / delta, s, k_a, k_l, k_u, s_a, s_l, s_u;
    if (k > 1000.0) {
        k = 1000.0;
        const double T = tanh(0.5 * k * delta);
        s = 1.0 / T;
        k_a = k_l = k_u = 0.0;
        s_a = 0.0;
        s_l = (1.0 - T * T) * k / (2.0 * levels * T * T);
        s_u = -s_l;
    } else {
        s = 1.0 / (1.0 - a);
        k_a = -2.0 / (a * (2.0 - a)) / delta;
        k_l = c / (levels * delta * delta);
        k_u = -k_l;
        s_a = 1.0 / ((1.0 - a) * (1.0 - a));
        s_l = s_u = 0.0;
    }
    p.l = l; p.u = u; p.delta = (float)delta; p.inv_delta = (float)(1.0 / delta);
    p.last_interval = (float)(levels - 1.0); p.inv_levels = (float)(1.0 / levels);
    p.k = (float)k; p.s = (float)s;
    p.k_a = (float)k_a; p.k_l = (float)k_l; p.k_u = (float)k_u;
    p.s_a = (float)s_a; p.s_l = (float)s_l; p.s_u = (float)s_u;
    return DSQ_OK;
}

}  // namespace

dsq_status dsq_soft_quantize_fwd(const float *x, size_t n, float l, float u, float alpha, int bits,
                                 float *y, void *hip_stream)
{
    if (!x || !y) return DSQ_ERR_NULL;
    if (n == 0 || n > (size_t)kMaxElems) return DSQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return DSQ_ERR_ALIGN;
    DsqSoftArgs p;
    const dsq_status st = soft_args(l, u, alpha, bits, p);
    if (st != DSQ_OK) return st;
    return dsq_launch_soft_fwd(x, y, n, p, (hipStream_t)hip_stream) == hipSuccess ? DSQ_OK : DSQ_ERR_HIP;
}

dsq_status dsq_soft_quantize_bwd(const float *x, const float *grad_y, size_t n, float l, float u,
                                 float alpha, int bits, float *grad_x, double *grad_alpha_l_u,
                                 void *hip_stream)
{
    if (!x || !grad_y || !grad_x || !grad_alpha_l_u) return DSQ_ERR_NULL;
    if (n == 0 || n > (size_t)kMaxElems) return DSQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(grad_y) || !aligned16(grad_x) || !aligned16(grad_alpha_l_u))
        return DSQ_ERR_ALIGN;
    DsqSoftArgs p;
    const dsq_status st = soft_args(l, u, alpha, bits, p);
    if (st != DSQ_OK) return st;
    return dsq_launch_soft_bwd(x, grad_y, grad_x, n, p, grad_alpha_l_u, (hipStream_t)hip_stream) == hipSuccess
               ? DSQ_OK : DSQ_ERR_HIP;
}

const char *dsq_status_string(dsq_status s)
{
    switch (s) {
    case DSQ_OK: return "ok";
    case DSQ_ERR_NULL: return "a required pointer is NULL";
    case DSQ_ERR_BITS: return "bits must be 1, 2, 3 or 4";
    case DSQ_ERR_RANGE: return "clip range must be finite with l < u";
    case DSQ_ERR_SHAPE: return "invalid tensor or filter shape";
    case DSQ_ERR_UNSUPPORTED: return "unsupported geometry, layout or tensor size";
    case DSQ_ERR_ALIGN: return "device pointer is not 16-byte aligned";
    case DSQ_ERR_SIZE: return "caller buffer is too small";
    case DSQ_ERR_HIP: return "HIP runtime error at kernel launch";
    }
    return "unknown status";
}

}  // extern "C"
