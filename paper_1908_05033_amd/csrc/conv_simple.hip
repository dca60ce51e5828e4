// dsq_conv2d, simple kernel: one wavefront per 32-pixel x 32-channel output
// tile, operands fetched straight from global memory and unpacked in
// registers (4-bit containers: int8 matrix instruction; 2-bit: the FP4 form, see
// dsq_device.h).  It supports every geometry the library accepts and serves as the
// fallback and as a cross-check for the tuned kernel.
//
// The GEMM view of Algorithm 1 step 5: rows = output channels, columns =
// output pixels, K = taps x input channels.  v_mfma_i32_32x32x32_i8 takes, per
// lane, 16 int8 of one row of the first operand (row = lane%32, K group =
// lane/32) and 16 int8 of one column of the second (column = lane%32, same K
// group), and leaves in lane L, register r, the int32 result of row
// 8*(r/4) + 4*(L/32) + r%4 of column L%32 -- i.e. four groups of four
// consecutive output channels of one pixel.
#include "conv_epilogue.h"

namespace {

template <int CONT>
__global__ __launch_bounds__(256) void conv_simple_kernel(DsqConvArgs a)
{
    // CONT: 2 / 4 = container width of the packed activation codes, 3 = dense 3-bit units
    // (the weights of such a layer are in the 4-bit layout)
    constexpr int WPL = CONT == 2 ? 1 : 2;       // packed weight words per lane per K half
    constexpr int KB_BYTES = 64 * CONT / 8;      // bytes of one pixel's 64-channel block
    constexpr int KG_BYTES = 16 * CONT / 8;      // bytes of 16 channels
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, h = lane >> 5;
    const int M = a.N * a.Ho * a.Wo;
    const int m = blockIdx.x * 32 + col;
    const int ct = blockIdx.y * 4 + wave;
    if (ct * 32 >= (a.rq ? a.rq_Cp : a.C_out)) return;     // (uniform per wave)
    const int T = a.R * a.R;
    const int NCB = a.Cp / 64;
    const int top = (1 << a.bits) - 1;
    const float delta_a = dsq_delta(a.l_a, a.u_a, top);

    const bool valid = m < M;
    const int mm = valid ? m : 0;
    const int ox = mm % a.Wo, oy = (mm / a.Wo) % a.Ho, n = mm / (a.Wo * a.Ho);
    const size_t row_bytes = (size_t)a.Cp * CONT / 8;
    const char *act = (const char *)a.act;
    const uint32_t *wq = (const uint32_t *)a.wq;

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
    if (CONT == 2) {
        // 2-bit layers: FP4 matrix instruction, 64 channels of one tap per step
        v16f facc;
#pragma unroll
        for (int r = 0; r < 16; ++r) facc[r] = 0.f;
        for (int cb = 0; cb < NCB; ++cb) {
            for (int tap = 0; tap < T; ++tap) {
                const int r = tap / a.R, s = tap % a.R;
                const int iy = oy * a.stride - a.pad + r, ix = ox * a.stride - a.pad + s;
                const bool inside = valid && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                v4i af = {0, 0, 0, 0};
                if (inside) {
                    const char *p = act + (((size_t)n * a.H + iy) * a.W + ix) * row_bytes + cb * KB_BYTES + 8 * h;
                    const v2i pk = *reinterpret_cast<const v2i *>(p);    // channels 32*h .. 32*h+31
                    af = dsq_fp4_from_c2((uint32_t)pk.x, (uint32_t)pk.y);
                }
                const v4i wf = *reinterpret_cast<const v4i *>(
                    wq + ((((size_t)ct * NCB + cb) * T + tap) * 64 + lane) * 4);
                facc = dsq_mfma_fp4(wf, af, facc);
            }
        }
        acc = dsq_fp4_acc_to_int(facc);
    }
    for (int cb = 0; cb < (CONT == 2 ? 0 : NCB); ++cb) {
        for (int tap = 0; tap < T; ++tap) {
            const int r = tap / a.R, s = tap % a.R;
            const int iy = oy * a.stride - a.pad + r, ix = ox * a.stride - a.pad + s;
            const bool inside = valid && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
            const char *p = act + (((size_t)n * a.H + iy) * a.W + ix) * row_bytes + cb * KB_BYTES;
            const uint32_t *wp = wq + ((((size_t)ct * NCB + cb) * T + tap) * 64 + lane) * 2 * WPL;
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                v4i af = {0, 0, 0, 0};
                if (inside) {
                    if (CONT == 3) {
                        // unit kh of the block: its low word h and its high-bit word
                        const uint32_t *u = reinterpret_cast<const uint32_t *>(p + kh * 12);
                        const uint32_t low = u[h], hi = u[2];
                        uint32_t g[8];
                        dsq_unpack32_d3(low, low, hi >> (4 * h), g);      // groups 4h..4h+3 land in g[0..3]
                        af = (v4i){(int)g[0], (int)g[1], (int)g[2], (int)g[3]};
                    } else {
                        const char *pk = p + (2 * kh + h) * KG_BYTES;   // channels 32*kh + 16*h ..
                        af = dsq_unpack16_c4(*reinterpret_cast<const v2i *>(pk));
                    }
                }
                const v4i wf = dsq_unpack16_c4(*reinterpret_cast<const v2i *>(wp + kh * WPL));
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, af, acc, 0, 0, 0);
            }
        }
    }
    const DsqPixel px = dsq_pixel_info(a, m, M);
    if (a.rq) {
        const int total = dsq_requant_tile(a, px, m, ct * 32, h, acc, delta_a);
        if (h == 0 && px.valid) atomicAdd(a.rq_pix + m, total);
        return;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const v4i part = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        dsq_store4(a, px, m, ct * 32 + 8 * q + 4 * h, part, delta_a);
    }
}

}  // namespace

hipError_t dsq_launch_conv_simple(const DsqConvArgs &a, hipStream_t stream)
{
    const int M = a.N * a.Ho * a.Wo;
    dim3 grid((M + 31) / 32, ((a.rq ? a.rq_Cp : a.C_out) + 127) / 128);
    // chained mode: the workgroups add to the next layer's pixel sums, which a
    // fill kernel clears first unless the caller did (no memset node: the call may be under graph capture)
    if (a.rq && !a.rq_zeroed) {
        const hipError_t e = dsq_launch_fill_zero(a.rq_pix, (size_t)M, stream);
        if (e != hipSuccess) return e;
    }
    if (a.cont == 4) conv_simple_kernel<4><<<grid, 256, 0, stream>>>(a);
    else if (a.cont == 3) conv_simple_kernel<3><<<grid, 256, 0, stream>>>(a);
    else conv_simple_kernel<2><<<grid, 256, 0, stream>>>(a);
    return hipGetLastError();
}
