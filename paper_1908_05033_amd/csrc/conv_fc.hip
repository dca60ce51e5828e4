// dsq_conv2d for 1x1 layers with few output pixels and a deep dot product: a
// quantized fully connected layer (H = W = 1, the pixels are the batch) and
// its relatives.  Algorithm 1 step 5 of the paper on such a layer is a GEMM
// with a handful of rows and thousands of K; the implicit-GEMM kernels, which
// give every workgroup a tile of pixels and walk K one 64-channel stage at a
// time, leave most of the chip idle there.
//
// Here a workgroup of eight waves owns one 32-pixel x 32-channel tile of the
// output and splits K among its waves: wave w multiplies channel blocks
// w*per .. w*per+per-1 (all loads of a wave are issued before its first matrix
// instruction, so a wave pays one memory latency), the eight partial tiles are
// added through LDS (integer adds: exact in any order), and four of the waves
// run the shared dequantizing epilogue on a quarter of the tile each.  The
// packed formats are those of the other kernels (activations as written by
// dsq_quantize_act, weights in matrix-instruction lane order), and so is the
// arithmetic: int8 matrix instruction for 3/4-bit layers, the FP4 form for
// 1/2-bit layers.
#include "conv_epilogue.h"

namespace {

constexpr int FC_WAVES = 8;
constexpr int FC_CHUNK = 8;      // channel blocks whose loads are in flight together per wave

template <int CONT>
__global__ __launch_bounds__(64 * FC_WAVES) void conv_fc_kernel(DsqConvArgs a)
{
    constexpr int KB_BYTES = 64 * CONT / 8;      // bytes of one pixel's 64-channel block
    constexpr int KG_BYTES = 16 * CONT / 8;      // bytes of 16 channels
    __shared__ v4i part[FC_WAVES][4][64];        // [wave][group of four channels][lane]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int col = lane & 31, h = lane >> 5;
    const int M = a.N * a.Ho * a.Wo;             // = N*H*W: 1x1, stride 1, no padding
    const int m = blockIdx.x * 32 + col;
    const int ct = blockIdx.y;                   // 32-channel tile; ct*32 < Cop by construction
    const int NCB = a.Cp / 64;
    const bool valid = m < M;
    const size_t row_bytes = (size_t)a.Cp * CONT / 8;
    const char *act = (const char *)a.act + (size_t)(valid ? m : 0) * row_bytes;
    const uint32_t *wq = (const uint32_t *)a.wq + ((size_t)ct * NCB * 64 + lane) * 4;

    const int per = (NCB + FC_WAVES - 1) / FC_WAVES;
    const int cb0 = wave * per;
    const int cb1 = min(NCB, cb0 + per);

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
    v16f facc;
#pragma unroll
    for (int r = 0; r < 16; ++r) facc[r] = 0.f;

    for (int base = cb0; base < cb1; base += FC_CHUNK) {
        // packed operands of up to FC_CHUNK channel blocks (blocks past the end: zeros)
        v4i ap[FC_CHUNK], wp[FC_CHUNK];
#pragma unroll
        for (int i = 0; i < FC_CHUNK; ++i) {
            const int cb = base + i;
            const bool on = cb < cb1;
            ap[i] = (v4i){0, 0, 0, 0};
            wp[i] = (v4i){0, 0, 0, 0};
            if (on) {
                wp[i] = *reinterpret_cast<const v4i *>(wq + (size_t)cb * 64 * 4);
                if (valid) {
                    const char *p = act + (size_t)cb * KB_BYTES;
                    if (CONT == 4) {
                        // K halves kh = 0, 1: channels 32*kh + 16*h .. +15
                        const v2i lo = *reinterpret_cast<const v2i *>(p + h * KG_BYTES);
                        const v2i hi = *reinterpret_cast<const v2i *>(p + (2 + h) * KG_BYTES);
                        ap[i] = (v4i){lo.x, lo.y, hi.x, hi.y};
                    } else {
                        const v2i pk = *reinterpret_cast<const v2i *>(p + 8 * h);    // channels 32*h .. 32*h+31
                        ap[i] = (v4i){pk.x, pk.y, 0, 0};
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < FC_CHUNK; ++i) {
            if (CONT == 4) {
                const v4i w0 = dsq_unpack16_c4((v2i){wp[i].x, wp[i].y});
                const v4i w1 = dsq_unpack16_c4((v2i){wp[i].z, wp[i].w});
                const v4i a0 = dsq_unpack16_c4((v2i){ap[i].x, ap[i].y});
                const v4i a1 = dsq_unpack16_c4((v2i){ap[i].z, ap[i].w});
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w0, a0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, a1, acc, 0, 0, 0);
            } else {
                const v4i af = dsq_fp4_from_c2((uint32_t)ap[i].x, (uint32_t)ap[i].y);
                facc = dsq_mfma_fp4(wp[i], af, facc);
            }
        }
    }
    if (CONT == 2) acc = dsq_fp4_acc_to_int(facc);

#pragma unroll
    for (int q = 0; q < 4; ++q)
        part[wave][q][lane] = (v4i){acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    __syncthreads();
    if (wave < 4) {
        const int q = wave;
        v4i sum = part[0][q][lane];
#pragma unroll
        for (int w = 1; w < FC_WAVES; ++w) {
            const v4i t = part[w][q][lane];
            sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
        }
        const DsqPixel px = dsq_pixel_info(a, m, M);
        dsq_store4(a, px, m, ct * 32 + 8 * q + 4 * h, sum, a.delta_a);
    }
}

}  // namespace

// 1x1, stride 1, no padding, no chained output; few enough 32x32 tiles that splitting K
// inside the workgroup pays, and K deep enough to split.
bool dsq_conv_fc_supported(const DsqConvArgs &a)
{
    if (a.R != 1 || a.stride != 1 || a.pad != 0 || a.rq) return false;
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long tiles = ((M + 31) / 32) * ((a.C_out + 31) / 32);
    return a.Cp >= 512 && tiles <= 2048;
}

hipError_t dsq_launch_conv_fc(const DsqConvArgs &a, hipStream_t stream)
{
    const int M = a.N * a.Ho * a.Wo;
    dim3 grid((M + 31) / 32, (a.C_out + 31) / 32);
    if (dsq_container(a.bits) == 4) conv_fc_kernel<4><<<grid, 64 * FC_WAVES, 0, stream>>>(a);
    else conv_fc_kernel<2><<<grid, 64 * FC_WAVES, 0, stream>>>(a);
    return hipGetLastError();
}
