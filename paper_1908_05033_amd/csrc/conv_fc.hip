// dsq_conv2d for 1x1 layers with few output pixels and a deep dot product: a
// quantized fully connected layer (H = W = 1, the pixels are the batch) and
// its relatives.  Algorithm 1 step 5 of the paper on such a layer is a GEMM
// with a handful of rows and thousands of K; the implicit-GEMM kernels, which
// give every workgroup a tile of pixels and walk K one 64-channel stage at a
// time, leave most of the chip idle there.
//
// Here a workgroup of eight waves owns one 32-pixel x 32-channel tile of the
// output and splits K among its waves: wave w multiplies channel blocks
// w*per .. w*per+per-1, eight blocks at a time (the loads of such a chunk are all
// issued together; activation codes come in as whole 16-byte units of the pixel
// rows and are turned into the matrix instruction's lane order through a
// wave-private LDS area), the eight partial tiles are
// added through LDS (integer adds: exact in any order), and four of the waves
// run the shared dequantizing epilogue (or, in chained mode, the next layer's
// quantizer) on a quarter of the tile each.  The
// packed formats are those of the other kernels (activations as written by
// dsq_quantize_act, weights in matrix-instruction lane order), and so is the
// arithmetic: int8 matrix instruction for 3/4-bit layers, the FP4 form for
// 1/2-bit layers.
#include "conv_epilogue.h"

namespace {

constexpr int FC_WAVES = 8;
constexpr int FC_CHUNK = 8;      // channel blocks whose loads are in flight together per wave

// LDS: each wave stages the activation codes of its 32 pixels x FC_CHUNK channel
// blocks (rows of ROW bytes; the row stride makes the column reads below free of
// bank conflicts), then the partial tiles of the eight waves reuse the space.
template <int CONT>
struct FcLayout {
    static constexpr int KB_BYTES = 64 * CONT / 8;            // one pixel's 64-channel block
    static constexpr int ROW_DATA = FC_CHUNK * KB_BYTES;      // 256 B (4-bit containers) or 128 B
    static constexpr int ROW = ROW_DATA + 8;                  // 66 or 34 dwords: odd multiple of 2
    static constexpr int WAVE_BYTES = 32 * ROW;
    static constexpr int STAGE_BYTES = FC_WAVES * WAVE_BYTES;
    static constexpr int PART_BYTES = FC_WAVES * 4 * 64 * 16;
    static constexpr int EXCH_BYTES = 2 * 4 * 64 * 4;         // chained mode: packed codes and code sums of four waves
    static constexpr int LDS_BYTES = STAGE_BYTES > PART_BYTES + EXCH_BYTES ? STAGE_BYTES : PART_BYTES + EXCH_BYTES;
};

template <int CONT>
__global__ __launch_bounds__(64 * FC_WAVES) void conv_fc_kernel(DsqConvArgs a)
{
    typedef FcLayout<CONT> Lay;
    constexpr int KB_BYTES = Lay::KB_BYTES;
    constexpr int KG_BYTES = 16 * CONT / 8;      // bytes of 16 channels
    constexpr int UPR = Lay::ROW_DATA / 16;      // 16-byte units per staged row: 16 or 8
    constexpr int PPI = 64 / UPR;                // pixels one load instruction of a wave covers: 4 or 8
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int col = lane & 31, h = lane >> 5;
    const int M = a.N * a.Ho * a.Wo;             // = N*H*W: 1x1, stride 1, no padding
    const int m0 = blockIdx.x * 32;
    const int m = m0 + col;
    const int ct = blockIdx.y;                   // 32-channel tile; ct*32 < Cop by construction (Cop >= rq_Cp)
    const int NCB = a.Cp / 64;
    const size_t row_bytes = (size_t)a.Cp * CONT / 8;
    const uint32_t *wq = (const uint32_t *)a.wq + ((size_t)ct * NCB * 64 + lane) * 4;
    char *stage = lds + wave * Lay::WAVE_BYTES;

    const int per = (NCB + FC_WAVES - 1) / FC_WAVES;
    const int cb0 = wave * per;
    const int cb1 = min(NCB, cb0 + per);

    // staging: lane -> (pixel inside a group of PPI, 16-byte unit of the row)
    const int s_unit = lane % UPR, s_pix = lane / UPR;

    v16i acc;
    v16f facc;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[r] = 0; facc[r] = 0.f; }

    for (int base = cb0; base < cb1; base += FC_CHUNK) {
        const int nblk = min(FC_CHUNK, cb1 - base);
        // weights: already in lane order, one 16-byte load per channel block
        v4i wp[FC_CHUNK];
#pragma unroll
        for (int i = 0; i < FC_CHUNK; ++i) {
            wp[i] = (v4i){0, 0, 0, 0};
            if (i < nblk) wp[i] = *reinterpret_cast<const v4i *>(wq + (size_t)(base + i) * 64 * 4);
        }
        // activations: contiguous 16-byte units of PPI pixel rows per instruction
        v4i au[32 / PPI];
        const bool unit_on = s_unit * 16 < nblk * KB_BYTES;
#pragma unroll
        for (int g = 0; g < 32 / PPI; ++g) {
            const int pm = m0 + g * PPI + s_pix;
            au[g] = (v4i){0, 0, 0, 0};
            if (unit_on && pm < M)
                au[g] = *reinterpret_cast<const v4i *>((const char *)a.act + (size_t)pm * row_bytes +
                                                       (size_t)base * KB_BYTES + s_unit * 16);
        }
#pragma unroll
        for (int g = 0; g < 32 / PPI; ++g) {
            char *d = stage + (g * PPI + s_pix) * Lay::ROW + s_unit * 16;      // 8-byte aligned
            *reinterpret_cast<v2i *>(d) = (v2i){au[g].x, au[g].y};
            *reinterpret_cast<v2i *>(d + 8) = (v2i){au[g].z, au[g].w};
        }
        // (the region is private to this wave and LDS operations of a wave execute in order)
        const char *rowp = stage + col * Lay::ROW;
#pragma unroll
        for (int i = 0; i < FC_CHUNK; ++i) {
            if (i < nblk) {
                const char *p = rowp + i * KB_BYTES;
                if (CONT == 4) {
                    // K halves kh = 0, 1: channels 32*kh + 16*h .. +15
                    const v2i lo = *reinterpret_cast<const v2i *>(p + h * KG_BYTES);
                    const v2i hi = *reinterpret_cast<const v2i *>(p + (2 + h) * KG_BYTES);
                    const v4i w0 = dsq_unpack16_c4((v2i){wp[i].x, wp[i].y});
                    const v4i w1 = dsq_unpack16_c4((v2i){wp[i].z, wp[i].w});
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w0, dsq_unpack16_c4(lo), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, dsq_unpack16_c4(hi), acc, 0, 0, 0);
                } else {
                    const v2i pk = *reinterpret_cast<const v2i *>(p + 8 * h);    // channels 32*h .. 32*h+31
                    facc = dsq_mfma_fp4(wp[i], dsq_fp4_from_c2((uint32_t)pk.x, (uint32_t)pk.y), facc);
                }
            }
        }
    }
    if (CONT == 2) acc = dsq_fp4_acc_to_int(facc);

    __syncthreads();                               // every wave is done with its staging area
    v4i *part = reinterpret_cast<v4i *>(lds);      // [wave][group of four channels][lane]
#pragma unroll
    for (int q = 0; q < 4; ++q)
        part[(wave * 4 + q) * 64 + lane] = (v4i){acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    __syncthreads();
    if (a.rq) {
        // chained mode: four waves turn a quarter of the tile each into the next
        // layer's codes; a lane pair of one wave then needs all four quarters
        // (it holds whole packed words of its pixel), so they meet in LDS and
        // wave 0 packs, stores and adds to the pixel sums
        uint32_t *exch = reinterpret_cast<uint32_t *>(lds + Lay::PART_BYTES);   // [codes | sums][quarter][lane]
        const DsqPixel px = dsq_pixel_info(a, m, M);
        if (wave < 4) {
            const int q = wave;
            v4i sum = part[q * 64 + lane];
#pragma unroll
            for (int w = 1; w < FC_WAVES; ++w) {
                const v4i t = part[(w * 4 + q) * 64 + lane];
                sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
            }
            const int top_n = (1 << a.rq_bits) - 1;
            int codes = 0;
            exch[q * 64 + lane] = dsq_requant_quarter(a, px, ct * 32 + 8 * q + 4 * h, sum, a.delta_a,
                                                      dsq_delta(a.rq_l, a.rq_u, top_n), top_n, codes);
            exch[(4 + q) * 64 + lane] = (uint32_t)codes;
        }
        __syncthreads();
        if (wave == 0) {
            uint32_t bytes[4];
            int codes = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bytes[q] = exch[q * 64 + lane];
                codes += (int)exch[(4 + q) * 64 + lane];
            }
            const int total = dsq_requant_store32(a, px.valid ? m : -1, ct * 32, h, bytes, codes);
            if (h == 0 && px.valid) atomicAdd(a.rq_pix + m, total);
        }
        return;
    }
    if (wave < 4) {
        const int q = wave;
        v4i sum = part[q * 64 + lane];
#pragma unroll
        for (int w = 1; w < FC_WAVES; ++w) {
            const v4i t = part[(w * 4 + q) * 64 + lane];
            sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
        }
        const DsqPixel px = dsq_pixel_info(a, m, M);
        dsq_store4(a, px, m, ct * 32 + 8 * q + 4 * h, sum, a.delta_a);
    }
}

template <int CONT>
hipError_t launch_fc(const DsqConvArgs &a, hipStream_t stream)
{
    auto kern = conv_fc_kernel<CONT>;
    const int lds = FcLayout<CONT>::LDS_BYTES;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    const int M = a.N * a.Ho * a.Wo;
    // (chained mode also writes the code-0 padding channels up to a multiple of 64)
    dim3 grid((M + 31) / 32, ((a.rq ? a.rq_Cp : a.C_out) + 31) / 32);
    // chained mode: the channel tiles add to the next layer's pixel sums, which a
    // fill kernel clears first unless the caller did (no memset node: the call may be under graph capture)
    if (a.rq && !a.rq_zeroed) {
        const hipError_t e = dsq_launch_fill_zero(a.rq_pix, (size_t)M, stream);
        if (e != hipSuccess) return e;
    }
    kern<<<grid, 64 * FC_WAVES, lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace

// What the kernel takes: 1x1, stride 1, no padding, K deep enough to split among
// eight waves, a bounded number of 32x32 tiles.
bool dsq_conv_fc_supported(const DsqConvArgs &a)
{
    if (a.R != 1 || a.stride != 1 || a.pad != 0) return false;
    if (a.cont == 3) return false;       // (dense 3-bit input: served by the implicit-GEMM kernels)
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long tiles = ((M + 31) / 32) * ((a.C_out + 31) / 32);
    return a.Cp >= 512 && tiles <= 2048;
}

// Where it is also the faster kernel (measured against the implicit-GEMM kernels
// on 1x1 layers of 49..12544 pixels and 512..4096 input channels): up to about
// 800 tiles, or 1536 when the dot product is at least 2048 deep; past that the
// per-tile cost of adding the partial tiles outweighs the idle compute units.
bool dsq_conv_fc_preferred(const DsqConvArgs &a)
{
    if (!dsq_conv_fc_supported(a)) return false;
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long tiles = ((M + 31) / 32) * ((a.C_out + 31) / 32);
    return tiles <= 800 || (a.Cp >= 2048 && tiles <= 1536);
}

hipError_t dsq_launch_conv_fc(const DsqConvArgs &a, hipStream_t stream)
{
    return a.cont == 4 ? launch_fc<4>(a, stream) : launch_fc<2>(a, stream);
}
