// dsq_conv2d, LDS-patch kernel (the tuned path).
//
// GEMM view of Algorithm 1 step 5 of the paper: rows = output channels,
// columns = output pixels, K = filter taps x input channels, run on
// v_mfma_i32_32x32x32_i8 with int32 accumulation (the integer-arithmetic
// deployment of Sec. 3.5 / 4.5, re-designed for the matrix cores; the
// 16x16x64 form of the instruction issues at half the rate on this chip).
//
// A workgroup (4 wavefronts, WP x WC) owns BP = 32*PF*WP consecutive output
// pixels of a strip of TW output columns (pixels are numbered row by row
// through the whole batch, so a tile may span rows and images) and
// BC = 32*CT*WC output channels; a wavefront owns PF fragments of 32 pixels and
// CT tiles of 32 channels.  K is walked in stages of 64 input channels.  For a
// stage, the input patch that all R*R taps of the tile touch is read from
// HBM/L2 once, unpacked from 2/4-bit codes to int8 and kept in LDS; the taps
// then read shifted windows of it, so the R*R-fold re-use of the activations
// never leaves the CU.  Positions of the patch that fall in the zero padding
// hold code 0: they add nothing to the integer sums, and the epilogue's SA /
// SW / KV terms leave them out as well.  Weight fragments were laid out per
// lane by dsq_pack_weights and go from global memory straight to registers,
// each refilled for the next stage right after its use.  The patch of the next
// stage is fetched while the current one is multiplied (two LDS buffers, one
// barrier per stage).
//
// Feed rates that shape the tiles (measured on MI355X): LDS delivers 128 B/clk
// per CU, the vector L1 one wave-wide load (<= 16 B per lane) per 16 clk per
// CU.  With 4 waves issuing MFMAs back to back, activation fragments keep the
// LDS busy 1/CT of the time and weight fragments keep the L1 busy 1/PF of the
// time.
#pragma once
#include <type_traits>

#include "conv_epilogue.h"

struct PatchPlan {
    int TW;            // strip width in output columns
    int BP;            // pixels per tile
    int tiles_w;       // strips per output row
    int row_tiles;     // tiles per strip
    int PR, PC;        // patch rows (max over tiles) x patch columns
    int RP;            // LDS bytes per patch row
    int buf_bytes;     // LDS bytes of one patch buffer (incl. a 64-byte dump slot at its end)
    int Hp;            // H + 2*pad: rows of one image in the padded row space
    int units;         // 16-byte fetch units per stage
    int aux_off;       // LDS offset of the small tables that follow the patch / staging area
    int tiles_c;       // channel tiles (workgroups per pixel tile)
    int total_blocks;  // pixel tiles * channel tiles
    int xcd_chunk;     // ceil(total_blocks / 8)
    uint32_t mg_tiles_c;   // division constants (see idiv) of tiles_c ...
    int step_q, step_r;   // (256 / units-per-pixel) divided by PC: quotient and remainder
    uint32_t mg_PC, mg_TW, mg_Hp, mg_Ho, mg_tiles_w;   // ... and of PC, TW, Hp, Ho, tiles_w
};

namespace {

// LDS bytes per patch pixel: 64 int8 (4-bit containers) or 32 bytes of FP4
// nibbles (2-bit) plus padding that makes the stride an odd multiple of 16, so
// that the 16-byte reads of 16 consecutive pixels fall into distinct bank groups.
constexpr int pix_stride(int cont) { return cont == 2 ? 48 : 80; }


// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains
// the vector-memory counter, which would expose the latency of the global
// loads that are deliberately left in flight across stage boundaries.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// x / d for x >= 0 and d >= 1 by multiplication: with m = min(floor(2^32 / d), 2^32 - 1)
// (computed on the host, division_constant below) the high word of x * m is the
// quotient or one less, so one correction suffices.  Wave-uniform operands stay
// on the scalar unit.
__device__ __forceinline__ int idiv(int x, int d, uint32_t m, int &rem)
{
    int q = (int)__umulhi((uint32_t)x, m);
    int r = x - q * d;
    if (r >= d) { ++q; r -= d; }
    rem = r;
    return q;
}

// The kernel's first argument where it lives: in the kernel-argument segment.
__device__ __forceinline__ const DsqConvArgs &kernarg_conv_args()
{
#if defined(__HIP_DEVICE_COMPILE__)
    return *reinterpret_cast<const DsqConvArgs *>(__builtin_amdgcn_kernarg_segment_ptr());
#else
    return *static_cast<const DsqConvArgs *>(nullptr);      // (host pass of the compiler: never executed)
#endif
}

// Epilogue for the cases the kernel's inline fast path does not cover; kept out
// of line so that its address arithmetic does not weigh on the main kernel.
__device__ __noinline__ void store4_general(const DsqConvArgs &a, int m, int o0, v4i acc, float delta_a)
{
    const DsqPixel px = dsq_pixel_info(a, m, a.N * a.Ho * a.Wo);
    dsq_store4(a, px, m, o0, acc, delta_a);
}

// Chained mode, per output channel o: the constants of the code-unit form of the
// layer-to-layer map.  With P = Da*Dw[o], Q = Da*l_w[o] (binary64, exact), scale sc
// and shift sh, the real value of the next layer's input in units of its quantizer
// step is
//   t = ((P*ACC + Q*SA)*sc + sh - l_n)/D_n + 1/2 = A*(ACC + rho*SA) + s,
//   A = P*sc/D_n, rho = Q/P = l_w/Dw, s = sh/D_n + c0, c0 = 1/2 - l_n/D_n,
// and the code is floor(t) clamped to the code range.  The kernel evaluates
//   u = fma(SA, rho32, ACC)             one rounding, of the small difference: the two
//                                       large terms cancel inside the fma
//   t = fma(u, A32, fma(SA, B32, s32))  B = A*(rho - rho32): the part of rho that
//                                       binary32 drops
// The exact sequence (fp32 value of the layer, times scale, plus shift: three
// roundings) and this one (three roundings, four rounded constants) each differ from
// the real t by a few 2^-24 of |t| + S, S = |sh|/D_n + |c0|, in total less than
//   E = 2^-21*(2^bits + S) + 2^-45*|Q*sc/D_n|*SA_max
// for t inside the code range (6|t| + 7S times 2^-24 to first order; the last term
// covers the rounding of B and of the fma that uses it).  Outside the range both
// clamp alike when E < 1/2.  Returns te = margin - E (margin: see DsqConvArgs), what
// |fract(t) - 1/2| must stay below for floor(t) to be the exact sequence's code;
// te = -1 (never safe) for channels whose magnitudes would let an intermediate of
// either sequence overflow, or lose bits to denormals, and when the host disabled
// the form: those keep harmless constants, so that t stays finite.  Channels past
// C_out get constants that give code 0 safely (their bytes are blanked anyway).
//
// `unit`: the kernel's accumulators hold ACC/unit (the FP4 form counts in quarter
// units): A*unit and rho32/unit are stored, both exact scalings by a power of two.
__device__ __forceinline__ float chained_channel_constants(const DsqConvArgs &a, int o, double P, double Q, float scale,
                                                           float shift, float unit, float4 &k)
{
    k = make_float4(0.f, 0.f, 0.f, 0.5f);
    if (o >= a.C_out) return 0.25f;
    const double sc = (double)scale, sh = (double)shift, inv_dn = a.rq_inv_dn;
    const double rho = Q / P;
    const float rho32 = (float)rho;
    const double A = P * sc * inv_dn;
    const double s = __builtin_fma(sh, inv_dn, a.rq_c0);
    const double S = __builtin_fabs(sh) * inv_dn + __builtin_fabs(a.rq_c0);
    const double samax = (double)a.rq_sa_max;
    const double E = 0x1p-21 * ((double)(1 << a.rq_bits) + S) + 0x1p-45 * __builtin_fabs(Q * sc * inv_dn) * samax;
    const double ymax = (__builtin_fabs(P) * (double)a.rq_w_max + __builtin_fabs(Q)) * samax;    // bound on the layer's |output|
    // (every comparison is false for a NaN, which then ends in te = -1)
    const bool ok = a.rq_fast && ymax < 0x1p100 && ymax * __builtin_fabs(sc) < 0x1p100 && __builtin_fabs(sh) < 0x1p100 &&
                    (__builtin_fabs(sc) + 1.0) * inv_dn < 0x1p100 && __builtin_fabs(A) < 0x1p60 &&
                    __builtin_fabs(rho) < 0x1p20 && E < (double)a.rq_t_margin;
    if (!ok) return -1.0f;
    k = make_float4((float)A * unit, rho32 / unit, (float)(A * (rho - (double)rho32)), (float)s);
    return (float)((double)a.rq_t_margin - E);
}

// RQ selects the chained-mode epilogue at compile time, so that the plain
// kernels' register allocation is exactly what it is without that mode.
template <int CONT, int R, int WP, int WC, int PF, int CT, int UPT, int WD, int OCC, int KS, bool RQ>
__global__ __launch_bounds__(256 * KS) __attribute__((amdgpu_waves_per_eu(OCC, OCC))) void conv_patch_kernel(DsqConvArgs a, PatchPlan pl)
{
    constexpr int T = R * R;
    // CONT: 2 / 4 = container width of the packed activation codes, 3 = dense 3-bit units
    // (12 bytes per 32 channels; everything after the patch store is the 4-bit path)
    constexpr int UPP = CONT == 2 ? 1 : 2;        // fetch units per patch pixel and 64 channels
    constexpr int UNIT_B = CONT == 3 ? 12 : 16;   // bytes of a fetch unit
    constexpr int KB_BYTES = 64 * CONT / 8;       // packed bytes of 64 channels
    constexpr int WLANE = 16;                     // weight bytes per lane per (tile, cb, tap)
    constexpr bool F4 = CONT == 2;                // 2-bit layers run on the FP4 matrix instruction
    constexpr int KH = F4 ? 1 : 2;                // matrix instructions per 64 channels
    constexpr int PIX_STRIDE = pix_stride(CONT);
    static_assert(WP * WC == 4, "four waves per workgroup");
    static_assert(64 * CT * WC <= 256, "one thread per staged channel constant");
    typedef v4i wpack_t;
    typedef typename std::conditional<F4, v16f, v16i>::type macc_t;   // main-loop accumulator

    extern __shared__ __attribute__((aligned(16))) char lds[];
    // LDS: [patch buffer 0][patch buffer 1] (re-used by the epilogue as staging)
    //      at aux_off: [double Da*Dw[BC]][double Da*l_w[BC]]
    //                  [int pixel code sums of the patch, PR*PC]
    constexpr int BC = 32 * CT * WC;
    double *pq_lds = reinterpret_cast<double *>(lds + pl.aux_off);
    int *pix_lds = reinterpret_cast<int *>(pq_lds + 2 * BC);
    // chained mode: scale and shift of the workgroup's channels (16-byte aligned)
    float *ss_lds = reinterpret_cast<float *>(lds + ((pl.aux_off + 2 * BC * 8 + pl.PR * pl.PC * 4 + 15) & ~15));
    // chained mode: the next quantizer's thresholds as 16 (lower, upper) pairs
    float2 *thr_lds = reinterpret_cast<float2 *>(ss_lds + 2 * BC);
    // chained mode: per channel the constants (A, rho, B, s) of the code-unit form, and the
    // largest distance from 1/2 of the fraction of t at which every channel's code is safe
    float4 *ft_lds = reinterpret_cast<float4 *>(thr_lds + 16);
    int *te_lds = reinterpret_cast<int *>(ft_lds + BC);              // (the bits of a float: see below)

    // KS = 2: two groups of four waves work on alternating 64-channel blocks of K
    // (each with its own patch buffers) and add their accumulators at the end, so
    // that every SIMD hosts two waves whose MFMA and VALU phases can overlap even
    // when the layer yields only one workgroup per CU.
    static_assert(KS == 1 || KS == 2, "one or two wave groups");
    const int tid = threadIdx.x & 255;                 // thread index inside its wave group
    const int lane = tid & 63;
    const int grp = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index inside the group
    const int col = lane & 31, h = lane >> 5;
    const int wp = wave % WP, wc = wave / WP;

    // The kernel arguments live in memory that is slow to reach.  Naming all of
    // them as scalar-register inputs of an (empty) asm statement right here makes
    // the compiler fetch them in one batch at the top of the kernel -- one round
    // trip instead of one per group of first uses -- at no instruction cost.
    asm volatile("" ::"s"(a.N), "s"(a.C_in), "s"(a.H), "s"(a.W), "s"(a.C_out), "s"(a.stride), "s"(a.pad),
                 "s"(a.bits), "s"(a.Ho), "s"(a.Wo), "s"(a.Cp), "s"(a.out_nchw), "s"(a.R), "s"(a.Cop),
                 "s"(a.l_a), "s"(a.u_a), "s"(a.delta_a), "s"(a.act), "s"(a.pix_sum), "s"(a.wq), "s"(a.delta_w), "s"(a.l_w),
                 "s"(a.out), "s"(a.acc));
    asm volatile("" ::"s"(pl.TW), "s"(pl.BP), "s"(pl.tiles_w), "s"(pl.PR), "s"(pl.PC), "s"(pl.RP),
                 "s"(pl.buf_bytes), "s"(pl.Hp), "s"(pl.aux_off), "s"(pl.step_q), "s"(pl.step_r),
                 "s"(pl.tiles_c), "s"(pl.total_blocks), "s"(pl.xcd_chunk), "s"(pl.mg_tiles_c), "s"(pl.mg_PC),
                 "s"(pl.mg_TW), "s"(pl.mg_Hp), "s"(pl.mg_Ho), "s"(pl.mg_tiles_w));

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give
    // every XCD a contiguous range of tiles, channel tiles of one pixel tile
    // first, so that the tiles that share activations (same pixels, halo rows of
    // neighbours) meet in one L2.
    const int logical = ((int)blockIdx.x & 7) * pl.xcd_chunk + ((int)blockIdx.x >> 3);
    if (logical >= pl.total_blocks) return;
    int blk_y;
    const int blk_x = idiv(logical, pl.tiles_c, pl.mg_tiles_c, blk_y);

    const int NCB = a.Cp / 64;
    const int NHo = a.N * a.Ho;

    // ---- weights first: their addresses need only the lane and block ids ----
    // lane-ordered fragments, [ct][cb][tap][lane][both K halves]
    const int ct0 = (blk_y * WC + wc) * CT;
    const uint32_t lane_woff = (uint32_t)lane * WLANE;
    // Packed weight fragments travel WD taps ahead of their use in a ring of
    // registers (slot = tap % WD; WD divides the tap count); a slot is refilled as
    // soon as it has been unpacked.
    static_assert(T % WD == 0, "ring period must divide the taps of a stage");
    wpack_t wreg[CT][WD];
    auto fetch_weight = [&](int c, int t, int cb) {
        const char *p = (const char *)a.wq +
                        ((((size_t)(ct0 + c) * NCB + cb) * T + t) * 64) * WLANE + lane_woff;
        wreg[c][t % WD] = *reinterpret_cast<const wpack_t *>(p);
    };
    // (a group whose first channel block does not exist fetches block 0 and never uses it)
    const int cb_first = grp < NCB ? grp : 0;
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int t = 0; t < WD; ++t) fetch_weight(c, t, cb_first);


    // ---- tile position -------------------------------------------------------
    int tile_w;
    const int tile_r = idiv(blk_x, pl.tiles_w, pl.mg_tiles_w, tile_w);
    const int t0 = tile_r * pl.BP;              // first pixel of the tile, numbered inside the strip
    const int ow0 = tile_w * pl.TW;
    int tc0;
    const int gr0 = idiv(t0, pl.TW, pl.mg_TW, tc0);   // its output row (batch-wide numbering)
    int oh0;
    const int n0 = idiv(gr0, a.Ho, pl.mg_Ho, oh0);
    const int v0 = n0 * pl.Hp + oh0 * a.stride;   // first padded input row of the patch
    const int vc0 = ow0 * a.stride;               // first padded input column of the patch
    const uint32_t row_bytes = (uint32_t)a.Cp * CONT / 8;

    // ---- per-thread fetch units of the patch ---------------------------------
    // unit u = tid + 256*k covers half `u % UPP` of patch pixel u / UPP; (prow, pcol)
    // and the image row behind prow advance by fixed steps from unit to unit
    uint32_t src_off[UPT];   // byte offset into act of the unit at channel block 0
    uint32_t src_pix[UPT];   // index of the unit's input pixel (0 if none)
    int dst_off[UPT];        // LDS byte offset inside a patch buffer (dump slot if no such unit)
    uint32_t src_valid = 0;  // bit k: unit k reads real data (else: zero padding)
    const int dump_off = pl.buf_bytes - 64;
    const int half = UPP == 2 ? (tid & 1) : 0;
    {
        int pcol, ihp;
        int prow = idiv(UPP == 2 ? (tid >> 1) : tid, pl.PC, pl.mg_PC, pcol);
        int n = idiv(v0 + prow, pl.Hp, pl.mg_Hp, ihp);
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            const int ih = ihp - a.pad, iw = vc0 + pcol - a.pad;
            const bool inpatch = prow < pl.PR;
            const bool valid = inpatch && n < a.N && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const uint32_t pix = valid ? (uint32_t)((n * a.H + ih) * a.W + iw) : 0u;
            src_pix[k] = pix;
            src_off[k] = pix * row_bytes + half * UNIT_B;
            dst_off[k] = inpatch ? prow * pl.RP + pcol * PIX_STRIDE + half * 32 : dump_off;
            src_valid |= (valid ? 1u : 0u) << k;
            int dp = pl.step_q;
            pcol += pl.step_r;
            if (pcol >= pl.PC) { pcol -= pl.PC; ++dp; }
            prow += dp;
            ihp += dp;
            while (ihp >= pl.Hp) { ihp -= pl.Hp; ++n; }  // seldom more than once
        }
    }

    v4i pre[UPT];            // packed patch units in flight
    auto fetch_patch = [&](int cb) {
        const char *base = (const char *)a.act + (size_t)cb * KB_BYTES;
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            if constexpr (CONT == 3) {
                typedef int v3i __attribute__((ext_vector_type(3)));
                const v3i t = *reinterpret_cast<const v3i *>(base + src_off[k]);      // (4-byte aligned)
                pre[k] = (v4i){t.x, t.y, t.z, 0};
            } else {
                pre[k] = *reinterpret_cast<const v4i *>(base + src_off[k]);
            }
        }
    };
    auto store_units = [&](char *buf, const v4i (&units)[UPT]) {
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            const v4i pk = (src_valid >> k & 1) ? units[k] : (v4i){0, 0, 0, 0};
            char *d = buf + dst_off[k];
            if (CONT == 3) {
                // 12 packed bytes = 32 channels -> 32 int8
                uint32_t g[8];
                dsq_unpack32_d3((uint32_t)pk.x, (uint32_t)pk.y, (uint32_t)pk.z, g);
                *reinterpret_cast<v4i *>(d) = (v4i){(int)g[0], (int)g[1], (int)g[2], (int)g[3]};
                *reinterpret_cast<v4i *>(d + 16) = (v4i){(int)g[4], (int)g[5], (int)g[6], (int)g[7]};
            } else if (CONT == 4) {
                // 16 packed bytes = 32 channels -> 32 int8
                *reinterpret_cast<v4i *>(d) = dsq_unpack16_c4((v2i){pk.x, pk.y});
                *reinterpret_cast<v4i *>(d + 16) = dsq_unpack16_c4((v2i){pk.z, pk.w});
            } else {
                // 16 packed bytes = 64 channels -> two K groups of 32 FP4 nibbles
                *reinterpret_cast<v4i *>(d) = dsq_fp4_from_c2((uint32_t)pk.x, (uint32_t)pk.y);
                *reinterpret_cast<v4i *>(d + 16) = dsq_fp4_from_c2((uint32_t)pk.z, (uint32_t)pk.w);
            }
        }
    };
    auto store_patch = [&](char *buf) { store_units(buf, pre); };
    fetch_patch(cb_first);
    // side tables, needed only after the main loop: the pixels' code sums and the
    // per-channel dequantization constants of this workgroup's channels
    int pix_val[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) pix_val[k] = a.pix_sum[src_pix[k]];
    // (every lane loads an entry, used or not: a load under a branch would drag
    // the wait for it, and for everything issued before it, up to this point)
    const int chan_i = tid < 2 * BC ? tid : 0;
    const int chan_o = blk_y * BC + (chan_i < BC ? chan_i : chan_i - BC);      // < Cop by construction
    const float chan_const = (chan_i < BC ? a.delta_w : a.l_w)[chan_o];
    float rq_const = 0.f;
    if (RQ && grp == 0 && tid < 2 * BC) {
        const int o = blk_y * BC + (tid < BC ? tid : tid - BC);
        const float *tab = tid < BC ? a.rq_scale : a.rq_shift;
        rq_const = tab != nullptr && o < a.C_out ? tab[o] : (tid < BC ? 1.0f : 0.0f);
    }

    // ---- per-lane LDS offsets of the fragments' pixels -----------------------
    // Tile pixels past the end of the strip multiply patch pixel 0 and are
    // never stored.
    int frag_off[PF];       // byte offset of the pixel's first tap inside a patch buffer
    int frag_pp[PF];        // index of that patch pixel (prow*PC + pcol)
    int frag_m[PF];         // output pixel index n*Ho*Wo + oy*Wo + ox, or -1
#pragma unroll
    for (int f = 0; f < PF; ++f) {
        const int t = t0 + (wp * PF + f) * 32 + col;
        int tc;
        const int gr = idiv(t, pl.TW, pl.mg_TW, tc);
        const int ow = ow0 + tc;
        const bool ok = gr < NHo && ow < a.Wo;
        int prow = 0, pcol = 0;
        if (ok) {
            int oh;
            const int n = idiv(gr, a.Ho, pl.mg_Ho, oh);
            prow = n * pl.Hp + oh * a.stride - v0;
            pcol = tc * a.stride;
        }
        frag_m[f] = ok ? gr * a.Wo + ow : -1;
        frag_pp[f] = prow * pl.PC + pcol;
        frag_off[f] = prow * pl.RP + pcol * PIX_STRIDE + 16 * h;
    }

    macc_t macc[PF][CT];
    const macc_t zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int f = 0; f < PF; ++f)
#pragma unroll
        for (int c = 0; c < CT; ++c) macc[f][c] = zero16;

    // One stage: all taps of 64 input channels.  HAS_NEXT: the weights and the
    // patch of stage next_cb are fetched / stored on the way.
    auto compute = [&](auto has_next, const char *buf, int cur_cb, int next_cb, char *nextbuf) {
        constexpr bool HAS_NEXT = decltype(has_next)::value;
        v4i af[2][PF][KH];
#pragma unroll
        for (int f = 0; f < PF; ++f)
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)
                af[0][f][kh] = *reinterpret_cast<const v4i *>(buf + frag_off[f] + 32 * kh);
        // (keep these LDS reads first in the stage: their latency then runs under the
        // unpacking of the first weight fragments instead of in front of the first MFMA.
        // Only where registers are plentiful: the one-group variants spill under
        // this constraint.)
        if constexpr (KS == 2) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            if (t + 1 < T) {
                const int tap_off = ((t + 1) / R) * pl.RP + ((t + 1) % R) * PIX_STRIDE;
#pragma unroll
                for (int f = 0; f < PF; ++f)
#pragma unroll
                    for (int kh = 0; kh < KH; ++kh)
                        af[(t + 1) & 1][f][kh] =
                            *reinterpret_cast<const v4i *>(buf + frag_off[f] + tap_off + 32 * kh);
            }
            v4i wf[CT][KH];
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const wpack_t wr = wreg[c][t % WD];
                if (F4) {
                    wf[c][0] = wr;                       // FP4 nibbles go to the matrix cores as they are
                } else {
                    wf[c][0] = dsq_unpack16_c4((v2i){wr[0], wr[1]});
                    wf[c][KH - 1] = dsq_unpack16_c4((v2i){wr[2], wr[3]});
                }
                if (t + WD < T) fetch_weight(c, t + WD, cur_cb);
                else if (HAS_NEXT) fetch_weight(c, t + WD - T, next_cb);
            }
            // (the loads just issued stay in front of this tap's matrix instructions:
            // left to itself the scheduler sinks each weight load to right before its
            // use, WD taps later, which exposes the full load latency at every tap.  Not
            // where the patch prefetch or the 4-bit 256x128 tile holds many registers (the
            // variants then spill), not on the 4-bit 128x128 tile (measured 3 % slower), and
            // not with two wave groups, where it measured slower)
            if constexpr (UPT <= 4 && KS == 1 && !(CONT >= 3 && (PF == 4 || (PF == 2 && WP == 2)))) __builtin_amdgcn_sched_barrier(0);
            // consecutive MFMAs go to different accumulators
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                for (int c = 0; c < CT; ++c)
#pragma unroll
                    for (int f = 0; f < PF; ++f) {
                        if constexpr (F4)
                            macc[f][c] = dsq_mfma_fp4(wf[c][kh], af[t & 1][f][kh], macc[f][c]);
                        else
                            macc[f][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[c][kh], af[t & 1][f][kh], macc[f][c], 0, 0, 0);
                    }
            // half way through the taps the next stage's patch has arrived:
            // unpack it into the other buffer while the matrix cores are busy
            if (HAS_NEXT && t == (T / 2)) store_patch(nextbuf);
        }
    };

    // patch buffers: [parity][group]
    auto patch_buf = [&](int parity) { return lds + (parity * KS + grp) * pl.buf_bytes; };
    // (have the fragment offsets computed here, under the latency of the patch
    // fetch, rather than after the barrier where nothing hides them)
#pragma unroll
    for (int f = 0; f < PF; ++f) asm volatile("" ::"v"(frag_off[f]), "v"(frag_pp[f]), "v"(frag_m[f]));
    // (likewise the zeroing of the accumulators, where registers are plentiful)
    if constexpr (KS == 2) {
#pragma unroll
        for (int f = 0; f < PF; ++f)
#pragma unroll
            for (int c = 0; c < CT; ++c) asm volatile("" : "+v"(macc[f][c]));
    }
    store_patch(patch_buf(0));
    if (grp == 0) {
        int pp = UPP == 2 ? (tid >> 1) : tid;
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            if (pp < pl.PR * pl.PC && half == 0) pix_lds[pp] = (src_valid >> k & 1) ? pix_val[k] : 0;
            pp += 256 / UPP;
        }
        // Da*Dw[o] and Da*l_w[o] of this workgroup's channels, in binary64
        const double da0 = (double)a.delta_a;
        if (tid < 2 * BC) pq_lds[tid] = da0 * (double)chan_const;
        if (RQ && tid < 2 * BC) ss_lds[tid] = rq_const;
        if (RQ && tid < 16) {
            // pair c = (thr[c], thr[c+1]); -inf below the first threshold, NaN above the last
            float lo = -__builtin_inff(), hi = __builtin_nanf("");
#pragma unroll
            for (int j = 1; j < 16; ++j) {
                lo = tid == j ? a.rq_thr[j] : lo;
                hi = tid + 1 == j ? a.rq_thr[j] : hi;
            }
            thr_lds[tid] = make_float2(lo, hi);
            if (tid == 0) *te_lds = __float_as_int(0.5f);
        }
    }
    lds_barrier();

    // stage i of this group works on channel block grp + i*KS.  Stages that have a
    // successor prefetch it; the last stage of a group is peeled off the loop.
    const int n_iter = (NCB + KS - 1) / KS;                  // stages of group 0
    const int n_full = (NCB - 1 - grp) / KS;                 // stages of this group with a successor
    for (int i = 0; i < n_full; ++i) {
        const int cb = grp + i * KS;
        fetch_patch(cb + KS);
        compute(std::true_type{}, patch_buf(i & 1), cb, cb + KS, patch_buf((i + 1) & 1));
        lds_barrier();
    }
    // ---- side values of the epilogue (see conv_epilogue.h for the algebra) ------
    const int top = (1 << a.bits) - 1;
    const float delta_a = a.delta_a;
    // fast path: NHWC fp32 output only, l_a = 0, C_out a multiple of 4
    const bool fast = !a.out_nchw && (a.C_out & 3) == 0 && a.l_a == 0.0f && a.acc == nullptr;
    // per fragment: SA = code sums of the patch pixels under the taps (0 in the padding)
    double dsa[PF];
    float fsa[PF];          // (the same sums in binary32: exact, they stay below 2^24 wherever this is used)
    auto sum_sa = [&]() {
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            int sa = 0;
#pragma unroll
            for (int t = 0; t < T; ++t) sa += pix_lds[frag_pp[f] + (t / R) * pl.PC + (t % R)];
            dsa[f] = (double)sa;
            fsa[f] = (float)sa;
        }
    };
    // Da*Dw and Da*l_w of this lane's channels of one tile: 4 groups of 4
    auto load_pq = [&](int c, double (&P)[16], double (&Q)[16]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ol = (wc * CT + c) * 32 + 8 * q + 4 * h;   // channel inside the workgroup
#pragma unroll
            for (int j = 0; j < 4; ++j) { P[4 * q + j] = pq_lds[ol + j]; Q[4 * q + j] = pq_lds[BC + ol + j]; }
        }
    };
    // With two wave groups (two waves per SIMD, registers to spare) a wave finishes a
    // single tile; its constants and code sums are fetched before the last stage so
    // that these LDS reads run under the matrix instructions instead of after them.
    // (The tables were written before the first barrier.)
    double P0[16], Q0[16];
    const bool early_tables = KS == 2 && CT == 2;
    if (early_tables) {
        sum_sa();
        if (fast) load_pq(grp, P0, Q0);
    }
    if (grp + n_full * KS < NCB) compute(std::false_type{}, patch_buf(n_full & 1), grp + n_full * KS, 0, nullptr);
    // every wave of the workgroup takes part in n_iter - 1 stage barriers
    if (KS > 1)
        for (int i = n_full; i < n_iter - 1; ++i) lds_barrier();

    // the exact integer sums (the FP4 form accumulates them in quarter units)
    v16i acc[PF][CT];
    if constexpr (!(RQ && F4 && KS == 1)) {
#pragma unroll
        for (int f = 0; f < PF; ++f)
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                if constexpr (F4) acc[f][c] = dsq_fp4_acc_to_int(macc[f][c]);
                else acc[f][c] = macc[f][c];
            }
    }

    // ---- epilogue --------------------------------------------------------------
    if (!early_tables) sum_sa();

    // The results of a 32x32 tile sit in the lanes as [pixel = lane%32][4 groups
    // of 4 channels].  They are staged through this wave's slice of the (now idle)
    // patch buffers so that each store instruction writes the 32 consecutive
    // channels (128 bytes) of 8 pixels instead of 16 bytes of 32 pixels.
    constexpr int ROWB = 128 + 16;                // staged bytes per pixel (+16: bank spread)
    constexpr int EPI_WAVE = 32 * ROWB + PF * 128;
    // chained mode, one wave group: the code-unit form reads the FP4 accumulators as
    // they are (quarter units); the integers are only formed where the exact sequence runs
    constexpr bool RAWF = RQ && F4 && KS == 1;
    if (RQ && grp == 0 && tid < BC) {
        const float te = chained_channel_constants(a, blk_y * BC + tid, pq_lds[tid], pq_lds[BC + tid], ss_lds[tid],
                                                   ss_lds[BC + tid], RAWF ? 4.0f : 1.0f, ft_lds[tid]);
        // the smallest margin of the workgroup's channels: reduced over the wave first
        // (BC is a multiple of 64, so whole waves get here), then one LDS operation per
        // wave (te is -1 or in (0, 1/2]: as signed integers the bit patterns of such
        // floats are ordered like the floats)
        float m = te;
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) m = __builtin_fminf(m, __shfl_xor(m, sft));
        if (lane == 0) atomicMin(te_lds, __float_as_int(m));
    }
    lds_barrier();                              // every wave is done with the patch buffers
    if (KS == 2) {
        // each group finishes the channel tiles c with c % 2 == grp: it hands the
        // partial sums of the other tiles to its partner wave through LDS and adds
        // the partner's partial sums to its own tiles (integer adds: exact in any
        // order)
        static_assert(KS == 1 || CT % 2 == 0, "two wave groups split the channel tiles evenly");
        char *part = lds + 8 * EPI_WAVE + lane * 16;
        const int mine = (grp * 4 + wave) * (PF * (CT / 2) * 4096);
        const int theirs = ((1 - grp) * 4 + wave) * (PF * (CT / 2) * 4096);
#pragma unroll
        for (int f = 0; f < PF; ++f)
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                if ((c & 1) == grp) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<v4i *>(part + mine + ((f * (CT / 2) + c / 2) * 4 + q) * 1024) =
                        (v4i){acc[f][c][4 * q], acc[f][c][4 * q + 1], acc[f][c][4 * q + 2], acc[f][c][4 * q + 3]};
            }
        lds_barrier();
#pragma unroll
        for (int f = 0; f < PF; ++f)
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                if ((c & 1) != grp) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4i o4 = *reinterpret_cast<const v4i *>(part + theirs + ((f * (CT / 2) + c / 2) * 4 + q) * 1024);
                    acc[f][c][4 * q] += o4.x; acc[f][c][4 * q + 1] += o4.y;
                    acc[f][c][4 * q + 2] += o4.z; acc[f][c][4 * q + 3] += o4.w;
                }
            }
    }
    char *stage = lds + (grp * 4 + wave) * EPI_WAVE;
    int *m_stage = reinterpret_cast<int *>(stage + 32 * ROWB);

    if (RQ) {
        // chained mode: the next layer's packed codes and pixel code sums instead
        // of the fp32 tensor (no transposition needed: a lane pair holds whole
        // 8-channel words of its pixel)
        int psum[PF];
#pragma unroll
        for (int f = 0; f < PF; ++f) psum[f] = 0;
        // (l_a = 0 here: the host sends chained layers with l_a != 0 to the simple
        // kernel.  Constants are fetched four channels at a time, right before
        // their use, to keep the register footprint of this path small.  Lanes of tile
        // pixels past the end compute on patch pixel 0 and are never stored; at worst
        // they send their wave through the exact sequence once more.)
        const int top_n = (1 << a.rq_bits) - 1;
        const float relu_floor = a.rq_relu ? 0.0f : -__builtin_inff();
        const float l_n = a.rq_l, u_n = a.rq_u, inv_delta_n = a.rq_inv_delta;
        const float t_lo = a.rq_t_lo, t_hi = a.rq_t_hi;
        const float te_wg = __int_as_float(*te_lds);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (KS == 2 && (c & 1) != grp) continue;
            const int o_tile = (ct0 + c) * 32;
            const int ol = (wc * CT + c) * 32 + 4 * h;   // this lane's first channel inside the workgroup
            // bytes of channels >= C_out are blanked (their codes must be 0)
            uint32_t mask[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int left = a.C_out - (o_tile + 8 * q + 4 * h);      // valid channels from here on
                mask[q] = left >= 4 ? 0xFFFFFFFFu : left <= 0 ? 0u : (1u << (8 * left)) - 1u;
            }
            // The code in code units, t = A*(ACC + rho*SA) + (B*SA + s) (see
            // chained_channel_constants): seven or eight binary32 instructions per output,
            // no binary64; the constants of four channels serve all fragments.  far[f]: the
            // largest distance of a fract(t) from 1/2 among the outputs of fragment f.
            uint32_t bytes[PF][4];
            float far[PF];
#pragma unroll
            for (int f = 0; f < PF; ++f) far[f] = 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float4 k[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) k[j] = ft_lds[ol + 8 * q + j];
#pragma unroll
                for (int f = 0; f < PF; ++f) {
                    int cd[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float fa;
                        if constexpr (RAWF) fa = macc[f][c][4 * q + j];
                        else fa = (float)acc[f][c][4 * q + j];
                        const float u = __builtin_fmaf(fsa[f], k[j].y, fa);
                        const float t = __builtin_fmaf(u, k[j].x, __builtin_fmaf(fsa[f], k[j].z, k[j].w));
                        const float tc = __builtin_amdgcn_fmed3f(t, t_lo, t_hi);
                        cd[j] = (int)tc;
                        far[f] = __builtin_fmaxf(far[f], __builtin_fabsf(__builtin_amdgcn_fractf(tc) - 0.5f));
                    }
                    bytes[f][q] = dsq_bytes4(cd[0], cd[1], cd[2], cd[3]) & mask[q];
                }
            }
#pragma unroll
            for (int f = 0; f < PF; ++f) {
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(far[f] < te_wg)) != 0, 0)) {
                    // the exact sequence: the binary32 value the plain call stores, scale,
                    // shift, ReLU and the quantizer as a step function
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float y[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            int ai;
                            if constexpr (RAWF) ai = (int)(macc[f][c][4 * q + j] * 4.0f);
                            else ai = acc[f][c][4 * q + j];
                            y[j] = (float)__builtin_fma(pq_lds[ol + 8 * q + j], (double)ai, pq_lds[BC + ol + 8 * q + j] * dsa[f]);
                        }
                        const float4 s4 = *reinterpret_cast<const float4 *>(ss_lds + ol + 8 * q);
                        const float4 b4 = *reinterpret_cast<const float4 *>(ss_lds + BC + ol + 8 * q);
                        const float sc[4] = {s4.x, s4.y, s4.z, s4.w}, sh[4] = {b4.x, b4.y, b4.z, b4.w};
                        bytes[f][q] = dsq_requant4_thr(y, sc, sh, relu_floor, l_n, u_n, inv_delta_n, top_n, thr_lds, mask[q]);
                    }
                }
                const int sum = (int)__builtin_amdgcn_sad_u8(bytes[f][3], 0u, __builtin_amdgcn_sad_u8(bytes[f][2], 0u,
                                __builtin_amdgcn_sad_u8(bytes[f][1], 0u, __builtin_amdgcn_sad_u8(bytes[f][0], 0u, 0u))));
                psum[f] += dsq_requant_store32(a, frag_m[f], o_tile, h, bytes[f], sum);
            }
        }
        // The waves that share a row of pixel fragments (wave columns, wave groups)
        // hand their sums to the row's first wave through their staging slices
        // (integer adds: exact in any order) ...
        constexpr int SHARE = WC * KS;
        const bool share = SHARE > 1 && a.rq_share;      // (uniform; otherwise every wave adds its own sums)
        const bool first = !share || (wc == 0 && grp == 0);
        if (share) {
            if (!first && h == 0) {
#pragma unroll
                for (int f = 0; f < PF; ++f) m_stage[f * 32 + col] = psum[f];
            }
            lds_barrier();
            if (first && h == 0) {
#pragma unroll
                for (int g = 0; g < KS; ++g)
#pragma unroll
                    for (int c2 = 0; c2 < WC; ++c2) {
                        if (g == 0 && c2 == 0) continue;
                        const int *theirs = reinterpret_cast<const int *>(lds + (g * 4 + wp + WP * c2) * EPI_WAVE + 32 * ROWB);
#pragma unroll
                        for (int f = 0; f < PF; ++f) psum[f] += theirs[f * 32 + col];
                    }
            }
        }
        // ... which adds them to the next layer's sums with one integer atomic per
        // pixel, or stores them where the workgroup holds all channels of the layer.
        // (The hand-over costs a barrier: measured, it pays where the sums can then
        // be stored and on 1x1 layers, whose time is mostly epilogue.)
        if (h == 0 && first) {
#pragma unroll
            for (int f = 0; f < PF; ++f) {
                if (frag_m[f] < 0) continue;
                if (a.rq_store) a.rq_pix[frag_m[f]] = psum[f];
                else atomicAdd(a.rq_pix + frag_m[f], psum[f]);
            }
        }
    } else if (fast) {
        if (h == 0) {
#pragma unroll
            for (int f = 0; f < PF; ++f) m_stage[f * 32 + col] = frag_m[f];
        }
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (KS == 2 && (c & 1) != grp) continue;
            double P[16], Q[16];
            if (KS == 2 && CT == 2) {
#pragma unroll
                for (int j = 0; j < 16; ++j) { P[j] = P0[j]; Q[j] = Q0[j]; }
            } else {
                load_pq(c, P, Q);
            }
            const int o = (ct0 + c) * 32 + (lane & 7) * 4;   // channels this lane stores
#pragma unroll
            for (int f = 0; f < PF; ++f) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    double v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] = __builtin_fma(P[4 * q + j], (double)acc[f][c][4 * q + j], Q[4 * q + j] * dsa[f]);
                    *reinterpret_cast<float4 *>(stage + col * ROWB + (8 * q + 4 * h) * 4) =
                        make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
                }
                // (LDS operations of one wave execute in order: no barrier needed)
                float4 rv[4];
                int rm[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int p = k * 8 + (lane >> 3);
                    rv[k] = *reinterpret_cast<const float4 *>(stage + p * ROWB + (lane & 7) * 16);
                    rm[k] = m_stage[f * 32 + p];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (rm[k] >= 0 && o < a.C_out)
                    {
                        // non-temporal: the output is not read again by this kernel, and
                        // streaming it out as it is produced leaves less for the write-back
                        // at the end of the kernel (measured 5-25 % off the kernel time of
                        // every layer class; a consumer that runs right after finds less of
                        // the tensor in the last-level cache, which costs it about as much)
                        typedef float v4f __attribute__((ext_vector_type(4)));
                        const v4f t = {rv[k].x, rv[k].y, rv[k].z, rv[k].w};
                        __builtin_nontemporal_store(t, reinterpret_cast<v4f *>(a.out + (size_t)rm[k] * a.C_out + o));
                    }
            }
        }
    } else {
        // general path: l_a != 0 (terms that depend on which taps are inside the
        // image), NCHW output, raw accumulators wanted, or C_out not a multiple of 4.
        // (the out-of-line function takes the arguments by reference: point it at the
        // kernel-argument segment, where `a` is the first argument, instead of copying the
        // structure to scratch memory -- the compiler hoists such a copy to the top of the
        // kernel, where it splits the one batch of argument loads into several round trips)
        const DsqConvArgs &a_copy = kernarg_conv_args();
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            const int m = frag_m[f];
            if (m < 0) continue;
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int o0 = (ct0 + c) * 32 + 8 * q + 4 * h;
                    if (o0 < a.C_out && (KS == 1 || (c & 1) == grp))
                        store4_general(a_copy, m, o0,
                                       (v4i){acc[f][c][4 * q], acc[f][c][4 * q + 1], acc[f][c][4 * q + 2], acc[f][c][4 * q + 3]},
                                       delta_a);
                }
        }
    }
}

// ---- host side ---------------------------------------------------------------

// m of idiv() for the divisor d >= 1
inline uint32_t division_constant(int d)
{
    const unsigned long long m = (1ull << 32) / (unsigned long long)d;
    return m > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)m;
}

inline int plan_lds_bytes(const PatchPlan &p, int BC, bool chained)
{
    // tables behind the buffers: Da*Dw, Da*l_w (binary64), the patch pixels' code
    // sums, the chained mode's scale, shift and quantizer thresholds and (chained
    // kernels only) its per-channel constants of the code-unit form
    return ((p.aux_off + 2 * BC * 8 + p.PR * p.PC * 4 + 15) & ~15) + 2 * BC * 4 + 16 * 8 + (chained ? BC * 16 + 16 : 0);
}

template <int CONT, int R, int WP, int WC, int PF, int CT, int UPT, int WD, int OCC, int KS, bool RQ>
hipError_t launch_kernel(const DsqConvArgs &a, const PatchPlan &pl, hipStream_t stream)
{
    auto kern = conv_patch_kernel<CONT, R, WP, WC, PF, CT, UPT, WD, OCC, KS, RQ>;
    const int BC = 32 * CT * WC;
    const size_t lds = (size_t)plan_lds_bytes(pl, BC, RQ);      // pl.aux_off already accounts for KS
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    // chained mode, layer wider than the tile: the workgroups add to the next
    // layer's pixel sums, which a fill kernel clears first (unless the caller did)
    if (RQ && !a.rq_store && !a.rq_zeroed) {
        const hipError_t e = dsq_launch_fill_zero(a.rq_pix, (size_t)a.N * a.Ho * a.Wo, stream);
        if (e != hipSuccess) return e;
    }
    PatchPlan p2 = pl;
    p2.tiles_c = (a.C_out + BC - 1) / BC;
    p2.mg_tiles_c = division_constant(p2.tiles_c);
    p2.total_blocks = pl.tiles_w * pl.row_tiles * p2.tiles_c;
    p2.xcd_chunk = (p2.total_blocks + 7) / 8;
    kern<<<dim3(8 * p2.xcd_chunk), 256 * KS, lds, stream>>>(a, p2);
    return hipGetLastError();
}

// Tile shapes (pixels x channels per workgroup; per wave PF x CT MFMA tiles):
//   small  128 x  64   waves 4x1, 1 x 2 tiles each  (few pixels: fill the chip)
//   medium 128 x 128   waves 2x2, 2 x 2
//   large  256 x 128   waves 2x2, 4 x 2
//   tall   256 x  64   waves 4x1, 2 x 2  (layers with at most 64 output channels)
template <int CONT, int R, int WP, int WC, int PF, int CT, int UPT, int WD, int OCC, int KS = 1>
hipError_t launch_cfg(const DsqConvArgs &a, const PatchPlan &pl, hipStream_t stream)
{
    if (a.rq) return launch_kernel<CONT, R, WP, WC, PF, CT, UPT, WD, OCC, KS, true>(a, pl, stream);
    return launch_kernel<CONT, R, WP, WC, PF, CT, UPT, WD, OCC, KS, false>(a, pl, stream);
}

enum { TILE_SMALL = 0, TILE_MEDIUM = 1, TILE_LARGE = 2, TILE_TALL = 3 };

// All variants of one (container, filter size) pair: tile, wave groups, and the
// number of 16-byte fetch units per thread (instantiated 2, 4, 8, 12).
// (The 128x64 tile with two fetch units per thread runs four waves per SIMD: layers of
// 784 k tiles, the 56x56 and 112x112 images, leave a nearly empty last round on 768
// resident workgroups; measured 5-8 % off such layers, 8-15 % off their chained call,
// no change elsewhere.)
template <int CONT, int RR>
hipError_t dispatch_variant(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream)
{
#define DSQ_TILE(CONT, RR, UPT)                                                                \
    do {                                                                                       \
        if (which == TILE_LARGE) {                                                             \
            if constexpr (CONT == 2) return launch_cfg<CONT, RR, 2, 2, 4, 2, UPT, (RR == 3 ? 3 : 1), 2>(a, pl, stream); \
            else return launch_kernel<CONT, RR, 2, 2, 4, 2, UPT, (RR == 3 ? 3 : 1), 2, 1, false>(a, pl, stream);  \
        }                                                                                      \
        if (which == TILE_MEDIUM && ks == 2) return launch_cfg<CONT, RR, 2, 2, 2, 2, UPT, (RR == 3 ? 3 : 1), 2, 2>(a, pl, stream); \
        if (which == TILE_MEDIUM) return launch_cfg<CONT, RR, 2, 2, 2, 2, UPT, (RR == 3 ? 3 : 1), 3>(a, pl, stream); \
        if (which == TILE_TALL) return launch_cfg<CONT, RR, 4, 1, 2, 2, UPT, (RR == 3 ? 3 : 1), 3>(a, pl, stream); \
        if (ks == 2) return launch_cfg<CONT, RR, 4, 1, 1, 2, UPT, (RR == 3 ? 3 : 1), 2, 2>(a, pl, stream); \
        return launch_cfg<CONT, RR, 4, 1, 1, 2, UPT, (RR == 3 ? 3 : 1), (UPT == 2 ? 4 : 3)>(a, pl, stream); \
    } while (0)
#define DSQ_GO(CONT, RR)                                                                       \
    do {                                                                                       \
        if (need <= 2) DSQ_TILE(CONT, RR, 2);                                                  \
        if (need <= 4) DSQ_TILE(CONT, RR, 4);                                                  \
        if (need <= 8) DSQ_TILE(CONT, RR, 8);                                                  \
        DSQ_TILE(CONT, RR, 12);                                                                \
    } while (0)
    DSQ_GO(CONT, RR);
#undef DSQ_TILE
#undef DSQ_GO
    return hipErrorInvalidValue;
}

}  // namespace

// One translation unit per (container, filter size) pair, so that they compile side by side.
hipError_t dsq_conv_patch_c4r3(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream);
hipError_t dsq_conv_patch_c4r1(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream);
hipError_t dsq_conv_patch_c2r3(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream);
hipError_t dsq_conv_patch_c2r1(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream);
hipError_t dsq_conv_patch_c3r3(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream);
hipError_t dsq_conv_patch_c3r1(const DsqConvArgs &a, const PatchPlan &pl, int which, int ks, int need, hipStream_t stream);
