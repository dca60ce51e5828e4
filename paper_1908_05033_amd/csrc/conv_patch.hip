// dsq_conv2d, LDS-patch kernel (the tuned path).
//
// GEMM view of Algorithm 1 step 5 of the paper: rows = output channels,
// columns = output pixels, K = filter taps x input channels, run on
// v_mfma_i32_16x16x64_i8 with int32 accumulation (the integer-arithmetic
// deployment of Sec. 3.5 / 4.5, re-designed for the matrix cores).
//
// A workgroup (4 wavefronts) owns a tile of TR output rows x TW output columns
// (TR*TW <= 16*FRAGS pixels; rows are counted through the whole batch, so a
// tile may span images) and BC = 16*CT*WC output channels.  K is walked in
// stages of 64 input channels.  For a stage, the input patch that all R*R taps
// of the tile touch is read from HBM/L2 once, unpacked from 2/4-bit codes to
// int8 and kept in LDS; the taps then read shifted windows of it, so the
// R*R-fold re-use of the activations never leaves the CU.  Positions of the
// patch that fall in the zero padding hold code 0: they add nothing to the
// integer sums, and the epilogue's SA/SW/KV terms leave them out as well.
// Weight fragments were laid out per lane by dsq_pack_weights and go from
// global memory straight to registers, one stage ahead.  The patch of the
// next stage is fetched while the current one is multiplied (two LDS buffers,
// one barrier per stage).
//
// LDS layout of a patch: pixel (prow, pcol) at prow*RP + pcol*80 bytes, 64
// bytes of int8 + 16 bytes of padding, so that the 16 pixels of a fragment
// (consecutive tile pixels) start in 16 different 16-byte bank groups; RP adds
// a per-row skew that keeps this true when a fragment wraps to the next row.
#include "conv_epilogue.h"

namespace {

constexpr int PIX_STRIDE = 80;   // LDS bytes per patch pixel (64 used)

struct PatchPlan {
    int TR, TW;        // tile: output rows x output columns
    int tiles_w;       // column tiles per output row
    int row_tiles;     // ceil(N*Ho / TR)
    int PR, PC;        // patch rows (max over tiles) x patch columns
    int RP;            // LDS bytes per patch row
    int buf_bytes;     // LDS bytes of one patch buffer
    int Hp;            // H + 2*pad: rows of one image in the padded row space
    int units;         // 16-byte fetch units per stage
};

template <int CONT, int R, int FRAGS, int WP, int WC, int CT, int UPT>
__global__ __launch_bounds__(256) void conv_patch_kernel(DsqConvArgs a, PatchPlan pl)
{
    constexpr int T = R * R;
    constexpr int WPL = CONT == 4 ? 2 : 1;        // packed weight words per lane per K64 block
    constexpr int UPP = CONT == 4 ? 2 : 1;        // 16-byte fetch units per patch pixel
    constexpr int KB_BYTES = 64 * CONT / 8;       // packed bytes of 64 channels
    constexpr int PF = (FRAGS + WP - 1) / WP;     // pixel fragments per wave (max)
    static_assert(WP * WC == 4, "four waves per workgroup");

    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, g = lane >> 4;
    const int wp = wave % WP, wc = wave / WP;

    const int tile_w = blockIdx.x % pl.tiles_w;
    const int tile_r = blockIdx.x / pl.tiles_w;
    const int NHo = a.N * a.Ho;
    const int gr0 = tile_r * pl.TR;             // first output row (batch-wide numbering)
    const int ow0 = tile_w * pl.TW;
    const int n0 = gr0 / a.Ho;
    const int v0 = n0 * pl.Hp + (gr0 - n0 * a.Ho) * a.stride;   // first padded input row
    const int vc0 = ow0 * a.stride;                              // first padded input column
    const int NCB = a.Cp / 64;
    const size_t row_bytes = (size_t)a.Cp * CONT / 8;
    const char *act = (const char *)a.act;

    // ---- per-thread fetch units of the patch -------------------------------
    int src_off[UPT];      // byte offset into act of the unit at channel block 0, or -1
    int dst_off[UPT];      // LDS byte offset inside a patch buffer, or -1 (no such unit)
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        const int u = tid + 256 * k;
        src_off[k] = -1;
        dst_off[k] = -1;
        if (u < pl.units) {
            const int pp = u / UPP, half = u - pp * UPP;
            const int prow = pp / pl.PC, pcol = pp - prow * pl.PC;
            dst_off[k] = prow * pl.RP + pcol * PIX_STRIDE + half * 32;
            const int v = v0 + prow;
            const int n = v / pl.Hp;
            const int ih = v - n * pl.Hp - a.pad;
            const int iw = vc0 + pcol - a.pad;
            if (n < a.N && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W)
                src_off[k] = (int)((((size_t)n * a.H + ih) * a.W + iw) * row_bytes) + half * 16;
        }
    }

    // ---- per-lane LDS offsets of the fragments' pixels ---------------------
    int frag_off[PF];
    int frag_gr[PF], frag_ow[PF];     // output row / column of this lane's pixel, -1 if none
#pragma unroll
    for (int f = 0; f < PF; ++f) {
        const int fi = wp + WP * f;                 // fragment index inside the tile
        const int t = fi * 16 + col;
        int tr = t / pl.TW, tc = t - tr * pl.TW;
        const int gr = gr0 + tr, ow = ow0 + tc;
        const bool ok = fi < FRAGS && tr < pl.TR && gr < NHo && ow < a.Wo;
        frag_gr[f] = ok ? gr : -1;
        frag_ow[f] = ow;
        int prow = 0, pcol = 0;
        if (ok) {
            const int n = gr / a.Ho;
            prow = n * pl.Hp + (gr - n * a.Ho) * a.stride - v0;
            pcol = tc * a.stride;
        }
        frag_off[f] = prow * pl.RP + pcol * PIX_STRIDE + 16 * g;
    }

    // ---- weights: lane-ordered fragments, [ct][cb][tap][lane][WPL] ---------
    const int ct0 = (blockIdx.y * WC + wc) * CT;
    const uint32_t *wq = (const uint32_t *)a.wq;
    auto wptr = [&](int c, int cb) {
        return wq + ((((size_t)(ct0 + c) * NCB + cb) * T) * 64 + lane) * WPL;
    };

    v4i acc[PF][CT];
#pragma unroll
    for (int f = 0; f < PF; ++f)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[f][c] = (v4i){0, 0, 0, 0};

    v4i pre[UPT];                 // packed patch units in flight
    uint32_t wreg[CT][T][WPL];    // packed weight fragments of the current stage; each is
                                  // refilled for the next stage as soon as it has been used

    auto fetch_patch = [&](int cb) {
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            pre[k] = (v4i){0, 0, 0, 0};
            if (src_off[k] >= 0)
                pre[k] = *reinterpret_cast<const v4i *>(act + (size_t)(uint32_t)src_off[k] + (size_t)cb * KB_BYTES);
        }
    };
    auto fetch_weight = [&](int c, int t, int cb) {
        const uint32_t *p = wptr(c, cb) + (size_t)t * 64 * WPL;
        if (WPL == 2) {
            v2i w2 = *reinterpret_cast<const v2i *>(p);
            wreg[c][t][0] = (uint32_t)w2.x;
            wreg[c][t][WPL - 1] = (uint32_t)w2.y;
        } else {
            wreg[c][t][0] = p[0];
        }
    };
    auto store_patch = [&](char *buf) {
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            if (dst_off[k] < 0) continue;
            char *d = buf + dst_off[k];
            if (CONT == 4) {
                // 16 packed bytes = 32 channels -> 32 int8
                *reinterpret_cast<v4i *>(d) = dsq_unpack16_c4((v2i){pre[k].x, pre[k].y});
                *reinterpret_cast<v4i *>(d + 16) = dsq_unpack16_c4((v2i){pre[k].z, pre[k].w});
            } else {
                // 16 packed bytes = 64 channels -> 64 int8
                *reinterpret_cast<v4i *>(d) = dsq_unpack2((uint32_t)pre[k].x);
                *reinterpret_cast<v4i *>(d + 16) = dsq_unpack2((uint32_t)pre[k].y);
                *reinterpret_cast<v4i *>(d + 32) = dsq_unpack2((uint32_t)pre[k].z);
                *reinterpret_cast<v4i *>(d + 48) = dsq_unpack2((uint32_t)pre[k].w);
            }
        }
    };
    // One stage: all taps of 64 input channels.  next_cb < 0: last stage.
    auto compute = [&](const char *buf, int next_cb, char *nextbuf) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int tap_off = (t / R) * pl.RP + (t % R) * PIX_STRIDE;
            v4i af[PF];
#pragma unroll
            for (int f = 0; f < PF; ++f)
                af[f] = *reinterpret_cast<const v4i *>(buf + frag_off[f] + tap_off);
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                v4i wf;
                if (CONT == 4) wf = dsq_unpack16_c4((v2i){(int)wreg[c][t][0], (int)wreg[c][t][WPL - 1]});
                else wf = dsq_unpack2(wreg[c][t][0]);
                if (next_cb >= 0) fetch_weight(c, t, next_cb);
#pragma unroll
                for (int f = 0; f < PF; ++f)
                    if (wp + WP * f < FRAGS)
                        acc[f][c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, af[f], acc[f][c], 0, 0, 0);
            }
            // half way through the taps the next stage's patch has arrived:
            // unpack it into the other buffer while the matrix cores are busy
            if (next_cb >= 0 && t == T / 2) store_patch(nextbuf);
        }
    };

    fetch_patch(0);
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int t = 0; t < T; ++t) fetch_weight(c, t, 0);
    store_patch(lds);
    __syncthreads();

    for (int cb = 0; cb < NCB; ++cb) {
        const bool more = cb + 1 < NCB;
        char *cur = lds + (cb & 1) * pl.buf_bytes;
        char *nxt = lds + ((cb + 1) & 1) * pl.buf_bytes;
        if (more) fetch_patch(cb + 1);
        compute(cur, more ? cb + 1 : -1, nxt);
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------
    const int top = (1 << a.bits) - 1;
    const float delta_a = dsq_delta(a.l_a, a.u_a, top);
    const int M = NHo * a.Wo;
#pragma unroll
    for (int f = 0; f < PF; ++f) {
        if (wp + WP * f >= FRAGS) continue;
        const int m = frag_gr[f] >= 0 ? frag_gr[f] * a.Wo + frag_ow[f] : M;
        const DsqPixel px = dsq_pixel_info(a, m, M);
#pragma unroll
        for (int c = 0; c < CT; ++c)
            dsq_store4(a, px, m, (ct0 + c) * 16 + 4 * g, acc[f][c], delta_a);
    }
}

// ---- host side: tile planning and dispatch ---------------------------------

struct TileCfg { int FRAGS, WP, WC, CT, UPT; };

// Picks TR x TW (TR*TW <= BP) minimising padded work, then patch size.
bool plan_patch(const DsqConvArgs &a, int BP, int UPT, int lds_limit, PatchPlan &best)
{
    const int cont = dsq_container(a.bits);
    const int UPP = cont == 4 ? 2 : 1;
    const int NHo = a.N * a.Ho;
    const int Hp = a.H + 2 * a.pad;
    bool found = false;
    long long best_cost = 0;
    for (int TW = 1; TW <= a.Wo && TW <= BP; ++TW) {
        int TR = BP / TW;
        if (TR > NHo) TR = NHo;
        if (TR < 1) continue;
        PatchPlan p;
        p.TR = TR; p.TW = TW; p.Hp = Hp;
        p.tiles_w = (a.Wo + TW - 1) / TW;
        p.row_tiles = (NHo + TR - 1) / TR;
        p.PC = (TW - 1) * a.stride + a.R;
        // patch rows: padded-row span of the tile's output rows, worst tile
        int PR = 0;
        for (int tr = 0; tr < p.row_tiles; ++tr) {
            int g0 = tr * TR, g1 = g0 + TR - 1;
            if (g1 >= NHo) g1 = NHo - 1;
            int nA = g0 / a.Ho, nB = g1 / a.Ho;
            int vA = nA * Hp + (g0 - nA * a.Ho) * a.stride;
            int vB = nB * Hp + (g1 - nB * a.Ho) * a.stride;
            int pr = vB - vA + a.R;
            if (pr > PR) PR = pr;
        }
        p.PR = PR;
        // row skew: consecutive tile pixels keep advancing by one pixel stride
        // (mod 256 bytes) when a fragment wraps from one tile row to the next
        int skew = ((TW * a.stride - p.PC) * PIX_STRIDE) % 256;
        if (skew < 0) skew += 256;
        // one output row down = `stride` patch rows down
        // (for stride 2 the skew is split over the two rows; any remainder is harmless)
        p.RP = p.PC * PIX_STRIDE + (a.stride == 1 ? skew : 0);
        p.buf_bytes = (p.PR * p.RP + 255) & ~255;
        p.units = p.PR * p.PC * UPP;
        if (2 * p.buf_bytes > lds_limit) continue;
        if (p.units > 256 * UPT) continue;
        const long long tiles = (long long)p.tiles_w * p.row_tiles;
        const long long cost = tiles * 100000 + (long long)p.PR * p.PC;
        if (!found || cost < best_cost) { best = p; best_cost = cost; found = true; }
    }
    return found;
}

template <int CONT, int R, int FRAGS, int WP, int WC, int CT, int UPT>
hipError_t launch_cfg(const DsqConvArgs &a, const PatchPlan &pl, hipStream_t stream)
{
    auto kern = conv_patch_kernel<CONT, R, FRAGS, WP, WC, CT, UPT>;
    const int BC = 16 * CT * WC;
    const size_t lds = 2 * (size_t)pl.buf_bytes;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    dim3 grid(pl.tiles_w * pl.row_tiles, (a.C_out + BC - 1) / BC);
    kern<<<grid, 256, lds, stream>>>(a, pl);
    return hipGetLastError();
}

// Tile shapes: small = 112 pixels x 64 channels, large = 224 x 128,
// tall = 224 x 64 (for layers with few output channels).
constexpr TileCfg kSmall = {7, 2, 2, 2, 4};
constexpr TileCfg kLarge = {14, 2, 2, 4, 8};
constexpr TileCfg kTall  = {14, 4, 1, 4, 8};

enum { TILE_SMALL = 0, TILE_LARGE = 1, TILE_TALL = 2 };

int pick_tile(const DsqConvArgs &a)
{
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long small_blocks = ((M + 111) / 112) * ((a.C_out + 63) / 64);
    if (a.C_out <= 64) return small_blocks >= 2048 ? TILE_TALL : TILE_SMALL;
    const long long large_blocks = ((M + 223) / 224) * ((a.C_out + 127) / 128);
    return large_blocks >= 1024 ? TILE_LARGE : TILE_SMALL;
}

const TileCfg &tile_cfg(int which)
{
    return which == TILE_LARGE ? kLarge : which == TILE_TALL ? kTall : kSmall;
}

constexpr int kLdsLimit = 150 * 1024;

}  // namespace

bool dsq_conv_patch_supported(const DsqConvArgs &a, int force_tile)
{
    if ((long long)a.N * a.H * a.W * (a.Cp * dsq_container(a.bits) / 8) > 0x7FFFFFFFLL) return false;
    PatchPlan pl;
    const TileCfg &tc = tile_cfg(force_tile >= 0 ? force_tile : pick_tile(a));
    return plan_patch(a, 16 * tc.FRAGS, tc.UPT, kLdsLimit, pl);
}

hipError_t dsq_launch_conv_patch(const DsqConvArgs &a, int force_tile, hipStream_t stream)
{
    const int which = force_tile >= 0 ? force_tile : pick_tile(a);
    const TileCfg &tc = tile_cfg(which);
    PatchPlan pl;
    if (!plan_patch(a, 16 * tc.FRAGS, tc.UPT, kLdsLimit, pl)) return hipErrorInvalidValue;
    const int cont = dsq_container(a.bits);
#define DSQ_GO(CONT, RR)                                                                       \
    do {                                                                                       \
        if (which == TILE_LARGE) return launch_cfg<CONT, RR, 14, 2, 2, 4, 8>(a, pl, stream);   \
        if (which == TILE_TALL) return launch_cfg<CONT, RR, 14, 4, 1, 4, 8>(a, pl, stream);    \
        return launch_cfg<CONT, RR, 7, 2, 2, 2, 4>(a, pl, stream);                             \
    } while (0)
    if (cont == 4) { if (a.R == 3) DSQ_GO(4, 3); else DSQ_GO(4, 1); }
    else           { if (a.R == 3) DSQ_GO(2, 3); else DSQ_GO(2, 1); }
#undef DSQ_GO
    return hipErrorInvalidValue;
}
