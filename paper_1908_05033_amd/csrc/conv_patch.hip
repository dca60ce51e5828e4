// dsq_conv2d, LDS-patch kernel: tile planning and dispatch (host side).  The
// kernel itself is in conv_patch_kernel.h.
#include <stdio.h>

#include "conv_patch_kernel.h"

namespace {

bool plan_patch(const DsqConvArgs &a, int BP, int BC, int PF, int CT, int UPT, int lds_limit, int KS, PatchPlan &best)
{
    // epilogue staging of the four waves (+ the partial sums of a second wave group)
    const int epi_bytes = 4 * KS * (32 * (128 + 16) + PF * 128) + (KS == 2 ? 8 * PF * (CT / 2) * 4096 : 0);
    const int cont = a.cont;
    const int UPP = cont == 2 ? 1 : 2;
    const int NHo = a.N * a.Ho;
    const int Hp = a.H + 2 * a.pad;
    bool found = false;
    long long best_cost = 0;
    for (int TW = 1; TW <= a.Wo; ++TW) {
        // widths that split the row evenly, the full row, or wide strips with a ragged last one
        const int tiles_w = (a.Wo + TW - 1) / TW;
        if (TW != a.Wo && a.Wo % TW != 0 && TW < 16) continue;
        PatchPlan p;
        p.TW = TW; p.BP = BP; p.Hp = Hp;
        p.tiles_w = tiles_w;
        const long long strip_pixels = (long long)NHo * TW;
        if (strip_pixels + BP >= (1 << 22)) continue;          // keeps every index well inside 32 bits
        p.row_tiles = (int)((strip_pixels + BP - 1) / BP);
        p.PC = (TW - 1) * a.stride + a.R;
        // patch rows: padded-row span of the tile's output rows, worst tile
        int PR = 0;
        for (int tr = 0; tr < p.row_tiles; ++tr) {
            long long tA = (long long)tr * BP, tB = tA + BP - 1;
            int g0 = (int)(tA / TW), g1 = (int)(tB / TW);
            if (g1 >= NHo) g1 = NHo - 1;
            int nA = g0 / a.Ho, nB = g1 / a.Ho;
            int vA = nA * Hp + (g0 - nA * a.Ho) * a.stride;
            int vB = nB * Hp + (g1 - nB * a.Ho) * a.stride;
            int pr = vB - vA + a.R;
            if (pr > PR) PR = pr;
        }
        p.PR = PR;
        // row skew: consecutive tile pixels keep advancing by one pixel stride
        // (mod 256 bytes) when a fragment wraps from one strip row to the next
        const int PIX_STRIDE = pix_stride(cont);
        int skew = ((TW * a.stride - p.PC) * PIX_STRIDE) % 256;
        if (skew < 0) skew += 256;
        p.RP = p.PC * PIX_STRIDE + (a.stride == 1 ? skew : 0);
        p.buf_bytes = (p.PR * p.RP + 64 + 255) & ~255;   // + dump slot for idle fetch units
        p.units = p.PR * p.PC * UPP;
        p.mg_TW = division_constant(TW); p.mg_Hp = division_constant(Hp); p.mg_Ho = division_constant(a.Ho);
        p.mg_PC = division_constant(p.PC); p.mg_tiles_w = division_constant(tiles_w);
        p.step_q = (256 / UPP) / p.PC;
        p.step_r = (256 / UPP) % p.PC;
        // a layer whose wave groups each see a single stage never touches the second
        // buffer of a group: leave it out, so that more workgroups fit a CU
        const int nbuf = a.Cp / 64 > KS ? 2 : 1;
        p.aux_off = nbuf * KS * p.buf_bytes > epi_bytes ? nbuf * KS * p.buf_bytes : epi_bytes;
        if (plan_lds_bytes(p, BC, a.rq != 0) > lds_limit) continue;
        if (p.units > 256 * UPT) continue;
        const long long tiles = (long long)p.tiles_w * p.row_tiles;
        // keep the operands of the index arithmetic small
        if (tiles * ((a.C_out + BC - 1) / BC) >= (1 << 22) || (long long)a.N * Hp >= (1 << 22) || NHo >= (1 << 22)) continue;
        // equal work: prefer a footprint that lets three (else two) workgroups share a CU,
        // then the smaller patch
        const int lds_bytes = plan_lds_bytes(p, BC, a.rq != 0);
        const long long cost = tiles * 100000 + (lds_bytes <= 52 * 1024 ? 0 : lds_bytes <= 78 * 1024 ? 20000 : 40000) +
                               (long long)p.PR * p.PC;
        if (!found || cost < best_cost) { best = p; best_cost = cost; found = true; }
    }
    return found;
}

struct TileCfg { int WP, WC, PF, CT; };
constexpr TileCfg kSmall  = {4, 1, 1, 2};
constexpr TileCfg kMedium = {2, 2, 2, 2};
constexpr TileCfg kLarge  = {2, 2, 4, 2};
constexpr TileCfg kTall   = {4, 1, 2, 2};
constexpr int kMaxUPT = 12;      // most 16-byte patch units a thread fetches per stage


const TileCfg &tile_cfg(int which)
{
    return which == TILE_LARGE ? kLarge : which == TILE_MEDIUM ? kMedium : which == TILE_TALL ? kTall : kSmall;
}

int pick_tile(const DsqConvArgs &a)
{
    const long long M = (long long)a.N * a.Ho * a.Wo;
    auto blocks = [&](const TileCfg &t) {
        const long long bp = 32 * t.PF * t.WP, bc = 32 * t.CT * t.WC;
        return ((M + bp - 1) / bp) * ((a.C_out + bc - 1) / bc);
    };
    // measured on the five benchmark configs: the 128x128 tile wins whenever it
    // yields enough workgroups (more for 1x1 layers, whose few channel blocks leave
    // nothing for two wave groups to split) and does not waste more than a quarter
    // of its channels; the 256x64 tile when it still runs in two rounds or more;
    // otherwise the 128x64 tile
    const int c_pad = ((a.C_out + 127) / 128) * 128;
    // (a 1x1 layer with at most 64 input channels is one matrix instruction deep:
    // wasted channels cost nothing there, fewer and wider output tiles still pay;
    // not in chained mode, whose epilogue quantizes the wasted channels too)
    const int waste_limit = (a.R == 1 && a.Cp <= 64 && !a.rq) ? 2 : 4;
    if (a.C_out > 64 && waste_limit * (c_pad - a.C_out) <= c_pad && blocks(kMedium) >= (a.R == 1 ? 320 : 192)) {
        // 2-bit layers (FP4 path: the 256x128 tile fits its registers): take that
        // tile when the 128x128 one leaves a nearly empty last round of workgroups
        // (3 per CU, 768 at a time) and the large one (2 per CU, 512) does not
        if (a.cont == 2) {
            const double bm = (double)blocks(kMedium), bl = (double)blocks(kLarge);
            const double waste_m = (double)((blocks(kMedium) + 767) / 768 * 768) / bm;
            const double waste_l = (double)((blocks(kLarge) + 511) / 512 * 512) / bl;
            if (bl >= 256 && waste_m > 1.35 * waste_l) return TILE_LARGE;
            // deep 3x3 layers with about one workgroup per CU (256 -> 256 at 14x14 x 64,
            // 512 -> 512 at 14x14 x 32): the 256x64 tile with one wave group measured 6-10 %
            // ahead of the 128x128 tile with two (plain call; the chained call measures the other way)
            if (!a.rq && a.R == 3 && a.stride == 1 && a.Cp >= 256 && !a.many_in_flight && blocks(kMedium) <= 320 &&
                blocks(kTall) >= 192)
                return TILE_TALL;
        }
        return TILE_MEDIUM;
    }
    if (blocks(kTall) >= 1536) return TILE_TALL;      // at least two rounds of workgroups; else finer tiles
    return TILE_SMALL;
}

constexpr int kLdsLimit = 150 * 1024;

}  // namespace

namespace {

// Tile, wave-group count and plan for a layer.  Two wave groups (K split inside
// the workgroup) only pay when the layer yields about one workgroup per CU.
bool choose_plan(const DsqConvArgs &a, int force_tile, int &which, int &ks, PatchPlan &pl)
{
    if ((long long)a.N * a.H * a.W * (a.Cp * a.cont / 8) > 0x7FFFFFFFLL) return false;
    which = force_tile >= 0 ? force_tile : pick_tile(a);
    // chained mode: the 256x128 tile has a variant for 2-bit containers only (at 3 and
    // 4 bits it does not fit the registers), and layers with l_a != 0 (border-dependent
    // terms) go to the simple kernel
    if (a.rq && ((which == TILE_LARGE && a.cont != 2) || a.l_a != 0.0f)) return false;
    const TileCfg &tc = tile_cfg(which);
    const int BP = 32 * tc.PF * tc.WP, BC = 32 * tc.CT * tc.WC;
    const long long M = (long long)a.N * a.Ho * a.Wo;
    const long long blocks = ((M + BP - 1) / BP) * ((a.C_out + BC - 1) / BC);
    // (with several calls in flight the CUs are shared by workgroups of different calls
    // anyway, and one wave group per workgroup -- half the LDS, no exchange of partial
    // sums -- gives the higher throughput: measured +9 % on config 2 with four in flight)
    ks = (!a.many_in_flight && (which == TILE_SMALL || which == TILE_MEDIUM) && a.Cp >= 128 && blocks <= 320) ? 2 : 1;
    if (ks == 2 && plan_patch(a, BP, BC, tc.PF, tc.CT, kMaxUPT, kLdsLimit, 2, pl)) return true;
    ks = 1;
    return plan_patch(a, BP, BC, tc.PF, tc.CT, kMaxUPT, kLdsLimit, 1, pl);
}

}  // namespace

bool dsq_conv_patch_supported(const DsqConvArgs &a, int force_tile)
{
    int which, ks;
    PatchPlan pl;
    return choose_plan(a, force_tile, which, ks, pl);
}

int dsq_conv_patch_describe(const DsqConvArgs &a, int force_tile, char *text, size_t n)
{
    int which, ks;
    PatchPlan pl;
    if (!choose_plan(a, force_tile, which, ks, pl)) return 0;
    const TileCfg &tc = tile_cfg(which);
    const int BC = 32 * tc.CT * tc.WC;
    const int need = (pl.units + 255) / 256;
    const int upt = need <= 2 ? 2 : need <= 4 ? 4 : need <= 8 ? 8 : 12;
    const int blocks = pl.tiles_w * pl.row_tiles * ((a.C_out + BC - 1) / BC);
    snprintf(text, n, "patch kernel: container %d, %dx%d filter, tile %dx%d (pixels x channels), %d wave group%s, "
             "%d fetch units per thread%s; strip width %d, patch %dx%d, %d workgroups, %d LDS bytes",
             a.cont, a.R, a.R, 32 * tc.PF * tc.WP, BC, ks, ks == 1 ? "" : "s", upt,
             a.rq ? ", chained epilogue" : "", pl.TW, pl.PR, pl.PC, blocks, plan_lds_bytes(pl, BC, a.rq != 0));
    return 1;
}

hipError_t dsq_launch_conv_patch(const DsqConvArgs &args, int force_tile, hipStream_t stream)
{
    int which, ks;
    PatchPlan pl;
    if (!choose_plan(args, force_tile, which, ks, pl)) return hipErrorInvalidValue;
    DsqConvArgs a = args;
    if (a.rq) {
        // Next layer's pixel sums: a layer no wider than the tile has each pixel's
        // sum complete in one workgroup, which stores it; otherwise the workgroups
        // add to sums that a fill kernel clears first.
        const TileCfg &tc = tile_cfg(which);
        a.rq_store = a.C_out <= 32 * tc.CT * tc.WC;
        a.rq_share = a.rq_store || a.R == 1;
    }
    const int need = (pl.units + 255) / 256;      // fetch units per thread: instantiated 2, 4, 8, 12
    switch (2 * a.cont + (a.R == 3 ? 0 : 1)) {
    case 8: return dsq_conv_patch_c4r3(a, pl, which, ks, need, stream);
    case 9: return dsq_conv_patch_c4r1(a, pl, which, ks, need, stream);
    case 6: return dsq_conv_patch_c3r3(a, pl, which, ks, need, stream);
    case 7: return dsq_conv_patch_c3r1(a, pl, which, ks, need, stream);
    case 4: return dsq_conv_patch_c2r3(a, pl, which, ks, need, stream);
    default: return dsq_conv_patch_c2r1(a, pl, which, ks, need, stream);
    }
}
