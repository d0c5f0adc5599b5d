// Variant selection and launch dispatch.
#include "plan.hpp"
#include <stdlib.h>

namespace dwc {

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Optional overrides for tuning runs, from the snapshot of tune.hpp (empty in normal use).
static int tune(const char *name, int dflt)
{
    const char *e = tune_env(name);
    if (!e) return dflt;
    int v = atoi(e);
    return v > 0 ? v : dflt;
}

static bool same_pad_s1(const Geom &g) { return g.s == 1 && (g.K == 3 || g.K == 5) && g.p == (g.K - 1) / 2; }
static bool k3s2p1(const Geom &g) { return g.s == 2 && g.K == 3 && g.p == 1; }

// channels per lane for the NHWC kernels, 0 if the fast path does not apply
static int nhwc_vec(const Geom &g, int dtype)
{
    // multiplier 2 has a fast path for 3x3 stride 1 only; the vector counts OUTPUT channels
    if (g.m == 2) { if (!(g.K == 3 && g.s == 1 && g.p == 1)) return 0; }
    else if (g.m != 1) return 0;
    if (dtype == DT_F32) return g.O % 4 == 0 ? 4 : 0;
    // 5x5: 25 taps x 8 channels would not fit in registers; 2 channels per lane take 110 registers
    // instead of the 208 of 4 channels and measured 1.25x faster.  These kernels address one image through a
    // buffer view of at most 2 GiB.
    if (g.K == 5) return (g.O % 2 == 0 && (long long)g.H * g.W * g.C * 2 <= (1LL << 31)) ? 2 : 0;
    return g.O % 8 == 0 ? 8 : (g.O % 4 == 0 ? 4 : 0);
}

// Rows loaded ahead in the NHWC stride-1 kernel.  fp32 3x3: four (inside the step the nine forward launches of the
// MobileNet stack take 522 us with four rows in flight against 531 with two; the small layers, whose wavefronts are
// all resident at once, gain most); bf16 3x3: three (input gradient 886 -> 870 us over the bf16 stack).  5x5 keeps
// 25 taps x V in registers: two rows.
static int nhwc_pf(const Geom &g, int dtype)
{
    int pf = tune("DWCONV_TUNE_PF", (g.K == 3 && g.m == 1) ? (dtype == DT_F32 ? 4 : 3) : 2);
    if (g.K == 5 && pf > 2) pf = 2;
    if (g.m != 1 && pf > 2) pf = 2;
    if (pf > 3 && !(dtype == DT_F32 && g.K == 3)) pf = 3;
    if (pf > 4) pf = 4;
    return pf;
}

// Rows per strip of the forward / backward-data row walks.  Measured on the benchmark layers:
// short strips win (14 input rows at stride 1, 7 output rows at stride 2) even though each strip
// re-reads K-1 halo rows (those come from L2): more, shorter walks keep the launch's accesses
// closer together in memory.
static int pick_th(int rows, int stride, int dflt1 = 14, int dflt2 = 0)
{
    // stride 2: 7 output rows, 4 on tall maps (56 output rows and more: 1-4 % on the 112x112 and 56x56 layers);
    // the input gradient takes 4 dy rows on every map (28 dy rows: NHWC 45.2 -> 42.2 us, NCHW 44.0 -> 42.5 us; 14 dy
    // rows: NHWC 21.1 -> 19.5 us) and in NCHW 2 on tall maps (its 112x112 layer: 118 -> 110 us inside the step; NHWC
    // lost 1 % with it)
    if (dflt2 == 0) dflt2 = rows >= 56 ? 4 : 7;
    const int target = stride == 1 ? tune("DWCONV_TUNE_TH1", dflt1) : tune("DWCONV_TUNE_TH2", dflt2);
    // balanced strips: the number of strips that brings their height closest to the target, then equal
    // heights (19 rows are one strip of 19, not 14 + 5; 37 rows are 13 + 13 + 11)
    int nstrips = (rows + target / 2) / target;
    if (nstrips < 1) nstrips = 1;
    const int th = ceil_div(rows, nstrips);
    return tune("DWCONV_TUNE_TH", th);
}

// Strip height of the NHWC stride-1 row walk: 14 rows for fp32; 28 for bf16, whose walks are bound by their
// vector-ALU work and pay for every halo row a strip computes again (5x5: 46.5 -> 44.2 us and 44.5 -> 41.9 us per
// launch over the bf16 stack; 3x3: 1 %).
static int nhwc_th1(int dtype) { return dtype == DT_BF16 ? 28 : 14; }

// Strip height of the NCHW stride-1 row walk.  The bf16 kernels are bound by their vector-ALU work (twice the
// elements per byte), so the K-1 halo rows a strip computes again cost them more than they cost the fp32 kernels:
// strips of 28 rows measured 2-9 % faster than 14 on the bf16 layers.
// fp32: 14 rows on rows of 112 elements; on rows of 56 and fewer (whole-line write-out in groups of four rows) 8 rows
// measured 3-4 % faster than 14 inside the step, on the forward pass and on the input gradient.
static int nchwd_th1(int dtype, int W) { return dtype == DT_BF16 ? 28 : (W <= 56 ? 8 : 14); }

// NCHW: rows per unit.  Small planes are taken whole; larger ones in strips of 8 output rows
// (halo rows come from L2), shrunk until the tile fits in LDS.
static int nchw_pick_tr(const Geom &g, bool (*fits)(const Geom &, int))
{
    int tr = g.Ho <= 16 ? g.Ho : 8;
    tr = tune("DWCONV_TUNE_TH", tr);
    if (tr > g.Ho) tr = g.Ho;
    while (tr > 1 && !fits(g, tr)) tr = (tr + 1) / 2;
    return fits(g, tr) ? tr : 0;
}
static bool fits_bwd_filter(const Geom &g, int tr) { return nchw_bwd_filter_parts(g, tr, 1) > 0; }

// Small-plane NCHW kernels: rows of up to 14 always, and whenever the row walk cannot take the shape (bf16 rows that
// are not whole 16-byte vectors).  Rows of 28, where both families apply, go to whichever measured faster inside the
// benchmark step: the filter gradient always to the small-plane kernel (37 against 46 us on the 28x28x256 layer at
// batch 128, 23 against 29 us on its stride-2 sibling), the fp32 forward and the fp32 input gradient at stride 2
// too (stride-1 forward 42 against 47 us, stride-2 forward 28 against 31 us, stride-2 input gradient 21 against
// 22 us); the fp32 stride-1 input gradient stays with the row walk; bf16 see below.
static bool use_small(const Geom &g, int dtype, int pass)
{
    if (!nchws_supported(g, pass)) return false;
    if (g.W <= 14 || nchwd_vec(g, dtype, pass) == 0) return true;
    if (const char *e = tune_env("DWCONV_TUNE_S28")) return atoi(e) == 1;
    if (pass == 2) return true;
    if (dtype == DT_F32) return pass == 0 || (pass == 1 && g.s == 2);
    // bf16 at stride 1 (the 28x28 layer at batch 256, outputs staged in place): 3x3 forward 46 against 73 us, 3x3
    // input gradient 39 against 59 us, 5x5 forward 56 against 74 us, 5x5 input gradient 50 against 63 us
    return g.s == 1;
}

Plan plan_fwd(const Geom &g, int layout, int dtype)
{
    Plan pl = {V_GENERIC, 0, 0, 0, 0, "generic"};
    if (layout == LAYOUT_NCHW) {
        if (use_small(g, dtype, 0)) { pl.variant = V_NCHWS_FWD; pl.name = g.K == 5 ? "nchw_smallplane_k5s1" : (g.s == 1 ? "nchw_smallplane_k3s1" : "nchw_smallplane_fwd_k3s2"); return pl; }
        const int V = nchwd_vec(g, dtype, 0);
        if (V) {
            pl.a = V;
            if (g.s == 1) { pl.variant = V_NCHWD_S1; pl.b = pick_th(g.H, 1, nchwd_th1(dtype, g.W)); pl.name = g.K == 3 ? "nchw_rowwalk_k3s1" : "nchw_rowwalk_k5s1"; }
            else { pl.variant = V_NCHWD_K3S2; pl.b = pick_th(g.Ho, 2); pl.name = "nchw_rowwalk_fwd_k3s2"; }
            return pl;
        }
        const int tr = nchw_pick_tr(g, nchw_fwd_supported);
        if (tr) { pl.variant = V_NCHW_FWD; pl.b = tr; pl.name = "nchw_tile_fwd"; }
        return pl;
    }
    if (layout == LAYOUT_NHWC) {
        const int V = nhwc_vec(g, dtype);
        if (V && same_pad_s1(g)) {
            pl.variant = V_NHWC_S1; pl.a = V; pl.b = pick_th(g.H, 1, nhwc_th1(dtype));
            pl.name = g.m == 2 ? "nhwc_rowwalk_k3s1_m2" : (g.K == 3 ? "nhwc_rowwalk_k3s1" : "nhwc_rowwalk_k5s1");
        } else if (V && k3s2p1(g)) {
            pl.variant = V_NHWC_K3S2; pl.a = V; pl.b = pick_th(g.Ho, 2);
            pl.name = "nhwc_rowwalk_fwd_k3s2";
        }
    }
    return pl;
}

Plan plan_bwd_data(const Geom &g, int layout, int dtype)
{
    Plan pl = {V_GENERIC, 0, 0, 0, 0, "generic"};
    if (layout == LAYOUT_NCHW) {
        if (use_small(g, dtype, 1)) {
            if (g.s == 1) { pl.variant = V_NCHWS_FWD; pl.name = g.K == 5 ? "nchw_smallplane_k5s1_flip" : "nchw_smallplane_k3s1_flip"; }
            else { pl.variant = V_NCHWS_BWD_DATA_S2; pl.name = "nchw_smallplane_bwd_data_k3s2"; }
            return pl;
        }
        const int V = nchwd_vec(g, dtype, 1);
        if (V) {
            pl.a = V;
            if (g.s == 1) { pl.variant = V_NCHWD_S1; pl.b = pick_th(g.H, 1, nchwd_th1(dtype, g.W)); pl.name = g.K == 3 ? "nchw_rowwalk_k3s1_flip" : "nchw_rowwalk_k5s1_flip"; }
            else { pl.variant = V_NCHWD_K3S2; pl.b = pick_th(g.Ho, 2, 14, g.Ho >= 56 ? 2 : 4); pl.name = "nchw_rowwalk_bwd_data_k3s2"; }
            return pl;
        }
        if (g.m == 1 && same_pad_s1(g)) {
            const int tr = nchw_pick_tr(g, nchw_fwd_supported);
            if (tr) { pl.variant = V_NCHW_FWD; pl.b = tr; pl.name = "nchw_tile_fwd_flip"; }
        } else if (g.m == 1 && k3s2p1(g)) {
            const int tr = nchw_pick_tr(g, nchw_bwd_data_k3s2_supported);
            if (tr) { pl.variant = V_NCHW_BWD_DATA_K3S2; pl.b = tr; pl.name = "nchw_tile_bwd_data_k3s2"; }
        }
        return pl;
    }
    if (layout == LAYOUT_NHWC) {
        const int V = nhwc_vec(g, dtype);
        if (V && same_pad_s1(g)) {
            pl.variant = V_NHWC_S1; pl.a = V; pl.b = pick_th(g.H, 1, nhwc_th1(dtype));
            pl.name = g.m == 2 ? "nhwc_rowwalk_k3s1_flip_m2" : (g.K == 3 ? "nhwc_rowwalk_k3s1_flip" : "nhwc_rowwalk_k5s1_flip");
        } else if (V && k3s2p1(g)) {
            pl.variant = V_NHWC_K3S2; pl.a = V; pl.b = pick_th(g.Ho, 2, 14, 4);
            pl.name = "nhwc_rowwalk_bwd_data_k3s2";
        }
    }
    return pl;
}

// NCHW filter gradient on the small-plane kernels / on the row walk; false if the family does not take the shape.
static bool plan_bwd_filter_nchws(const Geom &g, int dtype, Plan &pl)
{
    int U, NI, parts;
    nchws_bwd_filter_tiling(g, dtype, &U, &NI, &parts);
    NI = tune("DWCONV_TUNE_NI", NI);
    if (NI > g.N) NI = g.N;
    parts = ceil_div(g.N, NI);
    if ((long long)parts * g.O * g.K * g.K * 4 > (64ll << 20)) return false;
    pl.variant = V_NCHWS_BWD_FILTER; pl.a = U; pl.b = 0; pl.c = NI; pl.parts = parts;
    pl.name = g.K == 5 ? "nchw_smallplane_bwd_filter_k5s1"
                       : (g.s == 1 ? "nchw_smallplane_bwd_filter_k3s1" : "nchw_smallplane_bwd_filter_k3s2");
    return true;
}

static bool plan_bwd_filter_nchwd(const Geom &g, int dtype, Plan &pl)
{
    const int V = nchwd_vec(g, dtype, 2);
    if (!V) return false;
    // strip height (measured on the benchmark layers): stride 2 wants short strips of 7 output rows,
    // fp32 stride 1 on large planes 14 rows, everything else whole planes up to 56 rows
    int TH = g.s == 2 && g.Ho >= 28 ? 7
             : (g.s == 1 && dtype == DT_F32 && g.Ho >= 56 ? 14 : (g.Ho > 56 ? (g.Ho + 1) / 2 : g.Ho));
    TH = tune("DWCONV_TUNE_THW", tune("DWCONV_TUNE_TH", TH));
    int lg, nst, rounds, parts;
    nchwd_bwd_filter_tiling(g, V, TH, &lg, &nst, &rounds, &parts);
    // small batches: shorter strips until the launch has about two blocks per CU (one block = one
    // channel x a group of (image, strip) items)
    while (TH > 7 && parts >= 1 && (long long)parts * g.O < 512 && !tune_env("DWCONV_TUNE_THW") && !tune_env("DWCONV_TUNE_TH")) {
        TH = (TH + 1) / 2;
        nchwd_bwd_filter_tiling(g, V, TH, &lg, &nst, &rounds, &parts);
    }
    if (!(lg >= 1 && parts >= 1 && (long long)parts * g.O * g.K * g.K * 4 <= (64ll << 20))) return false;
    pl.variant = V_NCHWD_BWD_FILTER; pl.a = V; pl.b = TH; pl.c = 0; pl.parts = parts;
    pl.name = g.K == 5 ? "nchw_rowwalk_bwd_filter_k5s1"
                       : (g.s == 1 ? "nchw_rowwalk_bwd_filter_k3s1" : "nchw_rowwalk_bwd_filter_k3s2");
    return true;
}

// force_v > 0: channels per lane of the NHWC kernel (the fused backward kernel has four in either type)
static Plan plan_bwd_filter_v(const Geom &g, int layout, int dtype, int force_v)
{
    Plan pl = {V_GENERIC, generic_bwd_filter_parts(g), 0, 0, 0, "generic"};
    if (layout == LAYOUT_NCHW) {
        if (use_small(g, dtype, 2) && plan_bwd_filter_nchws(g, dtype, pl)) return pl;
        if (plan_bwd_filter_nchwd(g, dtype, pl)) return pl;
        const int tr = nchw_pick_tr(g, fits_bwd_filter);
        if (tr) {
            // images per block: keep about 4096 blocks in the launch
            const int wpl = g.Wo <= 8 ? 8 : g.Wo <= 16 ? 16 : g.Wo <= 32 ? 32 : g.Wo <= 64 ? 64 : g.Wo <= 128 ? 128 : 256;
            const long long ublocks = ((long long)g.O * ceil_div(g.Ho, tr) + (256 / wpl) - 1) / (256 / wpl);
            int NI = (int)((ublocks * g.N) / 4096);
            if (NI < 1) NI = 1;
            if (NI > g.N) NI = g.N;
            NI = tune("DWCONV_TUNE_NI", NI);
            int parts = nchw_bwd_filter_parts(g, tr, NI);
            while ((long long)parts * g.O * g.K * g.K * 4 > (64ll << 20) && NI < g.N) {
                NI *= 2;
                parts = nchw_bwd_filter_parts(g, tr, NI);
            }
            if ((long long)parts * g.O * g.K * g.K * 4 <= (64ll << 20)) {
                pl.variant = V_NCHW_BWD_FILTER; pl.b = tr; pl.c = NI; pl.parts = parts; pl.name = "nchw_tile_bwd_filter";
            }
        }
        return pl;
    }
    if (layout == LAYOUT_NHWC) {
        int V = nhwc_vec(g, dtype);
        // bf16 on small planes: four channels per lane (124 registers, four wavefronts per SIMD) measured faster
        // than eight (182 registers, two wavefronts)
        if (V == 8 && tune("DWCONV_TUNE_WV", g.W <= 14 ? 4 : 8) == 4) V = 4;
        if (force_v > 0 && V >= force_v) V = force_v;
        if (V && (same_pad_s1(g) || k3s2p1(g))) {
            // One block = 256 lanes over (columns x channel-vectors) x one strip x NI images.  Long
            // walks win (fewer partials, less stage-2 work): start from whole columns and one image
            // per block, and only split rows when the launch would have too few blocks to keep the
            // memory system busy.
            int CT, nct, nowt, nst, ngr;
            nhwc_bwd_filter_tiling(g, V, g.Ho, 1, &CT, &nct, &nowt, &nst, &ngr);
            const long long per_strip = (long long)nct * nowt * g.N;   // blocks with NI = 1 and one strip
            // Measured on all benchmark layers: about two blocks per CU (512) is the sweet spot, and a
            // block that walks two images beats two blocks with one image each; stride 2 tolerates
            // half as many blocks again.
            // 5x5 is bound by its multiply-adds and wants four wavefronts per SIMD (1024 blocks), not two
            const long long want = tune("DWCONV_TUNE_WBLOCKS", g.K == 5 ? 1024 : 512), floor_blocks = g.s == 1 ? want * 3 / 4 : want / 2;
            int TH = g.Ho, NI = 1;
            while (TH > 7 && per_strip * ceil_div(g.Ho, TH) * 4 < want * 3) TH = (TH + 1) / 2;
            while (NI < g.N && per_strip * ceil_div(g.Ho, TH) / (NI * 2) >= floor_blocks) NI *= 2;
            TH = tune("DWCONV_TUNE_THW", tune("DWCONV_TUNE_TH", TH)); NI = tune("DWCONV_TUNE_NI", NI);
            if (TH > g.Ho) TH = g.Ho;
            if (NI > g.N) NI = g.N;
            nhwc_bwd_filter_tiling(g, V, TH, NI, &CT, &nct, &nowt, &nst, &ngr);
            // keep the partials within 64 MiB: more images per block, then taller strips; a shape that is
            // still above it with whole columns of the whole batch per block (very many channels times very
            // wide rows) goes to the generic kernels, whose partials are a single O*K*K array in that case
            while ((long long)nowt * nst * ngr * g.O * g.K * g.K * 4 > (64ll << 20) && (NI < g.N || TH < g.Ho)) {
                if (NI < g.N) NI = NI * 2 < g.N ? NI * 2 : g.N; else TH = TH * 2 < g.Ho ? TH * 2 : g.Ho;
                nhwc_bwd_filter_tiling(g, V, TH, NI, &CT, &nct, &nowt, &nst, &ngr);
            }
            if ((long long)nowt * nst * ngr * g.O * g.K * g.K * 4 > (64ll << 20)) return pl;
            pl.variant = V_NHWC_BWD_FILTER; pl.a = V; pl.b = TH; pl.c = NI;
            pl.parts = nowt * nst * ngr;
            pl.name = g.m == 2 ? "nhwc_bwd_filter_k3s1_m2"
                               : (g.s == 2 ? "nhwc_bwd_filter_k3s2" : (g.K == 3 ? "nhwc_bwd_filter_k3s1" : "nhwc_bwd_filter_k5s1"));
        }
    }
    return pl;
}

Plan plan_bwd_filter(const Geom &g, int layout, int dtype) { return plan_bwd_filter_v(g, layout, dtype, 0); }

Plan plan_bwd(const Geom &g, int layout, int dtype)
{
    Plan pl = {V_GENERIC, 0, 0, 0, 0, "separate"};
    if (layout == LAYOUT_NHWC && !tune_env("DWCONV_TUNE_NOFUSE")) {
        // the fused kernel takes four channels per lane in either type (bf16 with eight would need more than 256 registers)
        int V = nhwc_vec(g, dtype);
        if (V == 8 && g.W <= tune("DWCONV_TUNE_FUSE_BF16W", 65536)) V = 4;
        if (V && nhwc_bwd_fused_supported(g, dtype, V)) {
            // tiling of the filter gradient: its block count and partial sums decide
            const Plan pf = plan_bwd_filter_v(g, layout, dtype, V);
            if (pf.variant == V_NHWC_BWD_FILTER && pf.a == V) {
                pl = pf;
                pl.variant = V_NHWC_BWD_FUSED;
                pl.name = g.m == 2 ? "nhwc_bwd_fused_k3s1_m2" : (g.s == 1 ? "nhwc_bwd_fused_k3s1" : "nhwc_bwd_fused_k3s2");
            }
        }
    }
    if (layout == LAYOUT_NCHW && !tune_env("DWCONV_TUNE_NOFUSE")) {
        // a fused kernel of either family, whichever the separate filter gradient would run on
        Plan pf = pl;
        // (28-wide fp32 rows at stride 1 are whole 16-byte vectors: they stay with the row-walk fused kernel below)
        const bool rowwalk28 = g.s == 1 && g.W == 28 && dtype == DT_F32;
        if (use_small(g, dtype, 2) && !rowwalk28 && nchws_bwd_fused_supported(g) && plan_bwd_filter_nchws(g, dtype, pf)) {
            int U, NI, parts;
            nchws_bwd_fused_tiling(g, dtype, &U, &NI, &parts);
            if ((long long)parts * g.O * g.K * g.K * 4 <= (64ll << 20)) {
                pl = pf;
                pl.variant = V_NCHWS_BWD_FUSED; pl.a = U; pl.c = NI; pl.parts = parts;
                pl.name = g.s == 1 ? "nchw_smallplane_bwd_fused_k3s1" : "nchw_smallplane_bwd_fused_k3s2";
                return pl;
            }
        }
        pf = pl;
        if (g.s == 2 && !use_small(g, dtype, 2) && !tune_env("DWCONV_TUNE_NOFUSE_NCHW_S2") && plan_bwd_filter_nchwd(g, dtype, pf)) {
            // stride 2 on row-walk shapes: two dy columns per lane, strips of the filter gradient's height made even
            // where a write-out group is four dx rows
            const int V2 = dtype == DT_F32 ? 2 : 4, rs = nchwd_bwd_fused_rs(g, dtype, V2);
            if (rs) {
                const int TH = (2 * pf.b) % rs == 0 ? pf.b : pf.b + 1;
                int lg, nst, rounds, parts;
                nchwd_bwd_filter_tiling(g, V2, TH, &lg, &nst, &rounds, &parts);
                if (lg >= 1 && parts >= 1 && (long long)parts * g.O * g.K * g.K * 4 <= (64ll << 20)) {
                    pl = pf;
                    pl.variant = V_NCHWD_BWD_FUSED; pl.a = V2; pl.b = TH; pl.parts = parts;
                    pl.name = "nchw_bwd_fused_k3s2";
                    return pl;
                }
            }
        }
        pf = pl;
        if (g.s == 1 && plan_bwd_filter_nchwd(g, dtype, pf)) {
            const int rs = nchwd_bwd_fused_rs(g, dtype, pf.a);
            if (rs) {
                // the filter gradient's tiling with the strip height rounded up to whole row groups
                const int TH = (pf.b + rs - 1) / rs * rs;
                int lg, nst, rounds, parts;
                nchwd_bwd_filter_tiling(g, pf.a, TH, &lg, &nst, &rounds, &parts);
                if (lg >= 1 && parts >= 1 && (long long)parts * g.O * g.K * g.K * 4 <= (64ll << 20)) {
                    pl = pf;
                    pl.variant = V_NCHWD_BWD_FUSED; pl.b = TH; pl.parts = parts;
                    pl.name = "nchw_bwd_fused_k3s1";
                }
            }
        }
    }
    return pl;
}

hipError_t launch_fwd(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *w, void *y,
                      hipStream_t st)
{
    switch (pl.variant) {
    case V_NHWC_S1: return nhwc_s1(g, dtype, pl.a, x, w, y, false, pl.b, nhwc_pf(g, dtype), st);
    case V_NHWC_K3S2: return nhwc_k3s2(g, dtype, pl.a, x, w, y, false, pl.b, st);
    case V_NCHW_FWD: return nchw_fwd(g, dtype, x, w, y, false, pl.b, st);
    case V_NCHWD_S1: return nchwd_s1(g, dtype, pl.a, x, w, y, false, pl.b, st);
    case V_NCHWS_FWD: return nchws_fwd(g, dtype, x, w, y, false, st);
    case V_NCHWD_K3S2: return nchwd_k3s2(g, dtype, pl.a, x, w, y, false, pl.b, st);
    default: return generic_fwd(g, layout, dtype, x, w, y, st);
    }
}

hipError_t launch_bwd_data(const Plan &pl, const Geom &g, int layout, int dtype, const void *dy, const void *w,
                           void *dx, hipStream_t st)
{
    switch (pl.variant) {
    case V_NHWC_S1: return nhwc_s1(g, dtype, pl.a, dy, w, dx, true, pl.b, nhwc_pf(g, dtype), st);
    case V_NHWC_K3S2: return nhwc_k3s2(g, dtype, pl.a, dy, w, dx, true, pl.b, st);
    case V_NCHW_FWD: return nchw_fwd(g, dtype, dy, w, dx, true, pl.b, st);
    case V_NCHWD_S1: return nchwd_s1(g, dtype, pl.a, dy, w, dx, true, pl.b, st);
    case V_NCHWS_FWD: return nchws_fwd(g, dtype, dy, w, dx, true, st);
    case V_NCHWS_BWD_DATA_S2: return nchws_bwd_data_s2(g, dtype, dy, w, dx, st);
    case V_NCHWD_K3S2: return nchwd_k3s2(g, dtype, pl.a, dy, w, dx, true, pl.b, st);
    case V_NCHW_BWD_DATA_K3S2: return nchw_bwd_data_k3s2(g, dtype, dy, w, dx, pl.b, st);
    default: return generic_bwd_data(g, layout, dtype, dy, w, dx, st);
    }
}

hipError_t launch_bwd_filter(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *dy,
                             float *ws, hipStream_t st)
{
    switch (pl.variant) {
    case V_NHWC_BWD_FILTER: return nhwc_bwd_filter(g, dtype, pl.a, x, dy, ws, pl.b, pl.c, st);
    case V_NCHW_BWD_FILTER: return nchw_bwd_filter(g, dtype, x, dy, ws, pl.b, pl.c, st);
    case V_NCHWD_BWD_FILTER: return nchwd_bwd_filter(g, dtype, pl.a, x, dy, ws, pl.b, st);
    case V_NCHWS_BWD_FILTER: return nchws_bwd_filter(g, dtype, x, dy, ws, pl.a, pl.c, st);
    default: return generic_bwd_filter(g, layout, dtype, x, dy, ws, pl.parts, st);
    }
}

hipError_t launch_bwd_fused(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *dy,
                            const void *w, void *dx, float *ws, hipStream_t st)
{
    (void)layout;
    if (pl.variant == V_NCHWD_BWD_FUSED) return nchwd_bwd_fused(g, dtype, pl.a, x, dy, w, dx, ws, pl.b, st);
    if (pl.variant == V_NCHWS_BWD_FUSED) return nchws_bwd_fused(g, dtype, x, dy, w, dx, ws, pl.a, pl.c, st);
    if (pl.variant != V_NHWC_BWD_FUSED) return hipErrorInvalidValue;
    return nhwc_bwd_fused(g, dtype, pl.a, x, dy, w, dx, ws, pl.b, pl.c, st);
}

}  // namespace dwc
