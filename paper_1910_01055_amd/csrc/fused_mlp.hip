// Host side of the whole-network fused int8 MLP: decides whether a network fits the kernel, picks
// rows per workgroup and feature tiles per wave, and dispatches to the compiled variant.
#include "fused_mlp.hpp"

namespace aq {

AQ_FUSED_DECL(1, 1, false, false, false);
AQ_FUSED_DECL(1, 1, false, true, false);
AQ_FUSED_DECL(2, 1, false, false, false);
AQ_FUSED_DECL(2, 1, false, true, false);
AQ_FUSED_DECL(4, 1, false, false, false);
AQ_FUSED_DECL(4, 1, false, true, false);
AQ_FUSED_DECL(1, 2, false, false, false);
AQ_FUSED_DECL(1, 2, false, true, false);
AQ_FUSED_DECL(2, 2, false, false, false);
AQ_FUSED_DECL(2, 2, false, true, false);
AQ_FUSED_DECL(1, 1, true, false, false);
AQ_FUSED_DECL(1, 1, true, true, false);
AQ_FUSED_DECL(2, 1, true, false, false);
AQ_FUSED_DECL(2, 1, true, true, false);
AQ_FUSED_DECL(1, 1, false, false, true);
AQ_FUSED_DECL(1, 1, false, true, true);
AQ_FUSED_DECL(1, 1, true, false, true);
AQ_FUSED_DECL(1, 1, true, true, true);

namespace {
struct Plan {
    int mt, nb, ld, cst_n, part_off, cst_dbl;
    bool half;  // 16 rows per workgroup
    size_t lds;
};

bool make_plan(const FwdArgs& a, Plan* p) {
    int maxw = 0, max_np = 0, max_nt = 0;
    for (int l = 0; l < a.net.n_layers; ++l) {
        const LayerDev& L = a.net.L[l];
        if (L.kh != 1 || L.kw != 1 || L.in_h != 1 || L.in_w != 1) return false;
        maxw = maxw > L.KS * 32 ? maxw : L.KS * 32;
        if (l < a.net.n_layers - 1) maxw = maxw > L.NT * 32 ? maxw : L.NT * 32;
        max_np = max_np > L.NT * 32 ? max_np : L.NT * 32;
        max_nt = max_nt > L.NT ? max_nt : L.NT;
    }
    if (max_np > CST_MAXN) return false;
    // the last layer's fp32 rows (NT * 32 floats) reuse an activation buffer
    const int lastw = a.net.L[a.net.n_layers - 1].NT * 32 * 4;
    maxw = maxw > lastw ? maxw : lastw;
    p->ld = maxw + 16;
    p->cst_n = max_np;
    // feature tiles per wave: wide layers take 2 (two passes of the 8 waves cover 32 tiles); more would
    // not leave registers for the operand pipeline at two waves per SIMD
    p->nb = (max_nt >= 32 && !a.net.asym) ? 2 : 1;
    auto ln_fits = [&](int nb) {  // LayerNorm needs its whole row resident in one pass
        for (int l = 0; l < a.net.n_layers - 1; ++l)
            if (a.net.L[l].act == AQ_ACT_LN_TANH && (a.net.L[l].NT + nb - 1) / nb > FW) return false;
        return true;
    };
    const bool narrow_last = a.net.L[a.net.n_layers - 1].NT <= NARROW_NT;
    const int nb_full = p->nb;
    // Rows per workgroup: 16 (one tile per wave only), 32, 64 or 128 (the latter with one tile per wave
    // only).  A workgroup's time grows roughly like 1 + rows/32 (a fixed latency chain plus epilogue work
    // per row), the 256 CUs take one workgroup each per round: take the cheapest rounds x time.
    struct Cand {
        int rows, mt, nb;
        bool half;
    };
    const Cand cands[4] = {{16, 1, 1, true}, {32, 1, nb_full, false}, {64, 2, nb_full, false}, {128, 4, 1, false}};
    double best = 0.0;
    bool found = false;
    for (const Cand& cd : cands) {
        if (cd.mt == 4 && (nb_full != 1 || a.net.asym)) continue;  // (the asymmetric 128-row variant does not fit the registers)
        if (!ln_fits(cd.nb)) continue;
        Plan q = *p;
        q.mt = cd.mt;
        q.nb = cd.nb;
        q.half = cd.half;
        // (a doubled constant area when everything still fits in 64 KB: small networks, where the
        // barrier it saves per layer is a visible share of the time)
        q.cst_dbl = cd.nb != 2 && cd.mt != 4 && fused_lds_bytes(32 * cd.mt, q.ld, q.cst_n, true) + PART_BYTES <= 64 * 1024;
        q.lds = fused_lds_bytes(32 * cd.mt, q.ld, q.cst_n, q.cst_dbl != 0);
        q.part_off = -1;
        // partial sums of a narrow last layer: in the idle activation buffer if it is large enough,
        // else in an area of their own behind everything else
        if (narrow_last && (size_t)32 * cd.mt * q.ld < (size_t)PART_BYTES) {
            q.part_off = (int)q.lds;
            q.lds += PART_BYTES;
        }
        if (q.lds > 160 * 1024) continue;
        const int64_t wgs = (a.c.batch + cd.rows - 1) / cd.rows;
        const double cost = (double)((wgs + 255) / 256) * (1.0 + cd.rows / 32.0);
        if (!found || cost < best) {
            best = cost;
            found = true;
            *p = q;
        }
    }
    return found;
}
}  // namespace

bool any_taps(const FwdArgs& a) {
    if (a.t.a0 || a.t.y) return true;
    for (int l = 0; l < a.net.n_layers; ++l)
        if (a.t.acc[l] || a.t.act[l] || a.t.ln[l]) return true;
    return false;
}

bool fused_mlp_supported(const FwdArgs& a, int* rows_out, size_t* lds_out, int* tiles_out) {
    Plan p;
    if (!make_plan(a, &p)) return false;
    *rows_out = p.half ? 16 : 32 * p.mt;
    *lds_out = p.lds;
    if (tiles_out) *tiles_out = p.nb;
    if (fused_mlp_kernel_kind(a) >= 2) {  // (given a 16-byte aligned observation buffer)
        *rows_out = 16 * rows16_mlp_row_tiles(a.c.batch);
        if (tiles_out) *tiles_out = 1;
    }
    return true;
}

int fused_mlp_kernel_kind(const FwdArgs& a) {
    Plan p;
    int ld;
    if (!make_plan(a, &p)) return 0;
    if (rows16_mlp_supported(a)) return rows16_mlp_alone_on_cu(a.c.batch) ? 3 : 2;
    if (p.half) return 0;
    if (p.nb == 2 && p.mt == 2 && wide_mlp_supported(a, &ld)) return 1;
    return 0;
}

aq_status launch_fused_mlp(const FwdArgs& a_in, hipStream_t st) {
    Plan p;
    if (!make_plan(a_in, &p)) return AQ_ESHAPE;
    // 64-row workgroups on wide layers: the pipelined kernel where the shapes and the address allow it
    // 16-row workgroups on small networks: the kernel built for that case
    const int kind = ((uintptr_t)a_in.c.obs & 15) == 0 ? fused_mlp_kernel_kind(a_in) : 0;
    if (kind == 1) return launch_wide_mlp(a_in, st);
    if (kind >= 2) return launch_rows16_mlp(a_in, st);
    FwdArgs a = a_in;
    a.c.ld = p.ld;
    a.c.cst_n = p.cst_n;
    a.c.wp0 = a.net.L[0].wp;
    a.c.pack0 = a.net.L[0].bias_fold;
    a.c.NT0 = a.net.L[0].NT;
    a.c.KS0 = a.net.L[0].KS;
    a.c.pieces0 = (a.net.n_layers == 1 ? 2 : 4) * a.net.L[0].NT * 8;
    a.c.part_off = p.part_off;
    a.c.cst_dbl = p.cst_dbl;
    a.c.ln0 = a.net.n_layers > 1 && a.net.L[0].act == AQ_ACT_LN_TANH;
    a.c.narrow0 = a.net.n_layers == 1 && a.net.L[0].NT <= NARROW_NT;
    const bool tp = any_taps(a);
    const bool as = a.net.asym != 0;
#define AQ_GO(MT, NB, AS, HF)                                                   \
    return tp ? launch_fused_t<MT, NB, AS, true, HF>(a, p.lds, st) \
              : launch_fused_t<MT, NB, AS, false, HF>(a, p.lds, st)
    if (p.half) {
        if (as) AQ_GO(1, 1, true, true);
        AQ_GO(1, 1, false, true);
    }
    if (p.nb == 2) {
        if (p.mt == 1) AQ_GO(1, 2, false, false);
        AQ_GO(2, 2, false, false);
    }
    if (as) {
        if (p.mt == 1) AQ_GO(1, 1, true, false);
        if (p.mt == 2) AQ_GO(2, 1, true, false);
        return AQ_ESHAPE;  // (no 128-row asymmetric variant: make_plan never picks it)
    }
    if (p.mt == 1) AQ_GO(1, 1, false, false);
    if (p.mt == 2) AQ_GO(2, 1, false, false);
    AQ_GO(4, 1, false, false);
#undef AQ_GO
}

}  // namespace aq
