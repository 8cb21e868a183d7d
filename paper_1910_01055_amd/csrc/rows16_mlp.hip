// Host side of the whole-network kernel for small policies (rows16_mlp.hpp): which networks it takes, how many
// 16-row tiles a workgroup owns at a given batch, and the launch.
#include "rows16_mlp.hpp"

namespace aq {
namespace r16 {
AQ_ROWS16_INST(1, false);
AQ_ROWS16_DECL(2, false);
AQ_ROWS16_DECL(4, false);
AQ_ROWS16_DECL(1, true);
AQ_ROWS16_DECL(2, true);
AQ_ROWS16_DECL(4, true);
AQ_ROWS16_LATE_DECL(false);
AQ_ROWS16_LATE_DECL(true);
}  // namespace r16

// Shapes the kernel takes (see the head of rows16_mlp.hpp).
bool rows16_mlp_supported(const FwdArgs& a) {
    const NetDev& n = a.net;
    if (n.n_layers < 1 || n.n_layers > r16::RMAXL) return false;
    for (int l = 0; l < n.n_layers; ++l) {
        const LayerDev& L = n.L[l];
        if (L.kh != 1 || L.kw != 1 || L.in_h != 1 || L.in_w != 1) return false;
        if (L.KS * 32 > r16::RMAXK) return false;
        if (l < n.n_layers - 1) {
            if (L.NT * 32 > r16::RMAXK) return false;
        } else if (L.NT > 2) {
            return false;
        }
    }
    return true;
}

// Row tiles per workgroup, from a sweep of cfg2's network over batch sizes (us per launch at 1 / 2 / 4 tiles:
// batch 4096: 6.8 / 9.3 / 13.5; 8192: 9.4 / 9.6 / 13.5; 16384: 16.4 / 13.0 / 13.7; 24576: 23.1 / 19.2 / 20.1;
// 32768: 29.8 / 23.7 / 20.2; 65536: 57.0 / 43.9 / 37.2): one tile while at most two workgroups share a CU, two
// tiles up to three workgroups per CU, four beyond (more rows per workgroup mean fewer weight bytes through the
// CU's vector memory path per row, and two resident workgroups overlap each other's barriers).
// Every workgroup has a CU to itself (256 CUs, 16 rows per workgroup): the variant that requests a layer's
// operands behind the epilogue two layers earlier.
bool rows16_mlp_alone_on_cu(int64_t batch) { return batch <= 16 * 256; }

int rows16_mlp_row_tiles(int64_t batch) {
    if (batch <= 16 * 512) return 1;
    if (batch <= 32 * 768) return 2;
    return 4;
}

aq_status launch_rows16_mlp(const FwdArgs& a, hipStream_t st) {
    if (!rows16_mlp_supported(a) || ((uintptr_t)a.c.obs & 15) != 0) return AQ_ESHAPE;
    r16::R16Args ra{};
    ra.obs = (const float*)a.c.obs;
    ra.actions = a.c.actions;
    ra.batch = a.c.batch;
    ra.K0 = a.net.L[0].K;
    ra.shape = a.net.n_layers | (a.net.in_u8 ? 1 << 8 : 0);
    ra.ex_sigma = a.c.ex_sigma;
    ra.ex_k0 = a.c.ex_k0;
    ra.ex_k1 = a.c.ex_k1;
    ra.ex_s0 = a.c.ex_s0;
    ra.ex_s1 = a.c.ex_s1;
    const bool tp = any_taps(a);
#define AQ_GO(MT)                                                                                         \
    return a.net.asym ? (tp ? r16::launch_rows16_t<MT, true, true>(a.d_net, ra, a.t, st)                  \
                            : r16::launch_rows16_t<MT, true, false>(a.d_net, ra, a.t, st))                \
                      : (tp ? r16::launch_rows16_t<MT, false, true>(a.d_net, ra, a.t, st)                 \
                            : r16::launch_rows16_t<MT, false, false>(a.d_net, ra, a.t, st))
    if (rows16_mlp_alone_on_cu(a.c.batch))
        return a.net.asym ? (tp ? r16::launch_rows16_t<1, true, true, true>(a.d_net, ra, a.t, st)
                                : r16::launch_rows16_t<1, true, false, true>(a.d_net, ra, a.t, st))
                          : (tp ? r16::launch_rows16_t<1, false, true, true>(a.d_net, ra, a.t, st)
                                : r16::launch_rows16_t<1, false, false, true>(a.d_net, ra, a.t, st));
    switch (rows16_mlp_row_tiles(a.c.batch)) {
        case 1: AQ_GO(1);
        case 2: AQ_GO(2);
        default: AQ_GO(4);
    }
#undef AQ_GO
}

}  // namespace aq
