// The leading convolution layers of a frame policy (Sec. 4.1: the Atari-style policies take stacked
// 8-bit frames through three convolutions before the fully connected layers) in one launch: one
// workgroup per image keeps the frame and every intermediate feature map in LDS, so the maps never
// travel through global memory and the three launches of the per-layer path become one.
//
// No im2col: with NHWC maps a 32-byte k-step of the implicit GEMM is 32 contiguous bytes of the input
// map (part of one kernel row), so an MFMA's activation operand is one 16-byte LDS read per lane at an
// address computed from the output position.  A wave owns a (32 output positions) x (32 features)
// tile at a time; weights stream from L2 in operand order, a few k-steps ahead.
//
// Shapes it takes (the host checks them, anything else goes one launch per layer): 8-bit frames,
// per-channel symmetric weights, K = kh*kw*in_c a multiple of 32, kw*in_c, stride*in_c and in_w*in_c
// multiples of 16 (operand reads stay aligned and inside one kernel row), N a multiple of 4.
#include "int8_device.hpp"

namespace aq {

namespace {
constexpr int CS_W = 8;    // waves per workgroup
constexpr int CS_PF = 8;   // weight k-steps in flight per wave
constexpr size_t CS_MAX_LDS = 96 * 1024;

struct StackPlan {
    int nc;          // leading convolution layers taken
    int off_b;       // LDS offset of the second map buffer
    size_t lds;
};

bool plan_stack(const FwdArgs& a, StackPlan* p) {
    const NetDev& net = a.net;
    if (!net.in_u8 || net.asym) return false;
    int nc = 0;
    while (nc < net.n_layers) {
        const LayerDev& L = net.L[nc];
        const bool fc = L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1;
        if (fc) break;
        ++nc;
    }
    if (nc < 2 || nc >= net.n_layers) return false;  // a fully connected layer must follow
    size_t sz[2] = {0, 0};
    for (int l = 0; l < nc; ++l) {
        const LayerDev& L = net.L[l];
        const int run = L.kw * L.in_c;
        if (L.act == AQ_ACT_LN_TANH) return false;
        if (L.K != L.KS * 32 || run % 16 || (L.stride * L.in_c) % 16 || (L.in_w * L.in_c) % 16 || (L.N & 3)) return false;
        if (a.t.ln[l]) return false;
        const size_t in_bytes = (size_t)L.in_h * L.in_w * L.in_c;
        if (in_bytes % 16) return false;
        if (in_bytes > sz[l & 1]) sz[l & 1] = in_bytes;
    }
    if (((uintptr_t)a.c.obs & 15) || a.c.batch > 0x7fffffffLL) return false;
    p->nc = nc;
    p->off_b = (int)sz[0];
    p->lds = sz[0] + sz[1];
    return p->lds <= CS_MAX_LDS;
}
}  // namespace

template <bool TAPS>
__global__ __launch_bounds__(CS_W * 64) void k_conv_stack(const NetDev* __restrict__ netp, const TapArgs t, const int nc,
                                                         const uint8_t* __restrict__ frames, int8_t* __restrict__ out,
                                                         const int off_b) {
    extern __shared__ __align__(16) int8_t smem[];
    const NetDev& a = *netp;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, n = lane & 31;
    const int64_t img = blockIdx.x;
    {   // the frame -> LDS, into the signed domain (code - 128)
        const LayerDev& L0 = a.L[0];
        const int pieces = (L0.in_h * L0.in_w * L0.in_c) >> 4;
        const v4i* src = (const v4i*)frames + img * pieces;
        v4i* dst = (v4i*)smem;
        for (int i = tid; i < pieces; i += CS_W * 64) {
            v4i v = src[i];
            v[0] ^= 0x80808080;
            v[1] ^= 0x80808080;
            v[2] ^= 0x80808080;
            v[3] ^= 0x80808080;
            dst[i] = v;
        }
    }
    __syncthreads();
    for (int l = 0; l < nc; ++l) {
        const LayerDev& L = a.L[l];
        const int8_t* in = smem + ((l & 1) ? off_b : 0);
        int8_t* map_out = smem + ((l & 1) ? 0 : off_b);
        const int R = L.oh * L.ow, RT = (R + 31) >> 5, NT = L.NT, KS = L.KS, N = L.N;
        const int run = L.kw * L.in_c, row_bytes = L.in_w * L.in_c;
        const bool to_global = l == nc - 1;
        const int z_out = a.actq[l + 1].z;
        const int lo = L.act == AQ_ACT_RELU ? z_out : 0;
        const bool fast = a.fast[l] != 0;
        LayerTaps T{nullptr, nullptr, nullptr};
        if (TAPS) T = LayerTaps{t.acc[l], t.act[l], nullptr};
        const CPtrs C = global_consts(L);
        for (int tile = wave; tile < RT * NT; tile += CS_W) {
            const int nt = tile % NT, rt = tile / NT;
            const int r = rt * 32 + n;           // this lane's output position (operand column)
            const int rc = r < R ? r : R - 1;    // a ragged last tile re-reads the last position; never stored
            const int oy = rc / L.ow, ox = rc - oy * L.ow;
            const int8_t* base = in + (oy * L.stride * L.in_w + ox * L.stride) * L.in_c;
            gv4i_ptr wptr = (gv4i_ptr)L.wp + (int64_t)nt * KS * 64 + lane;
            v4i w[CS_PF];
#pragma unroll
            for (int p = 0; p < CS_PF; ++p) w[p] = wptr[(int64_t)(p < KS ? p : KS - 1) * 64];
            v16i acc[1][1];
            acc[0][0] = zero16();
            // (ky, kr): kernel row and byte offset inside it of this lane's half of the current k-step
            int ky = 0, kr = g * 16;
            while (kr >= run) {
                kr -= run;
                ++ky;
            }
            for (int ks0 = 0; ks0 < KS; ks0 += CS_PF) {
#pragma unroll
                for (int p = 0; p < CS_PF; ++p) {
                    const int k = ks0 + p;
                    if (k < KS) {
                        const v4i x = *(const v4i*)(base + ky * row_bytes + kr);
                        acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[p], x, acc[0][0], 0, 0, 0);
                        kr += 32;
                        while (kr >= run) {
                            kr -= run;
                            ++ky;
                        }
                        const int kn = k + CS_PF;
                        w[p] = wptr[(int64_t)(kn < KS ? kn : KS - 1) * 64];
                    }
                }
            }
            v16i rs[1];
            rs[0] = zero16();
            const int64_t row_g = img * R + r;  // row of the layer's [batch * oh * ow][N] output
            int8_t* out0 = to_global ? out + row_g * N : map_out + r * N;
            if (fast)
                epi_hidden_wave<1, 1, false, TAPS, true>(N, NT, T, C, acc, rs, 0, nt, g, row_g, img * R + R, true, z_out, lo,
                                                        out0, 0, true, N);
            else
                epi_hidden_wave<1, 1, false, TAPS, false>(N, NT, T, C, acc, rs, 0, nt, g, row_g, img * R + R, true, z_out, lo,
                                                         out0, 0, true, N);
        }
        __syncthreads();
    }
}

int conv_stack_layers(const FwdArgs& a) {
    StackPlan p;
    return plan_stack(a, &p) ? p.nc : 0;
}

aq_status launch_conv_stack(const FwdArgs& a, int8_t* out, hipStream_t st) {
    StackPlan p;
    if (!plan_stack(a, &p)) return AQ_ESHAPE;
    const bool taps = any_taps(a);
    dim3 grid((unsigned)a.c.batch);
#define AQ_STACK(TP)                                                                                                 \
    do {                                                                                                             \
        static bool attr_set = false;                                                                                \
        if (!attr_set) {                                                                                             \
            if (hipFuncSetAttribute((const void*)k_conv_stack<TP>, hipFuncAttributeMaxDynamicSharedMemorySize,       \
                                    (int)CS_MAX_LDS) != hipSuccess)                                                  \
                return AQ_EHIP;                                                                                      \
            attr_set = true;                                                                                         \
        }                                                                                                            \
        hipLaunchKernelGGL((k_conv_stack<TP>), grid, dim3(CS_W * 64), p.lds, st, a.d_net, a.t, p.nc,                 \
                           (const uint8_t*)a.c.obs, out, p.off_b);                                                   \
    } while (0)
    if (taps) AQ_STACK(true);
    else AQ_STACK(false);
#undef AQ_STACK
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
