// The leading convolution layers of a frame policy (Sec. 4.1: the Atari-style policies take stacked
// 8-bit frames through three convolutions before the fully connected layers) in one launch: one
// workgroup per image keeps the frame, every intermediate feature map and the layers' epilogue
// constants in LDS.  Frame and constants are requested in one burst at its start (one round trip);
// the maps never travel through global memory, and the three launches of the per-layer path become one.
// Weights stream from L2 in operand order (staging them in LDS as well was measured slower: the burst
// grows to 100 KB per workgroup and only one workgroup fits a CU).
//
// No im2col: with NHWC maps a 32-byte k-step of the implicit GEMM is 32 contiguous bytes of the input
// map (part of one kernel row), so an MFMA's activation operand is one 16-byte LDS read per lane at an
// address computed from the output position.  A wave owns a (32 output positions) x (32 features)
// tile at a time.
//
// Shapes it takes (the host checks them, anything else goes one launch per layer): 8-bit frames,
// per-channel symmetric weights, K = kh*kw*in_c a multiple of 32, kw*in_c, stride*in_c and in_w*in_c
// multiples of 16 and kw*in_c a multiple of 32 (operand reads stay aligned and a k-step stays inside one
// kernel row), N a multiple of 4, and a frame and constants within the burst's register budget (32 KB,
// 2048 words).
#include "int8_device.hpp"

namespace aq {

namespace {
constexpr int CS_W = 8;          // waves per workgroup (16 when every image gets a CU to itself)
constexpr int CS_T = CS_W * 64;  // threads of the smaller workgroup: sizes the burst's limits
constexpr int CS_FU = 4;         // 16-byte pieces of the frame per thread
constexpr int CS_CU = 4;         // words of epilogue constants per thread
constexpr int CS_CONSTS = 5;     // arrays per layer: bias_fold | M0 | rz | sh (one contiguous pack), rshift
constexpr size_t CS_MAX_LDS = 160 * 1024;
constexpr int CS_MAXC = 4;       // convolution layers of a stack at most

// What the host knows of the stack at launch time, by value: the burst's requests and every layer's tile loop
// then need nothing but the kernel arguments (one scalar round trip at the start; read from the device-resident
// description the burst's addresses took four thousand clocks of dependent scalar loads to work out, and every
// layer began with a round trip for its own entry).  Only what the quantizer kernels write (activation zero-points,
// short-form flags) still comes from the description, requested at the start.
struct StackLayer {
    const int8_t* wp;
    int oh, ow, in_w, in_c, kw, stride, N, NT, KS, act;
};
struct StackArgs {
    int f_pieces;            // 16-byte pieces of a frame
    int c_words;             // constant words of all layers
    int cnt[CS_MAXC];        // ... of each layer, and where they come from: four arrays in one pack, then rshift
    int np4[CS_MAXC];
    const int32_t* pack[CS_MAXC];
    const int32_t* rsh[CS_MAXC];
    StackLayer L[CS_MAXC];
};

struct StackPlan {
    int nc;          // leading convolution layers taken
    int off_b;       // LDS offsets: second map buffer, constants
    int off_c;
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
    if (nc < 2 || nc > CS_MAXC || nc >= net.n_layers) return false;  // a fully connected layer must follow
    size_t sz[2] = {0, 0}, c_words = 0;
    for (int l = 0; l < nc; ++l) {
        const LayerDev& L = net.L[l];
        const int run = L.kw * L.in_c;
        if (L.act == AQ_ACT_LN_TANH) return false;
        if (L.K != L.KS * 32 || run % 32 || (L.stride * L.in_c) % 16 || (L.in_w * L.in_c) % 16 || (L.N & 3)) return false;
        if (a.t.ln[l]) return false;
        const size_t in_bytes = (size_t)L.in_h * L.in_w * L.in_c;
        if (in_bytes % 16) return false;
        if (in_bytes > sz[l & 1]) sz[l & 1] = in_bytes;
        c_words += (size_t)CS_CONSTS * L.NT * 32;
    }
    const size_t frame = (size_t)net.L[0].in_h * net.L[0].in_w * net.L[0].in_c;
    if (frame > (size_t)CS_FU * CS_T * 16 || c_words > (size_t)CS_CU * CS_T) return false;
    if (((uintptr_t)a.c.obs & 15) || a.c.batch > 0x7fffffffLL) return false;
    p->nc = nc;
    p->off_b = (int)sz[0];
    p->off_c = (int)(sz[0] + sz[1]);
    p->lds = sz[0] + sz[1] + c_words * 4;
    return p->lds <= CS_MAX_LDS;
}
}  // namespace

template <bool TAPS, int W, int NC>
__global__ __launch_bounds__(W * 64) void k_conv_stack(const NetDev* __restrict__ netp, const TapArgs t, const StackArgs sa,
                                                     const uint8_t* __restrict__ frames, int8_t* __restrict__ out,
                                                     const int off_b, const int off_c) {
    extern __shared__ __align__(16) int8_t smem[];
    const NetDev& a = *netp;
    // (the wave index stays a vector value here: it only selects tiles, in a loop; the tests that guard MFMAs are on
    // the scalar K.  An MFMA behind a lane-mask test could run under an empty mask, which the matrix cores ignore)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, n = lane & 31;
    const int64_t img = blockIdx.x;
    constexpr int NTHR = W * 64;
    constexpr int nc = NC;
    // (written by the quantizer kernels: requested now, used by the epilogues)
    int z_q[NC], fastf[NC];
#pragma unroll
    for (int l = 0; l < NC; ++l) {
        z_q[l] = a.actq[l + 1].z;
        fastf[l] = a.fast[l];
    }
    {   // the burst: frame pieces and the constant words of all layers, then their LDS stores
        const int f_pieces = sa.f_pieces;
        const int c_words = sa.c_words;
        const v4i* fsrc = (const v4i*)frames + img * f_pieces;
        v4i fr[CS_FU];
        int cr[CS_CU];
#pragma unroll
        for (int u = 0; u < CS_FU; ++u) {
            const int i = tid + u * NTHR;
            fr[u] = fsrc[i < f_pieces ? i : f_pieces - 1];
        }
#pragma unroll
        for (int u = 0; u < CS_CU; ++u) {
            int i = tid + u * NTHR;
            i = i < c_words ? i : c_words - 1;
            // which layer word i belongs to: per-lane selects over per-layer scalars
            const int32_t* pack = sa.pack[0];
            const int32_t* rsh = sa.rsh[0];
            int np4 = sa.np4[0];
            bool found = false;
#pragma unroll
            for (int j = 0; j + 1 < NC; ++j) {
                const int cnt = sa.cnt[j];
                if (!found && i >= cnt) {
                    i -= cnt;
                    pack = sa.pack[j + 1];
                    rsh = sa.rsh[j + 1];
                    np4 = sa.np4[j + 1];
                } else {
                    found = true;
                }
            }
            cr[u] = i < np4 ? pack[i] : rsh[i - np4];
        }
        v4i* fdst = (v4i*)smem;
        int* cdst = (int*)(smem + off_c);
#pragma unroll
        for (int u = 0; u < CS_FU; ++u) {
            const int i = tid + u * NTHR;
            if (i < f_pieces) {   // into the signed domain (code - 128)
                v4i x = fr[u];
                x[0] ^= 0x80808080;
                x[1] ^= 0x80808080;
                x[2] ^= 0x80808080;
                x[3] ^= 0x80808080;
                fdst[i] = x;
            }
        }
#pragma unroll
        for (int u = 0; u < CS_CU; ++u) {
            const int i = tid + u * NTHR;
            if (i < c_words) cdst[i] = cr[u];
        }
    }
    __syncthreads();
    int c_at = off_c;  // this layer's constants in LDS
    static_for<0, NC>([&](auto l_c) __attribute__((always_inline)) {
        constexpr int l = decltype(l_c)::value;
        const StackLayer& L = sa.L[l];
        const int8_t* in = smem + ((l & 1) ? off_b : 0);
        int8_t* map_out = smem + ((l & 1) ? 0 : off_b);
        const int R = L.oh * L.ow, RT = (R + 31) >> 5, NT = L.NT, KS = L.KS, N = L.N;
        const int run = L.kw * L.in_c, row_bytes = L.in_w * L.in_c;
        constexpr bool to_global = l == nc - 1;
        const int z_out = z_q[l];
        const int lo = L.act == AQ_ACT_RELU ? z_out : 0;
        const bool fast = fastf[l] != 0;
        LayerTaps T{nullptr, nullptr, nullptr};
        if (TAPS) T = LayerTaps{t.acc[l], t.act[l], nullptr};
        const int np = NT * 32;
        const int32_t* cst = (const int32_t*)(smem + c_at);
        const CPtrs C{cst, cst + np, cst + 4 * np, cst + 2 * np, cst + 3 * np, nullptr};
        for (int tile = wave; tile < RT * NT; tile += W) {
            const int nt = tile % NT, rt = tile / NT;
            const int r = rt * 32 + n;           // this lane's output position (operand column)
            const int rc = r < R ? r : R - 1;    // a ragged last tile re-reads the last position; never stored
            const int oy = rc / L.ow, ox = rc - oy * L.ow;
            const int8_t* base = in + (oy * L.stride * L.in_w + ox * L.stride) * L.in_c;
            gv4i_ptr wg = (gv4i_ptr)L.wp + (int64_t)nt * KS * 64 + lane;
            v16i acc[1][1];
            acc[0][0] = zero16();
            // Operands of four k-steps at a time, two sets in flight: the reads of one set run under the
            // MFMAs of the other.  px walks this lane's half of the k-steps through the input map: 32 bytes
            // on, and at the end of a kernel row (kr == run) down to the next map row.
            const int8_t* px = base + g * 16;
            int kr = 0;
            auto load4 = [&](int k0, v4i (&A)[4], v4i (&X)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k = k0 + j;
                    const int kc = k < KS ? k : KS - 1;
                    A[j] = wg[(int64_t)kc * 64];
                    X[j] = *(const v4i*)px;
                    if (k < KS - 1) {   // (uniform) never steps past the last k-step's bytes
                        kr += 32;
                        const bool wrap = kr == run;
                        px += wrap ? 32 + row_bytes - run : 32;
                        kr = wrap ? 0 : kr;
                    }
                }
            };
            auto mma4 = [&](int k0, v4i (&A)[4], v4i (&X)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (k0 + j < KS) acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[j], X[j], acc[0][0], 0, 0, 0);
            };
            v4i A0[4], X0[4], A1[4], X1[4];
            load4(0, A0, X0);
            int k0 = 0;
            for (; k0 + 8 < KS; k0 += 8) {
                load4(k0 + 4, A1, X1);
                mma4(k0, A0, X0);
                load4(k0 + 8, A0, X0);
                mma4(k0 + 4, A1, X1);
            }
            // the last eight k-steps or fewer, without the request for a group after them: past K a request
            // re-reads the last k-step and still takes its slot on the vector memory path
            if (k0 + 4 < KS) load4(k0 + 4, A1, X1);
            mma4(k0, A0, X0);
            mma4(k0 + 4, A1, X1);
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
        c_at += CS_CONSTS * np * 4;
        __syncthreads();
    });
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
    StackArgs sa{};
    {
        const LayerDev& L0 = a.net.L[0];
        sa.f_pieces = (L0.in_h * L0.in_w * L0.in_c) >> 4;
        for (int l = 0; l < p.nc; ++l) {
            const LayerDev& L = a.net.L[l];
            sa.cnt[l] = CS_CONSTS * L.NT * 32;
            sa.np4[l] = 4 * L.NT * 32;
            sa.pack[l] = L.bias_fold;
            sa.rsh[l] = L.rshift;
            sa.c_words += sa.cnt[l];
            sa.L[l] = StackLayer{L.wp, L.oh, L.ow, L.in_w, L.in_c, L.kw, L.stride, L.N, L.NT, L.KS, L.act};
        }
    }
#define AQ_STACK(TP, WV, NCV)                                                                                        \
    do {                                                                                                             \
        static std::atomic<bool> attr_set{false};                                                                    \
        if (!attr_set) {                                                                                             \
            if (hipFuncSetAttribute((const void*)k_conv_stack<TP, WV, NCV>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    (int)CS_MAX_LDS) != hipSuccess)                                                  \
                return AQ_EHIP;                                                                                      \
            attr_set = true;                                                                                         \
        }                                                                                                            \
        hipLaunchKernelGGL((k_conv_stack<TP, WV, NCV>), grid, dim3(WV * 64), p.lds, st, a.d_net, a.t, sa,            \
                           (const uint8_t*)a.c.obs, out, p.off_b, p.off_c);                                          \
    } while (0)
#define AQ_STACK_NC(TP, WV)                 \
    switch (p.nc) {                         \
        case 2: AQ_STACK(TP, WV, 2); break; \
        case 3: AQ_STACK(TP, WV, 3); break; \
        default: AQ_STACK(TP, WV, 4); break; \
    }
    // up to one image per CU: sixteen waves (the first layer's tiles then run in one round); beyond that
    // eight, so that two workgroups share a CU
    if (a.c.batch <= 256) {
        if (taps) AQ_STACK_NC(true, 16)
        else AQ_STACK_NC(false, 16)
    } else {
        if (taps) AQ_STACK_NC(true, 8)
        else AQ_STACK_NC(false, 8)
    }
#undef AQ_STACK_NC
#undef AQ_STACK
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
