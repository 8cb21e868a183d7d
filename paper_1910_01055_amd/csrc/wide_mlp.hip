// Whole-network int8 MLP for wide layers at large batch (Sec. 3.1 actor inference on the 8-bit policy of
// Sec. 3.2), software-pipelined: one workgroup of 8 wavefronts owns 64 batch rows from the observation to
// the action, as in the general fused kernel, but a wavefront never sits in a phase that uses only one of
// the CU's pipes.
//
// A layer's output features are split into passes of 512 (8 wavefronts x 2 feature tiles x 32); a wavefront
// keeps two sets of accumulators, the pass being multiplied and the pass before it.  While the matrix cores
// run the MFMAs of pass i, the vector ALU requantizes the accumulators of pass i - 1, one register quad per
// k-step, written between the MFMAs of that k-step.  Across a layer boundary this still works: the first
// k-steps of layer l + 1 read the features that layer l's earlier passes wrote, so the epilogue of layer l's
// last pass runs under them; one workgroup barrier in the middle of that pass then publishes the remaining
// features, and the k-steps that read them follow it.  Weights stream L2 -> registers in operand order, four
// k-steps in flight per wavefront, and the stream does not stop at a pass boundary: the last k-steps of a
// pass already request the first k-steps of the next one.
//
// Shapes: per-channel symmetric weights, fp32 observations at a 16-byte aligned address, every hidden layer
// ReLU / none (no LayerNorm) with a width that is a multiple of 64, every layer's K a multiple of 128, a
// last layer of at most 64 outputs.  Everything else takes the general fused kernel.
#include <mutex>

#include "fused_mlp.hpp"

namespace aq {
namespace {

constexpr int WROWS = 64;    // batch rows per workgroup: two row tiles per wavefront
constexpr int WPF = 4;       // weight k-steps in flight per wavefront
constexpr int WSLOT = 256;   // words of one wave-private constant slot: four arrays of 64 features
constexpr int WGROUP = 16;   // k-steps of a pass that carry the epilogue of the pass before (one quad each)

typedef const char AQ_GLOBAL* gbytes;

__host__ __device__ inline size_t wide_lds_bytes(int ld) {
    return (size_t)2 * WROWS * ld + (size_t)FW * 2 * WSLOT * 4 + 256 * 4;
}

template <bool TAPS>
__global__ __launch_bounds__(FT) void k_mlp_wide(const NetDev* __restrict__ netp, const CallArgs c, const TapArgs t) {
    extern __shared__ __align__(16) int8_t smem[];
    const NetDev& a = *netp;
    const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6), g = lane >> 5, mrow = lane & 31;
    const int64_t row0 = (int64_t)blockIdx.x * WROWS;
    const int ld = c.ld;
    int32_t* const cst_all = (int32_t*)(smem + 2 * WROWS * ld);
    int32_t* const my_cst = cst_all + wave * 2 * WSLOT;   // two slots: this pass's constants, the previous pass's
    int32_t* const cst_last = cst_all + FW * 2 * WSLOT;   // the narrow last layer's bias | scale
    auto buf = [&](int i) { return smem + (i & 1) * WROWS * ld; };
    const int n_layers = uni(a.n_layers), nh = n_layers - 1;

    // the weight stream of one pass of this wavefront: its two feature tiles, KS k-steps of 1 KiB each
    struct Stream {
        gbytes b0, b1;
        int KS;
    };
    auto stream_of = [&](int l, int grp) {
        const int KS = uni(a.L[l].KS);
        gbytes wp = (gbytes)uni_ptr(a.L[l].wp);
        return Stream{wp + (int64_t)(2 * grp) * KS * 1024, wp + (int64_t)(2 * grp + 1) * KS * 1024, KS};
    };
    const uint32_t lane_off = (uint32_t)lane * 16u;
    auto wload = [&](gbytes b, int ks) { return *(gv4i_ptr)(b + (int64_t)ks * 1024 + lane_off); };

    // first pass's first weights: requested before the observations are touched
    v4i wreg[WPF][2];
    {
        const int KS0 = c.KS0;
        gbytes wp = (gbytes)c.wp0;
        const int grp0 = 2 * wave < c.NT0 ? wave : 0;
#pragma unroll
        for (int p = 0; p < WPF; ++p) {
            const int k = p < KS0 ? p : KS0 - 1;
            wreg[p][0] = wload(wp + (int64_t)(2 * grp0) * KS0 * 1024, k);
            wreg[p][1] = wload(wp + (int64_t)(2 * grp0 + 1) * KS0 * 1024, k);
        }
    }

    // observation quantize: a0 = clamp(round(x / s0) + z0, 0, 255), kept in the signed domain.  The block's
    // rows are one contiguous 16-byte aligned run (the launcher checked the address; K0 is a multiple of 128):
    // 16-byte pieces, four in flight per lane, four codes at a time into their row of the LDS buffer.
    {
        const int K0 = c.K0;
        const float s0 = a.actq[0].s;
        const int z0 = a.actq[0].z;
        const QuantScale qs0 = make_quant_scale(s0);
        const float zf0 = (float)z0;
        int8_t* buf_in = buf(0);
        const int64_t left = c.batch - row0;
        const int vrows = left < WROWS ? (int)left : WROWS;
        const int n4 = (vrows * K0) >> 2, k4 = K0 >> 2;
        // idx / k4 by a reciprocal: (idx + 0.5) / k4 stays at least 0.5 / k4 away from every integer, far more
        // than the rounding error at these magnitudes (idx < 2^16)
        const float inv_k4 = __builtin_amdgcn_rcpf((float)k4);
        const float4* src = (const float4*)((const float*)c.obs + row0 * K0);
        for (int i0 = tid; i0 < n4; i0 += 4 * FT) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * FT < n4) v[u] = src[i0 + u * FT];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = i0 + u * FT;
                if (idx < n4) {
                    uint32_t pack = quant_u8x4(v[u], qs0, zf0);
                    if (TAPS) {
                        if (t.a0) *(uint32_t*)(t.a0 + row0 * K0 + 4 * idx) = pack;
                    }
                    const int m = (int)(((float)idx + 0.5f) * inv_k4), kq = idx - m * k4;
                    *(uint32_t*)(buf_in + m * ld + 4 * kq) = pack ^ 0x80808080u;
                }
            }
        }
        // rows past the batch: zero in the signed domain
        for (int m = vrows + wave; m < WROWS; m += FW)
            for (int k = lane * 4; k < K0; k += 256) *(uint32_t*)(buf_in + m * ld + k) = 0u;
    }
    lds_barrier();

    v16i cur[2][2], prev[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) cur[i][j] = prev[i][j] = zero16();

    // what the epilogue of the previous pass needs (all uniform)
    bool have_prev = false, prev_active = false;
    int prev_grp = 0, prev_N = 0, prev_zout = 0, prev_lo = 0, prev_fast = 0, prev_slot = 0;
    const int32_t* prev_rshift = nullptr;
    int8_t* prev_out = nullptr;
    int32_t* prev_tacc = nullptr;  // intermediate outputs asked for by a test (TAPS only)
    uint8_t* prev_tact = nullptr;

    // ---- epilogue of the previous pass, in pieces: quad Q = (feature tile nb, register quad j, row tile mt),
    // piece i = output i of the quad.  Constants of a (nb, j) pair are read from the wave's LDS slot one pair
    // ahead of their use.
    QuadConsts qc{}, qn{};
    uint32_t pack = 0;
    auto quad_consts = [&](int pair) {  // pair = nb * 4 + j
        const int32_t* s = my_cst + prev_slot * WSLOT + (pair >> 2) * 32 + 8 * (pair & 3) + 4 * g;
        QuadConsts q;
        q.bf = *(const int4*)(s);
        q.M = *(const int4*)(s + 64);
        q.Z = *(const int4*)(s + 128);
        q.S = *(const int4*)(s + 192);
        return q;
    };
    int lo_v = 0;
    auto epi_piece = [&](auto q_c, auto i_c, auto fast_c) __attribute__((always_inline)) {
        constexpr int Q = decltype(q_c)::value, i = decltype(i_c)::value;
        constexpr bool FAST = decltype(fast_c)::value;
        constexpr int pair = Q >> 1, mt = Q & 1, nb = pair >> 2, j = pair & 3;
        if (i == 0 && mt == 0) {
            qc = qn;
            if (pair + 1 < 8) qn = quad_consts(pair + 1);
        }
        const int bfv = i == 0 ? qc.bf.x : i == 1 ? qc.bf.y : i == 2 ? qc.bf.z : qc.bf.w;
        const int Mv = i == 0 ? qc.M.x : i == 1 ? qc.M.y : i == 2 ? qc.M.z : qc.M.w;
        const int Zv = i == 0 ? qc.Z.x : i == 1 ? qc.Z.y : i == 2 ? qc.Z.z : qc.Z.w;
        const int Sv = i == 0 ? qc.S.x : i == 1 ? qc.S.y : i == 2 ? qc.S.z : qc.S.w;
        const int val = prev[nb][mt][4 * j + i] + bfv;
        const int n = (2 * prev_grp + nb) * 32 + 8 * j + 4 * g + i;
        int code;
        if (FAST) code = clamp_code((__mulhi(val, Mv) + Zv) >> Sv, lo_v, 255);
        else code = requant_code(val, Mv, prev_rshift[n], prev_zout, prev_lo);
        if (TAPS) {
            const int64_t row = row0 + mt * 32 + mrow;
            if (row < c.batch) {
                if (prev_tacc) prev_tacc[row * prev_N + n] = val;
                if (prev_tact) prev_tact[row * prev_N + n] = (uint8_t)code;
            }
        }
        pack = i == 0 ? (uint32_t)code : pack | ((uint32_t)code << (8 * i));
        if (i == 3) *(uint32_t*)(prev_out + (mt * 32 + mrow) * ld + n - 3) = pack ^ 0x80808080u;
    };
    auto epi_begin = [&]() __attribute__((always_inline)) {
        qn = quad_consts(0);
        lo_v = prev_lo;
        asm volatile("" : "+v"(lo_v));
    };
    // the whole epilogue of the previous pass with nothing under it
    auto epi_standalone = [&](auto fast_c) __attribute__((always_inline)) {
        epi_begin();
        static_for<0, 16>([&](auto q_c) __attribute__((always_inline)) {
            static_for<0, 4>([&](auto i_c) __attribute__((always_inline)) { epi_piece(q_c, i_c, fast_c); });
        });
    };

    // ---- one k-step of this wavefront's 2 x 2 tiles; Q >= 0: with one quad of the previous pass's epilogue
    // between its MFMAs.  Then the activation operands of k-step k + 2 and the weight slot's refill: k-step
    // k + WPF of this pass, or, past its end, of the next pass (clamped to an address that exists when there
    // is nothing left to request; those registers are then never used).
    Stream sc{nullptr, nullptr, 1}, sn{nullptr, nullptr, 1};
    const int8_t* xrow = nullptr;
    v4i xf[2][2];
    auto kstep = [&](int k, auto p_c, auto q_c) __attribute__((always_inline)) {
        constexpr int p = decltype(p_c)::value, Q = decltype(q_c)::value;
        constexpr int xs = p & 1;
        using T = std::true_type;
        cur[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][0], xf[xs][0], cur[0][0], 0, 0, 0);
        if (Q >= 0) epi_piece(std::integral_constant<int, (Q >= 0 ? Q : 0)>{}, std::integral_constant<int, 0>{}, T{});
        cur[0][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][0], xf[xs][1], cur[0][1], 0, 0, 0);
        if (Q >= 0) epi_piece(std::integral_constant<int, (Q >= 0 ? Q : 0)>{}, std::integral_constant<int, 1>{}, T{});
        cur[1][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][1], xf[xs][0], cur[1][0], 0, 0, 0);
        if (Q >= 0) epi_piece(std::integral_constant<int, (Q >= 0 ? Q : 0)>{}, std::integral_constant<int, 2>{}, T{});
        cur[1][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][1], xf[xs][1], cur[1][1], 0, 0, 0);
        if (Q >= 0) epi_piece(std::integral_constant<int, (Q >= 0 ? Q : 0)>{}, std::integral_constant<int, 3>{}, T{});
        const int kk = k + 2 < sc.KS ? k + 2 : sc.KS - 1;
        xf[xs][0] = *(const v4i*)(xrow + kk * 32);
        xf[xs][1] = *(const v4i*)(xrow + 32 * ld + kk * 32);
        const int idx = k + WPF;
        const bool in = idx < sc.KS;
        const int past = idx - sc.KS < sn.KS ? idx - sc.KS : sn.KS - 1;
        const int ks = in ? idx : past;
        wreg[p][0] = wload(in ? sc.b0 : sn.b0, ks);
        wreg[p][1] = wload(in ? sc.b1 : sn.b1, ks);
        __builtin_amdgcn_sched_barrier(0);
    };
    using NoQ = std::integral_constant<int, -1>;
    auto group = [&](int k) __attribute__((always_inline)) {
        static_for<0, WPF>([&](auto p_c) __attribute__((always_inline)) { kstep(k + decltype(p_c)::value, p_c, NoQ{}); });
    };

    // the activation operand ring of the k-steps from k on (k even): k and k + 1
    auto start_ring = [&](int k) __attribute__((always_inline)) {
        const int k1 = k + 1 < sc.KS ? k + 1 : sc.KS - 1;
        xf[0][0] = *(const v4i*)(xrow + k * 32);
        xf[0][1] = *(const v4i*)(xrow + 32 * ld + k * 32);
        xf[1][0] = *(const v4i*)(xrow + k1 * 32);
        xf[1][1] = *(const v4i*)(xrow + 32 * ld + k1 * 32);
    };
    // Everything uniform a pass needs.  It is read from the network description one pass ahead of its use, so
    // that the scalar loads' round trips run under the previous pass's k-steps.
    struct Pass {
        bool valid, active;
        int l, p, grp, npass, N, Np, KS, act, z_out, fast;
        gbytes b0, b1;
        gv4i_ptr pack;
        const int32_t* rshift;
    };
    auto pass_of = [&](int l, int p) {
        Pass q{};
        q.valid = l < nh;
        q.l = l;
        q.p = p;
        if (q.valid) {
            const LayerDev& L = a.L[l];
            const int NT = uni(L.NT), ngroups = NT >> 1;
            q.npass = (ngroups + FW - 1) / FW;
            q.grp = p * FW + wave;
            q.active = q.grp < ngroups;
            q.N = uni(L.N);
            q.Np = NT * 32;
            q.KS = uni(L.KS);
            q.act = uni(L.act);
            q.z_out = uni(a.actq[l + 1].z);
            q.fast = uni(a.fast[l]);
            gbytes wp = (gbytes)uni_ptr(L.wp);
            const int grp = q.active ? q.grp : 0;
            q.b0 = wp + (int64_t)(2 * grp) * q.KS * 1024;
            q.b1 = wp + (int64_t)(2 * grp + 1) * q.KS * 1024;
            q.pack = (gv4i_ptr)uni_ptr(L.bias_fold);
            q.rshift = uni_ptr(L.rshift);
        }
        return q;
    };
    int npass_prev_layer = 0;
    int pass_no = 0;
    bool w_ready = 2 * wave < c.NT0;  // this wavefront's next pass finds its first weights requested already
    Pass P = pass_of(0, 0);
    while (P.valid) {
        const bool more = P.p + 1 < P.npass;
        const Pass Nx = pass_of(more ? P.l : P.l + 1, more ? P.p + 1 : 0);
        const int l = P.l;
        const bool active = P.active;
        sc = Stream{P.b0, P.b1, P.KS};
        // the pass after this one, for the weight stream (nothing to request: this pass's last tile again)
        if (Nx.valid && Nx.active) sn = Stream{Nx.b0, Nx.b1, Nx.KS};
        else sn = Stream{sc.b0 + (int64_t)(sc.KS - 1) * 1024, sc.b1 + (int64_t)(sc.KS - 1) * 1024, 1};
        // this pass's per-channel constants: one 16-byte piece per lane (four arrays x 64 features), parked in
        // the wave's slot at the end of the pass
        v4i cw = {0, 0, 0, 0};
        const int cw_word = (lane >> 4) * P.Np + 64 * P.grp + 4 * (lane & 15);
        if (active) cw = P.pack[cw_word >> 2];
        xrow = buf(l) + mrow * ld + g * 16;
        if (active && !w_ready) {  // (the pass before this one was not this wavefront's, or requested nothing)
#pragma unroll
            for (int q = 0; q < WPF; ++q) {
                wreg[q][0] = wload(sc.b0, q);
                wreg[q][1] = wload(sc.b1, q);
            }
        }
        // k-steps that may run before the previous pass's outputs are visible to every wavefront: all of them
        // within a layer; in a layer's first pass those that read what the previous layer's earlier passes wrote
        const int n_over = P.p > 0 ? sc.KS : WGROUP * (npass_prev_layer - 1);
        int k0 = 0;
        if (have_prev) {
            if (prev_active) {
                if (active && prev_fast && n_over >= WGROUP && sc.KS >= WGROUP) {
                    start_ring(0);
                    epi_begin();
                    static_for<0, WGROUP>([&](auto q_c) __attribute__((always_inline)) {
                        constexpr int q = decltype(q_c)::value;
                        kstep(q, std::integral_constant<int, q % WPF>{}, q_c);
                    });
                    k0 = WGROUP;
                } else if (prev_fast) {
                    epi_standalone(std::true_type{});
                } else {
                    epi_standalone(std::false_type{});
                }
            }
            // the previous pass's features are in LDS for every wavefront (the k-steps below, or a later pass of
            // any wavefront, read them)
            lds_barrier();
        }
        if (active) {
            if (k0 < sc.KS) start_ring(k0);  // (after the barrier: the ring reads two k-steps ahead)
            for (int k = k0; k < sc.KS; k += WPF) group(k);
            // park the constants: [bias_fold | M0 | rz | sh] x 64 features
            *(v4i*)(my_cst + (pass_no & 1) * WSLOT + (lane >> 4) * 64 + 4 * (lane & 15)) = cw;
        }
        w_ready = active && sn.KS > 1;  // (KS is at least 4: a one-step stream is the placeholder)
        // hand the accumulators to the next pass's epilogue
        have_prev = true;
        prev_active = active;
        prev_grp = P.grp;
        prev_N = P.N;
        prev_zout = P.z_out;
        prev_lo = P.act == AQ_ACT_RELU ? P.z_out : 0;
        prev_fast = P.fast;
        prev_slot = pass_no & 1;
        prev_rshift = P.rshift;
        prev_out = buf(l + 1);
        if (TAPS) {
            prev_tacc = t.acc[l];
            prev_tact = t.act[l];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                prev[i][j] = cur[i][j];
                cur[i][j] = zero16();
            }
        if (!more) npass_prev_layer = P.npass;
        P = Nx;
        ++pass_no;
    }
    // The narrow last layer's constants and this wavefront's first weights of it do not depend on the hidden
    // layers: requested before the last epilogue.
    const LayerView LL = layer_view(a, nh, n_layers);
    const NarrowMap nm = narrow_map<2>(LL.NT, LL.KS, wave);
    v4i cv0 = {0, 0, 0, 0}, cv1 = cv0;
    load_consts(LL, tid, cv0, cv1);
    gv4i_ptr nwptr[1];
    nwptr[0] = (gv4i_ptr)LL.wp + (int64_t)nm.nt * LL.KS * 64 + lane;
    v4i nw[4][1];
    if (nm.k0 < nm.k1) mma_prefetch<1, 4>(nwptr, nm.k0, nm.k1, nw);
    // the last hidden pass has nothing to hide under
    if (have_prev && prev_active) {
        if (prev_fast) epi_standalone(std::true_type{});
        else epi_standalone(std::false_type{});
    }

    // ---- narrow last layer (at most two feature tiles): spread over all eight wavefronts by splitting K
    {
        const int l = nh;
        const LayerView& L = LL;
        LayerTaps T{nullptr, nullptr, nullptr};
        if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
        const int Np = L.NT * 32;
        lds_barrier();  // every hidden feature is in LDS
        const int8_t* in = buf(l);
        const CPtrs C{cst_last, cst_last + Np, L.rshift, cst_last + 2 * Np, cst_last + 3 * Np, (const float*)(cst_last + Np)};
        v16i pacc[1][1], prs[1];
        pacc[0][0] = zero16();
        prs[0] = zero16();
        if (nm.k0 < nm.k1)
            mma_run<1, 1, false, 4>(nwptr, nw, in + nm.mt * 32 * ld, ld, nm.k0, nm.k1, 0, pacc, prs, lane);
        int32_t* part = (int32_t*)buf(l + 1);  // the idle activation buffer (64 * ld >= PART_BYTES, checked by the launcher)
        {
            int32_t* mine = part + wave * PART_WORDS + lane;
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[r * 64] = pacc[0][0][r];
        }
        park_consts(L.pieces, tid, cst_last, cv0, cv1);
        lds_barrier();  // partial sums and the layer's constants are in LDS; the layer's input is free
        float* yrow = (float*)buf(l);
        const int ldy = Np + 1;
        const int head = uni(a.head);
        float* direct = head != AQ_HEAD_ARGMAX ? (float*)c.actions : nullptr;
        float* tap_y = TAPS ? t.y : nullptr;
        if (L.NT == 1)
            narrow_reduce<2, 1, false, TAPS, false>(part, C, T, L.N, 0, row0, c.batch, yrow, ldy, tid, head, direct, tap_y, c);
        else
            narrow_reduce<2, 2, false, TAPS, false>(part, C, T, L.N, 0, row0, c.batch, yrow, ldy, tid, head, direct, tap_y, c);
        if (direct) return;
        lds_barrier();
        // argmax over the dequantized rows (lowest index wins ties)
        for (int m = tid; m < WROWS; m += FT) {
            const int64_t row = row0 + m;
            if (row >= c.batch) continue;
            int best = 0;
            for (int n = 0; n < L.N; ++n) {
                const float y = yrow[m * ldy + n];
                if (TAPS) {
                    if (t.y) t.y[row * L.N + n] = y;
                }
                if (y > yrow[m * ldy + best]) best = n;
            }
            ((int32_t*)c.actions)[row] = best;
        }
    }
}

template <bool TAPS>
aq_status launch_wide_t(const FwdArgs& a, size_t lds, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute((const void*)k_mlp_wide<TAPS>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    if (attr_err != hipSuccess) return AQ_EHIP;
    const unsigned grid = (unsigned)((a.c.batch + WROWS - 1) / WROWS);
    hipLaunchKernelGGL((k_mlp_wide<TAPS>), dim3(grid), dim3(FT), lds, st, a.d_net, a.c, a.t);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace

// Shapes the pipelined kernel takes (see the head of this file); `ld_out`: its LDS row stride.
bool wide_mlp_supported(const FwdArgs& a, int* ld_out) {
    const NetDev& n = a.net;
    if (n.asym || n.in_u8 || n.n_layers < 2) return false;
    int maxw = 0;
    for (int l = 0; l < n.n_layers; ++l) {
        const LayerDev& L = n.L[l];
        if (L.kh != 1 || L.kw != 1 || L.in_h != 1 || L.in_w != 1) return false;
        if (L.K % 128 != 0) return false;
        if (l < n.n_layers - 1) {
            if (L.N % 64 != 0 || L.N > CST_MAXN || L.act == AQ_ACT_LN_TANH) return false;
        } else if (L.NT > NARROW_NT) {
            return false;
        }
        maxw = maxw > L.K ? maxw : L.K;
    }
    const int ld = maxw + 16;
    // the narrow last layer parks its K-split partial sums in the idle activation buffer and its fp32 rows
    // (stride 32 * NT + 1 floats) in the other one
    if ((size_t)WROWS * ld < (size_t)PART_BYTES) return false;
    if ((size_t)ld < (size_t)(NARROW_NT * 32 + 1) * 4) return false;
    if (wide_lds_bytes(ld) > 160 * 1024) return false;
    *ld_out = ld;
    return true;
}

aq_status launch_wide_mlp(const FwdArgs& a_in, hipStream_t st) {
    int ld = 0;
    if (!wide_mlp_supported(a_in, &ld)) return AQ_ESHAPE;
    if (((uintptr_t)a_in.c.obs & 15) != 0) return AQ_ESHAPE;
    FwdArgs a = a_in;
    a.c.ld = ld;
    a.c.wp0 = a.net.L[0].wp;
    a.c.NT0 = a.net.L[0].NT;
    a.c.KS0 = a.net.L[0].KS;
    const size_t lds = wide_lds_bytes(ld);
    return any_taps(a) ? launch_wide_t<true>(a, lds, st) : launch_wide_t<false>(a, lds, st);
}

}  // namespace aq
