// Whole-network int8 MLP for small policies at small batch (Sec. 3.1 actor inference on the 8-bit policy of
// Sec. 3.2): one workgroup of 8 wavefronts owns 16 batch rows from the observation to the action.
//
// At these sizes (a few hundred features per layer, at most one 16-row block per CU) a launch holds a
// fraction of a microsecond of matrix-core work; its time is the chain of round trips inside one workgroup.
// This kernel is laid out to keep that chain short:
//   - v_mfma_i32_16x16x64_i8: a tile is 16 features x 16 batch rows, so a 16-row block fills it (no
//     don't-care rows, no fold afterwards) and K = 256 is four dependent MFMAs instead of eight; a wavefront
//     owns 32 features = two independent accumulator chains;
//   - the kernel arguments fit one 64-byte line (they live in host-visible memory: every line of them costs
//     a round trip over the host link on first touch, about 1800 clocks measured); everything else about the
//     network - every layer's pointers and sizes, the activation scales and zero-points, the short-form
//     flags - comes from the device-resident description by one burst of scalar loads at the start: no
//     layer waits for a descriptor;
//   - weights and per-channel constants go from global memory straight to registers, one layer ahead: all
//     of a layer's operands (at most 8 KiB per wavefront) are requested at the start of the previous layer,
//     the constants of its epilogue too.  A lane's four features of a tile are shared by the 16 lanes of its
//     row, so each lane fetches one 16-byte piece (array x tile) and the epilogue takes its operands from the
//     row's lanes by DPP row broadcasts: one load instruction per wavefront and layer instead of eight (the
//     CU's single vector memory path, 64 B / clock, is what the eight wavefronts queue for), no staging in
//     LDS, no barrier to publish them;
//   - LayerNorm statistics cross the wavefronts once: every wavefront reduces its 32 features to (sum, sum of
//     squared deviations from its own mean), and the eight pairs combine exactly (the pairwise update of
//     Chan, Golub, LeVeque 1979), so the layer has two barriers less than a mean pass followed by a
//     deviation pass;
//   - one barrier per layer; the narrow last layer is split over all wavefronts (feature tile x K).
//
// Weights are read from the library's 32 x 32 operand tiles unchanged: the 16-byte piece of lane
// (n % 32) + 32 * ((k % 32) / 16) of tile (n / 32, k / 32) is what lane (n % 16) + 16 * g of the 16 x 16 x 64
// operand needs when k-group g of a 64-wide k-step is taken to mean bytes 16 g .. 16 g + 15 of it.
//
// Shapes: per-channel symmetric weights, fp32 observations at a 16-byte aligned address, one to four fully
// connected layers, first-layer K and hidden widths at most 256, last layer at most 64 outputs.
#include <mutex>

#include "explore_device.hpp"
#include "int8_device.hpp"

namespace aq {
namespace {

constexpr int RW = 8;          // wavefronts per workgroup
constexpr int RT = RW * 64;    // threads per workgroup
constexpr int RROWS = 16;      // batch rows per workgroup
constexpr int RLD = 272;       // LDS row stride, bytes: 256 codes + 16 (rows land on different banks)
constexpr int RMAXL = 4;       // layers
constexpr int RMAXK = 256;     // widest layer input / hidden layer
constexpr int RSTEPS = 4;      // k-steps of 64 per layer at most

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float unif(float v) { return __int_as_float(uni(__float_as_int(v))); }

constexpr float K2_LOG2E = 2.885390081777927f;  // 2 log2(e): tanh(y) = 1 - 2 / (2^(K2 y) + 1)

// what the kernel uses of one layer, read from the device-resident description into scalar registers
struct R16Layer {
    const int8_t* wp;       // packed weights, [NT][KS] tiles of 1 KiB
    const int32_t* pack;    // four [32 NT] arrays: bias_fold | M0 or m | rz or gamma | sh or beta
    const int32_t* rshift;  // [32 NT] shifts of the general requantization form
    int N, NT, KS, act;
};
// the kernel arguments besides the description's address: 56 bytes, one line together with it
struct R16Args {
    const float* obs;
    void* actions;
    int64_t batch;
    const float* ex_sigma;  // Gaussian exploration noise added where the actions are written, or NULL
    uint32_t ex_k0, ex_k1, ex_s0, ex_s1;
    int K0, n_layers;
};
static_assert(sizeof(R16Args) == 56, "the kernel arguments must stay within one 64-byte line");

template <class T>
__device__ __forceinline__ T* uni_ptr(T* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (T*)(((uint64_t)hi << 32) | lo);
}

// lane N of every 16-lane row, broadcast to that row
template <int N>
__device__ __forceinline__ int row_bcast(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + N, 0xF, 0xF, false);
}

// The same as an operand of its own instruction.  Needed for shift amounts: the compiler folds a row broadcast
// into the shift (v_ashrrev_i32_dpp), and that instruction came back from the hardware with the broadcast
// applied to the shifted value instead of the amount (additions and plain moves are right).
template <int N>
__device__ __forceinline__ int row_bcast_mov(int v) {
    int r = row_bcast<N>(v);
    asm volatile("" : "+v"(r));
    return r;
}

// sum over the four 16-lane rows of a wavefront (lane ^ 16, then lane ^ 32), the same value in every lane
__device__ __forceinline__ float sum_rows4(float s) {
    const auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(s), false, false);
    s = __uint_as_float(p[0]) + __uint_as_float(p[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(s), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// NH = number of hidden layers (the network has NH + 1 layers): a compile-time fact, so that every global load
// sits in straight-line code and the compiler can count exactly which ones an instruction has to wait for (with
// the layer count a run-time value, epilogues waited for the loads of the next layer requested just before them)
template <int NH, bool TAPS>
__global__ __launch_bounds__(RT) void k_mlp_rows16(const NetDev* __restrict__ netp, const R16Args c, const TapArgs t) {
    __shared__ __align__(16) int8_t s_buf[2][RROWS * RLD];
    __shared__ __align__(16) float s_red[RROWS * RW * 2];
    __shared__ __align__(16) int32_t s_part[RW * 4 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
    const int b = lane & 15, g4 = lane >> 4;  // this lane's batch row and k-group (operands) / feature quad (results)
    const int64_t row0 = (int64_t)blockIdx.x * RROWS;
    const int64_t row = row0 + b;
    const bool row_ok = row < c.batch;
    constexpr int nh = NH;

    // The network, from the device-resident description: every layer's facts, (scale, zero-point) of every
    // activation tensor and the short-form flags, all requested here in one burst of scalar loads (slots past
    // the last layer exist in the description and are not used).
    struct {
        R16Layer L[RMAXL];
        int head;
        float ln_eps;
    } a;
#pragma unroll
    for (int i = 0; i < RMAXL; ++i) {
        const LayerDev& s = netp->L[i];
        a.L[i] = R16Layer{uni_ptr(s.wp), uni_ptr(s.bias_fold), uni_ptr(s.rshift), uni(s.N), uni(s.NT), uni(s.KS), uni(s.act)};
    }
    const R16Layer LL = a.L[NH];
    a.head = uni(netp->head);
    a.ln_eps = unif(netp->ln_eps);
    float s_q[RMAXL + 1];
    int z_q[RMAXL + 1], fastf[RMAXL];
#pragma unroll
    for (int i = 0; i <= RMAXL; ++i) {
        s_q[i] = unif(netp->actq[i].s);
        z_q[i] = uni(netp->actq[i].z);
    }
#pragma unroll
    for (int i = 0; i < RMAXL; ++i) fastf[i] = uni(netp->fast[i]);

    // ---- requests: observations, then the first layer's operands and constants
    const int K0 = c.K0;
    const int64_t left = c.batch - row0;
    const int vrows = left < RROWS ? (int)left : RROWS;
    // a thread takes up to two (row, four consecutive k) quads: one 16-byte load where the rows are 16-byte
    // aligned (K0 a multiple of 4), four 4-byte loads otherwise
    const int q4 = (K0 + 3) >> 2;  // quads per row, <= 64
    const float inv_q4 = 1.0f / (float)q4;
    const float* src1 = c.obs + row0 * K0;
    const bool k_al = (K0 & 3) == 0;
    float4 ov[2];
    int om[2], ok4[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = tid + u * RT;
        // q / q4: (q + 0.5) / q4 stays at least 0.5 / q4 away from every integer
        om[u] = (int)(((float)q + 0.5f) * inv_q4);
        ok4[u] = 4 * (q - om[u] * q4);
        ov[u] = float4{0.0f, 0.0f, 0.0f, 0.0f};
        if (om[u] < vrows) {
            const float* src = src1 + om[u] * K0 + ok4[u];
            if (k_al) {
                ov[u] = *(const float4*)src;
            } else {
                ov[u].x = src[0];
                if (ok4[u] + 1 < K0) ov[u].y = src[1];
                if (ok4[u] + 2 < K0) ov[u].z = src[2];
                if (ok4[u] + 3 < K0) ov[u].w = src[3];
            }
        }
    }

    // hidden layer operands of this wavefront's 32 features: [k-step][16-feature tile]; loads are unconditional
    // from clamped addresses (an idle wavefront re-reads the last tile, a k-group past K the last k-tile: those
    // registers are not used, or meet zero activations)
    // (`first`: the first layer's requests are the kernel's first, with nothing older in flight whose wait they
    // could blur, so the k-steps past its K - most of them for a narrow observation - are skipped)
    auto load_w = [&](const R16Layer& L, v4i (&w)[RSTEPS][2], bool first) __attribute__((always_inline)) {
        const int nt = wave < L.NT ? wave : L.NT - 1;
        gv4i_ptr base = (gv4i_ptr)L.wp + (int64_t)nt * L.KS * 64 + (b + 32 * (g4 & 1));
#pragma unroll
        for (int s = 0; s < RSTEPS; ++s) {
            int ks = 2 * s + (g4 >> 1);
            ks = ks < L.KS ? ks : L.KS - 1;
            if (!first || 2 * s < L.KS) {
#pragma unroll
                for (int tl = 0; tl < 2; ++tl) w[s][tl] = base[ks * 64 + 16 * tl];
            }
        }
    };
    // ... and the constants of its epilogue.  The lanes of a 16-lane row all need the same eight 16-byte
    // pieces (four arrays x two tiles, the row's four consecutive features of each tile): lane j (and j + 8)
    // of the row fetches piece j = 2 * array + tile, the epilogue reads piece j from lane j of its row.
    auto load_c = [&](const R16Layer& L, bool pack_sh) __attribute__((always_inline)) {
        const int nt = wave < L.NT ? wave : L.NT - 1;
        const int Np = L.NT * 32;
        const int arr = (b >> 1) & 3, tl = b & 1;
        const int32_t* base = L.pack + arr * Np;
        if (arr == 3 && !pack_sh) base = L.rshift;
        return *(gv4i_ptr)(base + 32 * nt + 16 * tl + 4 * g4);
    };
    // piece 2 * A + TL of this lane's row
#define AQ_R16_C(cm, A, TL, i) row_bcast<2 * (A) + (TL)>((cm)[i])
#define AQ_R16_CSH(cm, A, TL, i) row_bcast_mov<2 * (A) + (TL)>((cm)[i])
    // the narrow last layer: its 2 NT 16-feature tiles go to different wavefronts, the wavefronts left over
    // split K; at most two k-steps each
    struct LastMap {
        int t16, ksplit, tile, kp;
    };
    auto last_map = [&](const R16Layer& L) __attribute__((always_inline)) {
        LastMap m;
        m.t16 = 2 * L.NT;                       // 2 or 4
        m.ksplit = L.NT == 1 ? 4 : 2;           // RW / t16
        m.tile = wave & (m.t16 - 1);
        m.kp = L.NT == 1 ? wave >> 1 : wave >> 2;
        return m;
    };
    auto load_wl = [&](const R16Layer& L, v4i (&w)[2]) __attribute__((always_inline)) {
        const LastMap m = last_map(L);
        gv4i_ptr base = (gv4i_ptr)L.wp + (int64_t)(m.tile >> 1) * L.KS * 64 + (16 * (m.tile & 1) + b + 32 * (g4 & 1));
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int ks = 2 * (m.kp + j * m.ksplit) + (g4 >> 1);
            ks = ks < L.KS ? ks : L.KS - 1;
            w[j] = base[ks * 64];
        }
    };

    v4i w[2][RSTEPS][2];  // operands of the layer being multiplied, and of the next one
    v4i cst[2];           // this lane's piece of the constants of the layer whose epilogue runs, and of the next one
    v4i wl[2];            // operands of the last layer
    auto is_ln = [&](int l) { return a.L[l].act == AQ_ACT_LN_TANH; };
    if constexpr (nh > 0) {
        load_w(a.L[0], w[0], true);
        cst[0] = load_c(a.L[0], is_ln(0) || fastf[0]);
    } else {
        load_wl(LL, wl);
    }

    // ---- observation quantize: a0 = clamp(round(x / s0) + z0, 0, 255), kept in the signed domain: four
    // values at a time, one aligned 4-byte LDS store per quad
    {
        int8_t* buf = s_buf[0];
        const QuantScale qs0 = make_quant_scale(s_q[0]);
        const float zf0 = (float)z_q[0];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (om[u] < RROWS) {
                uint32_t pack = quant_u8x4(ov[u], qs0, zf0);
                const int left_k = K0 - ok4[u];  // real values in this quad: 1..4 (or more)
                if (TAPS) {
                    if (t.a0 && om[u] < vrows) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (i < left_k) t.a0[(row0 + om[u]) * K0 + ok4[u] + i] = (uint8_t)(pack >> (8 * i));
                    }
                }
                pack ^= 0x80808080u;
                // zero (signed domain) past K0 and in the rows past the batch
                if (left_k < 4) pack &= (1u << (8 * left_k)) - 1u;
                if (om[u] >= vrows) pack = 0u;
                *(uint32_t*)(buf + om[u] * RLD + ok4[u]) = pack;
            }
        }
        // ... and up to the end of the last 64-wide k-step
        const int kz4 = ((K0 + 63) & ~63) >> 2, extra = kz4 - q4;  // words per row
        if (extra > 0) {
            const float inv_e = 1.0f / (float)extra;
            for (int i = tid; i < RROWS * extra; i += RT) {
                const int m = (int)(((float)i + 0.5f) * inv_e), kq = q4 + i - m * extra;
                *(uint32_t*)(buf + m * RLD + 4 * kq) = 0u;
            }
        }
    }
    lds_barrier();

    // ---- hidden layers
    static_for<0, NH>([&](auto l_c) __attribute__((always_inline)) {
        constexpr int l = decltype(l_c)::value;
        {
            const R16Layer& L = a.L[l];
            const int8_t* in = s_buf[l & 1];
            int8_t* out = s_buf[(l + 1) & 1];
            const bool active = wave < L.NT;
            const int ks64 = (L.KS + 1) >> 1;
            const bool ln = is_ln(l);
            LayerTaps T{nullptr, nullptr, nullptr};
            if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};

            // The next layer's operands and constants are requested first: their eight loads per wavefront queue
            // at the CU's single vector memory path (64 KiB per 256 x 256 layer at 64 B / clock), and a
            // wavefront stuck there cannot start its epilogue; here it would be waiting for LDS anyway.
            if constexpr (l + 1 < nh) {
                load_w(a.L[l + 1], w[(l + 1) & 1], false);
                cst[(l + 1) & 1] = load_c(a.L[l + 1], is_ln(l + 1) || fastf[l + 1]);
            } else {
                load_wl(LL, wl);
            }
            v4i acc[2];
            acc[0] = acc[1] = v4i{0, 0, 0, 0};
            {
                v4i bx[RSTEPS];
                const int8_t* xrow = in + b * RLD + 16 * g4;
#pragma unroll
                for (int s = 0; s < RSTEPS; ++s) bx[s] = *(const v4i*)(xrow + 64 * s);
                if (active) {
#pragma unroll
                    for (int s = 0; s < RSTEPS; ++s) {
                        if (s < ks64) {
                            acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w[l & 1][s][0], bx[s], acc[0], 0, 0, 0);
                            acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w[l & 1][s][1], bx[s], acc[1], 0, 0, 0);
                        }
                    }
                }
            }
            const v4i cm = cst[l & 1];
            const float s_out = s_q[l + 1];
            const int z_out = z_q[l + 1];
            const int nbase = 32 * wave + 4 * g4;
            // a layer with an odd number of 32-feature tiles: the next layer's last 64-wide k-step reads 32
            // columns nobody computes; the first idle wavefront zeroes them
            if ((L.NT & 1) && wave == L.NT) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int e = lane + 64 * i;  // 16 rows x 8 words
                    *(uint32_t*)(out + (e >> 3) * RLD + 32 * L.NT + 4 * (e & 7)) = 0u;
                }
            }
            if (!ln) {
                if (active) {
                    const int lo = L.act == AQ_ACT_RELU ? z_out : 0;
                    int lo_v = lo;
                    asm volatile("" : "+v"(lo_v));
                    // (the form of the requantization is a fact of the layer: one branch around the whole tile pair)
                    auto tiles = [&](auto fast_c) __attribute__((always_inline)) {
                        constexpr bool fast = decltype(fast_c)::value;
                        static_for<0, 2>([&](auto tl_c) __attribute__((always_inline)) {
                            constexpr int tl = decltype(tl_c)::value;
                            const int n0 = nbase + 16 * tl;
                            uint32_t pack = 0;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int val = acc[tl][i] + AQ_R16_C(cm, 0, tl, i);
                                if (TAPS) {
                                    if (T.acc && row_ok && n0 + i < L.N) T.acc[row * L.N + n0 + i] = val;
                                }
                                int code;
                                if (fast)
                                    code = clamp_code((__mulhi(val, AQ_R16_C(cm, 1, tl, i)) + AQ_R16_C(cm, 2, tl, i)) >>
                                                          AQ_R16_CSH(cm, 3, tl, i), lo_v, 255);
                                else
                                    code = requant_code(val, AQ_R16_C(cm, 1, tl, i), AQ_R16_CSH(cm, 3, tl, i), z_out, lo);
                                if (TAPS) {
                                    if (T.act && row_ok && n0 + i < L.N) T.act[row * L.N + n0 + i] = (uint8_t)code;
                                }
                                pack |= (uint32_t)code << (8 * i);
                            }
                            *(uint32_t*)(out + b * RLD + n0) = pack ^ 0x80808080u;
                        });
                    };
                    if (fastf[l]) tiles(std::true_type{});
                    else tiles(std::false_type{});
                }
            } else {
                // LayerNorm over the layer's N features, tanh, re-quantize.  x = acc * (s_in s_w) in fp32; this
                // wavefront's features (32, fewer in the last tile) give (sum, squared deviations from their own
                // mean) per row.  Reciprocals of the feature counts and of the standard deviation come from the
                // reciprocal units (1 ulp, against a tolerance of 1e-4 on the result).
                const int n_w = L.N - 32 * wave < 0 ? 0 : (L.N - 32 * wave > 32 ? 32 : L.N - 32 * wave);
                float x[2][4];
                float s = 0.0f;
                static_for<0, 2>([&](auto tl_c) __attribute__((always_inline)) {
                    constexpr int tl = decltype(tl_c)::value;
                    const int n0 = nbase + 16 * tl;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int val = acc[tl][i] + AQ_R16_C(cm, 0, tl, i);
                        if (TAPS) {
                            if (T.acc && active && row_ok && n0 + i < L.N) T.acc[row * L.N + n0 + i] = val;
                        }
                        // (padding features: their scale is stored as zero, so x = 0; idle wavefronts hold
                        // zero accumulators and re-read the last tile's constants: their pair is not used)
                        x[tl][i] = (float)val * __int_as_float(AQ_R16_C(cm, 1, tl, i));
                        s += x[tl][i];
                    }
                });
                s = sum_rows4(s);
                const float mean_w = s * __builtin_amdgcn_rcpf((float)(n_w > 0 ? n_w : 1));
                float q = 0.0f;
                if (n_w == 32) {
#pragma unroll
                    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float d = x[tl][i] - mean_w;
                            q = fmaf(d, d, q);
                        }
                } else {
#pragma unroll
                    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float d = x[tl][i] - mean_w;
                            if (nbase + 16 * tl + i < L.N) q = fmaf(d, d, q);
                        }
                }
                q = sum_rows4(q);
                if (g4 == 0) *(float2*)(s_red + (b * RW + wave) * 2) = float2{s, q};
                // the output scale's reciprocal: needed after the barrier, computed while waiting for it
                const QuantScale qs_out = make_quant_scale(s_out);
                const float c0 = qs_out.inv + (float)z_out, c1 = 2.0f * qs_out.inv;
                const float inv_N = __builtin_amdgcn_rcpf((float)L.N);
                const int n_full = L.N >> 5, n_tail = L.N & 31;  // wavefronts with 32 features, features of the next one
                const float inv_tail = __builtin_amdgcn_rcpf((float)(n_tail > 0 ? n_tail : 1));
                lds_barrier();
                float sw[RW], qw[RW];
#pragma unroll
                for (int i = 0; i < RW / 2; ++i) {
                    const float4 v = *(const float4*)(s_red + b * RW * 2 + 4 * i);
                    sw[2 * i] = v.x;
                    qw[2 * i] = v.y;
                    sw[2 * i + 1] = v.z;
                    qw[2 * i + 1] = v.w;
                }
                float tot = 0.0f;
#pragma unroll
                for (int i = 0; i < RW; ++i)
                    if (i < n_full || (i == n_full && n_tail > 0)) tot += sw[i];
                const float mean = tot * inv_N;
                // pairwise combination: sum of squared deviations from the common mean
                float m2 = 0.0f;
#pragma unroll
                for (int i = 0; i < RW; ++i) {
                    if (i < n_full) {
                        const float d = sw[i] * 0.03125f - mean;
                        m2 += fmaf(32.0f * d, d, qw[i]);
                    } else if (i == n_full && n_tail > 0) {
                        const float d = sw[i] * inv_tail - mean;
                        m2 += fmaf((float)n_tail * d, d, qw[i]);
                    }
                }
                const float inv = __builtin_amdgcn_rsqf(fmaf(m2, inv_N, a.ln_eps));
                const float shift = -mean * inv;
                if (active) {
                    // code = round(t / s + z) with t = 1 - 2 r, r = 1 / (2^e + 1): round(c0 - c1 r)
                    static_for<0, 2>([&](auto tl_c) __attribute__((always_inline)) {
                        constexpr int tl = decltype(tl_c)::value;
                        const int n0 = nbase + 16 * tl;
                        float rv[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            // gain and offset times 2 log2(e); r = 1 / (e^{2y} + 1) on the exp2 and reciprocal
                            // units for either sign (exp2 saturates to 0 and +inf, rcp(inf) = 0)
                            const float gv = __int_as_float(AQ_R16_C(cm, 2, tl, i)) * K2_LOG2E;
                            const float bv = __int_as_float(AQ_R16_C(cm, 3, tl, i)) * K2_LOG2E;
                            const float e = __builtin_amdgcn_exp2f(fmaf(fmaf(x[tl][i], inv, shift), gv, bv));
                            rv[i] = __builtin_amdgcn_rcpf(e + 1.0f);
                        }
                        uint32_t pack;
                        if (qs_out.rcp_ok) {
                            // the tanh value already carries rounding differences of its own, so the code is taken
                            // from t * (1/s) + z directly (it can differ from round(t/s) only at a rounding tie)
                            pack = 0;
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                pack = __builtin_amdgcn_cvt_pk_u8_f32(rintf(fmaf(rv[i], -c1, c0)), i, pack);
                        } else {
                            pack = quant_code4(float4{fmaf(rv[0], -2.0f, 1.0f), fmaf(rv[1], -2.0f, 1.0f),
                                                      fmaf(rv[2], -2.0f, 1.0f), fmaf(rv[3], -2.0f, 1.0f)},
                                               qs_out, -z_out, 255 - z_out, z_out);
                        }
                        if (TAPS) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                if (row_ok && n0 + i < L.N) {
                                    if (T.ln) T.ln[row * L.N + n0 + i] = fmaf(rv[i], -2.0f, 1.0f);
                                    if (T.act) T.act[row * L.N + n0 + i] = (uint8_t)(pack >> (8 * i));
                                }
                            }
                        }
                        *(uint32_t*)(out + b * RLD + n0) = pack ^ 0x80808080u;
                    });
                }
            }
            lds_barrier();
        }
    });

    // ---- last layer: K split over the wavefronts, partial sums meet in LDS
    {
        const int l = nh;
        const R16Layer& L = LL;
        const int8_t* in = s_buf[l & 1];
        const int Np = L.NT * 32;
        const LastMap lm = last_map(L);
        const int ks64 = (L.KS + 1) >> 1;
        v4i acc = v4i{0, 0, 0, 0};
        {
            v4i bx[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int s = lm.kp + j * lm.ksplit;
                bx[j] = *(const v4i*)(in + b * RLD + 64 * (s < RSTEPS ? s : RSTEPS - 1) + 16 * g4);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (lm.kp + j * lm.ksplit < ks64) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wl[j], bx[j], acc, 0, 0, 0);
        }
        // this thread's outputs of the reduction: (tile, register, lane) = (o >> 8, (o >> 6) & 3, o & 63) for
        // o = tid (+ 512 with four tiles), so that its LDS reads are conflict-free; their bias and scale
        int bf[2];
        float ms[2];
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int o = tid + it * RT;
            const int n = 16 * (o >> 8) + 4 * ((o & 63) >> 4) + ((o >> 6) & 3);
            bf[it] = 0;
            ms[it] = 0.0f;
            if (n < Np) {
                bf[it] = *(gint_ptr)(L.pack + n);
                ms[it] = __int_as_float(*(gint_ptr)(L.pack + Np + n));
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) s_part[(wave * 4 + r) * 64 + lane] = acc[r];
        lds_barrier();
        float* ybuf = (float*)s_buf[l & 1];  // argmax policies: dequantized rows, stride Np + 1 (the input is free now)
        const int ldy = Np + 1;
        const int head = a.head;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            if (it < L.NT) {
                const int o = tid + it * RT;
                const int tile = o >> 8, r = (o >> 6) & 3, ln_ = o & 63;
                int v = 0;
#pragma unroll
                for (int kp = 0; kp < 4; ++kp)
                    if (kp < lm.ksplit) v += s_part[((tile + lm.t16 * kp) * 4 + r) * 64 + ln_];
                v += bf[it];
                const int n = 16 * tile + 4 * (ln_ >> 4) + r, m = ln_ & 15;
                const int64_t orow = row0 + m;
                const bool ok = orow < c.batch && n < L.N;
                if (TAPS) {
                    if (t.acc[l] && ok) t.acc[l][orow * L.N + n] = v;
                }
                const float y = (float)v * ms[it];
                if (head == AQ_HEAD_ARGMAX) {
                    ybuf[m * ldy + n] = y;
                } else if (ok) {
                    if (TAPS) {
                        if (t.y) t.y[orow * L.N + n] = y;
                    }
                    float act = head == AQ_HEAD_TANH ? tanh_head(y) : y;
                    if (c.ex_sigma)  // exploration noise of Sec. 4.1, sigma per actor (= per batch row)
                        act = act + c.ex_sigma[orow] * gaussian_draw((uint32_t)orow, n, c.ex_k0, c.ex_k1, c.ex_s0, c.ex_s1);
                    ((float*)c.actions)[orow * L.N + n] = act;
                }
            }
        }
        if (head != AQ_HEAD_ARGMAX) return;
        lds_barrier();
        // argmax over the dequantized rows (lowest index wins ties)
        if (tid < RROWS && row0 + tid < c.batch) {
            int best = 0;
            for (int n = 0; n < L.N; ++n) {
                const float y = ybuf[tid * ldy + n];
                if (TAPS) {
                    if (t.y) t.y[(row0 + tid) * L.N + n] = y;
                }
                if (y > ybuf[tid * ldy + best]) best = n;
            }
            ((int32_t*)c.actions)[row0 + tid] = best;
        }
    }
}

template <bool TAPS>
aq_status launch_rows16_t(const NetDev* d_net, const R16Args& ra, const TapArgs& t, hipStream_t st) {
    const unsigned grid = (unsigned)((ra.batch + RROWS - 1) / RROWS);
    switch (ra.n_layers) {
        case 1: hipLaunchKernelGGL((k_mlp_rows16<0, TAPS>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        case 2: hipLaunchKernelGGL((k_mlp_rows16<1, TAPS>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        case 3: hipLaunchKernelGGL((k_mlp_rows16<2, TAPS>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        case 4: hipLaunchKernelGGL((k_mlp_rows16<3, TAPS>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        default: return AQ_ESHAPE;
    }
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace

// Shapes the 16-row kernel takes (see the head of this file).
bool rows16_mlp_supported(const FwdArgs& a) {
    const NetDev& n = a.net;
    if (n.asym || n.in_u8 || n.n_layers < 1 || n.n_layers > RMAXL) return false;
    for (int l = 0; l < n.n_layers; ++l) {
        const LayerDev& L = n.L[l];
        if (L.kh != 1 || L.kw != 1 || L.in_h != 1 || L.in_w != 1) return false;
        if (L.KS * 32 > RMAXK) return false;
        if (l < n.n_layers - 1) {
            if (L.NT * 32 > RMAXK) return false;
        } else if (L.NT > 2) {
            return false;
        }
    }
    return true;
}

aq_status launch_rows16_mlp(const FwdArgs& a, hipStream_t st) {
    if (!rows16_mlp_supported(a) || ((uintptr_t)a.c.obs & 15) != 0) return AQ_ESHAPE;
    R16Args ra{};
    ra.obs = (const float*)a.c.obs;
    ra.actions = a.c.actions;
    ra.batch = a.c.batch;
    ra.K0 = a.net.L[0].K;
    ra.n_layers = a.net.n_layers;
    ra.ex_sigma = a.c.ex_sigma;
    ra.ex_k0 = a.c.ex_k0;
    ra.ex_k1 = a.c.ex_k1;
    ra.ex_s0 = a.c.ex_s0;
    ra.ex_s1 = a.c.ex_s1;
    return any_taps(a) ? launch_rows16_t<true>(a.d_net, ra, a.t, st) : launch_rows16_t<false>(a.d_net, ra, a.t, st);
}

}  // namespace aq
