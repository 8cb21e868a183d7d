// One launch per layer: FC and implicit-GEMM convolution on int8 MFMA (Sec. 3.1 actor inference on
// the quantized policy of Sec. 3.2), activations in global memory between layers.
//
// A workgroup of W waves owns ROWS = 32 * MT output rows (rows = batch * oh * ow positions) and, per
// pass, W * NB feature tiles; the rows' K bytes are staged in LDS (the whole K when it fits, else
// in chunks), weights stream from L2 straight into MFMA operand registers.  Each wave's tile is
// (NB*32 features) x (MT*32 rows): with MT = 4 a weight operand is reused for four MFMAs, which
// keeps the L2 -> register stream of a wide layer under a quarter KiB per MFMA; two waves per SIMD
// let one wave's epilogue overlap the other's MFMAs.
#include "int8_device.hpp"

namespace aq {

// address of the first of the contiguous input bytes that hold k .. of output row `row`
__device__ __forceinline__ int64_t gather_offset(const LayerDev& L, int64_t row, int k) {
    if (L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1) return row * L.K + k;
    const int per_img = L.oh * L.ow;
    const int64_t b = row / per_img;
    const int r = (int)(row - b * per_img);
    const int oy = r / L.ow, ox = r - oy * L.ow;
    const int run = L.kw * L.in_c;
    const int ky = k / run, kr = k - ky * run;
    return ((b * L.in_h + (int64_t)oy * L.stride + ky) * L.in_w + (int64_t)ox * L.stride) * L.in_c + kr;
}

// stage modes
constexpr int ST_BYTES = 0;   // generic byte gather (any shape; quantizes fp32 observations on the way)
constexpr int ST_VEC16 = 1;   // 16-byte gathers of 8-bit codes
constexpr int ST_F32X4 = 2;   // first FC layer on fp32 observations, K a multiple of 4: float4 -> 4 codes

// DEEP (single-tile waves only): 16 weight k-steps in flight per wave, requested before the
// activations are staged - for a long K at few rows, where few workgroups each walk a long weight
// stream and its latency, not bandwidth, sets the pace.  It costs registers, hence occupancy, so
// layers with many workgroups keep the shallow pipeline.
template <int W, int MT, int NB, bool ASYM, bool TAPS, bool DEEP>
__global__ __launch_bounds__(W * 64, (W <= 2 && !DEEP) ? 4 : 1) void k_layer_int8(const NetDev* __restrict__ netp, const TapArgs t, const int l,
                                                      const LayerIO io, const int64_t rows, const int stage_mode,
                                                      const int kc, const void* __restrict__ actions) {
    constexpr int ROWS = 32 * MT;
    constexpr int NT_ = W * 64;
    extern __shared__ __align__(16) int8_t xs[];
    const int LD = kc * 32 + 16;
    const NetDev& a = *netp;
    const LayerDev& L = a.L[l];
    LayerTaps T{nullptr, nullptr, nullptr};
    if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    const bool first = l == 0, last = l == a.n_layers - 1;
    const bool ln = !last && L.act == AQ_ACT_LN_TANH;
    const int grp = blockIdx.y * W + wave;
    const int ngroups = (L.NT + NB - 1) / NB;
    const bool active = grp < ngroups;
    float s0 = 1.0f;
    int z0 = 0;
    if (first) {
        s0 = a.actq[0].s;
        z0 = a.actq[0].z;
    }
    const QuantScale qs0 = make_quant_scale(s0);
    int z_out = 0;
    if (!last) z_out = a.actq[l + 1].z;
    const int lo = (!last && L.act == AQ_ACT_RELU) ? z_out : 0;
    const int zw_s = ASYM ? L.z_w[0] - 128 : 0;

    v16i acc[NB][MT];
    v16i rs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        rs[mt] = zero16();
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb][mt] = zero16();
    }
    gv4i_ptr wptr[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int nt = grp * NB + nb;
        nt = nt < L.NT ? nt : L.NT - 1;
        wptr[nb] = (gv4i_ptr)L.wp + (int64_t)nt * L.KS * 64 + lane;
    }

    static_assert(!DEEP || (NB == 1 && MT == 1), "deep weight pipeline: single-tile waves only");
    constexpr int PF = DEEP ? 16 : 4;
    v4i wreg[PF][NB];
    for (int ks0 = 0; ks0 < L.KS; ks0 += kc) {
        const int ks1 = ks0 + kc < L.KS ? ks0 + kc : L.KS;
        if (ks0) __syncthreads();
        if (DEEP && active) mma_prefetch<NB, PF>(wptr, ks0, ks1, wreg);
        // Staging loops keep SU independent loads in flight per thread: with one load per iteration the
        // block copy would run at one memory latency per 16 bytes per thread.
        constexpr int SU = 8;
        if (stage_mode == ST_VEC16) {
            // Every 16-byte piece of a row's K range is contiguous and aligned in the input.  A few threads
            // share a row (NT_ = 4 or 2 times ROWS), so the row's position in the
            // input (a 64-bit division for convolutions) is worked out once per thread, and each piece
            // costs one small division by the length of a kernel row, done in floating point (exact:
            // (k + 0.5) / run is never within 0.5 / run of an integer and k stays far below 2^21).
            constexpr int TPR = NT_ / ROWS;  // staging threads per row: 4, or 2 for the single-wave tile
            static_assert(TPR * ROWS == NT_ && (TPR == 4 || TPR == 2), "whole staging threads per row");
            const int chunks = (ks1 - ks0) * 2;
            const int m = tid / TPR, j = tid % TPR;
            const int64_t row = row0 + m;
            const bool row_ok = row < rows;
            const bool fc = L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1;
            int64_t base = 0;     // offset of the row's k = 0
            int run = L.K;        // contiguous K bytes per kernel row; the next kernel row is row_pitch further
            int64_t row_pitch = 0;
            if (row_ok) {
                if (fc) {
                    base = row * L.K;
                } else {
                    const int per_img = L.oh * L.ow;
                    const int64_t b = row / per_img;
                    const int r = (int)(row - b * per_img);
                    const int oy = r / L.ow, ox = r - oy * L.ow;
                    base = ((b * L.in_h + (int64_t)oy * L.stride) * L.in_w + (int64_t)ox * L.stride) * L.in_c;
                    run = L.kw * L.in_c;
                    row_pitch = (int64_t)L.in_w * L.in_c;
                }
            }
            const float inv_run = 1.0f / (float)run;
            for (int c0 = j; c0 < chunks; c0 += TPR * SU) {
                v4i v[SU];
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int c = c0 + TPR * u;
                    v[u][0] = v[u][1] = v[u][2] = v[u][3] = 0;
                    const int k = ks0 * 32 + c * 16;
                    if (c < chunks && row_ok && k < L.K) {
                        const int ky = fc ? 0 : (int)(((float)k + 0.5f) * inv_run);
                        const int kr = k - ky * run;
                        v[u] = *(const v4i*)((const int8_t*)io.in + base + ky * row_pitch + kr);
                        if (first) {  // raw unsigned codes -> signed domain
                            v[u][0] ^= 0x80808080;
                            v[u][1] ^= 0x80808080;
                            v[u][2] ^= 0x80808080;
                            v[u][3] ^= 0x80808080;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int c = c0 + TPR * u;
                    if (c < chunks) *(v4i*)(xs + m * LD + c * 16) = v[u];
                }
            }
        } else if (stage_mode == ST_F32X4) {
            const int K4 = L.K >> 2;
            const int q0 = ks0 * 8, q1 = ks1 * 8;  // quads of this chunk (zero beyond K4)
            const int nq = q1 - q0;
            const int total = ROWS * nq;
            for (int base = tid; base < total; base += NT_ * SU) {
                float4 v[SU];
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int idx = base + u * NT_;
                    v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (idx < total) {
                        const int m = idx / nq, q = q0 + (idx - m * nq);
                        if (row0 + m < rows && q < K4) v[u] = ((const float4*)io.in)[(row0 + m) * K4 + q];
                    }
                }
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int idx = base + u * NT_;
                    if (idx < total) {
                        const int m = idx / nq, q = q0 + (idx - m * nq);
                        const int64_t row = row0 + m;
                        uint32_t pack = 0;
                        if (row < rows && q < K4) {
                            pack = quant_code4(v[u], qs0, -z0, 255 - z0, z0);
                            if (TAPS) {
                                if (t.a0 && blockIdx.y == 0) *(uint32_t*)(t.a0 + row * L.K + 4 * q) = pack;
                            }
                            pack ^= 0x80808080u;
                        }
                        *(uint32_t*)(xs + m * LD + (q - q0) * 4) = pack;
                    }
                }
            }
        } else {
            const int kb = (ks1 - ks0) * 32;
            for (int idx = tid; idx < ROWS * kb; idx += NT_) {
                const int m = idx / kb, kk = idx - m * kb;
                const int k = ks0 * 32 + kk;
                const int64_t row = row0 + m;
                int sv = 0;
                if (row < rows && k < L.K) {
                    const int64_t off = gather_offset(L, row, k);
                    if (first) {
                        int code;
                        if (a.in_u8) code = ((const uint8_t*)io.in)[off];
                        else code = quant_code(((const float*)io.in)[off], qs0, -z0, 255 - z0) + z0;
                        if (TAPS) {
                            if (t.a0 && blockIdx.y == 0) t.a0[off] = (uint8_t)code;
                        }
                        sv = code - 128;
                    } else {
                        sv = ((const int8_t*)io.in)[off];
                    }
                }
                xs[m * LD + kk] = (int8_t)sv;
            }
        }
        __syncthreads();
        if (active) {
            if (!DEEP) mma_prefetch<NB, PF>(wptr, ks0, ks1, wreg);
            mma_run<MT, NB, ASYM, PF>(wptr, wreg, xs, LD, ks0, ks1, ks0, acc, rs, lane);
        }
    }

    const CPtrs C = global_consts(L);
    const bool fast = !last && !ln && a.fast[l] != 0;
    const int head = a.head;
    // Results leave through LDS so that global stores are whole 16-byte pieces of an output row: a lane
    // owns 4 consecutive features of ONE row, and 64 such 4-byte stores per instruction would each touch
    // a different cache line.  The activation block is no longer needed once every wave has left the
    // MFMA loop, so its LDS is reused: [ROWS][BNP + 16] bytes (hidden) or [ROWS][BNP + 4] floats (last).
    constexpr int BNP = W * NB * 32;                 // features per workgroup pass
    const int n_base = blockIdx.y * BNP;
    const bool via_lds = !ln && (last || (L.N & 15) == 0);
    if (!via_lds) {
        if (!active) return;
        const int64_t row_first = row0 + (lane & 31);
        if (ln) {
            // dequantized accumulators go to the LayerNorm kernel
            static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                constexpr int nb = decltype(nb_c)::value;
                const int nt = grp * NB + nb;
                if (nt < L.NT) {
                    static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                        constexpr int mt = decltype(mt_c)::value;
                        const int64_t row = row_first + mt * 32;
                        const bool row_ok = row < rows;
                        epi_last_tile<ASYM, TAPS>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok,
                                                  row_ok ? io.ln_x + row * L.N : nullptr, L.N, nullptr, 0);
                    });
                }
            });
        } else if (fast) {
            epi_hidden_wave<MT, NB, ASYM, TAPS, true>(L.N, L.NT, T, C, acc, rs, zw_s, grp, g, row_first, rows, true, z_out,
                                                      lo, io.out + row_first * L.N, (int64_t)32 * L.N, false, L.N);
        } else {
            epi_hidden_wave<MT, NB, ASYM, TAPS, false>(L.N, L.NT, T, C, acc, rs, zw_s, grp, g, row_first, rows, true, z_out,
                                                       lo, io.out + row_first * L.N, (int64_t)32 * L.N, false, L.N);
        }
        return;
    }
    __syncthreads();  // every wave is done reading the activation block
    if (last) {
        constexpr int LDY = BNP + 4;
        float* ys = (float*)xs;
        if (active) {
            static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                constexpr int nb = decltype(nb_c)::value;
                const int nt = grp * NB + nb;
                if (nt < L.NT) {
                    static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                        constexpr int mt = decltype(mt_c)::value;
                        const int m = mt * 32 + (lane & 31);
                        const int64_t row = row0 + m;
                        epi_last_tile<ASYM, TAPS>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row < rows,
                                                  ys + m * LDY - n_base, n_base + BNP, nullptr, 0);
                    });
                }
            });
        }
        __syncthreads();
        // y tap, elementwise head (tanh / identity) and coalesced stores; argmax is a separate row kernel
        const int nvalid = L.N - n_base < BNP ? L.N - n_base : BNP;
        for (int idx = tid; idx < ROWS * nvalid; idx += NT_) {
            const int m = idx / nvalid, n = idx - m * nvalid;
            const int64_t row = row0 + m;
            if (row >= rows) continue;
            const float y = ys[m * LDY + n];
            if (io.y) io.y[row * L.N + n_base + n] = y;
            if (actions) ((float*)actions)[row * L.N + n_base + n] = head == AQ_HEAD_TANH ? tanh_head(y) : y;
        }
    } else {
        constexpr int LDO = BNP + 16;
        if (active) {
            const int m0 = lane & 31;
            if (fast)
                epi_hidden_wave<MT, NB, ASYM, TAPS, true>(L.N, L.NT, T, C, acc, rs, zw_s, grp, g, row0 + m0, rows, false,
                                                          z_out, lo, xs + m0 * LDO - n_base, 32 * LDO, true, n_base + BNP);
            else
                epi_hidden_wave<MT, NB, ASYM, TAPS, false>(L.N, L.NT, T, C, acc, rs, zw_s, grp, g, row0 + m0, rows, false,
                                                           z_out, lo, xs + m0 * LDO - n_base, 32 * LDO, true, n_base + BNP);
        }
        __syncthreads();
        const int nvalid = L.N - n_base < BNP ? L.N - n_base : BNP;  // a multiple of 16
        const int chunks = nvalid >> 4;
        for (int idx = tid; idx < ROWS * chunks; idx += NT_) {
            const int m = idx / chunks, c = idx - m * chunks;
            const int64_t row = row0 + m;
            if (row < rows) *(v4i*)(io.out + row * L.N + n_base + c * 16) = *(const v4i*)(xs + m * LDO + c * 16);
        }
    }
}

// LayerNorm + tanh + re-quantize of fp32 rows (per-layer path): one wavefront per row.
__global__ __launch_bounds__(256) void k_ln_tanh_rows(const float* __restrict__ x, int64_t rows, int N,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      float eps, const ActQ* __restrict__ actq, int out_idx,
                                                      int8_t* __restrict__ out, float* __restrict__ tap_ln,
                                                      uint8_t* __restrict__ tap_act) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float s_out = actq[out_idx].s;
    const int z_out = actq[out_idx].z;
    const QuantScale qs_out = make_quant_scale(s_out);
    const float* xr = x + row * N;
    float s = 0.0f;
    for (int n = lane; n < N; n += 64) s += xr[n];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    const float mean = s / (float)N;
    float ss = 0.0f;
    for (int n = lane; n < N; n += 64) {
        float d = xr[n] - mean;
        ss += d * d;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    const float inv = 1.0f / sqrtf(ss / (float)N + eps);
    for (int n = lane; n < N; n += 64) {
        float y = (xr[n] - mean) * inv * gamma[n] + beta[n];
        float tv = tanh_fast(y);
        if (tap_ln) tap_ln[row * N + n] = tv;
        int code = quant_code(tv, qs_out, -z_out, 255 - z_out) + z_out;
        if (tap_act) tap_act[row * N + n] = (uint8_t)code;
        out[row * N + n] = (int8_t)(code - 128);
    }
}

// argmax head on the dequantized last-layer rows (per-layer path; lowest index wins ties)
__global__ void k_head_rows(const float* __restrict__ y, int64_t rows, int N, int head, void* __restrict__ actions) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (head == AQ_HEAD_ARGMAX) {
        if (i >= rows) return;
        const float* yr = y + i * N;
        int best = 0;
        for (int n = 1; n < N; ++n)
            if (yr[n] > yr[best]) best = n;
        ((int32_t*)actions)[i] = best;
    } else {
        if (i >= rows * N) return;
        ((float*)actions)[i] = head == AQ_HEAD_TANH ? tanh_head(y[i]) : y[i];
    }
}

namespace {
// Tile configuration of one layer launch.
struct LayerPlan {
    int w, mt, nb;
    bool deep;
};

LayerPlan plan_layer(const LayerDev& L, int64_t rows, bool asym) {
    // Wide layers with many rows: 128-row blocks, 64 features per wave, 8 waves (512 features per
    // workgroup pass).  Narrow layers: 32-row blocks and as many waves as there are feature tiles,
    // so that every SIMD of the chip gets work.  Everything else: 64-row blocks, 4 waves.
    if (!asym && rows >= 8192 && L.NT >= 16) return {8, 4, 2, false};  // (the asymmetric row-sum tiles would spill)
    // one feature tile and a short K: a second wave would only help staging, and idle afterwards
    if (rows >= 8192 && L.NT == 1 && L.KS <= 16) return {1, 1, 1, false};
    if (rows >= 8192 && L.NT <= 2) return {2, 1, 1, false};
    // few rows: the 64-row configuration would leave most CUs without a workgroup; take the smallest
    // tile, and with a long K the deep weight pipeline
    const int64_t wg_mid = ((rows + 63) / 64) * (((L.NT + 1) / 2 + 3) / 4);
    if (wg_mid < 128) return {2, 1, 1, L.KS >= 32};
    return {4, 2, 2, false};
}
}  // namespace

template <int W, int MT, int NB, bool DEEP = false>
static aq_status launch_layer_t(const FwdArgs& a, int l, const LayerIO& io, int64_t rows, int stage_mode,
                                const void* actions, hipStream_t st) {
    const LayerDev& L = a.net.L[l];
    constexpr int ROWS = 32 * MT;
    // stage as much of K as fits comfortably in LDS (whole K for K <= 2048 at 64 rows, 1024 at 128 rows)
    int kc = L.KS;
    const int kc_max = (144 * 1024 / ROWS - 16) / 32;
    if (kc > kc_max) kc = kc_max;
    if (kc < 1) kc = 1;
    size_t lds = (size_t)ROWS * (kc * 32 + 16);
    const size_t lds_out = (size_t)ROWS * (W * NB * 32 + 16) * (l == a.net.n_layers - 1 ? 4 : 1);
    if (lds_out > lds) lds = lds_out;
    const int ngroups = (L.NT + NB - 1) / NB;
    dim3 grid((unsigned)((rows + ROWS - 1) / ROWS), (unsigned)((ngroups + W - 1) / W));
    const bool taps = any_taps(a);
    const bool asym = a.net.asym != 0;
#define AQ_LAYER(AS, TP)                                                                                            \
    do {                                                                                                            \
        static std::atomic<bool> attr_set{false};                                                                          \
        if (!attr_set) {                                                                                            \
            if (hipFuncSetAttribute((const void*)k_layer_int8<W, MT, NB, AS, TP, DEEP>,                                   \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)          \
                return AQ_EHIP;                                                                                     \
            attr_set = true;                                                                                        \
        }                                                                                                           \
        hipLaunchKernelGGL((k_layer_int8<W, MT, NB, AS, TP, DEEP>), grid, dim3(W * 64), lds, st, a.d_net, a.t, l, io, rows, \
                           stage_mode, kc, actions);                                                                \
    } while (0)
    if (asym) {
        if (taps) AQ_LAYER(true, true);
        else AQ_LAYER(true, false);
    } else {
        if (taps) AQ_LAYER(false, true);
        else AQ_LAYER(false, false);
    }
#undef AQ_LAYER
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

bool layer_uses_skinny(const FwdArgs& a, int l) {
    const LayerDev& L = a.net.L[l];
    const int64_t rows = a.c.batch * L.oh * L.ow;
    const LayerPlan p = plan_layer(L, rows, a.net.asym != 0);
    return p.w == 2 && rows < 8192 && skinny_layer_supported(L, rows);
}

aq_status launch_layer_int8(const FwdArgs& a, int l, const LayerIO& io, hipStream_t st) {
    const LayerDev& L = a.net.L[l];
    const int64_t rows = a.c.batch * L.oh * L.ow;
    const bool first = l == 0, last = l == a.net.n_layers - 1;
    const bool fc = L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1;
    // 16-byte gathers need contiguous, aligned 16-byte pieces of K in an 8-bit input
    const int run = fc ? L.K : L.kw * L.in_c;
    int stage_mode = ST_BYTES;
    // (a caller's observation buffer may sit at any address; the library's own buffers are aligned)
    const bool aligned = ((uintptr_t)io.in & 15) == 0;
    if (aligned && run % 16 == 0 && !(first && !a.net.in_u8) && !(first && a.t.a0) &&
        (fc || ((L.stride * L.in_c) % 16 == 0 && (L.in_w * L.in_c) % 16 == 0)))
        stage_mode = ST_VEC16;
    else if (aligned && first && !a.net.in_u8 && fc && (L.K & 3) == 0)
        stage_mode = ST_F32X4;
    // elementwise heads are applied in the last layer's epilogue; argmax needs the whole row
    const void* actions = (last && a.net.head != AQ_HEAD_ARGMAX) ? a.c.actions : nullptr;
    const LayerPlan p = plan_layer(L, rows, a.net.asym != 0);
    // few workgroups and a fully connected layer: the K-split kernel makes one weight stream per wave
    if (layer_uses_skinny(a, l)) return launch_layer_skinny(a, l, io, st);
    if (p.w == 8) return launch_layer_t<8, 4, 2>(a, l, io, rows, stage_mode, actions, st);
    if (p.w == 1) return launch_layer_t<1, 1, 1>(a, l, io, rows, stage_mode, actions, st);
    if (p.w == 2 && p.deep) return launch_layer_t<2, 1, 1, true>(a, l, io, rows, stage_mode, actions, st);
    if (p.w == 2) return launch_layer_t<2, 1, 1>(a, l, io, rows, stage_mode, actions, st);
    return launch_layer_t<4, 2, 2>(a, l, io, rows, stage_mode, actions, st);
}

aq_status launch_ln_tanh_rows(const FwdArgs& a, int l, const float* x, int8_t* out, int64_t rows, hipStream_t st) {
    const LayerDev& L = a.net.L[l];
    hipLaunchKernelGGL(k_ln_tanh_rows, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, x, rows, L.N, L.gamma,
                       L.beta, a.net.ln_eps, a.d_net->actq, l + 1, out, a.t.ln[l], a.t.act[l]);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_head_rows(const float* y, int64_t rows, int N, int head, void* actions, hipStream_t st) {
    const int64_t n = head == AQ_HEAD_ARGMAX ? rows : rows * N;
    hipLaunchKernelGGL(k_head_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, y, rows, N, head, actions);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
