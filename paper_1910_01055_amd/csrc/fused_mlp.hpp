// Whole-network fused int8 MLP (Sec. 3.1 actor inference, quantized per Sec. 3.2): one workgroup
// of 8 wavefronts owns ROWS = 32 * MT batch rows from the observation to the action.
//   - activations never leave LDS (two ping-pong row-major int8 buffers, signed domain)
//   - weights stream from L2 straight into MFMA operand registers (pre-packed at quantize time)
//   - each wave owns NB feature tiles per pass; per-channel constants of the layer are fetched
//     while the MFMAs run and handed to the epilogue through LDS
//   - epilogues: requantize(+ReLU) / LayerNorm+tanh+requantize in registers, last layer dequantize,
//     then a coalesced head pass (tanh / identity / argmax)
#pragma once
#include "int8_device.hpp"

namespace aq {

constexpr int FW = 8;            // wavefronts per workgroup
constexpr int FT = FW * 64;      // threads per workgroup
constexpr int CST_MAXN = 1024;   // widest layer whose constants fit the LDS staging area

// LDS layout (bytes): [buf_in ROWS*ld][buf_out ROWS*ld][red 2*FW*ROWS floats][cst 6*cst_n words]
__host__ __device__ inline size_t fused_lds_bytes(int rows, int ld, int cst_n) {
    return (size_t)2 * rows * ld + (size_t)2 * FW * rows * 4 + (size_t)6 * cst_n * 4;
}

template <int MT, int NB, bool ASYM, bool TAPS>
__device__ __forceinline__ void fused_layer(const NetDev& a, const CallArgs& c, const TapArgs& t, int l,
                                            const int8_t* in, int8_t* out, float* red, int32_t* cst, int cst_n,
                                            int64_t row0) {
    constexpr int ROWS = 32 * MT;
    constexpr int PF = NB == 1 ? 8 : 4;
    const LayerDev& L = a.L[l];
    LayerTaps T{nullptr, nullptr, nullptr};
    if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
    const bool last = l == a.n_layers - 1;
    const bool ln = !last && L.act == AQ_ACT_LN_TANH;
    const int ngroups = (L.NT + NB - 1) / NB;
    const int Np = L.NT * 32;
    float s_out = 1.0f;
    int z_out = 0;
    if (!last) {
        s_out = a.actq[l + 1].s;
        z_out = a.actq[l + 1].z;
    }
    const int lo = (!last && L.act == AQ_ACT_RELU) ? z_out : 0;
    const int zw_s = ASYM ? L.z_w[0] - 128 : 0;
    const int ld = c.ld;
    const int ldy = Np;  // last layer: fp32 row stride of y in LDS

    // Per-channel constants: issue the global loads now, park them in LDS after the MFMA loop.
    // Six arrays of Np words: bias_fold, M0, rshift, m, gamma, beta (as 16-byte pieces).
    const int n4 = Np / 4;
    auto csrc = [&](int w) __attribute__((always_inline)) -> const int4* {
        return (const int4*)(w == 0 ? (const void*)L.bias_fold : w == 1 ? (const void*)L.M0 : w == 2 ? (const void*)L.rshift
                             : w == 3 ? (const void*)L.m : w == 4 ? (const void*)L.gamma : (const void*)L.beta);
    };
    int4 cv[3];
    const int pieces = (ln ? 6 : 4) * n4;  // <= 6 * 256 = 3 * FT for Np <= CST_MAXN
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int idx = tid + r * FT;
        if (idx < pieces) cv[r] = csrc(idx / n4)[idx % n4];
    }

    CPtrs C;
    C.bias_fold = cst;
    C.M0 = cst + cst_n;
    C.rshift = cst + 2 * cst_n;
    C.m = (const float*)(cst + 3 * cst_n);
    const float* c_gamma = (const float*)(cst + 4 * cst_n);
    const float* c_beta = (const float*)(cst + 5 * cst_n);

    for (int g0 = 0; g0 < ngroups; g0 += FW) {
        const int grp = g0 + wave;
        const bool active = grp < ngroups;
        v16i acc[NB][MT];
        v16i rs[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            rs[mt] = zero16();
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[nb][mt] = zero16();
        }
        if (active) {
            const v4i* wptr[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                int nt = grp * NB + nb;
                nt = nt < L.NT ? nt : L.NT - 1;
                wptr[nb] = (const v4i*)L.wp + (int64_t)nt * L.KS * 64 + lane;
            }
            mma_block<MT, NB, ASYM, PF>(wptr, in, ld, 0, L.KS, 0, acc, rs, lane);
        }
        if (g0 == 0) {
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int idx = tid + r * FT;
                if (idx < pieces) *(int4*)(cst + (idx / n4) * cst_n + (idx % n4) * 4) = cv[r];
            }
            __syncthreads();
        }
        if (!ln) {
            if (active) {
                static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                    constexpr int nb = decltype(nb_c)::value;
                    const int nt = grp * NB + nb;
                    if (nt < L.NT) {
                        static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                            constexpr int mt = decltype(mt_c)::value;
                            const int m = mt * 32 + (lane & 31);
                            const int64_t row = row0 + m;
                            const bool row_ok = row < c.batch;
                            if (last)
                                epi_last_tile<ASYM, TAPS>(L, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok,
                                                          (float*)out + m * ldy, ldy);
                            else
                                epi_hidden_tile<ASYM, TAPS>(L, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok,
                                                            z_out, lo, out + m * ld, true, Np);
                        });
                    }
                });
            }
        } else {
            // LayerNorm over the layer's N features (all resident in this one pass: ngroups <= FW),
            // tanh, re-quantize.  Row statistics: in-lane sums, lane ^ 32, then across waves via LDS.
            float* red1 = red;
            float* red2 = red + FW * ROWS;
            float mean[MT], inv[MT];
            static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                constexpr int mt = decltype(mt_c)::value;
                float s = 0.0f;
                const int64_t row = row0 + mt * 32 + (lane & 31);
                const bool row_ok = row < c.batch;
                static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                    constexpr int nb = decltype(nb_c)::value;
                    const int nt = grp * NB + nb;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int n0 = nt * 32 + 8 * j + 4 * g;
                        if (active && n0 < Np) {
                            int val[4];
                            quad_acc<ASYM, TAPS>(L, T, C, acc[nb][mt], j, n0, rs[mt][0], zw_s, row, row_ok, val);
                            const float4 mm = *(const float4*)(C.m + n0);
                            const float mv[4] = {mm.x, mm.y, mm.z, mm.w};
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                float x = n0 + i < L.N ? (float)val[i] * mv[i] : 0.0f;
                                acc[nb][mt][4 * j + i] = __float_as_int(x);
                                s += x;
                            }
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i) acc[nb][mt][4 * j + i] = 0;
                        }
                    }
                });
                s += __shfl_xor(s, 32, 64);
                if (g == 0) red1[wave * ROWS + mt * 32 + lane] = s;
            });
            __syncthreads();
            static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                constexpr int mt = decltype(mt_c)::value;
                const int m = mt * 32 + (lane & 31);
                float tot = 0.0f;
#pragma unroll
                for (int w = 0; w < FW; ++w) tot += red1[w * ROWS + m];
                mean[mt] = tot / (float)L.N;
                float ss = 0.0f;
                static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                    constexpr int nb = decltype(nb_c)::value;
                    const int nt = grp * NB + nb;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int n = nt * 32 + 8 * j + 4 * g + i;
                            if (active && n < L.N) {
                                float d = __int_as_float(acc[nb][mt][4 * j + i]) - mean[mt];
                                ss += d * d;
                            }
                        }
                });
                ss += __shfl_xor(ss, 32, 64);
                if (g == 0) red2[wave * ROWS + mt * 32 + lane] = ss;
            });
            __syncthreads();
            static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                constexpr int mt = decltype(mt_c)::value;
                const int m = mt * 32 + (lane & 31);
                float tot = 0.0f;
#pragma unroll
                for (int w = 0; w < FW; ++w) tot += red2[w * ROWS + m];
                inv[mt] = 1.0f / sqrtf(tot / (float)L.N + a.ln_eps);
                const int64_t row = row0 + m;
                const bool row_ok = row < c.batch;
                static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                    constexpr int nb = decltype(nb_c)::value;
                    const int nt = grp * NB + nb;
                    if (active && nt < L.NT) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int n0 = nt * 32 + 8 * j + 4 * g;
                            const float4 ga = *(const float4*)(c_gamma + n0);
                            const float4 be = *(const float4*)(c_beta + n0);
                            const float gv[4] = {ga.x, ga.y, ga.z, ga.w}, bv[4] = {be.x, be.y, be.z, be.w};
                            uint32_t pack = 0;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int n = n0 + i;
                                float x = __int_as_float(acc[nb][mt][4 * j + i]);
                                float y = (x - mean[mt]) * inv[mt] * gv[i] + bv[i];
                                float tv = tanh_fast(y);
                                int code = rint_clamp(tv / s_out, -z_out, 255 - z_out) + z_out;
                                if (n >= L.N) code = 128;
                                if (TAPS) {
                                    if (row_ok && n < L.N) {
                                        if (T.ln) T.ln[row * L.N + n] = tv;
                                        if (T.act) T.act[row * L.N + n] = (uint8_t)code;
                                    }
                                }
                                pack |= (uint32_t)((code ^ 0x80) & 255) << (8 * i);
                            }
                            *(uint32_t*)(out + m * ld + n0) = pack;
                        }
                    }
                });
            });
        }
    }
}

template <int MT, int NB, bool ASYM, bool TAPS>
__global__ __launch_bounds__(FT) void k_mlp_fused(const NetDev* __restrict__ netp, const CallArgs c,
                                                  const TapArgs t) {
    const NetDev& a = *netp;
    extern __shared__ __align__(16) int8_t smem[];
    constexpr int ROWS = 32 * MT;
    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    const int ld = c.ld;
    int8_t* buf_in = smem;
    int8_t* buf_out = smem + ROWS * ld;
    float* red = (float*)(smem + 2 * ROWS * ld);
    int32_t* cst = (int32_t*)(red + 2 * FW * ROWS);

    // observation quantize: a0 = clamp(round(x / s0) + z0, 0, 255), kept in the signed domain
    {
        const int K0 = a.L[0].K, Kp = a.L[0].KS * 32;
        const float s0 = a.actq[0].s;
        const int z0 = a.actq[0].z;
        if (!a.in_u8 && (K0 & 3) == 0) {
            // four observations per lane: one 16-byte load, one packed 32-bit LDS store
            const int K4 = K0 >> 2;
            const float4* src = (const float4*)c.obs + row0 * K4;
            for (int idx = tid; idx < ROWS * K4; idx += FT) {
                const int m = idx / K4, k4 = idx - m * K4;
                uint32_t pack = 0;
                if (row0 + m < c.batch) {
                    const float4 v = src[idx];
                    const int c0 = rint_clamp(v.x / s0, -z0, 255 - z0) + z0, c1 = rint_clamp(v.y / s0, -z0, 255 - z0) + z0;
                    const int c2 = rint_clamp(v.z / s0, -z0, 255 - z0) + z0, c3 = rint_clamp(v.w / s0, -z0, 255 - z0) + z0;
                    pack = (uint32_t)c0 | ((uint32_t)c1 << 8) | ((uint32_t)c2 << 16) | ((uint32_t)c3 << 24);
                    if (TAPS) {
                        if (t.a0) *(uint32_t*)(t.a0 + (row0 + m) * K0 + 4 * k4) = pack;
                    }
                    pack ^= 0x80808080u;
                }
                *(uint32_t*)(buf_in + m * ld + 4 * k4) = pack;
            }
        } else {
            for (int idx = tid; idx < ROWS * K0; idx += FT) {
                const int m = idx / K0, k = idx - m * K0;
                const int64_t row = row0 + m;
                int code = 128;
                if (row < c.batch) {
                    if (a.in_u8) {
                        code = ((const uint8_t*)c.obs)[row * K0 + k];
                    } else {
                        code = rint_clamp(((const float*)c.obs)[row * K0 + k] / s0, -z0, 255 - z0) + z0;
                    }
                    if (TAPS) {
                        if (t.a0) t.a0[row * K0 + k] = (uint8_t)code;
                    }
                }
                buf_in[m * ld + k] = (int8_t)(code - 128);
            }
        }
        const int padw = Kp - K0;
        for (int idx = tid; idx < ROWS * padw; idx += FT) {
            const int m = idx / padw, k = K0 + (idx - m * padw);
            buf_in[m * ld + k] = 0;
        }
    }
    __syncthreads();

    for (int l = 0; l < a.n_layers; ++l) {
        fused_layer<MT, NB, ASYM, TAPS>(a, c, t, l, buf_in, buf_out, red, cst, c.cst_n, row0);
        __syncthreads();
        int8_t* sw = buf_in;
        buf_in = buf_out;
        buf_out = sw;
    }

    // action head on the dequantized last-layer rows y (fp32, in LDS): tanh / identity / argmax
    {
        const LayerDev& L = a.L[a.n_layers - 1];
        const float* ybuf = (const float*)buf_in;
        const int ldy = L.NT * 32;
        const int N = L.N;
        if (a.head == AQ_HEAD_ARGMAX) {
            for (int m = tid; m < ROWS; m += FT) {
                const int64_t row = row0 + m;
                if (row >= c.batch) continue;
                int best = 0;
                for (int n = 0; n < N; ++n) {
                    const float y = ybuf[m * ldy + n];
                    if (TAPS) {
                        if (t.y) t.y[row * N + n] = y;
                    }
                    if (y > ybuf[m * ldy + best]) best = n;
                }
                ((int32_t*)c.actions)[row] = best;
            }
        } else {
            for (int idx = tid; idx < ROWS * N; idx += FT) {
                const int m = idx / N, n = idx - m * N;
                const int64_t row = row0 + m;
                if (row >= c.batch) continue;
                const float y = ybuf[m * ldy + n];
                if (TAPS) {
                    if (t.y) t.y[row * N + n] = y;
                }
                ((float*)c.actions)[row * N + n] = a.head == AQ_HEAD_TANH ? tanh_head(y) : y;
            }
        }
    }
}

template <int MT, int NB, bool ASYM, bool TAPS>
aq_status launch_fused_t(const FwdArgs& a, size_t lds, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_mlp_fused<MT, NB, ASYM, TAPS>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return AQ_EHIP;
        attr_set = true;
    }
    const int rows = 32 * MT;
    const unsigned grid = (unsigned)((a.c.batch + rows - 1) / rows);
    hipLaunchKernelGGL((k_mlp_fused<MT, NB, ASYM, TAPS>), dim3(grid), dim3(FT), lds, st, a.d_net, a.c, a.t);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

// one explicit instantiation per translation unit, so the variants compile in parallel
#define AQ_FUSED_DECL(MT, NB, AS, TP) \
    extern template aq_status launch_fused_t<MT, NB, AS, TP>(const FwdArgs&, size_t, hipStream_t)
#define AQ_FUSED_INST(MT, NB, AS, TP) \
    template aq_status launch_fused_t<MT, NB, AS, TP>(const FwdArgs&, size_t, hipStream_t)

}  // namespace aq
