// Actor inference on the 8-bit policy (Sec. 3.1; quantized weights and activations, Sec. 3.2).
//
// Arithmetic: activations are unsigned 8-bit codes a_u with zero-point z_a, weights 8-bit codes.
// The int8 MFMA is signed x signed, so both operands live in the signed domain (a_s = a_u - 128,
// unsigned weight codes likewise); the zero-point terms of
//   sum_k (a_u - z_a)(w_u - z_w) = sum_k a_s w_s - z_a' sum_k w_s - z_w' sum_k a_s + K z_a' z_w'
// are folded into a per-channel integer bias at quantize time, except "- z_w' sum_k a_s", which is
// applied here (per-tensor asymmetric weights only; the row sums come from one extra MFMA against
// an all-ones operand).  The canonical accumulator that leaves the MFMA + bias is therefore the
// exact integer sum_k (a_u - z_a)(w_u - z_w) + bias_q.
//
// MFMA mapping: v_mfma_i32_32x32x32_i8 computes D[32x32] += A[32x32] * B[32x32].  Weights are
// the A operand (rows = output features), batch rows are the B operand (columns), so that one
// lane owns one batch row and four consecutive output features per register quad: the requantized
// bytes of a quad pack into one 32-bit word of the next layer's row-major activation row.
//   A lane l: row  n = l % 32, bytes k = 16 * (l / 32) .. +15 of the 32-byte k-step
//   B lane l: col  m = l % 32, same bytes
//   D reg 4j+i of lane l: row n = 8 j + 4 (l / 32) + i, col m = l % 32
#include <type_traits>

#include "kernels.hpp"

namespace aq {

constexpr int PF = 4;  // weight k-steps in flight per wave (global -> register prefetch depth)

// compile-time loop: accumulator tiles are register arrays and must only ever be indexed by constants
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__device__ __forceinline__ v16i zero16() {
    v16i z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0;
    return z;
}

// tanh for hidden activations that are re-quantized to 8 bits right away: 1 - 2 / (e^{2|x|} + 1)
// on the hardware exp2 / rcp units; absolute error about 2e-7.
__device__ __forceinline__ float tanh_fast(float x) {
    float ax = fabsf(x);
    float e = __builtin_amdgcn_exp2f(fminf(ax, 20.0f) * 2.885390081777927f);  // e^{2|x|}
    float t = 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
    return copysignf(t, x);
}

// tanh for the action head: odd polynomial near zero (no cancellation), exponential form elsewhere;
// relative error below 1e-6.
__device__ __forceinline__ float tanh_head(float x) {
    float ax = fabsf(x);
    if (ax < 0.5f) {
        float u = x * x;
        // Taylor series of tanh(x)/x in u = x^2 up to u^6 (remainder < 2e-7 relative at |x| = 0.5)
        float p = 0.0035921280f;        // 21844/6081075
        p = fmaf(p, u, -0.0088632355f);  // -1382/155925
        p = fmaf(p, u, 0.0218694885f);   // 62/2835
        p = fmaf(p, u, -0.0539682540f);  // -17/315
        p = fmaf(p, u, 0.1333333333f);   // 2/15
        p = fmaf(p, u, -0.3333333333f);  // -1/3
        return fmaf(x * u, p, x);
    }
    float e = expf(2.0f * fminf(ax, 20.0f));
    float t = 1.0f - 2.0f / (e + 1.0f);
    return copysignf(t, x);
}

// ---------------------------------------------------------------------------------------------
// MFMA core: accumulates NB feature tiles x MT row tiles over k-steps [ks_begin, ks_end).
// Weights stream global -> registers (already in operand order), activations come from LDS
// (row-major int8, row stride ld, column 0 = k-step ks_lds0).
// ---------------------------------------------------------------------------------------------
template <int MT, int NB, bool ASYM>
__device__ __forceinline__ void mma_block(const v4i* (&wptr)[NB], const int8_t* xs, int ld, int ks_begin,
                                          int ks_end, int ks_lds0, v16i (&acc)[NB][MT], v16i (&rs)[MT], int lane) {
    v4i wreg[PF][NB];
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (ks_begin + p < ks_end) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) wreg[p][nb] = wptr[nb][(int64_t)(ks_begin + p) * 64];
        }
    const int8_t* xrow = xs + (lane & 31) * ld + (lane >> 5) * 16;
    v4i ones;
    ones[0] = ones[1] = ones[2] = ones[3] = 0x01010101;
    for (int ks = ks_begin; ks < ks_end; ks += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int k = ks + p;
            if (k < ks_end) {
                v4i xf[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    xf[mt] = *(const v4i*)(xrow + mt * 32 * ld + (k - ks_lds0) * 32);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[nb][mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][nb], xf[mt], acc[nb][mt], 0, 0, 0);
                if (ASYM) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        rs[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, xf[mt], rs[mt], 0, 0, 0);
                }
                if (k + PF < ks_end) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) wreg[p][nb] = wptr[nb][(int64_t)(k + PF) * 64];
                }
            }
        }
    }
}

// requantize one accumulator: v = (acc * M0 + 2^(r-1)) >> r, code = clamp(v + z_out, lo, 255)
__device__ __forceinline__ int requant_code(int acc, int M0, int r, int z_out, int lo) {
    long long p = (long long)acc * (long long)M0 + ((1LL << r) >> 1);
    long long v = (p >> r) + z_out;
    v = v < lo ? lo : v;
    v = v > 255 ? 255 : v;
    return (int)v;
}

// Epilogue of one 32x32 accumulator tile of a hidden (requantized) or last layer.
//   out_row: destination of this lane's row in the next activation buffer (hidden layers), or NULL
//   packed_store: four codes per 32-bit store (row length a multiple of 4), for features < n_store
template <bool ASYM>
__device__ __forceinline__ void epilogue_tile(const LayerDev& L, const v16i& c, int rs0, int zw_s, int nt, int g,
                                              int64_t row, bool row_ok, bool last, int z_out, int lo,
                                              int8_t* out_row, bool packed_store, int n_store, float* y_row,
                                              float* act_row, int head) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n0 = nt * 32 + 8 * j + 4 * g;
        const int4 bf = *(const int4*)(L.bias_fold + n0);
        const int bfv[4] = {bf.x, bf.y, bf.z, bf.w};
        int val[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            val[i] = c[4 * j + i] + bfv[i];
            if (ASYM) val[i] -= zw_s * rs0;
            if (L.tap_acc && row_ok && n0 + i < L.N) L.tap_acc[row * L.N + n0 + i] = val[i];
        }
        if (!last) {
            const int4 M = *(const int4*)(L.M0 + n0);
            const int4 R = *(const int4*)(L.rshift + n0);
            const int Mv[4] = {M.x, M.y, M.z, M.w}, Rv[4] = {R.x, R.y, R.z, R.w};
            uint32_t pack = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int code = requant_code(val[i], Mv[i], Rv[i], z_out, lo);
                if (n0 + i >= L.N) code = 128;  // padding features are zero in the signed domain
                if (L.tap_act && row_ok && n0 + i < L.N) L.tap_act[row * L.N + n0 + i] = (uint8_t)code;
                pack |= (uint32_t)((code ^ 0x80) & 255) << (8 * i);
            }
            if (out_row) {
                if (packed_store) {
                    if (n0 < n_store) *(uint32_t*)(out_row + n0) = pack;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n0 + i < L.N) out_row[n0 + i] = (int8_t)(pack >> (8 * i));
                }
            }
        } else {
            const float4 mm = *(const float4*)(L.m + n0);
            const float mv[4] = {mm.x, mm.y, mm.z, mm.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float y = (float)val[i] * mv[i];
                if (row_ok && n0 + i < L.N) {
                    if (y_row) y_row[n0 + i] = y;
                    if (act_row) act_row[n0 + i] = head == AQ_HEAD_TANH ? tanh_head(y) : y;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Whole-network fused MLP: one workgroup owns ROWS = 32 * MT batch rows from the observation
// to the action; activations never leave LDS, weights stream from L2 in operand order.
// ---------------------------------------------------------------------------------------------
template <int MT, int NB, bool ASYM>
__device__ __forceinline__ void fused_layer(const FwdArgs& a, int l, const int8_t* in, int8_t* out, float* red,
                                            int64_t row0) {
    constexpr int ROWS = 32 * MT;
    const LayerDev& L = a.L[l];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
    const bool last = l == a.n_layers - 1;
    const bool ln = !last && L.act == AQ_ACT_LN_TANH;
    const int ngroups = (L.NT + NB - 1) / NB;
    float s_out = 1.0f;
    int z_out = 0;
    if (!last) {
        s_out = a.actq[l + 1].s;
        z_out = a.actq[l + 1].z;
    }
    const int lo = (!last && L.act == AQ_ACT_RELU) ? z_out : 0;
    const int zw_s = ASYM ? L.z_w[0] - 128 : 0;
    const int ld = a.ld;

    for (int g0 = 0; g0 < ngroups; g0 += 4) {
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
            mma_block<MT, NB, ASYM>(wptr, in, ld, 0, L.KS, 0, acc, rs, lane);
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
                            const bool row_ok = row < a.batch;
                            float* y_row = (last && a.tap_y) ? a.tap_y + row * L.N : nullptr;
                            float* act_row = (last && a.head != AQ_HEAD_ARGMAX) ? (float*)a.actions + row * L.N : nullptr;
                            epilogue_tile<ASYM>(L, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok, last, z_out, lo,
                                                last ? nullptr : out + m * ld, true, L.NT * 32, y_row, act_row,
                                                a.head);
                        });
                    }
                });
                if (last && a.head == AQ_HEAD_ARGMAX) {
                    // single feature tile (checked on the host): each lane holds 16 of the 32 candidates of
                    // its row, the other 16 sit in lane ^ 32; lowest index wins ties
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        float best = -INFINITY;
                        int bi = 0x7fffffff;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int n = 8 * j + 4 * g + i;
                                if (n < L.N) {
                                    float y = (float)(acc[0][mt][4 * j + i] + L.bias_fold[n] -
                                                      (ASYM ? zw_s * rs[mt][0] : 0)) * L.m[n];
                                    if (y > best || (y == best && n < bi)) {
                                        best = y;
                                        bi = n;
                                    }
                                }
                            }
                        float ob = __shfl_xor(best, 32, 64);
                        int oi = __shfl_xor(bi, 32, 64);
                        if (ob > best || (ob == best && oi < bi)) bi = oi;
                        const int64_t row = row0 + mt * 32 + (lane & 31);
                        if (g == 0 && row < a.batch) ((int32_t*)a.actions)[row] = bi;
                    }
                }
            }
        } else {
            // LayerNorm over the layer's N features (all resident in this pass: ngroups <= 4), tanh,
            // re-quantize.  Row statistics: in-lane sums, lane ^ 32, then the four waves through LDS.
            float* red1 = red;
            float* red2 = red + 4 * ROWS;
            float mean[MT], inv[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float s = 0.0f;
                const int64_t row = row0 + mt * 32 + (lane & 31);
                const bool row_ok = row < a.batch;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int nt = grp * NB + nb;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int n = nt * 32 + 8 * j + 4 * g + i;
                            float x = 0.0f;
                            if (active && n < L.N) {
                                int val = acc[nb][mt][4 * j + i] + L.bias_fold[n];
                                if (ASYM) val -= zw_s * rs[mt][0];
                                if (L.tap_acc && row_ok) L.tap_acc[row * L.N + n] = val;
                                x = (float)val * L.m[n];
                            }
                            acc[nb][mt][4 * j + i] = __float_as_int(x);
                            s += x;
                        }
                }
                s += __shfl_xor(s, 32, 64);
                if (g == 0) red1[wave * ROWS + mt * 32 + lane] = s;
            }
            __syncthreads();
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = mt * 32 + (lane & 31);
                mean[mt] = (red1[m] + red1[ROWS + m] + red1[2 * ROWS + m] + red1[3 * ROWS + m]) / (float)L.N;
                float ss = 0.0f;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
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
                }
                ss += __shfl_xor(ss, 32, 64);
                if (g == 0) red2[wave * ROWS + mt * 32 + lane] = ss;
            }
            __syncthreads();
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = mt * 32 + (lane & 31);
                const float var = (red2[m] + red2[ROWS + m] + red2[2 * ROWS + m] + red2[3 * ROWS + m]) / (float)L.N;
                inv[mt] = 1.0f / sqrtf(var + a.ln_eps);
            }
            if (active) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int m = mt * 32 + (lane & 31);
                    const int64_t row = row0 + m;
                    const bool row_ok = row < a.batch;
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const int nt = grp * NB + nb;
                        if (nt < L.NT) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int n0 = nt * 32 + 8 * j + 4 * g;
                                uint32_t pack = 0;
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    const int n = n0 + i;
                                    int code = 128;
                                    if (n < L.N) {
                                        float x = __int_as_float(acc[nb][mt][4 * j + i]);
                                        float y = (x - mean[mt]) * inv[mt] * L.gamma[n] + L.beta[n];
                                        float t = tanh_fast(y);
                                        if (L.tap_ln && row_ok) L.tap_ln[row * L.N + n] = t;
                                        code = rint_clamp(t / s_out, -z_out, 255 - z_out) + z_out;
                                        if (L.tap_act && row_ok) L.tap_act[row * L.N + n] = (uint8_t)code;
                                    }
                                    pack |= (uint32_t)((code ^ 0x80) & 255) << (8 * i);
                                }
                                *(uint32_t*)(out + m * ld + n0) = pack;
                            }
                        }
                    }
                }
            }
        }
    }
}

// Feature tiles per wave and pass.  Narrow layers use fewer so that all four waves have work; a
// LayerNorm layer needs its whole row resident in one pass (at most 4 groups of NB tiles).
__host__ __device__ inline int pick_nb(int NT, int MT, bool ln) {
    const int nb_max = MT <= 2 ? 4 : 2;
    if (ln) {
        int nb = 1;
        while (nb < nb_max && (NT + nb - 1) / nb > 4) nb *= 2;
        return nb;
    }
    if (NT >= 16 && nb_max >= 4) return 4;
    return NT >= 8 ? 2 : 1;
}

template <int MT, bool ASYM>
__global__ __launch_bounds__(256) void k_mlp_fused(const FwdArgs a) {
    extern __shared__ __align__(16) int8_t smem[];
    constexpr int ROWS = 32 * MT;
    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    const int ld = a.ld;
    int8_t* buf_in = smem;
    int8_t* buf_out = smem + ROWS * ld;
    float* red = (float*)(smem + 2 * ROWS * ld);

    // observation quantize: a0 = clamp(round(x / s0) + z0, 0, 255), kept in the signed domain
    {
        const int K0 = a.L[0].K, Kp = a.L[0].KS * 32;
        const float s0 = a.actq[0].s;
        const int z0 = a.actq[0].z;
        for (int idx = tid; idx < ROWS * K0; idx += 256) {
            const int m = idx / K0, k = idx - m * K0;
            const int64_t row = row0 + m;
            int code = 128;
            if (row < a.batch) {
                if (a.in_u8) {
                    code = ((const uint8_t*)a.obs)[row * K0 + k];
                } else {
                    code = rint_clamp(((const float*)a.obs)[row * K0 + k] / s0, -z0, 255 - z0) + z0;
                }
                if (a.tap_a0) a.tap_a0[row * K0 + k] = (uint8_t)code;
            }
            buf_in[m * ld + k] = (int8_t)(code - 128);
        }
        const int padw = Kp - K0;
        for (int idx = tid; idx < ROWS * padw; idx += 256) {
            const int m = idx / padw, k = K0 + (idx - m * padw);
            buf_in[m * ld + k] = 0;
        }
    }
    __syncthreads();

    for (int l = 0; l < a.n_layers; ++l) {
        const bool ln = l < a.n_layers - 1 && a.L[l].act == AQ_ACT_LN_TANH;
        const int nb = pick_nb(a.L[l].NT, MT, ln);
        if (nb == 4) {
            if constexpr (MT <= 2) fused_layer<MT, 4, ASYM>(a, l, buf_in, buf_out, red, row0);
        } else if (nb == 2) {
            fused_layer<MT, 2, ASYM>(a, l, buf_in, buf_out, red, row0);
        } else {
            fused_layer<MT, 1, ASYM>(a, l, buf_in, buf_out, red, row0);
        }
        __syncthreads();
        int8_t* t = buf_in;
        buf_in = buf_out;
        buf_out = t;
    }
}


bool fused_mlp_supported(const FwdArgs& a, int* rows_out, size_t* lds_out) {
    int maxw = 0;
    for (int l = 0; l < a.n_layers; ++l) {
        const LayerDev& L = a.L[l];
        if (L.kh != 1 || L.kw != 1 || L.in_h != 1 || L.in_w != 1) return false;
        maxw = maxw > L.KS * 32 ? maxw : L.KS * 32;
        if (l < a.n_layers - 1) maxw = maxw > L.NT * 32 ? maxw : L.NT * 32;
    }
    if (a.head == AQ_HEAD_ARGMAX && a.L[a.n_layers - 1].NT != 1) return false;
    const int ld = maxw + 16;
    // rows per workgroup: enough workgroups to cover the 256 CUs, as many rows as LDS allows beyond that
    int mt = 1;
    if (a.batch >= 256 * 64) mt = 2;
    if (a.batch >= 512 * 128) mt = 4;
    for (; mt >= 1; mt >>= 1) {
        const int rows = 32 * mt;
        size_t lds = (size_t)2 * rows * ld + (size_t)8 * rows * sizeof(float);
        bool ok = lds <= 160 * 1024;
        for (int l = 0; l < a.n_layers - 1 && ok; ++l)
            if (a.L[l].act == AQ_ACT_LN_TANH) {
                int nb = pick_nb(a.L[l].NT, mt, true);
                if ((a.L[l].NT + nb - 1) / nb > 4) ok = false;  // LayerNorm needs the whole row in one pass
            }
        if (ok) {
            *rows_out = rows;
            *lds_out = lds;
            return true;
        }
    }
    return false;
}

template <int MT, bool ASYM>
static aq_status launch_fused_t(const FwdArgs& a, size_t lds, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_mlp_fused<MT, ASYM>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return AQ_EHIP;
        attr_set = true;
    }
    const int rows = 32 * MT;
    const unsigned grid = (unsigned)((a.batch + rows - 1) / rows);
    hipLaunchKernelGGL((k_mlp_fused<MT, ASYM>), dim3(grid), dim3(256), lds, st, a);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fused_mlp(const FwdArgs& a_in, hipStream_t st) {
    int rows;
    size_t lds;
    if (!fused_mlp_supported(a_in, &rows, &lds)) return AQ_ESHAPE;
    FwdArgs a = a_in;
    int maxw = 0;
    for (int l = 0; l < a.n_layers; ++l) {
        maxw = maxw > a.L[l].KS * 32 ? maxw : a.L[l].KS * 32;
        if (l < a.n_layers - 1) maxw = maxw > a.L[l].NT * 32 ? maxw : a.L[l].NT * 32;
    }
    a.ld = maxw + 16;
    const bool asym = a.asym != 0;
    switch (rows) {
        case 32: return asym ? launch_fused_t<1, true>(a, lds, st) : launch_fused_t<1, false>(a, lds, st);
        case 64: return asym ? launch_fused_t<2, true>(a, lds, st) : launch_fused_t<2, false>(a, lds, st);
        default: return asym ? launch_fused_t<4, true>(a, lds, st) : launch_fused_t<4, false>(a, lds, st);
    }
}

// ---------------------------------------------------------------------------------------------
// One layer per launch: FC or convolution as an implicit GEMM (rows = batch * oh * ow output
// positions, K = kh * kw * Cin gathered from the NHWC input).  A workgroup owns ROWS x (4*NB*32)
// outputs; the activation rows are staged in LDS KC k-steps at a time.
// ---------------------------------------------------------------------------------------------
constexpr int KC = 16;  // k-steps (of 32 bytes) staged per chunk

struct StageSrc {
    const void* in;
    int first;   // layer 0: input is the observation (fp32 to be quantized, or uint8 codes)
    int in_u8;
    float s0;
    int z0;
    uint8_t* tap_a0;
};

// address of the first of `run` contiguous input bytes that hold k .. k+run-1 of output row `row`
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

template <int MT, int NB, bool ASYM>
__global__ __launch_bounds__(256) void k_layer_int8(const FwdArgs a, const int l, const LayerIO io, const int64_t rows,
                                                    const int vec_ok) {
    constexpr int ROWS = 32 * MT;
    constexpr int LD = KC * 32 + 16;
    __shared__ __align__(16) int8_t xs[ROWS * LD];
    const LayerDev& L = a.L[l];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    const bool first = l == 0, last = l == a.n_layers - 1;
    const bool ln = !last && L.act == AQ_ACT_LN_TANH;
    const int grp = blockIdx.y * 4 + wave;
    const int ngroups = (L.NT + NB - 1) / NB;
    const bool active = grp < ngroups;
    float s0 = 1.0f;
    int z0 = 0;
    if (first) {
        s0 = a.actq[0].s;
        z0 = a.actq[0].z;
    }
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
    const v4i* wptr[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int nt = grp * NB + nb;
        nt = nt < L.NT ? nt : L.NT - 1;
        wptr[nb] = (const v4i*)L.wp + (int64_t)nt * L.KS * 64 + lane;
    }

    for (int ks0 = 0; ks0 < L.KS; ks0 += KC) {
        const int ks1 = ks0 + KC < L.KS ? ks0 + KC : L.KS;
        if (ks0) __syncthreads();
        if (vec_ok) {
            // 16-byte gathers: every 16-byte piece of a row's K range is contiguous in the input
            const int chunks = (ks1 - ks0) * 2;
            for (int idx = tid; idx < ROWS * chunks; idx += 256) {
                const int m = idx / chunks, c = idx - m * chunks;
                const int k = ks0 * 32 + c * 16;
                const int64_t row = row0 + m;
                v4i v;
                v[0] = v[1] = v[2] = v[3] = 0;
                if (row < rows && k < L.K) {
                    v = *(const v4i*)((const int8_t*)io.in + gather_offset(L, row, k));
                    if (first) {  // raw unsigned codes -> signed domain
                        v[0] ^= 0x80808080;
                        v[1] ^= 0x80808080;
                        v[2] ^= 0x80808080;
                        v[3] ^= 0x80808080;
                    }
                }
                *(v4i*)(xs + m * LD + c * 16) = v;
            }
        } else {
            const int kb = (ks1 - ks0) * 32;
            for (int idx = tid; idx < ROWS * kb; idx += 256) {
                const int m = idx / kb, kk = idx - m * kb;
                const int k = ks0 * 32 + kk;
                const int64_t row = row0 + m;
                int sv = 0;
                if (row < rows && k < L.K) {
                    const int64_t off = gather_offset(L, row, k);
                    if (first) {
                        int code;
                        if (a.in_u8) code = ((const uint8_t*)io.in)[off];
                        else code = rint_clamp(((const float*)io.in)[off] / s0, -z0, 255 - z0) + z0;
                        if (a.tap_a0 && blockIdx.y == 0) a.tap_a0[off] = (uint8_t)code;
                        sv = code - 128;
                    } else {
                        sv = ((const int8_t*)io.in)[off];
                    }
                }
                xs[m * LD + kk] = (int8_t)sv;
            }
        }
        __syncthreads();
        if (active) mma_block<MT, NB, ASYM>(wptr, xs, LD, ks0, ks1, ks0, acc, rs, lane);
    }

    if (!active) return;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int nt = grp * NB + nb;
        if (nt >= L.NT) continue;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int64_t row = row0 + mt * 32 + (lane & 31);
            const bool row_ok = row < rows;
            if (ln) {
                // dequantized accumulators go to the LayerNorm kernel
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int n = nt * 32 + 8 * j + 4 * g + i;
                        if (row_ok && n < L.N) {
                            int val = acc[nb][mt][4 * j + i] + L.bias_fold[n];
                            if (ASYM) val -= zw_s * rs[mt][0];
                            if (L.tap_acc) L.tap_acc[row * L.N + n] = val;
                            io.ln_x[row * L.N + n] = (float)val * L.m[n];
                        }
                    }
            } else {
                // the last layer leaves y = (float)acc * m in a.tap_y's place; the head kernel follows
                epilogue_tile<ASYM>(L, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok, last, z_out, lo,
                                    (!last && row_ok) ? io.out + row * L.N : nullptr, (L.N & 3) == 0, L.N,
                                    last ? a.tap_y + row * L.N : nullptr, nullptr, AQ_HEAD_LINEAR);
            }
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
        float t = tanh_fast(y);
        if (tap_ln) tap_ln[row * N + n] = t;
        int code = rint_clamp(t / s_out, -z_out, 255 - z_out) + z_out;
        if (tap_act) tap_act[row * N + n] = (uint8_t)code;
        out[row * N + n] = (int8_t)(code - 128);
    }
}

// action head on the dequantized last-layer rows (per-layer path)
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

aq_status launch_layer_int8(const FwdArgs& a, int l, const LayerIO& io, hipStream_t st) {
    const LayerDev& L = a.L[l];
    const int64_t rows = a.batch * L.oh * L.ow;
    const bool first = l == 0;
    // 16-byte gathers need contiguous, aligned 16-byte pieces of K in the input
    const bool fc = L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1;
    const int run = fc ? L.K : L.kw * L.in_c;
    bool vec_ok = run % 16 == 0 && !(first && !a.in_u8) && !(first && a.tap_a0);
    if (!fc && ((L.stride * L.in_c) % 16 != 0 || (L.in_w * L.in_c) % 16 != 0)) vec_ok = false;
    constexpr int MT = 2, NB = 2;
    const int ngroups = (L.NT + NB - 1) / NB;
    dim3 grid((unsigned)((rows + 32 * MT - 1) / (32 * MT)), (unsigned)((ngroups + 3) / 4));
    if (a.asym)
        hipLaunchKernelGGL((k_layer_int8<MT, NB, true>), grid, dim3(256), 0, st, a, l, io, rows, (int)vec_ok);
    else
        hipLaunchKernelGGL((k_layer_int8<MT, NB, false>), grid, dim3(256), 0, st, a, l, io, rows, (int)vec_ok);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_ln_tanh_rows(const FwdArgs& a, int l, const float* x, int8_t* out, int64_t rows, hipStream_t st) {
    const LayerDev& L = a.L[l];
    hipLaunchKernelGGL(k_ln_tanh_rows, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, x, rows, L.N, L.gamma,
                       L.beta, a.ln_eps, a.actq, l + 1, out, L.tap_ln, L.tap_act);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_head_rows(const float* y, int64_t rows, int N, int head, void* actions, hipStream_t st) {
    const int64_t n = head == AQ_HEAD_ARGMAX ? rows : rows * N;
    hipLaunchKernelGGL(k_head_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, y, rows, N, head, actions);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
