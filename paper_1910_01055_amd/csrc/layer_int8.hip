// One launch per layer: FC and implicit-GEMM convolution on int8 MFMA, activations in global memory.
#include "int8_device.hpp"

namespace aq {

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

template <int MT, int NB, bool ASYM, bool TAPS>
__global__ __launch_bounds__(256) void k_layer_int8(const NetDev* __restrict__ netp, const TapArgs t, const int l, const LayerIO io, const int64_t rows,
                                                    const int vec_ok) {
    constexpr int ROWS = 32 * MT;
    constexpr int LD = KC * 32 + 16;
    __shared__ __align__(16) int8_t xs[ROWS * LD];
    const NetDev& a = *netp;
    const LayerDev& L = a.L[l];
    LayerTaps T{nullptr, nullptr, nullptr};
    if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
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
        if (active) mma_block<MT, NB, ASYM, 4>(wptr, xs, LD, ks0, ks1, ks0, acc, rs, lane);
    }

    if (!active) return;
    const CPtrs C = global_consts(L);
    const bool fast = !last && !ln && a.fast[l] != 0;
    static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
        constexpr int nb = decltype(nb_c)::value;
        const int nt = grp * NB + nb;
        if (nt < L.NT) {
            static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                constexpr int mt = decltype(mt_c)::value;
                const int64_t row = row0 + mt * 32 + (lane & 31);
                const bool row_ok = row < rows;
                if (ln) {
                    // dequantized accumulators go to the LayerNorm kernel
                    epi_last_tile<ASYM, TAPS>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok,
                                              row_ok ? io.ln_x + row * L.N : nullptr, L.N);
                } else if (last) {
                    // y = (float)acc * m; the head kernel follows
                    epi_last_tile<ASYM, TAPS>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok,
                                              row_ok ? io.y + row * L.N : nullptr, L.N);
                } else if (fast) {
                    epi_hidden_tile<ASYM, TAPS, true>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok, z_out,
                                                      lo, row_ok ? io.out + row * L.N : nullptr, (L.N & 3) == 0, L.N);
                } else {
                    epi_hidden_tile<ASYM, TAPS, false>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row, row_ok, z_out,
                                                       lo, row_ok ? io.out + row * L.N : nullptr, (L.N & 3) == 0, L.N);
                }
            });
        }
    });
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
        float t = tanh_fast(y);
        if (tap_ln) tap_ln[row * N + n] = t;
        int code = quant_code(t, qs_out, -z_out, 255 - z_out) + z_out;
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
    const LayerDev& L = a.net.L[l];
    const int64_t rows = a.c.batch * L.oh * L.ow;
    const bool first = l == 0;
    // 16-byte gathers need contiguous, aligned 16-byte pieces of K in the input
    const bool fc = L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1;
    const int run = fc ? L.K : L.kw * L.in_c;
    bool vec_ok = run % 16 == 0 && !(first && !a.net.in_u8) && !(first && a.t.a0);
    if (!fc && ((L.stride * L.in_c) % 16 != 0 || (L.in_w * L.in_c) % 16 != 0)) vec_ok = false;
    constexpr int MT = 2, NB = 2;
    const int ngroups = (L.NT + NB - 1) / NB;
    dim3 grid((unsigned)((rows + 32 * MT - 1) / (32 * MT)), (unsigned)((ngroups + 3) / 4));
    const bool taps = any_taps(a);
#define AQ_LAYER(AS, TP) \
    hipLaunchKernelGGL((k_layer_int8<MT, NB, AS, TP>), grid, dim3(256), 0, st, a.d_net, a.t, l, io, rows, (int)vec_ok)
    if (a.net.asym) {
        if (taps) AQ_LAYER(true, true);
        else AQ_LAYER(true, false);
    } else {
        if (taps) AQ_LAYER(false, true);
        else AQ_LAYER(false, false);
    }
#undef AQ_LAYER
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
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
