// The half-precision actor (the paper's fp16 policies, Sec. 3.2, and actors at q = 16): parameters,
// observation and every operator's output are IEEE binary16 values; products are exact and sums are
// kept in fp32 by v_mfma_f32_32x32x16_f16, rounded to binary16 once per operator.
//
//   k_fp16_pack_weights   fp32 [N][K] -> binary16 in MFMA operand order (tile (n/32, k/16) = 1 KiB,
//                         lane = n % 32 + 32 * ((k % 16) / 8), 8 consecutive k per lane), zero padded
//   k_fp16_round_vec      biases / LayerNorm gain and offset rounded to binary16 (kept widened)
//   k_layer_fp16          affine layer (FC or implicit-GEMM convolution) + bias (+ReLU), one launch per layer
//   k_fp16_ln_tanh        LayerNorm, rounded, then tanh, rounded, in place
//   k_fp16_head           tanh / identity / argmax on the last layer's rows
#include "kernels.hpp"

namespace aq {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f16acc __attribute__((ext_vector_type(16)));

namespace {

constexpr int HR = 64;    // rows per workgroup (two 32-row MFMA tiles)
constexpr int HW = 4;     // waves per workgroup
constexpr int HNB = 2;    // feature tiles per wave
constexpr int HKC = 64;   // k per staged chunk
constexpr int HLD = HKC + 8;  // LDS row stride in halfs (144 bytes: 16-byte reads of 8 rows hit 32 banks)

__global__ __launch_bounds__(256) void k_fp16_pack_weights(const float* __restrict__ w, int N, int K, int KS16,
                                                           int NT, _Float16* __restrict__ wp, int* status) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)NT * KS16 * 512;
    if (i >= total) return;
    const int j = (int)(i & 7), lane = (int)((i >> 3) & 63);
    const int64_t tile = i >> 9;
    const int ks = (int)(tile % KS16), nt = (int)(tile / KS16);
    const int n = nt * 32 + (lane & 31), k = ks * 16 + 8 * (lane >> 5) + j;
    _Float16 v = (_Float16)0.0f;
    if (n < N && k < K) {
        v = (_Float16)w[(int64_t)n * K + k];
        if (!(fabsf((float)v) <= 65504.0f)) atomicOr(status, kStatNonFinite);
    }
    wp[i] = v;
}

__global__ __launch_bounds__(256) void k_fp16_round_vec(const float* __restrict__ src, int n, int n_pad, float fill,
                                                        float* __restrict__ dst, int* status) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_pad) return;
    float v = fill;
    if (i < n && src) {
        v = (float)(_Float16)src[i];
        if (!(fabsf(v) <= 65504.0f)) atomicOr(status, kStatNonFinite);
    }
    dst[i] = v;
}

struct RowPos {
    int64_t base;  // element offset of (row, k = 0) in the layer's input
    bool ok;
};

__device__ __forceinline__ RowPos row_pos(const Fp16Layer& L, int64_t row, int64_t rows) {
    RowPos r;
    r.ok = row < rows;
    if (L.fc) {
        r.base = row * L.K;
    } else {
        const int per_img = L.oh * L.ow;
        const int64_t b = row / per_img;
        const int q = (int)(row - b * per_img);
        const int oy = q / L.ow, ox = q - oy * L.ow;
        r.base = ((b * L.in_h + (int64_t)oy * L.stride) * L.in_w + (int64_t)ox * L.stride) * L.in_c;
    }
    return r;
}

// offset of reduction index k relative to the row's base
__device__ __forceinline__ int64_t k_offset(const Fp16Layer& L, int k) {
    if (L.fc) return k;
    const int run = L.kw * L.in_c;
    const int ky = k / run, kr = k - ky * run;
    return (int64_t)ky * L.in_w * L.in_c + kr;
}

// IN: 0 = binary16 activations, 1 = fp32 observations, 2 = uint8 observations (exact in binary16)
// VEC: 16-byte pieces of 8 consecutive k are contiguous and aligned in the input (binary16 input only)
template <int IN, bool VEC>
__global__ __launch_bounds__(256) void k_layer_fp16(const Fp16Layer L, const void* __restrict__ in,
                                                    _Float16* __restrict__ out, const int64_t rows) {
    __shared__ __align__(16) _Float16 xs[2][HR * HLD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * HR;
    const int nt0 = (blockIdx.y * HW + wave) * HNB;  // this wave's first feature tile
    const bool wave_on = nt0 < L.NT;
    const int KC = L.KS16 / 4;  // chunks of 64

    // staging: thread -> rows (tid >> 3) and (tid >> 3) + 32, k piece (tid & 7) * 8 of each chunk
    const int sr = tid >> 3, sk = (tid & 7) * 8;
    const RowPos rp0 = row_pos(L, row0 + sr, rows), rp1 = row_pos(L, row0 + sr + 32, rows);

    auto load_x = [&](int c, h8& x0, h8& x1) __attribute__((always_inline)) {
        const int k0 = c * HKC + sk;
        if (VEC) {
            const h8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            const int64_t off = k_offset(L, k0);
            const bool kok = k0 < L.K;  // K is a multiple of 8 here, so a piece is whole or empty
            x0 = (rp0.ok && kok) ? *(const h8*)((const _Float16*)in + rp0.base + off) : z;
            x1 = (rp1.ok && kok) ? *(const h8*)((const _Float16*)in + rp1.base + off) : z;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int k = k0 + j;
                _Float16 a = (_Float16)0.0f, b = (_Float16)0.0f;
                if (k < L.K) {
                    const int64_t off = k_offset(L, k);
                    if (IN == 0) {
                        if (rp0.ok) a = ((const _Float16*)in)[rp0.base + off];
                        if (rp1.ok) b = ((const _Float16*)in)[rp1.base + off];
                    } else if (IN == 1) {
                        if (rp0.ok) a = (_Float16)((const float*)in)[rp0.base + off];
                        if (rp1.ok) b = (_Float16)((const float*)in)[rp1.base + off];
                    } else {
                        if (rp0.ok) a = (_Float16)(float)((const uint8_t*)in)[rp0.base + off];
                        if (rp1.ok) b = (_Float16)(float)((const uint8_t*)in)[rp1.base + off];
                    }
                }
                x0[j] = a;
                x1[j] = b;
            }
        }
    };
    auto store_x = [&](int buf, const h8& x0, const h8& x1) __attribute__((always_inline)) {
        *(h8*)&xs[buf][sr * HLD + sk] = x0;
        *(h8*)&xs[buf][(sr + 32) * HLD + sk] = x1;
    };
    // this wave's weights of one chunk: 4 k-steps x HNB tiles, 16 bytes per lane each
    const h8* wbase = (const h8*)L.wp + lane;
    auto load_w = [&](int c, h8 (&wr)[4][HNB]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int nb = 0; nb < HNB; ++nb) {
                const int nt = nt0 + nb < L.NT ? nt0 + nb : L.NT - 1;  // (clamped: the tile is not stored)
                wr[s][nb] = wbase[((int64_t)nt * L.KS16 + c * 4 + s) * 64];
            }
    };

    f16acc acc[HNB][2];
#pragma unroll
    for (int nb = 0; nb < HNB; ++nb)
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[nb][mt][i] = 0.0f;

    h8 wc[4][HNB], wn[4][HNB];
    h8 x0, x1;
    if (wave_on) load_w(0, wc);
    load_x(0, x0, x1);
    store_x(0, x0, x1);
    __syncthreads();
    for (int c = 0; c < KC; ++c) {
        const bool more = c + 1 < KC;
        if (more) {
            if (wave_on) load_w(c + 1, wn);
            load_x(c + 1, x0, x1);
        }
        if (wave_on) {
            const _Float16* xb = xs[c & 1];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                h8 bx[2];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    bx[mt] = *(const h8*)&xb[(mt * 32 + (lane & 31)) * HLD + s * 16 + 8 * (lane >> 5)];
#pragma unroll
                for (int nb = 0; nb < HNB; ++nb)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
                        acc[nb][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wc[s][nb], bx[mt], acc[nb][mt], 0, 0, 0);
            }
        }
        if (more) {
            store_x((c + 1) & 1, x0, x1);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int nb = 0; nb < HNB; ++nb) wc[s][nb] = wn[s][nb];
        }
        __syncthreads();
    }
    if (!wave_on) return;

    // epilogue: + bias, rounded to binary16 once, ReLU; lane = one row, four consecutive features per quad
    const bool vec_out = (L.N & 3) == 0;
#pragma unroll
    for (int nb = 0; nb < HNB; ++nb) {
        if (nt0 + nb >= L.NT) continue;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int64_t row = row0 + mt * 32 + (lane & 31);
            if (row >= rows) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n0 = (nt0 + nb) * 32 + 8 * q + 4 * (lane >> 5);
                if (n0 >= L.N) continue;
                const float4 bv = *(const float4*)(L.bias + n0);  // padded to the tile
                const float b4[4] = {bv.x, bv.y, bv.z, bv.w};
                h4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    _Float16 v = (_Float16)(acc[nb][mt][4 * q + i] + b4[i]);
                    if (L.relu) v = v > (_Float16)0.0f ? v : (_Float16)0.0f;
                    o[i] = v;
                }
                _Float16* dst = out + row * L.N + n0;
                if (vec_out) {
                    *(h4*)dst = o;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n0 + i < L.N) dst[i] = o[i];
                }
            }
        }
    }
}

// LayerNorm (biased variance, eps inside the root) rounded to binary16, then tanh rounded to binary16;
// one wavefront per row, in place
__global__ __launch_bounds__(256) void k_fp16_ln_tanh(_Float16* __restrict__ x, int64_t rows, int N,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    _Float16* xr = x + row * N;
    float s = 0.0f;
    for (int n = lane; n < N; n += 64) s += (float)xr[n];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    const float mean = s / (float)N;
    float ss = 0.0f;
    for (int n = lane; n < N; n += 64) {
        const float d = (float)xr[n] - mean;
        ss += d * d;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    const float inv = 1.0f / sqrtf(ss / (float)N + eps);
    for (int n = lane; n < N; n += 64) {
        const _Float16 ln = (_Float16)(((float)xr[n] - mean) * inv * gamma[n] + beta[n]);
        xr[n] = (_Float16)tanhf((float)ln);
    }
}

__global__ __launch_bounds__(256) void k_fp16_head(const _Float16* __restrict__ y, int64_t rows, int N, int head,
                                                   void* __restrict__ actions) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (head == AQ_HEAD_ARGMAX) {
        if (i >= rows) return;
        const _Float16* yr = y + i * N;
        int best = 0;
        float bv = (float)yr[0];
        for (int n = 1; n < N; ++n) {
            const float v = (float)yr[n];
            if (v > bv) {
                bv = v;
                best = n;
            }
        }
        ((int32_t*)actions)[i] = best;
    } else {
        if (i >= rows * N) return;
        const float v = (float)y[i];
        ((float*)actions)[i] = head == AQ_HEAD_TANH ? (float)(_Float16)tanhf(v) : v;
    }
}

}  // namespace

aq_status launch_fp16_pack_weights(const float* w, int N, int K, int KS16, int NT, void* wp, int* status,
                                   hipStream_t st) {
    const int64_t total = (int64_t)NT * KS16 * 512;
    hipLaunchKernelGGL(k_fp16_pack_weights, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, N, K, KS16, NT,
                       (_Float16*)wp, status);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp16_round_vec(const float* src, int n, int n_pad, float fill, float* dst, int* status,
                                hipStream_t st) {
    hipLaunchKernelGGL(k_fp16_round_vec, dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st, src, n, n_pad, fill,
                       dst, status);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_layer_fp16(const Fp16Layer& L, const void* in, int in_mode, void* out, int64_t rows,
                            hipStream_t st) {
    if (rows < 1) return AQ_OK;
    if (L.KS16 % 4 != 0 || L.NT < 1) return AQ_ESHAPE;
    const dim3 grid((unsigned)((rows + HR - 1) / HR), (unsigned)((L.NT + HW * HNB - 1) / (HW * HNB)));
    _Float16* o = (_Float16*)out;
    // 16-byte pieces: binary16 input whose runs of consecutive k start and end on multiples of 8
    const bool vec = in_mode == 0 && ((uintptr_t)in & 15) == 0 && (L.fc ? L.K % 8 == 0 : L.in_c % 8 == 0);
    if (in_mode == 0) {
        if (vec) hipLaunchKernelGGL((k_layer_fp16<0, true>), grid, dim3(256), 0, st, L, in, o, rows);
        else hipLaunchKernelGGL((k_layer_fp16<0, false>), grid, dim3(256), 0, st, L, in, o, rows);
    } else if (in_mode == 1) {
        hipLaunchKernelGGL((k_layer_fp16<1, false>), grid, dim3(256), 0, st, L, in, o, rows);
    } else {
        hipLaunchKernelGGL((k_layer_fp16<2, false>), grid, dim3(256), 0, st, L, in, o, rows);
    }
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp16_ln_tanh(void* x, int64_t rows, int N, const float* gamma, const float* beta, float eps,
                              hipStream_t st) {
    hipLaunchKernelGGL(k_fp16_ln_tanh, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, (_Float16*)x, rows, N, gamma,
                       beta, eps);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp16_head(const void* y, int64_t rows, int N, int head, void* actions, hipStream_t st) {
    const int64_t n = head == AQ_HEAD_ARGMAX ? rows : rows * N;
    hipLaunchKernelGGL(k_fp16_head, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const _Float16*)y, rows, N,
                       head, actions);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
