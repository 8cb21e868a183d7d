// The full-precision actor (the paper's fp32 baseline policy, Sec. 3.1) and the min/max
// calibration of activation ranges.  Comparator only: a plain LDS-tiled fp32 GEMM (64x64 outputs
// per workgroup, 4x4 per thread) with the same implicit-GEMM gather as the 8-bit path.
#include "kernels.hpp"

namespace aq {

__device__ __forceinline__ int64_t gather_offset32(const Fp32Layer& L, int64_t row, int k) {
    if (L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1) return row * L.K + k;
    const int per_img = L.oh * L.ow;
    const int64_t b = row / per_img;
    const int r = (int)(row - b * per_img);
    const int oy = r / L.ow, ox = r - oy * L.ow;
    const int run = L.kw * L.in_c;
    const int ky = k / run, kr = k - ky * run;
    return ((b * L.in_h + (int64_t)oy * L.stride + ky) * L.in_w + (int64_t)ox * L.stride) * L.in_c + kr;
}

constexpr int TB = 64;  // tile edge
constexpr int TK = 16;  // k per stage

__global__ __launch_bounds__(256) void k_fp32_layer(const Fp32Layer L, const void* __restrict__ in, const int in_u8,
                                                    float* __restrict__ out, const int64_t rows, const int relu) {
    __shared__ float As[TK][TB + 4];
    __shared__ float Bs[TK][TB + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t row0 = (int64_t)blockIdx.x * TB;
    const int n0 = blockIdx.y * TB;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
    const int lr = tid >> 2;        // 0..63: tile row (A) / tile column (B) this thread loads
    const int lk = (tid & 3) * 4;   // first of its 4 k values
    for (int k0 = 0; k0 < L.K; k0 += TK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = k0 + lk + i;
            const int64_t row = row0 + lr;
            float av = 0.0f, bv = 0.0f;
            if (k < L.K) {
                if (row < rows) {
                    const int64_t off = gather_offset32(L, row, k);
                    av = in_u8 ? (float)((const uint8_t*)in)[off] : ((const float*)in)[off];
                }
                if (n0 + lr < L.N) bv = L.w[(int64_t)(n0 + lr) * L.K + k];
            }
            As[lk + i][lr] = av;
            Bs[lk + i][lr] = bv;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < TK; ++k) {
            float a4[4], b4[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a4[i] = As[k][ty * 4 + i];
                b4[i] = Bs[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a4[i], b4[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t row = row0 + ty * 4 + i;
        if (row >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= L.N) continue;
            float v = acc[i][j] + (L.b ? L.b[n] : 0.0f);
            if (relu) v = v > 0.0f ? v : 0.0f;
            out[row * L.N + n] = v;
        }
    }
}

// LayerNorm (biased variance, eps inside the root) + tanh in place, one wavefront per row
__global__ __launch_bounds__(256) void k_fp32_ln_tanh(float* __restrict__ x, int64_t rows, int N,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    float* xr = x + row * N;
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
        float g = gamma ? gamma[n] : 1.0f, b = beta ? beta[n] : 0.0f;
        xr[n] = tanhf((xr[n] - mean) * inv * g + b);
    }
}

__global__ void k_fp32_head(const float* __restrict__ y, int64_t rows, int N, int head, void* __restrict__ actions) {
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
        ((float*)actions)[i] = head == AQ_HEAD_TANH ? tanhf(y[i]) : y[i];
    }
}

// min / max of a tensor through order-preserving unsigned keys; keys[0] must start at 0xffffffff
// (min) and keys[1] at 0 (max).
__device__ __forceinline__ uint32_t f2key(float f) {
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key2f(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ __launch_bounds__(256) void k_minmax_keys(const void* __restrict__ x, int is_u8, int64_t n,
                                                     uint32_t* __restrict__ keys) {
    float lo = INFINITY, hi = -INFINITY;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float v = is_u8 ? (float)((const uint8_t*)x)[i] : ((const float*)x)[i];
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    if ((threadIdx.x & 63) == 0 && lo <= hi) {
        atomicMin(&keys[0], f2key(lo));
        atomicMax(&keys[1], f2key(hi));
    }
}

__global__ void k_keys_to_ranges(const uint32_t* __restrict__ keys, int n, float* __restrict__ out) {
    int i = threadIdx.x;
    if (i < n) out[i] = key2f(keys[i]);
}

__global__ void k_init_keys(uint32_t* keys, int n_pairs) {
    int i = threadIdx.x;
    if (i < n_pairs) {
        keys[2 * i] = 0xffffffffu;
        keys[2 * i + 1] = 0u;
    }
}

aq_status launch_fp32_layer(const Fp32Layer& L, const void* in, int in_u8, float* out, int64_t rows, int relu,
                            hipStream_t st) {
    dim3 grid((unsigned)((rows + TB - 1) / TB), (unsigned)((L.N + TB - 1) / TB));
    hipLaunchKernelGGL(k_fp32_layer, grid, dim3(256), 0, st, L, in, in_u8, out, rows, relu);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp32_ln_tanh(float* x, int64_t rows, int N, const float* gamma, const float* beta, float eps,
                              hipStream_t st) {
    hipLaunchKernelGGL(k_fp32_ln_tanh, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, x, rows, N, gamma, beta,
                       eps);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp32_head(const float* y, int64_t rows, int N, int head, void* actions, hipStream_t st) {
    const int64_t n = head == AQ_HEAD_ARGMAX ? rows : rows * N;
    hipLaunchKernelGGL(k_fp32_head, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, y, rows, N, head, actions);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_init_keys(uint32_t* keys, int n_pairs, hipStream_t st) {
    hipLaunchKernelGGL(k_init_keys, dim3(1), dim3(64), 0, st, keys, n_pairs);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_minmax_keys(const void* x, int is_u8, int64_t n, uint32_t* keys, hipStream_t st) {
    int64_t g = (n + 256 * 8 - 1) / (256 * 8);
    if (g < 1) g = 1;
    if (g > 2048) g = 2048;
    hipLaunchKernelGGL(k_minmax_keys, dim3((unsigned)g), dim3(256), 0, st, x, is_u8, n, keys);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_keys_to_ranges(const uint32_t* keys, int n, float* out, hipStream_t st) {
    hipLaunchKernelGGL(k_keys_to_ranges, dim3(1), dim3(64), 0, st, keys, n, out);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
