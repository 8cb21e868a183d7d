// Quantizer block (Sec. 3.1, Sec. 3.2): fp32 weights -> 8-bit codes + scales + integer layer constants.
//
// The weight passes are HBM-bandwidth bound (4 bytes read + 1 byte written per parameter);
// they are written as coalesced float4 streams with wavefront-shuffle reductions.  A whole
// output channel is kept in registers between the range reduction and the rounding, so a
// per-channel tensor is read from HBM exactly once.
#include "kernels.hpp"

#include <float.h>

namespace aq {

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, int n, uint32_t v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__device__ __forceinline__ bool finite_f(float v) { return fabsf(v) <= FLT_MAX; }
typedef float f4v __attribute__((ext_vector_type(4)));

// Sec. 3.2: delta = (|min(W,0)| + |max(W,0)|) / D ; zero-point z = round(-lo / delta).
// (n bits: D = 2^n - 1 or 2^n, codes and zero-point in [0, qmax = 2^n - 1])
__device__ __forceinline__ void asym_qparams(float hi, float nlo, float qdenom, int qmax, float& s, int& z) {
    float lo = -nlo;
    s = (hi - lo) / qdenom;
    if (hi == lo) s = 1.0f;
    z = rint_clamp(-lo / s, 0, qmax);
}

// ---------------------------------------------------------------------------------------------
// per-tensor range: hi = max(W, 0), nlo = max(-W, 0).  Both are non-negative floats, whose bit
// patterns order like unsigned integers, so the grid-wide reduction is one atomicMax each.
// mm[0] = hi bits, mm[1] = nlo bits, mm[2] = status flag; mm must be zero before the launch.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void range_nonneg_block(const float4* __restrict__ w4, int64_t n4,
                                                   const float* __restrict__ w, int64_t n,
                                                   uint32_t* __restrict__ mm, int blk, int nblk) {
    float hi = 0.0f, nlo = 0.0f;
    int bad = 0;
    const int64_t stride = (int64_t)nblk * blockDim.x;
    for (int64_t i = (int64_t)blk * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 v = w4[i];
        float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bad |= !finite_f(e[j]);
            hi = e[j] > hi ? e[j] : hi;
            float t = -e[j];
            nlo = t > nlo ? t : nlo;
        }
    }
    // scalar tail (tensor length not a multiple of 4)
    for (int64_t i = n4 * 4 + (int64_t)blk * blockDim.x + threadIdx.x; i < n; i += stride) {
        float e = w[i];
        bad |= !finite_f(e);
        hi = e > hi ? e : hi;
        float t = -e;
        nlo = t > nlo ? t : nlo;
    }
    hi = wave_max(hi);
    nlo = wave_max(nlo);
    bad = wave_or_i32(bad);
    __shared__ float s_hi[4], s_nlo[4];
    __shared__ int s_bad[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) {
        s_hi[wv] = hi;
        s_nlo[wv] = nlo;
        s_bad[wv] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < 4; ++i) {
            hi = fmaxf(hi, s_hi[i]);
            nlo = fmaxf(nlo, s_nlo[i]);
            bad |= s_bad[i];
        }
        atomicMax(&mm[0], __float_as_uint(hi));
        atomicMax(&mm[1], __float_as_uint(nlo));
        if (bad) atomicOr(&mm[2], 1u);
    }
}

// Pass 1 of the per-tensor scheme for a large flat tensor: every workgroup publishes its partial
// range (hi bits, -lo bits, non-finite flag) in part[3 * block]; nothing has to be cleared first.
__global__ __launch_bounds__(256) void k_range_partials(const float4* __restrict__ w4, int64_t n4,
                                                        uint32_t* __restrict__ part) {
    float hi = 0.0f, nlo = 0.0f;
    int bad = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const float4 v = w4[i];
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bad |= !finite_f(e[j]);
            hi = e[j] > hi ? e[j] : hi;
            const float t = -e[j];
            nlo = t > nlo ? t : nlo;
        }
    }
    hi = wave_max(hi);
    nlo = wave_max(nlo);
    bad = wave_or_i32(bad);
    __shared__ float s_hi[4], s_nlo[4];
    __shared__ int s_bad[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) {
        s_hi[wv] = hi;
        s_nlo[wv] = nlo;
        s_bad[wv] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        part[3 * blockIdx.x + 0] = __float_as_uint(fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3])));
        part[3 * blockIdx.x + 1] = __float_as_uint(fmaxf(fmaxf(s_nlo[0], s_nlo[1]), fmaxf(s_nlo[2], s_nlo[3])));
        part[3 * blockIdx.x + 2] = (uint32_t)(s_bad[0] | s_bad[1] | s_bad[2] | s_bad[3]);
    }
}

// Pass 2: every workgroup folds the partials (a few KiB, cache resident), then streams its share of
// the tensor: 16 bytes in, 4 codes out per thread and iteration.  The second read of the tensor
// comes from the last-level cache for tensors that fit it.
__global__ __launch_bounds__(256) void k_quant_asym_flat(const float4* __restrict__ w4, int64_t n4,
                                                         const uint32_t* __restrict__ part, int n_part, float qdenom,
                                                         int qmax, uint32_t* __restrict__ codes, float* __restrict__ scale,
                                                         int32_t* __restrict__ zp, uint32_t* __restrict__ flag) {
    float hi = 0.0f, nlo = 0.0f;
    int bad = 0;
    for (int b = threadIdx.x; b < n_part; b += 256) {
        hi = fmaxf(hi, __uint_as_float(part[3 * b + 0]));
        nlo = fmaxf(nlo, __uint_as_float(part[3 * b + 1]));
        bad |= (int)part[3 * b + 2];
    }
    hi = wave_max(hi);
    nlo = wave_max(nlo);
    bad = wave_or_i32(bad);
    __shared__ float s_hi[4], s_nlo[4];
    __shared__ int s_bad[4];
    if ((threadIdx.x & 63) == 0) {
        s_hi[threadIdx.x >> 6] = hi;
        s_nlo[threadIdx.x >> 6] = nlo;
        s_bad[threadIdx.x >> 6] = bad;
    }
    __syncthreads();
    hi = fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3]));
    nlo = fmaxf(fmaxf(s_nlo[0], s_nlo[1]), fmaxf(s_nlo[2], s_nlo[3]));
    float s;
    int z;
    asym_qparams(hi, nlo, qdenom, qmax, s, z);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        scale[0] = s;
        zp[0] = z;
        if (s_bad[0] | s_bad[1] | s_bad[2] | s_bad[3]) flag[0] = 1u;
    }
    const QuantScale qs = make_quant_scale(s);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const f4v q = __builtin_nontemporal_load((const f4v*)w4 + i);  // (last use of the tensor)
        __builtin_nontemporal_store(quant_code4(make_float4(q[0], q[1], q[2], q[3]), qs, -z, qmax - z, z), codes + i);
    }
}

// per-channel symmetric codes, canonical order: one wavefront per row, the row lives in
// registers (R float4 per lane) between the |w| reduction and the rounding.
template <int R>
__global__ __launch_bounds__(256) void k_quant_sym_rows_flat(const float4* __restrict__ w4, int64_t rows, int cols4, int qw,
                                                             uint32_t* __restrict__ codes, float* __restrict__ scale,
                                                             int32_t* __restrict__ zp, uint32_t* __restrict__ mm) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float4* src = w4 + row * cols4;
    float4 v[R];
    float amax = 0.0f;
    int bad = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int c = lane + 64 * r;
        v[r] = c < cols4 ? src[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        float a0 = fabsf(v[r].x), a1 = fabsf(v[r].y), a2 = fabsf(v[r].z), a3 = fabsf(v[r].w);
        bad |= !(a0 <= FLT_MAX) | !(a1 <= FLT_MAX) | !(a2 <= FLT_MAX) | !(a3 <= FLT_MAX);
        amax = fmaxf(fmaxf(amax, fmaxf(a0, a1)), fmaxf(a2, a3));
    }
    amax = wave_max(amax);
    bad = wave_or_i32(bad);
    float s = amax / (float)qw;
    if (amax == 0.0f) s = 1.0f;
    if (lane == 0) {
        scale[row] = s;
        zp[row] = 0;
        if (bad) atomicOr(&mm[2], 1u);
    }
    uint32_t* dst = codes + row * cols4;
    const QuantScale qs = make_quant_scale(s);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int c = lane + 64 * r;
        if (c < cols4) {
            __builtin_nontemporal_store(quant_code4(v[r], qs, -qw, qw, 0), dst + c);
        }
    }
}

// Longer rows: one workgroup per row, R float4 per thread held in registers between the |w|
// reduction and the rounding (still one pass over HBM).  Many small workgroups keep the memory
// pipeline of every CU busy while others are in their arithmetic phase.
template <int R>
__global__ __launch_bounds__(256) void k_quant_sym_row_wg(const float4* __restrict__ w4, int cols4, int qw,
                                                          uint32_t* __restrict__ codes, float* __restrict__ scale,
                                                          int32_t* __restrict__ zp, uint32_t* __restrict__ mm) {
    const int64_t row = blockIdx.x;
    const float4* src = w4 + row * cols4;
    float4 v[R];
    float amax = 0.0f;
    int bad = 0;
    // (the tensor is read once and the codes are written once: both bypass the cache hierarchy's retention)
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = threadIdx.x + 256 * r;
        if (c < cols4) {
            const f4v q = __builtin_nontemporal_load((const f4v*)src + c);
            v[r] = make_float4(q[0], q[1], q[2], q[3]);
        } else {
            v[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float a0 = fabsf(v[r].x), a1 = fabsf(v[r].y), a2 = fabsf(v[r].z), a3 = fabsf(v[r].w);
        bad |= !(a0 <= FLT_MAX) | !(a1 <= FLT_MAX) | !(a2 <= FLT_MAX) | !(a3 <= FLT_MAX);
        amax = fmaxf(fmaxf(amax, fmaxf(a0, a1)), fmaxf(a2, a3));
    }
    amax = wave_max(amax);
    __shared__ float s_max[4];
    if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = amax;
    if (bad) atomicOr(&mm[2], 1u);
    __syncthreads();
    amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    float s = amax / (float)qw;
    if (amax == 0.0f) s = 1.0f;
    if (threadIdx.x == 0) {
        scale[row] = s;
        zp[row] = 0;
    }
    const QuantScale qs = make_quant_scale(s);
    uint32_t* dst = codes + row * cols4;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int c = threadIdx.x + 256 * r;
        if (c < cols4) __builtin_nontemporal_store(quant_code4(v[r], qs, -qw, qw, 0), dst + c);
    }
}

// rows too long for the register-resident kernel: one workgroup per row, the row is read twice
// (the second read comes from cache for any realistic channel length).
__global__ __launch_bounds__(256) void k_quant_sym_rows_long(const float4* __restrict__ w4, int64_t rows, int cols4, int qw,
                                                             uint32_t* __restrict__ codes, float* __restrict__ scale,
                                                             int32_t* __restrict__ zp, uint32_t* __restrict__ mm) {
    const int64_t row = blockIdx.x;
    const float4* src = w4 + row * cols4;
    float amax = 0.0f;
    int bad = 0;
    for (int c = threadIdx.x; c < cols4; c += 256) {
        float4 v = src[c];
        float a0 = fabsf(v.x), a1 = fabsf(v.y), a2 = fabsf(v.z), a3 = fabsf(v.w);
        bad |= !(a0 <= FLT_MAX) | !(a1 <= FLT_MAX) | !(a2 <= FLT_MAX) | !(a3 <= FLT_MAX);
        amax = fmaxf(fmaxf(amax, fmaxf(a0, a1)), fmaxf(a2, a3));
    }
    amax = wave_max(amax);
    bad = wave_or_i32(bad);
    __shared__ float s_max[4];
    __shared__ int s_bad[4];
    if ((threadIdx.x & 63) == 0) {
        s_max[threadIdx.x >> 6] = amax;
        s_bad[threadIdx.x >> 6] = bad;
    }
    __syncthreads();
    amax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    bad = s_bad[0] | s_bad[1] | s_bad[2] | s_bad[3];
    float s = amax / (float)qw;
    if (amax == 0.0f) s = 1.0f;
    if (threadIdx.x == 0) {
        scale[row] = s;
        zp[row] = 0;
        if (bad) atomicOr(&mm[2], 1u);
    }
    uint32_t* dst = codes + row * cols4;
    const QuantScale qs = make_quant_scale(s);
    for (int c = threadIdx.x; c < cols4; c += 256) {
        dst[c] = quant_code4(src[c], qs, -qw, qw, 0);
    }
}

// ---------------------------------------------------------------------------------------------
// Policy weights: one wavefront per output channel n of W[N][K]; codes are written in the
// signed domain (unsigned codes minus 128; symmetric codes as they are) straight into the
// MFMA operand order used by the forward kernels:
//   tile (nt = n / 32, ks = k / 32) is 1 KiB: lane = n % 32 + 32 * ((k % 32) / 16), byte = k % 16.
// Also produced per channel: scale, zero-point, and the sum of the signed-domain codes (needed to
// fold the activation zero-point into the integer bias).
// ---------------------------------------------------------------------------------------------
template <bool SYM>
__device__ __forceinline__ void quant_row_packed(const float* __restrict__ w, int n, int N, int K, int KS,
                                                 float qdenom, int qmax, int qw, const uint32_t* __restrict__ mm,
                                                 int8_t* __restrict__ wp, float* __restrict__ s_w,
                                                 int32_t* __restrict__ z_w, int32_t* __restrict__ rowsum,
                                                 int* __restrict__ status) {
    const int lane = threadIdx.x & 63;
    if (n >= N) return;
    const float* src = w + (int64_t)n * K;
    float s;
    int z = 0;
    if (SYM) {
        float amax = 0.0f;
        int bad = 0;
        for (int k = lane; k < K; k += 64) {
            float a = fabsf(src[k]);
            bad |= !(a <= FLT_MAX);
            amax = fmaxf(amax, a);
        }
        amax = wave_max(amax);
        bad = wave_or_i32(bad);
        s = amax / (float)qw;
        if (amax == 0.0f) s = 1.0f;
        if (bad && lane == 0) atomicOr(status, kStatNonFinite);
    } else {
        asym_qparams(__uint_as_float(mm[0]), __uint_as_float(mm[1]), qdenom, qmax, s, z);
        if (mm[2] && lane == 0) atomicOr(status, kStatNonFinite);
    }
    int8_t* tile_row = wp + ((int64_t)(n >> 5) * KS * 64 + (n & 31)) * 16;
    int sum = 0;
    const QuantScale qs = make_quant_scale(s);
    for (int k = lane; k < K; k += 64) {
        int q = SYM ? quant_code(src[k], qs, -qw, qw) : quant_code(src[k], qs, -z, qmax - z) + z - 128;
        sum += q;
        tile_row[((int64_t)(k >> 5) * 64 + 32 * ((k & 31) >> 4)) * 16 + (k & 15)] = (int8_t)q;
    }
    sum = wave_sum_i32(sum);
    if (lane == 0) {
        s_w[n] = s;
        z_w[n] = z;
        rowsum[n] = sum;
    }
}

// packed signed-domain weights -> canonical codes (the inverse permutation), for export
__global__ void k_unpack_weights(const int8_t* __restrict__ wp, int N, int K, int KS, int asym,
                                 uint8_t* __restrict__ codes) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)N * K) return;
    int n = (int)(i / K), k = (int)(i % K);
    int8_t v = wp[(((int64_t)(n >> 5) * KS + (k >> 5)) * 64 + (n & 31) + 32 * ((k & 31) >> 4)) * 16 + (k & 15)];
    codes[i] = asym ? (uint8_t)((int)v + 128) : (uint8_t)v;
}

// ---------------------------------------------------------------------------------------------
// activation (scale, zero-point) from the supplied ranges: the same formula as for weights,
// the range being extended to contain zero.
// ---------------------------------------------------------------------------------------------
// One small launch opens a quantize pass: it also clears the status word and the per-layer range
// words, and presets the short-form flags (1 for requantized layers; a channel that does not
// qualify clears its layer's flag later).
__global__ void k_qp_prep(const QTab* __restrict__ tab, RangesArg r, ActQ* __restrict__ actq, int* __restrict__ fast,
                          int* __restrict__ status, uint32_t* __restrict__ mm) {
    const int i = threadIdx.x;
    const int nl = tab->n_layers;
    if (i == 63) *status = 0;
    if (i < 4 * AQ_MAX_LAYERS) mm[i] = 0u;
    if (i >= 32 && i < 32 + nl) fast[i - 32] = tab->L[i - 32].requant;
    if (i >= nl) return;
    if (i == 0 && tab->in_u8) {
        actq[0].s = 1.0f;
        actq[0].z = 0;
        return;
    }
    float hi = r.hi[i] > 0.0f ? r.hi[i] : 0.0f;
    float nlo = -r.lo[i] > 0.0f ? -r.lo[i] : 0.0f;
    float s;
    int z;
    asym_qparams(hi, nlo, tab->qdenom, 255, s, z);  // activations stay at 8 bits
    actq[i].s = s;
    actq[i].z = z;
}

// ---------------------------------------------------------------------------------------------
// per-channel layer constants (one thread per output channel):
//   m[n]      = s_in * s_w[n]                                   (fp32)
//   bias_q[n] = round(b[n] / (s_in * s_w[n]))                   (fp64, saturated)
//   M[n]      = s_in * s_w[n] / s_out = f * 2^e, f in [0.5,1);  M0 = round(f * 2^31), r = 31 - e
//   bias_fold = bias_q + zero-point terms of the signed-domain product:
//       sum_k (a_u - z_a)(w_u - z_w) = sum_k a_s w_s - z_a' sum_k w_s - z_w' sum_k a_s + K z_a' z_w'
//   with a_s = a_u - 128, z_a' = z_a - 128, and for unsigned weight codes w_s = w_u - 128,
//   z_w' = z_w - 128 (symmetric codes: w_s = w, z_w' = 0).  The "- z_w' sum_k a_s" term depends on
//   the batch row and is applied inside the forward kernel.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void layer_consts_channel(const ActQ* __restrict__ actq, int layer, int requant, int asym,
                                                     const float* __restrict__ s_w, const int32_t* __restrict__ z_w,
                                                     const float* __restrict__ bias, const int32_t* __restrict__ rowsum,
                                                     int n, int K, float* __restrict__ m, int32_t* __restrict__ bias_q,
                                                     int32_t* __restrict__ M0, int32_t* __restrict__ rshift,
                                                     int32_t* __restrict__ bias_fold, int32_t* __restrict__ pack1,
                                                     int32_t* __restrict__ rz, int32_t* __restrict__ sh,
                                                     int* __restrict__ fast, int* __restrict__ status) {
    const float s_in = actq[layer].s;
    const int z_a = actq[layer].z;
    m[n] = s_in * s_w[n];
    double sw = (double)s_in * (double)s_w[n];
    double bq = rint((double)(bias ? bias[n] : 0.0f) / sw);
    if (!(bq >= -2147483647.0)) bq = -2147483647.0;
    if (bq > 2147483647.0) bq = 2147483647.0;
    int32_t bqi = (int32_t)bq;
    bias_q[n] = bqi;
    if (requant) {
        double M = sw / (double)actq[layer + 1].s;
        int e;
        double f = frexp(M, &e);
        long long q = llround(f * 2147483648.0);
        if (q == 2147483648LL) {
            q = 1073741824LL;
            e += 1;
        }
        int r = 31 - e;
        if (r < 1 || r > 62 || !(M > 0.0) || !(M <= DBL_MAX)) {
            atomicOr(status, kStatRange);
            q = 0;
            r = 1;
        }
        M0[n] = (int32_t)q;
        pack1[n] = (int32_t)q;
        rshift[n] = r;
        // Short form of the same requantization for 33 <= r <= 54: the rounding constant 2^(r-1) has a
        // zero low word, so (acc*M0 + 2^(r-1)) >> r = (mulhi(acc, M0) + 2^(r-33)) >> (r-32), and the
        // output zero-point can ride along as z_out << (r-32).  One layer-wide flag says whether every
        // channel qualifies.
        if (r >= 33 && r <= 54) {
            sh[n] = r - 32;
            rz[n] = (1 << (r - 33)) + (actq[layer + 1].z << (r - 32));
        } else {
            sh[n] = 0;
            rz[n] = 0;
            atomicAnd(fast, 0);
        }
    } else {
        M0[n] = 0;
        rshift[n] = 0;
        pack1[n] = __float_as_int(s_in * s_w[n]);
    }
    const int za_s = z_a - 128;
    const int zw_s = asym ? z_w[n] - 128 : 0;
    // (a saturated integer bias can push the folded value out of the accumulator's range: reported, like a
    // multiplier outside the shift range, instead of wrapping silently)
    const long long bf = (long long)bqi - (long long)za_s * rowsum[n] + (long long)K * za_s * zw_s;
    if (bf > 2147483647LL || bf < -2147483648LL) atomicOr(status, kStatRange);
    bias_fold[n] = (int32_t)bf;
}

// ---------------------------------------------------------------------------------------------
// The whole policy in three or four launches: each grid covers every layer, a workgroup finds its
// layer from the table's first-workgroup indices (at most 8 compares).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int layer_of_block(const QTab& t, int blk, int which) {
    int l = t.n_layers - 1;
    while (l > 0 && blk < (which == 0 ? t.L[l].row_blk0 : which == 1 ? t.L[l].cst_blk0 : t.L[l].rng_blk0)) --l;
    return l;
}

__global__ __launch_bounds__(256) void k_qp_ranges(const QTab* __restrict__ tab, const QPtrs p, uint32_t* __restrict__ mm) {
    const QTab& t = *tab;
    const int l = layer_of_block(t, blockIdx.x, 2);
    const QLayerTab& L = t.L[l];
    const int64_t n = (int64_t)L.N * L.K;
    range_nonneg_block((const float4*)p.w[l], n / 4, p.w[l], n, mm + 4 * l, blockIdx.x - L.rng_blk0, L.rng_blks);
}

template <bool SYM>
__global__ __launch_bounds__(256) void k_qp_rows(const QTab* __restrict__ tab, const QPtrs p,
                                                 const uint32_t* __restrict__ mm, int* __restrict__ status) {
    const QTab& t = *tab;
    const int l = layer_of_block(t, blockIdx.x, 0);
    const QLayerTab& L = t.L[l];
    const int n = (blockIdx.x - L.row_blk0) * 4 + (threadIdx.x >> 6);
    quant_row_packed<SYM>(p.w[l], n, L.N, L.K, L.KS, t.w_qdenom, t.w_qmax, t.w_qw, mm + 4 * l, L.wp, L.s_w, L.z_w, L.rowsum, status);
}

__global__ __launch_bounds__(256) void k_qp_consts(const QTab* __restrict__ tab, const QPtrs p,
                                                   const ActQ* __restrict__ actq, int* __restrict__ fast,
                                                   int* __restrict__ status) {
    const QTab& t = *tab;
    const int l = layer_of_block(t, blockIdx.x, 1);
    const QLayerTab& L = t.L[l];
    const int n = (blockIdx.x - L.cst_blk0) * 256 + threadIdx.x;
    if (n >= L.N) return;
    layer_consts_channel(actq, l, L.requant, t.asym, L.s_w, L.z_w, p.b[l], L.rowsum, n, L.K, L.m, L.bias_q, L.M0,
                         L.rshift, L.bias_fold, L.pack1, L.rz, L.sh, fast + l, status);
    if (L.ln) {  // LayerNorm gain and offset (defaults 1 and 0) into their slots of the constant pack
        L.rz[n] = __float_as_int(p.gamma[l] ? p.gamma[l][n] : 1.0f);
        L.sh[n] = __float_as_int(p.beta[l] ? p.beta[l][n] : 0.0f);
    }
}

// ---------------------------------------------------------------------------------------------
// policy blob header: six words written / compared by one small launch (the expected words travel
// as kernel arguments, so neither call needs a host round trip)
// ---------------------------------------------------------------------------------------------
struct BlobWords {
    uint32_t w[6];
};
__global__ void k_blob_header_write(uint32_t* __restrict__ hdr, const BlobWords b) {
    // the 16 header words, and zeros over the 32 words behind them (the tail's padding; its
    // contents are copied in afterwards)
    const int i = threadIdx.x;
    if (i < 48) hdr[i] = i < 6 ? b.w[i] : 0u;
}
__global__ void k_blob_header_check(const uint32_t* __restrict__ hdr, const BlobWords b, int* __restrict__ status) {
    const int i = threadIdx.x;
    if (i < 6 && hdr[i] != b.w[i]) atomicOr(status, kStatBlob);
}

// ---------------------------------------------------------------------------------------------
// n-bit weight codes stored sub-byte (the packed policy blob): eight consecutive codes of the operand
// order -> n bytes and back.  Codes are kept in the signed domain in the library (symmetric: the code
// itself, in [-qw, qw]; per tensor: unsigned code - 128), the stored field is the code plus `off`
// (qw resp. 128), an n-bit unsigned number.  Padding entries (feature >= N or k >= K) are zero in the
// signed domain, which the per-tensor scheme cannot store in n < 8 bits: they are written as field 0
// and restored from their position when unpacking.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pack_bits(const int8_t* __restrict__ wp, uint8_t* __restrict__ out,
                                                   int64_t groups, int bits, int off) {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= groups) return;
    const uint64_t v = *(const uint64_t*)(wp + 8 * g);
    const int fmax = (1 << bits) - 1;
    uint64_t acc = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int u = (int)(int8_t)(v >> (8 * j)) + off;
        u = u < 0 ? 0 : (u > fmax ? 0 : u);
        acc |= (uint64_t)u << (j * bits);
    }
    uint8_t* dst = out + g * bits;
    for (int b = 0; b < bits; ++b) dst[b] = (uint8_t)(acc >> (8 * b));
}

__global__ __launch_bounds__(256) void k_unpack_bits(const uint8_t* __restrict__ in, int8_t* __restrict__ wp,
                                                     int64_t groups, int bits, int off, int N, int K, int KS) {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= groups) return;
    const uint8_t* src = in + g * bits;
    uint64_t acc = 0;
    for (int b = 0; b < bits; ++b) acc |= (uint64_t)src[b] << (8 * b);
    // position of the group's first element in the operand order: tile (n / 32, k / 32) = 1 KiB,
    // lane = n % 32 + 32 * ((k % 32) / 16), byte = k % 16
    const int64_t e = 8 * g;
    const int64_t tile = e >> 10;
    const int nt = (int)(tile / KS), ks = (int)(tile - (int64_t)nt * KS);
    const int lane = (int)((e & 1023) >> 4), byte0 = (int)(e & 15);
    const int n = nt * 32 + (lane & 31), k0 = ks * 32 + 16 * (lane >> 5) + byte0;
    const uint64_t fmask = ((uint64_t)1 << bits) - 1;
    uint64_t v = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int sgn = (int)((acc >> (j * bits)) & fmask) - off;
        if (n >= N || k0 + j >= K) sgn = 0;
        v |= (uint64_t)(uint8_t)(int8_t)sgn << (8 * j);
    }
    *(uint64_t*)(wp + 8 * g) = v;
}

// ---------------------------------------------------------------------------------------------
// Measurement aid: the memory traffic of the flat quantize pass without its arithmetic (4 bytes read and
// 1 byte written per element, no reduction, no dependence between the loads and the stores of a thread
// other than the data itself).  What this kernel reaches at a given size is the ceiling for the quantizer
// at that size.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_stream_reference(const float4* __restrict__ in4, int64_t n4,
                                                          uint32_t* __restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += 2 * stride) {
        const f4v a = __builtin_nontemporal_load((const f4v*)in4 + i);
        const bool two = i + stride < n4;
        f4v b = a;
        if (two) b = __builtin_nontemporal_load((const f4v*)in4 + i + stride);
        __builtin_nontemporal_store((__float_as_uint(a[0]) >> 24) | ((__float_as_uint(a[1]) >> 24) << 8) |
                                        ((__float_as_uint(a[2]) >> 24) << 16) | ((__float_as_uint(a[3]) >> 24) << 24),
                                    out + i);
        if (two)
            __builtin_nontemporal_store((__float_as_uint(b[0]) >> 24) | ((__float_as_uint(b[1]) >> 24) << 8) |
                                            ((__float_as_uint(b[2]) >> 24) << 16) | ((__float_as_uint(b[3]) >> 24) << 24),
                                        out + i + stride);
    }
}

aq_status launch_stream_reference(const float* d_in, int64_t n, void* d_out, hipStream_t st) {
    const int64_t n4 = n / 4;
    int64_t g = (n4 + 511) / 512;  // two 16-byte pieces per thread, like the per-channel kernel on 2048-wide rows
    if (g > 65536) g = 65536;
    hipLaunchKernelGGL(k_stream_reference, dim3((unsigned)g), dim3(256), 0, st, (const float4*)d_in, n4, (uint32_t*)d_out);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

// ---------------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------------
aq_status launch_pack_bits(const int8_t* wp, uint8_t* out, int64_t n_codes, int bits, int off, hipStream_t st) {
    const int64_t groups = n_codes / 8;
    hipLaunchKernelGGL(k_pack_bits, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, wp, out, groups, bits, off);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}
aq_status launch_unpack_bits(const uint8_t* in, int8_t* wp, int64_t n_codes, int bits, int off, int N, int K, int KS,
                             hipStream_t st) {
    const int64_t groups = n_codes / 8;
    hipLaunchKernelGGL(k_unpack_bits, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, in, wp, groups, bits, off,
                       N, K, KS);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_blob_header_write(uint32_t* d_hdr, const uint32_t* h_words, hipStream_t st) {
    BlobWords b;
    for (int i = 0; i < 6; ++i) b.w[i] = h_words[i];
    hipLaunchKernelGGL(k_blob_header_write, dim3(1), dim3(64), 0, st, d_hdr, b);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}
aq_status launch_blob_header_check(const uint32_t* d_hdr, const uint32_t* h_words, int* status, hipStream_t st) {
    BlobWords b;
    for (int i = 0; i < 6; ++i) b.w[i] = h_words[i];
    hipLaunchKernelGGL(k_blob_header_check, dim3(1), dim3(64), 0, st, d_hdr, b, status);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

static int grid_for(int64_t work_items, int per_block, int cap) {
    int64_t g = (work_items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

aq_status launch_fill_u32(uint32_t* p, int n, uint32_t v, hipStream_t st) {
    hipLaunchKernelGGL(k_fill_u32, dim3((n + 255) / 256), dim3(256), 0, st, p, n, v);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_quantize_tensor(const float* d_w, int64_t rows, int64_t cols, int wscheme, float qdenom,
                                 int qmax, int qw, void* d_codes, float* d_scale, int32_t* d_zp, uint32_t* d_ws, hipStream_t st) {
    const int64_t n = rows * cols;
    const float4* w4 = (const float4*)d_w;
    uint32_t* c4 = (uint32_t*)d_codes;
    if (wscheme == AQ_W_TENSOR_ASYM_U8) {
        const int64_t n4 = n / 4;
        // enough workgroups to keep every CU's memory pipeline full; partial ranges go to d_ws[16..]
        const int g1 = grid_for(n4, 256 * 4, 1024);
        hipLaunchKernelGGL(k_range_partials, dim3(g1), dim3(256), 0, st, w4, n4, d_ws + 16);
        const int g2 = grid_for(n4, 256 * 4, 2048);
        hipLaunchKernelGGL(k_quant_asym_flat, dim3(g2), dim3(256), 0, st, w4, n4, d_ws + 16, g1, qdenom, qmax, c4, d_scale,
                           d_zp, d_ws + 2);
    } else {
        const int cols4 = (int)(cols / 4);
        if (cols4 <= 64) {
            hipLaunchKernelGGL(k_quant_sym_rows_flat<1>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, w4, rows,
                               cols4, qw, c4, d_scale, d_zp, d_ws);
        } else {
#define AQ_ROW_WG(R) \
    hipLaunchKernelGGL(k_quant_sym_row_wg<R>, dim3((unsigned)rows), dim3(256), 0, st, w4, cols4, qw, c4, d_scale, d_zp, d_ws)
            if (cols4 <= 256) AQ_ROW_WG(1);
            else if (cols4 <= 512) AQ_ROW_WG(2);
            else if (cols4 <= 1024) AQ_ROW_WG(4);
            else if (cols4 <= 2048) AQ_ROW_WG(8);
            else
                hipLaunchKernelGGL(k_quant_sym_rows_long, dim3((unsigned)rows), dim3(256), 0, st, w4, rows, cols4, qw, c4,
                                   d_scale, d_zp, d_ws);
#undef AQ_ROW_WG
        }
    }
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_unpack_weights(const int8_t* wp, int N, int K, int KS, int asym, uint8_t* codes, hipStream_t st) {
    const int64_t n = (int64_t)N * K;
    hipLaunchKernelGGL(k_unpack_weights, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, wp, N, K, KS, asym,
                       codes);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_quantize_policy(const QTab* d_tab, const QTab& h_tab, const QPtrs& ptrs, const RangesArg& r,
                                 ActQ* actq, int* fast, int* status, uint32_t* mm, hipStream_t st) {
    hipLaunchKernelGGL(k_qp_prep, dim3(1), dim3(64), 0, st, d_tab, r, actq, fast, status, mm);
    if (h_tab.asym) {
        hipLaunchKernelGGL(k_qp_ranges, dim3(h_tab.rng_blks_total), dim3(256), 0, st, d_tab, ptrs, mm);
        hipLaunchKernelGGL(k_qp_rows<false>, dim3(h_tab.row_blks), dim3(256), 0, st, d_tab, ptrs, mm, status);
    } else {
        hipLaunchKernelGGL(k_qp_rows<true>, dim3(h_tab.row_blks), dim3(256), 0, st, d_tab, ptrs, mm, status);
    }
    hipLaunchKernelGGL(k_qp_consts, dim3(h_tab.cst_blks), dim3(256), 0, st, d_tab, ptrs, actq, fast, status);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
