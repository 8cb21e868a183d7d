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

constexpr int HW = 4;     // waves per workgroup
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

// tanh with relative error below 1e-6 (far inside half a binary16 spacing, 2.4e-4): odd polynomial
// near zero, where the exponential form would cancel, 1 - 2 / (e^{2|x|} + 1) elsewhere
__device__ __forceinline__ float tanh_rel(float x) {
    const float ax = fabsf(x);
    const float u = x * x;
    float p = 0.0035921280f;         // Taylor series of tanh(x) / x in u = x^2 up to u^6
    p = fmaf(p, u, -0.0088632355f);  // (remainder below 2e-7 relative at |x| = 0.5)
    p = fmaf(p, u, 0.0218694885f);
    p = fmaf(p, u, -0.0539682540f);
    p = fmaf(p, u, 0.1333333333f);
    p = fmaf(p, u, -0.3333333333f);
    const float small = fmaf(x * u, p, x);
    const float e = __builtin_amdgcn_exp2f(fminf(ax, 20.0f) * 2.885390081777927f);  // e^{2|x|}
    const float big = copysignf(fmaf(__builtin_amdgcn_rcpf(e + 1.0f), -2.0f, 1.0f), x);
    return ax < 0.5f ? small : big;
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
// PIECE: every run of 8 consecutive k starting at a multiple of 8 is contiguous in the input, whole
//        (K is a multiple of 8) and aligned for vector loads (16 bytes for binary16 and fp32, 4 for uint8)
// One workgroup = 4 waves = 32*MT rows x 128*NB features; a wave owns NB feature tiles and all MT row tiles.
// Operands are requested one chunk ahead: weights straight into registers in operand order, the
// activation chunk into registers and from there into the other LDS buffer after the chunk's MFMAs.
// Loads are unconditional from clamped addresses (a row past the end reads the last row, a piece
// past K reads piece 0) and the value is zeroed afterwards, so that no branch separates a load from
// its use.
// (compiled for two waves per SIMD: within 256 registers the accumulators stay in ordinary vector
// registers; with more the compiler parks them in accumulation registers and copies them back and
// forth around every chunk)
template <int MT, int NB, int IN, bool PIECE>
__global__ __launch_bounds__(256, 2) void k_layer_fp16(const Fp16Layer L, const void* __restrict__ in,
                                                    _Float16* __restrict__ out, const int64_t rows) {
    constexpr int ROWS = 32 * MT;
    constexpr int SW = NB * 32 + 8;  // row stride (halfs) of a wave's output staging tile
    constexpr int XBUF = ROWS * HLD;
    constexpr int XS = 2 * XBUF > HW * 32 * SW ? 2 * XBUF : HW * 32 * SW;
    __shared__ __align__(16) _Float16 xs[XS];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    const int nt0 = (blockIdx.y * HW + wave) * NB;  // this wave's first feature tile
    const bool wave_on = nt0 < L.NT;
    const int KC = L.KS16 / 4;  // chunks of 64

    // staging: thread -> rows (tid >> 3) + 32 j, k piece (tid & 7) * 8 of each chunk
    const int sr = tid >> 3, sk = (tid & 7) * 8;
    RowPos rp[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        const int64_t row = row0 + sr + 32 * j;
        rp[j] = row_pos(L, row < rows ? row : rows - 1, rows);
        rp[j].ok = row < rows;
    }

    auto load_x = [&](int c, h8 (&x)[MT]) __attribute__((always_inline)) {
        const int k0 = c * HKC + sk;
        if (PIECE) {
            const bool kok = k0 < L.K;
            const int64_t off = k_offset(L, kok ? k0 : 0);
            const h8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                h8 v;
                {
                    if (IN == 0) {
                        v = *(const h8*)((const _Float16*)in + rp[j].base + off);
                    } else if (IN == 1) {
                        const float4* s4 = (const float4*)((const float*)in + rp[j].base + off);
                        const float4 a = s4[0], b = s4[1];
                        v[0] = (_Float16)a.x; v[1] = (_Float16)a.y; v[2] = (_Float16)a.z; v[3] = (_Float16)a.w;
                        v[4] = (_Float16)b.x; v[5] = (_Float16)b.y; v[6] = (_Float16)b.z; v[7] = (_Float16)b.w;
                    } else {
                        const uint32_t* s1 = (const uint32_t*)((const uint8_t*)in + rp[j].base + off);
                        const uint32_t a = s1[0], b = s1[1];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            v[i] = (_Float16)(float)((a >> (8 * i)) & 0xffu);
                            v[4 + i] = (_Float16)(float)((b >> (8 * i)) & 0xffu);
                        }
                    }
                }
                x[j] = (rp[j].ok && kok) ? v : z;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = k0 + i;
                const bool kok = k < L.K;
                const int64_t off = k_offset(L, kok ? k : 0);
#pragma unroll
                for (int j = 0; j < MT; ++j) {
                    _Float16 a;
                    if (IN == 0) a = ((const _Float16*)in)[rp[j].base + off];
                    else if (IN == 1) a = (_Float16)((const float*)in)[rp[j].base + off];
                    else a = (_Float16)(float)((const uint8_t*)in)[rp[j].base + off];
                    x[j][i] = (kok && rp[j].ok) ? a : (_Float16)0.0f;
                }
            }
        }
    };
    auto store_x = [&](int buf, const h8 (&x)[MT]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < MT; ++j) *(h8*)&xs[buf * XBUF + (sr + 32 * j) * HLD + sk] = x[j];
    };
    // this wave's weights of one chunk: 4 k-steps x NB tiles, 16 bytes per lane each
    const h8* wbase = (const h8*)L.wp + lane;
    auto load_w = [&](int c, h8 (&wr)[4][NB]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int nt = nt0 + nb < L.NT ? nt0 + nb : L.NT - 1;  // (clamped: the tile is not stored)
                wr[s][nb] = wbase[((int64_t)nt * L.KS16 + c * 4 + s) * 64];
            }
    };

    f16acc acc[NB][MT];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[nb][mt][i] = 0.0f;

    h8 wc[4][NB], wn[4][NB];  // weights of chunks c, c + 1
    h8 xn[MT];                 // activations of chunk c + 1
    auto compute = [&](int buf, const h8 (&w)[4][NB]) __attribute__((always_inline)) {
        const _Float16* xb = xs + buf * XBUF;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            h8 bx[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                bx[mt] = *(const h8*)&xb[(mt * 32 + (lane & 31)) * HLD + s * 16 + 8 * (lane >> 5)];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[nb][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w[s][nb], bx[mt], acc[nb][mt], 0, 0, 0);
        }
    };
    if (MT < 4 && KC <= 2) {  // (the 128-row tile has no registers for it and never meets a short K)
        // short K (first layers: 17 or 67 observation features): everything is requested at once and both
        // LDS buffers are filled before the only barrier
        h8 x1[MT];
        load_w(0, wc);
        load_w(KC - 1, wn);
        load_x(0, xn);
        load_x(KC - 1, x1);
        store_x(0, xn);
        store_x(1, x1);
        __syncthreads();
        if (wave_on) {
            compute(0, wc);
            if (KC == 2) compute(1, wn);
        }
        __syncthreads();  // the epilogue reuses the buffers
    } else {
        load_w(0, wc);
        load_x(0, xn);
        store_x(0, xn);
        __syncthreads();
        for (int c = 0; c < KC; ++c) {
            const bool more = c + 1 < KC;
            {
                const int cn = more ? c + 1 : c;  // (clamped: loaded again, not used)
                load_w(cn, wn);
                load_x(cn, xn);
            }
            if (wave_on) compute(c & 1, wc);
            if (more) store_x((c + 1) & 1, xn);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) wc[s][nb] = wn[s][nb];
            __syncthreads();
        }
    }
    if (!wave_on) return;

    // epilogue: + bias, rounded to binary16 once, ReLU; lane = one row, four consecutive features per quad.
    // An elementwise action head (tanh / identity) is applied to the rounded value in the same sweep.
    auto quad_out = [&](int nb, int mt, int q, int n0) __attribute__((always_inline)) {
        const float4 bv = *(const float4*)(L.bias + n0);  // padded to the tile
        const float b4[4] = {bv.x, bv.y, bv.z, bv.w};
        h4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            _Float16 v = (_Float16)(acc[nb][mt][4 * q + i] + b4[i]);
            if (L.relu) v = v > (_Float16)0.0f ? v : (_Float16)0.0f;
            o[i] = v;
        }
        return o;
    };
    if ((L.N & 7) == 0) {
        // Rows of 16-byte pieces: each tile goes through a wave-private LDS region (the activation
        // buffers are idle after the last barrier) and leaves as whole contiguous runs of an output row,
        // NB * 64 bytes per row and wave, instead of 8 bytes per lane 2 * N bytes apart.
        _Float16* wsp = xs + wave * (32 * SW);
        constexpr int LPR = NB * 4;      // lanes per row on the way out
        constexpr int RPI = 64 / LPR;    // rows per store instruction
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n0 = (nt0 + nb) * 32 + 8 * q + 4 * (lane >> 5);
                    h4 o = {0, 0, 0, 0};
                    if (nt0 + nb < L.NT) o = quad_out(nb, mt, q, n0);
                    *(h4*)&wsp[(lane & 31) * SW + nb * 32 + 8 * q + 4 * (lane >> 5)] = o;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < 32 / RPI; ++j) {
                const int r = j * RPI + lane / LPR, pc = lane % LPR;
                const h8 v = *(const h8*)&wsp[r * SW + pc * 8];
                const int64_t row = row0 + mt * 32 + r;
                const int n = nt0 * 32 + pc * 8;
                if (row < rows && n < L.N) {
                    *(h8*)(out + row * L.N + n) = v;
                    if (L.head_actions) {
                        float a8[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            a8[i] = L.head_tanh ? (float)(_Float16)tanh_rel((float)v[i]) : (float)v[i];
                        float4* ad = (float4*)(L.head_actions + row * L.N + n);
                        ad[0] = make_float4(a8[0], a8[1], a8[2], a8[3]);
                        ad[1] = make_float4(a8[4], a8[5], a8[6], a8[7]);
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }
    const bool vec_out = (L.N & 3) == 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (nt0 + nb >= L.NT) continue;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int64_t row = row0 + mt * 32 + (lane & 31);
            if (row >= rows) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n0 = (nt0 + nb) * 32 + 8 * q + 4 * (lane >> 5);
                if (n0 >= L.N) continue;
                const h4 o = quad_out(nb, mt, q, n0);
                _Float16* dst = out + row * L.N + n0;
                if (vec_out) {
                    *(h4*)dst = o;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n0 + i < L.N) dst[i] = o[i];
                }
                if (L.head_actions) {
                    float* ad = L.head_actions + row * L.N + n0;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n0 + i < L.N)
                            ad[i] = L.head_tanh ? (float)(_Float16)tanh_rel((float)o[i]) : (float)o[i];
                }
            }
        }
    }
}

// Fully connected hidden layer at few rows (the paper's actors run one observation at a time, Sec. 3.1,
// on layers of 2048 units, Sec. 4.1): the time goes into streaming the binary16 weights once, so one
// workgroup of 8 waves owns a single 32-row x 32-feature output tile and its waves split K.  Both MFMA
// operands come straight from global memory, 16 bytes per lane and k-step (the activation rows are a
// few KB and stay in cache), SKH_PF k-steps of each in flight; partial tiles meet in LDS, then the 512
// threads reduce eight partial sums for two outputs each, add the bias, round once and store.
constexpr int SKH_W = 8;
constexpr int SKH_PF = 8;
constexpr int SKH_LD = 65;  // words per register row of a partial tile (conflict-free feature-major reads)

__global__ __launch_bounds__(SKH_W * 64) void k_layer_fp16_skinny(const Fp16Layer L, const _Float16* __restrict__ in,
                                                                   _Float16* __restrict__ out, const int64_t rows) {
    __shared__ float part[SKH_W * 16 * SKH_LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = blockIdx.x;
    const int64_t row0 = (int64_t)blockIdx.y * 32;
    const int KSr = (L.K + 15) / 16;                  // k-steps that hold real columns
    const int kc = (KSr + SKH_W - 1) / SKH_W;
    const int k0 = wave * kc, k1 = k0 + kc < KSr ? k0 + kc : KSr;
    const int64_t xrow = row0 + (lane & 31) < rows ? row0 + (lane & 31) : rows - 1;  // (clamped, zeroed below)
    const bool row_ok = row0 + (lane & 31) < rows;
    const h8* wsrc = (const h8*)L.wp + (int64_t)nt * L.KS16 * 64 + lane;
    const _Float16* xsrc = in + xrow * L.K + 8 * (lane >> 5);
    const h8 z8 = {0, 0, 0, 0, 0, 0, 0, 0};
    f16acc acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    for (int g0 = k0; g0 < k1; g0 += SKH_PF) {
        h8 a[SKH_PF], b[SKH_PF];
#pragma unroll
        for (int u = 0; u < SKH_PF; ++u) {
            const int ks = g0 + u < k1 ? g0 + u : k1 - 1;
            a[u] = wsrc[(int64_t)ks * 64];
            // K is a multiple of 8: a piece of 8 columns is whole or lies entirely in the zero padding
            const int kcol = ks * 16 + 8 * (lane >> 5);
            b[u] = *(const h8*)(xsrc + (kcol < L.K ? ks * 16 : 0));
            if (!(row_ok && kcol < L.K && g0 + u < k1)) b[u] = z8;
        }
#pragma unroll
        for (int u = 0; u < SKH_PF; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[u], b[u], acc, 0, 0, 0);
    }
    {
        float* mine = part + wave * 16 * SKH_LD + lane;
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[r * SKH_LD] = acc[r];
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int m = (tid >> 5) + 16 * it, nl = tid & 31;
        // accumulator register and lane that hold (feature nl, row m) of the tile
        const int reg = 4 * (nl >> 3) + (nl & 3), lsrc = m + 32 * ((nl >> 2) & 1);
        float v = 0.0f;
#pragma unroll
        for (int kp = 0; kp < SKH_W; ++kp) v += part[kp * 16 * SKH_LD + reg * SKH_LD + lsrc];
        const int n = nt * 32 + nl;
        const int64_t row = row0 + m;
        const bool ok = row < rows && n < L.N;
        _Float16 o = (_Float16)(v + L.bias[n]);  // (bias is padded to the tile)
        if (L.relu) o = o > (_Float16)0.0f ? o : (_Float16)0.0f;
        if (ok) {
            out[row * L.N + n] = o;
            if (L.head_actions)
                L.head_actions[row * L.N + n] = L.head_tanh ? (float)(_Float16)tanh_rel((float)o) : (float)o;
        }
        if (L.head_argmax) {
            // the whole output row sits in this tile, one feature per lane of a 32-lane group: the action
            // index (lowest index among equal values) is a shuffle reduction away
            float y = ok ? (float)o : -INFINITY;
            int best = n;
#pragma unroll
            for (int d = 16; d > 0; d >>= 1) {
                const float yo = __shfl_xor(y, d, 32);
                const int bo = __shfl_xor(best, d, 32);
                if (yo > y || (yo == y && bo < best)) {
                    y = yo;
                    best = bo;
                }
            }
            if (nl == 0 && row < rows) L.head_argmax[row] = best;
        }
    }
}

// LayerNorm (biased variance, eps inside the root) rounded to binary16, then tanh rounded to binary16,
// in place.  One wavefront per LN_R rows, the rows in registers between the statistics and the result,
// all of a wave's loads requested before the first is used (8-byte pieces when N is a multiple of 4).
constexpr int LN_R = 4;     // rows per wavefront
constexpr int LN_MAXV = 16; // elements per lane and row held in registers (N <= 1024)
template <bool VEC4>
__global__ __launch_bounds__(256) void k_fp16_ln_tanh(_Float16* __restrict__ x, int64_t rows, int N,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t r0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * LN_R;
    if (r0 >= rows) return;
    float v[LN_R][LN_MAXV];
    // element index of register i: VEC4: 4 * lane + 256 * (i / 4) + i % 4, else lane + 64 * i
#pragma unroll
    for (int r = 0; r < LN_R; ++r) {
        const int64_t row = r0 + r < rows ? r0 + r : rows - 1;
        const _Float16* xr = x + row * N;
        if (VEC4) {
#pragma unroll
            for (int i = 0; i < LN_MAXV / 4; ++i) {
                const int n = 4 * lane + 256 * i;
                h4 t = {0, 0, 0, 0};
                if (n < N) t = *(const h4*)(xr + n);
#pragma unroll
                for (int j = 0; j < 4; ++j) v[r][4 * i + j] = (float)t[j];
            }
        } else {
#pragma unroll
            for (int i = 0; i < LN_MAXV; ++i) {
                const int n = lane + 64 * i;
                v[r][i] = n < N ? (float)xr[n] : 0.0f;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < LN_R; ++r) {
        if (r0 + r >= rows) break;
        _Float16* xr = x + (r0 + r) * N;
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < LN_MAXV; ++i) s += v[r][i];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        const float mean = s / (float)N;
        float ss = 0.0f;
#pragma unroll
        for (int i = 0; i < LN_MAXV; ++i) {
            const int n = VEC4 ? 4 * lane + 256 * (i / 4) + i % 4 : lane + 64 * i;
            const float d = n < N ? v[r][i] - mean : 0.0f;
            ss += d * d;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        const float inv = 1.0f / sqrtf(ss / (float)N + eps);
        if (VEC4) {
#pragma unroll
            for (int i = 0; i < LN_MAXV / 4; ++i) {
                const int n = 4 * lane + 256 * i;
                if (n < N) {
                    const float4 g4 = *(const float4*)(gamma + n), b4 = *(const float4*)(beta + n);
                    const float gg[4] = {g4.x, g4.y, g4.z, g4.w}, bb[4] = {b4.x, b4.y, b4.z, b4.w};
                    h4 o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const _Float16 ln = (_Float16)((v[r][4 * i + j] - mean) * inv * gg[j] + bb[j]);
                        o[j] = (_Float16)tanh_rel((float)ln);
                    }
                    *(h4*)(xr + n) = o;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < LN_MAXV; ++i) {
                const int n = lane + 64 * i;
                if (n < N) {
                    const _Float16 ln = (_Float16)((v[r][i] - mean) * inv * gamma[n] + beta[n]);
                    xr[n] = (_Float16)tanh_rel((float)ln);
                }
            }
        }
    }
}

// rows wider than 64 * LN_MAXV: one wavefront per row, the row is read three times
__global__ __launch_bounds__(256) void k_fp16_ln_tanh_long(_Float16* __restrict__ x, int64_t rows, int N,
                                                           const float* __restrict__ gamma,
                                                           const float* __restrict__ beta, float eps) {
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
        xr[n] = (_Float16)tanh_rel((float)ln);
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
        ((float*)actions)[i] = head == AQ_HEAD_TANH ? (float)(_Float16)tanh_rel(v) : v;
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

namespace {
template <int MT, int NB>
void launch_layer_cfg(const Fp16Layer& L, const void* in, int in_mode, bool piece, _Float16* o, int64_t rows,
                      hipStream_t st) {
    const dim3 grid((unsigned)((rows + 32 * MT - 1) / (32 * MT)), (unsigned)((L.NT + HW * NB - 1) / (HW * NB)));
#define AQ_F16_GO(IN, PC) hipLaunchKernelGGL((k_layer_fp16<MT, NB, IN, PC>), grid, dim3(256), 0, st, L, in, o, rows)
    if constexpr (MT == 4) {  // (the 128-row tile serves hidden layers only)
        if (piece) AQ_F16_GO(0, true);
        else AQ_F16_GO(0, false);
    } else {
        if (in_mode == 0) {
            if (piece) AQ_F16_GO(0, true);
            else AQ_F16_GO(0, false);
        } else if (in_mode == 1) {
            if (piece) AQ_F16_GO(1, true);
            else AQ_F16_GO(1, false);
        } else {
            if (piece) AQ_F16_GO(2, true);
            else AQ_F16_GO(2, false);
        }
    }
#undef AQ_F16_GO
}
}  // namespace

bool fp16_layer_is_skinny(const Fp16Layer& L, const void* in, int in_mode, int64_t rows) {
    const int64_t tiled_wgs = ((rows + 31) / 32) * (int64_t)((L.NT + HW - 1) / HW);
    return in_mode == 0 && L.fc && L.K % 8 == 0 && ((uintptr_t)in & 15) == 0 && L.K >= 128 && tiled_wgs < 128 &&
           (rows + 31) / 32 <= 65535;
}

aq_status launch_layer_fp16(const Fp16Layer& L, const void* in, int in_mode, void* out, int64_t rows,
                            hipStream_t st) {
    if (rows < 1) return AQ_OK;
    if (L.KS16 % 4 != 0 || L.NT < 1) return AQ_ESHAPE;
    _Float16* o = (_Float16*)out;
    // whole aligned pieces of 8 consecutive k: runs of consecutive k are multiples of 8 long, and every
    // run starts at an element offset that is a multiple of 8 (binary16: 16 bytes) or 4 (fp32: 16 bytes,
    // uint8: 4 bytes)
    const int unit = in_mode == 0 ? 8 : 4;
    const bool piece = ((uintptr_t)in & 15) == 0 &&
                       (L.fc ? L.K % 8 == 0 : ((L.kw * L.in_c) % 8 == 0 && L.in_c % unit == 0));
    // Tile: 128 rows x 256 features (hidden layers: the conversion of an fp32 observation piece does not
    // fit the register budget beside 128 accumulators) when that still gives every CU two workgroups,
    // 64 x 256 when it gives one, else 32 x 128 (few rows or few features: as many workgroups as possible).
    auto wgs = [&](int mt, int nb) {
        return ((rows + 32 * mt - 1) / (32 * mt)) * (int64_t)((L.NT + HW * nb - 1) / (HW * nb));
    };
    // few rows: one workgroup per output tile with K split over its waves, whenever the tiled kernel would
    // leave most CUs without a workgroup (binary16 rows of whole, aligned 16-byte pieces)
    if (fp16_layer_is_skinny(L, in, in_mode, rows)) {
        const dim3 grid((unsigned)L.NT, (unsigned)((rows + 31) / 32));
        hipLaunchKernelGGL(k_layer_fp16_skinny, grid, dim3(SKH_W * 64), 0, st, L, (const _Float16*)in, o, rows);
        return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
    }
    if (in_mode == 0 && L.NT > HW && wgs(4, 2) >= 512) launch_layer_cfg<4, 2>(L, in, in_mode, piece, o, rows, st);
    else if (in_mode == 0 && L.NT > HW && wgs(2, 2) >= 256) launch_layer_cfg<2, 2>(L, in, in_mode, piece, o, rows, st);
    else launch_layer_cfg<1, 1>(L, in, in_mode, piece, o, rows, st);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp16_ln_tanh(void* x, int64_t rows, int N, const float* gamma, const float* beta, float eps,
                              hipStream_t st) {
    if (rows < 1) return AQ_OK;
    _Float16* xh = (_Float16*)x;
    if (N > 64 * LN_MAXV) {
        hipLaunchKernelGGL(k_fp16_ln_tanh_long, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, xh, rows, N, gamma,
                           beta, eps);
    } else {
        const dim3 grid((unsigned)((rows + 4 * LN_R - 1) / (4 * LN_R)));
        if (N % 4 == 0 && ((uintptr_t)x & 7) == 0)
            hipLaunchKernelGGL(k_fp16_ln_tanh<true>, grid, dim3(256), 0, st, xh, rows, N, gamma, beta, eps);
        else
            hipLaunchKernelGGL(k_fp16_ln_tanh<false>, grid, dim3(256), 0, st, xh, rows, N, gamma, beta, eps);
    }
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

aq_status launch_fp16_head(const void* y, int64_t rows, int N, int head, void* actions, hipStream_t st) {
    const int64_t n = head == AQ_HEAD_ARGMAX ? rows : rows * N;
    hipLaunchKernelGGL(k_fp16_head, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const _Float16*)y, rows, N,
                       head, actions);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
