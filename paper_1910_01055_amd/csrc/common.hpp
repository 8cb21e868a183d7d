// Shared device/host declarations of the ActorQ HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "actorq.h"

namespace aq {

constexpr int kWave = 64;
constexpr int kTile = 32;  // MFMA tile edge (features and batch rows); one k-step is 32 bytes

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
// Pointers that are known to address global memory.  A pointer read back from LDS is a generic
// ("flat") pointer to the compiler; flat loads are tracked by both memory counters and cannot be
// kept in flight selectively, so every prefetch through them would serialize.
#define AQ_GLOBAL __attribute__((address_space(1)))
typedef const v4i AQ_GLOBAL* gv4i_ptr;
typedef const int AQ_GLOBAL* gint_ptr;

// (scale, zero-point) of one activation tensor, produced on the device by the quantizer block.
struct ActQ {
    float s;
    int32_t z;
};

// Activation ranges travel to the device as a kernel argument (no host->device copy).
struct RangesArg {
    float lo[AQ_MAX_LAYERS];
    float hi[AQ_MAX_LAYERS];
};

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// round-half-even, clamped in float first so that huge values and NaN are defined
// (anything not >= lo, NaN included, gives lo) -- Sec. 3.2's round(W / delta) with saturation.
__device__ __forceinline__ int rint_clamp(float v, int lo, int hi) {
    float r = rintf(v);
    if (!(r >= (float)lo)) return lo;
    if (r > (float)hi) return hi;
    return (int)r;
}

// Sec. 3.2's round(W / delta), the quotient formed by IEEE fp32 division, at the price of one
// multiply in the common case.  m = w * (1/s) differs from the true quotient by a few ulp; unless m
// sits within a guard band of a half-integer (where that could flip the rounding, or where the
// fp32-rounded quotient could be an exact tie), round(m) IS round(fl(w / s)).  Lanes inside the band
// (a few in a million) take the division.  `rcp_ok` is false when 1/s is not usable (s denormal).
struct QuantScale {
    float s, inv;
    bool rcp_ok;
};
__device__ __forceinline__ QuantScale make_quant_scale(float s) {
    QuantScale q;
    q.s = s;
    q.inv = 1.0f / s;
    q.rcp_ok = q.inv <= 3.0e38f && s >= 1.2e-38f;
    return q;
}
__device__ __forceinline__ int quant_code(float w, const QuantScale& q, int lo, int hi) {
    if (!q.rcp_ok) return rint_clamp(w / q.s, lo, hi);
    const float m = w * q.inv;
    const float r = rintf(m);
    // distance to the nearest half-integer is 0.5 - |m - r|; guard band 2^-20 relative + 2^-20 absolute
    const float slack = 0.5f - fabsf(m - r);
    if (slack < fabsf(m) * 9.5367431640625e-7f + 9.5367431640625e-7f) return rint_clamp(w / q.s, lo, hi);
    if (!(r >= (float)lo)) return lo;
    if (r > (float)hi) return hi;
    return (int)r;
}

// Four codes at once, packed little-endian into one word (code & 255 each): the guard-band test of
// quant_code is shared by the four elements, so the common case has a single (not taken) branch.
__device__ __forceinline__ uint32_t quant_code4(float4 v, const QuantScale& q, int lo, int hi, int add) {
    float r0, r1, r2, r3;
    bool exact = !q.rcp_ok;
    if (!exact) {
        const float m0 = v.x * q.inv, m1 = v.y * q.inv, m2 = v.z * q.inv, m3 = v.w * q.inv;
        r0 = rintf(m0);
        r1 = rintf(m1);
        r2 = rintf(m2);
        r3 = rintf(m3);
        const float c = 9.5367431640625e-7f;  // 2^-20
        exact = (0.5f - fabsf(m0 - r0) < fabsf(m0) * c + c) | (0.5f - fabsf(m1 - r1) < fabsf(m1) * c + c) |
                (0.5f - fabsf(m2 - r2) < fabsf(m2) * c + c) | (0.5f - fabsf(m3 - r3) < fabsf(m3) * c + c);
    }
    if (exact) {
        r0 = rintf(v.x / q.s);
        r1 = rintf(v.y / q.s);
        r2 = rintf(v.z / q.s);
        r3 = rintf(v.w / q.s);
    }
    // fmaxf(NaN, lo) = lo: same saturation rule as rint_clamp
    const float flo = (float)lo, fhi = (float)hi;
    const int c0 = (int)fminf(fmaxf(r0, flo), fhi) + add, c1 = (int)fminf(fmaxf(r1, flo), fhi) + add;
    const int c2 = (int)fminf(fmaxf(r2, flo), fhi) + add, c3 = (int)fminf(fmaxf(r3, flo), fhi) + add;
    return (uint32_t)(c0 & 255) | ((uint32_t)(c1 & 255) << 8) | ((uint32_t)(c2 & 255) << 16) | ((uint32_t)c3 << 24);
}

// Four unsigned codes clamp(round(v / s) + z, 0, 255) packed little-endian: the form of quant_code4
// for activations and observations (lo = -z, hi = 255 - z, add = z), with the guard-band test folded
// into one comparison and the clamp, the conversion and the packing done by the saturating
// float -> byte conversion (the rounded value plus z is an integer, or saturates either way).
__device__ __forceinline__ uint32_t quant_u8x4(float4 v, const QuantScale& q, float zf) {
    float r0, r1, r2, r3;
    bool exact = !q.rcp_ok;
    if (!exact) {
        const float m0 = v.x * q.inv, m1 = v.y * q.inv, m2 = v.z * q.inv, m3 = v.w * q.inv;
        r0 = rintf(m0);
        r1 = rintf(m1);
        r2 = rintf(m2);
        r3 = rintf(m3);
        const float c = 9.5367431640625e-7f;  // 2^-20
        // 0.5 - |m - r| < |m| c + c  <=>  |m - r| + |m| c > 0.5 - c
        const float t0 = fmaf(fabsf(m0), c, fabsf(m0 - r0)), t1 = fmaf(fabsf(m1), c, fabsf(m1 - r1));
        const float t2 = fmaf(fabsf(m2), c, fabsf(m2 - r2)), t3 = fmaf(fabsf(m3), c, fabsf(m3 - r3));
        const float tm = fmaxf(fmaxf(t0, t1), fmaxf(t2, t3));
        // (a NaN or infinite lane drops out of the maximum; its code is the same on either path)
        exact = !(tm <= 0.5f - c);
    }
    if (exact) {
        r0 = rintf(v.x / q.s);
        r1 = rintf(v.y / q.s);
        r2 = rintf(v.z / q.s);
        r3 = rintf(v.w / q.s);
    }
    uint32_t pack = 0;
    pack = __builtin_amdgcn_cvt_pk_u8_f32(r0 + zf, 0, pack);
    pack = __builtin_amdgcn_cvt_pk_u8_f32(r1 + zf, 1, pack);
    pack = __builtin_amdgcn_cvt_pk_u8_f32(r2 + zf, 2, pack);
    pack = __builtin_amdgcn_cvt_pk_u8_f32(r3 + zf, 3, pack);
    return pack;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int wave_or_i32(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v |= __shfl_xor(v, o, 64);
    return v;
}

// Device status bits kept in the handle (sticky until the next aq_quantize_params).
constexpr int kStatNonFinite = 1;
constexpr int kStatRange = 2;
constexpr int kStatBlob = 4;  // an imported blob's header did not match the handle

// Per-layer descriptor handed to the forward kernels by value.
struct LayerDev {
    const int8_t* wp;          // packed signed-domain weights [NT][KS][64 lanes][16 bytes]
    // bias_fold heads a contiguous pack of four [N_pad] arrays: bias_fold | M0 or m | rz or gamma |
    // sh or beta (requantized layers take the first alternative, LayerNorm and last layers the second);
    // rz, sh, gamma and beta below point into that pack
    const int32_t* bias_fold;  // [N_pad] integer bias with the zero-point terms folded in
    const int32_t* M0;         // [N_pad] requantization multipliers (Q31, normalised)
    const int32_t* rshift;     // [N_pad] requantization right shifts
    const float* m;            // [N_pad] s_in * s_w[n]
    const float* gamma;        // [N_pad] LayerNorm gain / offset (LN layers)
    const float* beta;
    const int32_t* z_w;        // [N_pad] weight zero-points (unsigned domain)
    const int32_t* rz;         // [N_pad] short-form requantization: rounding constant + (z_out << sh)
    const int32_t* sh;         // [N_pad] short-form shift r - 32
    int K, N, KS, NT;
    int act;
    // conv geometry (per-layer kernel only); FC: all 1
    int in_h, in_w, in_c, kh, kw, stride, oh, ow;
};

// The static description of a quantized policy, kept in DEVICE memory and read by the forward
// kernels through one pointer: kernel arguments live in host-visible memory, and every cache line
// of a large by-value argument costs a round trip over the host link on first touch.
struct NetDev {
    LayerDev L[AQ_MAX_LAYERS];
    ActQ actq[AQ_MAX_LAYERS + 1];  // written by the quantizer kernels: (scale, zero-point) per activation tensor
    int fast[AQ_MAX_LAYERS];       // written by the quantizer kernels: layer qualifies for the short requant form
    int n_layers;
    int head;
    int in_u8;
    int asym;
    float ln_eps;
};

// The quantizer's view of a policy (device-resident, built once per handle): where every layer's
// outputs go, and where each layer starts in the three grids that cover all layers at once.
struct QLayerTab {
    int8_t* wp;
    float* s_w;
    int32_t* z_w;
    int32_t* rowsum;
    int32_t* bias_q;
    int32_t* M0;
    int32_t* rshift;
    float* m;
    int32_t* bias_fold;
    int32_t* pack1;
    int32_t* rz;  // LayerNorm layers: the gain slot of the constant pack
    int32_t* sh;  // LayerNorm layers: the offset slot
    int N, K, KS;
    int requant;  // hidden layer without LayerNorm
    int ln;
    int row_blk0;  // first workgroup of the row-quantize grid (4 output channels per workgroup)
    int cst_blk0;  // first workgroup of the constants grid (256 channels per workgroup)
    int rng_blk0;  // first workgroup of the range grid (per-tensor scheme)
    int rng_blks;
};
struct QTab {
    QLayerTab L[AQ_MAX_LAYERS];
    int n_layers, asym, in_u8;
    float qdenom;  // activations (8 bits)
    float w_qdenom;  // weights at n bits: denominator of delta, largest unsigned and symmetric codes
    int w_qmax, w_qw;
    int row_blks, cst_blks, rng_blks_total;
};
// The caller's fp32 parameters of one quantize pass (by value: they change from call to call).
struct QPtrs {
    const float* w[AQ_MAX_LAYERS];
    const float* b[AQ_MAX_LAYERS];
    const float* gamma[AQ_MAX_LAYERS];
    const float* beta[AQ_MAX_LAYERS];
};

// Per-call arguments (small, by value).
struct CallArgs {
    const void* obs;
    void* actions;
    int64_t batch;
    int ld;     // fused kernel: LDS row stride, bytes
    int cst_n;  // fused kernel: words per constant array in the LDS staging area
    int K0, Kp0, in_u8;  // first layer's input width (real, padded) and input type, so the observation
                         // loads can be issued before anything else has been read
    // fused kernel: the first layer's packed weights and constant pack, so that their loads do not
    // wait for the network description either
    const int8_t* wp0;
    const int32_t* pack0;
    int NT0, KS0, pieces0;
    int cst_dbl;   // fused kernel: the LDS constant area is doubled (next layer's constants parked early)
    int ln0;       // fused kernel: the first layer is followed by LayerNorm (its parked gain / offset are pre-scaled)
    int narrow0;   // fused kernel: the first layer is also the last and narrow (its weights are split over K)
    int part_off;  // fused kernel: LDS offset of the partial-sum area of a narrow last layer, or -1 when it
                   // fits the idle activation buffer
    // fused kernel: Gaussian exploration noise added where the actions are written (ex_sigma != NULL)
    const float* ex_sigma;
    uint32_t ex_k0, ex_k1, ex_s0, ex_s1;
};

// Optional intermediate outputs (by value, only read by the kernels compiled with TAPS).
struct TapArgs {
    int32_t* acc[AQ_MAX_LAYERS];
    uint8_t* act[AQ_MAX_LAYERS];
    float* ln[AQ_MAX_LAYERS];
    uint8_t* a0;
    float* y;
};
struct LayerTaps {
    int32_t* acc;
    uint8_t* act;
    float* ln;
};

}  // namespace aq

#define AQ_HIP_CHECK(expr)                        \
    do {                                          \
        hipError_t e_ = (expr);                   \
        if (e_ != hipSuccess) return AQ_EHIP;     \
    } while (0)
