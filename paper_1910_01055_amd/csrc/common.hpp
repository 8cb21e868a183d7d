// Shared device/host declarations of the ActorQ HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// Per-layer descriptor handed to the forward kernels by value.
struct LayerDev {
    const int8_t* wp;          // packed signed-domain weights [NT][KS][64 lanes][16 bytes]
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

// Per-call arguments (small, by value).
struct CallArgs {
    const void* obs;
    void* actions;
    int64_t batch;
    int ld;     // fused kernel: LDS row stride, bytes
    int cst_n;  // fused kernel: words per constant array in the LDS staging area
    int K0, Kp0, in_u8;  // first layer's input width (real, padded) and input type, so the observation
                         // loads can be issued before anything else has been read
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
