// Whole-network fused int8 MLP (Sec. 3.1 actor inference, quantized per Sec. 3.2): one workgroup
// of 8 wavefronts owns ROWS = 32 * MT batch rows from the observation to the action.
//   - activations never leave LDS (two ping-pong row-major int8 buffers, signed domain)
//   - weights stream from L2 straight into MFMA operand registers (pre-packed at quantize time);
//     the first k-steps of the NEXT pass or layer are requested before the current epilogue starts,
//     so no layer begins by waiting for its first operands; layer descriptors come by scalar loads
//   - each wave owns NB feature tiles per pass; per-channel constants of the layer are fetched
//     while the MFMAs run and handed to the epilogue through LDS
//   - epilogues: requantize(+ReLU) / LayerNorm+tanh+requantize in registers, last layer dequantize,
//     then a coalesced head pass (tanh / identity / argmax)
#pragma once
#include "explore_device.hpp"
#include "int8_device.hpp"

namespace aq {

constexpr int FW = 8;            // wavefronts per workgroup
constexpr int FT = FW * 64;      // threads per workgroup
constexpr int CST_MAXN = 1024;   // widest layer whose constants fit the LDS staging area


// LDS layout (bytes): [buf_in ROWS*ld][buf_out ROWS*ld][red 2*FW*ROWS floats][cst 4*cst_n words]
__host__ __device__ inline size_t fused_lds_bytes(int rows, int ld, int cst_n, bool cst_dbl = false) {
    return (size_t)2 * rows * ld + (size_t)2 * FW * rows * 4 + (size_t)4 * cst_n * 4 * (cst_dbl ? 2 : 1);
}

// The network description is read through the kernel's pointer argument with uniform indices, i.e. by
// scalar loads into scalar registers (measured faster than a copy in LDS read back through vector
// registers: 2 % on the headline workload).  readfirstlane keeps a value scalar wherever the compiler
// cannot prove it uniform, so that loop bounds and branches stay scalar.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float unif(float v) { return __int_as_float(uni(__float_as_int(v))); }
template <class T>
__device__ __forceinline__ T* uni_ptr(T* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (T*)(((uint64_t)hi << 32) | lo);
}

// One layer as the kernel needs it: plain scalars, built field by field from the LDS copy.
struct LayerView {
    const int8_t* wp;
    gv4i_ptr pack;        // the layer's epilogue constants: four contiguous [Np] arrays, as 16-byte pieces
    const int32_t* rshift;
    gint_ptr z_w;
    int N, NT, KS, act, pieces, fast, z_out;
    float s_out;
    bool last, ln;
};
// The pack holds bias_fold, then by layer type: requantized M0, rz, sh (the general requantization
// form reads its shifts from global memory); LayerNorm m, gamma, beta; last m (two arrays staged).
__device__ __forceinline__ LayerView layer_view(const NetDev& n, int l, int n_layers) {
    const LayerDev& s = n.L[l];
    LayerView v;
    v.last = l == n_layers - 1;
    v.act = uni(s.act);
    v.ln = !v.last && v.act == AQ_ACT_LN_TANH;
    v.wp = uni_ptr(s.wp);
    v.pack = (gv4i_ptr)uni_ptr(s.bias_fold);
    v.rshift = uni_ptr(s.rshift);
    v.z_w = (gint_ptr)uni_ptr(s.z_w);
    v.N = uni(s.N);
    v.NT = uni(s.NT);
    v.KS = uni(s.KS);
    v.pieces = (v.last ? 2 : 4) * v.NT * 8;
    v.s_out = 1.0f;
    v.z_out = 0;
    v.fast = 0;
    if (!v.last) {
        v.s_out = unif(n.actq[l + 1].s);
        v.z_out = uni(n.actq[l + 1].z);
        v.fast = uni(n.fast[l]);
    }
    return v;
}
// this thread's share of a layer's constants: up to two 16-byte pieces (Np <= CST_MAXN)
__device__ __forceinline__ void load_consts(const LayerView& v, int tid, v4i& c0, v4i& c1) {
    if (tid < v.pieces) c0 = v.pack[tid];
    if (tid + FT < v.pieces) c1 = v.pack[tid + FT];
}
// 2 log2(e): tanh(y) = 1 - 2 / (2^(K2 y) + 1).  A LayerNorm layer's gain and offset are parked already
// multiplied by it, so that the epilogue's fused multiply-add yields the exponent directly.
constexpr float K2_LOG2E = 2.885390081777927f;
__device__ __forceinline__ v4i scale_k2(const v4i& v) {
    v4i r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __float_as_int(__int_as_float(v[i]) * K2_LOG2E);
    return r;
}
// scale_from: first 16-byte piece that holds gain / offset values (LayerNorm layers), or a large number
__device__ __forceinline__ void park_consts(int pieces, int tid, int32_t* cst, const v4i& c0, const v4i& c1,
                                            int scale_from = 1 << 30) {
    if (tid < pieces) ((v4i*)cst)[tid] = tid >= scale_from ? scale_k2(c0) : c0;
    if (tid + FT < pieces) ((v4i*)cst)[tid + FT] = tid + FT >= scale_from ? scale_k2(c1) : c1;
}

template <int NB>
__device__ __forceinline__ void tile_ptrs(const int8_t* wp, int NT, int KS, int grp, int lane,
                                          gv4i_ptr (&wptr)[NB]) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int nt = grp * NB + nb;
        nt = nt < NT ? nt : NT - 1;
        wptr[nb] = (gv4i_ptr)wp + (int64_t)nt * KS * 64 + lane;
    }
}

// A last layer of at most two feature tiles would leave most waves idle.  It is spread over all
// eight instead: its (feature tile, row tile) pairs go to different waves, and the waves left over
// split K.  Partial accumulators meet in LDS (PART_WORDS ints per wave: 16 accumulator registers
// and the row sums of the activations, lane-major).
constexpr int NARROW_NT = 2;
constexpr int PART_WORDS = 17 * 64;
constexpr int PART_BYTES = FW * PART_WORDS * 4;
struct NarrowMap {
    int pairs, ksplit, pair, nt, mt, k0, k1;
};
template <int MT>
__device__ __forceinline__ NarrowMap narrow_map(int NT, int KS, int wave) {
    NarrowMap x;
    x.pairs = NT * MT;                        // 1, 2, 4 or 8
    const int lg = 31 - __builtin_clz(x.pairs);
    x.ksplit = FW >> lg;
    x.pair = wave & (x.pairs - 1);
    const int kpart = wave >> lg;
    x.nt = x.pair & (NT - 1);
    x.mt = x.pair >> (NT - 1);                // NT is 1 or 2
    const int kchunk = (KS + x.ksplit - 1) >> (3 - lg);
    x.k0 = kpart * kchunk;
    x.k1 = x.k0 + kchunk < KS ? x.k0 + kchunk : KS;
    return x;
}

// Sums the K-split partial accumulators of a narrow last layer and dequantizes: every thread owns
// 2 * NT * MT outputs (lane-major, so its LDS reads are conflict-free) and reads the KSPLIT partial
// sums of each; all reads of one output are independent and issued together.
template <int MT, int NT, bool ASYM, bool TAPS, bool HALF>
__device__ __forceinline__ void narrow_reduce(const int32_t* part, const CPtrs& C, const LayerTaps& T, int N, int zw_s,
                                              int64_t row0, int64_t batch, float* yrow, int ldy, int tid, int head,
                                              float* actions, float* tap_y, const CallArgs& c) {
    constexpr int PAIRS = NT * MT, KSPLIT = FW / PAIRS;
    // a 16-row workgroup enumerates only the lower half of the MFMA tile's rows (the rest is don't-care)
    constexpr int STEPS = HALF ? PAIRS : 2 * PAIRS;
#pragma unroll
    for (int it = 0; it < STEPS; ++it) {
        int pr, reg, ln;
        if (HALF) {
            pr = it;
            reg = (tid >> 5) & 15;
            ln = (tid & 15) + 32 * ((tid >> 4) & 1);
        } else {
            const int e = tid + it * FT;
            pr = it >> 1;  // FT = 512 outputs per step, 1024 per pair
            reg = (e >> 6) & 15;
            ln = tid & 63;
        }
        int v = 0, rsum = 0;
#pragma unroll
        for (int kp = 0; kp < KSPLIT; ++kp) {
            const int32_t* src = part + (kp * PAIRS + pr) * PART_WORDS + ln;
            v += src[reg * 64];
            if (ASYM) rsum += src[16 * 64];
        }
        const int nt = pr & (NT - 1), mt = pr / NT;
        const int n = nt * 32 + 8 * (reg >> 2) + 4 * (ln >> 5) + (reg & 3);
        const int m = mt * 32 + (ln & 31);
        v += C.bias_fold[n];
        if (ASYM) v -= zw_s * rsum;
        const int64_t row = row0 + m;
        const bool ok = row < batch && n < N;
        if (TAPS) {
            if (T.acc && ok) T.acc[row * N + n] = v;
        }
        const float y = (float)v * C.m[n];
        if (actions) {
            // elementwise heads leave from here; only argmax needs the whole row in one place
            if (ok) {
                if (TAPS) {
                    if (tap_y) tap_y[row * N + n] = y;
                }
                float act = head == AQ_HEAD_TANH ? tanh_head(y) : y;
                if (c.ex_sigma)  // exploration noise of Sec. 4.1, sigma per actor (= per batch row)
                    act = act + c.ex_sigma[row] * gaussian_draw((uint32_t)row, n, c.ex_k0, c.ex_k1, c.ex_s0, c.ex_s1);
                actions[row * N + n] = act;
            }
        } else {
            yrow[m * ldy + n] = y;
        }
    }
}

// HALF (MT = NB = 1 only): the workgroup owns 16 rows instead of 32, for batches too small to give
// every CU a 32-row workgroup.  The MFMAs still run on 32-row tiles (the upper 16 rows of the LDS
// buffers are don't-care); fold_rows16 then spreads the 16 valid rows over all 64 lanes, so that the
// epilogues, which are what bounds small networks, do half the work per lane.
template <int MT, int NB, bool ASYM, bool TAPS, bool HALF>
__global__ __launch_bounds__(FT) void k_mlp_fused(const NetDev* __restrict__ netp, const CallArgs c,
                                                  const TapArgs t) {
    extern __shared__ __align__(16) int8_t smem[];
    static_assert(!HALF || (MT == 1 && NB == 1), "16-row workgroups use one tile per wave");
    constexpr int ROWS = HALF ? 16 : 32 * MT;  // rows this workgroup owns
    constexpr int BROWS = 32 * MT;             // rows of each LDS activation buffer
    constexpr int QT = HALF ? 2 : 4;           // register quads per tile and lane in the epilogues
    constexpr int PF = NB == 1 ? 8 : 4;
    // requesting the next weights ahead of the epilogue keeps PF*NB operand registers alive through
    // it; the wide variant (NB = 2) has no registers to spare and fetches at the start of each pass
    constexpr bool XPF = NB == 1;
    const NetDev& a = *netp;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5;
    const int hh = HALF ? (lane >> 4) & 1 : 0;        // which half of the feature quads (after the fold)
    const int mrow = HALF ? lane & 15 : lane & 31;    // this lane's row within a row tile in the epilogues
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    const int ld = c.ld, cst_n = c.cst_n;
    int8_t* buf_in = smem;
    int8_t* buf_out = smem + BROWS * ld;
    float* red = (float*)(smem + 2 * BROWS * ld);
    int32_t* cst = (int32_t*)(red + 2 * FW * BROWS);
    // With LDS to spare the constant area is doubled: the next layer's constants are parked in the other
    // half before the barrier that ends the current layer, which saves the barrier that would publish them.
    // (two feature tiles per wave are only planned for layers too wide for a doubled constant area, and
    // 128-row workgroups never fit one)
    const int cst_dbl = (NB == 2 || MT == 4) ? 0 : c.cst_dbl;
    const int cst_half = cst_dbl ? 4 * cst_n : 0;  // words between the two halves

    // first layer's first weights: requested before the observations are touched
    v4i wreg[PF][NB];
    if (XPF) {
        gv4i_ptr wptr[NB];
        if (!c.narrow0) {
            tile_ptrs<NB>(c.wp0, c.NT0, c.KS0, wave, lane, wptr);
            if (wave * NB < c.NT0) mma_prefetch<NB, PF>(wptr, 0, c.KS0, wreg);
        }
    }
    // ... and its per-channel constants
    // (doubled constant area only; with a single area every wave fetches its own constants, see below)
    v4i cv0 = {0, 0, 0, 0}, cv1 = cv0;
    if (cst_dbl) {
        if (tid < c.pieces0) cv0 = ((gv4i_ptr)c.pack0)[tid];
        if (tid + FT < c.pieces0) cv1 = ((gv4i_ptr)c.pack0)[tid + FT];
    }

    // observation quantize: a0 = clamp(round(x / s0) + z0, 0, 255), kept in the signed domain
    {
        const int K0 = c.K0, Kp = c.Kp0;
        const float s0 = a.actq[0].s;
        const int z0 = a.actq[0].z;
        const QuantScale qs0 = make_quant_scale(s0);
        const float zf0 = (float)z0;
        if (!c.in_u8 && ((uintptr_t)c.obs & 15) == 0) {
            // The block's rows are one contiguous run in memory that starts 16-byte aligned (ROWS * K0
            // is a multiple of 4): read it as flat 16-byte pieces, four pieces in flight per lane,
            // quantize four values at a time, and scatter the codes to their (row, k) places in LDS.
            const int64_t left = c.batch - row0;
            const int vrows = left < ROWS ? (int)left : ROWS;
            const int n_el = vrows * K0, n4 = n_el >> 2;
            const float invK = 1.0f / (float)K0;
            const float* src1 = (const float*)c.obs + row0 * K0;
            const float4* src = (const float4*)src1;
            for (int i0 = tid; i0 < n4; i0 += 4 * FT) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (i0 + u * FT < n4) v[u] = src[i0 + u * FT];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = i0 + u * FT;
                    if (idx < n4) {
                        uint32_t pack = quant_u8x4(v[u], qs0, zf0);
                        if (TAPS) {
                            if (t.a0) *(uint32_t*)(t.a0 + row0 * K0 + 4 * idx) = pack;
                        }
                        pack ^= 0x80808080u;
                        const int e = 4 * idx;
                        // e / K0: (e + 0.5) / K0 stays at least 0.5 / K0 away from every integer, far more
                        // than the rounding error of the product at these magnitudes (all below 2^23, so
                        // the 24-bit multiplies are exact)
                        int m = (int)(((float)e + 0.5f) * invK);
                        int k = e - __mul24(m, K0);
                        if ((k & 3) == 0 && k + 4 <= K0) {
                            *(uint32_t*)(buf_in + __mul24(m, ld) + k) = pack;
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                buf_in[__mul24(m, ld) + k] = (int8_t)(pack >> (8 * i));
                                if (++k == K0) {
                                    k = 0;
                                    ++m;
                                }
                            }
                        }
                    }
                }
            }
            if (tid < n_el - 4 * n4) {  // at most three elements past the last whole piece
                const int e = 4 * n4 + tid;
                const int m = (int)(((float)e + 0.5f) * invK), k = e - m * K0;
                const int code = quant_code(src1[e], qs0, -z0, 255 - z0) + z0;
                if (TAPS) {
                    if (t.a0) t.a0[row0 * K0 + e] = (uint8_t)code;
                }
                buf_in[m * ld + k] = (int8_t)(code - 128);
            }
            // zero (signed domain) in the padding columns and in the rows past the batch
            const int padw = Kp - K0;
            if (padw > 0) {
                for (int m = tid >> 5; m < vrows; m += FT / 32) {
                    const int k = K0 + (tid & 31);
                    if (k < Kp) buf_in[m * ld + k] = 0;
                }
            }
            for (int m = vrows + wave; m < ROWS; m += FW)
                for (int k = lane; k < Kp; k += 64) buf_in[m * ld + k] = 0;
        } else {
            // 16 lanes per row; each lane requests up to eight elements before it converts the first,
            // and the zero padding up to the k-step boundary is written in the same sweep
            const int r32 = tid >> 4, l16 = tid & 15;
            for (int mb = 0; mb < ROWS; mb += 32) {
                const int m = mb + r32;
                const int64_t row = row0 + m;
                const bool ok = row < c.batch;
                for (int kb = 0; kb < (m < ROWS ? Kp : 0); kb += 128) {
                    float xv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int k = kb + l16 + 16 * u;
                        xv[u] = 0.0f;
                        if (ok && k < K0) {
                            if (c.in_u8) xv[u] = __int_as_float((int)((const uint8_t*)c.obs)[row * K0 + k]);
                            else xv[u] = ((const float*)c.obs)[row * K0 + k];
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int k = kb + l16 + 16 * u;
                        if (k < Kp) {
                            int code = 128;
                            if (ok && k < K0) {
                                code = c.in_u8 ? __float_as_int(xv[u]) : quant_code(xv[u], qs0, -z0, 255 - z0) + z0;
                                if (TAPS) {
                                    if (t.a0) t.a0[row * K0 + k] = (uint8_t)code;
                                }
                            }
                            buf_in[m * ld + k] = (int8_t)(code - 128);
                        }
                    }
                }
            }
        }
    }
    if (cst_dbl) park_consts(c.pieces0, tid, cst, cv0, cv1, c.ln0 ? c.NT0 * 16 : 1 << 30);
    lds_barrier();

    const int n_layers = uni(a.n_layers);
    const float ln_eps = unif(a.ln_eps);
    int N_last = 0;
    const float* ybuf = nullptr;  // dequantized last-layer rows in LDS and their stride, set by the last layer
    int ldy_h = 0;
    // a narrow last layer is handled after the loop, by all waves together
    const bool narrow = uni(a.L[n_layers - 1].NT) <= NARROW_NT;
    const int n_loop = narrow ? n_layers - 1 : n_layers;
    for (int l = 0; l < n_loop; ++l) {
        const LayerView L = layer_view(a, l, n_layers);
        const bool last = L.last, ln = L.ln;
        N_last = L.N;
        LayerTaps T{nullptr, nullptr, nullptr};
        if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
        const int ngroups = (L.NT + NB - 1) / NB;
        const int Np = L.NT * 32;
        const float s_out = L.s_out;
        const int z_out = L.z_out, fast = L.fast;
        const QuantScale qs_out = make_quant_scale(s_out);
        const float zf_out = (float)z_out;
        const int lo = (!last && L.act == AQ_ACT_RELU) ? z_out : 0;
        const int zw_s = ASYM ? L.z_w[0] - 128 : 0;
        const int ldy = Np;  // last layer: fp32 row stride of y in LDS
        const int8_t* in = buf_in;
        int8_t* out = buf_out;

        // This layer's per-channel constants.  Doubled constant area: they were parked in the other half
        // before the barrier that ended the previous layer.  Single area (wide layers): an epilogue only
        // reads the constants of its own wave's features, so every wave requests that slice (one
        // 16-byte piece per lane) at the start of each MFMA pass and parks it after the pass: nothing
        // is shared, no barrier is needed, and a wave that finishes its MFMA pass early goes straight
        // on to its epilogue while the other wave of its SIMD still has the matrix pipe.
        int32_t* cstl = cst + (l & 1) * cst_half;
        const CPtrs C{cstl, cstl + Np, L.rshift, cstl + 2 * Np, cstl + 3 * Np, (const float*)(cstl + Np)};
        const float* c_gamma = (const float*)(cstl + 2 * Np);
        const float* c_beta = (const float*)(cstl + 3 * Np);
        int pieces_next = 0, scale_next = 1 << 30;

        if (last) {
            ybuf = (const float*)out;
            ldy_h = ldy;
        }
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
            v4i cw = {0, 0, 0, 0};
            int cw_off = -1;  // word offset of this lane's piece within the constant pack, or none
            if (!cst_dbl && active) {
                constexpr int PER = 8 * NB;  // pieces per array in the slice of this wave's NB tiles
                const int arr = lane / PER, w0 = 32 * NB * grp + 4 * (lane % PER);
                if (arr < 4 && w0 < Np) {
                    cw_off = arr * Np + w0;
                    cw = L.pack[cw_off >> 2];
                }
            }
            if (active) {
                gv4i_ptr wptr[NB];
                tile_ptrs<NB>(L.wp, L.NT, L.KS, grp, lane, wptr);
                if (!XPF) mma_prefetch<NB, PF>(wptr, 0, L.KS, wreg);
                mma_run<MT, NB, ASYM, PF>(wptr, wreg, in, ld, 0, L.KS, 0, acc, rs, lane);
                if (HALF) {
                    fold_rows16(acc[0][0], lane);
                    if (ASYM) rs[0][0] = fold_rows16_scalar(rs[0][0], lane);
                }
            }
            // request the next pass's (or the next layer's) first weights before the epilogue
            if (XPF) {
                const bool more = g0 + FW < ngroups;
                const int ln_i = (more || last) ? l : l + 1;
                const int8_t* wp_n = uni_ptr(a.L[ln_i].wp);
                const int NT_n = uni(a.L[ln_i].NT), KS_n = uni(a.L[ln_i].KS);
                const int grp_n = more ? grp + FW : wave;
                // (a narrow last layer fetches its own weights: its waves split K instead of the tiles)
                const bool narrow_next = !more && l + 2 == n_layers && NT_n <= NARROW_NT;
                if ((more || !last) && !narrow_next && grp_n * NB < NT_n) {
                    gv4i_ptr wptr[NB];
                    tile_ptrs<NB>(wp_n, NT_n, KS_n, grp_n, lane, wptr);
                    mma_prefetch<NB, PF>(wptr, 0, KS_n, wreg);
                }
            }
            // ... and, on the last pass, the next layer's constants
            if (cst_dbl && !last && g0 + FW >= ngroups) {
                const LayerView vn = layer_view(a, l + 1, n_layers);
                load_consts(vn, tid, cv0, cv1);
                pieces_next = vn.pieces;
                if (vn.ln) scale_next = vn.NT * 16;  // pieces of the gain and offset arrays
            }
            if (!cst_dbl) {
                if (cw_off >= 0) *(v4i*)(cstl + cw_off) = (ln && cw_off >= 2 * Np) ? scale_k2(cw) : cw;
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_wave_barrier();
            }
            if (!ln) {
                if (active) {
                    const int m0 = mrow;
                    if (last) {
                        static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                            constexpr int nb = decltype(nb_c)::value;
                            const int nt = grp * NB + nb;
                            if (nt < L.NT) {
                                static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                                    constexpr int mt = decltype(mt_c)::value;
                                    const int m = mt * 32 + m0;
                                    const int64_t row = row0 + m;
                                    epi_last_tile<ASYM, TAPS, HALF>(L.N, T, C, acc[nb][mt], rs[mt][0], zw_s, nt, g, row,
                                                                    row < c.batch, (float*)out + m * ldy, ldy, nullptr,
                                                                    0, hh);
                                });
                            }
                        });
                    } else if (fast) {
                        epi_hidden_wave<MT, NB, ASYM, TAPS, true, HALF>(L.N, L.NT, T, C, acc, rs, zw_s, grp, g, row0 + m0,
                                                                        c.batch, false, z_out, lo, out + m0 * ld, 32 * ld,
                                                                        true, Np, hh);
                    } else {
                        epi_hidden_wave<MT, NB, ASYM, TAPS, false, HALF>(L.N, L.NT, T, C, acc, rs, zw_s, grp, g, row0 + m0,
                                                                         c.batch, false, z_out, lo, out + m0 * ld, 32 * ld,
                                                                         true, Np, hh);
                    }
                }
            } else {
                // LayerNorm over the layer's N features (all resident in this one pass: ngroups <= FW),
                // tanh, re-quantize.  Row statistics: in-lane sums, lane ^ 32, then across waves via LDS.
                float* red1 = red;
                float* red2 = red + FW * BROWS;
                float mean[MT], inv[MT];
                static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                    constexpr int mt = decltype(mt_c)::value;
                    float s = 0.0f;
                    const int64_t row = row0 + mt * 32 + mrow;
                    const bool row_ok = row < c.batch;
                    static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                        constexpr int nb = decltype(nb_c)::value;
                        const int nt = grp * NB + nb;
#pragma unroll
                        for (int j = 0; j < QT; ++j) {
                            const int n0 = nt * 32 + 8 * (j + 2 * hh) + 4 * g;
                            if (active && n0 < Np) {
                                int val[4];
                                quad_acc<ASYM, TAPS>(L.N, T, C, acc[nb][mt], j, n0, rs[mt][0], zw_s, row, row_ok, val);
                                const float4 mm = *(const float4*)(C.m + n0);
                                const float mv[4] = {mm.x, mm.y, mm.z, mm.w};
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    // (padding features: their scale m is stored as zero, so x = 0)
                                    float x = (float)val[i] * mv[i];
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
                    if (HALF) s += __shfl_xor(s, 16, 64);
                    if (g == 0 && hh == 0) red1[wave * BROWS + mt * 32 + mrow] = s;
                });
                lds_barrier();
                static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                    constexpr int mt = decltype(mt_c)::value;
                    const int m = mt * 32 + mrow;
                    float tot = 0.0f;
#pragma unroll
                    for (int w = 0; w < FW; ++w) tot += red1[w * BROWS + m];
                    mean[mt] = tot / (float)L.N;
                    // squared deviations over this wave's real tiles; the zeros standing in for the padding
                    // features of the last tile each add mean^2, taken out again below, once per row
                    float ss = 0.0f;
                    static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                        constexpr int nb = decltype(nb_c)::value;
                        const int nt = grp * NB + nb;
                        if (active && nt < L.NT) {
#pragma unroll
                            for (int j = 0; j < QT; ++j)
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    const float d = __int_as_float(acc[nb][mt][4 * j + i]) - mean[mt];
                                    ss = fmaf(d, d, ss);
                                }
                        }
                    });
                    ss += __shfl_xor(ss, 32, 64);
                    if (HALF) ss += __shfl_xor(ss, 16, 64);
                    if (g == 0 && hh == 0) red2[wave * BROWS + mt * 32 + mrow] = ss;
                });
                lds_barrier();
                static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                    constexpr int mt = decltype(mt_c)::value;
                    const int m = mt * 32 + mrow;
                    float tot = 0.0f;
#pragma unroll
                    for (int w = 0; w < FW; ++w) tot += red2[w * BROWS + m];
                    tot = fmaxf(tot - (float)(Np - L.N) * mean[mt] * mean[mt], 0.0f);  // the padding's share
                    inv[mt] = 1.0f / sqrtf(tot / (float)L.N + ln_eps);
                    const float shift = -mean[mt] * inv[mt];
                    // code = round(t / s + z) with t = 1 - 2 r, r = 1 / (2^e + 1): round(c0 - c1 r)
                    const float c0 = qs_out.inv + zf_out, c1 = 2.0f * qs_out.inv;
                    const int64_t row = row0 + m;
                    const bool row_ok = row < c.batch;
                    static_for<0, NB>([&](auto nb_c) __attribute__((always_inline)) {
                        constexpr int nb = decltype(nb_c)::value;
                        const int nt = grp * NB + nb;
                        if (active && nt < L.NT) {
#pragma unroll
                            for (int j = 0; j < QT; ++j) {
                                const int n0 = nt * 32 + 8 * (j + 2 * hh) + 4 * g;
                                const float4 ga = *(const float4*)(c_gamma + n0);
                                const float4 be = *(const float4*)(c_beta + n0);
                                const float gv[4] = {ga.x, ga.y, ga.z, ga.w}, bv[4] = {be.x, be.y, be.z, be.w};
                                // gv, bv: gain and offset times 2 log2(e); r = 1 / (e^{2y} + 1) on the exp2 and
                                // reciprocal units for either sign (exp2 saturates to 0 and +inf, rcp(inf) = 0)
                                float rv[4];
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    const float x = __int_as_float(acc[nb][mt][4 * j + i]);
                                    const float e = __builtin_amdgcn_exp2f(fmaf(fmaf(x, inv[mt], shift), gv[i], bv[i]));
                                    rv[i] = __builtin_amdgcn_rcpf(e + 1.0f);
                                }
                                uint32_t pack;
                                if (qs_out.rcp_ok) {
                                    // the tanh value already carries rounding differences of its own, so the
                                    // code is taken from t * (1/s) + z directly (it can differ from round(t/s)
                                    // only where t/s sits on a rounding tie)
                                    pack = 0;
#pragma unroll
                                    for (int i = 0; i < 4; ++i) {
                                        // float -> byte conversion: rounds half to even, saturates at 0 and 255, packs
                                        pack = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(rv[i], -c1, c0), i, pack);
                                    }
                                } else {
                                    pack = quant_code4(float4{fmaf(rv[0], -2.0f, 1.0f), fmaf(rv[1], -2.0f, 1.0f),
                                                              fmaf(rv[2], -2.0f, 1.0f), fmaf(rv[3], -2.0f, 1.0f)},
                                                       qs_out, -z_out, 255 - z_out, z_out);
                                }
                                if (n0 + 4 > L.N) {
                                    // padding features are zero in the signed domain
                                    const int keep = L.N - n0;  // < 4, may be <= 0
                                    const uint32_t kmask = keep <= 0 ? 0u : (1u << (8 * keep)) - 1u;
                                    pack = (pack & kmask) | (0x80808080u & ~kmask);
                                }
                                if (TAPS) {
#pragma unroll
                                    for (int i = 0; i < 4; ++i) {
                                        const int n = n0 + i;
                                        if (row_ok && n < L.N) {
                                            if (T.ln) T.ln[row * L.N + n] = fmaf(rv[i], -2.0f, 1.0f);
                                            if (T.act) T.act[row * L.N + n] = (uint8_t)(pack >> (8 * i));
                                        }
                                    }
                                }
                                *(uint32_t*)(out + m * ld + n0) = pack ^ 0x80808080u;
                            }
                        }
                    });
                });
            }
        }
        if (cst_dbl) park_consts(pieces_next, tid, cst + ((l + 1) & 1) * cst_half, cv0, cv1, scale_next);
        lds_barrier();
        int8_t* sw = buf_in;
        buf_in = buf_out;
        buf_out = sw;
    }

    if (narrow) {
        const int l = n_layers - 1;
        const LayerView L = layer_view(a, l, n_layers);
        N_last = L.N;
        LayerTaps T{nullptr, nullptr, nullptr};
        if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
        const int Np = L.NT * 32;
        const int zw_s = ASYM ? L.z_w[0] - 128 : 0;
        const int8_t* in = buf_in;
        int32_t* cstl = cst + (l & 1) * cst_half;
        if (!cst_dbl) load_consts(L, tid, cv0, cv1);  // parked below, after the MFMAs
        const CPtrs C{cstl, cstl + Np, L.rshift, cstl + 2 * Np, cstl + 3 * Np, (const float*)(cstl + Np)};
        // Everything below depends on the thread index only; left alone, the compiler computes it at
        // the top of the kernel and keeps it in registers through every layer.  The empty asm hides
        // the index from that motion.
        int tid_n = tid;
        asm volatile("" : "+v"(tid_n));
        const int lane = tid_n & 63, wave = __builtin_amdgcn_readfirstlane(tid_n >> 6);
        const NarrowMap nm = narrow_map<MT>(L.NT, L.KS, wave);
        v16i pacc[1][1], prs[1];
        pacc[0][0] = zero16();
        prs[0] = zero16();
        if (nm.k0 < nm.k1) {
            gv4i_ptr wptr[1];
            wptr[0] = (gv4i_ptr)L.wp + (int64_t)nm.nt * L.KS * 64 + lane;
            v4i w1[4][1];
            mma_prefetch<1, 4>(wptr, nm.k0, nm.k1, w1);
            mma_run<1, 1, ASYM, 4>(wptr, w1, in + nm.mt * 32 * ld, ld, nm.k0, nm.k1, 0, pacc, prs, lane);
        }
        int32_t* part = c.part_off >= 0 ? (int32_t*)(smem + c.part_off) : (int32_t*)buf_out;
        {
            int32_t* mine = part + wave * PART_WORDS + lane;
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[r * 64] = pacc[0][0][r];
            if (ASYM) mine[16 * 64] = prs[0][0];
        }
        if (!cst_dbl) park_consts(L.pieces, tid, cstl, cv0, cv1);
        lds_barrier();  // partial sums and this layer's constants are in LDS; the layer's input is free
        // y rows go where the layer's input was (stride Np + 1 floats keeps the banks apart)
        float* yrow = (float*)buf_in;
        ybuf = yrow;
        ldy_h = Np + 1;
        const int head_n = uni(a.head);
        float* direct = head_n != AQ_HEAD_ARGMAX ? (float*)c.actions : nullptr;
        float* tap_y = TAPS ? t.y : nullptr;
        if (L.NT == 1)
            narrow_reduce<MT, 1, ASYM, TAPS, HALF>(part, C, T, L.N, zw_s, row0, c.batch, yrow, ldy_h, tid_n, head_n, direct,
                                                   tap_y, c);
        else
            narrow_reduce<MT, 2, ASYM, TAPS, HALF>(part, C, T, L.N, zw_s, row0, c.batch, yrow, ldy_h, tid_n, head_n, direct,
                                                   tap_y, c);
        if (direct) return;  // actions are written; nothing below applies
        lds_barrier();
    }

    // action head on the dequantized last-layer rows y (fp32, in LDS): tanh / identity / argmax
    {
        const int head = uni(a.head);
        const int ldy = ldy_h;
        const int N = N_last;
        if (head == AQ_HEAD_ARGMAX) {
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
                ((float*)c.actions)[row * N + n] = head == AQ_HEAD_TANH ? tanh_head(y) : y;
            }
        }
    }
}

template <int MT, int NB, bool ASYM, bool TAPS, bool HALF>
aq_status launch_fused_t(const FwdArgs& a, size_t lds, hipStream_t st) {
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_mlp_fused<MT, NB, ASYM, TAPS, HALF>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return AQ_EHIP;
        attr_set = true;
    }
    const int rows = HALF ? 16 : 32 * MT;
    const unsigned grid = (unsigned)((a.c.batch + rows - 1) / rows);
    hipLaunchKernelGGL((k_mlp_fused<MT, NB, ASYM, TAPS, HALF>), dim3(grid), dim3(FT), lds, st, a.d_net, a.c, a.t);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

// one explicit instantiation per translation unit, so the variants compile in parallel
#define AQ_FUSED_DECL(MT, NB, AS, TP, HF) \
    extern template aq_status launch_fused_t<MT, NB, AS, TP, HF>(const FwdArgs&, size_t, hipStream_t)
#define AQ_FUSED_INST(MT, NB, AS, TP, HF) \
    template aq_status launch_fused_t<MT, NB, AS, TP, HF>(const FwdArgs&, size_t, hipStream_t)

}  // namespace aq
