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
#pragma once
#include <type_traits>

#include "kernels.hpp"

namespace aq {


// compile-time loop: accumulator tiles are register arrays and must only ever be indexed by constants
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits for every
// outstanding global access (vmcnt(0)), which would drain the weight / constant prefetches that
// are deliberately left in flight across the barrier; here only LDS traffic is waited for.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

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

// The same value without the sign handling: tanh(x) = 1 - 2 / (e^{2x} + 1) for either sign, because
// exp2 saturates to 0 and +inf and rcp(inf) = 0.  Absolute error about 2e-7.
__device__ __forceinline__ float tanh_exp2(float x) {
    const float e = __builtin_amdgcn_exp2f(x * 2.885390081777927f);
    return fmaf(__builtin_amdgcn_rcpf(e + 1.0f), -2.0f, 1.0f);
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
    // 1 - 2 / (e^{2|x|} + 1) on the exp2 and reciprocal units (each good to about one ulp; the result is
    // at least 0.46, so the absolute error of a few 1e-7 stays below 1e-6 relative)
    float e = __builtin_amdgcn_exp2f(fminf(ax, 20.0f) * 2.885390081777927f);
    float t = fmaf(__builtin_amdgcn_rcpf(e + 1.0f), -2.0f, 1.0f);
    return copysignf(t, x);
}

// ---------------------------------------------------------------------------------------------
// MFMA core: accumulates NB feature tiles x MT row tiles over k-steps [ks_begin, ks_end).
// Weights stream global -> registers (already in operand order), activations come from LDS
// (row-major int8, row stride ld, column 0 = k-step ks_lds0).
// ---------------------------------------------------------------------------------------------
// PF = weight k-steps in flight per wave (global -> register prefetch depth)
// mma_prefetch issues the first PF k-steps' weight loads; mma_run consumes them and keeps the
// pipeline full for the rest of K.  Splitting the two lets a caller issue the next layer's first
// loads before it starts the current layer's epilogue.
template <int NB, int PF>
__device__ __forceinline__ void mma_prefetch(gv4i_ptr (&wptr)[NB], int ks_begin, int ks_end, v4i (&wreg)[PF][NB]) {
    // unconditional (indices past the end are clamped, those registers are never used): straight-line
    // loads let the compiler count exactly how many are in flight when the first one is needed
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        const int k = ks_begin + p < ks_end - 1 ? ks_begin + p : ks_end - 1;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) wreg[p][nb] = wptr[nb][(int64_t)k * 64];
    }
}

template <int MT, int NB, bool ASYM, int PF>
__device__ __forceinline__ void mma_run(gv4i_ptr (&wptr)[NB], v4i (&wreg)[PF][NB], const int8_t* xs, int ld,
                                        int ks_begin, int ks_end, int ks_lds0, v16i (&acc)[NB][MT], v16i (&rs)[MT],
                                        int lane) {
    const int8_t* xrow = xs + (lane & 31) * ld + (lane >> 5) * 16;
    v4i ones;
    ones[0] = ones[1] = ones[2] = ones[3] = 0x01010101;
    // The activation operands are read R k-steps ahead of their MFMAs (a ring of R register sets;
    // R divides PF so that every slot index is static): each k-step sits in its own conditional
    // block, where the compiler cannot move the LDS read ahead of the wait by itself.
    constexpr int R = MT == 1 ? 4 : (MT == 2 ? 2 : 1);
    static_assert(PF % R == 0, "operand ring must divide the weight pipeline depth");
    v4i xf[R][MT];
    const int ks_last = ks_end - 1;
    if (R > 1) {
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int kk = ks_begin + i < ks_last ? ks_begin + i : ks_last;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xf[i][mt] = *(const v4i*)(xrow + mt * 32 * ld + (kk - ks_lds0) * 32);
        }
    }
    // Whole groups of PF k-steps run as straight-line code: with no branch between a weight load and
    // its use, the compiler can wait for exactly the oldest loads (a conditional block in between
    // makes it wait for all of them, which drains the pipeline once per group).
    //   refill 1: every slot is refilled with k + PF (the caller guarantees k + PF < ks_end)
    //   refill 2: the last whole group before a partial one; indices past the end are clamped and the
    //             tiles re-read there are never used
    //   refill 0: the last group of K, nothing left to load
    auto group = [&](int ks, auto refill_c) __attribute__((always_inline)) {
        constexpr int refill = decltype(refill_c)::value;
        static_for<0, PF>([&](auto p_c) __attribute__((always_inline)) {
            constexpr int p = decltype(p_c)::value;
            constexpr int slot = p % R;
            const int k = ks + p;
            if (R == 1) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) xf[0][mt] = *(const v4i*)(xrow + mt * 32 * ld + (k - ks_lds0) * 32);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[nb][mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][nb], xf[slot][mt], acc[nb][mt], 0, 0, 0);
            if (ASYM) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    rs[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, xf[slot][mt], rs[mt], 0, 0, 0);
            }
            if (R > 1) {
                const int kk = k + R < ks_last ? k + R : ks_last;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    xf[slot][mt] = *(const v4i*)(xrow + mt * 32 * ld + (kk - ks_lds0) * 32);
            }
            if (refill != 0) {
                const int kw = refill == 1 ? k + PF : (k + PF < ks_last ? k + PF : ks_last);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) wreg[p][nb] = wptr[nb][(int64_t)kw * 64];
                // keep each refill right behind the MFMAs that freed its registers: moved to the end of
                // the group, it would be needed again almost at once
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    int ks = ks_begin;
    if (MT * NB <= 4) {
        for (; ks + 2 * PF <= ks_end; ks += PF) group(ks, std::integral_constant<int, 1>{});
        if (ks + PF <= ks_end) {
            if (ks + PF < ks_end) group(ks, std::integral_constant<int, 2>{});
            else group(ks, std::integral_constant<int, 0>{});
            ks += PF;
        }
    } else {
        // eight accumulator tiles per wave: a second copy of the group body makes the register
        // allocator spill accumulators between the copies, so every whole group takes the clamped
        // form (the tiles re-read at the end of K hit in the vector L1)
        for (; ks + PF <= ks_end; ks += PF) group(ks, std::integral_constant<int, 2>{});
    }
    // the remaining k-steps (fewer than PF), one conditional block each
    if (ks < ks_end) {
        static_for<0, PF - 1>([&](auto p_c) __attribute__((always_inline)) {
            constexpr int p = decltype(p_c)::value;
            constexpr int slot = p % R;
            const int k = ks + p;
            if (k < ks_end) {
                if (R == 1) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        xf[0][mt] = *(const v4i*)(xrow + mt * 32 * ld + (k - ks_lds0) * 32);
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[nb][mt] =
                            __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][nb], xf[slot][mt], acc[nb][mt], 0, 0, 0);
                if (ASYM) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        rs[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, xf[slot][mt], rs[mt], 0, 0, 0);
                }
                if (R > 1) {
                    const int kk = k + R < ks_last ? k + R : ks_last;  // never past the staged columns
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        xf[slot][mt] = *(const v4i*)(xrow + mt * 32 * ld + (kk - ks_lds0) * 32);
                }
            }
        });
    }
}

// where an epilogue reads the per-channel constants from (global memory or a copy staged in LDS)
struct CPtrs {
    const int32_t* bias_fold;
    const int32_t* M0;
    const int32_t* rshift;  // general form
    const int32_t* rz;      // short form
    const int32_t* sh;
    const float* m;
};
__device__ __forceinline__ CPtrs global_consts(const LayerDev& L) {
    return CPtrs{L.bias_fold, L.M0, L.rshift, L.rz, L.sh, L.m};
}

// requantize one accumulator: v = (acc * M0 + 2^(r-1)) >> r, code = clamp(v + z_out, lo, 255)
__device__ __forceinline__ int requant_code(int acc, int M0, int r, int z_out, int lo) {
    long long p = (long long)acc * (long long)M0 + ((1LL << r) >> 1);
    long long v = (p >> r) + z_out;
    v = v < lo ? lo : v;
    v = v > 255 ? 255 : v;
    return (int)v;
}

// canonical accumulator of one register quad: MFMA sum + folded bias (- z_w' * row sum of a_s)
template <bool ASYM, bool TAPS>
__device__ __forceinline__ void quad_acc(const int N, const LayerTaps& T, const CPtrs& C, const v16i& c, int j, int n0, int rs0, int zw_s,
                                         int64_t row, bool row_ok, int (&val)[4]) {
    const int4 bf = *(const int4*)(C.bias_fold + n0);
    const int bfv[4] = {bf.x, bf.y, bf.z, bf.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        val[i] = c[4 * j + i] + bfv[i];
        if (ASYM) val[i] -= zw_s * rs0;
        if (TAPS) {
            if (T.acc && row_ok && n0 + i < N) T.acc[(int64_t)row * N + n0 + i] = val[i];
        }
    }
}

// 16-row workgroups still run 32x32x32 MFMAs (rows 16..31 of the operand are don't-care), then fold
// the tile: lanes that hold rows 16..31 take over feature quads 2 and 3 of the row 16 below them.
// Afterwards lane l owns row l & 15, half h = (l >> 4) & 1, and registers 4j+i (j = 0, 1) hold feature
// 8 (j + 2h) + 4 (l >> 5) + i of the tile: every lane does useful epilogue work on half the registers.
// v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of its
// second: (c[r], c[r+8]) -> c[r] = [own row 0 | c[r+8] row 0 | own row 2 | c[r+8] row 2], which is the fold.
__device__ __forceinline__ void fold_rows16(v16i& c, int lane) {
    (void)lane;
#pragma unroll
    for (int r = 0; r < 8; ++r) c[r] = (int)__builtin_amdgcn_permlane16_swap((unsigned)c[r], (unsigned)c[r + 8], false, false)[0];
}
__device__ __forceinline__ int fold_rows16_scalar(int v, int lane) {
    (void)lane;
    return (int)__builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false)[0];
}

// Hidden-layer epilogue of a wave's whole tile set (NB feature tiles x MT row tiles).  The
// per-channel constants of a feature quad are loaded once and shared by the MT row tiles, and the
// next quad's constants are requested before the current quad is processed, so the (global or LDS)
// load latency is paid once, not once per quad.
//   out0: this lane's row of row tile 0 in the destination (LDS staging buffer or global rows);
//   out_mt_stride: bytes between consecutive row tiles (32 rows); guard_rows: skip rows >= rows.
struct QuadConsts {
    int4 bf, M, Z, S;
};
template <bool FAST>
__device__ __forceinline__ QuadConsts load_quad_consts(const CPtrs& C, int n0) {
    QuadConsts q;
    q.bf = *(const int4*)(C.bias_fold + n0);
    q.M = *(const int4*)(C.M0 + n0);
    if (FAST) {
        q.Z = *(const int4*)(C.rz + n0);
        q.S = *(const int4*)(C.sh + n0);
    } else {
        q.Z = make_int4(0, 0, 0, 0);
        q.S = *(const int4*)(C.rshift + n0);
    }
    return q;
}
// FAST: every channel has 33 <= r <= 54, so (acc*M0 + 2^(r-1)) >> r + z_out collapses to
// (mulhi(acc, M0) + rz) >> sh with rz = 2^(r-33) + (z_out << sh), sh = r - 32 (same integers).
// HALF: the tiles were folded by fold_rows16 (two quads per tile, `hh` = this lane's half).
// clamp(x, lo, hi) for lo <= hi as one instruction: the median of the three
__device__ __forceinline__ int clamp_code(int x, int lo_v, int hi_s) {
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo_v), "s"(hi_s));
    return r;
}

template <int MT, int NB, bool ASYM, bool TAPS, bool FAST, bool HALF = false>
__device__ __forceinline__ void epi_hidden_wave(const int N, const int NT, const LayerTaps& T, const CPtrs& C,
                                                v16i (&acc)[NB][MT], v16i (&rs)[MT], int zw_s, int grp, int g,
                                                int64_t row_first, int64_t rows, bool guard_rows, int z_out, int lo,
                                                int8_t* out0, int64_t out_mt_stride, bool packed, int n_store,
                                                int hh = 0) {
    constexpr int QT = HALF ? 2 : 4;  // quads per tile
    constexpr int NQ = NB * QT;
    auto n0_of = [&](int q) { return (grp * NB + q / QT) * 32 + 8 * (q % QT + (HALF ? 2 * hh : 0)) + 4 * g; };
    auto valid = [&](int q) { return grp * NB + q / QT < NT; };
    QuadConsts cur = load_quad_consts<FAST>(C, valid(0) ? n0_of(0) : 0);
    // clamp bounds as operands of the three-input median: one vector register, one scalar (the
    // instruction takes a single scalar source)
    int lo_v = lo;
    asm volatile("" : "+v"(lo_v));
    const int c255 = 255;
    static_for<0, NQ>([&](auto q_c) __attribute__((always_inline)) {
        constexpr int q = decltype(q_c)::value;
        constexpr int nb = q / QT, j = q % QT;
        QuadConsts nxt = cur;
        if (q + 1 < NQ) nxt = load_quad_consts<FAST>(C, valid(q + 1) ? n0_of(q + 1) : 0);
        if (valid(q)) {
            const int n0 = n0_of(q);
            const int bfv[4] = {cur.bf.x, cur.bf.y, cur.bf.z, cur.bf.w}, Mv[4] = {cur.M.x, cur.M.y, cur.M.z, cur.M.w};
            const int Zv[4] = {cur.Z.x, cur.Z.y, cur.Z.z, cur.Z.w}, Sv[4] = {cur.S.x, cur.S.y, cur.S.z, cur.S.w};
            static_for<0, MT>([&](auto mt_c) __attribute__((always_inline)) {
                constexpr int mt = decltype(mt_c)::value;
                const int64_t row = row_first + mt * 32;
                const bool row_ok = row < rows;
                uint32_t pack = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int val = acc[nb][mt][4 * j + i] + bfv[i];
                    if (ASYM) val -= zw_s * rs[mt][0];
                    if (TAPS) {
                        if (T.acc && row_ok && n0 + i < N) T.acc[row * N + n0 + i] = val;
                    }
                    int code;
                    if (FAST) code = clamp_code((__mulhi(val, Mv[i]) + Zv[i]) >> Sv[i], lo_v, c255);
                    else code = requant_code(val, Mv[i], Sv[i], z_out, lo);
                    // Padding features are zero in the signed domain where that matters: the per-tensor
                    // scheme sums whole padded rows of activations for its zero-point term.  With symmetric
                    // weights a padding column only ever meets zero weights, so its code is left as it comes.
                    if (ASYM && n0 + i >= N) code = 128;
                    if (TAPS) {
                        if (T.act && row_ok && n0 + i < N) T.act[row * N + n0 + i] = (uint8_t)code;
                    }
                    pack |= (uint32_t)code << (8 * i);
                }
                pack ^= 0x80808080u;
                if (out0 && (!guard_rows || row_ok)) {
                    int8_t* dst = out0 + mt * out_mt_stride + n0;
                    if (packed) {
                        if (n0 < n_store) *(uint32_t*)dst = pack;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (n0 + i < n_store) dst[i] = (int8_t)(pack >> (8 * i));
                    }
                }
            });
        }
        cur = nxt;
    });
}

// Last layer: y = (float)acc * m[n] for one tile, stored to y_row[n] (n < n_store) when y_row is
// given; when act_row is given the elementwise head (tanh or identity) is applied and stored too.
template <bool ASYM, bool TAPS, bool HALF = false>
__device__ __forceinline__ void epi_last_tile(const int N, const LayerTaps& T, const CPtrs& C, const v16i& c, int rs0,
                                              int zw_s, int nt, int g, int64_t row, bool row_ok, float* y_row,
                                              int n_store, float* act_row, int head, int hh = 0) {
#pragma unroll
    for (int j = 0; j < (HALF ? 2 : 4); ++j) {
        const int n0 = nt * 32 + 8 * (j + (HALF ? 2 * hh : 0)) + 4 * g;
        int val[4];
        quad_acc<ASYM, TAPS>(N, T, C, c, j, n0, rs0, zw_s, row, row_ok, val);
        const float4 mm = *(const float4*)(C.m + n0);
        const float mv[4] = {mm.x, mm.y, mm.z, mm.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float y = (float)val[i] * mv[i];
            if (n0 + i < n_store) {
                if (y_row) y_row[n0 + i] = y;
                if (act_row) act_row[n0 + i] = head == AQ_HEAD_TANH ? tanh_head(y) : y;
            }
        }
    }
}

}  // namespace aq
