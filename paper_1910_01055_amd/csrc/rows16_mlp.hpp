// Whole-network int8 MLP for small policies (Sec. 3.1 actor inference on the 8-bit policy of Sec. 3.2): one
// workgroup of 8 wavefronts owns 16 * MT batch rows (MT = 1, 2 or 4 row tiles) from the observation to the action.
//
// At these sizes (a few hundred features per layer) a launch at small batch holds a fraction of a microsecond
// of matrix-core work; its time is the chain of round trips and vector-ALU phases inside one workgroup.  This
// kernel is laid out to keep that chain short:
//   - v_mfma_i32_16x16x64_i8: a tile is 16 features x 16 batch rows, so a 16-row block fills it (no
//     don't-care rows, no fold afterwards) and K = 256 is four dependent MFMAs instead of eight; a wavefront
//     owns 32 features = two independent accumulator chains;
//   - the kernel arguments fit one 64-byte line and hold what the observation addresses need; everything else
//     about the network - every layer's pointers and sizes, the activation scales and zero-points, the
//     short-form flags - comes from the device-resident description by one burst of scalar loads right after
//     the observation requests: no layer waits for a descriptor;
//   - weights and per-channel constants go from global memory straight to registers, one layer ahead: all
//     of a layer's operands (at most 8 KiB per wavefront) are requested at the start of the previous layer,
//     the constants of its epilogue too.  A lane's four features of a tile are shared by the 16 lanes of its
//     row, so each lane fetches one 16-byte piece (array x tile) and the epilogue takes its operands from the
//     row's lanes by DPP row broadcasts: one load instruction per wavefront and layer instead of eight (the
//     CU's single vector memory path, 64 B / clock, is what the eight wavefronts queue for), no staging in
//     LDS, no barrier to publish them;
//   - LayerNorm statistics cross the wavefronts once: every wavefront reduces its 32 features to (sum, sum of
//     squared deviations from its own mean), and the eight pairs combine exactly (the pairwise update of
//     Chan, Golub, LeVeque 1979), so the layer has one barrier where a mean pass followed by a deviation
//     pass has two;
//   - one barrier per layer; the narrow last layer is split over all wavefronts (feature tile x K).
//
// Weights are read from the library's 32 x 32 operand tiles unchanged: the 16-byte piece of lane
// (n % 32) + 32 * ((k % 32) / 16) of tile (n / 32, k / 32) is what lane (n % 16) + 16 * g of the 16 x 16 x 64
// operand needs when k-group g of a 64-wide k-step is taken to mean bytes 16 g .. 16 g + 15 of it.
//
// MT > 1 (large batches): a wavefront's operands serve MT row tiles, so the weight bytes through the CU's vector
// memory path per row shrink by MT, and the kernel is kept within 128 registers so that two workgroups share
// a CU: while one sits in a barrier or waits for LDS, the other's epilogue has the vector ALU.
//
// ASYM (per-tensor asymmetric weights, the scheme Sec. 3.2 writes out): the accumulator needs - z_w' sum_k a_s per
// batch row on top of the folded bias; the row sums come from one extra MFMA per k-step against an all-ones
// operand (the matrix cores are idle most of the time here), which leaves them in the lanes that hold the row's
// accumulators.  Padding features are then written as zero codes, because the next layer sums whole padded rows.
//
// Shapes: fp32 or 8-bit observations at a 16-byte aligned address, one to four fully connected layers, first-layer
// K and hidden widths at most 256, last layer at most 64 outputs.
#pragma once
#include "explore_device.hpp"
#include "int8_device.hpp"

namespace aq {
namespace r16 {

constexpr int RW = 8;          // wavefronts per workgroup
constexpr int RT = RW * 64;    // threads per workgroup
constexpr int RLD = 272;       // LDS row stride, bytes: 256 codes + 16 (16-byte operand reads of 8 rows hit 32 different banks)
constexpr int RMAXL = 4;       // layers
constexpr int RMAXK = 256;     // widest layer input / hidden layer
constexpr int RSTEPS = 4;      // k-steps of 64 per layer at most

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float unif(float v) { return __int_as_float(uni(__float_as_int(v))); }
template <class T>
__device__ __forceinline__ T* uni_ptr(T* p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (T*)(((uint64_t)hi << 32) | lo);
}

constexpr float K2_LOG2E = 2.885390081777927f;  // 2 log2(e): tanh(y) = 1 - 2 / (2^(K2 y) + 1)

// what the kernel uses of one layer, read from the device-resident description into scalar registers
struct R16Layer {
    const int8_t* wp;       // packed weights, [NT][KS] tiles of 1 KiB
    const int32_t* pack;    // four [32 NT] arrays: bias_fold | M0 or m | rz or gamma | sh or beta
    const int32_t* rshift;  // [32 NT] shifts of the general requantization form
    int N, NT, KS, act;
};
// the kernel arguments besides the description's address: 56 bytes, one 64-byte line together with it
struct R16Args {
    const float* obs;
    void* actions;
    int64_t batch;
    const float* ex_sigma;  // Gaussian exploration noise added where the actions are written, or NULL
    uint32_t ex_k0, ex_k1, ex_s0, ex_s1;
    int K0;
    int shape;  // number of layers | observations are 8-bit codes << 8
};
static_assert(sizeof(R16Args) == 56, "the kernel arguments must stay within one 64-byte line");

// lane N of every 16-lane row, broadcast to that row.  The old value is left undefined (a row broadcast writes
// every lane): no move that clears the destination first.
template <int N>
__device__ __forceinline__ int row_bcast(int v) {
    return __builtin_amdgcn_mov_dpp(v, 0x150 + N, 0xF, 0xF, true);
}
// r[i] = (lane N of the row's c[i]) + v[i] for a quad: the broadcast rides on the addition (v_add_u32_dpp, the
// form the compiler itself emits for some of these additions, but not for all), so a constant that is only
// ever added costs no instruction of its own.  The leading two wait states are the ones a DPP read needs after a
// vector instruction wrote its source; inside an asm block the compiler does not insert them.
template <int N>
__device__ __forceinline__ void add_row_bcast4(int (&r)[4], const v4i& c, const int (&v)[4]) {
    asm("s_nop 1\n\t"
        "v_add_u32_dpp %0, %4, %8 row_newbcast:%12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_u32_dpp %1, %5, %9 row_newbcast:%12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_u32_dpp %2, %6, %10 row_newbcast:%12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_u32_dpp %3, %7, %11 row_newbcast:%12 row_mask:0xf bank_mask:0xf bound_ctrl:1"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(c[0]), "v"(c[1]), "v"(c[2]), "v"(c[3]), "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "n"(N));
}
// The same as an operand of its own instruction.  Needed for shift amounts: the compiler folds a row broadcast
// into the shift (v_ashrrev_i32_dpp), and that instruction came back from the hardware with the broadcast
// applied to the shifted value instead of the amount (additions and plain moves are right).
template <int N>
__device__ __forceinline__ int row_bcast_mov(int v) {
    int r = row_bcast<N>(v);
    asm volatile("" : "+v"(r));
    return r;
}
// piece 2 * A + TL of this lane's row of constants (see load_c below)
#define AQ_R16_C(cm, A, TL, i) row_bcast<2 * (A) + (TL)>((cm)[i])
#define AQ_R16_CSH(cm, A, TL, i) row_bcast_mov<2 * (A) + (TL)>((cm)[i])

// sum over the four 16-lane rows of a wavefront (lane ^ 16, then lane ^ 32), the same value in every lane
__device__ __forceinline__ float sum_rows4(float s) {
    const auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(s), false, false);
    s = __uint_as_float(p[0]) + __uint_as_float(p[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(s), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// MT = row tiles of 16 batch rows per workgroup.  NH = number of hidden layers (the network has NH + 1 layers):
// a compile-time fact, so that every global load sits in straight-line code and the compiler can count exactly
// which ones an instruction has to wait for (with the layer count a run-time value, epilogues waited for the
// loads of the next layer requested just before them).
// LATE (one row tile, every workgroup with a CU to itself): when a layer's operands are requested, see
// request_layer below.
template <int MT, int NH, bool ASYM, bool TAPS, bool LATE = false>
__global__ __launch_bounds__(RT, MT == 1 ? 2 : 4) void k_mlp_rows16(const NetDev* __restrict__ netp, const R16Args c,
                                                                     const TapArgs t) {
    constexpr int ROWS = 16 * MT;
    constexpr int NQ = 2 * MT;  // observation quads per thread at most (64 quads per row)
    __shared__ __align__(16) int8_t s_buf[2][ROWS * RLD];
    __shared__ __align__(16) float s_red[ROWS * RW * 2];
    constexpr int NITEMS = MT == 4 ? 16 : 8;
    constexpr int PR = ASYM ? 5 : 4;  // words per lane and item: four accumulators (and the row sum of the activations)
    __shared__ __align__(16) int32_t s_part[NITEMS * PR * 64];  // accumulators of the last layer's items
    const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
    const int b = lane & 15, g4 = lane >> 4;  // this lane's batch row and k-group (operands) / feature quad (results)
    const int64_t row0 = (int64_t)blockIdx.x * ROWS;
    constexpr int nh = NH;

    // ---- the observations are requested first: their address needs nothing but the kernel arguments
    const int K0 = c.K0;
    const int64_t left = c.batch - row0;
    const int vrows = left < ROWS ? (int)left : ROWS;
    // a thread takes up to NQ (row, four consecutive k) quads: one 16-byte load where the rows are 16-byte aligned
    // (K0 a multiple of 4); otherwise four 4-byte loads (one row tile) or one 16-byte load at a 4-byte aligned
    // address (several row tiles; only the quad that ends the batch goes word by word)
    const int q4 = (K0 + 3) >> 2;  // quads per row, <= 64
    const float inv_q4 = __builtin_amdgcn_rcpf((float)q4);  // (1 ulp: far inside the margin below)
    const float* src1 = c.obs + row0 * K0;
    const bool k_al = (K0 & 3) == 0;
    const bool in_u8 = (c.shape >> 8) != 0;  // 8-bit observations are codes already (scale 1, zero-point 0)
    const int nquads = ROWS * q4;
    float4 ov[NQ];
    int om[NQ], ok4[NQ];
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        // (a slot past the last quad is skipped as a whole, by a scalar branch: with a narrow observation most
        // of the NQ slots are empty, and their index arithmetic alone was a tenth of the kernel's vector
        // instructions at four row tiles)
        om[u] = ROWS;
        ok4[u] = 0;
        ov[u] = float4{0.0f, 0.0f, 0.0f, 0.0f};
        if (u * RT >= nquads) continue;
        const int q = tid + u * RT;
        // q / q4: (q + 0.5) / q4 stays at least 0.5 / q4 away from every integer
        om[u] = (int)(((float)q + 0.5f) * inv_q4);
        ok4[u] = 4 * (q - om[u] * q4);
        if (om[u] < vrows) {
            if (in_u8) {
                // four codes: one word where the rows are 4-byte aligned, single bytes otherwise (kept in .x)
                const uint8_t* src = (const uint8_t*)c.obs + (row0 + om[u]) * K0 + ok4[u];
                uint32_t q4w;
                if (k_al) {
                    q4w = *(const uint32_t*)src;
                } else {
                    // (all four requested at once: bytes past the row's end re-read its last one and are masked
                    // out after the xor below)
                    const int last = K0 - 1 - ok4[u];  // >= 0
                    const uint32_t b0 = src[0], b1 = src[last < 1 ? last : 1], b2 = src[last < 2 ? last : 2],
                                   b3 = src[last < 3 ? last : 3];
                    q4w = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
                }
                ov[u].x = __uint_as_float(q4w);
            } else {
                const float* src = src1 + om[u] * K0 + ok4[u];
                if (k_al) {
                    ov[u] = *(const float4*)src;
                } else if (MT > 1 && !(left <= ROWS && om[u] == vrows - 1 && ok4[u] + 3 >= K0)) {
                    // rows at 4-byte aligned addresses, several row tiles per workgroup (where the requests
                    // count: cfg3 @ 65536 32.6 -> 31.75 us; a single 16-row tile, bound by latency, was 1 %
                    // slower with it): still one request, of 16 bytes at that alignment.  Past
                    // the row's end the words are the next row's first ones (they exist: only the batch's last
                    // row has none behind it) and are masked out once quantized
                    typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
                    const f4u v = *(const f4u*)src;
                    ov[u] = float4{v[0], v[1], v[2], v[3]};
                } else {  // the last words of the whole batch
                    ov[u].x = src[0];
                    if (ok4[u] + 1 < K0) ov[u].y = src[1];
                    if (ok4[u] + 2 < K0) ov[u].z = src[2];
                    if (ok4[u] + 3 < K0) ov[u].w = src[3];
                }
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // The network, from the device-resident description: every layer's facts, (scale, zero-point) of every
    // activation tensor and the short-form flags, all requested here in one burst of scalar loads (slots past
    // the last layer exist in the description and are not used).
    struct {
        R16Layer L[RMAXL];
        int head;
        float ln_eps;
    } a;
#pragma unroll
    for (int i = 0; i < RMAXL; ++i) {
        const LayerDev& s = netp->L[i];
        a.L[i] = R16Layer{uni_ptr(s.wp), uni_ptr(s.bias_fold), uni_ptr(s.rshift), uni(s.N), uni(s.NT), uni(s.KS), uni(s.act)};
    }
    const R16Layer LL = a.L[NH];
    a.head = uni(netp->head);
    a.ln_eps = unif(netp->ln_eps);
    float s_q[RMAXL + 1];
    int z_q[RMAXL + 1], fastf[RMAXL];
#pragma unroll
    for (int i = 0; i <= RMAXL; ++i) {
        s_q[i] = unif(netp->actq[i].s);
        z_q[i] = uni(netp->actq[i].z);
    }
#pragma unroll
    for (int i = 0; i < RMAXL; ++i) fastf[i] = uni(netp->fast[i]);
    // per-tensor weights: the tensor's zero-point in the signed domain (written by the quantizer)
    int zw_s[RMAXL];
#pragma unroll
    for (int i = 0; i < RMAXL; ++i) {
        zw_s[i] = 0;
        if (ASYM && i <= NH) zw_s[i] = uni(*(gint_ptr)uni_ptr(netp->L[i].z_w)) - 128;
    }
    v4i ones;
    ones[0] = ones[1] = ones[2] = ones[3] = 0x01010101;

    // hidden layer operands of this wavefront's 32 features: [k-step][16-feature tile]; loads are unconditional
    // from clamped addresses (an idle wavefront re-reads the last tile, a k-group past K the last k-tile: those
    // registers are not used, or meet zero activations)
    // (`first`: the first layer's requests are the kernel's first, with nothing older in flight whose wait they
    // could blur, so the k-steps past its K - most of them for a narrow observation - are skipped)
    auto load_w = [&](const R16Layer& L, v4i (&w)[RSTEPS][2], bool first) __attribute__((always_inline)) {
        const int nt = wave < L.NT ? wave : L.NT - 1;
        gv4i_ptr base = (gv4i_ptr)L.wp + (int64_t)nt * L.KS * 64 + (b + 32 * (g4 & 1));
#pragma unroll
        for (int s = 0; s < RSTEPS; ++s) {
            int ks = 2 * s + (g4 >> 1);
            ks = ks < L.KS ? ks : L.KS - 1;
            if (!first || 2 * s < L.KS) {
#pragma unroll
                for (int tl = 0; tl < 2; ++tl) w[s][tl] = base[ks * 64 + 16 * tl];
            }
        }
    };
    // ... and the constants of its epilogue.  The lanes of a 16-lane row all need the same eight 16-byte
    // pieces (four arrays x two tiles, the row's four consecutive features of each tile): lane j (and j + 8)
    // of the row fetches piece j = 2 * array + tile, the epilogue reads piece j from lane j of its row.
    auto load_c = [&](const R16Layer& L, bool pack_sh) __attribute__((always_inline)) {
        const int nt = wave < L.NT ? wave : L.NT - 1;
        const int Np = L.NT * 32;
        const int arr = (b >> 1) & 3, tl = b & 1;
        const int32_t* base = L.pack + arr * Np;
        if (arr == 3 && !pack_sh) base = L.rshift;
        return *(gv4i_ptr)(base + 32 * nt + 16 * tl + 4 * g4);
    };
    // The narrow last layer.  Its (16-feature tile, row tile) pairs go to different wavefronts; with fewer than
    // eight pairs the wavefronts left over split K.  item = pair + pairs * k-part; a wavefront takes items
    // wave and wave + 8 (sixteen pairs); every item covers at most two k-steps.
    struct LastMap {
        int t16, lg_t16, pairs, lg_pairs, ksplit;
    };
    auto last_map = [&](const R16Layer& L) __attribute__((always_inline)) {
        LastMap m;
        m.lg_t16 = L.NT;                                  // NT is 1 or 2: t16 = 2 NT = 2 or 4
        m.t16 = 1 << m.lg_t16;
        m.pairs = m.t16 * MT;                             // 2, 4, 8 or 16
        m.lg_pairs = m.lg_t16 + (MT == 4 ? 2 : MT - 1);
        m.ksplit = m.pairs >= RW ? 1 : RW >> m.lg_pairs;  // 4, 2 or 1
        return m;
    };
    constexpr int LI = MT == 4 ? 2 : 1;  // items per wavefront at most (sixteen pairs)
    constexpr int LJ = MT == 1 ? 2 : 4;  // k-steps per item at most: kp, kp + ksplit, ... below four
    auto load_wl = [&](const R16Layer& L, v4i (&w)[LI][LJ]) __attribute__((always_inline)) {
        const LastMap m = last_map(L);
#pragma unroll
        for (int it = 0; it < LI; ++it) {
            const int item = wave + RW * it;
            const int pair = item & (m.pairs - 1), kp = item >> m.lg_pairs;
            const int tile = pair & (m.t16 - 1);
            gv4i_ptr base = (gv4i_ptr)L.wp + (int64_t)(tile >> 1) * L.KS * 64 + (16 * (tile & 1) + b + 32 * (g4 & 1));
#pragma unroll
            for (int j = 0; j < LJ; ++j) {
                int ks = 2 * (kp + j * m.ksplit) + (g4 >> 1);
                ks = ks < L.KS ? ks : L.KS - 1;
                w[it][j] = base[ks * 64];
            }
        }
    };

    static_assert(!LATE || MT == 1, "two operand sets: one row tile only");
    constexpr bool WDBL = MT == 1;  // two operand sets: the next layer's are requested before this layer's MFMAs
    v4i w[WDBL ? 2 : 1][RSTEPS][2];  // operands of the layer being multiplied (and of the next one)
    v4i cst[2];           // this lane's piece of the constants of the layer whose epilogue runs, and of the next one
    v4i wl[LI][LJ];       // operands of the last layer
    auto is_ln = [&](int l) { return a.L[l].act == AQ_ACT_LN_TANH; };
    if constexpr (nh > 0) {
        load_w(a.L[0], w[0], true);
        cst[0] = load_c(a.L[0], is_ln(0) || fastf[0]);
    } else {
        load_wl(LL, wl);
    }

    // ---- observation quantize: a0 = clamp(round(x / s0) + z0, 0, 255), kept in the signed domain: four
    // values at a time, one aligned 4-byte LDS store per quad
    {
        int8_t* buf = s_buf[0];
        const QuantScale qs0 = make_quant_scale(s_q[0]);
        const float zf0 = (float)z_q[0];
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
            if (u * RT >= nquads) continue;  // (scalar branch: an empty slot costs nothing)
            if (om[u] < ROWS) {
                uint32_t pack = in_u8 ? __float_as_uint(ov[u].x) : quant_u8x4(ov[u], qs0, zf0);
                const int left_k = K0 - ok4[u];  // real values in this quad: 1..4 (or more)
                if (TAPS) {
                    if (t.a0 && om[u] < vrows) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (i < left_k) t.a0[(row0 + om[u]) * K0 + ok4[u] + i] = (uint8_t)(pack >> (8 * i));
                    }
                }
                pack ^= 0x80808080u;
                // zero (signed domain) past K0 and in the rows past the batch
                if (left_k < 4) pack &= (1u << (8 * left_k)) - 1u;
                if (om[u] >= vrows) pack = 0u;
                *(uint32_t*)(buf + om[u] * RLD + ok4[u]) = pack;
            }
        }
        // ... and up to the end of the last 64-wide k-step
        const int kz4 = ((K0 + 63) & ~63) >> 2, extra = kz4 - q4;  // words per row
        if (extra > 0) {
            const float inv_e = __builtin_amdgcn_rcpf((float)extra);
            for (int i = tid; i < ROWS * extra; i += RT) {
                const int m = (int)(((float)i + 0.5f) * inv_e), kq = q4 + i - m * extra;
                *(uint32_t*)(buf + m * RLD + 4 * kq) = 0u;
            }
        }
    }
    lds_barrier();

    // ---- hidden layers
    static_for<0, NH>([&](auto l_c) __attribute__((always_inline)) {
        constexpr int l = decltype(l_c)::value;
        const R16Layer& L = a.L[l];
        const int8_t* in = s_buf[l & 1];
        int8_t* out = s_buf[(l + 1) & 1];
        const bool active = wave < L.NT;
        const int ks64 = (L.KS + 1) >> 1;
        const bool ln = is_ln(l);
        LayerTaps T{nullptr, nullptr, nullptr};
        if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};

        // The operands and constants of a later layer j (j = nh: the last layer; beyond: nothing).  Their eight
        // loads per wavefront queue at the CU's single vector memory path (64 KiB per 256 x 256 layer at 64 B / clock):
        // eight wavefronts that request together leave the last one waiting a thousand clocks for its turn, and a
        // wavefront stuck there cannot start its epilogue.  One row tile (two operand sets): layer l + 1 is
        // requested in front of layer l's MFMAs, right behind the reads of its activations (the LDS round trip runs
        // while the requests queue).  LATE, a workgroup alone on its CU: only layer 1 is requested there; layer
        // l + 2 is requested at the end of layer l, behind its epilogue - the wavefronts get there one after the
        // other, the early ones would only wait at the barrier, and the set that layer l multiplied is free
        // (cfg2 at batch 4096 6.02 -> 5.91 us; with two workgroups on a CU it is the slower order: batch 8192
        // 7.88 -> 8.09 us).  More row tiles: layer l + 1 after layer l's MFMAs, into the registers they free (two
        // workgroups share the CU's register file, and the other workgroup's work hides the queueing).
        auto request_layer = [&](auto j_c) __attribute__((always_inline)) {
            constexpr int j = decltype(j_c)::value;
            if constexpr (j < nh) {
                load_w(a.L[j], w[WDBL ? j & 1 : 0], false);
                cst[j & 1] = load_c(a.L[j], is_ln(j) || fastf[j]);
            } else if constexpr (j == nh) {
                load_wl(LL, wl);
            }
        };
        auto request_next = [&]() __attribute__((always_inline)) { request_layer(std::integral_constant<int, l + 1>{}); };
        const v4i(&wcur)[RSTEPS][2] = w[WDBL ? l & 1 : 0];
        v4i acc[MT][2], rsa[MT];  // (rsa: every register of it ends up holding sum_k a_s of this lane's batch row)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][0] = acc[mt][1] = rsa[mt] = v4i{0, 0, 0, 0};
        {
            const int8_t* xrow = in + b * RLD + 16 * g4;
            if constexpr (MT == 1) {
                v4i bx[RSTEPS];
#pragma unroll
                for (int s = 0; s < RSTEPS; ++s) bx[s] = *(const v4i*)(xrow + 64 * s);
                // (the activation reads go first: their LDS round trip runs while the requests below queue)
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (!LATE || l == 0) request_next();
                __builtin_amdgcn_sched_barrier(0);
                if (active) {
#pragma unroll
                    for (int s = 0; s < RSTEPS; ++s) {
                        if (s < ks64) {
                            acc[0][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wcur[s][0], bx[s], acc[0][0], 0, 0, 0);
                            acc[0][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wcur[s][1], bx[s], acc[0][1], 0, 0, 0);
                            if (ASYM) rsa[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, bx[s], rsa[0], 0, 0, 0);
                        }
                    }
                }
            } else if (active) {
                // one k-step of the row tiles' operands is read ahead of the MFMAs of the step before
                v4i bx[2][MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) bx[0][mt] = *(const v4i*)(xrow + mt * 16 * RLD);
#pragma unroll
                for (int s = 0; s < RSTEPS; ++s) {
                    if (s < ks64) {
                        if (s + 1 < RSTEPS) {
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt) bx[(s + 1) & 1][mt] = *(const v4i*)(xrow + mt * 16 * RLD + 64 * (s + 1));
                        }
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            acc[mt][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wcur[s][0], bx[s & 1][mt], acc[mt][0], 0, 0, 0);
                            acc[mt][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wcur[s][1], bx[s & 1][mt], acc[mt][1], 0, 0, 0);
                            if (ASYM) rsa[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, bx[s & 1][mt], rsa[mt], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if constexpr (!WDBL) request_next();
        const v4i cm = cst[l & 1];
        const float s_out = s_q[l + 1];
        const int z_out = z_q[l + 1];
        const int nbase = 32 * wave + 4 * g4;
        int rowterm[MT];  // - z_w' sum_k a_s of this lane's row of each row tile
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) rowterm[mt] = ASYM ? -zw_s[l] * rsa[mt][0] : 0;
        // a layer with an odd number of 32-feature tiles: the next layer's last 64-wide k-step reads 32
        // columns nobody computes; the first idle wavefront zeroes them
        if ((L.NT & 1) && wave == L.NT) {
#pragma unroll
            for (int i = 0; i < 2 * MT; ++i) {
                const int e = lane + 64 * i;  // ROWS rows x 8 words
                *(uint32_t*)(out + (e >> 3) * RLD + 32 * L.NT + 4 * (e & 7)) = 0u;
            }
        }
        if (!ln) {
            if (active) {
                const int lo = L.act == AQ_ACT_RELU ? z_out : 0;
                int lo_v = lo;
                asm volatile("" : "+v"(lo_v));
                // (the form of the requantization is a fact of the layer: one branch around all the tiles)
                auto tiles = [&](auto fast_c) __attribute__((always_inline)) {
                    constexpr bool fast = decltype(fast_c)::value;
                    static_for<0, 2>([&](auto tl_c) __attribute__((always_inline)) {
                        constexpr int tl = decltype(tl_c)::value;
                        const int n0 = nbase + 16 * tl;
                        // multipliers and shift amounts once per tile (every row tile uses them); the integer
                        // bias and the rounding term ride on their additions
                        int cmul[4], csh[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            cmul[i] = AQ_R16_C(cm, 1, tl, i);
                            csh[i] = AQ_R16_CSH(cm, 3, tl, i);
                        }
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            const int64_t row = row0 + 16 * mt + b;
                            const bool row_ok = row < c.batch;
                            const int a4[4] = {acc[mt][tl][0], acc[mt][tl][1], acc[mt][tl][2], acc[mt][tl][3]};
                            int val[4];
                            add_row_bcast4<tl>(val, cm, a4);
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                if (ASYM) val[i] += rowterm[mt];
                                if (TAPS) {
                                    if (T.acc && row_ok && n0 + i < L.N) T.acc[row * L.N + n0 + i] = val[i];
                                }
                            }
                            int code[4];
                            if (fast) {
                                const int hi[4] = {__mulhi(val[0], cmul[0]), __mulhi(val[1], cmul[1]),
                                                   __mulhi(val[2], cmul[2]), __mulhi(val[3], cmul[3])};
                                int t[4];
                                add_row_bcast4<4 + tl>(t, cm, hi);
#pragma unroll
                                for (int i = 0; i < 4; ++i) code[i] = clamp_code(t[i] >> csh[i], lo_v, 255);
                            } else {
#pragma unroll
                                for (int i = 0; i < 4; ++i) code[i] = requant_code(val[i], cmul[i], csh[i], z_out, lo);
                            }
                            uint32_t pack = 0;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                // per-tensor weights: padding features are zero in the signed domain (the next
                                // layer sums whole padded rows); with symmetric weights they only meet zero weights
                                if (ASYM && n0 + i >= L.N) code[i] = 128;
                                if (TAPS) {
                                    if (T.act && row_ok && n0 + i < L.N) T.act[row * L.N + n0 + i] = (uint8_t)code[i];
                                }
                                pack |= (uint32_t)code[i] << (8 * i);
                            }
                            *(uint32_t*)(out + (16 * mt + b) * RLD + n0) = pack ^ 0x80808080u;
                        }
                    });
                };
                if (fastf[l]) tiles(std::true_type{});
                else tiles(std::false_type{});
            }
        } else {
            // LayerNorm over the layer's N features, tanh, re-quantize.  x = acc * (s_in s_w) in fp32; this
            // wavefront's features (32, fewer in the last tile) give (sum, squared deviations from their own
            // mean) per row.  Reciprocals of the feature counts and of the standard deviation come from the
            // reciprocal units (1 ulp, against a tolerance of 1e-4 on the result).
            const int n_w = L.N - 32 * wave < 0 ? 0 : (L.N - 32 * wave > 32 ? 32 : L.N - 32 * wave);
            const float inv_nw = __builtin_amdgcn_rcpf((float)(n_w > 0 ? n_w : 1));
            float x[MT][2][4];
            static_for<0, 2>([&](auto tl_c) __attribute__((always_inline)) {
                constexpr int tl = decltype(tl_c)::value;
                const int n0 = nbase + 16 * tl;
                // (padding features: their scale is stored as zero, so x = 0; idle wavefronts hold zero
                // accumulators and re-read the last tile's constants: their pair is not used)
                float cmul[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) cmul[i] = __int_as_float(AQ_R16_C(cm, 1, tl, i));
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const int a4[4] = {acc[mt][tl][0], acc[mt][tl][1], acc[mt][tl][2], acc[mt][tl][3]};
                    int val[4];
                    add_row_bcast4<tl>(val, cm, a4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (ASYM) val[i] += rowterm[mt];
                        if (TAPS) {
                            const int64_t row = row0 + 16 * mt + b;
                            if (T.acc && active && row < c.batch && n0 + i < L.N) T.acc[row * L.N + n0 + i] = val[i];
                        }
                        x[mt][tl][i] = (float)val[i] * cmul[i];
                    }
                }
            });
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float s = 0.0f;
#pragma unroll
                for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                    for (int i = 0; i < 4; ++i) s += x[mt][tl][i];
                s = sum_rows4(s);
                const float mean_w = s * inv_nw;
                float q = 0.0f;
                if (n_w == 32) {
#pragma unroll
                    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float d = x[mt][tl][i] - mean_w;
                            q = fmaf(d, d, q);
                        }
                } else {
#pragma unroll
                    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float d = x[mt][tl][i] - mean_w;
                            if (nbase + 16 * tl + i < L.N) q = fmaf(d, d, q);
                        }
                }
                q = sum_rows4(q);
                if (g4 == 0) *(float2*)(s_red + ((16 * mt + b) * RW + wave) * 2) = float2{s, q};
            }
            // the output scale's reciprocal: needed after the barrier, computed while waiting for it
            const QuantScale qs_out = make_quant_scale(s_out);
            const float c0 = qs_out.inv + (float)z_out, c1 = 2.0f * qs_out.inv;
            const float inv_N = __builtin_amdgcn_rcpf((float)L.N);
            // The eight (sum, squared deviations) pairs of a row are combined by the four lanes that hold the row:
            // lane group g4 takes the pairs of wavefronts 2 g4 and 2 g4 + 1 (one 16-byte read), the groups meet by
            // two lane exchanges.  A wavefront past the layer's width counts no features, the last one with
            // features may count fewer than 32.
            static_assert(RW == 8, "two pairs for each of the four lane groups of a row");
            float cnt[2], inv_cnt[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int left = L.N - 32 * (2 * g4 + j);
                const int n_j = left < 0 ? 0 : (left > 32 ? 32 : left);
                cnt[j] = (float)n_j;
                inv_cnt[j] = __builtin_amdgcn_rcpf((float)(n_j > 0 ? n_j : 1));
            }
            lds_barrier();
            float inv[MT], shift[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float4 v = *(const float4*)(s_red + (16 * mt + b) * RW * 2 + 4 * g4);
                const float sw[2] = {cnt[0] > 0.0f ? v.x : 0.0f, cnt[1] > 0.0f ? v.z : 0.0f};
                const float qw[2] = {cnt[0] > 0.0f ? v.y : 0.0f, cnt[1] > 0.0f ? v.w : 0.0f};
                const float mean = sum_rows4(sw[0] + sw[1]) * inv_N;
                // pairwise combination: sum of squared deviations from the common mean
                const float d0 = sw[0] * inv_cnt[0] - mean, d1 = sw[1] * inv_cnt[1] - mean;
                const float m2 = sum_rows4(fmaf(cnt[0] * d0, d0, qw[0]) + fmaf(cnt[1] * d1, d1, qw[1]));
                // (2 log2 e rides on the row's scale and shift and on the offset: exp2 then yields e^{2y})
                inv[mt] = __builtin_amdgcn_rsqf(fmaf(m2, inv_N, a.ln_eps)) * K2_LOG2E;
                shift[mt] = -mean * inv[mt];
            }
            if (active) {
                // code = round(t / s + z) with t = 1 - 2 r, r = 1 / (2^e + 1): round(c0 - c1 r)
                static_for<0, 2>([&](auto tl_c) __attribute__((always_inline)) {
                    constexpr int tl = decltype(tl_c)::value;
                    const int n0 = nbase + 16 * tl;
                    float gv[4], bv[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        gv[i] = __int_as_float(AQ_R16_C(cm, 2, tl, i));
                        bv[i] = __int_as_float(AQ_R16_C(cm, 3, tl, i)) * K2_LOG2E;
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        float rv[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            // r = 1 / (e^{2y} + 1) on the exp2 and reciprocal units for either sign (exp2
                            // saturates to 0 and +inf, rcp(inf) = 0)
                            const float e = __builtin_amdgcn_exp2f(fmaf(fmaf(x[mt][tl][i], inv[mt], shift[mt]), gv[i], bv[i]));
                            rv[i] = __builtin_amdgcn_rcpf(e + 1.0f);
                        }
                        uint32_t pack;
                        if (qs_out.rcp_ok) {
                            // the tanh value already carries rounding differences of its own, so the code is taken
                            // from t * (1/s) + z directly (it can differ from round(t/s) only at a rounding tie);
                            // the float -> byte conversion rounds half to even itself and saturates at 0 and 255
                            pack = 0;
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                pack = __builtin_amdgcn_cvt_pk_u8_f32(fmaf(rv[i], -c1, c0), i, pack);
                        } else {
                            pack = quant_code4(float4{fmaf(rv[0], -2.0f, 1.0f), fmaf(rv[1], -2.0f, 1.0f),
                                                      fmaf(rv[2], -2.0f, 1.0f), fmaf(rv[3], -2.0f, 1.0f)},
                                               qs_out, -z_out, 255 - z_out, z_out);
                        }
                        if (ASYM && n0 + 4 > L.N) {  // padding features: zero in the signed domain
                            const int keep = L.N - n0;  // < 4, may be <= 0
                            const uint32_t kmask = keep <= 0 ? 0u : (1u << (8 * keep)) - 1u;
                            pack = (pack & kmask) | (0x80808080u & ~kmask);
                        }
                        if (TAPS) {
                            const int64_t row = row0 + 16 * mt + b;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                if (row < c.batch && n0 + i < L.N) {
                                    if (T.ln) T.ln[row * L.N + n0 + i] = fmaf(rv[i], -2.0f, 1.0f);
                                    if (T.act) T.act[row * L.N + n0 + i] = (uint8_t)(pack >> (8 * i));
                                }
                            }
                        }
                        *(uint32_t*)(out + (16 * mt + b) * RLD + n0) = pack ^ 0x80808080u;
                    }
                });
            }
        }
        if constexpr (LATE) {
            __builtin_amdgcn_sched_barrier(0);
            request_layer(std::integral_constant<int, l + 2>{});
        }
        lds_barrier();
    });

    // ---- last layer: (feature tile, row tile) pairs over the wavefronts, K split where there are fewer than
    // eight pairs; accumulators meet in LDS, where the reduction pass finds them lane-major
    {
        const int l = nh;
        const R16Layer& L = LL;
        const int8_t* in = s_buf[l & 1];
        const int Np = L.NT * 32;
        const LastMap lm = last_map(L);
        const int ks64 = (L.KS + 1) >> 1;
#pragma unroll
        for (int it = 0; it < LI; ++it) {
            const int item = wave + RW * it;
            const int pair = item & (lm.pairs - 1), kp = item >> lm.lg_pairs;
            const int mt = pair >> lm.lg_t16;
            v4i acc = v4i{0, 0, 0, 0}, rsl = v4i{0, 0, 0, 0};
            if (item < lm.pairs * lm.ksplit) {
                v4i bx[LJ];
#pragma unroll
                for (int j = 0; j < LJ; ++j) {
                    const int s = kp + j * lm.ksplit;
                    bx[j] = *(const v4i*)(in + (16 * mt + b) * RLD + 64 * (s < RSTEPS ? s : RSTEPS - 1) + 16 * g4);
                }
#pragma unroll
                for (int j = 0; j < LJ; ++j)
                    if (kp + j * lm.ksplit < ks64) {
                        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wl[it][j], bx[j], acc, 0, 0, 0);
                        if (ASYM) rsl = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, bx[j], rsl, 0, 0, 0);
                    }
#pragma unroll
                for (int r = 0; r < 4; ++r) s_part[(item * PR + r) * 64 + lane] = acc[r];
                if (ASYM) s_part[(item * PR + 4) * 64 + lane] = rsl[0];
            }
        }
        // this thread's outputs of the reduction: (pair, register, lane) = (o >> 8, (o >> 6) & 3, o & 63) for
        // o = tid + 512 it, so that its LDS reads are conflict-free; their bias and scale (pair -> feature tile)
        constexpr int OI = 2 * MT;  // outputs per thread at most: pairs / 2
        int bf[OI];
        float ms[OI];
#pragma unroll
        for (int it = 0; it < OI; ++it) {
            const int o = tid + it * RT;
            const int pair = o >> 8;
            const int n = 16 * (pair & (lm.t16 - 1)) + 4 * ((o & 63) >> 4) + ((o >> 6) & 3);
            bf[it] = 0;
            ms[it] = 0.0f;
            if (pair < lm.pairs) {
                bf[it] = *(gint_ptr)(L.pack + n);
                ms[it] = __int_as_float(*(gint_ptr)(L.pack + Np + n));
            }
        }
        lds_barrier();
        float* ybuf = (float*)s_buf[l & 1];  // argmax policies: dequantized rows, stride Np + 1 (the input is free now)
        const int ldy = Np + 1;
        const int head = a.head;
        float held[OI];  // elementwise heads: this thread's actions, for the exploration pass below
#pragma unroll
        for (int it = 0; it < OI; ++it) {
            const int o = tid + it * RT;
            const int pair = o >> 8, r = (o >> 6) & 3, ln_ = o & 63;
            held[it] = 0.0f;
            if (pair < lm.pairs) {
                int v = 0, rsum = 0;
#pragma unroll
                for (int kp = 0; kp < 4; ++kp)
                    if (kp < lm.ksplit) {
                        v += s_part[((pair + lm.pairs * kp) * PR + r) * 64 + ln_];
                        if (ASYM) rsum += s_part[((pair + lm.pairs * kp) * PR + 4) * 64 + ln_];
                    }
                v += bf[it];
                if (ASYM) v -= zw_s[nh] * rsum;
                const int tile = pair & (lm.t16 - 1), mt = pair >> lm.lg_t16;
                const int n = 16 * tile + 4 * (ln_ >> 4) + r, m = 16 * mt + (ln_ & 15);
                const int64_t orow = row0 + m;
                const bool ok = orow < c.batch && n < L.N;
                if (TAPS) {
                    if (t.acc[l] && ok) t.acc[l][orow * L.N + n] = v;
                }
                const float y = (float)v * ms[it];
                if (head == AQ_HEAD_ARGMAX) {
                    ybuf[m * ldy + n] = y;
                } else if (ok) {
                    if (TAPS) {
                        if (t.y) t.y[orow * L.N + n] = y;
                    }
                    const float act = head == AQ_HEAD_TANH ? tanh_head(y) : y;
                    held[it] = act;
                    if (!c.ex_sigma) ((float*)c.actions)[orow * L.N + n] = act;
                }
            }
        }
        if (head != AQ_HEAD_ARGMAX) {
            // Exploration noise of Sec. 4.1, sigma per actor (= per batch row).  Its code (a counter-based generator
            // and Box-Muller per output) is long; inside the loop above a forward pass without exploration would
            // jump over it once per output, and each jump lands on instructions that are not in the cache.
            if (c.ex_sigma) {
#pragma unroll
                for (int it = 0; it < OI; ++it) {
                    const int o = tid + it * RT;
                    const int pair = o >> 8, r = (o >> 6) & 3, ln_ = o & 63;
                    const int tile = pair & (lm.t16 - 1), mt = pair >> lm.lg_t16;
                    const int n = 16 * tile + 4 * (ln_ >> 4) + r, m = 16 * mt + (ln_ & 15);
                    const int64_t orow = row0 + m;
                    if (pair < lm.pairs && orow < c.batch && n < L.N)
                        ((float*)c.actions)[orow * L.N + n] =
                            held[it] + c.ex_sigma[orow] * gaussian_draw((uint32_t)orow, n, c.ex_k0, c.ex_k1, c.ex_s0, c.ex_s1);
                }
            }
            return;
        }
        lds_barrier();
        // argmax over the dequantized rows (lowest index wins ties)
        if (tid < ROWS && row0 + tid < c.batch) {
            int best = 0;
            for (int n = 0; n < L.N; ++n) {
                const float y = ybuf[tid * ldy + n];
                if (TAPS) {
                    if (t.y) t.y[(row0 + tid) * L.N + n] = y;
                }
                if (y > ybuf[tid * ldy + best]) best = n;
            }
            ((int32_t*)c.actions)[row0 + tid] = best;
        }
    }
}

template <int MT, bool ASYM, bool TAPS, bool LATE = false>
aq_status launch_rows16_t(const NetDev* d_net, const R16Args& ra, const TapArgs& t, hipStream_t st) {
    const unsigned grid = (unsigned)((ra.batch + 16 * MT - 1) / (16 * MT));
    switch (ra.shape & 255) {
        case 1: hipLaunchKernelGGL((k_mlp_rows16<MT, 0, ASYM, TAPS, LATE>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        case 2: hipLaunchKernelGGL((k_mlp_rows16<MT, 1, ASYM, TAPS, LATE>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        case 3: hipLaunchKernelGGL((k_mlp_rows16<MT, 2, ASYM, TAPS, LATE>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        case 4: hipLaunchKernelGGL((k_mlp_rows16<MT, 3, ASYM, TAPS, LATE>), dim3(grid), dim3(RT), 0, st, d_net, ra, t); break;
        default: return AQ_ESHAPE;
    }
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}
// one translation unit per (MT, ASYM), so that the variants compile in parallel
#define AQ_ROWS16_DECL(MT, AS) \
    extern template aq_status launch_rows16_t<MT, AS, false>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t); \
    extern template aq_status launch_rows16_t<MT, AS, true>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t)
#define AQ_ROWS16_INST(MT, AS) \
    template aq_status launch_rows16_t<MT, AS, false>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t); \
    template aq_status launch_rows16_t<MT, AS, true>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t)
// ... and the one-row-tile variants for a workgroup that has its CU to itself
#define AQ_ROWS16_LATE_DECL(AS) \
    extern template aq_status launch_rows16_t<1, AS, false, true>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t); \
    extern template aq_status launch_rows16_t<1, AS, true, true>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t)
#define AQ_ROWS16_LATE_INST(AS) \
    template aq_status launch_rows16_t<1, AS, false, true>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t); \
    template aq_status launch_rows16_t<1, AS, true, true>(const NetDev*, const R16Args&, const TapArgs&, hipStream_t)

}  // namespace r16
}  // namespace aq
