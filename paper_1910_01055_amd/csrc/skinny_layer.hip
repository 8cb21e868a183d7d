// Fully connected layer at few rows (Sec. 3.1: the paper's actors run their policy on one observation
// at a time; Sec. 4.1: three hidden layers of 2048 units): the time goes into streaming the layer's
// 8-bit weights once, so the layer is cut into as many independent weight streams as possible.
//
// One workgroup of 8 waves owns one 32-row x 32-feature output tile; its waves split K eight ways.
// Each wave requests its whole share of the weights at once (up to 16 KiB in flight), stages its own
// K-slice of the activations in a private LDS region (no barrier before the MFMAs), and leaves a
// partial accumulator tile in LDS; after one barrier the 512 threads sum the eight partial sums of two
// outputs each and run the layer's epilogue (requantize, or dequantize for a LayerNorm / last layer).
// A 2048 x 2048 layer at batch 1 is 64 workgroups x 8 waves with all 4 MiB of weights in flight.
//
// Weights of at most 4 bits (the precision sweep of the paper's appendix on quantization-aware training; per-channel
// symmetric codes in [-7, 7]) can stay sub-byte in device memory (W4): two codes per byte, stored as c + 8, half
// the bytes to stream.  A wave expands them on the way into the operand registers with three vector instructions
// per 8 codes -- mask, shift, mask: the nibbles enter the MFMA as the unsigned values c + 8, and the surplus
// 8 * sum_k a[k] leaves again in the epilogue through the row sums of the activations, which four 4-byte dot
// products per k-step against all-ones collect beside the MFMA -- the accumulator the epilogue sees is the 8-bit
// path's, bit for bit.
#include "int8_device.hpp"

namespace aq {

namespace {
constexpr int SK_W = 8;                    // waves per workgroup = K split
// Weight k-steps a wave requests up front (template parameter PF): 4 or 8 for 8-bit weights (shares up to 4
// k-steps / longer ones, refilled as they are used), 8 or 16 = the whole share for nibble weights, whichever
// covers it.  Requests beyond the share re-read its last k-step (straight-line loads, so that the waits can
// be counted), and every such re-read takes its 16 clocks of the CU's vector memory path like a useful one: with
// 16 in flight for a share of 8, a 2048 x 2048 layer at batch 1 took 3.7 us instead of 3.2.
constexpr int SK_MAX_KCHUNK = 15;          // k-steps per wave that fit the LDS budget below
constexpr int SK_PART_LD = 65;             // words per register row of a partial tile (64 lanes + 1: the
                                           // feature-major reduction then spreads over the banks)
constexpr int SK_PART_WORDS = 17 * SK_PART_LD;

__host__ __device__ inline size_t skinny_lds_bytes(int kchunk) {
    return (size_t)SK_W * 32 * (kchunk * 32 + 16) + (size_t)SK_W * SK_PART_WORDS * 4;
}

// What the host knows of the layer at launch time, by value: with the pointers among the kernel arguments the
// weight requests go out after one scalar round trip instead of two (arguments, then the layer's entry of the
// device-resident description); only what the quantizer kernels write (activation scales and zero-points, the
// short-form flag, the weight zero-point) is still read from the description, off the critical path.
struct SkinnyLayer {
    const int8_t* wp;
    const uint8_t* w4;  // the same weights as nibbles (k_pack_nibbles), or NULL
    const int32_t *bias_fold, *M0, *rz, *sh, *rshift, *z_w;
    const float* m;
    int K, KS, N, act;
    int first, last, head, in_u8;
};

typedef int v2i __attribute__((ext_vector_type(2)));

// 16 signed codes in [-7, 7] (one lane's 16 bytes of a k-step, words d0 .. d3) -> 8 bytes: word j holds the codes of
// d(2j) as the low nibbles of its bytes and those of d(2j + 1) as the high nibbles, each stored as c + 8
__global__ __launch_bounds__(256) void k_pack_nibbles(const v4i* __restrict__ wp, v2i* __restrict__ w4, int64_t pieces) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= pieces) return;
    const v4i d = wp[i];
    auto nib = [](int w) {  // per byte: (c + 8) & 15
        uint32_t r = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) r |= ((((uint32_t)w >> (8 * b)) + 8u) & 15u) << (8 * b);
        return r;
    };
    v2i q;
    q[0] = (int)(nib(d[0]) | (nib(d[1]) << 4));
    q[1] = (int)(nib(d[2]) | (nib(d[3]) << 4));
    w4[i] = q;
}
}  // namespace

// TR: batch rows per workgroup, 32 or 16 (where 32 would leave CUs without a workgroup).
// W4: weights read as nibbles (per-channel symmetric only).  PF: see above.
template <bool ASYM, bool TAPS, int TR, bool W4, int PF>
__global__ __launch_bounds__(SK_W * 64) void k_layer_skinny(const NetDev* __restrict__ netp, const SkinnyLayer L,
                                                           const TapArgs t, const int l,
                                                           const LayerIO io, const int64_t rows, const int kchunk,
                                                           const int in_mode, const void* __restrict__ actions,
                                                           void* __restrict__ argmax_out) {
    extern __shared__ __align__(16) int8_t smem[];
    static_assert(!(ASYM && W4), "nibble weights are per-channel symmetric codes");
    constexpr bool RS = ASYM || W4;  // the epilogue needs the row sums of the activations
    const NetDev& a = *netp;
    LayerTaps T{nullptr, nullptr, nullptr};
    if (TAPS) T = LayerTaps{t.acc[l], t.act[l], t.ln[l]};
    // (the wave index as a scalar: what depends on it - this wave's k-steps - then branches on the scalar unit.
    // Left in a vector register it makes those tests lane masks, and a block that holds nothing but an MFMA may
    // lose its skip branch: the matrix cores do not honour an empty lane mask, the k-step would be added anyway)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = blockIdx.x;
    constexpr int tile_rows = TR;
    const int64_t row0 = (int64_t)blockIdx.y * tile_rows;
    const bool first = L.first != 0, last = L.last != 0;
    const bool ln = !last && L.act == AQ_ACT_LN_TANH;
    const int K = L.K, KS = L.KS, N = L.N;
    const int k0 = wave * kchunk, k1 = k0 + kchunk < KS ? k0 + kchunk : KS;
    const int LDX = kchunk * 32 + 16;
    int8_t* xs = smem + (size_t)wave * 32 * LDX;  // this wave's rows x its K slice
    int32_t* part = (int32_t*)(smem + (size_t)SK_W * 32 * LDX);

    // this thread's epilogue constants (its two outputs share one feature): requested up front, they
    // arrive behind the weights
    const int n_e = nt * 32 + (tid & 31);  // < N_pad: the constant arrays are padded
    const int c_bias = L.bias_fold[n_e], c_M0 = L.M0[n_e], c_rz = L.rz[n_e], c_sh = L.sh[n_e], c_r = L.rshift[n_e];
    const float c_m = L.m[n_e];
    const int z_out = last ? 0 : a.actq[l + 1].z;
    const int lo = (!last && L.act == AQ_ACT_RELU) ? z_out : 0;
    const int zw_s = W4 ? 8 : (ASYM ? L.z_w[0] - 128 : 0);
    const bool fast = !last && !ln && a.fast[l] != 0;
    const int head = L.head;
    const bool argmax_here = argmax_out != nullptr;  // last layer, argmax head, a single feature tile

    v16i pacc[1][1], prs[1];
    pacc[0][0] = zero16();
    prs[0] = zero16();
    if (k0 < k1) {
        // this wave's K slice of the tile's rows -> LDS (signed domain; zero beyond K).  Rows past the batch are
        // not staged at all: a batch row is a column of the MFMA's second operand, so whatever LDS holds there
        // only reaches accumulators of rows that are never stored (at batch 1 that is 31 of the 32 rows)
        const int kb0 = k0 * 32, kb1 = k1 * 32;  // byte range of K
        const int64_t left = rows - row0;
        const int vrows = left < tile_rows ? (int)left : tile_rows;
        // 8-bit activations, rows of K bytes with K a multiple of 16, 16-byte aligned: whole pieces.  The first
        // eight pieces per lane (all of them for slices up to 256 bytes) are requested ahead of the weights: they
        // are few, the MFMAs cannot start before they have been through LDS, and behind the eight wavefronts'
        // weight requests they would wait for 128 KiB to pass the CU's vector memory path.
        const int ppr = (kb1 - kb0) >> 4;  // pieces per row
        const int total = in_mode == 1 ? vrows * ppr : 0;
        // idx / ppr by a reciprocal: (idx + 0.5) / ppr stays at least 0.5 / ppr away from every integer, far
        // more than the rounding error at these magnitudes (an integer division costs about thirty vector
        // instructions, and this staging loop sits in front of the layer's MFMAs)
        const float inv_ppr = __builtin_amdgcn_rcpf((float)ppr);
        constexpr int SU = 8;
        auto piece_load = [&](int idx) __attribute__((always_inline)) {
            v4i v = {0, 0, 0, 0};
            if (idx < total) {
                const int m = (int)(((float)idx + 0.5f) * inv_ppr), c = idx - m * ppr;
                const int k = kb0 + c * 16;
                if (k < K) v = *(const v4i*)((const int8_t*)io.in + (row0 + m) * K + k);
            }
            return v;
        };
        auto piece_store = [&](int idx, const v4i& v) __attribute__((always_inline)) {
            if (idx < total) {
                const int m = (int)(((float)idx + 0.5f) * inv_ppr), c = idx - m * ppr;
                *(v4i*)(xs + m * LDX + c * 16) = v;
            }
        };
        v4i v0[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) v0[u] = piece_load(lane + u * 64);

        // the wave's whole weight share
        gv4i_ptr wptr[1];
        wptr[0] = (gv4i_ptr)L.wp + (int64_t)nt * KS * 64 + lane;
        v4i wreg[W4 ? 1 : PF][1];
        v2i w4r[W4 ? PF : 1];
        if constexpr (W4) {
            const v2i AQ_GLOBAL* w4p = (const v2i AQ_GLOBAL*)L.w4 + (int64_t)nt * KS * 64 + lane;
#pragma unroll
            for (int p = 0; p < PF; ++p) {  // (indices past the share are clamped; those registers are not used)
                const int k = k0 + p < k1 - 1 ? k0 + p : k1 - 1;
                w4r[p] = w4p[(int64_t)k * 64];
            }
        } else {
            mma_prefetch<1, PF>(wptr, k0, k1, wreg);
        }

        if (in_mode == 1) {
#pragma unroll
            for (int u = 0; u < SU; ++u) piece_store(lane + u * 64, v0[u]);
            for (int base = lane + 64 * SU; base < total; base += 64 * SU) {
                v4i v[SU];
#pragma unroll
                for (int u = 0; u < SU; ++u) v[u] = piece_load(base + u * 64);
#pragma unroll
                for (int u = 0; u < SU; ++u) piece_store(base + u * 64, v[u]);
            }
        } else {
            float s0 = 1.0f;
            int z0 = 0;
            if (first) {
                s0 = a.actq[0].s;
                z0 = a.actq[0].z;
            }
            const QuantScale qs0 = make_quant_scale(s0);
            const int kb = kb1 - kb0;
            const float inv_kb = __builtin_amdgcn_rcpf((float)kb);
            for (int idx = lane; idx < vrows * kb; idx += 64) {
                const int m = (int)(((float)idx + 0.5f) * inv_kb), kk = idx - m * kb;
                const int k = kb0 + kk;
                const int64_t row = row0 + m;
                int sv = 0;
                if (k < K) {
                    const int64_t off = row * K + k;
                    if (first) {
                        int code;
                        if (L.in_u8) code = ((const uint8_t*)io.in)[off];
                        else code = quant_code(((const float*)io.in)[off], qs0, -z0, 255 - z0) + z0;
                        if (TAPS) {
                            if (t.a0 && nt == 0) t.a0[off] = (uint8_t)code;
                        }
                        sv = code - 128;
                    } else {
                        sv = ((const int8_t*)io.in)[off];
                    }
                }
                xs[m * LDX + kk] = (int8_t)sv;
            }
        }
        // the slice is private to this wave: its own LDS writes only have to land
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        if constexpr (W4) {
            // the share is at most PF k-steps (the host's choice): every one of them has its registers already
            const int8_t* xrow = xs + (lane & 31) * LDX + (lane >> 5) * 16;
            int rsl = 0;  // this lane's share of its row's sum: the 16 bytes per k-step it feeds the MFMA
            // activation operands four k-steps ahead of their MFMAs (every k-step sits in its own conditional
            // block, where the compiler cannot move the LDS read up by itself)
            const int n_last = k1 - k0 - 1;
            v4i xr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xr[i] = *(const v4i*)(xrow + (i < n_last ? i : n_last) * 32);
            static_for<0, PF>([&](auto p_c) __attribute__((always_inline)) {
                constexpr int p = decltype(p_c)::value;
                if (k0 + p < k1) {
                    const v4i x = xr[p & 3];
                    xr[p & 3] = *(const v4i*)(xrow + (p + 4 < n_last ? p + 4 : n_last) * 32);
                    const v2i q = w4r[p];
                    v4i w;
                    w[0] = q[0] & 0x0F0F0F0F;
                    w[1] = (int)((uint32_t)q[0] >> 4) & 0x0F0F0F0F;
                    w[2] = q[1] & 0x0F0F0F0F;
                    w[3] = (int)((uint32_t)q[1] >> 4) & 0x0F0F0F0F;
                    pacc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x, pacc[0][0], 0, 0, 0);
#pragma unroll
                    for (int j = 0; j < 4; ++j) rsl = __builtin_amdgcn_sdot4(x[j], 0x01010101, rsl, false);
                }
            });
            // a row's two k-halves sit in lanes r and r + 32; both get the whole sum (where the all-ones MFMA of
            // the per-tensor scheme leaves it)
            prs[0][0] = rsl + __shfl_xor(rsl, 32, 64);
        } else {
            mma_run<1, 1, ASYM, PF>(wptr, wreg, xs, LDX, k0, k1, k0, pacc, prs, lane);
        }
    }
    {
        int32_t* mine = part + wave * SK_PART_WORDS + lane;
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[r * SK_PART_LD] = pacc[0][0][r];
        if (RS) mine[16 * SK_PART_LD] = prs[0][0];
    }
    __syncthreads();

    // reduction + epilogue: thread -> (row m, feature n) with the feature index fastest, so that the
    // global stores of a row are contiguous
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int m = (tid >> 5) + 16 * it, nl = tid & 31;
        if (m >= tile_rows) break;  // (a 16-row tile: the upper half of the MFMA tile belongs to nobody)
        const int reg = 4 * (nl >> 3) + (nl & 3), lsrc = m + 32 * ((nl >> 2) & 1);
        int v = 0, rsum = 0;
#pragma unroll
        for (int kp = 0; kp < SK_W; ++kp) {
            const int32_t* src = part + kp * SK_PART_WORDS + lsrc;
            v += src[reg * SK_PART_LD];
            if (RS) rsum += src[16 * SK_PART_LD];
        }
        const int n = nt * 32 + nl;
        const int64_t row = row0 + m;
        if (argmax_here) {
            // the whole output row sits in this tile, one feature per lane of a 32-lane group: the
            // action index (lowest index among equal logits) is a shuffle reduction away
            const bool ok = row < rows && n < N;
            int vv = v + c_bias;
            if (RS) vv -= zw_s * rsum;
            if (TAPS) {
                if (T.acc && ok) T.acc[row * N + n] = vv;
            }
            float y = ok ? (float)vv * c_m : -INFINITY;
            if (ok && io.y) io.y[row * N + n] = y;
            int best = n;
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) {
                const float yo = __shfl_xor(y, o, 32);
                const int bo = __shfl_xor(best, o, 32);
                if (yo > y || (yo == y && bo < best)) {
                    y = yo;
                    best = bo;
                }
            }
            if (nl == 0 && row < rows) ((int32_t*)argmax_out)[row] = best;
            continue;
        }
        if (row >= rows || n >= N) continue;
        v += c_bias;
        if (RS) v -= zw_s * rsum;
        if (TAPS) {
            if (T.acc) T.acc[row * N + n] = v;
        }
        if (ln) {
            io.ln_x[row * N + n] = (float)v * c_m;
        } else if (last) {
            const float y = (float)v * c_m;
            if (io.y) io.y[row * N + n] = y;
            if (actions) ((float*)actions)[row * N + n] = head == AQ_HEAD_TANH ? tanh_head(y) : y;
        } else {
            int code;
            if (fast) code = min(max((__mulhi(v, c_M0) + c_rz) >> c_sh, lo), 255);
            else code = requant_code(v, c_M0, c_r, z_out, lo);
            if (TAPS) {
                if (T.act) T.act[row * N + n] = (uint8_t)code;
            }
            io.out[row * N + n] = (int8_t)(code - 128);
        }
    }
}

// the last layer of an argmax policy whose logits fit one tile: the action index comes out of the
// same launch
bool skinny_layer_does_argmax(const FwdArgs& a, int l) {
    return l == a.net.n_layers - 1 && a.net.head == AQ_HEAD_ARGMAX && a.net.L[l].NT == 1;
}

bool skinny_layer_supported(const LayerDev& L, int64_t rows) {
    const bool fc = L.kh == 1 && L.kw == 1 && L.in_h == 1 && L.in_w == 1;
    if (!fc) return false;
    const int kchunk = (L.KS + SK_W - 1) / SK_W;
    if (kchunk > SK_MAX_KCHUNK) return false;
    return (rows + 15) / 16 <= 65535;
}

aq_status launch_pack_nibbles(const int8_t* wp, uint8_t* w4, int64_t pieces, hipStream_t st) {
    hipLaunchKernelGGL(k_pack_nibbles, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (const v4i*)wp, (v2i*)w4, pieces);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

namespace {
struct SkinnyCall {
    dim3 grid;
    size_t lds;
    hipStream_t st;
    const NetDev* d_net;
    SkinnyLayer sl;
    TapArgs t;
    int l;
    LayerIO io;
    int64_t rows;
    int kchunk, in_mode;
    const void* actions;
    void* argmax_out;
};
template <bool AS, bool TP, int TRV, bool W4V, int PFV>
aq_status skinny_launch(const SkinnyCall& c) {
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_layer_skinny<AS, TP, TRV, W4V, PFV>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return AQ_EHIP;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_layer_skinny<AS, TP, TRV, W4V, PFV>), c.grid, dim3(SK_W * 64), c.lds, c.st, c.d_net, c.sl, c.t,
                       c.l, c.io, c.rows, c.kchunk, c.in_mode, c.actions, c.argmax_out);
    return AQ_OK;
}
template <bool AS, bool TP, int TRV, bool W4V>
aq_status skinny_pick_depth(const SkinnyCall& c) {
    if (!W4V && c.kchunk <= 4) return skinny_launch<AS, TP, TRV, W4V, W4V ? 8 : 4>(c);
    if (c.kchunk <= 8 || !W4V) return skinny_launch<AS, TP, TRV, W4V, 8>(c);
    return skinny_launch<AS, TP, TRV, W4V, W4V ? 16 : 8>(c);
}
template <bool AS, bool W4V>
aq_status skinny_pick_tile(const SkinnyCall& c, bool taps, int tile_rows) {
    if (taps) return tile_rows == 16 ? skinny_pick_depth<AS, true, 16, W4V>(c) : skinny_pick_depth<AS, true, 32, W4V>(c);
    return tile_rows == 16 ? skinny_pick_depth<AS, false, 16, W4V>(c) : skinny_pick_depth<AS, false, 32, W4V>(c);
}
}  // namespace

aq_status launch_layer_skinny(const FwdArgs& a, int l, const LayerIO& io, hipStream_t st) {
    const LayerDev& L = a.net.L[l];
    const int64_t rows = a.c.batch;
    const bool first = l == 0, last = l == a.net.n_layers - 1;
    const int kchunk = (L.KS + SK_W - 1) / SK_W;
    const size_t lds = skinny_lds_bytes(kchunk);
    // whole 16-byte pieces need 8-bit rows whose length is a multiple of 16, at an aligned address
    const int in_mode = (!first && (L.K & 15) == 0 && ((uintptr_t)io.in & 15) == 0) ? 1 : 0;
    const void* actions = (last && a.net.head != AQ_HEAD_ARGMAX) ? a.c.actions : nullptr;
    void* argmax_out = skinny_layer_does_argmax(a, l) ? a.c.actions : nullptr;
    // 16-row tiles where 32-row tiles would give fewer workgroups than CUs (half of each MFMA tile is then idle,
    // but a workgroup stages half the activation bytes and twice as many CUs stream weights)
    const int tile_rows = (rows > 16 && (int64_t)L.NT * ((rows + 31) / 32) < 256) ? 16 : 32;
    dim3 grid((unsigned)L.NT, (unsigned)((rows + tile_rows - 1) / tile_rows));
    const bool taps = any_taps(a);
    const bool asym = a.net.asym != 0;
    const uint8_t* w4 = asym ? nullptr : a.w4[l];
    const SkinnyLayer sl{L.wp, w4, L.bias_fold, L.M0, L.rz, L.sh, L.rshift, L.z_w, L.m, L.K, L.KS, L.N, L.act,
                         first, last, a.net.head, a.net.in_u8};
    const SkinnyCall call{grid, lds, st, a.d_net, sl, a.t, l, io, rows, kchunk, in_mode, actions, argmax_out};
    aq_status s;
    if (asym) s = skinny_pick_tile<true, false>(call, taps, tile_rows);
    else if (w4) s = skinny_pick_tile<false, true>(call, taps, tile_rows);
    else s = skinny_pick_tile<false, false>(call, taps, tile_rows);
    if (s != AQ_OK) return s;
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
