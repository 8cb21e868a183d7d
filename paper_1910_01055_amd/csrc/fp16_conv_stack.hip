// Half-precision actor (Sec. 3.2: fp16 policies): the leading convolutions of a frame policy in one
// launch, the binary16 counterpart of the 8-bit convolution stack.  One workgroup of 16 waves per image
// keeps the frame (converted from 8-bit codes, exact in binary16), every intermediate feature map and
// the layers' biases in LDS; only the last map goes to global memory.  With NHWC maps a k-step of 16
// values is 32 contiguous bytes of one kernel row of the input map, so an MFMA's activation operand is
// one 16-byte LDS read per lane.  Arithmetic and its order are those of the per-layer kernel: fp32
// accumulation over k in ascending order on the fp16 matrix cores, + bias, one rounding to binary16, ReLU.
//
// Shapes it takes (the host checks them; anything else goes one launch per layer): 8-bit frames at a
// 16-byte aligned address, two to four convolutions followed by a fully connected layer, kw*in_c a
// multiple of 16, stride*in_c and in_w*in_c multiples of 8, N a multiple of 4, frame up to 64 KB of
// codes, maps and biases within the LDS of one CU.
#include "kernels.hpp"

namespace aq {

namespace {
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f16acc __attribute__((ext_vector_type(16)));
typedef int i4v __attribute__((ext_vector_type(4)));

constexpr int FS_W = 16;          // waves per workgroup
constexpr int FS_T = FS_W * 64;
constexpr int FS_FU = 4;          // 16-byte pieces of the 8-bit frame per thread
constexpr int FS_MAXL = 4;        // convolution layers at most
constexpr size_t FS_MAX_LDS = 160 * 1024;

struct Fp16Stack {
    Fp16Layer L[FS_MAXL];
    int nc;
    int off_b;     // LDS byte offsets: second map buffer, biases
    int off_bias;
};

struct FsPlan {
    int nc, off_b, off_bias;
    size_t lds;
};

bool plan_fs(const Fp16Layer* L, int n_layers, const void* obs, int in_mode0, int64_t batch, FsPlan* p) {
    if (in_mode0 != 2 || ((uintptr_t)obs & 15) || batch > 0x7fffffffLL) return false;
    int nc = 0;
    while (nc < n_layers && !L[nc].fc) ++nc;
    if (nc < 2 || nc > FS_MAXL || nc >= n_layers) return false;
    size_t sz[2] = {0, 0}, bias_words = 0;
    for (int l = 0; l < nc; ++l) {
        const Fp16Layer& X = L[l];
        const int run = X.kw * X.in_c;
        if (run % 16 || (X.stride * X.in_c) % 8 || (X.in_w * X.in_c) % 8 || (X.N & 3)) return false;
        const size_t in_elems = (size_t)X.in_h * X.in_w * X.in_c;
        if (in_elems % 16) return false;
        if (in_elems * 2 > sz[l & 1]) sz[l & 1] = in_elems * 2;
        bias_words += (size_t)X.NT * 32;
    }
    const size_t frame = (size_t)L[0].in_h * L[0].in_w * L[0].in_c;
    if (frame > (size_t)FS_FU * FS_T * 16 || bias_words > FS_T) return false;
    p->nc = nc;
    p->off_b = (int)sz[0];
    p->off_bias = (int)(sz[0] + sz[1]);
    p->lds = sz[0] + sz[1] + bias_words * 4;
    return p->lds <= FS_MAX_LDS;
}

__global__ __launch_bounds__(FS_T) void k_fp16_conv_stack(const Fp16Stack S, const uint8_t* __restrict__ frames,
                                                         _Float16* __restrict__ out) {
    extern __shared__ __align__(16) int8_t smem[];
    // (the wave index stays a vector value here: it only selects tiles, in a loop; the tests that guard MFMAs are on
    // the scalar K.  An MFMA behind a lane-mask test could run under an empty mask, which the matrix cores ignore)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, n = lane & 31;
    const int64_t img = blockIdx.x;
    const int nc = S.nc;
    {   // frame (8-bit codes -> binary16) and all layers' biases -> LDS, requested together
        const Fp16Layer& L0 = S.L[0];
        const int pieces = (L0.in_h * L0.in_w * L0.in_c) >> 4;
        const i4v* src = (const i4v*)frames + img * pieces;
        i4v fr[FS_FU];
#pragma unroll
        for (int u = 0; u < FS_FU; ++u) {
            const int i = tid + u * FS_T;
            fr[u] = src[i < pieces ? i : pieces - 1];
        }
        float bv = 0.0f;
        int bias_words = 0;
        {
            int i = tid;
            const float* bp = nullptr;
#pragma unroll
            for (int l = 0; l < FS_MAXL; ++l) {
                if (l < nc) {
                    const int cnt = S.L[l].NT * 32;
                    if (bp == nullptr && i < cnt) bp = S.L[l].bias + i;
                    if (bp == nullptr) i -= cnt;
                    bias_words += cnt;
                }
            }
            if (bp) bv = *bp;
        }
        _Float16* fdst = (_Float16*)smem;
#pragma unroll
        for (int u = 0; u < FS_FU; ++u) {
            const int i = tid + u * FS_T;
            if (i < pieces) {
                h8 lo8, hi8;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    lo8[j] = (_Float16)(float)(((uint32_t)fr[u][j >> 2] >> (8 * (j & 3))) & 0xffu);
                    hi8[j] = (_Float16)(float)(((uint32_t)fr[u][2 + (j >> 2)] >> (8 * (j & 3))) & 0xffu);
                }
                *(h8*)(fdst + (int64_t)i * 16) = lo8;
                *(h8*)(fdst + (int64_t)i * 16 + 8) = hi8;
            }
        }
        if (tid < bias_words) ((float*)(smem + S.off_bias))[tid] = bv;
    }
    __syncthreads();
    int bias_at = 0;
#pragma unroll
    for (int l = 0; l < FS_MAXL; ++l) {
        if (l >= nc) break;
        const Fp16Layer& L = S.L[l];
        const _Float16* in = (const _Float16*)(smem + ((l & 1) ? S.off_b : 0));
        _Float16* map_out = (_Float16*)(smem + ((l & 1) ? 0 : S.off_b));
        const float* bias = (const float*)(smem + S.off_bias) + bias_at;
        const int R = L.oh * L.ow, RT = (R + 31) >> 5, NT = L.NT, N = L.N;
        const int KS = L.K >> 4;  // real k-steps (K is a multiple of 16; the packed tiles beyond hold zeros)
        const int run = L.kw * L.in_c, row_elems = L.in_w * L.in_c;
        const bool to_global = l == nc - 1;
        for (int tile = wave; tile < RT * NT; tile += FS_W) {
            const int nt = tile % NT, rt = tile / NT;
            const int r = rt * 32 + n;
            const int rc = r < R ? r : R - 1;  // a ragged last tile re-reads the last position; never stored
            const int oy = rc / L.ow, ox = rc - oy * L.ow;
            const _Float16* px = in + (oy * L.stride * L.in_w + ox * L.stride) * L.in_c + g * 8;
            const h8* wg = (const h8*)L.wp + ((int64_t)nt * L.KS16) * 64 + lane;
            f16acc acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
            int kr = 0;
            // operands of four k-steps at a time, two sets in flight
            auto load4 = [&](int k0, h8 (&A)[4], h8 (&X)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k = k0 + j;
                    A[j] = wg[(int64_t)(k < KS ? k : KS - 1) * 64];
                    X[j] = *(const h8*)px;
                    if (k < KS - 1) {   // 16 values on; at the end of a kernel row, down one map row
                        kr += 16;
                        const bool wrap = kr == run;
                        px += wrap ? 16 + row_elems - run : 16;
                        kr = wrap ? 0 : kr;
                    }
                }
            };
            auto mma4 = [&](int k0, h8 (&A)[4], h8 (&X)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (k0 + j < KS) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A[j], X[j], acc, 0, 0, 0);
            };
            h8 A0[4], X0[4], A1[4], X1[4];
            load4(0, A0, X0);
            int k0 = 0;
            for (; k0 + 8 < KS; k0 += 8) {
                load4(k0 + 4, A1, X1);
                mma4(k0, A0, X0);
                load4(k0 + 8, A0, X0);
                mma4(k0 + 4, A1, X1);
            }
            // the last eight k-steps or fewer, without the request for a group after them: past K a request
            // re-reads the last k-step and still takes its slot on the vector memory path
            if (k0 + 4 < KS) load4(k0 + 4, A1, X1);
            mma4(k0, A0, X0);
            mma4(k0 + 4, A1, X1);
            // + bias, one rounding to binary16, ReLU; lane = one output position, four features per quad
            _Float16* dst = to_global ? out + (img * R + r) * N : map_out + r * N;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n0 = nt * 32 + 8 * q + 4 * g;
                const float4 b4 = *(const float4*)(bias + n0);
                const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
                h4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    _Float16 v = (_Float16)(acc[4 * q + i] + bb[i]);
                    if (L.relu) v = v > (_Float16)0.0f ? v : (_Float16)0.0f;
                    o[i] = v;
                }
                if (r < R && n0 < N) *(h4*)(dst + n0) = o;
            }
        }
        bias_at += NT * 32;
        __syncthreads();
    }
}
}  // namespace

int fp16_conv_stack_layers(const Fp16Layer* L, int n_layers, const void* obs, int in_mode0, int64_t batch) {
    FsPlan p;
    return plan_fs(L, n_layers, obs, in_mode0, batch, &p) ? p.nc : 0;
}

aq_status launch_fp16_conv_stack(const Fp16Layer* L, int n_layers, const void* obs, int in_mode0, int64_t batch,
                                 void* out, hipStream_t st) {
    FsPlan p;
    if (!plan_fs(L, n_layers, obs, in_mode0, batch, &p)) return AQ_ESHAPE;
    Fp16Stack S{};
    for (int l = 0; l < p.nc; ++l) S.L[l] = L[l];
    S.nc = p.nc;
    S.off_b = p.off_b;
    S.off_bias = p.off_bias;
    static std::atomic<bool> attr_set{false};
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)k_fp16_conv_stack, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)FS_MAX_LDS) != hipSuccess)
            return AQ_EHIP;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_fp16_conv_stack, dim3((unsigned)batch), dim3(FS_T), p.lds, st, S, (const uint8_t*)obs,
                       (_Float16*)out);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
