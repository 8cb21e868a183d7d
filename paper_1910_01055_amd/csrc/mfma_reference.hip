// Measurement aid for the whole-network int8 kernels (Sec. 3.1 actor inference): the inner loop of the
// pipelined wide kernel and nothing else, so that a benchmark can report what the matrix cores sustain in that
// loop shape on the operands it is given -- the ceiling of k_mlp_wide's passes on this machine.
//
// One workgroup of 8 wavefronts per CU owns 64 activation rows of K = 1024 in LDS.  A k-step of a wavefront is
// four 32x32x32 MFMAs (2 feature tiles x 2 row tiles) on 2 x 1 KiB of weight operands read L2 -> registers in
// operand order, four k-steps in flight, and on two activation operands read from LDS two k-steps ahead: 16 KiB
// of weights and 32 MFMAs per CU and k-step, the ratio at which a CU's vector memory path (64 B/clock) and its
// matrix cores (8192 op/clock) are both saturated.  No epilogue, no barrier, no output but the accumulators of
// workgroup 0, which a test checks.  The matrix cores' clock under load depends on the operands (a loop on
// zeros runs about a third faster than one on random bytes), which is why the operands are arguments.
#include <mutex>

#include "kernels.hpp"

namespace aq {
namespace {

constexpr int RPF = 4;      // weight k-steps in flight per wavefront
constexpr int RLD = 1040;   // LDS row stride in bytes (K + 16: rows 16 bytes apart in the banks)
// LDS asked for: more than half of a CU's 160 KiB, so that every CU holds one workgroup, as under k_mlp_wide
constexpr int RLDS = 96 * 1024;
static_assert(64 * RLD <= RLDS, "the activation rows fit");

typedef int rv4i __attribute__((ext_vector_type(4)));
typedef int rv16i __attribute__((ext_vector_type(16)));

// weights: 16 feature tiles x 64 k-steps x 1 KiB; wavefront w owns tiles 2w and 2w + 1 and walks their 64 k-steps
// round and round.  acts: 64 rows x 1024 bytes, walked 32 k-steps round and round.
template <bool STREAM>
__global__ __launch_bounds__(512) void k_mfma_reference(const char* __restrict__ weights, const int8_t* __restrict__ acts,
                                                        int ksteps, int32_t* __restrict__ acc_out) {
    extern __shared__ __align__(16) int8_t x[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < 64 * 64; i += 512) {  // 16-byte pieces
        const int m = i >> 6, k16 = i & 63;
        *(rv4i*)(x + m * RLD + 16 * k16) = *(const rv4i*)(acts + m * 1024 + 16 * k16);
    }
    __syncthreads();
    const int8_t* xrow = x + (lane & 31) * RLD + (lane >> 5) * 16;
    const char* b0 = weights + (size_t)(2 * wave) * 64 * 1024 + lane * 16;
    const char* b1 = b0 + 64 * 1024;
    rv4i wreg[RPF][2], xf[2][2];
#pragma unroll
    for (int p = 0; p < RPF; ++p) {
        wreg[p][0] = *(const rv4i*)(b0 + p * 1024);
        wreg[p][1] = *(const rv4i*)(b1 + p * 1024);
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        xf[s][0] = *(const rv4i*)(xrow + s * 32);
        xf[s][1] = *(const rv4i*)(xrow + 32 * RLD + s * 32);
    }
    rv16i c[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0;
    for (int k = 0; k < ksteps; k += RPF) {
#pragma unroll
        for (int p = 0; p < RPF; ++p) {
            const int s = p & 1;
            c[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][0], xf[s][0], c[0][0], 0, 0, 0);
            c[0][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][0], xf[s][1], c[0][1], 0, 0, 0);
            c[1][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][1], xf[s][0], c[1][0], 0, 0, 0);
            c[1][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[p][1], xf[s][1], c[1][1], 0, 0, 0);
            const int kk = (k + p + 2) & 31;
            xf[s][0] = *(const rv4i*)(xrow + kk * 32);
            xf[s][1] = *(const rv4i*)(xrow + 32 * RLD + kk * 32);
            if (STREAM) {
                const int ks = (k + p + RPF) & 63;
                wreg[p][0] = *(const rv4i*)(b0 + ks * 1024);
                wreg[p][1] = *(const rv4i*)(b1 + ks * 1024);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // workgroup 0's accumulators, [wave][feature tile][row tile][register][lane]; the other workgroups computed
    // the same values
    if (blockIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_out[(((wave * 2 + i) * 2 + j) * 16 + r) * 64 + lane] = c[i][j][r];
    }
}

}  // namespace

aq_status launch_mfma_reference(const void* d_weights, const void* d_acts, int ksteps, bool stream_weights, int workgroups,
                                int32_t* d_acc, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute((const void*)k_mfma_reference<true>, hipFuncAttributeMaxDynamicSharedMemorySize, RLDS);
        if (attr_err == hipSuccess)
            attr_err = hipFuncSetAttribute((const void*)k_mfma_reference<false>, hipFuncAttributeMaxDynamicSharedMemorySize, RLDS);
    });
    if (attr_err != hipSuccess) return AQ_EHIP;
    if (stream_weights)
        hipLaunchKernelGGL((k_mfma_reference<true>), dim3((unsigned)workgroups), dim3(512), RLDS, st, (const char*)d_weights,
                           (const int8_t*)d_acts, ksteps, d_acc);
    else
        hipLaunchKernelGGL((k_mfma_reference<false>), dim3((unsigned)workgroups), dim3(512), RLDS, st, (const char*)d_weights,
                           (const int8_t*)d_acts, ksteps, d_acc);
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
