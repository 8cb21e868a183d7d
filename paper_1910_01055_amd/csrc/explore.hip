// Exploration on the actor (Sec. 4.1): Gaussian noise with a per-actor sigma on continuous actions,
// epsilon-greedy on argmax actions, applied in place to the actions a forward pass produced.
// Random numbers: the counter-based generator Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel
// random numbers: as easy as 1, 2, 3", SC'11), key = the caller's seed, counter = (batch row, block,
// step low word, step high word): every (row, step) has its own stream, nothing is stored.
#include "explore_device.hpp"
#include "kernels.hpp"

namespace aq {

namespace {
// one thread per (row, block of four features)
__global__ __launch_bounds__(256) void k_explore_gaussian(float* __restrict__ actions, int64_t rows, int A, int blocks,
                                                          const float* __restrict__ sigma, uint32_t k0, uint32_t k1,
                                                          uint32_t s0, uint32_t s1) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * blocks) return;
    const int64_t b = i / blocks;
    const int q = (int)(i - b * blocks);
    const U4 r = philox4x32_10(U4{(uint32_t)b, (uint32_t)q, s0, s1}, k0, k1);
    float z[4];
    box_muller(r.x, r.y, z[0], z[1]);
    box_muller(r.z, r.w, z[2], z[3]);
    const float sg = sigma[b];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = 4 * q + j;
        if (n < A) actions[b * A + n] = actions[b * A + n] + sg * z[j];
    }
}

__global__ __launch_bounds__(256) void k_explore_eps_greedy(int32_t* __restrict__ idx, int64_t rows, int A, float epsilon,
                                                            uint32_t k0, uint32_t k1, uint32_t s0, uint32_t s1) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= rows) return;
    const U4 r = philox4x32_10(U4{(uint32_t)b, 0xFFFFFFFFu, s0, s1}, k0, k1);
    const float u = (float)(r.x >> 8) * 5.9604644775390625e-8f;
    if (u < epsilon) idx[b] = (int32_t)__umulhi(r.y, (uint32_t)A);
}
}  // namespace

aq_status launch_explore(void* d_actions, int64_t rows, int A, int head, const float* d_sigma, float epsilon,
                         uint64_t seed, uint64_t step, hipStream_t st) {
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32), s0 = (uint32_t)step, s1 = (uint32_t)(step >> 32);
    if (head == AQ_HEAD_ARGMAX) {
        hipLaunchKernelGGL(k_explore_eps_greedy, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st,
                           (int32_t*)d_actions, rows, A, epsilon, k0, k1, s0, s1);
    } else {
        const int blocks = (A + 3) / 4;
        const int64_t n = rows * blocks;
        hipLaunchKernelGGL(k_explore_gaussian, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (float*)d_actions,
                           rows, A, blocks, d_sigma, k0, k1, s0, s1);
    }
    return hipGetLastError() == hipSuccess ? AQ_OK : AQ_EHIP;
}

}  // namespace aq
