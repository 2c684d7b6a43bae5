// Sign binarisation and bit packing (paper Eq. 3), and the per-layer scale mean|w|.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

// One wavefront turns 64 consecutive elements of a row into one 64-bit ballot: a coalesced 256-byte
// read, two 32-bit words written.  `w32` is the row length of the output in 32-bit words (for 64-bit
// packing it is twice the 64-bit word count, so the bytes are the same little-endian words).
__global__ __launch_bounds__(256) void pack_sign_kernel(const float* __restrict__ X, int64_t rows, int64_t K,
                                                        int64_t w32, uint32_t* __restrict__ out) {
    const int lane = lane_id();
    const int64_t chunks = (K + 63) / 64;
    const int64_t tasks = rows * chunks;
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);
    for (int64_t task = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave); task < tasks;
         task += nwaves) {
        const int64_t row = task / chunks;
        const int64_t c = task - row * chunks;
        const int64_t k = c * 64 + lane;
        const bool p = (k < K) && sign_bit(X[row * K + k]);
        const unsigned long long mask = __ballot(p);
        if (lane < 2) {
            const int64_t w = 2 * c + lane;
            if (w < w32) out[row * w32 + w] = (uint32_t)(mask >> (32 * lane));
        }
    }
}

// mean|w| over `count` elements: one workgroup, every thread keeps an fp64 partial over a fixed
// strided subset, then a fixed tree over LDS.  The order never depends on timing, so the result is
// reproducible bit for bit.  Off the per-frame path (runs once per layer when a model is prepared).
__global__ __launch_bounds__(1024) void mean_abs_kernel(const float* __restrict__ W, int64_t count,
                                                        float* __restrict__ out) {
    __shared__ double part[1024];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += 1024) s += (double)__builtin_fabsf(W[i]);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int stride = 512; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) part[threadIdx.x] += part[threadIdx.x + stride];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = (float)(part[0] / (double)count);
}

}  // namespace bnn
