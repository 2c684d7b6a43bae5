// Row-wise log-Softmax (paper Alg. 2 forward, last layer), in place on fp32 pre-activations.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// One workgroup of 256 threads per frame: logp[n] = z[n] - max - log(sum exp(z - max)).
// The row (a few thousand floats) is read three times; after the first pass it sits in L1/L2.
__global__ __launch_bounds__(256) void log_softmax_rows_kernel(float* __restrict__ Z, int M, int N) {
    __shared__ float red[4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        float* z = Z + (size_t)m * N;
        float mx = -__builtin_inff();
        for (int n = threadIdx.x; n < N; n += 256) mx = fmaxf(mx, z[n]);
        mx = wave_max(mx);
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        __syncthreads();
        float s = 0.0f;
        for (int n = threadIdx.x; n < N; n += 256) s += expf(z[n] - mx);
        s = wave_sum(s);
        if (lane == 0) red[wave] = s;
        __syncthreads();
        s = (red[0] + red[1]) + (red[2] + red[3]);
        __syncthreads();
        const float shift = mx + logf(s);
        for (int n = threadIdx.x; n < N; n += 256) z[n] = z[n] - shift;
    }
}

}  // namespace bnn
