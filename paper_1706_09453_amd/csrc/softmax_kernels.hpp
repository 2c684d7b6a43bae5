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

// The same with the whole row held in registers (N <= 256 * PER): one read and one write of the tensor.
// Thread t owns elements 4 t .. 4 t + 3 of every 1024-element chunk (16-byte accesses when N % 4 == 0).
template <int PER>
__global__ __launch_bounds__(256) void log_softmax_rows_reg_kernel(float* __restrict__ Z, int M, int N) {
    __shared__ float red[4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const bool vec = (N & 3) == 0;
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        float* z = Z + (size_t)m * N;
        float v[PER];
        const float neg_inf = -__builtin_inff();
#pragma unroll
        for (int c = 0; c < PER / 4; ++c) {
            const int n = c * 1024 + 4 * (int)threadIdx.x;
            if (vec && n + 3 < N) {
                const float4 q = *reinterpret_cast<const float4*>(z + n);
                v[4 * c] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[4 * c + i] = (n + i < N) ? z[n + i] : neg_inf;
            }
        }
        float mx = neg_inf;
#pragma unroll
        for (int i = 0; i < PER; ++i) mx = fmaxf(mx, v[i]);
        mx = wave_max(mx);
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        __syncthreads();
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < PER; ++i) s += __expf(v[i] - mx);
        s = wave_sum(s);
        if (lane == 0) red[wave] = s;
        __syncthreads();
        s = (red[0] + red[1]) + (red[2] + red[3]);
        __syncthreads();
        const float shift = mx + __logf(s);
#pragma unroll
        for (int c = 0; c < PER / 4; ++c) {
            const int n = c * 1024 + 4 * (int)threadIdx.x;
            if (vec && n + 3 < N) {
                float4 q;
                q.x = v[4 * c] - shift; q.y = v[4 * c + 1] - shift; q.z = v[4 * c + 2] - shift; q.w = v[4 * c + 3] - shift;
                *reinterpret_cast<float4*>(z + n) = q;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (n + i < N) z[n + i] = v[4 * c + i] - shift;
            }
        }
    }
}

// Output layer, second half: the row starts with N int16 integer products (written by the product kernel);
// z[n] = fma(scale[n], dot[n], bias[n]) is formed here, then log-Softmax, and the fp32 log-posteriors replace
// the row.  Every thread holds its elements in registers across the barriers of the two reductions, so all
// reads of the row are complete before the first write.  Needs N % 4 == 0, N <= 256 * PER, 16-byte aligned rows.
template <int PER>
__global__ __launch_bounds__(256) void log_softmax_rows_i16_kernel(float* __restrict__ Z, const float* __restrict__ scale,
                                                                   const float* __restrict__ bias, int M, int N) {
    __shared__ float red[4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const float neg_inf = -__builtin_inff();
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        float* z = Z + (size_t)m * N;
        const uint16_t* d16 = reinterpret_cast<const uint16_t*>(z);
        float v[PER];
#pragma unroll
        for (int c = 0; c < PER / 4; ++c) {
            const int n = c * 1024 + 4 * (int)threadIdx.x;
            if (n < N) {
                const uint2 h = *reinterpret_cast<const uint2*>(d16 + n);
                const float4 sc = scale ? *reinterpret_cast<const float4*>(scale + n) : make_float4(1.f, 1.f, 1.f, 1.f);
                const float4 bi = bias ? *reinterpret_cast<const float4*>(bias + n) : make_float4(0.f, 0.f, 0.f, 0.f);
                v[4 * c + 0] = affine(sc.x, (float)(int)(int16_t)(h.x & 0xFFFFu), bi.x);
                v[4 * c + 1] = affine(sc.y, (float)(int)(int16_t)(h.x >> 16), bi.y);
                v[4 * c + 2] = affine(sc.z, (float)(int)(int16_t)(h.y & 0xFFFFu), bi.z);
                v[4 * c + 3] = affine(sc.w, (float)(int)(int16_t)(h.y >> 16), bi.w);
            } else {
                v[4 * c] = v[4 * c + 1] = v[4 * c + 2] = v[4 * c + 3] = neg_inf;
            }
        }
        float mx = neg_inf;
#pragma unroll
        for (int i = 0; i < PER; ++i) mx = fmaxf(mx, v[i]);
        mx = wave_max(mx);
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        __syncthreads();
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < PER; ++i) s += __expf(v[i] - mx);
        s = wave_sum(s);
        if (lane == 0) red[wave] = s;
        __syncthreads();
        s = (red[0] + red[1]) + (red[2] + red[3]);
        __syncthreads();
        const float shift = mx + __logf(s);
#pragma unroll
        for (int c = 0; c < PER / 4; ++c) {
            const int n = c * 1024 + 4 * (int)threadIdx.x;
            if (n < N) {
                float4 q;
                q.x = v[4 * c] - shift; q.y = v[4 * c + 1] - shift; q.z = v[4 * c + 2] - shift; q.w = v[4 * c + 3] - shift;
                *reinterpret_cast<float4*>(z + n) = q;
            }
        }
    }
}

}  // namespace bnn
