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
// reads of a row are complete before its first write.  A workgroup takes ROWS consecutive frames at a time and
// fetches its scale/bias values once for all of them.
// Needs N % 4 == 0, N <= 256 * PER, 16-byte aligned rows.
template <int PER, int ROWS>
__global__ __launch_bounds__(256) void log_softmax_rows_i16_kernel(float* __restrict__ Z, const float* __restrict__ scale,
                                                                   const float* __restrict__ bias, int M, int N) {
    __shared__ float red[ROWS][4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const float neg_inf = -__builtin_inff();
    float sc[PER], bi[PER];
#pragma unroll
    for (int c = 0; c < PER / 4; ++c) {
        const int n = c * 1024 + 4 * (int)threadIdx.x;
        float4 s4 = make_float4(1.f, 1.f, 1.f, 1.f), b4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n < N) {
            if (scale) s4 = *reinterpret_cast<const float4*>(scale + n);
            if (bias) b4 = *reinterpret_cast<const float4*>(bias + n);
        }
        sc[4 * c] = s4.x; sc[4 * c + 1] = s4.y; sc[4 * c + 2] = s4.z; sc[4 * c + 3] = s4.w;
        bi[4 * c] = b4.x; bi[4 * c + 1] = b4.y; bi[4 * c + 2] = b4.z; bi[4 * c + 3] = b4.w;
    }
    for (int m0 = blockIdx.x * ROWS; m0 < M; m0 += gridDim.x * ROWS) {
        float v[ROWS][PER];
#pragma unroll
        for (int t = 0; t < ROWS; ++t) {
            const int m = m0 + t < M ? m0 + t : M - 1;     // a row past the end repeats the last one and is not written
            const uint16_t* d16 = reinterpret_cast<const uint16_t*>(Z + (size_t)m * N);
#pragma unroll
            for (int c = 0; c < PER / 4; ++c) {
                const int n = c * 1024 + 4 * (int)threadIdx.x;
                if (n < N) {
                    const uint2 h = *reinterpret_cast<const uint2*>(d16 + n);
                    v[t][4 * c + 0] = affine(sc[4 * c + 0], (float)(int)(int16_t)(h.x & 0xFFFFu), bi[4 * c + 0]);
                    v[t][4 * c + 1] = affine(sc[4 * c + 1], (float)(int)(int16_t)(h.x >> 16), bi[4 * c + 1]);
                    v[t][4 * c + 2] = affine(sc[4 * c + 2], (float)(int)(int16_t)(h.y & 0xFFFFu), bi[4 * c + 2]);
                    v[t][4 * c + 3] = affine(sc[4 * c + 3], (float)(int)(int16_t)(h.y >> 16), bi[4 * c + 3]);
                } else {
                    v[t][4 * c] = v[t][4 * c + 1] = v[t][4 * c + 2] = v[t][4 * c + 3] = neg_inf;
                }
            }
        }
        float mx[ROWS], s[ROWS];
#pragma unroll
        for (int t = 0; t < ROWS; ++t) {
            mx[t] = neg_inf;
#pragma unroll
            for (int i = 0; i < PER; ++i) mx[t] = fmaxf(mx[t], v[t][i]);
            mx[t] = wave_max(mx[t]);
            if (lane == 0) red[t][wave] = mx[t];
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < ROWS; ++t) mx[t] = fmaxf(fmaxf(red[t][0], red[t][1]), fmaxf(red[t][2], red[t][3]));
        __syncthreads();
#pragma unroll
        for (int t = 0; t < ROWS; ++t) {
            s[t] = 0.0f;
#pragma unroll
            for (int i = 0; i < PER; ++i) s[t] += __expf(v[t][i] - mx[t]);
            s[t] = wave_sum(s[t]);
            if (lane == 0) red[t][wave] = s[t];
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < ROWS; ++t) s[t] = (red[t][0] + red[t][1]) + (red[t][2] + red[t][3]);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < ROWS; ++t) {
            if (m0 + t >= M) break;
            float* z = Z + (size_t)(m0 + t) * N;
            const float shift = mx[t] + __logf(s[t]);
#pragma unroll
            for (int c = 0; c < PER / 4; ++c) {
                const int n = c * 1024 + 4 * (int)threadIdx.x;
                if (n < N) {
                    float4 q;
                    q.x = v[t][4 * c] - shift; q.y = v[t][4 * c + 1] - shift; q.z = v[t][4 * c + 2] - shift; q.w = v[t][4 * c + 3] - shift;
                    *reinterpret_cast<float4*>(z + n) = q;
                }
            }
        }
    }
}

// Scaled log-likelihoods for decoding with a hybrid system: logp[m][n] -= log_prior[n] (log-posterior minus the log of
// the tied state's prior; one fp32 subtraction).  One thread per element, grid-stride.
__global__ __launch_bounds__(256) void subtract_log_prior_kernel(float* __restrict__ logp, const float* __restrict__ log_prior,
                                                                 int64_t M, int N) {
    const int64_t total = M * (int64_t)N;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int n = (int)(e % N);
        logp[e] = logp[e] - log_prior[n];
    }
}

}  // namespace bnn
