// Training-side kernels (paper Alg. 1 and Alg. 2, backward propagation and update; Sec. 2.1-2.3).
//
// The two matrix products of the backward pass are the forward products with the operands' roles exchanged and run
// on the forward kernels:
//   g_{h_{l-1}} = g_{h^_l} w^b_l      realx kernels on the TRANSPOSED packed signs (pack_sign_transposed_kernel below)
//   g_{w_l}     = g_{h^_l}^T h_{l-1}  realw kernels on the two transposed operands (transpose_f32_kernel below)
// so their sums run in ascending n and ascending frame m, one accumulator per result.  What is here are the remaining
// steps: the transposes, the gradient through the Softmax/cross-entropy and through the binarisation layer (Mask),
// the bias gradient, the clipped update, gradient-norm clipping and the semi-stochastic binarisation.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

// WpT[k][n / 32] bit (n % 32) = (W[n][k] > 0): the signs of W^T, packed along n.  A workgroup turns a tile of 64 rows n
// x 64 columns k through LDS (rows read along k, coalesced); a wave then takes one k at a time, lane <-> n, and the
// ballot of (value > 0) is the two output words.  Pad bits (n >= N) are 0.  Grid: x = ceil(K / 64), y = ceil(N / 64).
__global__ __launch_bounds__(256) void pack_sign_transposed_kernel(const float* __restrict__ W, int N, int K, int w32t,
                                                                   uint32_t* __restrict__ WpT) {
    __shared__ float tile[64][65];
    const int k0 = (int)blockIdx.x * 64, n0 = (int)blockIdx.y * 64;
    const int wave = (int)threadIdx.x >> 6, lane = lane_id();
    for (int r = wave; r < 64; r += 4) {   // row n0 + r, column k0 + lane
        const int n = n0 + r, k = k0 + lane;
        tile[r][lane] = (n < N && k < K) ? W[(size_t)n * K + k] : 0.0f;
    }
    __syncthreads();
    for (int c = wave; c < 64; c += 4) {
        const int k = k0 + c;
        const unsigned long long mask = __ballot(sign_bit(tile[lane][c]));   // lanes with n >= N hold 0: bit 0
        if (lane == 0 && k < K) {
            uint32_t* row = WpT + (size_t)k * w32t;
            const int w = n0 >> 5;
            row[w] = (uint32_t)mask;
            if (w + 1 < w32t) row[w + 1] = (uint32_t)(mask >> 32);
        }
    }
}

// out[c][r] = A[r][c], 64 x 64 tiles through LDS, both sides coalesced.  Grid: x = ceil(C / 64), y = ceil(R / 64).
__global__ __launch_bounds__(256) void transpose_f32_kernel(const float* __restrict__ A, int R, int C, float* __restrict__ out) {
    __shared__ float tile[64][65];
    const int c0 = (int)blockIdx.x * 64, r0 = (int)blockIdx.y * 64;
    const int wave = (int)threadIdx.x >> 6, lane = lane_id();
    for (int i = wave; i < 64; i += 4)
        if (r0 + i < R && c0 + lane < C) tile[i][lane] = A[(size_t)(r0 + i) * C + c0 + lane];
    __syncthreads();
    for (int i = wave; i < 64; i += 4)
        if (c0 + i < C && r0 + lane < R) out[(size_t)(c0 + i) * R + r0 + lane] = tile[lane][i];
}

// Alg. 1/2: gradient of the summed cross entropy through the Softmax layer, g[m][n] = exp(logp[m][n]) - (n == label[m]),
// evaluated in fp64 from the fp32 log-posteriors and rounded once.  Grid-stride over M x N elements.
__global__ __launch_bounds__(256) void softmax_xent_grad_kernel(const float* __restrict__ logp, const int32_t* __restrict__ labels,
                                                                int64_t M, int N, float* __restrict__ g) {
    const int64_t total = M * (int64_t)N;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t m = e / N;
        const int n = (int)(e - m * N);
        const double p = exp((double)logp[e]);
        g[e] = (float)(n == labels[m] ? p - 1.0 : p);
    }
}

// Sec. 2.2: g_{h^} = g_h (.) Mask(h^, k); Mask = 0 where |h^| > k, 1 otherwise.  out may be g_h itself.
__global__ __launch_bounds__(256) void mask_grad_kernel(const float* __restrict__ g_h, const float* __restrict__ hhat,
                                                        int64_t count, float k, float* __restrict__ out) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256)
        out[e] = __builtin_fabsf(hhat[e]) > k ? 0.0f : g_h[e];
}

// Alg. 1 backward through a Sigmoid layer: g_{h^} = g_h * (h * (1 - h)) with h the layer's output, every operation
// rounded in fp32 (no contraction: the library is built with -ffp-contract=off).  out may be g_h itself.
__global__ __launch_bounds__(256) void sigmoid_grad_kernel(const float* __restrict__ g_h, const float* __restrict__ h,
                                                           int64_t count, float* __restrict__ out) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        const float v = h[e];
        const float d = v * (1.0f - v);
        out[e] = g_h[e] * d;
    }
}

// g_r[n] = sum_m g[m][n] in fp32, ascending m, one accumulator per n (lanes <-> n: every row is read coalesced; 32
// rows are requested at a time, the additions stay in order).  Grid: x = ceil(N / 64), one wave per workgroup.
__global__ __launch_bounds__(64) void colsum_kernel(const float* __restrict__ g, int M, int N, float* __restrict__ out) {
    const int n = (int)blockIdx.x * 64 + (int)threadIdx.x;
    if (n >= N) return;
    float s = 0.0f;
    int m = 0;
    for (; m + 32 <= M; m += 32) {
        float v[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = g[(size_t)(m + i) * N + n];
#pragma unroll
        for (int i = 0; i < 32; ++i) s = s + v[i];
    }
    for (; m < M; ++m) s = s + g[(size_t)m * N + n];
    out[n] = s;
}

// Alg. 1 Update: w <- Clip(w - eta g) with Clip to [-1, +1] (Sec. 2.1); clip == 0: the plain update.  One fma.
__global__ __launch_bounds__(256) void update_clip_kernel(float* __restrict__ w, const float* __restrict__ g, int64_t count,
                                                          float eta, int clip) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        float v = __builtin_fmaf(-eta, g[e], w[e]);
        if (clip) {
            v = v > 1.0f ? 1.0f : v;
            v = v < -1.0f ? -1.0f : v;
        }
        w[e] = v;
    }
}

// Sec. 2.3, gradient-norm clipping, in three launches whose order of additions is fixed (reproducible bit for bit):
// 256 workgroups each sum the squares of a fixed strided subset in fp64 (per thread, then a tree over LDS) ...
constexpr int kSumsqBlocks = 256;
__global__ __launch_bounds__(256) void sumsq_partial_kernel(const float* __restrict__ g, int64_t count, double* __restrict__ partial) {
    __shared__ double part[256];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)kSumsqBlocks * 256) {
        const double v = (double)g[i];
        s += v * v;
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int stride = 128; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) part[threadIdx.x] += part[threadIdx.x + stride];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = part[0];
}
// ... one workgroup adds the 256 partial sums with the same tree and stores ||g||_2 as fp32 ...
__global__ __launch_bounds__(256) void sumsq_final_kernel(const double* __restrict__ partial, float* __restrict__ norm_out) {
    __shared__ double part[256];
    part[threadIdx.x] = partial[threadIdx.x];
    __syncthreads();
    for (int stride = 128; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) part[threadIdx.x] += part[threadIdx.x + stride];
        __syncthreads();
    }
    if (threadIdx.x == 0) norm_out[0] = (float)sqrt(part[0]);
}
// ... and every element is multiplied by alpha / ||g||_2 if the norm is above alpha.
__global__ __launch_bounds__(256) void scale_if_above_kernel(float* __restrict__ g, int64_t count, float alpha,
                                                             const float* __restrict__ norm) {
    const float nrm = norm[0];
    if (!(nrm > alpha)) return;
    const float factor = alpha / nrm;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) g[e] = g[e] * factor;
}

// Sec. 2.1 (Alg. 1 Update, optional step): w <- Sign(w) where the given draw u in [0, 1) is below p(|w|) = |w|.
__global__ __launch_bounds__(256) void semi_stochastic_kernel(float* __restrict__ w, const float* __restrict__ u, int64_t count) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        const float v = w[e];
        if (u[e] < __builtin_fabsf(v)) w[e] = v > 0.0f ? 1.0f : -1.0f;
    }
}

}  // namespace bnn
