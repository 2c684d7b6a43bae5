// Layers that keep real-valued weights (paper Sec. 2.2, last paragraph, and Sec. 3.1: the input layer and the Softmax
// layer are not binarised): acc[m][n] = sum_k W[n][k] x[m][k] in fp32, ascending k, one accumulator per output, one
// fused multiply-add per step -- the order of the binary-weight product of valu_kernels.hpp, to which this reduces
// bit for bit when every weight is +1 or -1.  Then h^ = acc + bias (one rounding) and the activation.
//
//   realw_valu_kernel         K a multiple of 4, X and W 16-byte aligned
//   realw_valu_simple_kernel  any K (element loads)
//   bits_to_real_kernel       packed bits of a binary layer -> the fp32 numbers they stand for (-1/+1 or 0/1), for a
//                             real-weight layer that follows a binary one
#pragma once

#include "valu_kernels.hpp"

namespace bnn {

constexpr int kRealwKC = 16;     // k per chunk
constexpr int kRealwLD = 20;     // LDS row pitch in floats: 16-byte aligned rows, 8 consecutive lanes cover all 32 banks

// Lanes <-> outputs n (4 waves x 64), TM frames per workgroup.  Per chunk of 16 k:
//   - the workgroup copies W[n0 .. n0+255][kc .. kc+15] to LDS with 16-byte loads (4 threads per row piece of 64
//     bytes; fetched into registers before the products of the current chunk, stored after them: two LDS stages,
//     one barrier per chunk), and a lane reads its own row back (4 x ds_read_b128);
//   - lane l holds x[m][kc + (l mod 16)] for each frame (the same in each row of 16 lanes) and the fmac takes
//     x[m][k] by the DPP row broadcast, as in realx_valu_kernel<., ., true>.
// The k past the last whole chunk (fewer than 16) are done with element loads.
// Grid: x = ceil(M / TM), y = ceil(N / 256).  TM = 16, or 2 for batches of a few frames.
template <int TM, int ACT>
__global__ __launch_bounds__(256) void realw_valu_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                         const float* __restrict__ bias, int M, int K, int N,
                                                         void* __restrict__ Y, int yw32) {
    constexpr int KC = kRealwKC, LD = kRealwLD, KV = 1, NP = 256 * KC / 4 / 256;   // NP pieces of W per thread
    __shared__ __attribute__((aligned(16))) float wt[2][256 * LD];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int nb0 = (int)blockIdx.y * 256;
    const int n0 = nb0 + wave * kWave;
    const bool active = n0 < N;   // wave-uniform; an inactive wave still copies its share of W and meets the barriers
    const int n = n0 + lane;
    const int m0 = (int)blockIdx.x * TM;

    const float* xr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) xr[i] = X + (size_t)(m0 + i < M ? m0 + i : M - 1) * K;
    // this thread's NP pieces of the W tile: piece p is row (t + 256 p) / 4, floats 4 ((t + 256 p) % 4) .. + 3
    const int prow = (int)threadIdx.x >> 2, pcol = ((int)threadIdx.x & 3) * 4;
    const float* wsrc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int row = nb0 + prow + 64 * p;
        wsrc[p] = W + (size_t)(row < N ? row : N - 1) * K + pcol;
    }

    float acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[i] = 0.0f;

    const int nchunks = K / KC;
    const int lk = (lane & 15) * KV;
    float pre[NP][4];
    auto fetch_w = [&](int c) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const float4 t = *reinterpret_cast<const float4*>(wsrc[p] + c * KC);
            pre[p][0] = t.x, pre[p][1] = t.y, pre[p][2] = t.z, pre[p][3] = t.w;
        }
    };
    auto stash_w = [&](int stage) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<float4*>(&wt[stage][(prow + 64 * p) * LD + pcol]) = make_float4(pre[p][0], pre[p][1], pre[p][2], pre[p][3]);
    };
    auto fetch_x = [&](float (&v)[TM][KV], int c) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            v[i][0] = xr[i][c * KC + lk];
        }
    };
    auto products = [&](const float (&v)[TM][KV], int stage) {
        float wv[KC];
        const float* mine = &wt[stage][(wave * kWave + lane) * LD];
#pragma unroll
        for (int q4 = 0; q4 < KC / 4; ++q4) {
            const float4 t = *reinterpret_cast<const float4*>(mine + 4 * q4);
            wv[4 * q4] = t.x, wv[4 * q4 + 1] = t.y, wv[4 * q4 + 2] = t.z, wv[4 * q4 + 3] = t.w;
        }
        static_for<16>([&](auto jc) {
            constexpr int J = decltype(jc)::value;
#pragma unroll
            for (int q = 0; q < KV; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i) fmac_row_bcast<J>(acc[i], v[i][q], wv[KV * J + q]);
        });
    };

    if (nchunks > 0) {
        // every fetch unconditional (those past the end re-read the last chunk, unused)
        float va[TM][KV], vb[TM][KV];
        const int last = nchunks - 1;
        fetch_w(0);
        fetch_x(va, 0);
        stash_w(0);
        __syncthreads();
        int c = 0;
        for (; c + 1 < nchunks; c += 2) {
            fetch_w(c + 1);
            fetch_x(vb, c + 1);
            if (active) products(va, 0);
            stash_w(1);   // stage 1 was last read before the previous barrier
            __syncthreads();
            fetch_w(c + 2 < last ? c + 2 : last);
            fetch_x(va, c + 2 < last ? c + 2 : last);
            if (active) products(vb, 1);
            stash_w(0);
            __syncthreads();
        }
        if (c < nchunks && active) products(va, 0);
    }
    if (!active) return;
    const float* wrow = W + (size_t)(n < N ? n : N - 1) * K;
    for (int k = nchunks * KC; k < K; ++k) {
        const float w = wrow[k];
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[i] = __builtin_fmaf(w, xr[i][k], acc[i]);
    }
    int dummy[TM];
    epilogue_lanes_n<TM, ACT>(acc, dummy, nullptr, bias, m0, M, n0, n, N, Y, yw32);
}

// Any K: lanes <-> outputs n, a lane walks its own weight row, the frame value is a wave-uniform (scalar) load.
// Grid: x = ceil(M / TM), y = ceil(N / 256).
template <int TM, int ACT>
__global__ __launch_bounds__(256) void realw_valu_simple_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                                const float* __restrict__ bias, int M, int K, int N,
                                                                void* __restrict__ Y, int yw32) {
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n0 = ((int)blockIdx.y * 4 + wave) * kWave;
    if (n0 >= N) return;
    const int n = n0 + lane;
    const int m0 = (int)blockIdx.x * TM;
    const float* wrow = W + (size_t)(n < N ? n : N - 1) * K;
    const float* xr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) xr[i] = X + (size_t)(m0 + i < M ? m0 + i : M - 1) * K;
    float acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[i] = 0.0f;
    for (int k = 0; k < K; ++k) {
        const float w = wrow[k];
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[i] = __builtin_fmaf(w, xr[i][k], acc[i]);
    }
    int dummy[TM];
    epilogue_lanes_n<TM, ACT>(acc, dummy, nullptr, bias, m0, M, n0, n, N, Y, yw32);
}

// out[m][k] = bit k of row m ? 1.0f : (zero_one ? 0.0f : -1.0f).  One thread per element, grid-stride.
__global__ __launch_bounds__(256) void bits_to_real_kernel(const uint32_t* __restrict__ Xp, int64_t M, int K, int w32,
                                                           int zero_one, float* __restrict__ out) {
    const int64_t total = M * (int64_t)K;
    const float low = zero_one ? 0.0f : -1.0f;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t m = e / K;
        const int k = (int)(e - m * K);
        out[e] = ((Xp[m * w32 + (k >> 5)] >> (k & 31)) & 1u) ? 1.0f : low;
    }
}

}  // namespace bnn
