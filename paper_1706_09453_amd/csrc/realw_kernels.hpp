// Layers that keep real-valued weights (paper Sec. 2.2, last paragraph, and Sec. 3.1: the input layer and the Softmax
// layer are not binarised): acc[m][n] = sum_k W[n][k] x[m][k] in fp32, ascending k, one accumulator per output, one
// fused multiply-add per step -- the order of the binary-weight product of valu_kernels.hpp, to which this reduces
// bit for bit when every weight is +1 or -1.  Then h^ = acc + bias (one rounding) and the activation.
//
//   realw_valu_kernel         K a multiple of 4, X and W 16-byte aligned
//   realw_valu_simple_kernel  any K (element loads)
//   realw_gemv_kernel         a few frames, outputs that go into the log-Softmax: K split over the lanes
//   bits_to_real_kernel       packed bits of a binary layer -> the fp32 numbers they stand for (-1/+1 or 0/1), for a
//                             real-weight layer that follows a binary one
#pragma once

#include "valu_kernels.hpp"

namespace bnn {

// Lanes <-> outputs n (4 waves x 64), TM frames per workgroup.  Per chunk of KC k (16 or 64):
//   - the workgroup copies W[n0 .. n0+255][kc .. kc+KC-1] to LDS with 16-byte loads (KC/4 threads per row piece;
//     fetched into registers before the products of the current chunk, stored after them: two LDS stages, one
//     barrier per chunk; row pitch KC + 4 floats, so the 16-byte reads of 8 consecutive lanes cover all 32 banks),
//     and a lane reads its own row back (KC/4 x ds_read_b128);
//   - lane l holds x[m][kc + (KC/16) (l mod 16) .. ] for each frame (the same in each row of 16 lanes) and the fmac
//     takes x[m][k] by the DPP row broadcast, as in realx_valu_kernel<., ., true>.
// Columns of a partial last chunk are staged as 0 in both operands: fma(0, 0, acc) returns acc (an accumulator that
// starts at +0 is never -0), so the sum over k < K is unchanged.
// TM = 16 with KC = 16 for large batches; TM = 2 with KC = 64 for batches of a few frames, where a workgroup's time
// is its number of memory round trips (one per chunk).
// Dynamic LDS: realw_lds_bytes(KC).  Grid: x = ceil(M / TM), y = ceil(N / 256).
constexpr unsigned realw_lds_bytes(int KC) { return 2u * 256u * (unsigned)(KC + 4) * 4u; }

template <int TM, int ACT, int KC>
__global__ __launch_bounds__(256) void realw_valu_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                         const float* __restrict__ bias, int M, int K, int N,
                                                         void* __restrict__ Y, int yw32) {
    constexpr int LD = KC + 4, KV = KC / 16, TPR = KC / 4, NP = TPR, RPP = 256 / TPR;   // threads per row, pieces per thread, rows per pass
    extern __shared__ __attribute__((aligned(16))) float wt[];   // [2][256 * LD]
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
    // this thread's NP pieces of the W tile: piece p is row t / TPR + RPP p, floats 4 (t % TPR) .. + 3
    const int prow = (int)threadIdx.x / TPR, pcol = ((int)threadIdx.x % TPR) * 4;
    const float* wsrc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int row = nb0 + prow + RPP * p;
        wsrc[p] = W + (size_t)(row < N ? row : N - 1) * K;
    }

    float acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[i] = 0.0f;

    const int nchunks = (K + KC - 1) / KC;
    const int lk = (lane & 15) * KV;
    float pre[NP][4];
    // K % 4 == 0: a 16-byte piece lies wholly inside the row or wholly past it; past it, the row's first piece is read
    // again and dropped
    auto fetch_w = [&](int c) {
        const int k = c * KC + pcol;
        const bool in = k < K;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const float4 t = *reinterpret_cast<const float4*>(wsrc[p] + (in ? k : 0));
            pre[p][0] = in ? t.x : 0.0f, pre[p][1] = in ? t.y : 0.0f, pre[p][2] = in ? t.z : 0.0f, pre[p][3] = in ? t.w : 0.0f;
        }
    };
    auto stash_w = [&](int stage) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<float4*>(&wt[stage * 256 * LD + (prow + RPP * p) * LD + pcol]) =
                make_float4(pre[p][0], pre[p][1], pre[p][2], pre[p][3]);
    };
    auto fetch_x = [&](float (&v)[TM][KV], int c) {
        const int k = c * KC + lk;
        const bool in = k < K;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float* p = xr[i] + (in ? k : 0);
            if constexpr (KV == 4) {
                const float4 t = *reinterpret_cast<const float4*>(p);
                v[i][0] = in ? t.x : 0.0f, v[i][1] = in ? t.y : 0.0f, v[i][2] = in ? t.z : 0.0f, v[i][3] = in ? t.w : 0.0f;
            } else {
                const float t = *p;
                v[i][0] = in ? t : 0.0f;
            }
        }
    };
    auto products = [&](const float (&v)[TM][KV], int stage) {
        float wv[KC];
        const float* mine = &wt[stage * 256 * LD + (wave * kWave + lane) * LD];
#pragma unroll
        for (int q4 = 0; q4 < KC / 4; ++q4) {
            const float4 t = *reinterpret_cast<const float4*>(mine + 4 * q4);
            wv[4 * q4] = t.x, wv[4 * q4 + 1] = t.y, wv[4 * q4 + 2] = t.z, wv[4 * q4 + 3] = t.w;
        }
        // the zeroed frame values of a partial chunk come from v_cndmask: keep the DPP reads two instructions away
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 1");
        static_for<16>([&](auto jc) {
            constexpr int J = decltype(jc)::value;
#pragma unroll
            for (int q = 0; q < KV; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i) fmac_row_bcast<J>(acc[i], v[i][q], wv[KV * J + q]);
        });
    };

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
    if (!active) return;
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

// Real-weight layer in front of the log-Softmax for a handful of frames (streaming): z[m][n] = sum_k W[n][k] x[m][k]
// + bias[n] with K split over the lanes.  27.9 MB of fp32 weights (the paper's 2048 -> 3400 Softmax layer) have to
// pass through the chip once per FR frames; with lanes <-> outputs only N / 64 waves would pull them, here
// N / 4 waves do, each reading whole rows with 16-byte loads (a wave reads 1 KiB of a row at a time).  Lane l
// sums k = 256 s + 4 l .. + 3 over s in fp32, then the 64 partial sums are added by a butterfly of lane exchanges:
// a fixed order, but not the ascending-k chain, so this serves only the layer whose outputs go straight into the
// log-Softmax (the same rule as the matrix-core kernel for large batches).
// K a multiple of 4, X and W 16-byte aligned.  Grid: x = ceil(N / 16), y = ceil(M / FR); 4 waves x 4 rows.
template <int FR>
__global__ __launch_bounds__(256) void realw_gemv_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                         const float* __restrict__ bias, int M, int K, int N,
                                                         float* __restrict__ Z) {
    constexpr int R = 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n0 = ((int)blockIdx.x * 4 + wave) * R;
    if (n0 >= N) return;
    const int m0 = (int)blockIdx.y * FR;
    const float* wr[R];
    const float* xr[FR];
#pragma unroll
    for (int r = 0; r < R; ++r) wr[r] = W + (size_t)(n0 + r < N ? n0 + r : N - 1) * K;
#pragma unroll
    for (int i = 0; i < FR; ++i) xr[i] = X + (size_t)(m0 + i < M ? m0 + i : M - 1) * K;

    float acc[R][FR];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < FR; ++i) acc[r][i] = 0.0f;

    const int nsteps = (K + 255) / 256;
#pragma unroll 2
    for (int s = 0; s < nsteps; ++s) {
        const int k = 256 * s + 4 * lane;
        const bool in = k < K;            // K % 4 == 0: all four or none; past K the row's first four are read and dropped
        const int kk = in ? k : 0;
        float4 w[R], x[FR];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            w[r] = *reinterpret_cast<const float4*>(wr[r] + kk);
            if (!in) w[r] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);   // fma(0, 0, acc) returns acc: no branch around the loads
        }
#pragma unroll
        for (int i = 0; i < FR; ++i) {
            x[i] = *reinterpret_cast<const float4*>(xr[i] + kk);
            if (!in) x[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < FR; ++i) {
                acc[r][i] = __builtin_fmaf(w[r].x, x[i].x, acc[r][i]);
                acc[r][i] = __builtin_fmaf(w[r].y, x[i].y, acc[r][i]);
                acc[r][i] = __builtin_fmaf(w[r].z, x[i].z, acc[r][i]);
                acc[r][i] = __builtin_fmaf(w[r].w, x[i].w, acc[r][i]);
            }
    }
    // butterfly: after the step with distance d every lane holds the sum over its group of 2 d lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < FR; ++i) acc[r][i] += __shfl_xor(acc[r][i], d, 64);
    // lane r * FR + i stores output (frame m0 + i, row n0 + r)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < FR; ++i)
            if (lane == r * FR + i && n0 + r < N && m0 + i < M)
                Z[(size_t)(m0 + i) * N + n0 + r] = affine(1.0f, acc[r][i], bias ? bias[n0 + r] : 0.0f);
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
