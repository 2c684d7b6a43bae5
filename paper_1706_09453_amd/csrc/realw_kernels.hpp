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

// ---- real weights, large batches: every fma with three VGPR operands ----
// The product of realw_valu_kernel (same chains, same bits) at the issue rate of realx_valu_lds_kernel: an fp32 fma with
// three VGPR operands issues about every 2.7 clocks when two waves share a SIMD, the DPP form of realw_valu_kernel every
// 4 or more.  A workgroup owns 64 frames x 256 outputs: wave w takes frames 16 w .. 16 w + 15, lane l the outputs
// n0 + l + 64 j (j < 4): 64 accumulators per lane.  The frames go through LDS in chunks of 64 k (two stages, one barrier
// per chunk; x[m][k .. k+3] is one broadcast ds_read_b128: one LDS read per 16 fmas).  The weights come from a
// transposed copy Wt[k][n] (weights_transposed_kernel, once per call): the 64 lanes of a wave read 64 consecutive
// numbers per k and j, the four waves of a workgroup read the same ones (one fetch from L2 for four), and the numbers
// of the next four k are requested while these four are used.
// Rows K .. kpad - 1 of Wt hold 0 and the frames are staged as 0 there: fma(0, 0, acc) returns acc.
// K a multiple of 4, X 16-byte aligned, kpad = K rounded up to 64.  Grid: x = ceil(M / 64), y = ceil(N / 256).
constexpr int kRealwLdsKC = 64, kRealwLdsFrames = 64;
__host__ __device__ inline int realw_lds_kpad(int K) { return (K + kRealwLdsKC - 1) / kRealwLdsKC * kRealwLdsKC; }

// Wt[k][n] = W[n][k] for k < K, 0 for K <= k < kpad.  Tiles of 32 x 32 through LDS.  Grid: x = ceil(N / 32),
// y = kpad / 32; block = 256 threads (32 x 8).
__global__ __launch_bounds__(256) void weights_transposed_kernel(const float* __restrict__ W, int N, int K, int kpad,
                                                                 float* __restrict__ Wt) {
    __shared__ float tile[32][33];
    const int tx = (int)threadIdx.x & 31, ty = (int)threadIdx.x >> 5;
    const int nb = (int)blockIdx.x * 32, kb = (int)blockIdx.y * 32;
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int n = nb + r, k = kb + tx;
        tile[r][tx] = (n < N && k < K) ? W[(size_t)n * K + k] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int k = kb + r, n = nb + tx;
        if (n < N && k < kpad) Wt[(size_t)k * N + n] = tile[tx][r];
    }
}

template <int ACT>
__global__ __launch_bounds__(256, 2) void realw_valu_lds_kernel(const float* __restrict__ X, const float* __restrict__ Wt,
                                                                const float* __restrict__ bias, int M, int K, int kpad, int N,
                                                                void* __restrict__ Y, int yw32) {
    constexpr int KC = kRealwLdsKC, FR = kRealwLdsFrames, TM = 16, TNN = 4, NP = FR * (KC / 4) / 256;
    __shared__ __attribute__((aligned(16))) float xs[2][FR][KC];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n0 = (int)blockIdx.y * (kWave * TNN);
    const int m0 = (int)blockIdx.x * FR;
    const int mw = m0 + TM * wave;
    const bool active = mw < M;   // wave-uniform; an inactive wave still stages its share of x and meets the barriers
    uint32_t wofs[TNN];   // byte offset of the lane's outputs in a row of Wt (past the last output: its values again, not stored)
#pragma unroll
    for (int j = 0; j < TNN; ++j) wofs[j] = 4u * (uint32_t)min(n0 + 64 * j + lane, N - 1);
    // this thread's NP pieces of the x tile: piece p is row t / 16 + 16 p, floats 4 (t % 16) .. + 3
    const int prow = (int)threadIdx.x >> 4, pcol = ((int)threadIdx.x & 15) * 4;
    const float* xsrc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) xsrc[p] = X + (size_t)min(m0 + prow + 16 * p, M - 1) * K + pcol;

    float acc[TNN][TM];
#pragma unroll
    for (int j = 0; j < TNN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[j][i] = 0.0f;

    const int nchunks = kpad / KC;
    float pre[NP][4];
    auto fetch_x = [&](int c) {
        const bool in = c * KC + pcol < K;   // K % 4 == 0: all four values or none; past K re-read the row's first four, unused
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const float4 t = *reinterpret_cast<const float4*>(in ? xsrc[p] + c * KC : xsrc[p] - pcol);
            pre[p][0] = in ? t.x : 0.0f, pre[p][1] = in ? t.y : 0.0f, pre[p][2] = in ? t.z : 0.0f, pre[p][3] = in ? t.w : 0.0f;
        }
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<float4*>(&xs[stage][prow + 16 * p][pcol]) = make_float4(pre[p][0], pre[p][1], pre[p][2], pre[p][3]);
    };
    // the weights of k0 .. k0 + 3 (k0 + 3 < kpad): a row's address is wave-uniform, the lane adds its 32-bit offset.
    // Requested last to first and used first to last, like the LDS reads of a step: the first use waits for all of them
    // (one wait instead of sixteen; the other wave of the SIMD has work meanwhile).
    auto fetch_w = [&](float (&w)[4][TNN], int k0) {
#pragma unroll
        for (int kk = 3; kk >= 0; --kk) {
            const char* row = reinterpret_cast<const char*>(Wt + (size_t)(k0 + kk) * N);
#pragma unroll
            for (int j = TNN - 1; j >= 0; --j) {
                // keeps the 32-bit offset next to its load (scalar base + 32-bit lane offset: no address arithmetic per load)
                asm volatile("" : "+v"(wofs[j]));
                w[kk][j] = *reinterpret_cast<const float*>(row + wofs[j]);
            }
        }
    };
    // A step of 4 k in two halves of 8 frames: the LDS reads of a half are requested before the half in front of it is
    // multiplied, so only the first half of a chunk waits for LDS.
    constexpr int HF = TM / 2;
    auto read_x = [&](float (&xv)[HF][4], int stage, int q, int h) {
#pragma unroll
        for (int i = 0; i < HF; ++i) {
            const float4 t = *reinterpret_cast<const float4*>(&xs[stage][TM * wave + HF * h + i][4 * q]);
            xv[i][0] = t.x, xv[i][1] = t.y, xv[i][2] = t.z, xv[i][3] = t.w;
        }
    };
    auto multiply = [&](const float (&w)[4][TNN], const float (&xv)[HF][4], int h) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int i = 0; i < HF; ++i)
#pragma unroll
                for (int j = 0; j < TNN; ++j) acc[j][HF * h + i] = __builtin_fmaf(w[kk][j], xv[i][kk], acc[j][HF * h + i]);
    };

    // two sets of weights in turn: the numbers of step q + 1 are requested before step q is multiplied
    float wa[4][TNN], wb[4][TNN];
    float xa[HF][4], xb[HF][4];
    const int klast = kpad - 4;
    fetch_x(0);
    fetch_w(wa, 0);
    stash(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int stage = c & 1;
        if (c + 1 < nchunks) fetch_x(c + 1);   // workgroup-uniform
        const int kc = c * KC;
        if (active) {   // wave-uniform
            read_x(xa, stage, 0, 0);
#pragma unroll 1
            for (int q = 0; q < KC / 4; q += 2) {   // the request past the last step reads the last four rows again, unused
                // (nothing moves across the scheduling barriers: reads and requests stay one half-step ahead, no further)
                fetch_w(wb, min(kc + 4 * q + 4, klast));
                read_x(xb, stage, q, 1);
                multiply(wa, xa, 0);
                __builtin_amdgcn_sched_barrier(0);
                read_x(xa, stage, q + 1, 0);
                multiply(wa, xb, 1);
                __builtin_amdgcn_sched_barrier(0);
                fetch_w(wa, min(kc + 4 * q + 8, klast));
                read_x(xb, stage, q + 1, 1);
                multiply(wb, xa, 0);
                __builtin_amdgcn_sched_barrier(0);
                read_x(xa, stage, min(q + 2, KC / 4 - 1), 0);   // behind the chunk's last step: read again, unused
                multiply(wb, xb, 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (c + 1 < nchunks) stash(stage ^ 1);   // that stage was last read before the previous barrier
        __syncthreads();
    }
    if (!active) return;
    int dummy[TM];
#pragma unroll
    for (int j = 0; j < TNN; ++j)
        if (n0 + 64 * j < N) epilogue_lanes_n<TM, ACT>(acc[j], dummy, nullptr, bias, mw, M, n0 + 64 * j, n0 + 64 * j + lane, N, Y, yw32);
}

}  // namespace bnn
