// Vector-ALU kernels: lanes <-> outputs n.
//
//   realx_valu_lds_kernel  binary weights x real input, large batches  (paper Alg. 1 forward: add/subtract product)
//   realx_valu_kernel      the same for batches of a few frames and for rows that are not 16-byte aligned
//   binx_valu_kernel       binary weights x binary input (paper Sec. 2.3: XOR + popcount), -1/+1 or 0/1 reading
//
// All are output-stationary: one wavefront owns 64 outputs n per lane slot for TM frames, so every output has
// exactly one accumulator and one writer and its sum runs in ascending k.  What a lane needs of the weights is its
// own packed row (vector loads).  What it needs of the frames is the same for all 64 lanes; it arrives, depending
// on the kernel, as a broadcast read of a tile staged in LDS, by the DPP row broadcast of a value held once per 16
// lanes, or through the scalar cache as an SGPR operand (the binary kernel's frame words).
#pragma once

#include <type_traits>

#include "bnn_device.hpp"

namespace bnn {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a compile-time constant
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

// Epilogue for the lanes<->n layout.  v[i] is the product term of frame m0+i and output n (this lane).
//   ACT_RAW_I32            Y int32 [M][N]          (vi[i], no affine step)
//   ACT_LINEAR / HARDTANH  Y fp32  [M][N]
//   ACT_SIGN               Y words [M][yw32]       one ballot per frame packs the 64 outputs of the wave
template <int TM, int ACT>
__device__ __forceinline__ void epilogue_lanes_n(const float (&v)[TM], const int (&vi)[TM], const float* __restrict__ scale,
                                                 const float* __restrict__ bias, int m0, int M, int n0, int n, int N,
                                                 void* __restrict__ Y, int yw32) {
    const bool nvalid = n < N;
    const int lane = lane_id();
    if constexpr (ACT == ACT_RAW_I32) {
        int* Yi = (int*)Y;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            if (nvalid && m0 + i < M) Yi[(size_t)(m0 + i) * N + n] = vi[i];
    } else {
        const float sc = (scale && nvalid) ? scale[n] : 1.0f;
        const float bi = (bias && nvalid) ? bias[n] : 0.0f;
        if constexpr (ACT == ACT_SIGN) {
            unsigned long long mine = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const bool p = nvalid && sign_bit(affine(sc, v[i], bi));
                const unsigned long long mask = __ballot(p);
                if (lane == i) mine = mask;
            }
            if (lane < TM && m0 + lane < M) {
                uint32_t* yr = (uint32_t*)Y + (size_t)(m0 + lane) * yw32;
                const int w = n0 >> 5;
                yr[w] = (uint32_t)mine;
                if (w + 1 < yw32) yr[w + 1] = (uint32_t)(mine >> 32);
            }
        } else {
            float* Yf = (float*)Y;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                float h = affine(sc, v[i], bi);
                if constexpr (ACT == ACT_HARDTANH) h = hardtanh(h);
                if constexpr (ACT == ACT_SIGMOID) h = sigmoid(h);
                if (nvalid && m0 + i < M) Yf[(size_t)(m0 + i) * N + n] = h;
            }
        }
    }
}

// acc += x[lane J of this lane's row of 16] * w: the frame operand comes through the DPP row broadcast of the fmac
// itself, so it costs no instruction of its own.  (The compiler does not fold a DPP move into a three-operand fma.)
// x must have been written by a memory load, not by a VALU instruction within the two instructions before: the
// assembler adds no wait states for inline assembly.
template <int J>
__device__ __forceinline__ void fmac_row_bcast(float& acc, float x, float w) {
    asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(x), "v"(w), "n"(J));
}

// acc[m][n] = sum_k (w[n][k] ? +x[m][k] : -x[m][k]) in fp32, k ascending, one accumulator per output:
// each step is fma(+-1.0f, x, acc), which rounds exactly like acc +- x.  The +-1.0f is built per lane
// from the lane's weight bit (2 VALU ops per k, shared by the TM frames).
//   BCAST  (K a multiple of 4, X 16-byte aligned): lane l holds x[m][kc + KV (l mod 16) .. + KV - 1] of a chunk of
//          16 KV k (one load per frame and chunk, the same in each row of 16 lanes); the fmac takes x[m][k] by a
//          row broadcast.
//   !BCAST x[m][k] is a wave-uniform load and arrives through the scalar cache as an SGPR operand (61 % of the
//          4-cycle VALU issue rate measured; BCAST reaches 73 % with TM = 16, where 16 of 18 instructions are fmas).
// Grid: x = ceil(M / TM), y = ceil(N / 256) (4 waves x 64 outputs).
template <int TM, int ACT, bool BCAST>
__global__ __launch_bounds__(256) void realx_valu_kernel(const float* __restrict__ X, const uint32_t* __restrict__ Wp,
                                                         const float* __restrict__ scale, const float* __restrict__ bias,
                                                         int M, int K, int N, int w32, void* __restrict__ Y, int yw32) {
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n0 = ((int)blockIdx.y * 4 + wave) * kWave;
    if (n0 >= N) return;
    const int n = n0 + lane;
    const int m0 = (int)blockIdx.x * TM;
    const uint32_t* wrow = Wp + (size_t)(n < N ? n : N - 1) * w32;

    const float* xr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) xr[i] = X + (size_t)(m0 + i < M ? m0 + i : M - 1) * K;

    float acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[i] = 0.0f;

    if constexpr (BCAST) {
        // KV floats per lane and chunk: a chunk is 16 KV k; two register sets of TM x KV values
        constexpr int KV = TM <= 8 ? 4 : (TM <= 16 ? 2 : 1);
        constexpr int KC = 16 * KV;
        const int nchunks = K / KC;          // whole chunks
        const int lk = (lane & 15) * KV;
        constexpr int NW = KV == 4 ? 2 : 1;   // weight words a chunk touches
        // fetch of chunk c; `in` = this lane's KV values lie inside the row (K is a multiple of 4, so they lie wholly
        // inside or wholly past it); past it the row's first values and its last weight word are read again
        auto fetch = [&](float (&v)[TM][KV], uint32_t (&wv)[NW], int c, bool in = true) {
            const int wlast = w32 - 1;
            if constexpr (KV == 4) {
                wv[0] = wrow[2 * c < wlast ? 2 * c : wlast], wv[1] = wrow[2 * c + 1 < wlast ? 2 * c + 1 : wlast];
            } else {
                wv[0] = wrow[(c * KC) >> 5];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float* p = xr[i] + (in ? c * KC + lk : 0);
                if constexpr (KV == 4) {
                    const float4 t = *reinterpret_cast<const float4*>(p);
                    v[i][0] = t.x, v[i][1] = t.y, v[i][2] = t.z, v[i][3] = t.w;
                } else if constexpr (KV == 2) {
                    const float2 t = *reinterpret_cast<const float2*>(p);
                    v[i][0] = t.x, v[i][1] = t.y;
                } else {
                    v[i][0] = *p;
                }
            }
        };
        // The partial chunk after the whole ones (if any) is requested first and used last.  Its columns past K are taken
        // as 0: fma(w, 0, acc) returns acc (an accumulator that starts at +0 is never -0), so the sum over k < K is
        // unchanged.
        const bool has_tail = nchunks * KC < K;
        const bool tail_in = nchunks * KC + lk < K;
        float vt[TM][KV];
        uint32_t wt[NW];
        fetch(vt, wt, has_tail ? nchunks : 0, has_tail && tail_in);
        auto products = [&](const float (&v)[TM][KV], const uint32_t (&wv)[NW], int c) {
            // bit (KV J + q) of inv[.] is the complement of the weight of the chunk's k number KV J + q
            uint32_t inv[NW];
            if constexpr (KV == 4) {
                inv[0] = ~wv[0], inv[1] = ~wv[1];
            } else {
                inv[0] = ~wv[0] >> ((c * KC) & 31);
            }
            static_for<16>([&](auto jc) {
                constexpr int J = decltype(jc)::value;
#pragma unroll
                for (int q = 0; q < KV; ++q) {
                    const float w = pm1_from_inverted_bit(inv[(KV * J + q) >> 5], (KV * J + q) & 31);
#pragma unroll
                    for (int i = 0; i < TM; ++i) fmac_row_bcast<J>(acc[i], v[i][q], w);
                }
            });
        };
        if (nchunks > 0) {
            // every fetch unconditional (the one past the end re-reads the last chunk, unused)
            float va[TM][KV], vb[TM][KV];
            uint32_t wa[NW], wb[NW];
            const int last = nchunks - 1;
            fetch(va, wa, 0);
            int c = 0;
            for (; c + 1 < nchunks; c += 2) {
                fetch(vb, wb, c + 1);
                products(va, wa, c);
                fetch(va, wa, c + 2 < last ? c + 2 : last);
                products(vb, wb, c + 1);
            }
            if (c < nchunks) products(va, wa, c);
        }
        if (has_tail) {
            // The selects are vector instructions and their results feed DPP reads: every value passes through an
            // "s_nop 1" of its own (two wait states), which the data dependence keeps between the two.
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < KV; ++q) {
                    vt[i][q] = tail_in ? vt[i][q] : 0.0f;
                    asm volatile("s_nop 1" : "+v"(vt[i][q]));
                }
            products(vt, wt, nchunks);
        }
    } else {
        const int kfull = K >> 5;
        for (int kw = 0; kw < kfull; ++kw) {
            const uint32_t inv = ~wrow[kw];
            const int kb = kw << 5;
#pragma unroll
            for (int kk = 0; kk < 32; ++kk) {
                const float w = pm1_from_inverted_bit(inv, kk);
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i] = __builtin_fmaf(w, xr[i][kb + kk], acc[i]);
            }
        }
        if (K & 31) {
            const uint32_t inv = ~wrow[kfull];
            const int kb = kfull << 5;
            for (int kk = 0; kb + kk < K; ++kk) {
                const float w = pm1_from_inverted_bit(inv, kk);
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i] = __builtin_fmaf(w, xr[i][kb + kk], acc[i]);
            }
        }
    }
    int dummy[TM];
    epilogue_lanes_n<TM, ACT>(acc, dummy, scale, bias, m0, M, n0, n, N, Y, yw32);
}

// The same product for large batches, built so that every fma has three VGPR operands: on this chip such an fp32 fma
// issues every 2.5-2.9 clocks when two or more waves share a SIMD, against 3.8-4.4 with an SGPR or DPP operand
// (measured).  A workgroup stages x[16 frames][64 k] in LDS (two stages, one barrier per 64 k); a wave reads
// x[m][k..k+3] with one broadcast ds_read_b128 (all lanes the same address) and uses each value for TNN = 4 outputs per
// lane (n = n0 + lane + 64 j), so there is one LDS read per 16 fmas and the 2 sign-building instructions per k and
// output are shared by 16 frames (TM = 16, TNN = 4; measured: 8 x 8 is 14 % slower, 16 x 2 7 %, 8 x 4 8 %).  Columns of a partial last chunk are staged as 0: fma(w, 0, acc) returns acc (an
// accumulator that starts at +0 is never -0), so the sum over k < K is unchanged.
// K a multiple of 4, X 16-byte aligned.  Grid: x = ceil(M / TM), y = ceil(N / (256 TNN)).
constexpr int kRealxLdsKC = 64;
template <int TM, int TNN, int ACT>
__global__ __launch_bounds__(256, 3) void realx_valu_lds_kernel(const float* __restrict__ X, const uint32_t* __restrict__ Wp,
                                                             const float* __restrict__ scale, const float* __restrict__ bias,
                                                             int M, int K, int N, int w32, void* __restrict__ Y, int yw32) {
    constexpr int KC = kRealxLdsKC;
    static_assert(TM <= 16, "one 16-byte piece of the frame tile per thread");
    __shared__ __attribute__((aligned(16))) float xs[2][TM][KC];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n0 = ((int)blockIdx.y * 4 + wave) * (kWave * TNN);
    const bool active = n0 < N;   // wave-uniform; an inactive wave still stages its share of x and meets the barriers
    const int m0 = (int)blockIdx.x * TM;
    const uint32_t* wrow[TNN];
#pragma unroll
    for (int j = 0; j < TNN; ++j) {
        const int n = n0 + 64 * j + lane;
        wrow[j] = Wp + (size_t)(n < N ? n : N - 1) * w32;
    }
    // this thread's piece of the x tile: row t / 16, floats 4 (t % 16) .. + 3 (threads past TM x 16 have none)
    const int prow = (int)threadIdx.x >> 4, pcol = ((int)threadIdx.x & 15) * 4;
    const bool has_piece = prow < TM;
    const float* xsrc = X + (size_t)(m0 + prow < M ? m0 + prow : M - 1) * K + pcol;

    float acc[TNN][TM];
#pragma unroll
    for (int j = 0; j < TNN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[j][i] = 0.0f;

    const int nchunks = (K + KC - 1) / KC;
    const int wlast = w32 - 1;
    float pre[4];
    uint32_t wa[TNN][2], wb[TNN][2];
    auto fetch = [&](uint32_t (&wv)[TNN][2], int c) {
        const int k = c * KC + pcol;
        const bool in = k < K;   // K % 4 == 0: all four values or none; past K re-read the row's first four, unused
        const float4 t = *reinterpret_cast<const float4*>(in ? xsrc + c * KC : xsrc - pcol);
        pre[0] = in ? t.x : 0.0f, pre[1] = in ? t.y : 0.0f, pre[2] = in ? t.z : 0.0f, pre[3] = in ? t.w : 0.0f;
#pragma unroll
        for (int j = 0; j < TNN; ++j) {   // words past the row's end belong to zero columns: any value will do
            wv[j][0] = wrow[j][2 * c < wlast ? 2 * c : wlast];
            wv[j][1] = wrow[j][2 * c + 1 < wlast ? 2 * c + 1 : wlast];
        }
    };
    auto stash = [&](int stage) {
        if (has_piece) *reinterpret_cast<float4*>(&xs[stage][prow][pcol]) = make_float4(pre[0], pre[1], pre[2], pre[3]);
    };
    auto products = [&](const uint32_t (&wv)[TNN][2], int stage) {
        uint32_t inv[TNN][2];
#pragma unroll
        for (int j = 0; j < TNN; ++j) inv[j][0] = ~wv[j][0], inv[j][1] = ~wv[j][1];
        // 8 steps of 4 k per weight word; the step loop stays a loop (fully unrolled, the three copies of a chunk are
        // 50 KiB of code and no faster)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll 1
        for (int q8 = 0; q8 < 8; ++q8) {
            const int q = 8 * h + q8;
            float xv[TM][4];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float4 t = *reinterpret_cast<const float4*>(&xs[stage][i][4 * q]);
                xv[i][0] = t.x, xv[i][1] = t.y, xv[i][2] = t.z, xv[i][3] = t.w;
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                float w[TNN];
#pragma unroll
                for (int j = 0; j < TNN; ++j) w[j] = pm1_from_inverted_bit(inv[j][h], 4 * q8 + kk);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TNN; ++j) acc[j][i] = __builtin_fmaf(w[j], xv[i][kk], acc[j][i]);
            }
        }
    };

    const int last = nchunks - 1;
    fetch(wa, 0);
    stash(0);
    __syncthreads();
    int c = 0;
    for (; c + 1 < nchunks; c += 2) {   // every fetch unconditional (past the end: the last chunk again, unused)
        fetch(wb, c + 1);
        if (active) products(wa, 0);
        stash(1);   // stage 1 was last read before the previous barrier
        __syncthreads();
        fetch(wa, c + 2 < last ? c + 2 : last);
        if (active) products(wb, 1);
        stash(0);
        __syncthreads();
    }
    if (c < nchunks && active) products(wa, 0);
    if (!active) return;
    int dummy[TM];
#pragma unroll
    for (int j = 0; j < TNN; ++j)
        if (n0 + 64 * j < N)
            epilogue_lanes_n<TM, ACT>(acc[j], dummy, scale, bias, m0, M, n0 + 64 * j, n0 + 64 * j + lane, N, Y, yw32);
}

// dot[m][n] = K - 2 * sum_w popcount(x[m][w] XOR w[n][w]): v_xor_b32 with the frame word as SGPR
// operand, then v_bcnt_u32_b32, whose second operand is the running count (the add is free).
// VEC4: rows are 16-byte aligned and a multiple of 4 words long, so a lane fetches 4 words per load.
// X01:  the input bits are read as 0/1 (paper Sec. 3.2): dot = 2 * sum_w popcount(x AND w) - sum_w popcount(x).
// With TM = 1, 2 or 4 this is also the small-batch (streaming) kernel: ceil(M / TM) x N / 64 waves, each of which
// walks whole weight rows, so a layer takes one memory round trip however few frames there are.
template <int TM, int ACT, bool VEC4, bool X01 = false>
__global__ __launch_bounds__(256) void binx_valu_kernel(const uint32_t* __restrict__ Xp, const uint32_t* __restrict__ Wp,
                                                        const float* __restrict__ scale, const float* __restrict__ bias,
                                                        int M, int K, int N, int w32, void* __restrict__ Y, int yw32) {
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n0 = ((int)blockIdx.y * 4 + wave) * kWave;
    if (n0 >= N) return;
    const int n = n0 + lane;
    const int m0 = (int)blockIdx.x * TM;
    const uint32_t* wrow = Wp + (size_t)(n < N ? n : N - 1) * w32;

    const uint32_t* xr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) xr[i] = Xp + (size_t)(m0 + i < M ? m0 + i : M - 1) * w32;

    uint32_t cnt[TM];
    int ones[TM];   // X01: popcount of the frame's own bits (wave-uniform)
#pragma unroll
    for (int i = 0; i < TM; ++i) cnt[i] = 0, ones[i] = 0;

    auto step = [&](uint32_t b, int i, int kw) {
        const uint32_t x = xr[i][kw];
        if constexpr (X01) {
            cnt[i] += __builtin_popcount(b & x);
            ones[i] += __builtin_popcount(x);
        } else {
            cnt[i] += __builtin_popcount(b ^ x);
        }
    };
    if constexpr (VEC4) {
        // Pieces of 32 words (8 loads of 16 bytes per lane), the next piece in flight while the current one is counted:
        // with few frames per workgroup the kernel's time is the number of memory round trips, and this makes it
        // about one per 64 words instead of one per 4.
        // (For TM > 4 the frames' words of one such piece would not fit the scalar registers: 4 words at a time, as below.)
        constexpr int PW = 32;
        const int npieces = TM <= 4 ? w32 / PW : 0;
        auto fetch = [&](uint4 (&b)[PW / 4], int p) {
#pragma unroll
            for (int q = 0; q < PW / 4; ++q) b[q] = *reinterpret_cast<const uint4*>(wrow + p * PW + 4 * q);
        };
        auto count = [&](const uint4 (&b)[PW / 4], int p) {
#pragma unroll
            for (int q = 0; q < PW / 4; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    step(b[q].x, i, p * PW + 4 * q + 0);
                    step(b[q].y, i, p * PW + 4 * q + 1);
                    step(b[q].z, i, p * PW + 4 * q + 2);
                    step(b[q].w, i, p * PW + 4 * q + 3);
                }
        };
        if (npieces > 0) {
            uint4 ba[PW / 4], bb[PW / 4];
            const int last = npieces - 1;
            fetch(ba, 0);
            int p = 0;
            for (; p + 1 < npieces; p += 2) {   // every fetch unconditional (past the end: the last piece again, unused)
                fetch(bb, p + 1);
                count(ba, p);
                fetch(ba, p + 2 < last ? p + 2 : last);
                count(bb, p + 1);
            }
            if (p < npieces) count(ba, p);
        }
        for (int kw = npieces * PW; kw < w32; kw += 4) {
            const uint4 b = *reinterpret_cast<const uint4*>(wrow + kw);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                step(b.x, i, kw + 0);
                step(b.y, i, kw + 1);
                step(b.z, i, kw + 2);
                step(b.w, i, kw + 3);
            }
        }
    } else {
        for (int kw = 0; kw < w32; ++kw) {
            const uint32_t b = wrow[kw];
#pragma unroll
            for (int i = 0; i < TM; ++i) step(b, i, kw);
        }
    }

    float v[TM];
    int vi[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        vi[i] = X01 ? 2 * (int)cnt[i] - ones[i] : K - 2 * (int)cnt[i];
        v[i] = (float)vi[i];
    }
    epilogue_lanes_n<TM, ACT>(v, vi, scale, bias, m0, M, n0, n, N, Y, yw32);
}

}  // namespace bnn
