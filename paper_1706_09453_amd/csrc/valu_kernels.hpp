// Vector-ALU kernels: lanes <-> outputs n, frames streamed through scalar registers.
//
//   realx_valu_kernel  binary weights x real input   (paper Alg. 1 forward: add/subtract product)
//   binx_valu_kernel   binary weights x binary input (paper Sec. 2.3: XOR + popcount)
//
// Both are output-stationary: one wavefront owns 64 outputs n (one per lane) for TM frames, so every
// output has exactly one accumulator and one writer.  What a lane needs of the weights is its own
// packed row (vector loads); what it needs of the frames is the same for all 64 lanes, so the frame
// operands are wave-uniform and arrive through the scalar cache as SGPR operands of the VALU
// instruction: no LDS traffic and no cross-lane exchange in the inner loop.
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
//          row broadcast.  The k of the last, partial chunk go the way of !BCAST.
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
        const int nchunks = K / KC;
        const int lk = (lane & 15) * KV;
        constexpr int NW = KV == 4 ? 2 : 1;   // weight words a chunk touches
        auto fetch = [&](float (&v)[TM][KV], uint32_t (&wv)[NW], int c) {
            if constexpr (KV == 4) {
                wv[0] = wrow[2 * c], wv[1] = wrow[2 * c + 1];
            } else {
                wv[0] = wrow[(c * KC) >> 5];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float* p = xr[i] + c * KC + lk;
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
        for (int k = nchunks * KC; k < K; ++k) {   // fewer than 16 KV of them
            const float w = pm1_from_inverted_bit(~wrow[k >> 5], k & 31);
#pragma unroll
            for (int i = 0; i < TM; ++i) acc[i] = __builtin_fmaf(w, xr[i][k], acc[i]);
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
        constexpr int PW = 32;
        const int npieces = w32 / PW;
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
