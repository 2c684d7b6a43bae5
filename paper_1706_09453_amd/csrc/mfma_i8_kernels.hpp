// Third arm of the binary x binary product (paper Sec. 2.3): +-1 as int8 on the matrix cores,
// V_MFMA_I32_16X16X64_I8 with exact int32 accumulation.  Kept for the measured comparison with the XOR/popcount arm
// and the 4-bit-float arm: it moves the same packed bits but expands every bit to a byte (3 vector instructions per
// 4 elements, against 2 per 8 for the 4-bit format) and the int8 MFMA rate is half the 4-bit rate.
//
// Tiling as in mfma_kernels.hpp: a workgroup of 2 x 2 waves, each wave 4 x 4 accumulator fragments of 16 x 16; K in
// super-steps of 512 bits, lane (r = lane % 16, g = lane / 16) fetches words 4g..4g+3 of the super-step of row r of
// every fragment.  One packed word feeds two MFMAs: dword c (0..7) of the expansion holds, in byte i, the element of
// bit c + 8 i, and dwords 4t..4t+3 are the lane's 16 elements of MFMA t.  Both operands use the same map, so the order
// of k inside a super-step is permuted identically for both.  A byte is 0x01 for bit 0 and 0xFF for bit 1: the sign
// convention is flipped in both operands, products are unchanged; zero pad bits give (+1)(+1) and are subtracted.
#pragma once

#include "mfma_kernels.hpp"

namespace bnn {

typedef int v4i __attribute__((ext_vector_type(4)));

// Byte i of the result is +1 (0x01) or -1 (0xFF) for bit c + 8 i of w: the 0/1 bytes select byte 0 or 1 of the table.
__device__ __forceinline__ int expand_pm1_i8(uint32_t w, int c, uint32_t table) {
    return (int)__builtin_amdgcn_perm(0u, table, (w >> c) & 0x01010101u);
}

// Grid: x = ceil(M / 128), y = ceil(N / 128); block = 256 threads.
template <int ACT, bool ALIGNED>
__global__ __launch_bounds__(256) void binx_mfma_i8_kernel(const uint32_t* __restrict__ Xp, const uint32_t* __restrict__ Wp,
                                                           const float* __restrict__ scale, const float* __restrict__ bias,
                                                           int M, int K, int N, int w32, void* __restrict__ Y, int yw32) {
    constexpr int WM = 4, WN = 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15, g = lane >> 4;
    const int m_base = ((int)blockIdx.x * 2 + (wave >> 1)) * (WM * 16);
    const int n_base = ((int)blockIdx.y * 2 + (wave & 1)) * (WN * 16);
    if (m_base >= M || n_base >= N) return;   // wave-uniform

    const uint32_t* arow[WM];
    const uint32_t* brow[WN];
#pragma unroll
    for (int f = 0; f < WM; ++f) {
        const int m = m_base + f * 16 + r;
        arow[f] = Xp + (size_t)(m < M ? m : M - 1) * w32;
    }
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        const int n = n_base + f * 16 + r;
        brow[f] = Wp + (size_t)(n < N ? n : N - 1) * w32;
    }

    v4i acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    uint32_t table = 0x0000FF01u;   // byte 0: +1, byte 1: -1
    asm volatile("" : "+v"(table));
    const int nS = (K + 511) >> 9;
    uint4 araw[WM], braw[WN];
#pragma unroll
    for (int f = 0; f < WM; ++f) araw[f] = load_words<ALIGNED>(arow[f], 0, g, w32);
#pragma unroll
    for (int f = 0; f < WN; ++f) braw[f] = load_words<ALIGNED>(brow[f], 0, g, w32);

    for (int S = 0; S < nS; ++S) {
        uint4 anext[WM], bnext[WN];
        const int Sn = (S + 1 < nS) ? S + 1 : S;   // the last prefetch re-reads the last step (in bounds, unused)
#pragma unroll
        for (int f = 0; f < WM; ++f) anext[f] = load_words<ALIGNED>(arow[f], Sn, g, w32);
#pragma unroll
        for (int f = 0; f < WN; ++f) bnext[f] = load_words<ALIGNED>(brow[f], Sn, g, w32);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                v4i bx[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f)
#pragma unroll
                    for (int c = 0; c < 4; ++c) bx[f][c] = expand_pm1_i8(word_of(braw[f], j), 4 * t + c, table);
#pragma unroll
                for (int fm = 0; fm < WM; ++fm) {
                    v4i ax;
#pragma unroll
                    for (int c = 0; c < 4; ++c) ax[c] = expand_pm1_i8(word_of(araw[fm], j), 4 * t + c, table);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ax, bx[fn], acc[fm][fn], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int f = 0; f < WM; ++f) araw[f] = anext[f];
#pragma unroll
        for (int f = 0; f < WN; ++f) braw[f] = bnext[f];
    }

    // ---- epilogue.  Accumulator fragment (fm, fn), register q of lane (r, g) is
    //      dot[m_base + 16 fm + 4 g + q][n_base + 16 fn + r] + pad.
    const int pad = nS * 512 - K;
    float sc[WN], bi[WN];
    bool nvalid[WN];
#pragma unroll
    for (int fn = 0; fn < WN; ++fn) {
        const int n = n_base + fn * 16 + r;
        nvalid[fn] = n < N;
        sc[fn] = (scale && nvalid[fn]) ? scale[n] : 1.0f;
        bi[fn] = (bias && nvalid[fn]) ? bias[n] : 0.0f;
    }

    if constexpr (ACT == ACT_SIGN) {
        uint32_t* Yw = (uint32_t*)Y;
        const int wcol = n_base >> 5;   // first 32-bit word of this wave's 64 outputs
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned long long b[WN];
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    const float h = affine(sc[fn], (float)(acc[fm][fn][q] - pad), bi[fn]);
                    b[fn] = __ballot(nvalid[fn] && sign_bit(h));
                }
                // ballot bit 16*gg + rr belongs to row 4*gg + q, column 16*fn + rr.  Lane gg (< 4) assembles row 4*gg + q.
                if (lane < 4) {
                    const int sh = 16 * lane;
                    const uint32_t lo = (uint32_t)((b[0] >> sh) & 0xFFFFu) | ((uint32_t)((b[1] >> sh) & 0xFFFFu) << 16);
                    const uint32_t hi = (uint32_t)((b[2] >> sh) & 0xFFFFu) | ((uint32_t)((b[3] >> sh) & 0xFFFFu) << 16);
                    const int m = m_base + fm * 16 + 4 * lane + q;
                    if (m < M) {
                        uint32_t* yr = Yw + (size_t)m * yw32;
                        yr[wcol] = lo;
                        if (wcol + 1 < yw32) yr[wcol + 1] = hi;
                    }
                }
            }
        }
    } else {
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = m_base + fm * 16 + 4 * g + q;
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    const int n = n_base + fn * 16 + r;
                    const int dot = acc[fm][fn][q] - pad;
                    if (m < M && nvalid[fn]) {
                        if constexpr (ACT == ACT_RAW_I32) {
                            ((int*)Y)[(size_t)m * N + n] = dot;
                        } else {
                            float h = affine(sc[fn], (float)dot, bi[fn]);
                            if constexpr (ACT == ACT_HARDTANH) h = hardtanh(h);
                            if constexpr (ACT == ACT_SIGMOID) h = sigmoid(h);
                            ((float*)Y)[(size_t)m * N + n] = h;
                        }
                    }
                }
            }
        }
    }
}

}  // namespace bnn
