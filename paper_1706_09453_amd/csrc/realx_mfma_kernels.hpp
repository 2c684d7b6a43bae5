// Real input x binary weights with fp32 outputs (paper Alg. 1 forward: every product is +-x, the sum needs no
// multiplier) on the matrix cores: V_MFMA_F32_32X32X2_F32 with the weight bits expanded to +-1.0f.
//
// Products +-1.0f * x are exact; the 2 x K/2 partial sums are added in fp32 in the matrix core's own order, so the
// result differs from the sum taken in ascending k by ordinary fp32 rounding (a few units in the last place of the
// largest partial sum) and is checked against the fp64 value of the same sum within the stated tolerance.  Layers
// whose outputs are Sign bits never use this kernel: bits are defined from the sum in ascending k.
//
// Tiling: a workgroup of 2 x 2 waves, each wave 4 x 2 accumulator fragments of 32 x 32 (128 frames x 64 outputs).
// K advances in chunks of 16: lane (r = lane % 32, g = lane / 32) holds, per frames fragment, the 8 values
// x[m_base + 32 fm + r][16 c + 8 g .. + 7] (two 16-byte loads) and, per weights fragment, the packed word of row
// n_base + 32 fn + r that contains these k; step t of a chunk multiplies element 8 g + t of both (the order of k
// inside a chunk is permuted identically for both operands).  The next chunk's loads are pinned ahead of the 64
// MFMAs of the current one (two register sets).  A lane expands one weight bit to +-1.0f per MFMA pair (2 vector
// instructions), so the 64-clock MFMAs run back to back.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

typedef float v16f32 __attribute__((ext_vector_type(16)));

// VEC: K % 16 == 0 and X rows 16-byte aligned (16-byte loads); otherwise element loads, zero past K.
// WREAL: the layer keeps real-valued weights (paper Sec. 3.1: input and Softmax layer): Wv is fp32 [N][K] (16-byte
//        aligned too if VEC), fetched exactly like the frames; otherwise Wv is packed bits [N][w32].
// Grid: x = ceil(M / 256), y = ceil(N / 128); block = 256 threads.  ACT: ACT_LINEAR, ACT_HARDTANH or ACT_SIGMOID.
// One wave per SIMD, i.e. one workgroup per CU, stated to the compiler (it sizes the register claim of the kernel so
// that a second wave does not fit): two workgroups on a CU evict each other's operand rows from the L1.
template <int ACT, bool VEC, bool WREAL = false>
__global__ __launch_bounds__(256, 1) __attribute__((amdgpu_waves_per_eu(1, 1))) void realx_f32_mfma_kernel(const float* __restrict__ X, const void* __restrict__ Wv,
                                                               const float* __restrict__ scale, const float* __restrict__ bias,
                                                               int M, int K, int N, int w32, float* __restrict__ Y) {
    const uint32_t* Wp = static_cast<const uint32_t*>(Wv);
    const float* Wf = static_cast<const float*>(Wv);
    constexpr int WM = 4, WN = 2;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 31, g = lane >> 5;
    const int m_base = ((int)blockIdx.x * 2 + (wave >> 1)) * (WM * 32);
    const int n_base = ((int)blockIdx.y * 2 + (wave & 1)) * (WN * 32);
    if (m_base >= M || n_base >= N) return;   // wave-uniform

    const float* arow[WM];
    const uint32_t* brow[WN];
    const float* brow_f[WN];
#pragma unroll
    for (int f = 0; f < WM; ++f) {
        const int m = m_base + f * 32 + r;
        arow[f] = X + (size_t)(m < M ? m : M - 1) * K + 8 * g;
    }
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        const int n = n_base + f * 32 + r;
        brow[f] = Wp + (size_t)(n < N ? n : N - 1) * w32;
        brow_f[f] = Wf + (size_t)(n < N ? n : N - 1) * K + 8 * g;
    }
    float sc[WN], bi[WN];
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        const int n = n_base + f * 32 + r;
        sc[f] = (n < N && scale) ? scale[n] : 1.0f;
        bi[f] = (n < N && bias) ? bias[n] : 0.0f;
    }

    v16f32 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int nC = (K + 15) >> 4;
    struct Set {
        float a[WM][8];
        uint32_t b[WN];
        float bf[WREAL ? WN : 1][8];
    };
    // the lane's 8 values of chunk cc of a row of floats; p points at element 8 g of the row
    auto fetch8 = [&](float (&dst)[8], const float* p, int cc) {
        if constexpr (VEC) {
            const float4 lo = *reinterpret_cast<const float4*>(p + 16 * cc);
            const float4 hi = *reinterpret_cast<const float4*>(p + 16 * cc + 4);
            dst[0] = lo.x; dst[1] = lo.y; dst[2] = lo.z; dst[3] = lo.w;
            dst[4] = hi.x; dst[5] = hi.y; dst[6] = hi.z; dst[7] = hi.w;
        } else {
            const float* row = p - 8 * g;   // start of the row
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int k = 16 * cc + 8 * g + t;
                const float v = row[k < K ? k : K - 1];   // index clamped into the row, value dropped past K
                dst[t] = k < K ? v : 0.0f;
            }
        }
    };
    auto fetch = [&](Set& s, int c) {
        const int cc = c < nC ? c : nC - 1;   // past the end: re-read the last chunk (in bounds, unused)
#pragma unroll
        for (int f = 0; f < WM; ++f) fetch8(s.a[f], arow[f], cc);
#pragma unroll
        for (int f = 0; f < WN; ++f) {
            if constexpr (WREAL) fetch8(s.bf[f], brow_f[f], cc);
            else s.b[f] = brow[f][cc >> 1];
        }
    };
    auto products = [&](const Set& s, int c) {
        // bit 16 (c & 1) + 8 g + t of the complemented word, moved to bit 24 + t: weight bit 1 <=> +1.0f <=> sign bit clear
        const int base = 16 * (c & 1) + 8 * g;
        uint32_t q[WN];
        if constexpr (!WREAL) {
#pragma unroll
            for (int f = 0; f < WN; ++f) q[f] = ((~s.b[f]) >> base) << 24;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float bx[WN];
#pragma unroll
            for (int f = 0; f < WN; ++f) {
                if constexpr (WREAL) bx[f] = s.bf[f][t];
                else bx[f] = __uint_as_float(((q[f] << (7 - t)) & 0x80000000u) | 0x3f800000u);
            }
#pragma unroll
            for (int fm = 0; fm < WM; ++fm)
#pragma unroll
                for (int fn = 0; fn < WN; ++fn)
                    acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x2f32(s.a[fm][t], bx[fn], acc[fm][fn], 0, 0, 0);
        }
    };
    Set s0, s1;
    // Both fetches of a round are unconditional: a fetch whose only use sits behind a branch is moved behind it.
    // (A third set, fetched two rounds ahead, measured the same time: the kernel does not wait for memory.)
    fetch(s0, 0);
    int c = 0;
    for (; c + 1 < nC; c += 2) {
        fetch(s1, c + 1);
        __builtin_amdgcn_sched_barrier(0);
        products(s0, c);
        __builtin_amdgcn_sched_barrier(0);
        fetch(s0, c + 2);
        __builtin_amdgcn_sched_barrier(0);
        products(s1, c + 1);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (c < nC) products(s0, c);   // odd number of chunks: the last one is already in the first set

    // ---- epilogue.  Accumulator fragment (fm, fn), register v of lane (r, g) is the sum for frame
    //      m_base + 32 fm + 8 (v/4) + 4 g + v%4 and output n_base + 32 fn + r.  Each wave turns 32 rows x 64 columns at
    //      a time through its own slice of LDS so that 16 lanes write 256 contiguous bytes of a row.
    constexpr int LDW = 32 * WN + 4;
    __shared__ __attribute__((aligned(16))) float stage[4][32 * LDW];
    float* st = stage[wave];
    const bool rows_vec = ((N & 3) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
    const int c4 = (lane & 15) * 4;
#pragma unroll
    for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
        for (int fn = 0; fn < WN; ++fn)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float h = affine(sc[fn], acc[fm][fn][v], bi[fn]);
                if constexpr (ACT == ACT_HARDTANH) h = hardtanh(h);
                if constexpr (ACT == ACT_SIGMOID) h = sigmoid(h);
                st[(8 * (v >> 2) + 4 * g + (v & 3)) * LDW + fn * 32 + r] = h;
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // this wave's LDS writes are done before it reads them back
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 4 + (lane >> 4);
            const int m = m_base + fm * 32 + row;
            const int n = n_base + c4;
            const float4 qv = *reinterpret_cast<const float4*>(st + row * LDW + c4);
            if (m < M) {
                float* y = Y + (size_t)m * N + n;
                if (rows_vec && n + 3 < N) {
                    *reinterpret_cast<float4*>(y) = qv;
                } else {
                    if (n + 0 < N) y[0] = qv.x;
                    if (n + 1 < N) y[1] = qv.y;
                    if (n + 2 < N) y[2] = qv.z;
                    if (n + 3 < N) y[3] = qv.w;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // reads done before the next fragment row overwrites the slice
    }
}

}  // namespace bnn
