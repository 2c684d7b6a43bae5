// Matrix-core arm of the binary x binary product (paper Sec. 2.3) for gfx950.
//
// A +-1 value is exactly representable in the 4-bit float operand format (E2M1) of the CDNA4
// V_MFMA_F32_16X16X128_F8F6F4 instruction: nibble 0b0010 = +1.0, 0b1010 = -1.0.  Products of +-1 are
// +-1 and the fp32 accumulator holds every partial sum exactly (|sum| <= K < 2^24), so the MFMA result
// IS the integer dot product; nothing is approximated.
//
// Operands stay bit-packed (1 bit per element) all the way from HBM into registers.  A lane's share of
// a 16x128 operand fragment is 32 elements of one row = ONE 32-bit packed word, which it expands in
// registers into four dwords of eight nibbles:  d_j = ((w << (3-j)) & 0x88888888) | 0x22222222.
// The nibble sign is the packed bit itself (bit 1 -> -1.0): the convention is flipped in BOTH operands,
// which leaves every product unchanged.  Dword j, nibble i holds bit 4i+j: the order of k inside a
// fragment is permuted, identically for both operands, which leaves the sum unchanged.  Zero pad bits
// expand to (+1)(+1) and are subtracted afterwards as a constant.
//
// Tiling: a workgroup of 4 waves (2 x 2) computes a (2*WM*16) x (2*WN*16) tile of [M][N]; each wave owns
// WM x WN accumulator fragments of 16 x 16.  K advances in super-steps of 512 bits: lane (r = lane%16,
// g = lane/16) fetches 16 bytes (words 4g..4g+3 of the super-step) of row r of each fragment in one
// global_load_dwordx4, and word j feeds MFMA step j.  The next super-step is fetched while the current
// one is expanded and multiplied.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// The two constants of the expansion, held in registers so that each dword costs one shift and one
// v_and_or_b32 (a 32-bit literal cannot be an operand of that instruction).
struct ExpandConsts {
    uint32_t sign_mask;   // 0x88888888, lives in an SGPR
    uint32_t one_bits;    // 0x22222222, lives in a VGPR
};
__device__ __forceinline__ ExpandConsts expand_consts() {
    ExpandConsts c{0x88888888u, 0x22222222u};
    asm volatile("" : "+s"(c.sign_mask));
    asm volatile("" : "+v"(c.one_bits));
    return c;
}

__device__ __forceinline__ v8i expand_pm1_fp4(uint32_t w, const ExpandConsts& c) {
    v8i d;
    d[0] = (int)(((w << 3) & c.sign_mask) | c.one_bits);
    d[1] = (int)(((w << 2) & c.sign_mask) | c.one_bits);
    d[2] = (int)(((w << 1) & c.sign_mask) | c.one_bits);
    d[3] = (int)((w & c.sign_mask) | c.one_bits);
    d[4] = 0; d[5] = 0; d[6] = 0; d[7] = 0;   // unused by the 4-bit format
    return d;
}

// Fetch words [16*S + 4*g, +4) of a packed row.  ALIGNED: rows are 16-byte aligned and whole
// super-steps long.  Otherwise each word is bounds-checked against the row length and reads as 0.
template <bool ALIGNED>
__device__ __forceinline__ uint4 load_words(const uint32_t* __restrict__ row, int S, int g, int w32) {
    const int base = S * 16 + g * 4;
    if constexpr (ALIGNED) {
        return *reinterpret_cast<const uint4*>(row + base);
    } else {
        uint4 v;
        v.x = (base + 0 < w32) ? row[base + 0] : 0u;
        v.y = (base + 1 < w32) ? row[base + 1] : 0u;
        v.z = (base + 2 < w32) ? row[base + 2] : 0u;
        v.w = (base + 3 < w32) ? row[base + 3] : 0u;
        return v;
    }
}

__device__ __forceinline__ uint32_t word_of(const uint4& v, int j) {
    return j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w));
}

// Grid: x = ceil(M / (32*WM)), y = ceil(N / (32*WN)); block = 256 threads.
template <int WM, int WN, int ACT, bool ALIGNED>
__global__ __launch_bounds__(256) void binx_mfma_kernel(const uint32_t* __restrict__ Xp, const uint32_t* __restrict__ Wp,
                                                        const float* __restrict__ scale, const float* __restrict__ bias,
                                                        int M, int K, int N, int w32, void* __restrict__ Y, int yw32) {
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15;   // row of the operand fragment / column of the accumulator fragment
    const int g = lane >> 4;   // k-group of the operand fragment / row-group of the accumulator fragment
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int m_base = ((int)blockIdx.x * 2 + wave_m) * (WM * 16);
    const int n_base = ((int)blockIdx.y * 2 + wave_n) * (WN * 16);
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

    v4f acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    const ExpandConsts ec = expand_consts();
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
            v8i bx[WN];
#pragma unroll
            for (int f = 0; f < WN; ++f) bx[f] = expand_pm1_fp4(word_of(braw[f], j), ec);
#pragma unroll
            for (int fm = 0; fm < WM; ++fm) {
                const v8i ax = expand_pm1_fp4(word_of(araw[fm], j), ec);
#pragma unroll
                for (int fn = 0; fn < WN; ++fn)
                    acc[fm][fn] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ax, bx[fn], acc[fm][fn], 4, 4, 0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int f = 0; f < WM; ++f) araw[f] = anext[f];
#pragma unroll
        for (int f = 0; f < WN; ++f) braw[f] = bnext[f];
    }

    // ---- epilogue.  Accumulator fragment (fm, fn), register q of lane (r, g) is
    //      dot[m_base + 16 fm + 4 g + q][n_base + 16 fn + r] + pad.
    const float pad = (float)(nS * 512 - K);
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
        static_assert(ACT != ACT_SIGN || WN == 4, "the packed epilogue assumes 64 outputs per wave");
        uint32_t* Yw = (uint32_t*)Y;
        const int wcol = n_base >> 5;   // first 32-bit word of this wave's 64 outputs
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned long long b[WN];
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    const float h = affine(sc[fn], acc[fm][fn][q] - pad, bi[fn]);
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
                    const float dot = acc[fm][fn][q] - pad;
                    if (m < M && nvalid[fn]) {
                        if constexpr (ACT == ACT_RAW_I32) {
                            ((int*)Y)[(size_t)m * N + n] = (int)dot;
                        } else {
                            float h = affine(sc[fn], dot, bi[fn]);
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

// ---------------------------------------------------------------------------------------------------------
// Output layer (paper Alg. 2, l = L): binary product, affine step and log-Softmax in ONE kernel.
//
// A workgroup of 8 waves owns 16 frames and ALL N outputs, so the row maximum and the row sum of
// exponentials never leave the chip and the log-posteriors are the only thing written to HBM (one pass
// over the largest tensor of the network instead of write + read + write).  Wave v holds the NF accumulator
// fragments of outputs [16 NF v, 16 NF (v + 1)).
//
// K advances in super-steps of LW * 128 bits.  Lane (r, g) holds, per fragment, LW consecutive packed words
// of row r (one wide load: 4 lanes of a row read 16 LW contiguous bytes); word j feeds MFMA step j.  The
// registers of a fragment are reloaded for the NEXT super-step right after its LW products have been
// issued, so every load has the time of all other fragments' work to arrive and nothing is double-buffered:
// the register file holds the whole 16 x N accumulator tile plus one super-step of all N weight rows.
// Buffer addressing: per-lane byte offset of (row, lane group) in a VGPR, the super-step in the scalar
// offset; a read past the end of either matrix (rows past M or N) returns 0 and its results are never stored.
// Requires K % (128 LW) == 0, N <= 16 * 8 * NF and both packed matrices smaller than 2 GiB.
// Grid: x = ceil(M / 16); block = 512 threads.
template <int LW> struct RawWords;
template <> struct RawWords<4> {
    typedef unsigned int vec __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ vec load(__amdgpu_buffer_rsrc_t rs, int voff, int soff) {
        return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
    }
};
template <> struct RawWords<2> {
    typedef unsigned int vec __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ vec load(__amdgpu_buffer_rsrc_t rs, int voff, int soff) {
        return __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, 0);
    }
};

template <int NF, int LW>
__global__ __launch_bounds__(512) void binx_mfma_logsoftmax_kernel(const uint32_t* __restrict__ Xp,
                                                                   const uint32_t* __restrict__ Wp,
                                                                   const float* __restrict__ scale,
                                                                   const float* __restrict__ bias, int M, int K, int N,
                                                                   int w32, float* __restrict__ Y, unsigned int a_bytes,
                                                                   unsigned int b_bytes) {
    typedef typename RawWords<LW>::vec raw_t;
    __shared__ float red[8][16];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15, g = lane >> 4;
    const int m_base = (int)blockIdx.x * 16;
    const int n_wave = wave * NF * 16;
    const ExpandConsts ec = expand_consts();

    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(Xp), 0, (int)a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(Wp), 0, (int)b_bytes, 0x00020000);
    const int a_off = ((m_base + r) * w32 + LW * g) * 4;
    const int b_off = ((n_wave + r) * w32 + LW * g) * 4;   // fragment 0; fragment i adds i * frag_bytes (uniform)
    const int frag_bytes = 16 * w32 * 4;

    v4f acc[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) acc[i] = v4f{0.f, 0.f, 0.f, 0.f};

    const int nsuper = K / (128 * LW);
    raw_t braw[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) braw[i] = RawWords<LW>::load(wrs, b_off, i * frag_bytes);
    raw_t araw = RawWords<LW>::load(xrs, a_off, 0);
    for (int S = 0; S < nsuper; ++S) {
        const int so = 16 * LW * ((S + 1 < nsuper) ? S + 1 : S);   // bytes (4 LW words per row and super-step); the last reload is unused
        v8i ax[LW];
#pragma unroll
        for (int j = 0; j < LW; ++j) ax[j] = expand_pm1_fp4(araw[j], ec);
        araw = RawWords<LW>::load(xrs, a_off, so);
#pragma unroll
        for (int i = 0; i < NF; ++i) {
#pragma unroll
            for (int j = 0; j < LW; ++j) {
                const v8i bx = expand_pm1_fp4(braw[i][j], ec);
                acc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ax[j], bx, acc[i], 4, 4, 0, 0, 0, 0);
            }
            braw[i] = RawWords<LW>::load(wrs, b_off, so + i * frag_bytes);
        }
    }

    // ---- z = fma(scale, dot, bias); register q of lane (r, g), fragment i: frame m_base + 4 g + q, output n_wave + 16 i + r
    const float neg_inf = -__builtin_inff();
    float mx[4] = {neg_inf, neg_inf, neg_inf, neg_inf};
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int n = n_wave + i * 16 + r;
        const bool nv = n < N;
        const float sc = (scale && nv) ? scale[n] : 1.0f;
        const float bi = (bias && nv) ? bias[n] : 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float z = nv ? affine(sc, acc[i][q], bi) : neg_inf;
            acc[i][q] = z;
            mx[q] = fmaxf(mx[q], z);
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) mx[q] = fmaxf(mx[q], __shfl_xor(mx[q], off, kWave));
        if (r == 0) red[wave][4 * g + q] = mx[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float v = red[0][4 * g + q];
#pragma unroll
        for (int w = 1; w < 8; ++w) v = fmaxf(v, red[w][4 * g + q]);
        mx[q] = v;
    }
    __syncthreads();
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) sum[q] += __expf(acc[i][q] - mx[q]);      // exp(-inf) = 0 for outputs past N
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) sum[q] += __shfl_xor(sum[q], off, kWave);
        if (r == 0) red[wave][4 * g + q] = sum[q];
    }
    __syncthreads();
    float shift[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float v = red[0][4 * g + q];
#pragma unroll
        for (int w = 1; w < 8; ++w) v += red[w][4 * g + q];
        shift[q] = mx[q] + __logf(v);
    }
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int n = n_wave + i * 16 + r;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m_base + 4 * g + q;
            if (m < M && n < N) Y[(size_t)m * N + n] = acc[i][q] - shift[q];
        }
    }
}

}  // namespace bnn
