// Real-input layer with Sign output (paper Alg. 1 forward followed by Alg. 2's Sign) in ONE kernel on the
// matrix cores, bit-exact with the fp32 sum taken in ascending k.
//
// The output of this layer is one bit per unit: bit = (fma(scale, acc32, bias) > 0), where acc32 is the fp32
// sum of +-x[k] accumulated in ascending k.  A matrix core cannot reproduce that sum (its internal order is
// its own) but it can almost always reproduce the DECISION, by a filter with a rigorous error bound:
//
//   quantise   each frame x[m][:] is scaled by a power of two 2^s (from the row's largest exponent) and
//              rounded to integers |xq| <= 2^20, split into three digits of 7 bits (int8 MFMA operands);
//              per frame: R = sum xq, 2^-s, and a bound E on |acc32 - a 2^-s| (a = the exact integer sum of
//              +-xq): quantisation error (<= K/2 units) + the classical bound of a K-term recursive fp32 sum,
//              (K-1) u / (1 - K u) * sum|x|, + the int->float conversion error, inflated by 1 %.
//   multiply   three int8 MFMA products (one per digit) of the digits with the weight bits as 0/1 bytes give
//              P = sum_k b_k xq_k exactly; a = 2 P - R.
//   decide     acc -> (fma(scale, acc, bias) > 0) is monotone, so if both ends of [a - E, a + E] give the same
//              bit, that bit is the bit of acc32.  Otherwise the output is "uncertain" (a few in 10^4 on N(0,1)
//              inputs) and goes to a list in LDS; if the list is full the lane takes the fp32 sum itself.
//   resolve    for every listed (m, n) one lane takes the fp32 sum in ascending k exactly as the vector-ALU
//              kernel does (frame from LDS, weight words from memory), and sets the bit in the LDS copy of
//              the output tile.
//
// One workgroup (8 waves) owns 16 frames and all N outputs (up to 8192).  The frames are read once, kept in LDS
// in fp32 (for the resolution) and as three digit planes (for the products).  The weight rows stream through
// two LDS stages, 512 rows at a time: while one chunk is multiplied, the next one is in flight in registers
// (issue order pinned by scheduling barriers).  With M = 4096 that is 256 workgroups, one per CU.
//
// Operand order inside a 64-wide k step is permuted so that a lane expands its 16 weight bytes with shift+mask
// only: byte i of dword c' of lane group g is bit (4 (g & 1) + c' + 8 i) of packed word 2*step + (g >> 1).
// The digit bytes are written in the very same order, so both MFMA operands agree on which k sits where.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

typedef int v4i32 __attribute__((ext_vector_type(4)));

constexpr int kDigits = 3;
constexpr int kDigitBits = 7;
constexpr int kQuantBits = 20;         // |xq| <= 2^20
constexpr int kRealxMfmaMaxK = 512;    // LDS budget (frames in two forms + two weight stages); also 2 K 2^20 < 2^31
constexpr int kRealxBM = 16;           // frames per workgroup
constexpr int kRealxThreads = 512;     // 8 waves: two per SIMD, so one wave's latencies hide behind the other's work
constexpr int kRealxChunk = 512;       // outputs multiplied at a time (8 waves x 64)
constexpr int kRealxMaxNB = 8192;      // outputs per workgroup, at most
constexpr int kRealxListCap = 512;     // uncertain outputs a workgroup can list (expected: about a dozen)

struct RowMeta {
    int R;             // sum_k xq[k]
    float inv_scale;   // 2^-s
    float E;           // bound on |acc32 - a * 2^-s|
    int flags;         // 1: the row holds NaN/Inf or values too large to quantise -> every output is resolved exactly
};

// Byte offset (0..63) of element kk (0..63 of a k step) in the permuted operand order.
__device__ __forceinline__ int permuted_byte_of_k(int kk) {
    const int hw = kk >> 5, bitpos = kk & 31;
    const int c = bitpos & 7, i = bitpos >> 3;
    const int g = 2 * hw + (c >> 2), cp = c & 3;
    return 16 * g + 4 * cp + i;
}

// LDS layout (bytes from the start of the dynamic LDS): digit planes | fp32 frames | two weight stages | output tile
__host__ __device__ constexpr int realx_plane_row(int kpad) { return kpad + 16; }   // +16 spreads the 16 rows over the banks
// Words per weight row in an LDS stage.  16 lanes read the same word of 16 consecutive rows: a row length of
// 2 * odd words puts them in 16 different banks, and then a chunk is one contiguous copy; otherwise pad to odd.
__host__ __device__ constexpr int realx_wrow(int w32) { return (w32 & 3) == 2 ? w32 : (w32 | 1); }
__host__ __device__ constexpr size_t realx_off_xs(int kpad) { return (size_t)kDigits * kRealxBM * realx_plane_row(kpad); }
__host__ __device__ constexpr size_t realx_off_w(int K, int kpad) {
    return realx_off_xs(kpad) + ((size_t)kRealxBM * (K + 1) * 4 + 15) / 16 * 16;
}
__host__ __device__ constexpr size_t realx_stage_bytes(int w32) { return (size_t)kRealxChunk * realx_wrow(w32) * 4; }
__host__ __device__ constexpr size_t realx_off_tile(int K, int kpad, int w32) {
    return realx_off_w(K, kpad) + 2 * realx_stage_bytes(w32);
}
__host__ __device__ constexpr size_t realx_dynamic_lds(int K, int kpad, int w32, int nb) {
    return realx_off_tile(K, kpad, w32) + (size_t)kRealxBM * (nb / 32) * 4;
}

// The fp32 sum in ascending k for one output, operands in global memory (used only when the list overflows).
__device__ __noinline__ float canonical_acc_global(const float* __restrict__ x, const uint32_t* __restrict__ wrow, int K) {
    float acc = 0.0f;
    for (int k = 0; k < K; ++k) {
        const uint32_t inv = ~wrow[k >> 5];
        acc = __builtin_fmaf(pm1_from_inverted_bit(inv, k & 31), x[k], acc);
    }
    return acc;
}

// Grid: x = ceil(M / 16), y = ceil(N / NB); block = 512 threads; dynamic LDS = realx_dynamic_lds(K, kpad, w32, NB).
// NB is a multiple of 512.  VEC16: Wp is 16-byte aligned (16-byte loads of the weight chunks).
template <bool VEC16>
__global__ __launch_bounds__(kRealxThreads) void realx_sign_fused_kernel(const float* __restrict__ X, const uint32_t* __restrict__ Wp,
                                                               const float* __restrict__ scale, const float* __restrict__ bias,
                                                               int M, int K, int kpad, int N, int NB, int w32,
                                                               uint32_t* __restrict__ Y, int yw32) {
    constexpr int WN = 4;   // 16-output fragments per wave and chunk
    extern __shared__ __attribute__((aligned(16))) int8_t lds_raw[];
    __shared__ RowMeta meta[kRealxBM];
    __shared__ unsigned int list_count;
    __shared__ unsigned int list[kRealxListCap];   // (frame in tile) << 16 | (output in block)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15, g = lane >> 4;
    const int m_base = (int)blockIdx.x * kRealxBM;
    const int n_block = (int)blockIdx.y * NB;
    const int nb = min(NB, N - n_block);             // outputs of this workgroup
    const int plrow = realx_plane_row(kpad);
    const int ldw = realx_wrow(w32);
    const int xstride = K + 1;
    int8_t* planes = lds_raw;                                                            // [3][16][plrow]
    float* xs = reinterpret_cast<float*>(lds_raw + realx_off_xs(kpad));                  // [16][K + 1]
    uint32_t* wst = reinterpret_cast<uint32_t*>(lds_raw + realx_off_w(K, kpad));          // [2][512][ldw]
    uint32_t* tile = reinterpret_cast<uint32_t*>(lds_raw + realx_off_tile(K, kpad, w32)); // [16][NB / 32] packed outputs
    const int stage_words = kRealxChunk * ldw;
    const int tw = NB >> 5;
    if (threadIdx.x == 0) list_count = 0u;

    // ---- a chunk of weight rows: 512 rows = one contiguous run of words; a thread carries up to WPT 16-byte pieces
    constexpr int WPT = (kRealxChunk * ((kRealxMfmaMaxK + 31) / 32) / 4 + kRealxThreads - 1) / kRealxThreads;
    uint4 wreg[WPT];
    auto fetch_chunk = [&](int c0) {
        const int rows = min(kRealxChunk, nb - c0);
        const int total = rows * w32;                                     // words
        const uint32_t* src = Wp + (size_t)(n_block + c0) * w32;
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const int f = (int)threadIdx.x + i * kRealxThreads;
            wreg[i] = make_uint4(0u, 0u, 0u, 0u);
            if (VEC16 && 4 * f + 3 < total) {
                wreg[i] = reinterpret_cast<const uint4*>(src)[f];
            } else {                                                       // tail piece or unaligned matrix
                if (4 * f + 0 < total) wreg[i].x = src[4 * f + 0];
                if (4 * f + 1 < total) wreg[i].y = src[4 * f + 1];
                if (4 * f + 2 < total) wreg[i].z = src[4 * f + 2];
                if (4 * f + 3 < total) wreg[i].w = src[4 * f + 3];
            }
        }
    };
    auto store_chunk = [&](int c0, uint32_t* stage) {
        const int total = min(kRealxChunk, nb - c0) * w32;
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const int f = (int)threadIdx.x + i * kRealxThreads;
            if (ldw == w32 && 4 * f + 3 < total) {             // unpadded rows: the chunk is one contiguous run in LDS too
                reinterpret_cast<uint4*>(stage)[f] = wreg[i];
            } else if (4 * f < total) {
                int row = (4 * f) / w32, col = 4 * f - row * w32;
                const uint32_t w4[4] = {wreg[i].x, wreg[i].y, wreg[i].z, wreg[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (4 * f + j < total) stage[row * ldw + col] = w4[j];
                    if (++col == w32) { col = 0; ++row; }
                }
            }
        }
    };

    // ---- frames: wave w takes frames 2w and 2w+1, lane l elements l, l + 64, ...; every load of both rows and of
    //      the first weight chunk is issued before the first value is used
    constexpr int KPL = (kRealxMfmaMaxK + 63) / 64;            // elements per lane and row, at most
    constexpr int FPW = kRealxBM / (kRealxThreads / kWave);     // frames per wave
    float xv[FPW][KPL];
#pragma unroll
    for (int t = 0; t < FPW; ++t) {
        const int m = m_base + wave * FPW + t;
        const float* x = X + (size_t)(m < M ? m : M - 1) * K;
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            const int k = lane + 64 * i;
            xv[t][i] = (i * 64 < kpad && k < K) ? x[k] : 0.0f;   // first test is wave-uniform: unused slots cost nothing
        }
    }
    fetch_chunk(0);
#pragma unroll
    for (int t = 0; t < FPW; ++t) {
        const int ml = wave * FPW + t;
        unsigned int mx = 0;   // largest |x| of the row as a bit pattern (NaN/Inf have the largest patterns)
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            mx = max(mx, __float_as_uint(xv[t][i]) & 0x7fffffffu);
            if (i * 64 < kpad && lane + 64 * i < K) xs[ml * xstride + lane + 64 * i] = xv[t][i];
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned int)__shfl_xor((int)mx, off, kWave));
        const int e = (int)(mx >> 23) - 127;                 // floor(log2 max|x|) for normal numbers
        const int flags = (mx >= 0x7f800000u || e >= 100) ? 1 : 0;
        int s = kQuantBits - 1 - e;                           // max|x| < 2^(e+1)  =>  |x| 2^s < 2^20
        s = s > 100 ? 100 : s;
        const float qs = __uint_as_float((unsigned int)(s + 127) << 23);
        int R = 0, A = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            if (i * 64 < kpad) {   // wave-uniform
                const int xq = flags ? 0 : (int)__builtin_rintf(xv[t][i] * qs);   // slots past K hold 0
                R += xq;
                A += xq < 0 ? -xq : xq;
                const int pos = ml * plrow + i * 64 + permuted_byte_of_k(lane);
                planes[pos] = (int8_t)(xq & 127);
                planes[kRealxBM * plrow + pos] = (int8_t)((xq >> kDigitBits) & 127);
                planes[2 * kRealxBM * plrow + pos] = (int8_t)(xq >> (2 * kDigitBits));
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            R += __shfl_xor(R, off, kWave);
            A += __shfl_xor(A, off, kWave);
        }
        if (lane == 0) {
            const float u = 5.9604644775390625e-08f;                            // 2^-24; all terms in units of 2^-s
            const float Kf = (float)K;
            const float sum_abs = (float)A + 0.5f * Kf;                         // >= sum |x| 2^s
            const float e_seq = (Kf - 1.0f) * u / (1.0f - Kf * u) * sum_abs;    // recursive fp32 summation
            const float e_quant = 0.5f * Kf;                                     // |x 2^s - xq| <= 1/2 each
            const float e_conv = u * (float)A;                                   // (float)a
            const float inv = __uint_as_float((unsigned int)(127 - s) << 23);
            RowMeta rm;
            rm.R = R; rm.inv_scale = inv; rm.flags = flags;
            rm.E = flags ? __builtin_inff() : (e_seq + e_quant + e_conv) * 1.01f * inv;   // infinite bound: every output uncertain
            meta[ml] = rm;
        }
    }
    store_chunk(0, wst);
    __syncthreads();

    // ---- products and decisions, 512 outputs at a time; this wave's 64 outputs are nw .. nw+63 of the block
    const int nsteps = kpad >> 6;
    const int sh = 4 * (g & 1);
    const int8_t* al = planes + (size_t)r * plrow + 16 * g;
    RowMeta rmeta[4];
    unsigned long long mv[4];   // lanes whose frame 4g+q exists
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        rmeta[q] = meta[4 * g + q];
        mv[q] = __builtin_amdgcn_ballot_w64(m_base + 4 * g + q < M);
    }

    for (int c0 = 0, ci = 0; c0 < nb; c0 += kRealxChunk, ++ci) {
        const uint32_t* stage = wst + (ci & 1) * stage_words;
        const bool more = c0 + kRealxChunk < nb;     // workgroup-uniform
        if (more) fetch_chunk(c0 + kRealxChunk);
        __builtin_amdgcn_sched_barrier(0);
        const int nw = c0 + wave * (WN * 16);
        if (nw < nb) {   // wave-uniform
            // Outputs past the block's end get scale 0 and bias -1: pre-activation -1, certain, bit 0.
            float sc[WN], bi[WN], asc[WN];
            unsigned long long nv[WN];   // lanes whose output exists
#pragma unroll
            for (int fn = 0; fn < WN; ++fn) {
                const int nl = nw + fn * 16 + r;
                const bool nvalid = nl < nb;
                nv[fn] = __builtin_amdgcn_ballot_w64(nvalid);
                sc[fn] = nvalid ? (scale ? scale[n_block + nl] : 1.0f) : 0.0f;
                bi[fn] = nvalid ? (bias ? bias[n_block + nl] : 0.0f) : -1.0f;
                // |scale| (1 + 2^-16.6) covers the roundings of the margin; the floor covers a product that underflows
                asc[fn] = __builtin_fmaxf(__builtin_fabsf(sc[fn]) * 1.00001f, 1e-30f);
            }
            v4i32 acc[kDigits][WN];
#pragma unroll
            for (int d = 0; d < kDigits; ++d)
#pragma unroll
                for (int j = 0; j < WN; ++j) acc[d][j] = v4i32{0, 0, 0, 0};

            const uint32_t* bl = stage + (size_t)(wave * (WN * 16) + r) * ldw + (g >> 1);
            for (int st = 0; st < nsteps; ++st) {
                v4i32 bx[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f) {
                    const int wi = 2 * st + (g >> 1);
                    // rows past the block's outputs hold stale LDS (never stored); words past the row read as 0 (pad)
                    const uint32_t w = (wi < w32) ? bl[(size_t)f * 16 * ldw + 2 * st] : 0u;
                    const uint32_t ws = w >> sh;
                    bx[f][0] = (int)(ws & 0x01010101u);
                    bx[f][1] = (int)((ws >> 1) & 0x01010101u);
                    bx[f][2] = (int)((ws >> 2) & 0x01010101u);
                    bx[f][3] = (int)((ws >> 3) & 0x01010101u);
                }
#pragma unroll
                for (int d = 0; d < kDigits; ++d) {
                    const v4i32 ax = *reinterpret_cast<const v4i32*>(al + (size_t)d * kRealxBM * plrow + st * 64);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[d][fn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ax, bx[fn], acc[d][fn], 0, 0, 0);
                }
            }

            // accumulator register q of lane (r, g), fragment fn: frame 4g+q of the tile, output nw + 16 fn + r of the block.
            // With t = fma(scale, a, bias): if |t| > |scale| E (1 + 2^-16.6) + 1e-30, then scale x + bias has the sign
            // of t, and at least 1e-30 in magnitude, for every real x within E of a, so its rounding has that sign
            // too and the bit of the fp32 sum is (t > 0).  Anything else (NaN included) is uncertain.
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ml = 4 * g + q;
                const RowMeta rm = rmeta[q];
                unsigned long long b[WN], u[WN];
                unsigned long long any_u = 0ull;
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    const unsigned int P = ((((unsigned int)acc[2][fn][q] << kDigitBits) + (unsigned int)acc[1][fn][q]) << kDigitBits) +
                                           (unsigned int)acc[0][fn][q];
                    const float a = (float)(int)((P << 1) - (unsigned int)rm.R) * rm.inv_scale;
                    const float t = affine(sc[fn], a, bi[fn]);
                    const float margin = __builtin_fmaf(asc[fn], rm.E, 1e-30f);
                    const unsigned long long certain = __builtin_amdgcn_ballot_w64(__builtin_fabsf(t) > margin);
                    const unsigned long long pos = __builtin_amdgcn_ballot_w64(t > 0.0f);
                    u[fn] = ~certain & nv[fn] & mv[q];
                    b[fn] = pos & certain;
                    any_u |= u[fn];
                }
                if (any_u != 0ull) {   // wave-uniform, a few in 10^4 outputs
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn) {
                        bool bit = false;
                        if ((u[fn] >> lane) & 1ull) {
                            const int nl = nw + fn * 16 + r;
                            const unsigned int slot = atomicAdd(&list_count, 1u);
                            if (slot < (unsigned int)kRealxListCap) {
                                list[slot] = ((unsigned int)ml << 16) | (unsigned int)nl;   // resolved below; set by an LDS atomic OR if it is 1
                            } else {
                                const int m = m_base + ml;
                                bit = sign_bit(affine(sc[fn], canonical_acc_global(X + (size_t)m * K, Wp + (size_t)(n_block + nl) * w32, K), bi[fn]));
                            }
                        }
                        b[fn] |= __builtin_amdgcn_ballot_w64(bit);
                    }
                }
                if (lane < 4) {   // ballot bit 16 gg + rr: frame 4 gg + q, output 16 fn + rr; lane gg assembles frame 4 gg + q
                    const int shb = 16 * lane;
                    const uint32_t lo32 = (uint32_t)((b[0] >> shb) & 0xFFFFu) | ((uint32_t)((b[1] >> shb) & 0xFFFFu) << 16);
                    const uint32_t hi32 = (uint32_t)((b[2] >> shb) & 0xFFFFu) | ((uint32_t)((b[3] >> shb) & 0xFFFFu) << 16);
                    uint32_t* trow = tile + (size_t)(4 * lane + q) * tw + (nw >> 5);
                    trow[0] = lo32;
                    trow[1] = hi32;
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) store_chunk(c0 + kRealxChunk, wst + ((ci + 1) & 1) * stage_words);
        __syncthreads();
    }

    // ---- resolve the listed outputs exactly: fp32 sum in ascending k, one lane per output; the frame comes from
    //      LDS, the packed weight row (all its words fetched first: one memory latency) from global memory
    const int count = (int)min(list_count, (unsigned int)kRealxListCap);
    for (int i = threadIdx.x; i < count; i += kRealxThreads) {
        const unsigned int e = list[i];
        const int ml = (int)(e >> 16), nl = (int)(e & 0xFFFFu);
        const int n = n_block + nl;
        const uint32_t* wrow = Wp + (size_t)n * w32;
        const float* xr = xs + ml * xstride;
        constexpr int WMAX = (kRealxMfmaMaxK + 31) / 32;
        uint32_t wq[WMAX];
#pragma unroll
        for (int kw = 0; kw < WMAX; ++kw) wq[kw] = (kw * 32 < K) ? wrow[kw] : 0u;
        float acc = 0.0f;
        const int kfull = K >> 5;
#pragma unroll
        for (int kw = 0; kw < WMAX; ++kw) {
            if (kw >= kfull) break;
            const uint32_t inv = ~wq[kw];
            float xq[32];
#pragma unroll
            for (int kk = 0; kk < 32; ++kk) xq[kk] = xr[kw * 32 + kk];      // 32 independent LDS reads, then the chain
#pragma unroll
            for (int kk = 0; kk < 32; ++kk) acc = __builtin_fmaf(pm1_from_inverted_bit(inv, kk), xq[kk], acc);
        }
        if (K & 31) {
            const uint32_t inv = ~wrow[kfull];
            for (int kk = 0; kfull * 32 + kk < K; ++kk)
                acc = __builtin_fmaf(pm1_from_inverted_bit(inv, kk), xr[kfull * 32 + kk], acc);
        }
        const float s1 = scale ? scale[n] : 1.0f, b1 = bias ? bias[n] : 0.0f;
        if (sign_bit(affine(s1, acc, b1))) atomicOr(&tile[(size_t)ml * tw + (nl >> 5)], 1u << (nl & 31));
    }
    __syncthreads();

    // ---- write the tile: each frame's words are contiguous in memory
    const int words_here = min(tw, yw32 - (n_block >> 5));           // words of this block that exist in a row of Y
    const int words_filled = ((nb + 63) >> 6) << 1;                   // words some wave has filled
    for (int i = threadIdx.x; i < kRealxBM * tw; i += kRealxThreads) {
        const int ml = i / tw, wi = i - ml * tw;
        const int m = m_base + ml;
        if (m < M && wi < words_here && wi < words_filled) Y[(size_t)m * yw32 + (n_block >> 5) + wi] = tile[i];
    }
}

}  // namespace bnn
