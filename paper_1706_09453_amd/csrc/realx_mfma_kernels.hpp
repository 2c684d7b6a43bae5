// Real-input layer with Sign output (paper Alg. 1 forward followed by Alg. 2's Sign) on the matrix cores,
// bit-exact with the fp32 sum taken in ascending k.
//
// The output of this layer is one bit per unit: bit = (fma(scale, acc32, bias) > 0), where acc32 is the
// fp32 sum of +-x[k] accumulated in ascending k.  That sum cannot be reproduced by a matrix core (its
// internal order is its own), but its SIGN DECISION almost always can, by a filter:
//
//   1. quantize_rows_kernel: each frame x[m][:] is scaled by a power of two 2^s (from the row's largest
//      exponent) and rounded to integers |xq| <= 2^20, split into three digits of 7 bits (int8 operands).
//      Per row it also stores R = sum xq, 2^-s, and a rigorous bound E on |acc32 - a| where a is the
//      integer result scaled back: E = quantisation error (<= K/2 units) + the classical bound of a
//      K-term recursive fp32 sum, (K-1) u / (1 - K u) * sum|x|, + the int->float conversion error.
//   2. realx_mfma_sign_kernel: three int8 MFMA products (one per digit) of the digits with the weight
//      bits as 0/1 bytes give P = sum_k b_k xq_k exactly; a = 2 P - R is the exact integer sum of +-xq.
//      The map acc -> (fma(scale, acc, bias) > 0) is monotone, so if both ends of [a - E, a + E] give the
//      same bit, that bit is the bit of acc32.  Otherwise the output is "uncertain" (a few in 10^4 on
//      N(0,1) inputs) and goes to a small list in LDS; if the list is full the lane takes the fp32 sum itself.
//   3. Still in the same workgroup, after its products are done: for every listed (m, n) the frame is staged
//      in LDS and one lane takes the fp32 sum in ascending k, exactly as the vector-ALU kernel does; the
//      bit is set with an atomic OR if it is 1.  No global queue, no global counter, no second kernel.
//
// Operand order inside a 64-wide k step is permuted so that a lane expands its 16 weight bytes with
// shift+mask only: byte i of dword c' of lane group g is bit (4 (g & 1) + c' + 8 i) of packed word
// 2*step + (g >> 1).  quantize_rows_kernel writes the digit bytes in the very same order, so both MFMA
// operands agree on which k sits where; the sum over a step does not depend on that order.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

typedef int v4i32 __attribute__((ext_vector_type(4)));

struct RowMeta {        // 16 bytes per frame
    int R;              // sum_k xq[k]
    float inv_scale;    // 2^-s
    float E;            // bound on |acc32 - a * 2^-s|, already inflated; +inf never used: see flags
    int flags;          // 1: the row holds NaN/Inf or values too large to quantise -> every output uncertain
};

constexpr int kDigits = 3;
constexpr int kDigitBits = 7;
constexpr int kQuantBits = 20;      // |xq| <= 2^20
constexpr int kRealxMfmaMaxK = 1023; // 2 * K * 2^20 must stay below 2^31

// Position of element k (0 <= k < 64 within its step) in the permuted operand order: byte offset in [0, 64).
__device__ __forceinline__ int permuted_byte_of_k(int kk) {
    const int hw = kk >> 5, bitpos = kk & 31;
    const int c = bitpos & 7, i = bitpos >> 3;
    const int g = 2 * hw + (c >> 2), cp = c & 3;
    return 16 * g + 4 * cp + i;
}

// One wavefront per frame.  planes: [3][M][kpad] int8, kpad = 64 * ceil(K / 64), pad bytes 0.
__global__ __launch_bounds__(256) void quantize_rows_kernel(const float* __restrict__ X, int M, int K, int kpad,
                                                            int8_t* __restrict__ planes, RowMeta* __restrict__ meta) {
    const int lane = lane_id();
    const int m = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (m >= M) return;
    const float* x = X + (size_t)m * K;

    // largest magnitude of the row, as the bit pattern of |x| (NaN/Inf have the largest patterns)
    unsigned int mx = 0;
    for (int k = lane; k < K; k += kWave) mx = max(mx, __float_as_uint(x[k]) & 0x7fffffffu);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned int)__shfl_xor((int)mx, off, kWave));
    const int e = (int)(mx >> 23) - 127;                 // floor(log2 max|x|) for normal numbers
    int flags = (mx >= 0x7f800000u || e >= 100) ? 1 : 0;
    int s = kQuantBits - 1 - e;                           // max|x| < 2^(e+1)  =>  |x| 2^s < 2^20
    s = s > 100 ? 100 : s;
    const float scale = __uint_as_float((unsigned int)(s + 127) << 23);
    const float inv_scale = __uint_as_float((unsigned int)(127 - s) << 23);

    int8_t* p0 = planes + (size_t)m * kpad;
    int8_t* p1 = p0 + (size_t)M * kpad;
    int8_t* p2 = p1 + (size_t)M * kpad;
    int R = 0, A = 0;
    // each lane produces whole output dwords: dword (g, c') of a step holds k = 32 (g>>1) + 4 (g&1) + c' + 8 i
    const int ndw = kpad >> 2;
    for (int q = lane; q < ndw; q += kWave) {
        const int step = q >> 4, g = (q >> 2) & 3, cp = q & 3;
        unsigned int d0 = 0, d1 = 0, d2 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = step * 64 + 32 * (g >> 1) + 4 * (g & 1) + cp + 8 * i;
            int xq = 0;
            if (k < K && !flags) xq = (int)__builtin_rintf(x[k] * scale);
            R += xq;
            A += xq < 0 ? -xq : xq;
            d0 |= (unsigned int)(xq & 127) << (8 * i);
            d1 |= (unsigned int)((xq >> kDigitBits) & 127) << (8 * i);
            d2 |= (unsigned int)((xq >> (2 * kDigitBits)) & 255) << (8 * i);
        }
        reinterpret_cast<unsigned int*>(p0)[q] = d0;
        reinterpret_cast<unsigned int*>(p1)[q] = d1;
        reinterpret_cast<unsigned int*>(p2)[q] = d2;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        R += __shfl_xor(R, off, kWave);
        A += __shfl_xor(A, off, kWave);
    }
    if (lane == 0) {
        // all terms in units of 2^-s; u = 2^-24
        const float u = 5.9604644775390625e-08f;
        const float Kf = (float)K;
        const float sum_abs = (float)A + 0.5f * Kf;                         // >= sum |x| 2^s
        const float e_seq = (Kf - 1.0f) * u / (1.0f - Kf * u) * sum_abs;    // recursive fp32 summation
        const float e_quant = 0.5f * Kf;                                     // |x 2^s - xq| <= 1/2 each
        const float e_conv = u * (float)A;                                   // (float)a
        RowMeta r;
        r.R = R;
        r.inv_scale = inv_scale;
        r.E = (e_seq + e_quant + e_conv) * 1.01f * inv_scale;
        r.flags = flags;
        meta[m] = r;
    }
}

// The fp32 sum in ascending k for one output, as the vector-ALU kernel takes it (x read from global memory).
__device__ __noinline__ float canonical_acc_global(const float* __restrict__ x, const uint32_t* __restrict__ wrow, int K) {
    float acc = 0.0f;
    for (int k = 0; k < K; ++k) {
        const uint32_t inv = ~wrow[k >> 5];
        acc = __builtin_fmaf(pm1_from_inverted_bit(inv, k & 31), x[k], acc);
    }
    return acc;
}

// LDS row stride of a staged digit plane: kpad + 16 bytes keeps the 16 rows of a fragment on different banks.
__host__ __device__ constexpr int realx_lds_row(int kpad) { return kpad + 16; }
constexpr int kRealxBM = 32;    // frames per workgroup
constexpr int kRealxBN = 256;   // outputs per workgroup (4 waves x 64)

// LDS row stride (in words) of the staged weight rows: odd, so the 16 rows of a fragment hit different banks.
__host__ __device__ constexpr int realx_lds_wrow(int w32) { return w32 | 1; }
__host__ __device__ constexpr size_t realx_lds_bytes(int kpad, int w32) {
    return (size_t)kDigits * kRealxBM * realx_lds_row(kpad) + (size_t)kRealxBN * realx_lds_wrow(w32) * 4;
}

constexpr int kRealxListCap = 256;   // uncertain outputs a workgroup can list (expected: a handful)

// Grid: x = ceil(M / 32), y = ceil(N / 256); block = 256 threads; dynamic LDS = realx_lds_bytes(kpad, w32).
// K is short (a few hundred), so there is no steady state to pipeline: the workgroup first brings its 32
// frames of all three digit planes and its 256 packed weight rows into LDS, and every wave also fetches the
// per-frame bounds and per-output scale/bias it will need, with every global load in flight at once.  After
// one barrier each wave multiplies the whole tile of frames with its own 64 weight rows (2 x 4 accumulator
// fragments per digit) out of LDS only, decides the bits, and lists the uncertain ones; after a second
// barrier the workgroup resolves its list exactly (the frames' fp32 values take over the LDS of the digit
// planes, the weight rows are still there).
__global__ __launch_bounds__(256) void realx_mfma_sign_kernel(
    const float* __restrict__ X, const int8_t* __restrict__ planes, const RowMeta* __restrict__ meta,
    const uint32_t* __restrict__ Wp, const float* __restrict__ scale, const float* __restrict__ bias, int M, int K,
    int kpad, int N, int w32, uint32_t* __restrict__ Y, int yw32) {
    constexpr int WM = 2, WN = 4;
    extern __shared__ __attribute__((aligned(16))) int8_t lds_a[];
    __shared__ unsigned int list_count;
    __shared__ unsigned int list[kRealxListCap];          // (frame in tile) << 16 | (output in tile)
    __shared__ uint32_t tile_words[kRealxBM][kRealxBN / 32];   // the packed output tile, written to memory at the end
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15, g = lane >> 4;
    const int m_base = (int)blockIdx.x * kRealxBM;
    const int n_block = (int)blockIdx.y * kRealxBN;
    const int n_base = n_block + wave * (WN * 16);
    const int ldrow = realx_lds_row(kpad);
    const int ldw = realx_lds_wrow(w32);
    const int a_bytes = kDigits * kRealxBM * ldrow;
    uint32_t* lds_b = reinterpret_cast<uint32_t*>(lds_a + a_bytes);
    const size_t plane_stride = (size_t)M * kpad;
    if (threadIdx.x == 0) list_count = 0u;

    // ---- stage the frames: 8 threads per frame, 16-byte chunks, three digit planes
    {
        const int row = (int)threadIdx.x >> 3, c0 = (int)threadIdx.x & 7;
        const int m = m_base + row;
        const int8_t* src = planes + (size_t)(m < M ? m : M - 1) * kpad;
        const int cpr = kpad >> 4;
        for (int col = c0; col < cpr; col += 8) {
#pragma unroll
            for (int d = 0; d < kDigits; ++d)
                *reinterpret_cast<v4i32*>(lds_a + (size_t)(d * kRealxBM + row) * ldrow + 16 * col) =
                    *reinterpret_cast<const v4i32*>(src + d * plane_stride + 16 * col);
        }
    }
    // ---- stage the packed weight rows: one thread per output of the workgroup
    {
        const int n = n_block + (int)threadIdx.x;
        const uint32_t* src = Wp + (size_t)(n < N ? n : N - 1) * w32;
        uint32_t* dst = lds_b + (size_t)threadIdx.x * ldw;
        for (int w = 0; w < w32; ++w) dst[w] = src[w];
    }
    // ---- what the epilogue needs, fetched now so that its latency hides behind the products
    RowMeta rmeta[WM][4];
#pragma unroll
    for (int fm = 0; fm < WM; ++fm)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m_base + fm * 16 + 4 * g + q;
            rmeta[fm][q] = meta[m < M ? m : M - 1];
        }
    float sc[WN], bi[WN];
    bool nvalid[WN];
#pragma unroll
    for (int fn = 0; fn < WN; ++fn) {
        const int n = n_base + fn * 16 + r;
        nvalid[fn] = n < N;
        sc[fn] = (scale && nvalid[fn]) ? scale[n] : 1.0f;
        bi[fn] = (bias && nvalid[fn]) ? bias[n] : 0.0f;
    }
    __syncthreads();

    if (n_base < N) {   // wave-uniform; waves past the last output skip the products but keep the barriers
        v4i32 acc[kDigits][WM][WN];
#pragma unroll
        for (int d = 0; d < kDigits; ++d)
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) acc[d][i][j] = v4i32{0, 0, 0, 0};

        const int nsteps = kpad >> 6;
        const int sh = 4 * (g & 1);
        const uint32_t* bl = lds_b + (size_t)(wave * (WN * 16) + r) * ldw + (g >> 1);
        const int8_t* al = lds_a + (size_t)r * ldrow + 16 * g;
        for (int st = 0; st < nsteps; ++st) {
            v4i32 bx[WN];
#pragma unroll
            for (int f = 0; f < WN; ++f) {
                const int wi = 2 * st + (g >> 1);
                const uint32_t w = (wi < w32) ? bl[(size_t)f * 16 * ldw + 2 * st] : 0u;   // words past the row read as 0 (pad)
                const uint32_t ws = w >> sh;
                bx[f][0] = (int)(ws & 0x01010101u);
                bx[f][1] = (int)((ws >> 1) & 0x01010101u);
                bx[f][2] = (int)((ws >> 2) & 0x01010101u);
                bx[f][3] = (int)((ws >> 3) & 0x01010101u);
            }
#pragma unroll
            for (int d = 0; d < kDigits; ++d) {
#pragma unroll
                for (int fm = 0; fm < WM; ++fm) {
                    const v4i32 ax = *reinterpret_cast<const v4i32*>(al + (size_t)(d * kRealxBM + fm * 16) * ldrow + st * 64);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[d][fm][fn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ax, bx[fn], acc[d][fm][fn], 0, 0, 0);
                }
            }
        }

        // ---- decide: accumulator register q of lane (r, g), fragment (fm, fn) is frame m_base+16fm+4g+q, output n_base+16fn+r
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ml = fm * 16 + 4 * g + q;
                const int m = m_base + ml;
                const bool mvalid = m < M;
                const RowMeta rm = rmeta[fm][q];
                unsigned long long b[WN];
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    const int P = acc[0][fm][fn][q] + acc[1][fm][fn][q] * (1 << kDigitBits) + acc[2][fm][fn][q] * (1 << (2 * kDigitBits));
                    const float a = (float)(2 * P - rm.R) * rm.inv_scale;
                    const float Ew = rm.E + __builtin_fabsf(a) * 2.384185791015625e-07f;   // + 2^-22 |a| for the two roundings below
                    const bool lo = sign_bit(affine(sc[fn], a - Ew, bi[fn]));
                    const bool hi = sign_bit(affine(sc[fn], a + Ew, bi[fn]));
                    bool bit = lo;
                    if (mvalid && nvalid[fn] && (lo != hi || rm.flags)) {
                        const int nl = wave * (WN * 16) + fn * 16 + r;
                        const unsigned int slot = atomicAdd(&list_count, 1u);
                        if (slot < (unsigned int)kRealxListCap) {
                            list[slot] = ((unsigned int)ml << 16) | (unsigned int)nl;
                            bit = false;                       // resolved below; set by an LDS atomic OR if it is 1
                        } else {
                            bit = sign_bit(affine(sc[fn], canonical_acc_global(X + (size_t)m * K, Wp + (size_t)(n_block + nl) * w32, K), bi[fn]));
                        }
                    }
                    b[fn] = __ballot(nvalid[fn] && bit);
                }
                if (lane < 4) {
                    const int shb = 16 * lane;
                    const uint32_t lo32 = (uint32_t)((b[0] >> shb) & 0xFFFFu) | ((uint32_t)((b[1] >> shb) & 0xFFFFu) << 16);
                    const uint32_t hi32 = (uint32_t)((b[2] >> shb) & 0xFFFFu) | ((uint32_t)((b[3] >> shb) & 0xFFFFu) << 16);
                    const int mlw = fm * 16 + 4 * lane + q;
                    tile_words[mlw][2 * wave] = lo32;
                    tile_words[mlw][2 * wave + 1] = hi32;
                }
            }
        }
    }
    __syncthreads();   // products done everywhere: the digit planes' LDS can be reused

    // ---- resolve the listed outputs exactly: fp32 sum in ascending k, one lane per output
    const int count = (int)min(list_count, (unsigned int)kRealxListCap);
    float* xs = reinterpret_cast<float*>(lds_a);
    const int xstride = K + 1;
    int rows = a_bytes / (xstride * 4);
    rows = rows > 64 ? 64 : rows;
    for (int base = 0; base < count; base += rows) {
        const int nr = min(rows, count - base);
        for (int t = 0; t < nr; ++t) {
            const float* x = X + (size_t)(m_base + (int)(list[base + t] >> 16)) * K;
            for (int k = threadIdx.x; k < K; k += 256) xs[t * xstride + k] = x[k];
        }
        __syncthreads();
        if ((int)threadIdx.x < nr) {
            const unsigned int e = list[base + threadIdx.x];
            const int ml = (int)(e >> 16), nl = (int)(e & 0xFFFFu);
            const uint32_t* wrow = lds_b + (size_t)nl * ldw;
            const float* xr = xs + threadIdx.x * xstride;
            float acc = 0.0f;
            const int kfull = K >> 5;
            for (int kw = 0; kw < kfull; ++kw) {
                const uint32_t inv = ~wrow[kw];
                float xv[32];
#pragma unroll
                for (int kk = 0; kk < 32; ++kk) xv[kk] = xr[kw * 32 + kk];      // 32 independent LDS reads, then the chain
#pragma unroll
                for (int kk = 0; kk < 32; ++kk) acc = __builtin_fmaf(pm1_from_inverted_bit(inv, kk), xv[kk], acc);
            }
            if (K & 31) {
                const uint32_t inv = ~wrow[kfull];
                for (int kk = 0; kfull * 32 + kk < K; ++kk)
                    acc = __builtin_fmaf(pm1_from_inverted_bit(inv, kk), xr[kfull * 32 + kk], acc);
            }
            const int n = n_block + nl;
            const float s1 = scale ? scale[n] : 1.0f, b1 = bias ? bias[n] : 0.0f;
            if (sign_bit(affine(s1, acc, b1))) atomicOr(&tile_words[ml][nl >> 5], 1u << (nl & 31));
        }
        __syncthreads();
    }

    // ---- write the tile: 8 consecutive words per frame
    {
        const int ml = (int)threadIdx.x >> 3, wl = (int)threadIdx.x & 7;
        const int m = m_base + ml, w = (n_block >> 5) + wl;
        const bool wave_had_outputs = n_block + 64 * (wl >> 1) < N;   // words of skipped waves were never filled
        if (m < M && w < yw32 && wave_had_outputs) Y[(size_t)m * yw32 + w] = tile_words[ml][wl];
    }
}

}  // namespace bnn
