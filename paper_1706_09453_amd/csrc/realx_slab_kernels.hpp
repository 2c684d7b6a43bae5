// Real-input layer with Sign output for any input width (paper Alg. 1 forward followed by Alg. 2's Sign), bit-exact with
// the fp32 sum taken in ascending k: the matrix-core filter of realx_fused_kernel.hpp with K streamed in slabs.
//
// The filter is the one described there: quantise every frame to integers split into three 7-bit digits, three int8
// MFMA products against the weight bits as 0/1 bytes, decide every output whose interval [a - E, a + E] lies on one
// side of the threshold, and take the exact ascending-k fp32 sum for the rest.  What differs:
//   - the frames are quantised by a kernel of their own (realx_quantize_kernel) into digit planes in global memory,
//     [digit][frame][kpad] bytes in the MFMA's operand order, with one RowMeta per frame; any layer of a network can
//     then use the filter (the Sigmoid -> Sign layer of the paper's Table 2 topology has 2048 inputs), not only a
//     first layer of at most 512 inputs whose frames fit in LDS;
//   - a workgroup owns 16 frames x 512 outputs and walks K in slabs of 512: digit planes and weight words of a slab
//     go through LDS (two buffers: the next slab is in flight in registers while the current one is multiplied), the
//     int32 accumulators stay in registers across slabs;
//   - quantisation to |xq| <= 2^qb with qb = 29 - ceil(log2 K) (18 bits at K = 2048): 2 K 2^qb stays below 2^31;
//   - the exact sums of the listed outputs run slab by slab as well: all threads form the signed terms +-x[k] of the
//     listed sums for one slab in LDS (frames and weight words fetched side by side: one memory latency per slab), then
//     one lane per output adds its 512 terms in ascending k.  acc + (+-x) rounds exactly as fma(+-1, x, acc) does.
#pragma once

#include "realx_fused_kernel.hpp"

namespace bnn {

constexpr int kSlabK = 512;              // inputs per slab: 8 MFMA steps of 64
constexpr int kSlabNB = 512;             // outputs per workgroup (8 waves x 64)
constexpr int kSlabThreads = 512;
constexpr int kSlabMaxK = 8192;          // qb = 16 there
constexpr int kSlabPlaneRow = kSlabK + 16;   // bytes per frame row of a plane slab in LDS (+16 spreads the rows over the banks)
constexpr int kSlabWRow = 17;            // words per weight row of a slab in LDS (odd: 16 consecutive rows hit 16 banks)
constexpr int kSlabListCap = 512;
constexpr int kSlabTermRow = kSlabK + 4; // floats per listed output in the term table

__host__ __device__ constexpr int slab_quant_bits(int K) {
    int lg = 0;
    while ((1 << lg) < K) ++lg;          // ceil(log2 K)
    const int qb = 29 - lg;
    return qb > kQuantBits ? kQuantBits : qb;
}
__host__ __device__ constexpr size_t slab_planes_bytes() { return (size_t)2 * kDigits * kRealxBM * kSlabPlaneRow; }
__host__ __device__ constexpr size_t slab_weights_bytes() { return (size_t)2 * kSlabNB * kSlabWRow * 4; }
__host__ __device__ constexpr size_t slab_dynamic_lds() {
    return slab_planes_bytes() + slab_weights_bytes() + (size_t)kRealxBM * (kSlabNB / 32) * 4;
}

// One wave per frame: scale, digits, RowMeta.  planes: [kDigits][M][kpad] bytes; within every 64 elements the bytes sit
// in the permuted operand order (permuted_byte_of_k).  Elements past K are 0.
// INREG: K % 4 == 0, K <= 2048 and X 16-byte aligned: the frame is read once, 16 bytes per lane and request, all eight
// requests in flight together, and stays in registers between the search for its largest element and the quantisation.
// Otherwise it is read twice, element by element.
// Grid: ceil(M / 4) workgroups of 256 threads.
template <bool INREG>
__global__ __launch_bounds__(256) void realx_quantize_kernel(const float* __restrict__ X, int M, int K, int kpad, int qbits,
                                                             int8_t* __restrict__ planes, RowMeta* __restrict__ meta) {
    const int m = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (m >= M) return;   // wave-uniform
    const int lane = lane_id();
    const float* x = X + (size_t)m * K;
    unsigned int mx = 0;   // largest |x| of the row as a bit pattern (NaN/Inf have the largest patterns)
    float4 xr[8];          // INREG: elements 256 c + 4 lane .. + 3 of the frame
    if constexpr (INREG) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int k = 256 * c + 4 * lane;
            xr[c] = k < K ? *reinterpret_cast<const float4*>(x + k) : make_float4(0.f, 0.f, 0.f, 0.f);   // K % 4 == 0
        }
#pragma unroll
        for (int c = 0; c < 8; ++c)
            mx = max(max(mx, max(__float_as_uint(xr[c].x) & 0x7fffffffu, __float_as_uint(xr[c].y) & 0x7fffffffu)),
                     max(__float_as_uint(xr[c].z) & 0x7fffffffu, __float_as_uint(xr[c].w) & 0x7fffffffu));
    } else {
        for (int k0 = 0; k0 < K; k0 += 64) {
            const int k = k0 + lane;
            if (k < K) mx = max(mx, __float_as_uint(x[k]) & 0x7fffffffu);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned int)__shfl_xor((int)mx, off, kWave));
    const int e = (int)(mx >> 23) - 127;                 // floor(log2 max|x|) for normal numbers
    const int flags = (mx >= 0x7f800000u || e >= 100) ? 1 : 0;
    int s = qbits - 1 - e;                                // max|x| < 2^(e+1)  =>  |x| 2^s < 2^qbits
    s = s > 100 ? 100 : s;
    const float qs = __uint_as_float((unsigned int)(s + 127) << 23);
    const size_t plane = (size_t)M * kpad;
    int8_t* row = planes + (size_t)m * kpad;
    // 256 elements at a time: the digit bytes go to their permuted places in a slice of LDS, and leave as whole dwords,
    // 256 contiguous bytes per digit and store instruction
    __shared__ __attribute__((aligned(16))) int8_t qstage[4][kDigits][256];
    int8_t (*qs3)[256] = qstage[threadIdx.x >> 6];
    int R = 0, A = 0;
    auto put = [&](float v, int at) {
        const int xq = flags ? 0 : (int)__builtin_rintf(v * qs);
        R += xq;
        A += xq < 0 ? -xq : xq;
        qs3[0][at] = (int8_t)(xq & 127);
        qs3[1][at] = (int8_t)((xq >> kDigitBits) & 127);
        qs3[2][at] = (int8_t)(xq >> (2 * kDigitBits));
    };
    auto flush = [&](int k0) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // this wave's LDS writes before it reads them back
        const int kd = k0 + 4 * lane;
        if (kd < kpad) {   // (kpad is a multiple of 64: a dword is inside or outside as a whole)
#pragma unroll
            for (int d = 0; d < kDigits; ++d)
                *reinterpret_cast<int*>(row + d * plane + kd) = *reinterpret_cast<const int*>(&qs3[d][4 * lane]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // reads done before the next round overwrites the slice
    };
    if constexpr (INREG) {
        // this lane's four elements of a round sit in block lane / 16 of the round, at 4 (lane % 16) .. + 3 of the block
        const int blk = 64 * (lane >> 4), kk = 4 * (lane & 15);
        const int p0 = blk + permuted_byte_of_k(kk), p1 = blk + permuted_byte_of_k(kk + 1), p2 = blk + permuted_byte_of_k(kk + 2),
                  p3 = blk + permuted_byte_of_k(kk + 3);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if (256 * c < kpad) {   // wave-uniform
                put(xr[c].x, p0); put(xr[c].y, p1); put(xr[c].z, p2); put(xr[c].w, p3);
                flush(256 * c);
            }
        }
    } else {
        const int pos = permuted_byte_of_k(lane);
        for (int k0 = 0; k0 < kpad; k0 += 256) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int kb = k0 + 64 * b;
                if (kb < kpad) {   // wave-uniform
                    const int k = kb + lane;
                    put(k < K ? x[k] : 0.0f, 64 * b + pos);
                }
            }
            flush(k0);
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
        const float sum_abs = (float)A * 1.0000002f + 0.5f * Kf;            // >= sum |x| 2^s ((float)A rounds: one ulp added)
        const float e_seq = (Kf - 1.0f) * u / (1.0f - Kf * u) * sum_abs;    // recursive fp32 summation
        const float e_quant = 0.5f * Kf;                                     // |x 2^s - xq| <= 1/2 each
        const float e_conv = u * (float)A * 1.0000002f;                      // (float)a
        const float inv = __uint_as_float((unsigned int)(127 - s) << 23);
        RowMeta rm;
        rm.R = R; rm.inv_scale = inv; rm.flags = flags;
        rm.E = flags ? __builtin_inff() : (e_seq + e_quant + e_conv) * 1.01f * inv;   // infinite bound: every output uncertain
        meta[m] = rm;
    }
}

// Grid: x = ceil(M / 16), y = ceil(N / 512); block = 512 threads; dynamic LDS = slab_dynamic_lds().
// VEC16: Wp is 16-byte aligned and w32 % 4 == 0 (16-byte loads of the weight words of a slab).
template <bool VEC16>
__global__ __launch_bounds__(kSlabThreads) void realx_sign_slab_kernel(const float* __restrict__ X, const int8_t* __restrict__ planes,
                                                                      const RowMeta* __restrict__ meta, const uint32_t* __restrict__ Wp,
                                                                      const float* __restrict__ scale, const float* __restrict__ bias,
                                                                      int M, int K, int kpad, int N, int w32,
                                                                      uint32_t* __restrict__ Y, int yw32) {
    constexpr int WN = 4;   // 16-output fragments per wave
    extern __shared__ __attribute__((aligned(16))) int8_t lds_raw[];
    __shared__ RowMeta meta_s[kRealxBM];
    __shared__ unsigned int list_count;
    __shared__ unsigned int list[kSlabListCap];   // (frame in tile) << 16 | (output in block)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15, g = lane >> 4;
    const int m_base = (int)blockIdx.x * kRealxBM;
    const int n_block = (int)blockIdx.y * kSlabNB;
    const int nb = min(kSlabNB, N - n_block);             // outputs of this workgroup
    int8_t* pl = lds_raw;                                                                 // [2][3][16][kSlabPlaneRow]
    uint32_t* wst = reinterpret_cast<uint32_t*>(lds_raw + slab_planes_bytes());            // [2][512][kSlabWRow]
    uint32_t* tile = reinterpret_cast<uint32_t*>(lds_raw + slab_planes_bytes() + slab_weights_bytes());   // [16][16] packed outputs
    constexpr int tw = kSlabNB / 32;
    constexpr int pl_buf = kDigits * kRealxBM * kSlabPlaneRow;
    constexpr int w_buf = kSlabNB * kSlabWRow;
    if (threadIdx.x == 0) list_count = 0u;
    if (threadIdx.x < kRealxBM) {
        const int m = m_base + (int)threadIdx.x;
        meta_s[threadIdx.x] = meta[m < M ? m : M - 1];
    }
    const int nsl = (kpad + kSlabK - 1) / kSlabK;
    const size_t plane = (size_t)M * kpad;

    // ---- a slab on its way: 3 pieces of the digit planes and 4 of the weight words per thread, 16 bytes each
    uint4 preg[3], wreg[4];
    auto fetch_slab = [&](int sl) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;        // 0 .. 1535
            const int rowi = p >> 5, c16 = p & 31;                    // (digit, frame) row 0 .. 47, 16-byte column
            const int d = rowi >> 4, f = rowi & 15;
            const int m = m_base + f;
            const int k = sl * kSlabK + c16 * 16;
            preg[i] = make_uint4(0u, 0u, 0u, 0u);
            if (k < kpad)   // kpad is a multiple of 64: a piece is inside or outside as a whole
                preg[i] = *reinterpret_cast<const uint4*>(planes + d * plane + (size_t)(m < M ? m : M - 1) * kpad + k);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;        // 0 .. 2047
            const int rowi = p >> 2, q = p & 3;
            const int wi = sl * 16 + q * 4;
            const uint32_t* src = Wp + (size_t)(n_block + (rowi < nb ? rowi : nb - 1)) * w32;
            wreg[i] = make_uint4(0u, 0u, 0u, 0u);
            if (VEC16 && wi + 3 < w32) {
                wreg[i] = *reinterpret_cast<const uint4*>(src + wi);
            } else {
                if (wi + 0 < w32) wreg[i].x = src[wi + 0];
                if (wi + 1 < w32) wreg[i].y = src[wi + 1];
                if (wi + 2 < w32) wreg[i].z = src[wi + 2];
                if (wi + 3 < w32) wreg[i].w = src[wi + 3];
            }
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;
            const int rowi = p >> 5, c16 = p & 31;
            *reinterpret_cast<uint4*>(pl + buf * pl_buf + rowi * kSlabPlaneRow + c16 * 16) = preg[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;
            const int rowi = p >> 2, q = p & 3;
            uint32_t* dst = wst + buf * w_buf + rowi * kSlabWRow + q * 4;
            dst[0] = wreg[i].x; dst[1] = wreg[i].y; dst[2] = wreg[i].z; dst[3] = wreg[i].w;
        }
    };

    fetch_slab(0);
    store_slab(0);
    __syncthreads();

    // ---- products: this wave's 64 outputs are nw .. nw + 63 of the block; accumulators live across the slabs
    const int nw = wave * (WN * 16);
    const int sh = 4 * (g & 1);
    v4i32 acc[kDigits][WN];
#pragma unroll
    for (int d = 0; d < kDigits; ++d)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[d][j] = v4i32{0, 0, 0, 0};
    for (int sl = 0; sl < nsl; ++sl) {
        const int buf = sl & 1;
        const bool more = sl + 1 < nsl;          // workgroup-uniform
        if (more) fetch_slab(sl + 1);
        __builtin_amdgcn_sched_barrier(0);
        if (nw < nb) {   // wave-uniform
            const int8_t* al = pl + buf * pl_buf + r * kSlabPlaneRow + 16 * g;
            const uint32_t* bl = wst + buf * w_buf + (nw + r) * kSlabWRow + (g >> 1);
            const int steps = min(kSlabK, kpad - sl * kSlabK) >> 6;
            for (int st = 0; st < steps; ++st) {
                v4i32 bx[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f) {
                    // (rows past the block's outputs repeat its last row; their outputs are never written)
                    const uint32_t ws = bl[f * 16 * kSlabWRow + 2 * st] >> sh;
                    bx[f][0] = (int)(ws & 0x01010101u);
                    bx[f][1] = (int)((ws >> 1) & 0x01010101u);
                    bx[f][2] = (int)((ws >> 2) & 0x01010101u);
                    bx[f][3] = (int)((ws >> 3) & 0x01010101u);
                }
#pragma unroll
                for (int d = 0; d < kDigits; ++d) {
                    const v4i32 ax = *reinterpret_cast<const v4i32*>(al + d * kRealxBM * kSlabPlaneRow + st * 64);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[d][fn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ax, bx[fn], acc[d][fn], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) store_slab(buf ^ 1);
        __syncthreads();
    }

    // ---- decisions (the margin test of realx_fused_kernel.hpp): accumulator register q of lane (r, g), fragment fn is
    //      frame 4 g + q of the tile, output nw + 16 fn + r of the block
    if (nw < nb) {   // wave-uniform
        float sc[WN], bi[WN], asc[WN];
        unsigned long long nv[WN];   // lanes whose output exists
#pragma unroll
        for (int fn = 0; fn < WN; ++fn) {
            const int nl = nw + fn * 16 + r;
            const bool nvalid = nl < nb;
            nv[fn] = __builtin_amdgcn_ballot_w64(nvalid);
            sc[fn] = nvalid ? (scale ? scale[n_block + nl] : 1.0f) : 0.0f;
            bi[fn] = nvalid ? (bias ? bias[n_block + nl] : 0.0f) : -1.0f;
            asc[fn] = __builtin_fmaxf(__builtin_fabsf(sc[fn]) * 1.00001f, 1e-30f);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ml = 4 * g + q;
            const RowMeta rm = meta_s[ml];
            const unsigned long long mvalid = __builtin_amdgcn_ballot_w64(m_base + ml < M);
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
                u[fn] = ~certain & nv[fn] & mvalid;
                b[fn] = pos & certain;
                any_u |= u[fn];
            }
            if (any_u != 0ull) {   // wave-uniform
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    bool bit = false;
                    if ((u[fn] >> lane) & 1ull) {
                        const int nl = nw + fn * 16 + r;
                        const unsigned int slot = atomicAdd(&list_count, 1u);
                        if (slot < (unsigned int)kSlabListCap) {
                            list[slot] = ((unsigned int)ml << 16) | (unsigned int)nl;   // resolved below
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
                uint32_t* trow = tile + (4 * lane + q) * tw + (nw >> 5);
                trow[0] = lo32;
                trow[1] = hi32;
            }
        }
    }
    __syncthreads();

    // ---- the listed outputs, exactly: slab by slab, a table of signed terms in LDS (the slab buffers are free now),
    //      then one lane per output down its row of the table
    const int count = (int)min(list_count, (unsigned int)kSlabListCap);
    float* terms = reinterpret_cast<float*>(lds_raw);
    constexpr int kTermRows = 56;   // 7 preparing waves x 8 outputs (the table has room for 58)
    static_assert((size_t)kTermRows * kSlabTermRow * 4 <= slab_planes_bytes() + slab_weights_bytes(), "term table");
    constexpr int kWaves = kSlabThreads / kWave - 1;               // waves 1 .. 7 prepare terms, wave 0 adds them up
    constexpr int kPerWave = (kTermRows + kWaves - 1) / kWaves;   // listed outputs a wave prepares per pass: 8
    const int pw = wave - 1;                                       // preparing wave 0 .. 6 (wave 0 of the workgroup: -1)
    for (int base = 0; base < count; base += kTermRows) {   // workgroup-uniform
        const int ne = min(kTermRows, count - base);
        // Preparing wave w takes outputs w, w + 7, ...; lane l their terms of k = 64 j + l.  The frames' values and the weight
        // words of a slab are requested for all of a wave's outputs at once (no request is conditional: past the last
        // listed output the last one is fetched again) and one slab ahead of the sums, so that a slab costs one pass
        // over its 512 terms and no memory round trip of its own.
        float xv[kPerWave][8];
        uint32_t wv[kPerWave][8];
        auto request = [&](int sl) {
            if (pw < 0) return;   // wave-uniform
#pragma unroll
            for (int q = 0; q < kPerWave; ++q) {
                const int i = min(pw + kWaves * q, ne - 1);
                const unsigned int e = list[base + i];
                const int ml = (int)(e >> 16), nl = (int)(e & 0xFFFFu);
                const float* xr = X + (size_t)(m_base + ml) * K;
                const uint32_t* wr = Wp + (size_t)(n_block + nl) * w32;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = min(sl * kSlabK + 64 * j + lane, K - 1);   // past K: in bounds, unused
                    xv[q][j] = xr[k];
                    wv[q][j] = wr[k >> 5];
                }
            }
        };
        request(0);
        float acc32 = 0.0f;
        for (int sl = 0; sl < nsl; ++sl) {
#pragma unroll
            for (int q = 0; q < kPerWave; ++q) {
                const int i = pw + kWaves * q;
                if (pw >= 0 && i < ne) {   // wave-uniform
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t flip = (~wv[q][j] >> (lane & 31)) << 31;             // weight bit 0: -x
                        terms[i * kSlabTermRow + 64 * j + lane] = __uint_as_float(__float_as_uint(xv[q][j]) ^ flip);
                    }
                }
            }
            __syncthreads();
            if (sl + 1 < nsl) request(sl + 1);
            if ((int)threadIdx.x < ne) {
                const float* tr = terms + threadIdx.x * kSlabTermRow;
                const int kn = min(kSlabK, K - sl * kSlabK);
                // 32 terms per batch of LDS reads; the next batch is requested before this one is added up (past the end
                // of the row the reads stay inside the table and are not used)
                float4 t4[8], n4[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t4[j] = *reinterpret_cast<const float4*>(tr + 4 * j);
                int k = 0;
                for (; k + 32 <= kn; k += 32) {
                    const int kn4 = k + 32 < kSlabK ? k + 32 : k;
#pragma unroll
                    for (int j = 0; j < 8; ++j) n4[j] = *reinterpret_cast<const float4*>(tr + kn4 + 4 * j);
#pragma unroll
                    for (int j = 0; j < 8; ++j) { acc32 += t4[j].x; acc32 += t4[j].y; acc32 += t4[j].z; acc32 += t4[j].w; }
#pragma unroll
                    for (int j = 0; j < 8; ++j) t4[j] = n4[j];
                }
                for (; k < kn; ++k) acc32 += tr[k];
            }
            __syncthreads();
        }
        if ((int)threadIdx.x < ne) {
            const unsigned int e = list[base + threadIdx.x];
            const int ml = (int)(e >> 16), nl = (int)(e & 0xFFFFu);
            const int n = n_block + nl;
            const float s1 = scale ? scale[n] : 1.0f, b1 = bias ? bias[n] : 0.0f;
            if (sign_bit(affine(s1, acc32, b1))) atomicOr(&tile[ml * tw + (nl >> 5)], 1u << (nl & 31));
        }
    }
    __syncthreads();

    // ---- write the tile: each frame's words are contiguous in memory
    const int words_here = min(tw, yw32 - (n_block >> 5));           // words of this block that exist in a row of Y
    const int words_filled = ((nb + 63) >> 6) << 1;                   // words some wave has filled
    for (int i = threadIdx.x; i < kRealxBM * tw; i += kSlabThreads) {
        const int ml = i / tw, wi = i - ml * tw;
        const int m = m_base + ml;
        if (m < M && wi < words_here && wi < words_filled) Y[(size_t)m * yw32 + (n_block >> 5) + wi] = tile[i];
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Real input x binary weights with fp32 outputs that feed the log-Softmax (the output layer of a network with real
// hidden activations), on the int8 matrix cores: the same digit-plane product with FOUR 7-bit digits, |xq| <= 2^27.
// The integer sum a = sum +-xq is exact, and x differs from xq 2^-s by at most half a unit, so
//     | sum +-x  -  a 2^-s |  <=  K / 2 * 2^-s  <  K 2^-27 max|x|
// (4e-6 max|x| at K = 2048): below what the order of an fp32 summation changes (the sum in ascending k, the fp32
// matrix-core kernel and this one agree within a few 1e-6 of the sum's scale), and only used where nothing but the
// log-Softmax follows.  Frames with NaN, Inf or values too large to quantise take the fp32 sum in ascending k.
//   realx_quantize4_kernel   one wave per frame -> planes [4][M][kpad] + RowMeta4
//   realx_i8_linear_kernel   16 frames x 512 outputs per workgroup, K in slabs of 512 through LDS, z = fma(scale, sum, bias)
constexpr int kDigits4 = 4;
constexpr int kQuantBits4 = 27;
struct RowMeta4 {
    long long R;       // sum_k xq[k]
    float inv_scale;   // 2^-s
    int flags;         // 1: the row holds NaN/Inf or values too large to quantise
};
__host__ __device__ constexpr size_t slab4_planes_bytes() { return (size_t)2 * kDigits4 * kRealxBM * kSlabPlaneRow; }
__host__ __device__ constexpr size_t slab4_dynamic_lds() { return slab4_planes_bytes() + slab_weights_bytes(); }

// Grid: ceil(M / 4) workgroups of 256 threads.
__global__ __launch_bounds__(256) void realx_quantize4_kernel(const float* __restrict__ X, int M, int K, int kpad,
                                                              int8_t* __restrict__ planes, RowMeta4* __restrict__ meta) {
    const int m = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (m >= M) return;   // wave-uniform
    const int lane = lane_id();
    const float* x = X + (size_t)m * K;
    unsigned int mx = 0;
    for (int k0 = 0; k0 < K; k0 += 256) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = k0 + 64 * b + lane;
            if (k < K) mx = max(mx, __float_as_uint(x[k]) & 0x7fffffffu);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned int)__shfl_xor((int)mx, off, kWave));
    const int e = (int)(mx >> 23) - 127;
    const int flags = (mx >= 0x7f800000u || e >= 90) ? 1 : 0;
    int s = kQuantBits4 - 1 - e;                          // max|x| < 2^(e+1)  =>  |x| 2^s < 2^27
    s = s > 100 ? 100 : s;
    const float qs = __uint_as_float((unsigned int)(s + 127) << 23);
    const size_t plane = (size_t)M * kpad;
    int8_t* row = planes + (size_t)m * kpad;
    __shared__ __attribute__((aligned(16))) int8_t qstage[4][kDigits4][256];
    int8_t (*qs4)[256] = qstage[threadIdx.x >> 6];
    const int pos = permuted_byte_of_k(lane);
    long long R = 0;
    for (int k0 = 0; k0 < kpad; k0 += 256) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int kb = k0 + 64 * b;
            if (kb < kpad) {   // wave-uniform
                const int k = kb + lane;
                const float v = k < K ? x[k] : 0.0f;
                const int xq = flags ? 0 : (int)__builtin_rintf(v * qs);
                R += xq;
                qs4[0][64 * b + pos] = (int8_t)(xq & 127);
                qs4[1][64 * b + pos] = (int8_t)((xq >> kDigitBits) & 127);
                qs4[2][64 * b + pos] = (int8_t)((xq >> (2 * kDigitBits)) & 127);
                qs4[3][64 * b + pos] = (int8_t)(xq >> (3 * kDigitBits));
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        const int kd = k0 + 4 * lane;
        if (kd < kpad) {
#pragma unroll
            for (int d = 0; d < kDigits4; ++d)
                *reinterpret_cast<int*>(row + d * plane + kd) = *reinterpret_cast<const int*>(&qs4[d][4 * lane]);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) R += __shfl_xor(R, off, kWave);
    if (lane == 0) {
        RowMeta4 rm;
        rm.R = R;
        rm.inv_scale = __uint_as_float((unsigned int)(127 - s) << 23);
        rm.flags = flags;
        meta[m] = rm;
    }
}

// Grid: x = ceil(M / 16), y = ceil(N / 512); block = 512 threads; dynamic LDS = slab4_dynamic_lds().
// Z: fp32 [M][N], z = fma(scale, sum, bias) (the log-Softmax row kernel follows).
template <bool VEC16>
__global__ __launch_bounds__(kSlabThreads) void realx_i8_linear_kernel(const float* __restrict__ X, const int8_t* __restrict__ planes,
                                                                      const RowMeta4* __restrict__ meta, const uint32_t* __restrict__ Wp,
                                                                      const float* __restrict__ scale, const float* __restrict__ bias,
                                                                      int M, int K, int kpad, int N, int w32, float* __restrict__ Z) {
    constexpr int WN = 4;
    extern __shared__ __attribute__((aligned(16))) int8_t lds_raw[];
    __shared__ RowMeta4 meta_s[kRealxBM];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int r = lane & 15, g = lane >> 4;
    const int m_base = (int)blockIdx.x * kRealxBM;
    const int n_block = (int)blockIdx.y * kSlabNB;
    const int nb = min(kSlabNB, N - n_block);
    int8_t* pl = lds_raw;                                                                 // [2][4][16][kSlabPlaneRow]
    uint32_t* wst = reinterpret_cast<uint32_t*>(lds_raw + slab4_planes_bytes());           // [2][512][kSlabWRow]
    constexpr int pl_buf = kDigits4 * kRealxBM * kSlabPlaneRow;
    constexpr int w_buf = kSlabNB * kSlabWRow;
    if (threadIdx.x < kRealxBM) {
        const int m = m_base + (int)threadIdx.x;
        meta_s[threadIdx.x] = meta[m < M ? m : M - 1];
    }
    const int nsl = (kpad + kSlabK - 1) / kSlabK;
    const size_t plane = (size_t)M * kpad;

    uint4 preg[4], wreg[4];
    auto fetch_slab = [&](int sl) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;        // 0 .. 2047
            const int rowi = p >> 5, c16 = p & 31;                    // (digit, frame) row 0 .. 63, 16-byte column
            const int d = rowi >> 4, f = rowi & 15;
            const int m = m_base + f;
            const int k = sl * kSlabK + c16 * 16;
            preg[i] = make_uint4(0u, 0u, 0u, 0u);
            if (k < kpad) preg[i] = *reinterpret_cast<const uint4*>(planes + d * plane + (size_t)(m < M ? m : M - 1) * kpad + k);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;
            const int rowi = p >> 2, q = p & 3;
            const int wi = sl * 16 + q * 4;
            const uint32_t* src = Wp + (size_t)(n_block + (rowi < nb ? rowi : nb - 1)) * w32;
            wreg[i] = make_uint4(0u, 0u, 0u, 0u);
            if (VEC16 && wi + 3 < w32) {
                wreg[i] = *reinterpret_cast<const uint4*>(src + wi);
            } else {
                if (wi + 0 < w32) wreg[i].x = src[wi + 0];
                if (wi + 1 < w32) wreg[i].y = src[wi + 1];
                if (wi + 2 < w32) wreg[i].z = src[wi + 2];
                if (wi + 3 < w32) wreg[i].w = src[wi + 3];
            }
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;
            const int rowi = p >> 5, c16 = p & 31;
            *reinterpret_cast<uint4*>(pl + buf * pl_buf + rowi * kSlabPlaneRow + c16 * 16) = preg[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = (int)threadIdx.x + i * kSlabThreads;
            const int rowi = p >> 2, q = p & 3;
            uint32_t* dst = wst + buf * w_buf + rowi * kSlabWRow + q * 4;
            dst[0] = wreg[i].x; dst[1] = wreg[i].y; dst[2] = wreg[i].z; dst[3] = wreg[i].w;
        }
    };
    fetch_slab(0);
    store_slab(0);
    __syncthreads();

    const int nw = wave * (WN * 16);
    const int sh = 4 * (g & 1);
    v4i32 acc[kDigits4][WN];
#pragma unroll
    for (int d = 0; d < kDigits4; ++d)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[d][j] = v4i32{0, 0, 0, 0};
    for (int sl = 0; sl < nsl; ++sl) {
        const int buf = sl & 1;
        const bool more = sl + 1 < nsl;
        if (more) fetch_slab(sl + 1);
        __builtin_amdgcn_sched_barrier(0);
        if (nw < nb) {   // wave-uniform
            const int8_t* al = pl + buf * pl_buf + r * kSlabPlaneRow + 16 * g;
            const uint32_t* bl = wst + buf * w_buf + (nw + r) * kSlabWRow + (g >> 1);
            const int steps = min(kSlabK, kpad - sl * kSlabK) >> 6;
            for (int st = 0; st < steps; ++st) {
                v4i32 bx[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f) {
                    const uint32_t ws = bl[f * 16 * kSlabWRow + 2 * st] >> sh;
                    bx[f][0] = (int)(ws & 0x01010101u);
                    bx[f][1] = (int)((ws >> 1) & 0x01010101u);
                    bx[f][2] = (int)((ws >> 2) & 0x01010101u);
                    bx[f][3] = (int)((ws >> 3) & 0x01010101u);
                }
#pragma unroll
                for (int d = 0; d < kDigits4; ++d) {
                    const v4i32 ax = *reinterpret_cast<const v4i32*>(al + d * kRealxBM * kSlabPlaneRow + st * 64);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[d][fn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ax, bx[fn], acc[d][fn], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) store_slab(buf ^ 1);
        __syncthreads();
    }

    // accumulator register q of lane (r, g), fragment fn: frame 4 g + q of the tile, output nw + 16 fn + r of the block
    if (nw < nb) {   // wave-uniform
#pragma unroll
        for (int fn = 0; fn < WN; ++fn) {
            const int nl = nw + fn * 16 + r;
            const int n = n_block + nl;
            const float sc1 = (nl < nb && scale) ? scale[n] : 1.0f, bi1 = (nl < nb && bias) ? bias[n] : 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ml = 4 * g + q, m = m_base + ml;
                const RowMeta4 rm = meta_s[ml];
                // P = sum_k b_k xq_k from its four digit sums (each below 2^18), a = 2 P - R: 64-bit integers, then one rounding
                const long long P = ((((long long)acc[3][fn][q] * 128 + acc[2][fn][q]) * 128 + acc[1][fn][q]) * 128) + acc[0][fn][q];
                float a = (float)(double)(2 * P - rm.R) * rm.inv_scale;
                if (m < M && nl < nb) {
                    if (rm.flags) a = canonical_acc_global(X + (size_t)m * K, Wp + (size_t)n * w32, K);   // rare: NaN, Inf, huge values
                    Z[(size_t)m * N + n] = affine(sc1, a, bi1);
                }
            }
        }
    }
}

}  // namespace bnn
