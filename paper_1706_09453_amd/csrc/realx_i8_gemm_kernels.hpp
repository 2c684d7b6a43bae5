// Real input x binary weights on the int8 matrix cores for batches of 128 frames or more (paper Alg. 1 forward; Alg. 2:
// Sign at a hidden layer, Softmax at l = L): the digit-plane product of realx_slab_kernels.hpp as a tiled matrix
// product with V_MFMA_I32_32X32X32_I8, workgroups of 128 frames x 256 outputs instead of 16 x 512, so that a weight
// byte fetched into LDS serves 128 frames.
//
// What is computed is the filter described in realx_fused_kernel.hpp and realx_slab_kernels.hpp: every frame is scaled by
// a power of two and rounded to integers xq, P = sum_k b_k xq_k is exact (b = the weight bit), a = 2 P - sum_k xq_k.
//   Sign layers (three 7-bit digits, |xq| <= 2^qb, qb = 29 - ceil(log2 K) at most 20): an output whose interval
//     [a - E, a + E] lies on one side of the threshold is decided; the others are listed in global memory, frame by
//     frame, and resolved by the fp32 sum in ascending k (realx_resolve_rows_kernel), so every bit is the bit of that sum.
//   Log-Softmax layers (four digits, |xq| <= 2^27): z = fma(scale, a 2^-s, bias), |a 2^-s - sum +-x| < K 2^-27 max|x|.
//
// Digits.  xq = d0 + 128 d1 + 16384 d2 (+ 2097152 d3) with d0, d1 (, d2) in 0..127 and the top digit signed.  Two
// digits share an accumulator: the odd digits are stored NEGATED and multiplied with -128 b (b << 7 as a byte), so
//     acc_lo = sum_k b (d0 + 128 d1),    acc_hi = sum_k b d2   or   sum_k b (d2 + 128 d3),    P = acc_lo + 16384 acc_hi,
// all exact in int32 (K <= 8192: below 2^27 each).  A fragment of b is read once from LDS and shifted in registers.
//
// Layout.  Planes [digit][frame][kpad] and weight bytes [output][kpad] (0 or 1), both in natural k order, kpad = K
// rounded up to 64, zeros past K.  The product kernel is the pipeline of realw_split_kernels.hpp (steps of 64 k = 64
// bytes of a row, two LDS buffers, loads of step j + 2 in flight, one barrier per step, memory instructions between
// MFMAs): 2 x 2 waves of 64 frames x 128 outputs each, 2 x 4 accumulator fragments of 32 x 32, twice.
#pragma once

#include <utility>

#include "realx_slab_kernels.hpp"

namespace bnn {

typedef int v16i32g __attribute__((ext_vector_type(16)));
typedef int v4i32g __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4g __attribute__((ext_vector_type(4)));

constexpr int kI8KStep = 64;                       // k per pipeline step
constexpr int kI8TileM = 128, kI8TileN = 256;      // workgroup tile
constexpr int kI8RowBytes = 64;
constexpr int kI8Threads = 256;
constexpr int kI8StageB = kI8TileN * kI8RowBytes;  // 16384
__host__ __device__ constexpr int i8_stage_a(int digits) { return digits * kI8TileM * kI8RowBytes; }
__host__ __device__ constexpr int i8_stage(int digits) { return i8_stage_a(digits) + kI8StageB; }             // 40960 / 49152
__host__ __device__ constexpr unsigned i8_gemm_lds(int digits) { return 2u * (unsigned)i8_stage(digits); }    // 81920 / 98304
__host__ __device__ inline int i8_kpad(int K) { return (K + kI8KStep - 1) / kI8KStep * kI8KStep; }

// The outputs the filter could not decide, per frame and tile of 256 outputs: a record of 32 bytes, byte 0 = how many
// (at most 31), then the outputs' positions in the tile.  Records: [frame][tile], written whole by the one workgroup
// that owns frame and tile (no atomics in global memory, nothing to clear beforehand).
constexpr int kUndecidedRecord = 32;
constexpr int kUndecidedMax = kUndecidedRecord - 1;

// B[n][k] = bit k of weight row n as a byte (0 past K).  One thread per 16 k.  Grid: any number of blocks of 256.
__global__ __launch_bounds__(256) void bits_to_bytes_kernel(const uint32_t* __restrict__ Wp, int64_t N, int K, int w32, int kpad,
                                                            int8_t* __restrict__ B) {
    const int per_row = kpad >> 4;
    const int64_t total = N * per_row;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t n = i / per_row;
        const int k0 = (int)(i - n * per_row) * 16;
        uint32_t bits = 0;
        if (k0 < K) bits = (Wp[(size_t)n * w32 + (k0 >> 5)] >> (k0 & 31)) & 0xFFFFu;
        if (K - k0 < 16 && K > k0) bits &= (1u << (K - k0)) - 1u;
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t nib = (bits >> (4 * j)) & 0xFu;
            w[j] = (nib & 1u) | ((nib & 2u) << 7) | ((nib & 4u) << 14) | ((nib & 8u) << 21);
        }
        *reinterpret_cast<uint4*>(B + (size_t)n * kpad + k0) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// One wave per frame: scale, digits (odd digits negated), RowMeta (D = 3) or RowMeta4 (D = 4).  planes: [D][M][kpad].
// The frame is read twice (largest element, then digits), four consecutive elements per lane.  VEC: K % 4 == 0 and X
// 16-byte aligned.  Grid: ceil(M / 4) workgroups of 256 threads.
template <int D, bool VEC>
__global__ __launch_bounds__(256) void realx_quantize_nat_kernel(const float* __restrict__ X, int M, int K, int kpad, int qbits,
                                                                 int8_t* __restrict__ planes, void* __restrict__ meta_out) {
    static_assert(D == 3 || D == 4, "three digits for Sign layers, four in front of the log-Softmax");
    const int m = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (m >= M) return;   // wave-uniform
    const int lane = lane_id();
    const float* x = X + (size_t)m * K;
    auto load4 = [&](int k, float (&v)[4]) {
        if (VEC && k + 3 < K) {
            const float4 q = *reinterpret_cast<const float4*>(x + k);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = (k + t < K) ? x[k + t] : 0.0f;
        }
    };
    unsigned int mx = 0;   // largest |x| of the row as a bit pattern (NaN/Inf have the largest patterns)
    for (int k0 = 0; k0 < K; k0 += 256) {
        float v[4];
        load4(k0 + 4 * lane, v);
#pragma unroll
        for (int t = 0; t < 4; ++t) mx = max(mx, __float_as_uint(v[t]) & 0x7fffffffu);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = max(mx, (unsigned int)__shfl_xor((int)mx, off, kWave));
    const int e = (int)(mx >> 23) - 127;                 // floor(log2 max|x|) for normal numbers
    const int flags = (mx >= 0x7f800000u || e >= (D == 3 ? 100 : 90)) ? 1 : 0;
    int s = qbits - 1 - e;                                // max|x| < 2^(e+1)  =>  |x| 2^s < 2^qbits
    s = s > 100 ? 100 : s;
    const float qs = __uint_as_float((unsigned int)(s + 127) << 23);
    const size_t plane = (size_t)M * kpad;
    int8_t* row = planes + (size_t)m * kpad;
    long long R = 0, A = 0;
    for (int k0 = 0; k0 < kpad; k0 += 256) {
        const int k = k0 + 4 * lane;
        if (k < kpad) {   // kpad is a multiple of 64: the lane's four elements are inside or outside together
            float v[4];
            load4(k, v);
            uint32_t w[D] = {};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int xq = flags ? 0 : (int)__builtin_rintf(v[t] * qs);   // elements past K hold 0
                R += xq;
                A += xq < 0 ? -xq : xq;
                const int d0 = xq & 127, d1 = (xq >> 7) & 127;
                w[0] |= (uint32_t)d0 << (8 * t);
                w[1] |= ((uint32_t)(-d1) & 0xFFu) << (8 * t);
                if constexpr (D == 3) {
                    w[2] |= ((uint32_t)(xq >> 14) & 0xFFu) << (8 * t);
                } else {
                    const int d2 = (xq >> 14) & 127, d3 = xq >> 21;
                    w[2] |= (uint32_t)d2 << (8 * t);
                    w[3] |= ((uint32_t)(-d3) & 0xFFu) << (8 * t);
                }
            }
#pragma unroll
            for (int d = 0; d < D; ++d) *reinterpret_cast<uint32_t*>(row + d * plane + k) = w[d];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        R += __shfl_xor(R, off, kWave);
        A += __shfl_xor(A, off, kWave);
    }
    if (lane == 0) {
        const float inv = __uint_as_float((unsigned int)(127 - s) << 23);
        if constexpr (D == 3) {
            const float u = 5.9604644775390625e-08f;                            // 2^-24; all terms in units of 2^-s
            const float Kf = (float)K;
            const float sum_abs = (float)A * 1.0000002f + 0.5f * Kf;            // >= sum |x| 2^s ((float)A rounds: one ulp added)
            const float e_seq = (Kf - 1.0f) * u / (1.0f - Kf * u) * sum_abs;    // recursive fp32 summation
            const float e_quant = 0.5f * Kf;                                     // |x 2^s - xq| <= 1/2 each
            const float e_conv = u * (float)A * 1.0000002f;                      // (float)a
            RowMeta rm;
            rm.R = (int)R; rm.inv_scale = inv; rm.flags = flags;
            rm.E = flags ? __builtin_inff() : (e_seq + e_quant + e_conv) * 1.01f * inv;   // infinite bound: every output uncertain
            static_cast<RowMeta*>(meta_out)[m] = rm;
        } else {
            RowMeta4 rm;
            rm.R = R; rm.inv_scale = inv; rm.flags = flags;
            static_cast<RowMeta4*>(meta_out)[m] = rm;
        }
    }
}

// The product kernel.  D = 3: Sign bits into Yv (uint32 words [M][yw32]; bits of listed outputs are left 0) and the
// records of undecided outputs into `undecided` ([M][gridDim.y] records); D = 4: z = fma(scale, a 2^-s, bias) into Yv
// (fp32 [M][N]), `undecided` unused.
// planes [D][M][kpad], Bb [N][kpad], both 16-byte aligned, kpad % 64 == 0; meta: RowMeta (D = 3) or RowMeta4 (D = 4) [M].
// X, Wp: the layer's own operands, for the fp32 sum in ascending k of outputs that do not fit a record (D = 3) or of
// frames that could not be quantised (D = 4).  Grid: x = ceil(M / 128), y = ceil(N / 256); block = 256 threads;
// dynamic LDS i8_gemm_lds(D).
template <int D>
__global__ __launch_bounds__(kI8Threads) __attribute__((amdgpu_waves_per_eu(1, 1))) void realx_i8_gemm_kernel(
    const int8_t* __restrict__ planes, const int8_t* __restrict__ Bb, const void* __restrict__ meta_in, const float* __restrict__ X,
    const uint32_t* __restrict__ Wp, const float* __restrict__ scale, const float* __restrict__ bias, int M, int K, int kpad, int N,
    int w32, void* __restrict__ Yv, int yw32, unsigned char* __restrict__ undecided) {
    static_assert(D == 3 || D == 4, "three digits for Sign layers, four in front of the log-Softmax");
    extern __shared__ __attribute__((aligned(16))) unsigned char i8_lds[];
    constexpr int WM = 2, WN = 4;
    constexpr int LR = kI8Threads / 4;                       // rows one load instruction of the workgroup covers: 64
    constexpr int AL = kI8TileM / LR, BL = kI8TileN / LR;     // 2, 4
    constexpr int NL = D * AL + BL;                           // loads per thread and step: 10 / 12
    constexpr int NR = D * WM + WN;                           // fragment reads per wave and block: 10 / 12
    constexpr int NM = D * WM * WN;                           // MFMAs per wave and block: 24 / 32
    constexpr int kStageA = i8_stage_a(D), kStage = i8_stage(D);
    const int tid = (int)threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = lane_id();
    const int r = lane & 31, g = lane >> 5;
    const int m_tile = (int)blockIdx.x * kI8TileM, n_tile = (int)blockIdx.y * kI8TileN;
    const int m_base = m_tile + (wave >> 1) * (WM * 32);
    const int n_base = n_tile + (wave & 1) * (WN * 32);

    // ---- the thread's share of a step's loads: row (tid / 4) + 64 j, slot tid % 4
    const int lrow = tid >> 2, lslot = tid & 3;
    const int8_t* srcA[AL];
    const int8_t* srcB[BL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const int m = m_tile + lrow + LR * j;
        srcA[j] = planes + (size_t)(m < M ? m : M - 1) * kpad + lslot * 16;
    }
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int n = n_tile + lrow + LR * j;
        srcB[j] = Bb + (size_t)(n < N ? n : N - 1) * kpad + lslot * 16;
    }
    const size_t planeA = (size_t)M * kpad;
    const int st_off = lrow * kI8RowBytes + ((lslot ^ ((lrow >> 2) & 3)) << 4);
    // load i: digit i / AL, frames row block i % AL for i < D AL; then weights row block i - D AL
    struct Loads { u32x4 v[NL]; };
    auto gload_one = [&](Loads& L, int step, int i) {
        const int off = step * kI8KStep;
        if (i < D * AL) L.v[i] = *reinterpret_cast<const u32x4*>(srcA[i < D * AL ? i % AL : 0] + (i / AL) * planeA + off);
        else L.v[i] = *reinterpret_cast<const u32x4*>(srcB[i < D * AL ? 0 : i - D * AL] + off);
    };
    auto lstore_one = [&](unsigned char* stage, const Loads& L, int i) {
        if (i < D * AL)
            *reinterpret_cast<u32x4*>(stage + (i / AL) * (kI8TileM * kI8RowBytes) + (i % AL) * (LR * kI8RowBytes) + st_off) = L.v[i];
        else
            *reinterpret_cast<u32x4*>(stage + kStageA + (i - D * AL) * (LR * kI8RowBytes) + st_off) = L.v[i];
    };

    // ---- the wave's operand fragments of block h (0 or 1) of a stage: digit fragments, then weight fragments
    struct Frags { v4i32g a[D][WM]; v4i32g b[WN]; };
    const int swz = (r >> 2) & 3;
    const int a_off = ((wave >> 1) * (WM * 32) + r) * kI8RowBytes;
    const int b_off = kStageA + ((wave & 1) * (WN * 32) + r) * kI8RowBytes;
    auto lread_one = [&](Frags& F, const unsigned char* stage, int h, int i) {
        const int so = ((2 * h + g) ^ swz) << 4;
        if (i < D * WM)
            F.a[i < D * WM ? i / WM : 0][i % WM] =
                *reinterpret_cast<const v4i32g*>(stage + (i / WM) * (kI8TileM * kI8RowBytes) + a_off + (i % WM) * (32 * kI8RowBytes) + so);
        else
            F.b[i < D * WM ? 0 : i - D * WM] = *reinterpret_cast<const v4i32g*>(stage + b_off + (i - D * WM) * (32 * kI8RowBytes) + so);
    };

    v16i32g acc[2][WM][WN];   // [0]: digits 0 and 1, [1]: digits 2 (and 3)
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[p][i][j][v] = 0;

    auto products = [&](const Frags& F) {
        v4i32g bneg[WN];   // -128 b: the byte 1 becomes 0x80
#pragma unroll
        for (int fn = 0; fn < WN; ++fn) bneg[fn] = F.b[fn] << 7;
#pragma unroll
        for (int d = 0; d < D; ++d)
#pragma unroll
            for (int fm = 0; fm < WM; ++fm)
#pragma unroll
                for (int fn = 0; fn < WN; ++fn)
                    acc[d >> 1][fm][fn] =
                        __builtin_amdgcn_mfma_i32_32x32x32_i8(F.a[d][fm], (d & 1) ? bneg[fn] : F.b[fn], acc[d >> 1][fm][fn], 0, 0, 0);
    };

    // One half of a step (the pipeline and the issue pattern of realw_bf16x3_kernel): after every fragment read one load
    // or one LDS write, alternately, while there are any, then one MFMA; the rest of the MFMAs at the end.
    constexpr int G1 = (NL + 1) / 2, G2 = NL - G1;
    static_assert(NL <= NR, "one load or write per fragment read");
    auto half = [&](int hf, const Frags& now, Frags& next, const unsigned char* rd, int rd_h, unsigned char* wr, Loads& L, int sl) {
        const int g0 = hf ? G1 : 0, ng = hf ? G2 : G1, w0 = hf ? 0 : G1, nw = hf ? G1 : G2;
        const int mn = ng < nw ? ng : nw;
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            lread_one(next, rd, rd_h, i);
            const int e = i - 2 * mn;
            if (i < 2 * mn) {
                if ((i & 1) == 0) gload_one(L, sl, g0 + i / 2);
                else lstore_one(wr, L, w0 + i / 2);
            } else {
                if (ng > nw && e < ng - mn) gload_one(L, sl, g0 + mn + e);
                if (nw > ng && e < nw - mn) lstore_one(wr, L, w0 + mn + e);
            }
        }
        products(now);
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
            const int e = i - 2 * mn;
            if (i < 2 * mn) {
                if ((i & 1) == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // load from memory
                else __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);              // LDS write
            } else {
                if (ng > nw && e < ng - mn) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (nw > ng && e < nw - mn) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NM - NR, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int nS = kpad / kI8KStep;
    unsigned char* buf0 = i8_lds;
    unsigned char* buf1 = i8_lds + kStage;
    Loads L;
    Frags F0, F1;
#pragma unroll
    for (int i = 0; i < NL; ++i) gload_one(L, 0, i);
#pragma unroll
    for (int i = 0; i < NL; ++i) lstore_one(buf0, L, i);
#pragma unroll
    for (int i = 0; i < NL; ++i) gload_one(L, nS > 1 ? 1 : 0, i);
#pragma unroll
    for (int i = 0; i < G1; ++i) lstore_one(buf1, L, i);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NR; ++i) lread_one(F0, buf0, 0, i);
    for (int j = 0; j < nS; ++j) {
        unsigned char* cur = (j & 1) ? buf1 : buf0;
        unsigned char* nxt = (j & 1) ? buf0 : buf1;
        const int sl = j + 2 < nS ? j + 2 : nS - 1;   // past the end: the last step again (in bounds, never used)
        half(0, F0, F1, cur, 1, nxt, L, sl);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        half(1, F1, F0, nxt, 0, cur, L, sl);
    }
    __syncthreads();   // the buffers are free: the epilogue reuses them

    // ---- epilogue.  Accumulator fragment (fm, fn), register v of lane (r, g) belongs to frame
    //      m_base + 32 fm + 8 (v/4) + 4 g + v%4 and output n_base + 32 fn + r.
    if constexpr (D == 3) {
        const RowMeta* meta = static_cast<const RowMeta*>(meta_in);
        uint32_t* Y = static_cast<uint32_t*>(Yv);
        // A lane decides its 16 frames of a fragment on its own and keeps the answers as bit masks (bit v: frame v of
        // the fragment): no ballots, no scalar logic, no branch per sum.  The masks of all lanes go to LDS,
        // colmask[frame block of 32][g][output of the tile], and are turned into output words afterwards.
        // LDS: column masks 4 x 2 x 256 x 2 bytes | the frames' quantisation records | per frame: how many undecided
        // outputs | per frame: their records (about one output per frame is expected at K = 2048).
        uint16_t* colmask = reinterpret_cast<uint16_t*>(i8_lds);
        constexpr int kMaskBytes = 4 * 2 * kI8TileN * 2;
        RowMeta* meta_s = reinterpret_cast<RowMeta*>(i8_lds + kMaskBytes);
        unsigned int* und_count = reinterpret_cast<unsigned int*>(i8_lds + kMaskBytes + kI8TileM * sizeof(RowMeta));
        unsigned char* und = reinterpret_cast<unsigned char*>(und_count + kI8TileM);   // [frame][kUndecidedRecord]
        static_assert((kMaskBytes + kI8TileM * sizeof(RowMeta)) % 16 == 0 &&
                          kMaskBytes + kI8TileM * (sizeof(RowMeta) + 4 + kUndecidedRecord) <= i8_gemm_lds(3),
                      "epilogue LDS");
        if (tid < kI8TileM) {
            const int m = m_tile + tid;
            meta_s[tid] = meta[m < M ? m : M - 1];
            und_count[tid] = 0u;
        }
        __syncthreads();
        float sc[WN], bi[WN], asc[WN];
        bool nvalid[WN];
#pragma unroll
        for (int fn = 0; fn < WN; ++fn) {
            const int n = n_base + fn * 32 + r;
            nvalid[fn] = n < N;
            sc[fn] = nvalid[fn] ? (scale ? scale[n] : 1.0f) : 0.0f;
            bi[fn] = nvalid[fn] ? (bias ? bias[n] : 0.0f) : -1.0f;
            // |scale| (1 + 2^-16.6) covers the roundings of the margin; the floor covers a product that underflows
            asc[fn] = __builtin_fmaxf(__builtin_fabsf(sc[fn]) * 1.00001f, 1e-30f);
        }
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
            const int fb = (wave >> 1) * WM + fm;   // block of 32 frames of the tile
            uint32_t bits[WN], ubits[WN];
#pragma unroll
            for (int fn = 0; fn < WN; ++fn) bits[fn] = ubits[fn] = 0u;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int ml = fb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);   // frame in the tile
                const RowMeta rm = meta_s[ml];
                const bool mvalid = m_tile + ml < M;
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    // With t = fma(scale, a, bias): if |t| > |scale| E (1 + 2^-16.6) + 1e-30, then scale x + bias has the
                    // sign of t, and at least 1e-30 in magnitude, for every real x within E of a, so its rounding has that
                    // sign too and the bit of the fp32 sum is (t > 0).  Anything else (NaN included) is uncertain.
                    const int P = acc[0][fm][fn][v] + (acc[1][fm][fn][v] << (2 * kDigitBits));
                    const float a = (float)(int)(((unsigned int)P << 1) - (unsigned int)rm.R) * rm.inv_scale;
                    const float t = affine(sc[fn], a, bi[fn]);
                    const float margin = __builtin_fmaf(asc[fn], rm.E, 1e-30f);
                    const bool certain = __builtin_fabsf(t) > margin;
                    bits[fn] |= (certain && t > 0.0f) ? (1u << v) : 0u;
                    ubits[fn] |= (!certain && mvalid) ? (1u << v) : 0u;
                }
            }
#pragma unroll
            for (int fn = 0; fn < WN; ++fn) {
                const int nl = (wave & 1) * (WN * 32) + fn * 32 + r;   // output in the tile
                uint32_t ub = nvalid[fn] ? ubits[fn] : 0u;
                uint32_t bt = nvalid[fn] ? bits[fn] : 0u;              // outputs past the layer's end: bit 0
                while (ub) {   // rare: about one lane in twenty has one
                    const int v = __builtin_ctz(ub);
                    ub &= ub - 1u;
                    const int ml = fb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                    const unsigned int slot = atomicAdd(&und_count[ml], 1u);
                    if (slot < (unsigned int)kUndecidedMax) {
                        und[ml * kUndecidedRecord + 1 + (int)slot] = (unsigned char)nl;
                    } else {   // more than the frame's record holds: summed here
                        const int m = m_tile + ml, n = n_tile + nl;
                        if (sign_bit(affine(sc[fn], canonical_acc_global(X + (size_t)m * K, Wp + (size_t)n * w32, K), bi[fn]))) bt |= 1u << v;
                    }
                }
                colmask[(fb * 2 + g) * kI8TileN + nl] = (uint16_t)bt;
            }
        }
        __syncthreads();
        // Output words: thread (frame f = tid / 2, half = tid % 2) builds words 4 half .. + 3 of its frame; bit j of word c
        // is bit v(f) of the mask of output 32 c + j, where f = 32 fb + 8 (v / 4) + 4 g + v % 4.
        {
            const int f = tid >> 1, wq = (tid & 1) * 4;
            const int fb = f >> 5, fg = (f >> 2) & 1, fv = ((f >> 3) & 3) * 4 + (f & 3);
            const uint32_t* cm = reinterpret_cast<const uint32_t*>(colmask + (fb * 2 + fg) * kI8TileN);   // two masks per dword
            const int m = m_tile + f;
            const int w_first = (n_tile >> 5) + wq;
            uint32_t words[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint32_t w = 0u;
#pragma unroll
                for (int j2 = 0; j2 < 16; ++j2) {
                    const uint32_t two = cm[(wq + c) * 16 + j2] >> fv;   // outputs 32 (wq + c) + 2 j2 and + 1
                    w |= (two & 1u) << (2 * j2);
                    w |= ((two >> 16) & 1u) << (2 * j2 + 1);
                }
                words[c] = w;
            }
            if (m < M) {
                uint32_t* y = Y + (size_t)m * yw32 + w_first;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (w_first + c < yw32) y[c] = words[c];
            }
        }
        // the frames' records, 16 bytes per thread (the barrier above also ordered the entries written to them)
        {
            const int f = tid >> 1, h = tid & 1;
            const int m = m_tile + f;
            u32x4 rec = *reinterpret_cast<const u32x4*>(und + f * kUndecidedRecord + 16 * h);
            const unsigned int cnt = und_count[f] < (unsigned int)kUndecidedMax ? und_count[f] : (unsigned int)kUndecidedMax;
            if (h == 0) rec.x = (rec.x & ~0xFFu) | cnt;
            if (m < M)
                *reinterpret_cast<u32x4*>(undecided + ((size_t)m * gridDim.y + blockIdx.y) * kUndecidedRecord + 16 * h) = rec;
        }
    } else {
        const RowMeta4* meta = static_cast<const RowMeta4*>(meta_in);
        float* Z = static_cast<float*>(Yv);
        if (m_base >= M || n_base >= N) return;   // wave-uniform, after the last barrier
        // per wave 32 rows x 128 columns of outputs on their way to memory (a row is 512 contiguous bytes)
        constexpr int LDW = 32 * WN + 4;
        static_assert(4 * 32 * LDW * 4 <= (int)i8_gemm_lds(4), "epilogue LDS");
        float* stg = reinterpret_cast<float*>(i8_lds) + wave * (32 * LDW);
        float sc[WN], bi[WN];
#pragma unroll
        for (int fn = 0; fn < WN; ++fn) {
            const int n = n_base + fn * 32 + r;
            sc[fn] = (n < N && scale) ? scale[n] : 1.0f;
            bi[fn] = (n < N && bias) ? bias[n] : 0.0f;
        }
        const bool rows_vec = ((N & 3) == 0) && ((reinterpret_cast<uintptr_t>(Z) & 15) == 0);
        const int c4 = (lane & 31) * 4;
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rowl = 8 * (v >> 2) + 4 * g + (v & 3);
                const int m = m_base + fm * 32 + rowl;
                const RowMeta4 rm = meta[m < M ? m : M - 1];
#pragma unroll
                for (int fn = 0; fn < WN; ++fn) {
                    // P = sum_k b_k xq_k from its two accumulators, a = 2 P - R as a 64-bit integer (below 2^40), rounded
                    // once: its upper part (below 2^24) and its lower 16 bits are exact floats, and one fma adds them
                    const long long P = (long long)acc[0][fm][fn][v] + ((long long)acc[1][fm][fn][v] << (2 * kDigitBits));
                    const long long a64 = 2 * P - rm.R;
                    const int hi = (int)(a64 >> 16);
                    const int lo = (int)(a64 & 0xFFFF);
                    float a = __builtin_fmaf((float)hi, 65536.0f, (float)lo) * rm.inv_scale;
                    const int n = n_base + fn * 32 + r;
                    if (rm.flags && m < M && n < N)   // rare: NaN, Inf, huge values
                        a = canonical_acc_global(X + (size_t)m * K, Wp + (size_t)n * w32, K);
                    stg[rowl * LDW + fn * 32 + r] = affine(sc[fn], a, bi[fn]);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // this wave's LDS writes are done before it reads them back
            // two rows per pass: 32 lanes x 16 bytes each
#pragma unroll 4
            for (int it = 0; it < 16; ++it) {
                const int rowl = it * 2 + (lane >> 5);
                const int m = m_base + fm * 32 + rowl;
                const int n = n_base + c4;
                const float4 qv = *reinterpret_cast<const float4*>(stg + rowl * LDW + c4);
                if (m < M) {
                    float* y = Z + (size_t)m * N + n;
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
}

// The undecided outputs, exactly: the fp32 sum in ascending k, acc + (+-x) at every step, written as fma(+-1, x, acc)
// (the product with +-1 is exact, so it rounds as the addition does), then bit = Sign(fma(scale, sum, bias)) ORed into Y
// (the product kernel left these bits 0).
// A sum is a chain of K dependent operations, and an output's terms are its frame's values with the signs of its weight
// row, so the frames are what is worth sharing: a workgroup of 256 threads takes 16 frames, collects their undecided
// outputs from the records (about 130 at K = 2048, N = 2048) and gives each to a lane.  The frames go through LDS in
// slabs of 256 k, twice buffered (the next slab is on its way from memory while this one is added up, one barrier per
// slab); a lane reads its frame's values from there (lanes of one frame read the same address, the 16 frames lie in
// different banks), forms the signs from its own weight words (eight per slab, read one slab ahead) and adds.
// More than 256 outputs: further passes over the frames; more than kResolveCap: the lane that finds them sums them
// from global memory.  The last slab of a frame is padded with +0 and added up to the end of the block of 32 in which the
// frame ends.
// VEC: K % 4 == 0 and X 16-byte aligned.  Grid: ceil(M / 16) workgroups of 256 threads.
constexpr int kResolveFrames = 16;
constexpr int kResolveSlab = 256;
constexpr int kResolveLd = kResolveSlab + 4;   // floats per frame in a buffer: frame r starts at bank 4 r
constexpr int kResolveThreads = 256;
constexpr int kResolveCap = 1024;

// Term T of a slab and what stands around it (see the kernel); T = -16 .. -1 only start the stream.
// The factor +-1 of a term is a half-precision number: bits j and j + 16 of a weight word, moved to the sign bits of
// the two halves of a register over the bit pattern of (1.0, 1.0), serve terms j and j + 16 of the word's 32, and the
// mixed-precision fused multiply-add takes either half as its first factor (widened exactly; the operation itself is
// the fp32 one).  Two instructions per pair and one per term instead of three per term.
// Rings: a shifted word lives for four terms, a pair for twenty, an LDS read for twenty.
typedef _Float16 f16x2g __attribute__((ext_vector_type(2)));
// Returns false behind the last term of a block of 32 when the frame ends there or before (kn: terms of this slab).
template <int T>
__device__ __forceinline__ bool resolve_term(int kn, const float* xr, const uint32_t (&wc)[kResolveSlab / 32], uint32_t (&sh)[8], uint32_t (&pr)[16],
                                             f32x4g (&xv)[8], float& acc, uint32_t ones) {
    if constexpr (T + 16 < kResolveSlab && ((T + 16) & 3) == 0) xv[((T + 16) >> 2) & 7] = *reinterpret_cast<const f32x4g*>(xr + T + 16);
    if constexpr (T >= 0) {
        const f16x2g pm = __builtin_bit_cast(f16x2g, pr[T & 15]);
        acc = __builtin_fmaf((float)pm[(T >> 4) & 1], xv[(T >> 2) & 7][T & 3], acc);
    }
    if constexpr (T + 4 >= 0 && T + 4 < kResolveSlab && ((T + 4) & 31) < 16)   // one bit-field insert
        pr[(T + 4) & 15] = (sh[(T + 4) & 7] & 0x80008000u) | (ones & ~0x80008000u);
    if constexpr (T + 8 >= 0 && T + 8 < kResolveSlab && ((T + 8) & 31) < 16)
        sh[(T + 8) & 7] = ~wc[(T + 8) >> 5] << (15 - ((T + 8) & 31));   // weight bit 0: -x
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (T >= 0 && (T & 31) == 31 && T + 1 < kResolveSlab) return T + 1 < kn;   // wave-uniform
    return true;
}
template <int... I>
__device__ __forceinline__ void resolve_slab(int kn, const float* xr, const uint32_t (&wc)[kResolveSlab / 32], float& acc,
                                             std::integer_sequence<int, I...>) {
    uint32_t sh[8];
    uint32_t pr[16];
    f32x4g xv[8];
    uint32_t ones = 0x3C003C00u;   // (1.0, 1.0) in half precision, kept in a register as the insert's third operand
    asm volatile("" : "+v"(ones));
    (void)(resolve_term<I - 16>(kn, xr, wc, sh, pr, xv, acc, ones) && ...);
}

template <bool VEC>
__global__ __launch_bounds__(kResolveThreads) void realx_resolve_rows_kernel(const float* __restrict__ X, const uint32_t* __restrict__ Wp,
                                                                           const float* __restrict__ scale, const float* __restrict__ bias,
                                                                           int M, int K, int w32, const unsigned char* __restrict__ undecided,
                                                                           int tiles, uint32_t* __restrict__ Y, int yw32) {
    __shared__ __attribute__((aligned(16))) float xs[2][kResolveFrames][kResolveLd];
    __shared__ u32x4 ws[2][kResolveThreads][2];   // a lane's eight weight words of a slab
    __shared__ unsigned int ent[kResolveCap];   // (frame of the workgroup) << 28 | output
    __shared__ unsigned int total_s;
    const int tid = (int)threadIdx.x;
    const int m0 = (int)blockIdx.x * kResolveFrames;
    const int nsl = (K + kResolveSlab - 1) / kResolveSlab;
    // a slab is 16 frames x 64 pieces of four k: four pieces per thread
    constexpr int kPPR = kResolveSlab / 4, kPer = kResolveFrames * kPPR / kResolveThreads;
    struct Pieces { f32x4g x[kPer]; };   // native vectors: an array of them stays in registers
    auto request = [&](Pieces& P, int sl) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int p = tid + kResolveThreads * i;
            const int m = min(m0 + p / kPPR, M - 1);   // past the last frame: the last one again (unused)
            const int k = sl * kResolveSlab + 4 * (p % kPPR);
            const float* xr = X + (size_t)m * K;
            if (VEC) {   // past K: values of the frame's end (in bounds), replaced by deposit()
                P.x[i] = *reinterpret_cast<const f32x4g*>(xr + min(k, K - 4));
            } else {
                P.x[i] = f32x4g{xr[min(k, K - 1)], xr[min(k + 1, K - 1)], xr[min(k + 2, K - 1)], xr[min(k + 3, K - 1)]};
            }
        }
    };
    // past K: +0, which leaves a sum as it is with either sign in front (a sum that starts at +0 never becomes -0).
    // The first use of what was requested is here, after the slab in between has been added up.
    auto deposit = [&](const Pieces& P, int sl) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int p = tid + kResolveThreads * i;
            const int k = sl * kResolveSlab + 4 * (p % kPPR);
            f32x4g v = P.x[i];
            v.x = k < K ? v.x : 0.0f;
            v.y = k + 1 < K ? v.y : 0.0f;
            v.z = k + 2 < K ? v.z : 0.0f;
            v.w = k + 3 < K ? v.w : 0.0f;
            *reinterpret_cast<f32x4g*>(&xs[sl & 1][p / kPPR][4 * (p % kPPR)]) = v;
        }
    };
    Pieces P;
    request(P, 0);   // the frames' first slab is on its way while the records are read
    if (tid == 0) total_s = 0u;
    __syncthreads();
    for (int t = tid; t < kResolveFrames * tiles; t += kResolveThreads) {
        const int r = t / tiles, tile = t - r * tiles;
        const int m = m0 + r;
        if (m >= M) continue;
        const u32x4* rec = reinterpret_cast<const u32x4*>(undecided + ((size_t)m * tiles + tile) * kUndecidedRecord);
        const u32x4 lo = rec[0];
        const int cnt = min((int)(lo.x & 0xFFu), kUndecidedMax);
        if (cnt == 0) continue;
        const u32x4 hi = rec[1];
        const unsigned int base = atomicAdd(&total_s, (unsigned int)cnt);
        for (int i = 0; i < cnt; ++i) {
            const int b = i + 1;   // byte of the record
            const unsigned int word = b < 16 ? (b < 8 ? (b < 4 ? lo.x : lo.y) : (b < 12 ? lo.z : lo.w))
                                             : (b < 24 ? (b < 20 ? hi.x : hi.y) : (b < 28 ? hi.z : hi.w));
            const int n = tile * kI8TileN + (int)((word >> (8 * (b & 3))) & 0xFFu);
            if (base + i < (unsigned int)kResolveCap) {
                ent[base + i] = ((unsigned int)r << 28) | (unsigned int)n;
            } else {
                const float s1 = scale ? scale[n] : 1.0f, b1 = bias ? bias[n] : 0.0f;
                if (sign_bit(affine(s1, canonical_acc_global(X + (size_t)m * K, Wp + (size_t)n * w32, K), b1)))
                    atomicOr(&Y[(size_t)m * yw32 + (n >> 5)], 1u << (n & 31));
            }
        }
    }
    __syncthreads();
    const int total = (int)min(total_s, (unsigned int)kResolveCap);   // workgroup-uniform
    if (total == 0) return;
    for (int first = 0; first < total; first += kResolveThreads) {   // workgroup-uniform
        const bool active = first + tid < total;
        const unsigned int e = ent[active ? first + tid : 0];
        const int r = (int)(e >> 28), n = (int)(e & 0x0FFFFFFFu);
        const uint32_t* wrow = Wp + (size_t)n * w32;
        const int wlast = (K - 1) >> 5;
        constexpr int kWords = kResolveSlab / 32;
        static_assert(kWords == 8, "eight weight words per slab and lane");
        float acc32 = 0.0f;
        struct Words { u32x4 lo, hi; };
        auto words = [&](Words& w, int sl) {
            uint32_t v[kWords];
#pragma unroll
            for (int b = 0; b < kWords; ++b) v[b] = wrow[min(sl * kWords + b, wlast)];
            w.lo = u32x4{v[0], v[1], v[2], v[3]};
            w.hi = u32x4{v[4], v[5], v[6], v[7]};
        };
        // What comes from global memory (the frames' next slab, the lane's next eight weight words) is requested before
        // the slab is added up and goes to LDS after it: nothing in between waits for memory.
        Words W;
        __syncthreads();   // the previous pass no longer reads the buffers
        if (first > 0) request(P, 0);
        words(W, 0);
        deposit(P, 0);
        ws[0][tid][0] = W.lo;
        ws[0][tid][1] = W.hi;
        __syncthreads();
        for (int sl = 0; sl < nsl; ++sl) {
            if (sl + 1 < nsl) {   // workgroup-uniform
                request(P, sl + 1);
                words(W, sl + 1);
            }
            if (active) {
                // The slab's 256 terms as one stream (the last slab of a frame is padded with +0).  A result is ready some
                // clocks after its instruction, and a wave has nothing else to issue meanwhile, so no instruction reads
                // what one of the two before it wrote: around the addition of term t stand the mask of term t + 4, the
                // shift of term t + 8 and, every fourth term, the LDS read of terms t + 16 .. t + 19.
                const u32x4 lo = ws[sl & 1][tid][0], hi = ws[sl & 1][tid][1];
                const uint32_t wc[kWords] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                resolve_slab(K - sl * kResolveSlab, &xs[sl & 1][r][0], wc, acc32, std::make_integer_sequence<int, kResolveSlab + 16>{});
            }
            if (sl + 1 < nsl) {
                deposit(P, sl + 1);
                ws[(sl + 1) & 1][tid][0] = W.lo;
                ws[(sl + 1) & 1][tid][1] = W.hi;
            }
            __syncthreads();
        }
        if (active) {
            const int m = m0 + r;
            const float s1 = scale ? scale[n] : 1.0f, b1 = bias ? bias[n] : 0.0f;
            if (sign_bit(affine(s1, acc32, b1))) atomicOr(&Y[(size_t)m * yw32 + (n >> 5)], 1u << (n & 31));
        }
    }
}

}  // namespace bnn
