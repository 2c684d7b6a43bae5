// A layer with real-valued weights and real-valued inputs in front of the log-Softmax (paper Sec. 3.1: the Softmax
// layer keeps real weights; Sec. 4.3: sigmoid networks hand it real inputs) on the bf16 matrix cores,
// V_MFMA_F32_32X32X16_BF16, at fp32 accuracy.
//
// Every fp32 operand v is written as v = p0 + p1 + p2 + rest with three bf16 pieces: p0 = bf16(v), p1 = bf16(v - p0),
// p2 = bf16(v - p0 - p1), each rounded to nearest, each difference exact in fp32; |rest| <= 2^-24 |v| (a bf16 keeps
// 8 significant bits).  A product x w is taken as the six piece products whose weights are 2^-16 or more,
//     x0 w2 + x1 w1 + x2 w0 + x0 w1 + x1 w0 + x0 w0,
// every one exact in the matrix core's fp32 (8 x 8 significant bits) and added to an fp32 accumulator.  What is left
// out (x1 w2, x2 w1, x2 w2 and the two rests) is below 2^-22 |x w| per term, so the sum differs from the exact one by
// at most 2^-22 sum_k |x_k w_k| plus ordinary fp32 rounding of the accumulation, the same kind of difference the fp32
// matrix-core kernel has (its own rounding bound is K 2^-24 sum_k |x_k w_k|).  One V_MFMA_F32_32X32X16_BF16 does 16 k
// in 8 passes where V_MFMA_F32_32X32X2_F32 needs 8 instructions of 16 passes: six of them are 2.7 times cheaper.
// Layers whose outputs are Sign bits never use this kernel: bits are defined from the fp32 sum in ascending k.
//
// Two kernels: the split (one pass over each operand, pieces to planes [piece][row][kpad] of bf16 in the caller's
// workspace, kpad = K rounded up to 32, zeros past K), then the product kernel below.
#pragma once

#include "bnn_device.hpp"

namespace bnn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f32s __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSplitPieces = 3;
constexpr int kSplitKStep = 32;                                  // k per pipeline step: 64 bytes of a plane row
constexpr int kSplitTileM = 256, kSplitTileN = 128;              // workgroup tile: 2 x 2 waves of 128 x 64
constexpr int kSplitRowBytes = kSplitKStep * 2;
constexpr int kSplitStageA = kSplitPieces * kSplitTileM * kSplitRowBytes;   // 49152
constexpr int kSplitStageB = kSplitPieces * kSplitTileN * kSplitRowBytes;   // 24576
constexpr int kSplitStage = kSplitStageA + kSplitStageB;                    // 73728
constexpr unsigned split_dynamic_lds() { return 2u * kSplitStage; }         // 147456 of the CU's 163840 bytes

__host__ __device__ inline int split_kpad(int K) { return (K + kSplitKStep - 1) / kSplitKStep * kSplitKStep; }

// bf16 nearest to v (ties to even) as its 16 bits; a finite v that would round to infinity is truncated instead, so that
// the pieces of a finite value stay finite.
__device__ inline uint32_t bf16_bits(float v) {
    uint32_t h = (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)v);
    const uint32_t u = __float_as_uint(v);
    if ((h & 0x7fffu) == 0x7f80u && (u & 0x7f800000u) != 0x7f800000u) h = u >> 16;
    return h;
}

// The three pieces of v.  A non-finite v gives p0 = v and NaN further down, so every sum it enters ends up NaN or
// infinite, as the exact sum does before the log-Softmax turns the row into NaN.
__device__ inline void split3(float v, uint32_t& p0, uint32_t& p1, uint32_t& p2) {
    p0 = bf16_bits(v);
    const float r1 = v - __uint_as_float(p0 << 16);
    p1 = bf16_bits(r1);
    const float r2 = r1 - __uint_as_float(p1 << 16);
    p2 = bf16_bits(r2);
}

// planes[p][row][kpad] <- piece p of A[row][k] (zero for K <= k < kpad).  One thread per 8 consecutive k.
// VEC: K % 4 == 0 and A 16-byte aligned.  Grid: any number of blocks of 256 threads (grid-stride).
template <bool VEC>
__global__ __launch_bounds__(256) void split_bf16x3_kernel(const float* __restrict__ A, int64_t rows, int K, int kpad,
                                                            uint16_t* __restrict__ planes) {
    const int per_row = kpad >> 3;
    const int64_t total = rows * per_row;
    const size_t plane = (size_t)rows * (size_t)kpad;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / per_row;
        const int k0 = (int)(i - row * per_row) * 8;
        const float* a = A + (size_t)row * K;
        float v[8];
        if (VEC && k0 + 7 < K) {
            const float4 lo = *reinterpret_cast<const float4*>(a + k0);
            const float4 hi = *reinterpret_cast<const float4*>(a + k0 + 4);
            v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
            v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
        } else {
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = (k0 + t < K) ? a[k0 + t] : 0.0f;
        }
        uint32_t w[kSplitPieces][4];
#pragma unroll
        for (int t = 0; t < 8; t += 2) {
            uint32_t a0, a1, a2, b0, b1, b2;
            split3(v[t], a0, a1, a2);
            split3(v[t + 1], b0, b1, b2);
            w[0][t >> 1] = a0 | (b0 << 16);
            w[1][t >> 1] = a1 | (b1 << 16);
            w[2][t >> 1] = a2 | (b2 << 16);
        }
        const size_t at = (size_t)row * kpad + k0;
#pragma unroll
        for (int p = 0; p < kSplitPieces; ++p)
            *reinterpret_cast<uint4*>(planes + p * plane + at) = make_uint4(w[p][0], w[p][1], w[p][2], w[p][3]);
    }
}

// Y[m][n] = bias[n] + sum_k X[m][k] W[n][k] from the planes Xs [3][M][kpad] and Ws [3][N][kpad] (16-byte aligned,
// kpad % 32 == 0).  Grid: x = ceil(M / 256), y = ceil(N / 128); block = 64 NW threads; dynamic LDS split_dynamic_lds().
// NW = 4: 2 x 2 waves of 128 x 64, one wave per SIMD; NW = 8: 4 x 2 waves of 64 x 64, two waves per SIMD (each fills the
// other's waits).
//
// Pipeline, one step = 32 k = two MFMA blocks of 16: the workgroup's 384 rows x 3 pieces x 64 bytes of step j + 2 are
// loaded into registers (16 bytes per lane and load, four lanes per 64-byte row segment) while step j runs, and stored
// into the LDS buffer of step j once every wave has taken its last operands out of it (one barrier per step).  A wave
// reads its operand fragments out of LDS one block ahead of the MFMAs that use them.  In LDS a row's four 16-byte slots
// are stored at slot ^ ((row / 4) % 4), which spreads both the stores and the fragment reads of 16 lanes over all
// banks.  Lane (r = lane % 32, g = lane / 32) feeds row r, k = 8 g .. 8 g + 7 of a block to both operands.
template <int ACT, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void realw_bf16x3_kernel(
    const uint16_t* __restrict__ Xs, const uint16_t* __restrict__ Ws, const float* __restrict__ bias, int M, int kpad, int N,
    float* __restrict__ Y) {
    static_assert(NW == 4 || NW == 8, "2 x 2 or 4 x 2 waves");
    extern __shared__ __attribute__((aligned(16))) unsigned char split_lds[];
    constexpr int WM = 16 / NW, WN = 2;              // 32 x 32 accumulator fragments per wave
    constexpr int LR = 16 * NW;                      // rows one load instruction of the workgroup covers
    constexpr int AL = kSplitTileM / LR, BL = kSplitTileN / LR, NL = kSplitPieces * (AL + BL);   // loads per thread and step
    constexpr int NR = kSplitPieces * (WM + WN);     // fragment reads per wave and block
    constexpr int NM = 6 * WM * WN;                  // MFMAs per wave and block
    const int tid = (int)threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = lane_id();
    const int r = lane & 31, g = lane >> 5;
    const int m_tile = (int)blockIdx.x * kSplitTileM, n_tile = (int)blockIdx.y * kSplitTileN;
    const int m_base = m_tile + (wave >> 1) * (WM * 32);
    const int n_base = n_tile + (wave & 1) * (WN * 32);

    // ---- the thread's share of a step's loads: row (tid / 4) + LR j of the tile's frames or weights rows, slot tid % 4
    const int lrow = tid >> 2, lslot = tid & 3;
    const uint16_t* srcA[AL];
    const uint16_t* srcB[BL];
#pragma unroll
    for (int j = 0; j < AL; ++j) {
        const int m = m_tile + lrow + LR * j;
        srcA[j] = Xs + (size_t)(m < M ? m : M - 1) * kpad + lslot * 8;
    }
#pragma unroll
    for (int j = 0; j < BL; ++j) {
        const int n = n_tile + lrow + LR * j;
        srcB[j] = Ws + (size_t)(n < N ? n : N - 1) * kpad + lslot * 8;
    }
    const size_t planeA = (size_t)M * kpad, planeB = (size_t)N * kpad;
    const int st_off = lrow * kSplitRowBytes + ((lslot ^ ((lrow >> 2) & 3)) << 4);   // + LR j rows: (row / 4) % 4 unchanged

    // NL loads per thread and step, numbered i: piece i / (AL + BL); then frames row block i % (AL + BL) if that is
    // below AL, else weights row block i % (AL + BL) - AL
    struct Loads { u32x4 v[NL]; };
    auto gload_one = [&](Loads& L, int step, int i) {
        const int off = step * kSplitKStep, p = i / (AL + BL), sub = i % (AL + BL);
        if (sub < AL) L.v[i] = *reinterpret_cast<const u32x4*>(srcA[sub < AL ? sub : 0] + p * planeA + off);
        else L.v[i] = *reinterpret_cast<const u32x4*>(srcB[sub < AL ? 0 : sub - AL] + p * planeB + off);
    };
    auto lstore_one = [&](unsigned char* stage, const Loads& L, int i) {
        const int p = i / (AL + BL), sub = i % (AL + BL);
        if (sub < AL)
            *reinterpret_cast<u32x4*>(stage + p * (kSplitTileM * kSplitRowBytes) + sub * (LR * kSplitRowBytes) + st_off) = L.v[i];
        else
            *reinterpret_cast<u32x4*>(stage + kSplitStageA + p * (kSplitTileN * kSplitRowBytes) + (sub - AL) * (LR * kSplitRowBytes) +
                                      st_off) = L.v[i];
    };

    // ---- the wave's operand fragments of block h (0 or 1) of a stage: NR reads, numbered like the loads
    struct Frags { bf16x8 a[kSplitPieces][WM]; bf16x8 b[kSplitPieces][WN]; };
    const int swz = (r >> 2) & 3;
    const int a_off = ((wave >> 1) * (WM * 32) + r) * kSplitRowBytes;
    const int b_off = kSplitStageA + ((wave & 1) * (WN * 32) + r) * kSplitRowBytes;
    auto lread_one = [&](Frags& F, const unsigned char* stage, int h, int i) {
        const int so = ((2 * h + g) ^ swz) << 4;
        const int p = i / (WM + WN), sub = i % (WM + WN);
        if (sub < WM)
            F.a[p][sub < WM ? sub : 0] = *reinterpret_cast<const bf16x8*>(stage + p * (kSplitTileM * kSplitRowBytes) + a_off +
                                                                         sub * (32 * kSplitRowBytes) + so);
        else
            F.b[p][sub < WM ? 0 : sub - WM] = *reinterpret_cast<const bf16x8*>(stage + p * (kSplitTileN * kSplitRowBytes) + b_off +
                                                                              (sub - WM) * (32 * kSplitRowBytes) + so);
    };

    v16f32s acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // the six piece products of a block, smallest first; each accumulator is touched once per WM WN MFMAs
    auto products = [&](const Frags& F) {
        constexpr int px[6] = {0, 1, 2, 0, 1, 0};
        constexpr int pw[6] = {2, 1, 0, 1, 0, 0};
#pragma unroll
        for (int q = 0; q < 6; ++q)
#pragma unroll
            for (int fm = 0; fm < WM; ++fm)
#pragma unroll
                for (int fn = 0; fn < WN; ++fn)
                    acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F.a[px[q]][fm], F.b[pw[q]][fn], acc[fm][fn], 0, 0, 0);
    };

    // Step s lives in buffer s % 2.  The first G1 loads of step j + 2 are issued in the first half of step j and stored
    // in its second half; the others are issued in the second half and stored in the first half of step j + 1: the
    // buffer of step j is free from the barrier in the middle of step j to the one in the middle of step j + 1, and
    // nothing reads it in between.
    //
    // A wave issues in order, and the waves share one path to memory and one to LDS: loads in a row hold the MFMAs behind
    // them back for as long as the path takes to accept them.  So the memory instructions of a half go between its MFMAs:
    // after every fragment read one load or one LDS write, alternately, while there are any, then MPR MFMAs; the last
    // 12 MFMAs of a half come after all of them, so that what the next half needs has been issued that long before it
    // starts.  The scheduler is told this pattern; it keeps LDS reads and writes in source order, so the source has it too.
    constexpr int G1 = (NL + 1) / 2, G2 = NL - G1;
    constexpr int MPR = (NM - 12) / NR;
    static_assert(NL <= NR && MPR >= 1, "one load or write per fragment read");
    // half 0: loads [0, G1) of step `sl`, writes of loads [G1, NL) into `wr`; half 1: loads [G1, NL), writes of [0, G1)
    auto half = [&](int hf, const Frags& now, Frags& next, const unsigned char* rd, int rd_h, unsigned char* wr, Loads& L,
                    int sl) {
        const int g0 = hf ? G1 : 0, ng = hf ? G2 : G1, w0 = hf ? 0 : G1, nw = hf ? G1 : G2;
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            lread_one(next, rd, rd_h, i);
            // op i: loads at even i (or once the writes have run out), writes at odd i (or once the loads have run out)
            const int k = i / 2;
            if (i < 2 * (ng < nw ? ng : nw)) {
                if ((i & 1) == 0) gload_one(L, sl, g0 + k);
                else lstore_one(wr, L, w0 + k);
            } else {
                const int m = ng < nw ? ng : nw, e = i - 2 * m;   // the longer list alone
                if (ng > nw && e < ng - m) gload_one(L, sl, g0 + m + e);
                if (nw > ng && e < nw - m) lstore_one(wr, L, w0 + m + e);
            }
        }
        products(now);
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
            const int m = ng < nw ? ng : nw, e = i - 2 * m;
            if (i < 2 * m) {
                if ((i & 1) == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // load from memory
                else __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);              // LDS write
            } else {
                if (ng > nw && e < ng - m) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (nw > ng && e < nw - m) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);   // MFMA
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NM - MPR * NR, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int nS = kpad / kSplitKStep;
    unsigned char* buf0 = split_lds;
    unsigned char* buf1 = split_lds + kSplitStage;
    Loads L;
    Frags F0, F1;
    // start: step 0 complete, step 1 up to its loads [G1, NL), which are on their way
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
        // block 0 of step j; fragment reads of its block 1; the last loads of step j + 1 land in that step's buffer
        half(0, F0, F1, cur, 1, nxt, L, sl);
        // every wave has its last fragments of `cur` in registers, and step j + 1 is complete in `nxt`
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        // block 1 of step j; fragment reads of block 0 of step j + 1 (after the last step: unused); the first loads of
        // step j + 2 land in the buffer of step j
        half(1, F1, F0, nxt, 0, cur, L, sl);
    }
    __syncthreads();   // the buffers are free: the epilogue reuses them

    // ---- epilogue.  Accumulator fragment (fm, fn), register v of lane (r, g) is the sum for frame
    //      m_base + 32 fm + 8 (v/4) + 4 g + v%4 and output n_base + 32 fn + r.  Each wave turns 32 rows x 64 columns at
    //      a time through its own slice of LDS so that 16 lanes write 256 contiguous bytes of a row.
    if (m_base >= M || n_base >= N) return;   // wave-uniform, after the last barrier
    constexpr int LDW = 32 * WN + 4;
    float* stg = reinterpret_cast<float*>(split_lds) + wave * (32 * LDW);
    float bi[WN];
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        const int n = n_base + f * 32 + r;
        bi[f] = (n < N && bias) ? bias[n] : 0.0f;
    }
    const bool rows_vec = ((N & 3) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
    const int c4 = (lane & 15) * 4;
#pragma unroll
    for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
        for (int fn = 0; fn < WN; ++fn)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float h = acc[fm][fn][v] + bi[fn];
                if constexpr (ACT == ACT_HARDTANH) h = hardtanh(h);
                if constexpr (ACT == ACT_SIGMOID) h = sigmoid(h);
                stg[(8 * (v >> 2) + 4 * g + (v & 3)) * LDW + fn * 32 + r] = h;
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // this wave's LDS writes are done before it reads them back
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 4 + (lane >> 4);
            const int m = m_base + fm * 32 + row;
            const int n = n_base + c4;
            const float4 qv = *reinterpret_cast<const float4*>(stg + row * LDW + c4);
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
