// Matrix-core arm of the binary x binary product (paper Sec. 2.3), large-batch version:
// V_MFMA_F32_32X32X64_F8F6F4 with both operands in the 4-bit float format (+-1.0 exactly, see
// mfma_kernels.hpp for the encoding and for why the result is the exact integer dot product).
//
// Why this shape: every operand word a lane holds (32 elements of one row) has to be expanded from bits to
// nibbles by the vector ALU (7 instructions), and the SIMD issues either a VALU instruction or an MFMA per
// 4 clocks.  What counts is therefore expansions per multiply-accumulate: a wave that owns a 128 x 64 tile of
// [M][N] as 4 x 2 accumulator fragments of 32 x 32 expands 6 words for 8 MFMAs of 65536 MACs each, about
// half the expansion work per MAC of the 16 x 16 x 128 kernel with 64 x 64 wave tiles.
//
// K advances in super-steps of 512 bits: lane (r = lane%32, g = lane/32) fetches 32 contiguous bytes (words
// 8g..8g+7 of the super-step) of row r of every fragment in two 16-byte loads; word j feeds MFMA step j.
// Inside a fragment the order of k is therefore permuted, identically for both operands.  The next
// piece of K is fetched while the current one is expanded and multiplied.
// A workgroup is 2 x 2 waves: a (64 WM) x (64 WN) tile; at M = 4096, N = 2048 with WM = 4, WN = 2 that is
// 256 workgroups, one wave per SIMD of the chip.
#pragma once

#include "mfma_kernels.hpp"

namespace bnn {

typedef float v16f __attribute__((ext_vector_type(16)));

struct Raw8 {
    uint4 lo, hi;   // words 0..3 and 4..7 of a lane's share of a super-step
};

// Fetch words [16*S + 8*g, +8) of a packed row.  ALIGNED: rows are 16-byte aligned and whole super-steps
// long.  Otherwise each word is bounds-checked against the row length and reads as 0.
template <bool ALIGNED>
__device__ __forceinline__ Raw8 load_raw8(const uint32_t* __restrict__ row, int S, int g, int w32) {
    const int base = S * 16 + g * 8;
    Raw8 v;
    if constexpr (ALIGNED) {
        v.lo = *reinterpret_cast<const uint4*>(row + base);
        v.hi = *reinterpret_cast<const uint4*>(row + base + 4);
    } else {
        v.lo.x = (base + 0 < w32) ? row[base + 0] : 0u;
        v.lo.y = (base + 1 < w32) ? row[base + 1] : 0u;
        v.lo.z = (base + 2 < w32) ? row[base + 2] : 0u;
        v.lo.w = (base + 3 < w32) ? row[base + 3] : 0u;
        v.hi.x = (base + 4 < w32) ? row[base + 4] : 0u;
        v.hi.y = (base + 5 < w32) ? row[base + 5] : 0u;
        v.hi.z = (base + 6 < w32) ? row[base + 6] : 0u;
        v.hi.w = (base + 7 < w32) ? row[base + 7] : 0u;
    }
    return v;
}

// words[lane_lo] = lo, words[lane_hi] = hi (wave-uniform values; the lanes must be compile-time constants after
// unrolling).
// On this core a vector instruction that reads an SGPR needs two wait states after the vector instruction (here
// the compare behind a ballot) that wrote it.  The compiler inserts them for its own instructions but does not
// look inside inline assembly, so the two wait states are part of the statement.
__device__ __forceinline__ void write_lane_pair(int& words, uint32_t lo, uint32_t hi, int lane_lo, int lane_hi) {
    asm volatile("s_nop 1\n\tv_writelane_b32 %0, %1, %3\n\tv_writelane_b32 %0, %2, %4"
                 : "+v"(words) : "s"(lo), "s"(hi), "n"(lane_lo), "n"(lane_hi));
}

// Called inside the product loop, after the first products: the loads that produced sc/bi then stay in front of
// the loop, where they were written, instead of moving next to their use in the epilogue, and by the time this
// point is reached they have long returned (the operand words used by those products were requested later).
template <int WN>
__device__ __forceinline__ void pin_loaded(float (&sc)[WN], float (&bi)[WN]) {
#pragma unroll
    for (int f = 0; f < WN; ++f) asm volatile("" : "+v"(sc[f]), "+v"(bi[f]));
}

// 16 bytes at byte offset voff (per lane) + soff (wave-uniform) of a buffer.
__device__ __forceinline__ uint4 load16(__amdgpu_buffer_rsrc_t rs, int voff, int soff) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ uint32_t word_of(const Raw8& v, int j) {
    return j < 4 ? word_of(v.lo, j) : word_of(v.hi, j - 4);
}

// PINGPONG (aligned rows only): the operand fetch runs ahead of the products in separate register sets, with the
// issue order pinned by scheduling barriers: two whole super-steps for 64-row wave tiles (WM = 2), three half
// super-steps in rotation for 128-row tiles (WM = 4), whose half-steps are also written out instruction slot by
// slot.  Without it (current = next, order left to the compiler) the two sets get merged and every super-step
// waits for its own loads; kept for ragged rows and for comparison.
// X01: the activation bits are read as 0/1 instead of -1/+1 (paper Sec. 3.2).  With a the -1/+1 reading of the same
// bits, h = (a + 1) / 2 and h.w = (a.w + sum_k w_k) / 2: the product runs unchanged, every lane counts the 1 bits of
// the weight words it fetches anyway (the two lanes that share a row add theirs up), and the epilogue forms
// 0.5 (a.w) + (popcount(w) - K/2), exact in fp32.
// SPLITK (128-row pinned variant only, K a multiple of 1024): the workgroup has 8 waves; waves 4..7 own the same four
// wave tiles as waves 0..3 and take the second half of K, so that a grid of one workgroup per CU still puts TWO waves
// on every SIMD (a single wave per SIMD cannot cover its own operand latencies: measured 28 ns per MFMA against 17-19
// with two).  Their partial sums (small integers, exact in fp32 in any order) go to waves 0..3 through LDS, 64
// accumulator registers at a time; waves 0..3 run the epilogue.
// Grid: x = ceil(M / (64*WM)), y = ceil(N / (64*WN)); block = 256 threads (512 with SPLITK).
template <int WM, int WN, int ACT, bool ALIGNED, bool PINGPONG = false, bool X01 = false, bool SPLITK = false>
__global__ __launch_bounds__(SPLITK ? 512 : 256, SPLITK ? 1 : 2) void binx_mfma32_kernel(const uint32_t* __restrict__ Xp, const uint32_t* __restrict__ Wp,
                                                          const float* __restrict__ scale, const float* __restrict__ bias,
                                                          int M, int K, int N, int w32, void* __restrict__ Y, int yw32,
                                                          unsigned int a_bytes, unsigned int b_bytes, int xcd_order,
                                                          const CoopLsm coop) {
    static_assert(!SPLITK || (WM == 4 && PINGPONG && !X01 && ACT != ACT_LSM_COOP), "split K: 128-row pinned variant, -1/+1 inputs");
    const int wave_all = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wave = SPLITK ? (wave_all & 3) : wave_all;   // which wave tile of the workgroup
    const int khalf = SPLITK ? (wave_all >> 2) : 0;        // which half of K
    const int lane = lane_id();
    const int r = lane & 31;   // row of the operand fragment / column of the accumulator fragment
    const int g = lane >> 5;   // k-group of the operand fragment / row-group of the accumulator fragment
    int tile_m = (int)blockIdx.x, tile_n = (int)blockIdx.y;
    if (xcd_order) {
        // Workgroups go to the 8 XCDs round-robin in dispatch order, and every XCD has its own L2.  Give XCD x a
        // contiguous run of tiles in (frames tile, outputs tile) order, outputs fastest: the workgroups that share
        // a frames tile then run on the same XCD, one after the other, and its rows are fetched into one L2 once.
        const int total = (int)(gridDim.x * gridDim.y);
        const int lin = (int)(blockIdx.y * gridDim.x + blockIdx.x);
        const int x = lin & 7, q = total >> 3, rem = total & 7;
        const int t = x * q + (x < rem ? x : rem) + (lin >> 3);
        tile_m = t / (int)gridDim.y;
        tile_n = t - tile_m * (int)gridDim.y;
    }
    const int m_base = (tile_m * 2 + (wave >> 1)) * (WM * 32);
    const int n_base = (tile_n * 2 + (wave & 1)) * (WN * 32);
    // (the cooperative epilogue has workgroup barriers: there a wave without rows or columns of its own runs along on
    // clamped rows and contributes nothing)
    if constexpr (ACT != ACT_LSM_COOP) {
        if (m_base >= M || n_base >= N) return;   // wave-uniform
    }

    const uint32_t* arow[WM];
    const uint32_t* brow[WN];
#pragma unroll
    for (int f = 0; f < WM; ++f) {
        const int m = m_base + f * 32 + r;
        arow[f] = Xp + (size_t)(m < M ? m : M - 1) * w32;
    }
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        const int n = n_base + f * 32 + r;
        brow[f] = Wp + (size_t)(n < N ? n : N - 1) * w32;
    }

    // Scale and bias of this lane's columns, requested before the product so that the epilogue does not wait for
    // them.  Columns past N get scale = bias = 0: their pre-activation is 0, their Sign bit 0 (pad bits stay 0).
    float sc[WN], bi[WN];
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        const int n = n_base + f * 32 + r;
        sc[f] = n < N ? (scale ? scale[n] : 1.0f) : 0.0f;
        bi[f] = n < N ? (bias ? bias[n] : 0.0f) : 0.0f;
    }

    int ones[WN];   // X01: 1 bits of this lane's share of the weight rows
#pragma unroll
    for (int f = 0; f < WN; ++f) ones[f] = 0;
    auto count4 = [&](const uint4 (&b)[WN]) {
        if constexpr (X01) {
#pragma unroll
            for (int f = 0; f < WN; ++f)
                ones[f] += __builtin_popcount(b[f].x) + __builtin_popcount(b[f].y) + __builtin_popcount(b[f].z) + __builtin_popcount(b[f].w);
        }
    };

    v16f acc[WM][WN];
    if constexpr (!PINGPONG || WM >= 4) {   // (the 64-row pinned variant starts its accumulators with a zero addend instead)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    }

    const ExpandConsts ec = expand_consts();
    const int nS = (K + 511) >> 9;
    static_assert(ALIGNED || !PINGPONG, "the pinned pipelines fetch whole 16-byte pieces of whole super-steps");
    const v16f zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (PINGPONG) {
        // Buffer addressing: one byte offset per fragment row in a VGPR, the position along K in an SGPR, so the loop
        // carries no 64-bit address arithmetic.  (The host selects these variants only for operands below 2 GiB.)
        const __amdgpu_buffer_rsrc_t ars = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(Xp), 0, (int)a_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(Wp), 0, (int)b_bytes, 0x00020000);
        int aoff[WM], boff[WN];
#pragma unroll
        for (int f = 0; f < WM; ++f) {
            const int m = m_base + f * 32 + r;
            aoff[f] = ((m < M ? m : M - 1) * w32 + g * 8) * 4;
        }
#pragma unroll
        for (int f = 0; f < WN; ++f) {
            const int n = n_base + f * 32 + r;
            boff[f] = ((n < N ? n : N - 1) * w32 + g * 8) * 4;
        }
        // the first product into each accumulator takes a zero addend instead of a cleared register
        auto products = [&](const uint4 (&a)[WM], const uint4 (&b)[WN], bool first) {
            count4(b);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v8i bx[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f) bx[f] = expand_pm1_fp4(word_of(b[f], j), ec);
#pragma unroll
                for (int fm = 0; fm < WM; ++fm) {
                    const v8i ax = expand_pm1_fp4(word_of(a[fm], j), ec);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ax, bx[fn], (first && j == 0) ? zero16 : acc[fm][fn],
                                                                                    4, 4, 0, 0, 0, 0);
                }
            }
        };
        if constexpr (WM >= 4) {
            // 128-row wave tiles leave no room for two whole operand sets beside the 128 accumulator registers: the
            // two sets are the two halves of a super-step (words 0..3 and 4..7 of every lane's share) instead.
            // Three sets in rotation, fetched two half-steps ahead: with one wave per SIMD (4096 x 2048 outputs fill the
            // chip exactly once) nothing else covers the memory latency, and one half-step of products is shorter.
            uint4 a0[WM], b0[WN], a1[WM], b1[WN], a2[WM], b2[WN];
            const int H = SPLITK ? nS : 2 * nS;   // half-steps of this wave (split K: nS is even, each half has nS / 2 super-steps)
            if constexpr (SPLITK) {
#pragma unroll
                for (int f = 0; f < WM; ++f) arow[f] += khalf * (nS >> 1) * 16;
#pragma unroll
                for (int f = 0; f < WN; ++f) brow[f] += khalf * (nS >> 1) * 16;
            }
            // (plain pointer loads here: buffer addressing saves the address arithmetic but measured 3 % slower on
            //  this variant, as did a peeled first round with zero addends: more code to fetch for four rounds)
            auto fetch = [&](uint4 (&a)[WM], uint4 (&b)[WN], int h) {
                const int hc = h < H ? h : H - 1;   // past the end: re-read the last half-step (in bounds, unused)
                const int base = (hc >> 1) * 16 + g * 8 + (hc & 1) * 4;
#pragma unroll
                for (int f = 0; f < WM; ++f) a[f] = *reinterpret_cast<const uint4*>(arow[f] + base);
#pragma unroll
                for (int f = 0; f < WN; ++f) b[f] = *reinterpret_cast<const uint4*>(brow[f] + base);
            };
            // Every fetch is unconditional: a fetch whose only use sits behind a branch gets moved behind that
            // branch by the compiler, next to its use, and then nothing overlaps.
            // Issue order inside a half-step, written out and pinned slot by slot.  A wave issues in order, and an
            // MFMA that finds the pipe busy (32 clocks per 32x32x64) blocks whatever follows it: left to the
            // compiler's order (expansions in clumps, MFMAs back to back) one wave per SIMD ran at 70 clocks per
            // MFMA.  Here every MFMA is followed by the 5-6 expansion instructions of an operand needed two to
            // eight MFMAs later, which issue in its shadow: the frames fragment fm+1 of this step while fm is
            // multiplied, and the two weights fragments and frames fragment 0 of the NEXT step (taken from the next
            // register set after the last step of a half-step) spread over the eight slots.
            static_assert(WM == 4 && WN == 2, "the slot plan below is written for 4 x 2 fragments");
            v8i bx[2][WN];   // expanded weights: [parity of the step][fragment]
            v8i ax[2];       // expanded frames: fragment fm lives in ax[fm & 1]
            auto piece = [&](v8i& dst, uint32_t w, int part) {   // part 0..2: shifted dwords (2 instructions), 3: unshifted (1)
                dst[part] = (int)((((part < 3) ? (w << (3 - part)) : w) & ec.sign_mask) | ec.one_bits);
            };
            auto clear_hi = [&](v8i& d) { d[4] = 0; d[5] = 0; d[6] = 0; d[7] = 0; };   // unused by the 4-bit format
            clear_hi(ax[0]); clear_hi(ax[1]);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int f = 0; f < WN; ++f) clear_hi(bx[t][f]);
            auto half_step = [&](const uint4 (&a)[WM], const uint4 (&b)[WN], const uint4 (&an)[WM], const uint4 (&bn)[WN]) {
                count4(b);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int pc = j & 1, pn = pc ^ 1;
                    // words of the next step: the next word of this set, or the first word of the next set
                    const uint32_t wb0 = j < 3 ? word_of(b[0], j + 1) : word_of(bn[0], 0);
                    const uint32_t wb1 = j < 3 ? word_of(b[1], j + 1) : word_of(bn[1], 0);
                    const uint32_t wa0 = j < 3 ? word_of(a[0], j + 1) : word_of(an[0], 0);
                    const uint32_t wa1 = word_of(a[1], j), wa2 = word_of(a[2], j), wa3 = word_of(a[3], j);
#define BNN_MFMA(fm, fn) acc[fm][fn] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ax[(fm) & 1], bx[pc][fn], acc[fm][fn], 4, 4, 0, 0, 0, 0)
#define BNN_SLOT_END __builtin_amdgcn_sched_barrier(0)
                    BNN_MFMA(0, 0); piece(ax[1], wa1, 0); piece(ax[1], wa1, 1); piece(ax[1], wa1, 3); BNN_SLOT_END;
                    BNN_MFMA(0, 1); piece(ax[1], wa1, 2); piece(bx[pn][0], wb0, 0); piece(bx[pn][0], wb0, 3); BNN_SLOT_END;
                    BNN_MFMA(1, 0); piece(ax[0], wa2, 0); piece(ax[0], wa2, 1); piece(ax[0], wa2, 3); BNN_SLOT_END;
                    BNN_MFMA(1, 1); piece(ax[0], wa2, 2); piece(bx[pn][0], wb0, 1); piece(bx[pn][0], wb0, 2); BNN_SLOT_END;
                    BNN_MFMA(2, 0); piece(ax[1], wa3, 0); piece(ax[1], wa3, 1); piece(ax[1], wa3, 3); BNN_SLOT_END;
                    BNN_MFMA(2, 1); piece(ax[1], wa3, 2); piece(bx[pn][1], wb1, 0); piece(bx[pn][1], wb1, 3); BNN_SLOT_END;
                    BNN_MFMA(3, 0); piece(bx[pn][1], wb1, 1); piece(bx[pn][1], wb1, 2); BNN_SLOT_END;
                    BNN_MFMA(3, 1); BNN_SLOT_END;
                    // frames fragment 0 of the next step overwrites ax[0], which MFMA (2, *) has finished reading
                    piece(ax[0], wa0, 0); piece(ax[0], wa0, 1); piece(ax[0], wa0, 2); piece(ax[0], wa0, 3); BNN_SLOT_END;
#undef BNN_MFMA
#undef BNN_SLOT_END
                }
            };
            // Every fetch is unconditional: a fetch whose only use sits behind a branch gets moved behind that
            // branch by the compiler, next to its use, and then nothing overlaps.
            fetch(a0, b0, 0);
            fetch(a1, b1, 1);
            {   // operands of the very first step
                const uint32_t wb0 = word_of(b0[0], 0), wb1 = word_of(b0[1], 0), wa0 = word_of(a0[0], 0);
#pragma unroll
                for (int part = 0; part < 4; ++part) { piece(bx[0][0], wb0, part); piece(bx[0][1], wb1, part); piece(ax[0], wa0, part); }
            }
            int h = 0;
            for (; h + 2 < H; h += 3) {
                fetch(a2, b2, h + 2);
                __builtin_amdgcn_sched_barrier(0);
                half_step(a0, b0, a1, b1);
                pin_loaded(sc, bi);
                __builtin_amdgcn_sched_barrier(0);
                fetch(a0, b0, h + 3);
                __builtin_amdgcn_sched_barrier(0);
                half_step(a1, b1, a2, b2);
                __builtin_amdgcn_sched_barrier(0);
                fetch(a1, b1, h + 4);
                __builtin_amdgcn_sched_barrier(0);
                half_step(a2, b2, a0, b0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (h < H) half_step(a0, b0, a1, b1);       // one or two half-steps left, already fetched
            if (h + 1 < H) half_step(a1, b1, a2, b2);
        } else {
            // two whole super-steps in registers; set 0 holds the even ones at first, then the sets alternate
            uint4 a0l[WM], a0h[WM], b0l[WN], b0h[WN], a1l[WM], a1h[WM], b1l[WN], b1h[WN];
            auto fetch = [&](uint4 (&al)[WM], uint4 (&ah)[WM], uint4 (&bl)[WN], uint4 (&bh)[WN], int S) {
                const int so = (S < nS ? S : nS - 1) * 64;
#pragma unroll
                for (int f = 0; f < WM; ++f) { al[f] = load16(ars, aoff[f], so); ah[f] = load16(ars, aoff[f], so + 16); }
#pragma unroll
                for (int f = 0; f < WN; ++f) { bl[f] = load16(brs, boff[f], so); bh[f] = load16(brs, boff[f], so + 16); }
            };
            fetch(a0l, a0h, b0l, b0h, 0);
            fetch(a1l, a1h, b1l, b1h, 1);
            __builtin_amdgcn_sched_barrier(0);
            products(a0l, b0l, true);
            products(a0h, b0h, false);
            __builtin_amdgcn_sched_barrier(0);
            int S = 1;   // set 1 holds super-step S, set 0 is free
            for (; S + 1 < nS; S += 2) {
                fetch(a0l, a0h, b0l, b0h, S + 1);
                __builtin_amdgcn_sched_barrier(0);
                products(a1l, b1l, false);
                products(a1h, b1h, false);
                pin_loaded(sc, bi);
                __builtin_amdgcn_sched_barrier(0);
                fetch(a1l, a1h, b1l, b1h, S + 2);
                __builtin_amdgcn_sched_barrier(0);
                products(a0l, b0l, false);
                products(a0h, b0h, false);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (S < nS) {   // one super-step left, already in set 1
                products(a1l, b1l, false);
                products(a1h, b1h, false);
            }
        }
    } else {
        Raw8 araw[WM], braw[WN];
#pragma unroll
        for (int f = 0; f < WM; ++f) araw[f] = load_raw8<ALIGNED>(arow[f], 0, g, w32);
#pragma unroll
        for (int f = 0; f < WN; ++f) braw[f] = load_raw8<ALIGNED>(brow[f], 0, g, w32);

        for (int S = 0; S < nS; ++S) {
            Raw8 anext[WM], bnext[WN];
            const int Sn = (S + 1 < nS) ? S + 1 : S;   // the last prefetch re-reads the last step (in bounds, unused)
#pragma unroll
            for (int f = 0; f < WM; ++f) anext[f] = load_raw8<ALIGNED>(arow[f], Sn, g, w32);
#pragma unroll
            for (int f = 0; f < WN; ++f) bnext[f] = load_raw8<ALIGNED>(brow[f], Sn, g, w32);

            if constexpr (X01) {
                uint4 lo[WN], hi[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f) { lo[f] = braw[f].lo; hi[f] = braw[f].hi; }
                count4(lo);
                count4(hi);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v8i bx[WN];
#pragma unroll
                for (int f = 0; f < WN; ++f) bx[f] = expand_pm1_fp4(word_of(braw[f], j), ec);
#pragma unroll
                for (int fm = 0; fm < WM; ++fm) {
                    const v8i ax = expand_pm1_fp4(word_of(araw[fm], j), ec);
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
                        acc[fm][fn] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ax, bx[fn], acc[fm][fn], 4, 4, 0, 0, 0, 0);
                }
            }
            pin_loaded(sc, bi);
#pragma unroll
            for (int f = 0; f < WM; ++f) araw[f] = anext[f];
#pragma unroll
            for (int f = 0; f < WN; ++f) braw[f] = bnext[f];
        }
    }

    if constexpr (SPLITK) {
        // the second half of K joins the first: 64 accumulator registers per round through 64 KiB of LDS
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        __shared__ f32x4 xch[4][16][kWave];   // [wave tile][four registers][lane]
#pragma unroll
        for (int round = 0; round < 2; ++round) {
            if (khalf == 1) {
#pragma unroll
                for (int fmh = 0; fmh < 2; ++fmh)
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v16f& c = acc[2 * round + fmh][fn];
                            xch[wave][(fmh * 2 + fn) * 4 + q][lane] = f32x4{c[4 * q], c[4 * q + 1], c[4 * q + 2], c[4 * q + 3]};
                        }
            }
            __syncthreads();
            if (khalf == 0) {
#pragma unroll
                for (int fmh = 0; fmh < 2; ++fmh)
#pragma unroll
                    for (int fn = 0; fn < WN; ++fn)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const f32x4 p = xch[wave][(fmh * 2 + fn) * 4 + q][lane];
                            v16f& c = acc[2 * round + fmh][fn];
                            c[4 * q] += p[0]; c[4 * q + 1] += p[1]; c[4 * q + 2] += p[2]; c[4 * q + 3] += p[3];
                        }
            }
            if (round == 0) __syncthreads();   // everything read before the second round overwrites it
        }
        if (khalf == 1) return;   // wave-uniform; no barrier follows
    }

    // ---- epilogue.  Accumulator fragment (fm, fn), register v of lane (r, g) is
    //      dot[m_base + 32 fm + 8 (v/4) + 4 g + v%4][n_base + 32 fn + r] + pad.
    const float pad = (float)(nS * 512 - K);
    float half_wsum[WN];   // X01: popcount(w) - K/2 = (sum_k w_k) / 2 of this lane's columns
#pragma unroll
    for (int f = 0; f < WN; ++f) {
        half_wsum[f] = 0.0f;
        if constexpr (X01) half_wsum[f] = (float)(ones[f] + __shfl_xor(ones[f], 32, kWave)) - 0.5f * (float)K;
    }
    auto dot_of = [&](float a, int fn) -> float {
        const float d = ALIGNED ? a : a - pad;   // whole super-steps: no pad
        if constexpr (X01) return __builtin_fmaf(d, 0.5f, half_wsum[fn]);
        else return d;
    };
    if constexpr (ACT == ACT_SIGN) {
        uint32_t* Yw = (uint32_t*)Y;
#pragma unroll
        for (int fn = 0; fn < WN; ++fn) {
            const int wcol = (n_base >> 5) + fn;
#pragma unroll
            for (int fm = 0; fm < WM; ++fm) {
                // One ballot is two output words: lanes 0..31 are the 32 outputs of frame row 8(v/4)+v%4,
                // lanes 32..63 the same outputs of the frame 4 rows below.  Word v is parked in lane v
                // (and 32+v) of one register, so the whole fragment leaves with a single store.
                int words = 0;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float dot = dot_of(acc[fm][fn][v], fn);
                    const unsigned long long b = __builtin_amdgcn_ballot_w64(sign_bit(affine(sc[fn], dot, bi[fn])));
                    write_lane_pair(words, (uint32_t)b, (uint32_t)(b >> 32), v, 32 + v);
                }
                if (r < 16) {
                    const int m = m_base + fm * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (m < M && wcol < yw32) Yw[(size_t)m * yw32 + wcol] = (uint32_t)words;
                }
            }
        }
    } else if constexpr (ACT == ACT_LSM_COOP) {
        // log-Softmax of whole rows without a second kernel.  The rows of this workgroup's tile continue in the other
        // tiles of the same frames (grid row tile_m): every workgroup reduces its 128 columns of each row to
        // (max, sum of exp(h - max)), publishes the pair, waits for the other tiles of its grid row, combines the pairs
        // to max + log sum exp and only then writes its share of the rows, normalised, straight from the accumulators.
        // Publishing: write-through stores (sc1), wait until they are acknowledged, then the flag.  Readers poll the
        // flags with loads that bypass the non-coherent caches (sc1) and then read the pairs with plain loads: no
        // cache of this launch can hold an older copy of a pair, because nothing reads a pair before its flag is up
        // and what earlier launches left in the caches is dropped at the kernel boundary.  The wait is bounded.
        static_assert(WN == 2, "the transposing epilogue is written for 64-column wave tiles");
        constexpr int LDW = 32 * WN + 4;
        constexpr int ROWS = 32 * WM;                          // rows of a wave; the workgroup has 2 ROWS
        __shared__ __attribute__((aligned(16))) uint32_t stage[4][32 * LDW];
        __shared__ float2 wave_part[4][ROWS];
        __shared__ float lse_s[2 * ROWS];
        uint32_t* st = stage[wave];
        const int c4 = (lane & 15) * 4;
        const int T = (int)gridDim.y;
        const float ninf = -__builtin_inff();
        // (a) pre-activations, in place; columns past N count as -inf (no share in any maximum or sum)
#pragma unroll
        for (int fm = 0; fm < WM; ++fm)
#pragma unroll
            for (int fn = 0; fn < WN; ++fn) {
                const bool col = n_base + fn * 32 + r < N;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float h = affine(sc[fn], dot_of(acc[fm][fn][v], fn), bi[fn]);
                    acc[fm][fn][v] = col ? h : ninf;
                }
            }
        // (b) this wave's 64 columns of each of its rows: through its LDS slice, 32 rows at a time, so that lane
        //     (row = lane % 32, half = lane / 32) holds 32 consecutive columns of one row in registers: the maximum and
        //     the sum are then taken inside a lane, with a single exchange between the two halves of a row for each
        //     (8 consecutive lanes read 16 bytes each from rows 68 words apart: 32 different banks)
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int fn = 0; fn < WN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    st[(8 * (v >> 2) + 4 * g + (v & 3)) * LDW + fn * 32 + r] = __float_as_uint(acc[fm][fn][v]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            float hv[32];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint4 q = *reinterpret_cast<const uint4*>(st + r * LDW + g * 32 + j * 4);
                hv[4 * j] = __uint_as_float(q.x); hv[4 * j + 1] = __uint_as_float(q.y);
                hv[4 * j + 2] = __uint_as_float(q.z); hv[4 * j + 3] = __uint_as_float(q.w);
            }
            float m4[4] = {hv[0], hv[1], hv[2], hv[3]};        // four chains: the maximum does not care about order
#pragma unroll
            for (int j = 4; j < 32; ++j) m4[j & 3] = __builtin_fmaxf(m4[j & 3], hv[j]);
            float mx = __builtin_fmaxf(__builtin_fmaxf(m4[0], m4[1]), __builtin_fmaxf(m4[2], m4[3]));
            mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, kWave));
            float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (mx != ninf) {
#pragma unroll
                for (int j = 0; j < 32; ++j) s4[j & 3] += __expf(hv[j] - mx);
            }
            float s = (s4[0] + s4[1]) + (s4[2] + s4[3]);
            s += __shfl_xor(s, 32, kWave);
            if (g == 0) wave_part[wave][fm * 32 + r] = make_float2(mx, s);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        }
        __syncthreads();
        // (c) the two waves that share a row, then out to memory
        const int trow = (int)threadIdx.x;                     // row of the workgroup tile (threads below 2 ROWS)
        if (trow < 2 * ROWS) {
            const float2 pa = wave_part[2 * (trow / ROWS)][trow % ROWS], pb = wave_part[2 * (trow / ROWS) + 1][trow % ROWS];
            const float mx = __builtin_fmaxf(pa.x, pb.x);
            float s = 0.0f;
            if (pa.x != ninf) s += pa.y * __expf(pa.x - mx);
            if (pb.x != ninf) s += pb.y * __expf(pb.x - mx);
            const unsigned long long pair = (unsigned long long)__float_as_uint(mx) | ((unsigned long long)__float_as_uint(s) << 32);
            __hip_atomic_store(reinterpret_cast<unsigned long long*>(coop.partials + ((size_t)tile_m * T + tile_n) * (2 * ROWS) + trow), pair,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the pairs have arrived ...
        __syncthreads();
        if (threadIdx.x == 0)                                  // ... before the flag says so
            __hip_atomic_store(coop.flags + (size_t)tile_m * T + tile_n, coop.stamp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (wave == 0) {
            const unsigned long long* f = coop.flags + (size_t)tile_m * T;
            bool ok = false;
            for (int spin = 0; spin < coop.spin_limit; ++spin) {
                unsigned long long v = coop.stamp;
                if (lane < T) v = __hip_atomic_load(f + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (__builtin_amdgcn_ballot_w64(v == coop.stamp) == ~0ull) { ok = true; break; }
                __builtin_amdgcn_s_sleep(1);
            }
            if (!ok && lane == 0) atomicAdd(coop.timeouts, 1u);
        }
        __syncthreads();
        // (d) max + log sum exp of each row over all tiles of the grid row
        if (trow < 2 * ROWS) {
            // (consecutive lanes read consecutive rows of one tile's pairs: whole cache lines per request; 32 requests in
            // flight before the first pair is used)
            const unsigned long long* src = reinterpret_cast<const unsigned long long*>(coop.partials + (size_t)tile_m * T * (2 * ROWS) + trow);
            float mx = ninf, s = 0.0f;
            for (int t0 = 0; t0 < T; t0 += 32) {
                unsigned long long pr[32];
#pragma unroll
                for (int i = 0; i < 32; ++i)                    // (clamped: the same pair again, skipped below)
                    pr[i] = src[(size_t)(t0 + i < T ? t0 + i : T - 1) * (2 * ROWS)];
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const float pm = __uint_as_float((uint32_t)pr[i]), ps = __uint_as_float((uint32_t)(pr[i] >> 32));
                    if (t0 + i < T && pm != ninf) {
                        if (pm > mx) { s = s * __expf(mx - pm) + ps; mx = pm; }   // (mx = -inf: s = 0, exp gives 0)
                        else s += ps * __expf(pm - mx);
                    }
                }
            }
            lse_s[trow] = mx + __logf(s);
        }
        __syncthreads();
        // (e) normalise and write: rows leave as contiguous 256-byte pieces, as in the plain fp32 epilogue
        const bool rows_vec = ((N & 3) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int fn = 0; fn < WN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    st[(8 * (v >> 2) + 4 * g + (v & 3)) * LDW + fn * 32 + r] = __float_as_uint(acc[fm][fn][v]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int row = it * 4 + (lane >> 4);
                const int m = m_base + fm * 32 + row;
                const int n = n_base + c4;
                const uint4 q = *reinterpret_cast<const uint4*>(st + row * LDW + c4);
                const float l = lse_s[(wave >> 1) * ROWS + fm * 32 + row];
                float4 o;
                o.x = __uint_as_float(q.x) - l; o.y = __uint_as_float(q.y) - l; o.z = __uint_as_float(q.z) - l; o.w = __uint_as_float(q.w) - l;
                if (m < M) {
                    float* y = (float*)Y + (size_t)m * N + n;
                    if (rows_vec && n + 3 < N) {
                        *reinterpret_cast<float4*>(y) = o;
                    } else {
                        if (n + 0 < N) y[0] = o.x;
                        if (n + 1 < N) y[1] = o.y;
                        if (n + 2 < N) y[2] = o.z;
                        if (n + 3 < N) y[3] = o.w;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        }
    } else {
        // 32-bit outputs: the accumulator layout gives a lane one column and 16 scattered rows, which would
        // store 128-byte pieces.  Each wave turns 32 rows x (32 WN) columns at a time through its own slice
        // of LDS so that 16 lanes write 256 contiguous bytes of a row (16 bytes per lane).
        static_assert(WN == 2, "the transposing epilogue is written for 64-column wave tiles");
        constexpr int LDW = 32 * WN + 4;                       // padded row length in words
        __shared__ __attribute__((aligned(16))) uint32_t stage[4][32 * LDW];
        uint32_t* st = stage[wave];
        const bool rows_vec = ((N & 3) == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
        const int c4 = (lane & 15) * 4;                        // this lane's 4 columns of the 64
#pragma unroll
        for (int fm = 0; fm < WM; ++fm) {
#pragma unroll
            for (int fn = 0; fn < WN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float dot = dot_of(acc[fm][fn][v], fn);
                    uint32_t bits;
                    if constexpr (ACT == ACT_RAW_I32 || ACT == ACT_DOT_I16) {
                        bits = (uint32_t)(int)dot;
                    } else {
                        float h = affine(sc[fn], dot, bi[fn]);
                        if constexpr (ACT == ACT_HARDTANH) h = hardtanh(h);
                        if constexpr (ACT == ACT_SIGMOID) h = sigmoid(h);
                        bits = __float_as_uint(h);
                    }
                    st[(8 * (v >> 2) + 4 * g + (v & 3)) * LDW + fn * 32 + r] = bits;
                }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // this wave's LDS writes are done before it reads them back
            if constexpr (ACT == ACT_DOT_I16) {
                // int16 outputs: 8 lanes write the 128 bytes a row has in this wave tile (eight int16 = 16 bytes per lane),
                // so a store instruction covers 8 rows and the tile takes half as many of them as with 8 bytes per lane
                // (the stores, not their bytes, are what this epilogue costs).  The caller guarantees N % 4 == 0 and a
                // 16-byte aligned Y.
                const int c8 = (lane & 7) * 8;
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = it * 8 + (lane >> 3);
                    const int m = m_base + fm * 32 + row;
                    const int n = n_base + c8;
                    const uint4 q0 = *reinterpret_cast<const uint4*>(st + row * LDW + c8);
                    const uint4 q1 = *reinterpret_cast<const uint4*>(st + row * LDW + c8 + 4);
                    uint4 h;
                    h.x = (q0.x & 0xFFFFu) | (q0.y << 16);
                    h.y = (q0.z & 0xFFFFu) | (q0.w << 16);
                    h.z = (q1.x & 0xFFFFu) | (q1.y << 16);
                    h.w = (q1.z & 0xFFFFu) | (q1.w << 16);
                    if (m < M) {
                        uint16_t* y = reinterpret_cast<uint16_t*>(Y) + (size_t)m * 2 * N + n;
                        if (n + 7 < N) {
                            *reinterpret_cast<uint4*>(y) = h;
                        } else if (n < N) {   // N % 8 == 4: the last four outputs of the row
                            *reinterpret_cast<uint2*>(y) = make_uint2(h.x, h.y);
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // reads done before the next fragment row overwrites the slice
                continue;
            }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int row = it * 4 + (lane >> 4);
                const int m = m_base + fm * 32 + row;
                const int n = n_base + c4;
                const uint4 q = *reinterpret_cast<const uint4*>(st + row * LDW + c4);
                if (m < M) {
                    uint32_t* y = (uint32_t*)Y + (size_t)m * N + n;
                    if (rows_vec && n + 3 < N) {
                        *reinterpret_cast<uint4*>(y) = q;
                    } else {
                        if (n + 0 < N) y[0] = q.x;
                        if (n + 1 < N) y[1] = q.y;
                        if (n + 2 < N) y[2] = q.z;
                        if (n + 3 < N) y[3] = q.w;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // reads done before the next fragment row overwrites the slice
        }
    }
}

}  // namespace bnn
