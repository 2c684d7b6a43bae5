// Device-side helpers shared by the gfx950 kernels of the binary-network forward pass.
// Written for CDNA4 only: 64-wide wavefronts, no portability layer.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bnn {

constexpr int kWave = 64;

// Activation selectors; numerically identical to bnn_act in include/bnn.h.
enum : int { ACT_RAW_I32 = 0, ACT_LINEAR = 1, ACT_HARDTANH = 2, ACT_SIGN = 3, ACT_LOGSOFTMAX = 4, ACT_SIGMOID = 5 };
// Kernel-internal: the integer product as int16 in the first 2 N bytes of each fp32 output row (|dot| <= K < 2^15);
// the log-Softmax row kernel turns the row into fp32 log-posteriors in place.
enum : int { ACT_DOT_I16 = 100 };
// Kernel-internal: log-Softmax finished inside the product kernel.  The workgroups that share rows of frames hand each
// other their share of every row's maximum and sum of exponentials through memory (see CoopLsm); needs every workgroup
// of the launch resident at once.
enum : int { ACT_LSM_COOP = 101 };

// Hand-over area of ACT_LSM_COOP.  Tile (tm, tn) of the launch writes partials[(tm * n_tiles + tn) * rows_per_tile + row]
// = (max, sum of exp(h - max)) of `row` over its columns, then flags[tm * n_tiles + tn] = stamp.  Stamps are unique per
// launch, so what an earlier launch left in the area never reads as this launch's.
struct CoopLsm {
    float2* partials;
    unsigned long long* flags;
    unsigned long long stamp;
    unsigned int* timeouts;   // incremented by a workgroup whose bounded wait ran out (its rows are then wrong)
    int spin_limit;           // polls of the flags before a workgroup gives up
};

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Eq. 3 of the paper: +1 exactly when v > 0 (0, -0 and NaN give -1, i.e. bit 0).
__device__ __forceinline__ bool sign_bit(float v) { return v > 0.0f; }

// Eq. 1 with the per-layer scale: one fused multiply-add, a single rounding.
__device__ __forceinline__ float affine(float scale, float v, float bias) { return __builtin_fmaf(scale, v, bias); }

__device__ __forceinline__ float hardtanh(float v) {
    v = v > 1.0f ? 1.0f : v;
    v = v < -1.0f ? -1.0f : v;
    return v;
}

// Sigmoid of the paper's real hidden layers (Sec. 3), evaluated in fp64 and rounded once to fp32, as the reference
// definition does: a layer of Sign units that reads these values must see the same fp32 numbers, bit for bit, or a
// unit whose pre-activation is nearly zero flips and every binary layer after it diverges.  (An fp32 exp is within
// 1e-6, which is fine for the values and fatal for the bits.)  Two fp64 exp implementations can differ in the last
// place of the fp64 result; that survives the rounding to fp32 with probability about 2^-29 per value.
__device__ __forceinline__ float sigmoid(float v) { return (float)(1.0 / (1.0 + exp(-(double)v))); }

// +1.0f or -1.0f from bit `pos` of `inv` where inv holds the COMPLEMENT of the weight bits
// (weight bit 1 <=> +1 <=> float sign bit clear).
__device__ __forceinline__ float pm1_from_inverted_bit(uint32_t inv, int pos) {
    const uint32_t s = (inv << (31 - pos)) & 0x80000000u;
    return __uint_as_float(s | 0x3f800000u);
}

}  // namespace bnn
