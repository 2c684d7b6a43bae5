/*
 * CPU oracle for the forward pass of a feedforward acoustic model with binary
 * (+1/-1) weights and, optionally, binary activations, and for the steps of its
 * backward pass and update (second half of this file and oracle/train_oracle.py).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code, header, table or helper with the
 * HIP path, and the product never calls it: only the tests, the smoke check and
 * the benchmark's CPU-baseline leg may build or load it.
 *
 * Every function states the passage of the paper it follows (arXiv 1706.09453):
 *   Eq. 1-2   layer:  h^_l = w_l h_{l-1} + r_l ,  h_l = f_l(h^_l)
 *   Eq. 3     Sign(w) = +1 if w > 0, -1 otherwise (so Sign(0) = -1)
 *   Alg. 1    forward with binary weights  w^b_l = Sign(w_l)
 *   Alg. 2    forward with binary activations: Sign for l < L, Softmax for l = L
 *   Sec. 2.3  with both binarised the products reduce to XOR operations
 *
 * Readings taken where the paper is silent (also listed in the design notes):
 *   - bit encoding: bit 1 <=> +1; element k of a row lives in word k / wb, bit
 *     k % wb counted from the least significant bit; pad bits are 0;
 *   - per-layer scale alpha = mean|w| multiplies the product only:
 *     h^ = alpha * (w^b h) + r, evaluated as ONE fused multiply-add in fp32;
 *   - a real-input product is accumulated in fp32 in ascending k with one
 *     accumulator per output (the order any output-stationary kernel can keep),
 *     with an fp64 shadow sum for tolerance checks;
 *   - the output layer returns log-Softmax, evaluated in fp64, rounded to fp32.
 *
 * Parity pins (tests/test_oracle_*.py): brute force against numpy's matmul on
 * +-1 floats, the XOR/popcount identity and its closed forms, sign symmetry,
 * numpy's sequential fp32 cumsum, exact rational arithmetic for the fused
 * multiply-add, scipy's fp64 log-softmax, and hand-worked examples under
 * tests/golden/.  The paper prints no worked numeric example, so no pin comes
 * from printed values.
 *
 * Loops over frames carry an OpenMP pragma: frames are independent, the
 * arithmetic inside one frame is untouched.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORC_API __attribute__((visibility("default")))

/* Eq. 3: +1 if v > 0, -1 otherwise.  0, -0 and NaN all fail "v > 0" and give -1. */
static inline int sign_pm1(float v) { return (v > 0.0f) ? 1 : -1; }

/* Words per packed row: ceil(K / word_bits). */
ORC_API int64_t orc_words_per_row(int64_t K, int word_bits) { return (K + word_bits - 1) / word_bits; }

/*
 * Eq. 3 applied elementwise, then the storage reading: element k -> word k/wb,
 * bit k%wb (LSB first), bit = 1 for +1.  rows x K floats -> rows x Kw words.
 */
ORC_API void orc_pack_sign(const float* x, int64_t rows, int64_t K, int word_bits, void* out) {
    const int64_t Kw = orc_words_per_row(K, word_bits);
    if (word_bits == 32) {
        uint32_t* o = (uint32_t*)out;
        memset(o, 0, (size_t)(rows * Kw) * sizeof(uint32_t));
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t k = 0; k < K; ++k)
                if (sign_pm1(x[r * K + k]) == 1) o[r * Kw + k / 32] |= (uint32_t)1 << (k % 32);
    } else {
        uint64_t* o = (uint64_t*)out;
        memset(o, 0, (size_t)(rows * Kw) * sizeof(uint64_t));
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t k = 0; k < K; ++k)
                if (sign_pm1(x[r * K + k]) == 1) o[r * Kw + k / 64] |= (uint64_t)1 << (k % 64);
    }
}

/* Inverse of the storage reading: packed rows -> +1/-1 as int8, rows x K. */
ORC_API void orc_unpack_pm1(const void* words, int64_t rows, int64_t K, int word_bits, int8_t* out) {
    const int64_t Kw = orc_words_per_row(K, word_bits);
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            int bit;
            if (word_bits == 32) bit = (int)((((const uint32_t*)words)[r * Kw + k / 32] >> (k % 32)) & 1u);
            else                 bit = (int)((((const uint64_t*)words)[r * Kw + k / 64] >> (k % 64)) & 1u);
            out[r * K + k] = bit ? 1 : -1;
        }
}

/* Per-layer scale: mean of |w| over the real-valued weights, fp64 running sum in index order. */
ORC_API float orc_mean_abs(const float* w, int64_t count) {
    double s = 0.0;
    for (int64_t i = 0; i < count; ++i) s += fabs((double)w[i]);
    return (float)(s / (double)count);
}

/*
 * Eq. 1 with both operands in {-1,+1}: dot[m][n] = sum_k a[m][k] * b[n][k].
 * The plain definition, exact in int32.
 */
ORC_API void orc_dot_pm1(const int8_t* a, const int8_t* b, int64_t M, int64_t N, int64_t K, int32_t* dot) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)a[m * K + k] * (int32_t)b[n * K + k];
            dot[m * N + n] = s;
        }
}

/*
 * Sec. 2.3: the same product on packed rows.  Equal bits multiply to +1 and
 * differing bits to -1, so dot = (K - d) - d with d = popcount(a XOR b);
 * zero pad bits are equal in both operands and add nothing to d.
 */
ORC_API void orc_dot_xor(const void* a, const void* b, int64_t M, int64_t N, int64_t K, int word_bits,
                         int32_t* dot) {
    const int64_t Kw = orc_words_per_row(K, word_bits);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t d = 0;
            if (word_bits == 32) {
                const uint32_t* ar = (const uint32_t*)a + m * Kw;
                const uint32_t* br = (const uint32_t*)b + n * Kw;
                for (int64_t w = 0; w < Kw; ++w) d += __builtin_popcount(ar[w] ^ br[w]);
            } else {
                const uint64_t* ar = (const uint64_t*)a + m * Kw;
                const uint64_t* br = (const uint64_t*)b + n * Kw;
                for (int64_t w = 0; w < Kw; ++w) d += __builtin_popcountll(ar[w] ^ br[w]);
            }
            dot[m * N + n] = (int32_t)(K - 2 * d);
        }
}

/*
 * Activations binarised to (0, 1) instead of (-1, +1) (Sec. 2.1 remark; Sec. 3.2, Tables 3 and 4): the weights stay in
 * {-1, +1}, the activation is h = 1 where the pre-activation is positive and 0 otherwise, so the stored bit is the
 * same and only the product reads it differently: dot[m][n] = sum_k h[m][k] * w[n][k].  The plain definition.
 */
ORC_API void orc_dot_x01_wpm1(const int8_t* h01, const int8_t* wpm1, int64_t M, int64_t N, int64_t K, int32_t* dot) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)h01[m * K + k] * (int32_t)wpm1[n * K + k];
            dot[m * N + n] = s;
        }
}

/*
 * The same product on packed rows: an element adds +1 where activation and weight bit are both 1 and -1 where the
 * activation bit is 1 and the weight bit 0, so dot = popcount(h AND w) - popcount(h AND NOT w)
 *                                                  = 2 popcount(h AND w) - popcount(h).  Zero pad bits add nothing.
 */
ORC_API void orc_dot_and(const void* h, const void* w, int64_t M, int64_t N, int64_t K, int word_bits, int32_t* dot) {
    const int64_t Kw = orc_words_per_row(K, word_bits);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t both = 0, ones = 0;
            if (word_bits == 32) {
                const uint32_t* hr = (const uint32_t*)h + m * Kw;
                const uint32_t* wr = (const uint32_t*)w + n * Kw;
                for (int64_t i = 0; i < Kw; ++i) { both += __builtin_popcount(hr[i] & wr[i]); ones += __builtin_popcount(hr[i]); }
            } else {
                const uint64_t* hr = (const uint64_t*)h + m * Kw;
                const uint64_t* wr = (const uint64_t*)w + n * Kw;
                for (int64_t i = 0; i < Kw; ++i) { both += __builtin_popcountll(hr[i] & wr[i]); ones += __builtin_popcountll(hr[i]); }
            }
            dot[m * N + n] = (int32_t)(2 * both - ones);
        }
}

/*
 * Alg. 1 forward, product term with real input: acc[m][n] = sum_k w^b[n][k] * x[m][k],
 * which is an add where w^b = +1 and a subtract where w^b = -1 (no multiplications).
 * acc32: fp32, k ascending, one accumulator, every add/sub rounded to nearest.
 * acc64: the same sum carried in fp64 (reference for tolerance checks).
 */
ORC_API void orc_realx_acc(const float* x, const int8_t* wpm1, int64_t M, int64_t N, int64_t K,
                           float* acc32, double* acc64) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float s32 = 0.0f; /* built without fast-math or contraction: the order below is the order executed */
            double s64 = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const float v = x[m * K + k];
                if (wpm1[n * K + k] > 0) { s32 = s32 + v; s64 += (double)v; }
                else                     { s32 = s32 - v; s64 -= (double)v; }
            }
            if (acc32) acc32[m * N + n] = s32;
            if (acc64) acc64[m * N + n] = s64;
        }
}

/*
 * Eq. 1 for a layer whose weights stay real-valued (Sec. 2.2, last paragraph, and Sec. 3.1: the input layer and the
 * Softmax layer of the paper's systems keep the real-valued weights of the model they were initialised from):
 * acc[m][n] = sum_k w[n][k] * x[m][k].  Reading: fp32, ascending k, one accumulator per output, each step ONE fused
 * multiply-add (a single rounding per step), the same order as the binary-weight product above, to which it
 * reduces bit for bit when every w is +1 or -1.  acc64 is the fp64 shadow sum (every product of two fp32 numbers
 * is exact in fp64).
 */
ORC_API void orc_realw_acc(const float* x, const float* w, int64_t M, int64_t N, int64_t K,
                           float* acc32, double* acc64) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float s32 = 0.0f;
            double s64 = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                s32 = fmaf(w[n * K + k], x[m * K + k], s32);
                s64 += (double)w[n * K + k] * (double)x[m * K + k];
            }
            if (acc32) acc32[m * N + n] = s32;
            if (acc64) acc64[m * N + n] = s64;
        }
}

/* Bits of a binary hidden layer as the real numbers the next, real-weight layer multiplies: bit 1 -> +1.0, bit 0 ->
 * -1.0 (Sign units, Alg. 2) or bit 1 -> 1.0, bit 0 -> 0.0 (the (0, 1) units of Sec. 3.2). */
ORC_API void orc_bits_to_real(const void* words, int64_t M, int64_t K, int word_bits, int zero_one, float* out) {
    const int64_t Kw = (K + word_bits - 1) / word_bits;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            uint64_t word;
            if (word_bits == 64) word = ((const uint64_t*)words)[m * Kw + k / 64];
            else                 word = ((const uint32_t*)words)[m * Kw + k / 32];
            const int bit = (int)((word >> (k % word_bits)) & 1u);
            out[m * K + k] = bit ? 1.0f : (zero_one ? 0.0f : -1.0f);
        }
}

/* ---------------------------------------------------------------------------------------------------------------
 * Training side (Alg. 1 and Alg. 2, backward propagation and update; Sec. 2.1-2.3).  The two matrix products of the
 * backward pass, g_{h_{l-1}} = g_{h^_l} w_l^b and g_{w_l} = g_{h^_l} h_{l-1}, are the products above with the operands'
 * roles exchanged (orc_realx_acc with the transposed weight signs, orc_realw_acc with both operands transposed), so
 * they are composed in oracle/train_oracle.py; what follows are the remaining steps.
 * ------------------------------------------------------------------------------------------------------------- */

/* Alg. 1/2 backward, g_{r_l} = g_{h^_l} summed over the frames of the minibatch: out[n] = sum_m g[m][n], fp32,
 * ascending m, one accumulator per output (reading: the same order rule as every other sum here). */
ORC_API void orc_colsum_f32(const float* g, int64_t M, int64_t N, float* out) {
    for (int64_t n = 0; n < N; ++n) {
        float s = 0.0f;
        for (int64_t m = 0; m < M; ++m) s = s + g[m * N + n];
        out[n] = s;
    }
}

/* Alg. 1 Update: w <- Clip(w - eta g) (Clip of Sec. 2.1: to [-1, +1]); with clip == 0 the plain update of Alg. 2 and
 * of the bias.  w - eta g is ONE fused multiply-add in fp32. */
ORC_API void orc_update_clip(float* w, const float* g, int64_t count, float eta, int clip) {
    for (int64_t i = 0; i < count; ++i) {
        float v = fmaf(-eta, g[i], w[i]);
        if (clip) {
            if (v > 1.0f) v = 1.0f;
            if (v < -1.0f) v = -1.0f;
        }
        w[i] = v;
    }
}

/* Sec. 2.3, gradient-norm clipping: the squared l2 norm of a gradient matrix, fp64 running sum in index order. */
ORC_API double orc_sumsq_f64(const float* g, int64_t count) {
    double s = 0.0;
    for (int64_t i = 0; i < count; ++i) s += (double)g[i] * (double)g[i];
    return s;
}

/*
 * Eq. 1 with the per-layer scale: h^[m][n] = scale[n] * v[m][n] + bias[n] as one
 * fp32 fused multiply-add (single rounding).  scale == NULL means 1, bias == NULL means 0.
 */
ORC_API void orc_affine_f32(const float* v, const float* scale, const float* bias, int64_t M, int64_t N,
                            float* hhat) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            hhat[m * N + n] = fmaf(scale ? scale[n] : 1.0f, v[m * N + n], bias ? bias[n] : 0.0f);
}

/* The same affine map carried in fp64 from an fp64 product (tolerance reference, not a parity definition). */
ORC_API void orc_affine_f64(const double* v, const float* scale, const float* bias, int64_t M, int64_t N,
                            double* hhat) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            hhat[m * N + n] = (double)(scale ? scale[n] : 1.0f) * v[m * N + n] + (double)(bias ? bias[n] : 0.0f);
}

/* int32 -> fp32, exact for |dot| < 2^24. */
ORC_API void orc_i32_to_f32(const int32_t* dot, int64_t count, float* out) {
    for (int64_t i = 0; i < count; ++i) out[i] = (float)dot[i];
}

/* Real hidden nonlinearity of the real-activation configuration: clip to [-1, 1]. */
ORC_API void orc_hardtanh(const float* hhat, int64_t count, float* out) {
    for (int64_t i = 0; i < count; ++i) {
        float v = hhat[i];
        if (v > 1.0f) v = 1.0f;
        if (v < -1.0f) v = -1.0f;
        out[i] = v;
    }
}

/*
 * The real hidden nonlinearity of the paper's own networks (Sec. 3: Sigmoid hidden layers in the baselines and in the
 * first and last hidden layer of the binary-activation systems, Table 2): sigma(v) = 1 / (1 + exp(-v)), evaluated in
 * fp64 from the fp32 pre-activation and rounded to fp32.
 */
ORC_API void orc_sigmoid(const float* hhat, int64_t count, float* out) {
    for (int64_t i = 0; i < count; ++i) out[i] = (float)(1.0 / (1.0 + exp(-(double)hhat[i])));
}

/*
 * Alg. 2, last layer: Softmax over the N outputs of each frame, returned as
 * log-posteriors: logp[n] = z[n] - max_j z[j] - log sum_j exp(z[j] - max_j z[j]).
 * Evaluated in fp64 from the fp32 pre-activations; result kept in fp64 and also rounded to fp32.
 */
ORC_API void orc_log_softmax(const float* z, int64_t M, int64_t N, float* out32, double* out64) {
    for (int64_t m = 0; m < M; ++m) {
        const float* zr = z + m * N;
        double mx = (double)zr[0];
        for (int64_t n = 1; n < N; ++n) if ((double)zr[n] > mx) mx = (double)zr[n];
        double s = 0.0;
        for (int64_t n = 0; n < N; ++n) s += exp((double)zr[n] - mx);
        const double lse = log(s);
        for (int64_t n = 0; n < N; ++n) {
            const double v = (double)zr[n] - mx - lse;
            if (out64) out64[m * N + n] = v;
            if (out32) out32[m * N + n] = (float)v;
        }
    }
}
