/*
 * bnn.h - C ABI of the MI355X (gfx950) forward pass for feedforward acoustic
 * models with binary weights and, optionally, binary activations
 * (arXiv 1706.09453, "Toward Computation and Memory Efficient Neural Network
 * Acoustic Models with Binary Weights and Activations").
 *
 * What the library computes, per layer l (paper Eq. 1-2):
 *     h^_l = scale_l * (w^b_l h_{l-1}) + r_l ,   h_l = f_l(h^_l)
 * with w^b_l = Sign(w_l) (Eq. 3: +1 if w > 0, -1 otherwise, so Sign(0) = -1),
 * f_l = Sign for binary hidden activations (Alg. 2 forward), hard-tanh for real
 * hidden activations, and log-Softmax at the last layer (Alg. 2: Softmax at l = L).
 * scale_l = 1 is the paper's layer; a per-layer scale mean|w_l| is what
 * bnn_pack_weights reports.
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer unless marked HOST.  The caller owns all
 *     memory; the library never allocates, frees or keeps a caller pointer.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; they never synchronise.  Results are valid once the
 *     stream has reached the end of the call's work.
 *   - Matrices are row-major and dense.  Weights are [N][K] (N outputs, K inputs),
 *     activations [M][K] (M frames), outputs [M][N].
 *   - Packed rows: element k of a row is bit (k % word_bits) of word (k / word_bits),
 *     least significant bit first, bit 1 <=> +1, words little-endian; a row holds
 *     bnn_packed_words(K, word_bits) words and its pad bits are 0.  Every producer
 *     here writes pad bits as 0 and every consumer assumes they are 0.  A 64-bit
 *     packed row is byte-identical to the 32-bit packed row padded to a multiple of 8 bytes.
 *   - word_bits is 32 or 64.  Packed pointers must be aligned to word_bits/8 bytes, fp32 pointers to 4.
 *   - M and K are at most 2^30 (K < 2^24 for a binary input), N at most 2^22; beyond that: BNN_ESHAPE.
 *   - Calls may be made from several host threads and on several streams at once, as long as their outputs and
 *     workspaces are distinct (inputs and the packed model may be shared): the library keeps no per-call state on
 *     the host or the device.  Two exceptions, each stated at its entry point or option: bnn_forward_static (one
 *     scratch array per device) and BNN_OPT_COOPERATIVE (one such kernel on a device at a time).  Several batches
 *     in flight on several streams is also how the device is used best: a layer launch of a few thousand frames
 *     leaves half of every CU's wave slots free for the launch beside it.
 *   - Output buffers must not overlap input buffers.
 *   - Return value: BNN_OK (0) or a negative bnn_status.  On error nothing has been
 *     enqueued.  M == 0 is valid and does nothing.
 */
#ifndef BNN_H_
#define BNN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bnn_status {
    BNN_OK = 0,
    BNN_EINVAL = -1,     /* null pointer, unknown act / arm, act not allowed for this call, overlapping buffers */
    BNN_ESHAPE = -2,     /* M < 0, K <= 0, N <= 0, word_bits not in {32, 64}, inconsistent layer chain */
    BNN_EALIGN = -3,     /* a packed or fp32 pointer is not aligned as required */
    BNN_EWORKSPACE = -4, /* workspace missing or smaller than bnn_forward_workspace_bytes() */
    BNN_EDEVICE = -5     /* a HIP call failed (launch error) */
} bnn_status;

typedef enum bnn_act {
    BNN_ACT_RAW_I32 = 0,   /* bnn_layer_binw_binx only: int32 product, scale and bias ignored            */
    BNN_ACT_LINEAR = 1,    /* fp32 h^                                                                     */
    BNN_ACT_HARDTANH = 2,  /* fp32 min(1, max(-1, h^))                                                    */
    BNN_ACT_SIGN = 3,      /* packed bits of Sign(h^): bit = (h^ > 0), packed along n                     */
    BNN_ACT_LOGSOFTMAX = 4, /* fp32 log-posteriors: h^ - max_n h^ - log sum_n exp(h^ - max_n h^)          */
    BNN_ACT_SIGMOID = 5     /* fp32 1 / (1 + exp(-h^)): the real hidden layers of the paper's networks (Sec. 3) */
} bnn_act;

/* Which arithmetic unit carries the binary x binary product (same results, different speed). */
typedef enum bnn_binx_arm {
    BNN_ARM_AUTO = 0,      /* the arm measurement showed to be faster for the shape */
    BNN_ARM_VALU_XOR = 1,  /* v_xor + accumulating v_bcnt on packed words (Sec. 2.3 of the paper, literally) */
    BNN_ARM_MFMA = 2,      /* +-1 expanded in registers to the 4-bit float matrix-core operand format (exact)  */
    BNN_ARM_MFMA_I8 = 3    /* +-1 expanded in registers to int8, int8 MFMA with int32 accumulate (comparison)  */
} bnn_binx_arm;

/* Kernel-selection knobs for bnn_set_option (measurement and tuning; results never change, except that
 * BNN_OPT_REALX_F32_MFMA moves fp32 outputs within rounding, as its comment says). */
typedef enum bnn_option {
    BNN_OPT_BINX_ARM = 1,      /* arm used for BNN_ARM_AUTO: BNN_ARM_VALU_XOR, BNN_ARM_MFMA or BNN_ARM_MFMA_I8   */
    BNN_OPT_REALX_TM = 2,      /* real-input vector-ALU kernel: 0 (default) = frames staged through LDS, 16 frames x 4
                                  outputs per lane, where K % 4 == 0 and X is 16-byte aligned; 1, 2, 4, 8, 16 or 32 =
                                  that many frames per wavefront on the row-broadcast kernel.  Same results.        */
    BNN_OPT_BINX_VALU_TM = 3,  /* frames per wavefront of the XOR/popcount kernel: 1, 2, 4, 8, 16 (default) or 32  */
    BNN_OPT_MFMA_WM = 4,       /* 16-row accumulator fragments per wavefront of the matrix-core kernel: 2 or 4  */
    BNN_OPT_REALX_SIGN_MFMA = 5, /* bnn_forward, binary-weight layers real input -> Sign (the first layer of a
                                   binary-activation network; the layer behind a Sigmoid layer in the paper's Table 2
                                   topology): 1 = matrix-core filter with exact sums for the outputs it cannot decide
                                   (default; K <= 8192, scratch from the forward workspace for K > 512 or layers other
                                   than the first: for 128 frames or more a tiled product, 128 frames x 256 outputs per
                                   workgroup, followed by a kernel that sums the undecided outputs; workgroups of 16
                                   frames otherwise), 2 = the same with workgroups of 16 frames for every batch size,
                                   0 = vector-ALU kernel; same bits in all three                                  */
    BNN_OPT_FUSED_LOGSOFTMAX = 6, /* binary-input LOGSOFTMAX layer on the matrix-core arm: 1 = product and
                                   log-Softmax in one kernel (needs K % 256 == 0 and N <= 4096),
                                   0 = product kernel followed by a row kernel (default: measured faster)        */
    BNN_OPT_MFMA_SHAPE = 7,      /* matrix-core arm: 16 = 16x16x128 MFMA (64 x 64 wave tiles), 32 = 32x32x64 MFMA
                                   (128 x 64 wave tiles), 0 = by batch size (32 from 1024 frames; default)       */
    BNN_OPT_MFMA32_WM = 8,       /* 32-row accumulator fragments per wavefront of the 32x32x64 kernel: 2, 4, or 0 =
                                   by grid size (default)                                                        */
    BNN_OPT_MFMA32_XCD_ORDER = 11, /* 32x32x64 kernel: 1 = tiles that share rows of frames run on the same XCD (one L2),
                                   2 = tiles in dispatch order, 0 = by problem size (default)                     */
    BNN_OPT_REALX_F32_MFMA = 10, /* real-input layers with fp32 outputs of 128 frames or more: which of them run on the fp32
                                   matrix-core kernel (about 3x faster; sums in the matrix core's order, within 2e-6 of
                                   the layer's output scale of the ascending-k sum) instead of the vector-ALU kernel
                                   (ascending k, bit-identical to the reference definition): 0 = LOGSOFTMAX layers only
                                   (default: nothing follows them), 1 = LINEAR, HARDTANH and SIGMOID layers too, 2 =
                                   none.  A deep hard-tanh network amplifies the different rounding from layer to layer
                                   (measured: 8e-4 of the output scale after 7 layers of 2048 units), hence the default */
    BNN_OPT_MFMA32_PIPELINE = 9, /* operand fetch of the 32x32x64 kernel on 16-byte aligned rows with K % 512 == 0:
                                   0 or 1 = two register sets, the fetch of the next piece of K pinned ahead of
                                   the products of the current one (default), 2 = one set, order left to the
                                   compiler (kept for comparison)                                                */
    BNN_OPT_STREAM_MAX_FRAMES = 12, /* batches of at most this many frames (streaming; the paper's motivation is on-device,
                                       frame-by-frame inference) run every layer on the vector-ALU kernels with 1 or 2 frames
                                       per workgroup, so that a layer is spread over the whole chip and takes one pass
                                       over its weight rows; 0 = never.  Default 64.  Same results either way.          */
    BNN_OPT_MFMA32_SPLITK = 14,     /* Sign layers on the 128-row 32x32x64 kernel with K % 1024 == 0: 1 = a workgroup of 8
                                       waves, the second four taking the second half of K and handing their sums over
                                       through LDS (two waves per SIMD from a grid of one workgroup per CU); 0 = no
                                       (default: measured 12.4 against 9.9 us at 4096 x 2048 x 2048).  Same bits.       */
    BNN_OPT_REALX_I8_LOGSOFTMAX = 16, /* bnn_forward, LOGSOFTMAX layer with binary weights and real inputs, 128 frames or more,
                                       K <= 8192: 1 = the sum of +-x on the int8 matrix cores from four 7-bit digit planes of
                                       the frames (|sum - exact| < K 2^-27 max|x| per frame: below what the order of an fp32
                                       summation changes; about 3x faster than the fp32 matrix cores; default, unless
                                       BNN_OPT_REALX_F32_MFMA = 2 asks for the ascending-k sum everywhere; a tiled product,
                                       128 frames x 256 outputs per workgroup), 2 = the same sums with workgroups of 16
                                       frames x 512 outputs (identical results), 0 = as BNN_OPT_REALX_F32_MFMA says       */
    BNN_OPT_REALW_SPLIT_LOGSOFTMAX = 17, /* bnn_forward, LOGSOFTMAX layer with real-valued weights, 128 frames or more:
                                       1 = the products run on the bf16 matrix cores with every fp32 operand split into
                                       three bf16 pieces (v = p0 + p1 + p2 to 2^-24 |v|) and the six piece products of
                                       weight 2^-16 or more added in fp32: |sum - exact| <= 2^-22 sum_k |x_k w_k| plus
                                       ordinary fp32 rounding, no more than the fp32 matrix cores give, in half their time
                                       (default, unless BNN_OPT_REALX_F32_MFMA = 2 asks for the ascending-k sum
                                       everywhere); 2 = the same with workgroups of eight waves, two per SIMD (measured
                                       2 % slower); 0 = as BNN_OPT_REALX_F32_MFMA says.  The planes of both operands
                                       (six bytes per element, K padded to 32) are part of bnn_forward_workspace_bytes */
    BNN_OPT_REALW_VALU_LDS = 18,    /* bnn_forward, layer with real-valued weights whose outputs do not go into the
                                       log-Softmax, 512 frames or more, K a multiple of 4, X 16-byte aligned: 1 = the
                                       ascending-k sums on fused multiply-adds with three register operands (frames through
                                       LDS, weights from a transposed copy made once per call: K padded to 64, times N, fp32,
                                       part of bnn_forward_workspace_bytes); 0 = the kernel of bnn_layer_realw.  Same bits
                                       (default 1: 130 against 192 us at 4096 x 440 x 2048)                              */
    BNN_OPT_COOPERATIVE_SPIN = 15,  /* polls of the other workgroups' flags before a workgroup of a cooperative kernel gives
                                       up (>= 1; default 2^20, about a second).  A small value makes the bounded wait run
                                       out on purpose: the kernel still ends, its rows are wrong and
                                       bnn_cooperative_timeouts counts the workgroups that gave up (for tests of that path) */
    BNN_OPT_COOPERATIVE = 13        /* 1 = kernels whose workgroups wait for each other may be used: a binary-input
                                       LOGSOFTMAX layer on the matrix-core arm then finishes its rows inside the product
                                       kernel (the tiles of a row exchange their maxima and sums of exponentials through
                                       memory) instead of running a second kernel over the rows.  Such a kernel needs all its
                                       workgroups resident at once: the library sizes it for an otherwise idle device, so
                                       the caller promises that nothing else runs on that device beside it (one stream, or
                                       streams the caller serialises).  The waits are bounded: a launch that could not
                                       get its workgroups resident ends anyway, with wrong rows, and is counted
                                       (bnn_cooperative_timeouts).  0 = never (default).  Results within the same
                                       tolerance as the two-kernel path (sums of exponentials taken in another order).   */
} bnn_option;

/* One layer of a network for bnn_forward.  HOST struct; the three pointers are DEVICE pointers. */
typedef struct bnn_layer_desc {
    int64_t K;            /* inputs                                                        */
    int64_t N;            /* outputs                                                       */
    int32_t act;          /* bnn_act of this layer (not BNN_ACT_RAW_I32)                   */
    int32_t word_bits;    /* 32 or 64: packing of Wp, of a binary input and of a SIGN output */
    int32_t x_is_binary;  /* 0: input is fp32 [M][K]; 1: packed bits [M][Kw] read as -1/+1;
                             2: packed bits read as 0/1 (see bnn_layer_binw_binx01)            */
    int32_t w_is_real;    /* 0: Wp is packed bits [N][Kw]; 1: the layer keeps real-valued weights (see
                             bnn_layer_realw): Wp is fp32 [N][K] and scale must be NULL      */
    const void* Wp;       /* weights, see w_is_real                                         */
    const float* scale;   /* [N] or NULL (= 1)                                              */
    const float* bias;    /* [N] or NULL (= 0)                                              */
} bnn_layer_desc;

/* ceil(K / word_bits); 0 if K <= 0 or word_bits is not 32 or 64.  HOST helper. */
size_t bnn_packed_words(int64_t K, int word_bits);

/* Static, never-freed description of a status code.  HOST helper. */
const char* bnn_status_string(int status);

/* Set a kernel-selection knob (bnn_option); BNN_EINVAL for an unknown option or value.  HOST helper.
 * The knobs are process-wide state (one atomic integer each, shared by every thread, stream and device): a call takes
 * effect for every layer call that STARTS after it, in any thread.  Setting one while another thread is inside a layer
 * or forward call is safe (no torn state: each entry point reads each knob once per kernel choice) but which of the
 * two values that call sees is unspecified; a multi-layer bnn_forward may then pick its kernels from both.  Results do
 * not depend on the knobs beyond what bnn_option documents; callers that tune set them once, before serving. */
int bnn_set_option(int option, int value);

/* *count = number of workgroups, since the library was loaded, whose bounded wait inside a cooperative kernel
 * (BNN_OPT_COOPERATIVE) ran out on the current device; 0 means every such launch was complete.  Waits for the device to
 * be idle first (hipDeviceSynchronize).  BNN_EINVAL for a NULL pointer, BNN_EDEVICE if the device cannot be read.
 * HOST helper; count is a host pointer. */
int bnn_cooperative_timeouts(uint64_t* count);

/*
 * Binarise real-valued weights (Eq. 3; Alg. 1 forward, first step): Wp[n][k-bit] = (W[n][k] > 0).
 *   W         fp32 [N][K]
 *   Wp        out, words [N][bnn_packed_words(K, word_bits)]
 *   scale_out out, nullable: ONE float = mean over all N*K elements of |W| (fp64 accumulation in a
 *             fixed order, rounded once to fp32; deterministic)
 */
int bnn_pack_weights(const float* W, int64_t N, int64_t K, int word_bits, void* Wp, float* scale_out,
                     void* stream);

/*
 * Binarise activations with the same Sign (Sec. 2.2): Xp[m][k-bit] = (X[m][k] > 0).
 *   X  fp32 [M][K];  Xp out, words [M][bnn_packed_words(K, word_bits)]
 * Inside bnn_forward this step is fused into the producing layer; this call is for standalone use.
 */
int bnn_pack_activations(const float* X, int64_t M, int64_t K, int word_bits, void* Xp, void* stream);

/*
 * One layer with binary weights and REAL input (Alg. 1 forward): the product is a sign-selected
 * add/subtract, acc[m][n] = sum_k (Wp bit ? +X[m][k] : -X[m][k]), accumulated in fp32 in ascending k
 * with one accumulator per output; then h^ = fmaf(scale[n], acc, bias[n]) and the activation.
 *   X [M][K] fp32; Wp [N][Kw]; scale, bias [N] or NULL
 *   act: LINEAR, HARDTANH, SIGMOID, LOGSOFTMAX -> Y fp32 [M][N];  SIGN -> Y words [M][bnn_packed_words(N, word_bits)]
 */
int bnn_layer_binw_realx(const float* X, const void* Wp, const float* scale, const float* bias,
                         int64_t M, int64_t K, int64_t N, int act, int word_bits, void* Y, void* stream);

/*
 * One layer with binary weights and BINARY input (Sec. 2.3): dot[m][n] = sum_k x[m][k] w[n][k] over +-1
 * values = K - 2 * popcount(Xp[m] XOR Wp[n]), exact in int32; then h^ = fmaf(scale[n], (float)dot, bias[n])
 * and the activation.
 *   Xp [M][Kw]; Wp [N][Kw]; K < 2^24
 *   act: RAW_I32 -> Y int32 [M][N] (scale, bias ignored); LINEAR, HARDTANH, SIGMOID, LOGSOFTMAX -> Y fp32 [M][N];
 *        SIGN -> Y words [M][bnn_packed_words(N, word_bits)]
 */
int bnn_layer_binw_binx(const void* Xp, const void* Wp, const float* scale, const float* bias,
                        int64_t M, int64_t K, int64_t N, int act, int word_bits, void* Y, void* stream);

/*
 * As bnn_layer_binw_binx, with the input bits read as 0/1 instead of -1/+1: the activations binarised to (0, 1) of
 * Sec. 3.2 (Tables 3 and 4; the paper calls it the hard version of Sigmoid: 1 where the pre-activation is positive,
 * so the producing layer stores the same bit as Sign and uses BNN_ACT_SIGN).  Weights stay in {-1, +1}:
 * dot[m][n] = sum_k h[m][k] w[n][k] = 2 * popcount(Xp[m] AND Wp[n]) - popcount(Xp[m]), exact in int32.
 * Arguments, outputs and errors as bnn_layer_binw_binx.
 */
int bnn_layer_binw_binx01(const void* Xp, const void* Wp, const float* scale, const float* bias,
                          int64_t M, int64_t K, int64_t N, int act, int word_bits, void* Y, void* stream);

/*
 * One layer that keeps REAL-valued weights (Eq. 1-2; Sec. 2.2, last paragraph, and Sec. 3.1: the paper's systems keep
 * the real-valued weights of the input layer and of the Softmax layer, only the intermediate hidden layers are
 * binarised): acc[m][n] = sum_k W[n][k] X[m][k], then h^ = acc + bias[n] (one rounding) and the activation.
 *   X [M][K] fp32; W [N][K] fp32; bias [N] or NULL
 *   act: LINEAR, HARDTANH, SIGMOID -> Y fp32 [M][N]: the sum is taken in fp32 in ascending k, one fused multiply-add
 *        per step, one accumulator per output (the order of bnn_layer_binw_realx);
 *        SIGN -> Y words [M][bnn_packed_words(N, word_bits)], bits from that same sum;
 *        LOGSOFTMAX -> Y fp32 [M][N]; for M >= 128 the sum is taken on the fp32 matrix cores in their own order
 *        (within ordinary fp32 rounding of the ascending-k sum; BNN_OPT_REALX_F32_MFMA = 2 turns this off, = 1
 *        extends it to LINEAR, HARDTANH and SIGMOID).
 *   word_bits only sets the packing of a SIGN output.
 * Errors as bnn_layer_binw_realx.
 */
int bnn_layer_realw(const float* X, const float* W, const float* bias, int64_t M, int64_t K, int64_t N, int act,
                    int word_bits, void* Y, void* stream);

/*
 * The inverse of bnn_pack_activations for a real-weight layer that follows a binary one: X[m][k] = +1.0 where bit k
 * of row m is set, else -1.0 (zero_one = 0: Sign units, Alg. 2) or 0.0 (zero_one = 1: the (0, 1) units of Sec. 3.2).
 *   Xp words [M][bnn_packed_words(K, word_bits)];  X out, fp32 [M][K]
 */
int bnn_unpack_activations(const void* Xp, int64_t M, int64_t K, int word_bits, int zero_one, float* X, void* stream);

/* As bnn_layer_binw_binx, with the arithmetic unit chosen by the caller (bnn_binx_arm); same results. */
int bnn_layer_binw_binx_arm(const void* Xp, const void* Wp, const float* scale, const float* bias,
                            int64_t M, int64_t K, int64_t N, int act, int word_bits, void* Y, int arm,
                            void* stream);

/*
 * Bytes of scratch bnn_forward needs for M frames: two ping-pong buffers, each large enough for the
 * largest inter-layer activation (packed bits or fp32), each 256-byte aligned, plus a third region: for the bits of a
 * binary layer as fp32 if a real-weight layer reads them, or for the matrix-core filter of a binary-weight layer with
 * real inputs and Sign units (3 bytes per input and frame, 16 bytes per frame; not needed by a first layer of at most
 * 512 inputs), or for the digit planes of a binary-weight LOGSOFTMAX layer with real inputs (4 bytes per input and
 * frame, 16 per frame, from 128 frames on), whichever is larger; with 128 frames or more these two also hold a byte per
 * weight (K padded to 64) and, for Sign units, a record of 32 bytes per frame and 256 outputs; a real-weight layer adds
 * the bf16 pieces of both operands (LOGSOFTMAX, 128 frames or more: 6 bytes per element, K padded to 32) or a
 * transposed copy of its weights (other activations, 512 frames or more: 4 bytes per weight, K padded to 64).
 * 0 on invalid arguments, and for a one-layer network without such a layer.
 * HOST helper; layers is a HOST array.
 */
size_t bnn_forward_workspace_bytes(const bnn_layer_desc* layers, int n_layers, int64_t M);

/*
 * Whole forward pass (Alg. 2 forward with Alg. 1's binary weights): layer 0 reads X, every layer reads the
 * previous layer's output, the last layer writes `out`.
 *   layers    HOST array of n_layers descriptors.  layers[0].x_is_binary says whether X is fp32 [M][K0] or
 *             packed bits; for l > 0, x_is_binary must be nonzero exactly when layers[l-1].act == BNN_ACT_SIGN
 *             (1: the bits are read as -1/+1, 2: as 0/1),
 *             K must equal layers[l-1].N and word_bits must match across a binary link.
 *   X         input of layer 0
 *   out       output of the last layer: fp32 [M][N_last] (log-posteriors when its act is LOGSOFTMAX),
 *             or packed bits when its act is SIGN
 *   workspace DEVICE scratch of at least bnn_forward_workspace_bytes() bytes, 256-byte aligned
 *             (may be NULL when that is 0)
 * A layer with w_is_real = 1 runs as bnn_layer_realw (after bnn_unpack_activations if its input is binary).
 * Enqueues one kernel per layer (two for a LOGSOFTMAX layer or a real-input Sign layer on the slab filter) on `stream`,
 * no host synchronisation.
 */
int bnn_forward(const bnn_layer_desc* layers, int n_layers, const void* X, int64_t M, void* out,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * bnn_forward for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same forward pass with the ping-pong buffers in a fixed
 * BNN_FORWARD_STATIC_MAX_BYTES array inside the library's device image.  Calls no hipMalloc / hipFree or any other
 * allocating routine.  Arguments, results and errors as bnn_forward, except:
 *   - BNN_EWORKSPACE if bnn_forward_workspace_bytes(layers, n_layers, M) exceeds BNN_FORWARD_STATIC_MAX_BYTES
 *     (16 MiB: Config-3-sized networks up to 32768 frames, 4096-unit ones up to 16384; a network with a real-input
 *     Sign layer that is not its first layer, or has more than 512 inputs, also keeps 3 bytes per input and frame of
 *     that layer there: 2048 inputs fit up to about 2600 frames).  The extra scratch of the tiled matrix-core products
 *     (a byte per weight of a real-input layer with binary weights, six bytes per weight of a Softmax layer with real
 *     weights) is left out when it does not fit: those layers then run on the kernels with 16-frame workgroups and on
 *     the fp32 matrix cores, with the results those give in bnn_forward (same bits for Sign layers);
 *   - BNN_EDEVICE if the array's address cannot be obtained on the current device.
 * Every call on a GPU shares that GPU's one array: calls that overlap in time on one GPU (different streams or threads)
 * race on it; calls on one stream are ordered and safe.  Nothing in the array has to be cleared between calls: every
 * layer writes all of its output, pad bits included, before the next layer reads it.
 */
#define BNN_FORWARD_STATIC_MAX_BYTES (16u << 20)
int bnn_forward_static(const bnn_layer_desc* layers, int n_layers, const void* X, int64_t M, void* out, void* stream);

/* ------------------------------------------------------------------------------------------------------------------
 * Training side: backward propagation and update of Alg. 1 (binary weights) and Alg. 2 (binary activations), the
 * gradient-norm clipping of Sec. 2.3 and the semi-stochastic binarisation of Sec. 2.1.  All buffers are DEVICE memory,
 * fp32 unless said otherwise, dense row-major; calls only enqueue on `stream`; errors as above.
 * The paper's layers have no per-layer scale; a caller that uses one multiplies g_hhat by it before the products.
 * ---------------------------------------------------------------------------------------------------------------- */

/* Signs of W^T, packed along n: WpT[k][n / wb] bit (n % wb) = (W[n][k] > 0)  (Eq. 3), the operand of
 * bnn_backward_input_binw.   W [N][K];  WpT out, words [K][bnn_packed_words(N, word_bits)]. */
int bnn_pack_weights_transposed(const float* W, int64_t N, int64_t K, int word_bits, void* WpT, void* stream);

/* out[c][r] = A[r][c].   A [R][C];  out [C][R] (must not overlap A). */
int bnn_transpose_f32(const float* A, int64_t R, int64_t C, float* out, void* stream);

/* Gradient of the cross entropy (Sec. 3), summed over the frames of the minibatch, through the Softmax layer (Alg. 1 and
 * Alg. 2, first backward step at l = L): g[m][n] = exp(logp[m][n]) - (n == labels[m]).
 *   logp [M][N] log-posteriors (the output of a LOGSOFTMAX layer);  labels int32 [M], 0 <= label < N (not checked);
 *   g out [M][N] (may be logp itself). */
int bnn_softmax_xent_grad(const float* logp, const int32_t* labels, int64_t M, int64_t N, float* g, void* stream);

/* Gradient through a binarisation layer (Sec. 2.2, Alg. 2): g_hhat = g_h (.) Mask(hhat, k), Mask = 0 where |hhat| > k,
 * 1 otherwise; k > 0.   g_h, hhat [count];  g_hhat out [count] (may be g_h itself). */
int bnn_mask_grad(const float* g_h, const float* hhat, int64_t count, float k, float* g_hhat, void* stream);

/* Gradient through a Sigmoid layer (Alg. 1, "gradients through f_l"; the real hidden layers of Sec. 3):
 * g_hhat = g_h * (h * (1 - h)), h = the layer's OUTPUT; fp32, each operation rounded.  A hard-tanh layer's derivative is
 * bnn_mask_grad with k = 1 on its pre-activation; a linear layer's is the identity.
 *   g_h, h [count];  g_hhat out [count] (may be g_h itself). */
int bnn_sigmoid_grad(const float* g_h, const float* h, int64_t count, float* g_hhat, void* stream);

/* Alg. 1 backward, g_{h_{l-1}} = g_{hhat_l} w^b_l: g_h[m][k] = sum_n (WpT bit (k, n) ? +g_hhat[m][n] : -g_hhat[m][n]),
 * fp32, ascending n, one accumulator per result (the kernels of bnn_layer_binw_realx on the transposed signs).
 *   g_hhat [M][N];  WpT [K][bnn_packed_words(N, word_bits)] from bnn_pack_weights_transposed;  g_h out [M][K]. */
int bnn_backward_input_binw(const float* g_hhat, const void* WpT, int64_t M, int64_t N, int64_t K, int word_bits,
                            float* g_h, void* stream);

/* The product of bnn_layer_binw_realx with fp32 outputs, Y[m][n] = fma(scale[n], sum_k (Wp bit ? +X[m][k] : -X[m][k]),
 * bias[n]) (Alg. 1 forward; with the roles exchanged also both backward products of Alg. 1 and Alg. 2, see
 * bnn_backward_input_binw and bnn_backward_weight_binh), on the int8 matrix cores: every row of X is scaled by a power of
 * two and rounded to integers of 27 bits, whose sum is exact, so
 *     | sum - exact sum |  <  K max(2^-27 max_k |X[m][k]|, 2^-101)       for every row m
 * (the ascending-k fp32 sum of bnn_layer_binw_realx differs from the exact one by up to (K - 1) 2^-24 sum_k |X[m][k]|).
 * NOT the bits of the ascending-k sum: for gradients and for outputs that feed nothing but a log-Softmax.  Rows holding
 * NaN, Inf or values beyond 2^90 take the ascending-k sum.  About four times faster than bnn_layer_binw_realx at
 * 4096 x 2048 x 2048 (a training step of a 6 x 2048 network on 4096 frames: 8.3 -> 3.2 ms).
 *   X fp32 [M][K];  Wp words [N][bnn_packed_words(K, word_bits)];  scale, bias [N] or NULL;  Y out fp32 [M][N];
 *   K <= 8192 (BNN_ESHAPE beyond);  workspace: DEVICE scratch of at least bnn_layer_binw_realx_i8_workspace_bytes(M, K, N)
 *   bytes, 256-byte aligned, overlapping none of the operands (BNN_EWORKSPACE, BNN_EALIGN, BNN_EINVAL); its contents
 *   mean nothing between calls.  The size helper returns 0 for shapes the call refuses.  HOST helper. */
size_t bnn_layer_binw_realx_i8_workspace_bytes(int64_t M, int64_t K, int64_t N);
int bnn_layer_binw_realx_i8(const float* X, const void* Wp, const float* scale, const float* bias, int64_t M, int64_t K,
                            int64_t N, int word_bits, float* Y, void* workspace, size_t workspace_bytes, void* stream);

/* The same with real-valued weights (Alg. 2, and the layers that keep their weights): g_h[m][k] = sum_n g_hhat[m][n]
 * Wt[k][n], ascending n, one fused multiply-add per step.   Wt [K][N] = the transposed weight matrix (bnn_transpose_f32). */
int bnn_backward_input_realw(const float* g_hhat, const float* Wt, int64_t M, int64_t N, int64_t K, float* g_h,
                             void* stream);

/* Alg. 1 and Alg. 2 backward, g_{w_l} = g_{hhat_l}^T h_{l-1}: g_w[n][k] = sum_m g_hhat_t[n][m] h_t[k][m], fp32, ascending
 * frame m, one fused multiply-add per step (the kernels of bnn_layer_realw).
 *   g_hhat_t [N][M] and h_t [K][M]: the transposed gradient and the transposed input of the layer (bnn_transpose_f32; a
 *   binary input first through bnn_unpack_activations);  g_w out [N][K]. */
int bnn_backward_weight(const float* g_hhat_t, const float* h_t, int64_t N, int64_t K, int64_t M, float* g_w, void* stream);

/* The same gradient when the layer's input is the output of Sign units (Alg. 2: h_{l-1} in {-1, +1}): every product is
 * an add or a subtract, g_w[n][k] = sum_m (HpT bit (k, m) ? +g_hhat_t[n][m] : -g_hhat_t[n][m]), ascending m: the kernels of
 * bnn_layer_binw_realx with the frames as the summed index.  Same results as bnn_backward_weight on the unpacked input.
 *   HpT words [K][bnn_packed_words(M, word_bits)]: the bits of h_{l-1}^T packed along the frames, e.g. from
 *   bnn_pack_weights_transposed(hhat_{l-1}, M, K, ...), since h_{l-1} = Sign(hhat_{l-1}). */
int bnn_backward_weight_binh(const float* g_hhat_t, const void* HpT, int64_t N, int64_t K, int64_t M, int word_bits,
                             float* g_w, void* stream);

/* Alg. 1 and Alg. 2 backward, g_{r_l} = g_{hhat_l} summed over the minibatch: g_r[n] = sum_m g_hhat[m][n], ascending m. */
int bnn_bias_grad(const float* g_hhat, int64_t M, int64_t N, float* g_r, void* stream);

/* Alg. 1 Update: w <- Clip(w - eta g), Clip to [-1, +1] (Sec. 2.1); clip = 0: w <- w - eta g (Alg. 2; the bias).
 * w - eta g is one fused multiply-add.   w in/out [count];  g [count]. */
int bnn_update_clip(float* w, const float* g, int64_t count, float eta, int clip, void* stream);

/* Sec. 2.3: if ||g||_2 > alpha then g <- (alpha / ||g||_2) g; the norm is summed in fp64 in a fixed order.
 *   g in/out [count];  workspace: DEVICE scratch of at least 2048 bytes, 8-byte aligned;
 *   norm_out: DEVICE float that receives ||g||_2 (before clipping). */
int bnn_grad_norm_clip(float* g, int64_t count, float alpha, void* workspace, float* norm_out, void* stream);

/* Sec. 2.1, optional step of Alg. 1's Update (semi-stochastic binarisation): w <- Sign(w) with probability p(|w|),
 * taken as p(|w|) = |w| (the paper gives no formula), the uniform draws in [0, 1) supplied by the caller:
 * w[i] <- Sign(w[i]) where u[i] < |w[i]|.   w in/out [count];  u [count]. */
int bnn_semi_stochastic_binarize(float* w, const float* u, int64_t count, void* stream);

/* After the output layer (Alg. 2, Softmax at l = L), for decoding with a hybrid system as the recipe of Sec. 3 does (the
 * paper's equations end at the Softmax): scaled log-likelihoods log p(x | s) + const = log P(s | x) - log P(s).
 *   logp in/out: DEVICE fp32 [M][N], the log-posteriors bnn_forward wrote;  log_prior: DEVICE fp32 [N], log of each
 *   tied state's prior (the caller's, e.g. from state counts);  logp[m][n] <- logp[m][n] - log_prior[n], one fp32
 *   subtraction.  The two buffers must not overlap (BNN_EINVAL).  M = 0 is a no-op. */
int bnn_subtract_log_prior(float* logp, const float* log_prior, int64_t M, int64_t N, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BNN_H_ */
