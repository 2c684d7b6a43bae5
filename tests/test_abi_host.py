"""Host-side checks of the C-ABI library that need no GPU: exported symbols and argument validation.

Every call below is rejected by the library's own checks before any HIP call is made
(the pointers are made-up addresses that are never dereferenced).
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bnn.h")


@pytest.fixture(scope="module")
def bnn():
    import paper_1706_09453_amd as b
    return b


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(bnn_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(bnn):
    names = _declared_functions()
    for required in ("bnn_pack_weights", "bnn_pack_activations", "bnn_layer_binw_realx", "bnn_layer_binw_binx",
                     "bnn_forward"):
        assert required in names
    lib = ctypes.CDLL(bnn.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/bnn.h but not exported"
    assert set(bnn.EXPORTED) == set(names), "the Python binding mirrors the header one to one"


def test_packed_words(bnn):
    assert bnn.bnn_packed_words(440, 32) == 14 and bnn.bnn_packed_words(440, 64) == 7
    assert bnn.bnn_packed_words(2048, 32) == 64 and bnn.bnn_packed_words(1, 64) == 1
    assert bnn.bnn_packed_words(0, 32) == 0 and bnn.bnn_packed_words(64, 16) == 0


def test_status_strings(bnn):
    seen = {bnn.bnn_status_string(s) for s in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6 and bnn.bnn_status_string(-99) == "unknown status"


P = 0x10000   # fake, 64 KiB-aligned "device pointers" far apart from each other
Q = 0x900000
R = 0x1200000


def _status(fn, *a):
    with pytest.raises(Exception) as e:
        fn(*a)
    return e.value.status


def test_layer_argument_validation(bnn):
    S, L = bnn.BNN_ACT_SIGN, bnn.BNN_ACT_LINEAR
    for fn in (bnn.bnn_layer_binw_realx, bnn.bnn_layer_binw_binx):
        assert _status(fn, 0, Q, 0, 0, 4, 64, 64, S, 32, R, 0) == bnn.BNN_EINVAL        # null X
        assert _status(fn, P, 0, 0, 0, 4, 64, 64, S, 32, R, 0) == bnn.BNN_EINVAL        # null Wp
        assert _status(fn, P, Q, 0, 0, 4, 64, 64, S, 32, 0, 0) == bnn.BNN_EINVAL        # null Y
        assert _status(fn, P, Q, 0, 0, -1, 64, 64, S, 32, R, 0) == bnn.BNN_ESHAPE       # M < 0
        assert _status(fn, P, Q, 0, 0, 4, 0, 64, S, 32, R, 0) == bnn.BNN_ESHAPE         # K = 0
        assert _status(fn, P, Q, 0, 0, 4, 64, 0, S, 32, R, 0) == bnn.BNN_ESHAPE         # N = 0
        assert _status(fn, P, Q, 0, 0, 4, 64, 64, S, 16, R, 0) == bnn.BNN_ESHAPE        # word_bits
        assert _status(fn, P, Q, 0, 0, 4, 64, (1 << 22) + 1, S, 32, R, 0) == bnn.BNN_ESHAPE   # N beyond the grid's reach
        assert _status(fn, P, Q, 0, 0, (1 << 30) + 1, 64, 64, S, 32, R, 0) == bnn.BNN_ESHAPE  # M beyond 2^30
        assert _status(fn, P, Q, 0, 0, 4, 64, 64, 9, 32, R, 0) == bnn.BNN_EINVAL        # unknown act
        assert _status(fn, P, Q + 4, 0, 0, 4, 64, 64, S, 64, R, 0) == bnn.BNN_EALIGN    # 64-bit words at 4 mod 8
        assert _status(fn, P, Q, 0, 0, 4, 64, 64, L, 32, R + 2, 0) == bnn.BNN_EALIGN    # fp32 out at 2 mod 4
        assert _status(fn, P, Q, 0, 0, 4, 64, 64, L, 32, P, 0) == bnn.BNN_EINVAL        # Y aliases X
        assert _status(fn, P, Q, 0, 0, 4, 64, 64, L, 32, Q + 8, 0) == bnn.BNN_EINVAL    # Y overlaps Wp
    assert _status(bnn.bnn_layer_binw_realx, P, Q, 0, 0, 4, 64, 64, bnn.BNN_ACT_RAW_I32, 32, R, 0) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_layer_binw_binx, P, Q, 0, 0, 4, 1 << 24, 64, S, 32, R, 0) == bnn.BNN_ESHAPE
    assert _status(bnn.bnn_layer_binw_binx_arm, P, Q, 0, 0, 4, 64, 64, S, 32, R, 7, 0) == bnn.BNN_EINVAL


def test_real_weight_layer_argument_validation(bnn):
    S, L = bnn.BNN_ACT_SIGN, bnn.BNN_ACT_LINEAR
    fn = bnn.bnn_layer_realw
    assert _status(fn, 0, Q, 0, 4, 64, 64, L, 32, R, 0) == bnn.BNN_EINVAL            # null X
    assert _status(fn, P, 0, 0, 4, 64, 64, L, 32, R, 0) == bnn.BNN_EINVAL            # null W
    assert _status(fn, P, Q, 0, 4, 64, 64, L, 32, 0, 0) == bnn.BNN_EINVAL            # null Y
    assert _status(fn, P, Q, 0, -1, 64, 64, L, 32, R, 0) == bnn.BNN_ESHAPE           # M < 0
    assert _status(fn, P, Q, 0, 4, 0, 64, L, 32, R, 0) == bnn.BNN_ESHAPE             # K = 0
    assert _status(fn, P, Q, 0, 4, 64, 64, S, 48, R, 0) == bnn.BNN_ESHAPE            # word_bits of the Sign output
    assert _status(fn, P, Q, 0, 4, 64, 64, bnn.BNN_ACT_RAW_I32, 32, R, 0) == bnn.BNN_EINVAL
    assert _status(fn, P, Q + 2, 0, 4, 64, 64, L, 32, R, 0) == bnn.BNN_EALIGN        # fp32 weights at 2 mod 4
    assert _status(fn, P, Q, 0, 4, 64, 64, L, 32, Q + 64 * 64 * 4 - 4, 0) == bnn.BNN_EINVAL   # Y overlaps the fp32 weights
    assert bnn.bnn_layer_realw(0, 0, 0, 0, 64, 64, L, 32, 0, 0) == 0                 # M = 0: nothing to do
    un = bnn.bnn_unpack_activations
    assert _status(un, 0, 4, 64, 32, 0, R, 0) == bnn.BNN_EINVAL                      # null Xp
    assert _status(un, P, 4, 64, 32, 0, 0, 0) == bnn.BNN_EINVAL                      # null X
    assert _status(un, P, 4, 64, 32, 2, R, 0) == bnn.BNN_EINVAL                      # zero_one not 0 or 1
    assert _status(un, P, 4, 0, 32, 0, R, 0) == bnn.BNN_ESHAPE
    assert _status(un, P, 4, 64, 16, 0, R, 0) == bnn.BNN_ESHAPE
    assert _status(un, P + 4, 4, 64, 64, 0, R, 0) == bnn.BNN_EALIGN
    assert _status(un, P, 4, 64, 32, 0, P + 8, 0) == bnn.BNN_EINVAL                  # output overlaps the bits
    assert un(0, 0, 64, 32, 0, 0, 0) == 0


def test_real_weight_layers_in_a_chain(bnn):
    S, G, Z = bnn.BNN_ACT_SIGN, bnn.BNN_ACT_SIGMOID, bnn.BNN_ACT_LOGSOFTMAX
    d = _chain(bnn, (440, 2048, 2048, 3400), (G, S, Z))
    d[0]["w_is_real"] = 1
    d[2]["w_is_real"] = 1          # reads the bits of layer 2: the third region holds them as 4096 x 2048 fp32, and
    arr = bnn.make_layer_array(d)  # behind them three bf16 planes of the frames and of the 3400 weight rows
    planes = 3 * 2 * 2048 * (4096 + 3400)
    assert bnn.bnn_forward_workspace_bytes(arr, 3, 4096) == 2 * 4096 * 2048 * 4 + 4096 * 2048 * 4 + planes
    # fewer than 128 frames: no matrix-core Softmax layer, no planes (the first two regions: 64 x 2048 fp32 each)
    assert bnn.bnn_forward_workspace_bytes(arr, 3, 64) == 2 * 64 * 2048 * 4 + 64 * 2048 * 4
    # a real-weight layer that is not the Softmax layer, 512 frames or more: its weights transposed (K padded to 64)
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d[:1]), 1, 4096) == 448 * 2048 * 4
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d[:1]), 1, 511) == 0
    d[2]["w_is_real"] = 0
    # layer 2 reads 2048 real inputs and has Sign units: the third region then holds the scratch of its matrix-core
    # filter instead.  128 frames or more (the tiled product): three digit bytes per input and frame, one byte per
    # weight, 16 bytes per frame, and a record of 32 bytes per frame and tile of 256 outputs for the undecided ones
    pingpong = 2 * 4096 * 2048 * 4
    sign_scratch = 3 * 4096 * 2048 + 2048 * 2048 + 4096 * 16 + 32 * 4096 * (2048 // 256)
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d), 3, 4096) == pingpong + sign_scratch
    # fewer than 128 frames (workgroups of 16 frames): three digit bytes per input and frame plus 16 bytes per frame
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d), 3, 64) == 2 * 64 * 2048 * 4 + 3 * 64 * 2048 + 64 * 16
    d[1]["act"] = G                # no Sign layer behind real inputs, but a binary-weight output layer that reads real
    d[2]["x_is_binary"] = 0        # inputs: four digit bytes per input and frame, one byte per weight, 16 bytes per frame
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d), 3, 4096) == pingpong + 4 * 4096 * 2048 + 3400 * 2048 + 4096 * 16
    d[2]["w_is_real"] = 1          # real weights there: the planes of both operands only
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d), 3, 4096) == 2 * 4096 * 2048 * 4 + planes
    d[2]["K"], d[1]["N"] = 2041, 2041   # K is padded to a multiple of 32 in the planes (2041 -> 2048), rows to 256 bytes
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d), 3, 4096) == 2 * 4096 * 2048 * 4 + planes
    d[2]["K"], d[1]["N"] = 2048, 2048
    d[2]["w_is_real"] = 2
    assert _status(bnn.bnn_forward, bnn.make_layer_array(d), 3, P, 8, R, 0x4000000, 1 << 26, 0) == bnn.BNN_EINVAL
    d[2]["w_is_real"] = 1
    d[2]["scale"] = Q               # a real-weight layer has no scale
    assert _status(bnn.bnn_forward, bnn.make_layer_array(d), 3, P, 8, R, 0x4000000, 1 << 26, 0) == bnn.BNN_EINVAL
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d), 3, 4096) == 0


def test_int8_layer_argument_validation(bnn):
    fn, size = bnn.bnn_layer_binw_realx_i8, bnn.bnn_layer_binw_realx_i8_workspace_bytes
    # four digit bytes per input and frame, one byte per weight (K padded to 64), 16 bytes per frame
    assert size(4096, 2048, 3400) == 4 * 4096 * 2048 + 3400 * 2048 + 4096 * 16
    assert size(3, 5, 7) == 4 * 3 * 64 + (7 * 64 + 255) // 256 * 256 + 256
    assert size(4, 8193, 7) == 0 and size(0, 8, 8) == 0 and size(4, 0, 8) == 0
    W = 0x40000000
    need = size(4, 64, 64)
    assert _status(fn, 0, Q, 0, 0, 4, 64, 64, 32, R, W, need, 0) == bnn.BNN_EINVAL        # null X
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 32, 0, W, need, 0) == bnn.BNN_EINVAL        # null Y
    assert _status(fn, P, Q, 0, 0, 4, 8193, 64, 32, R, W, 1 << 30, 0) == bnn.BNN_ESHAPE   # K beyond 8192
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 48, R, W, need, 0) == bnn.BNN_ESHAPE        # word_bits
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 32, R, 0, need, 0) == bnn.BNN_EWORKSPACE    # no workspace
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 32, R, W, need - 1, 0) == bnn.BNN_EWORKSPACE
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 32, R, W + 128, need, 0) == bnn.BNN_EALIGN  # workspace at 128 mod 256
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 32, R + 2, W, need, 0) == bnn.BNN_EALIGN    # fp32 out at 2 mod 4
    assert _status(fn, P, Q, 0, 0, 4, 64, 64, 32, W + 256, W, need, 0) == bnn.BNN_EINVAL  # Y inside the workspace
    assert _status(fn, W, Q, 0, 0, 4, 64, 64, 32, R, W, need, 0) == bnn.BNN_EINVAL        # X inside the workspace
    assert fn(0, 0, 0, 0, 0, 64, 64, 32, 0, 0, 0, 0) == 0                                  # M = 0: nothing to do


def test_training_argument_validation(bnn):
    E, S, A = bnn.BNN_EINVAL, bnn.BNN_ESHAPE, bnn.BNN_EALIGN
    assert _status(bnn.bnn_pack_weights_transposed, 0, 4, 64, 32, Q, 0) == E
    assert _status(bnn.bnn_pack_weights_transposed, P, 0, 64, 32, Q, 0) == S
    assert _status(bnn.bnn_pack_weights_transposed, P, 4, 64, 48, Q, 0) == S
    assert _status(bnn.bnn_pack_weights_transposed, P, 4, 64, 64, Q + 4, 0) == A
    assert _status(bnn.bnn_transpose_f32, P, 4, 0, Q, 0) == S
    assert _status(bnn.bnn_transpose_f32, P, 4, 64, 0, 0) == E
    assert _status(bnn.bnn_transpose_f32, P, 4, 64, P + 16, 0) == E                 # overlapping
    assert _status(bnn.bnn_softmax_xent_grad, P, 0, 4, 64, R, 0) == E                # null labels
    assert _status(bnn.bnn_softmax_xent_grad, P, Q, 4, 0, R, 0) == S
    assert bnn.bnn_softmax_xent_grad(0, 0, 0, 64, 0, 0) == 0                          # no frames: nothing to do
    assert _status(bnn.bnn_mask_grad, P, Q, 16, 0.0, R, 0) == E                      # k must be positive
    assert _status(bnn.bnn_mask_grad, P, Q, -1, 1.0, R, 0) == S
    assert _status(bnn.bnn_mask_grad, P, 0, 16, 1.0, R, 0) == E
    assert _status(bnn.bnn_sigmoid_grad, P, 0, 16, R, 0) == E
    assert _status(bnn.bnn_sigmoid_grad, P, Q, -2, R, 0) == S
    assert _status(bnn.bnn_backward_input_binw, P, 0, 4, 64, 64, 32, R, 0) == E
    assert _status(bnn.bnn_backward_input_binw, P, Q, 4, 64, 64, 16, R, 0) == S
    assert _status(bnn.bnn_backward_input_realw, P, Q + 2, 4, 64, 64, R, 0) == A
    assert _status(bnn.bnn_backward_weight, P, Q, 64, 64, 0, R, 0) == S              # an empty minibatch has no gradient
    assert _status(bnn.bnn_backward_weight, P, Q, 64, 64, 8, P, 0) == E              # output aliases an operand
    assert _status(bnn.bnn_bias_grad, 0, 4, 64, R, 0) == E
    assert _status(bnn.bnn_update_clip, P, Q, 16, 0.1, 2, 0) == E                    # clip is 0 or 1
    assert _status(bnn.bnn_update_clip, P, P, 16, 0.1, 1, 0) == E                    # w and g overlap
    assert bnn.bnn_update_clip(0, 0, 0, 0.1, 1, 0) == 0
    assert _status(bnn.bnn_grad_norm_clip, P, 16, 0.0, Q, R, 0) == E                 # alpha must be positive
    assert _status(bnn.bnn_grad_norm_clip, P, 16, 15.0, 0, R, 0) == E                # no workspace
    assert _status(bnn.bnn_grad_norm_clip, P, 16, 15.0, Q + 4, R, 0) == A
    assert _status(bnn.bnn_subtract_log_prior, 0, P, 4, 8, 0) == E                   # null log-posteriors
    assert _status(bnn.bnn_subtract_log_prior, P, 0, 4, 8, 0) == E                   # null priors
    assert _status(bnn.bnn_subtract_log_prior, P, P + 64, 4, 8, 0) == E              # the priors inside the output
    assert _status(bnn.bnn_subtract_log_prior, P, Q, 4, 0, 0) == bnn.BNN_ESHAPE
    assert _status(bnn.bnn_subtract_log_prior, P, Q, -1, 8, 0) == bnn.BNN_ESHAPE
    assert _status(bnn.bnn_subtract_log_prior, P + 2, Q, 4, 8, 0) == bnn.BNN_EALIGN
    assert bnn.bnn_subtract_log_prior(0, 0, 0, 8, 0) == 0                            # no frames: nothing to do
    assert _status(bnn.bnn_semi_stochastic_binarize, P, 0, 16, 0) == E
    assert _status(bnn.bnn_semi_stochastic_binarize, P, P + 8, 16, 0) == E


def test_pack_argument_validation(bnn):
    assert _status(bnn.bnn_pack_weights, 0, 4, 64, 32, Q, 0, 0) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_pack_weights, P, 0, 64, 32, Q, 0, 0) == bnn.BNN_ESHAPE
    assert _status(bnn.bnn_pack_weights, P, 4, 64, 48, Q, 0, 0) == bnn.BNN_ESHAPE
    assert _status(bnn.bnn_pack_weights, P, 4, 64, 64, Q + 4, 0, 0) == bnn.BNN_EALIGN
    assert _status(bnn.bnn_pack_weights, P, 4, 64, 32, P + 16, 0, 0) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_pack_activations, P, 4, 64, 32, 0, 0) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_pack_activations, P, -4, 64, 32, Q, 0) == bnn.BNN_ESHAPE
    assert bnn.bnn_pack_activations(0, 0, 64, 32, 0, 0) == 0                               # M = 0: nothing to do


def test_set_option_validation(bnn):
    assert _status(bnn.bnn_set_option, 99, 1) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_set_option, bnn.BNN_OPT_REALX_TM, 5) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_set_option, bnn.BNN_OPT_BINX_ARM, 0) == bnn.BNN_EINVAL
    assert bnn.bnn_set_option(bnn.BNN_OPT_BINX_ARM, bnn.BNN_ARM_MFMA) == 0
    assert bnn.bnn_set_option(bnn.BNN_OPT_REALX_TM, 0) == 0


def _chain(bnn, dims, acts, wb=32, first_binary=False, Wp=Q):
    descs, binary = [], first_binary
    for (K, N), a in zip(zip(dims[:-1], dims[1:]), acts):
        descs.append(dict(K=K, N=N, act=a, word_bits=wb, x_is_binary=binary, Wp=Wp, scale=0, bias=0))
        binary = a == bnn.BNN_ACT_SIGN
    return descs


def test_forward_chain_validation_and_workspace(bnn):
    S, H, Z = bnn.BNN_ACT_SIGN, bnn.BNN_ACT_HARDTANH, bnn.BNN_ACT_LOGSOFTMAX
    d = _chain(bnn, (440, 2048, 2048, 3400), (S, S, Z))
    arr = bnn.make_layer_array(d)
    # two ping-pong buffers of 4096 x 2048 bits = 1 MiB each
    assert bnn.bnn_forward_workspace_bytes(arr, 3, 4096) == 2 * 4096 * 256
    binfirst = _chain(bnn, (2048, 2048, 3400), (S, Z), first_binary=True)
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(binfirst), 2, 4096) == 2 * 4096 * 256
    d2 = _chain(bnn, (440, 2048, 2048, 3400), (H, H, Z))
    # two buffers of 4096 x 2048 fp32, and for the output layer's real inputs four digit planes, one byte per weight,
    # and 16 bytes per frame
    assert (bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d2), 3, 4096) ==
            2 * 4096 * 2048 * 4 + 4 * 4096 * 2048 + 3400 * 2048 + 4096 * 16)
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d2), 3, 100) == 2 * 100 * 2048 * 4   # fewer than 128 frames: no planes
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d[:1]), 1, 4096) == 0
    assert bnn.bnn_forward_workspace_bytes(bnn.make_layer_array(d2[:1]), 1, 4096) == 0
    # workspace too small / missing
    assert _status(bnn.bnn_forward, arr, 3, P, 4096, R, 0, 0, 0) == bnn.BNN_EWORKSPACE
    assert _status(bnn.bnn_forward, arr, 3, P, 4096, R, 0x4000000, 100, 0) == bnn.BNN_EWORKSPACE
    assert _status(bnn.bnn_forward, arr, 3, P, 4096, R, 0x4000000 + 64, 1 << 26, 0) == bnn.BNN_EALIGN
    # K of a layer must equal N of the one before
    bad = _chain(bnn, (440, 2048, 2048, 3400), (S, S, Z)); bad[1]["K"] = 1024
    assert _status(bnn.bnn_forward, bnn.make_layer_array(bad), 3, P, 8, R, 0x4000000, 1 << 22, 0) == bnn.BNN_ESHAPE
    # x_is_binary must follow the previous activation
    bad = _chain(bnn, (440, 2048, 3400), (H, Z)); bad[1]["x_is_binary"] = 1
    assert _status(bnn.bnn_forward, bnn.make_layer_array(bad), 2, P, 8, R, 0x4000000, 1 << 22, 0) == bnn.BNN_ESHAPE
    # Softmax only at the end; RAW_I32 is not a layer activation of a network
    bad = _chain(bnn, (440, 2048, 3400), (Z, Z))
    assert _status(bnn.bnn_forward, bnn.make_layer_array(bad), 2, P, 8, R, 0x4000000, 1 << 22, 0) == bnn.BNN_ESHAPE
    bad = _chain(bnn, (440, 3400), (bnn.BNN_ACT_RAW_I32,))
    assert _status(bnn.bnn_forward, bnn.make_layer_array(bad), 1, P, 8, R, 0, 0, 0) == bnn.BNN_EINVAL
    # null weights, null input, no layers
    bad = _chain(bnn, (440, 3400), (Z,), Wp=0)
    assert _status(bnn.bnn_forward, bnn.make_layer_array(bad), 1, P, 8, R, 0, 0, 0) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_forward, arr, 3, 0, 8, R, 0x4000000, 1 << 26, 0) == bnn.BNN_EINVAL
    assert _status(bnn.bnn_forward, arr, 0, P, 8, R, 0x4000000, 1 << 22, 0) == bnn.BNN_EINVAL
    # zero frames: nothing to do, nothing touched
    assert bnn.bnn_forward(arr, 3, 0, 0, 0, 0, 0, 0) == 0


def test_product_does_not_reach_the_oracle():
    """The package holds no reference to oracle/ (no CPU fallback can hide behind the C ABI)."""
    pkg = os.path.join(ROOT, "paper_1706_09453_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    assert "oracle" not in open(HEADER).read().lower()
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_1706_09453_amd" not in text and "libbnn_hip" not in text, f
