"""ctypes binding of libbnn_hip.so: the same names as include/bnn.h, argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI.  There is no CPU fallback: if the
library has not been built, importing this module raises.  Pointers are plain integers (for example
``tensor.data_ptr()`` of a PyTorch tensor on the GPU, or 0 for NULL); ``stream`` is a hipStream_t as an
integer (``torch.cuda.current_stream().cuda_stream``, 0 = default stream).
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from typing import Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbnn_hip.so")

BNN_OK, BNN_EINVAL, BNN_ESHAPE, BNN_EALIGN, BNN_EWORKSPACE, BNN_EDEVICE = 0, -1, -2, -3, -4, -5
BNN_ACT_RAW_I32, BNN_ACT_LINEAR, BNN_ACT_HARDTANH, BNN_ACT_SIGN, BNN_ACT_LOGSOFTMAX, BNN_ACT_SIGMOID = 0, 1, 2, 3, 4, 5
BNN_ARM_AUTO, BNN_ARM_VALU_XOR, BNN_ARM_MFMA, BNN_ARM_MFMA_I8 = 0, 1, 2, 3
BNN_OPT_BINX_ARM, BNN_OPT_REALX_TM, BNN_OPT_BINX_VALU_TM, BNN_OPT_MFMA_WM = 1, 2, 3, 4
BNN_OPT_REALX_SIGN_MFMA, BNN_OPT_FUSED_LOGSOFTMAX, BNN_OPT_MFMA_SHAPE, BNN_OPT_MFMA32_WM = 5, 6, 7, 8
BNN_OPT_MFMA32_PIPELINE = 9
BNN_OPT_REALX_F32_MFMA = 10
BNN_OPT_MFMA32_XCD_ORDER = 11
BNN_OPT_STREAM_MAX_FRAMES = 12
BNN_OPT_COOPERATIVE = 13
BNN_OPT_MFMA32_SPLITK = 14
BNN_OPT_COOPERATIVE_SPIN = 15
BNN_OPT_REALX_I8_LOGSOFTMAX = 16
BNN_OPT_REALW_SPLIT_LOGSOFTMAX = 17
BNN_OPT_REALW_VALU_LDS = 18

ACT_BY_NAME = {"raw": BNN_ACT_RAW_I32, "linear": BNN_ACT_LINEAR, "hardtanh": BNN_ACT_HARDTANH,
               "sign": BNN_ACT_SIGN, "step01": BNN_ACT_SIGN, "logsoftmax": BNN_ACT_LOGSOFTMAX,
               "sigmoid": BNN_ACT_SIGMOID}


class bnn_layer_desc(ctypes.Structure):
    _fields_ = [("K", c_int64), ("N", c_int64), ("act", c_int32), ("word_bits", c_int32),
                ("x_is_binary", c_int32), ("w_is_real", c_int32),
                ("Wp", c_void_p), ("scale", c_void_p), ("bias", c_void_p)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")

_lib = ctypes.CDLL(LIB_PATH)

_SIGNATURES = {
    "bnn_packed_words": (c_size_t, [c_int64, c_int]),
    "bnn_status_string": (c_char_p, [c_int]),
    "bnn_set_option": (c_int, [c_int, c_int]),
    "bnn_cooperative_timeouts": (c_int, [ctypes.POINTER(ctypes.c_uint64)]),
    "bnn_pack_weights": (c_int, [c_void_p, c_int64, c_int64, c_int, c_void_p, c_void_p, c_void_p]),
    "bnn_pack_activations": (c_int, [c_void_p, c_int64, c_int64, c_int, c_void_p, c_void_p]),
    "bnn_layer_binw_realx": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_int,
                                     c_void_p, c_void_p]),
    "bnn_layer_binw_binx": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_int,
                                    c_void_p, c_void_p]),
    "bnn_layer_binw_binx01": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_int,
                                      c_void_p, c_void_p]),
    "bnn_layer_realw": (c_int, [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_int, c_void_p, c_void_p]),
    "bnn_unpack_activations": (c_int, [c_void_p, c_int64, c_int64, c_int, c_int, c_void_p, c_void_p]),
    "bnn_layer_binw_binx_arm": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_int,
                                        c_void_p, c_int, c_void_p]),
    "bnn_pack_weights_transposed": (c_int, [c_void_p, c_int64, c_int64, c_int, c_void_p, c_void_p]),
    "bnn_transpose_f32": (c_int, [c_void_p, c_int64, c_int64, c_void_p, c_void_p]),
    "bnn_softmax_xent_grad": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_void_p]),
    "bnn_mask_grad": (c_int, [c_void_p, c_void_p, c_int64, c_float, c_void_p, c_void_p]),
    "bnn_sigmoid_grad": (c_int, [c_void_p, c_void_p, c_int64, c_void_p, c_void_p]),
    "bnn_backward_input_binw": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_void_p, c_void_p]),
    "bnn_backward_input_realw": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p]),
    "bnn_backward_weight": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p]),
    "bnn_backward_weight_binh": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_void_p, c_void_p]),
    "bnn_layer_binw_realx_i8_workspace_bytes": (c_size_t, [c_int64, c_int64, c_int64]),
    "bnn_layer_binw_realx_i8": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_void_p,
                                c_void_p, c_size_t, c_void_p]),
    "bnn_bias_grad": (c_int, [c_void_p, c_int64, c_int64, c_void_p, c_void_p]),
    "bnn_update_clip": (c_int, [c_void_p, c_void_p, c_int64, c_float, c_int, c_void_p]),
    "bnn_grad_norm_clip": (c_int, [c_void_p, c_int64, c_float, c_void_p, c_void_p, c_void_p]),
    "bnn_semi_stochastic_binarize": (c_int, [c_void_p, c_void_p, c_int64, c_void_p]),
    "bnn_subtract_log_prior": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_void_p]),
    "bnn_forward_workspace_bytes": (c_size_t, [c_void_p, c_int, c_int64]),
    "bnn_forward": (c_int, [c_void_p, c_int, c_void_p, c_int64, c_void_p, c_void_p, c_size_t, c_void_p]),
    "bnn_forward_static": (c_int, [c_void_p, c_int, c_void_p, c_int64, c_void_p, c_void_p]),
}
for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTED = tuple(_SIGNATURES)


class BnnError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"bnn status {status}: {bnn_status_string(status)}")


def _check(status: int) -> int:
    if status != BNN_OK:
        raise BnnError(status)
    return status


def bnn_packed_words(K: int, word_bits: int) -> int:
    return int(_lib.bnn_packed_words(K, word_bits))


def bnn_status_string(status: int) -> str:
    return _lib.bnn_status_string(status).decode()


def bnn_set_option(option: int, value: int) -> int:
    return _check(_lib.bnn_set_option(option, value))


def bnn_cooperative_timeouts() -> int:
    count = ctypes.c_uint64(0)
    _check(_lib.bnn_cooperative_timeouts(ctypes.byref(count)))
    return int(count.value)


def bnn_pack_weights(W: int, N: int, K: int, word_bits: int, Wp: int, scale_out: int = 0, stream: int = 0) -> int:
    return _check(_lib.bnn_pack_weights(W, N, K, word_bits, Wp, scale_out or None, stream or None))


def bnn_pack_activations(X: int, M: int, K: int, word_bits: int, Xp: int, stream: int = 0) -> int:
    return _check(_lib.bnn_pack_activations(X, M, K, word_bits, Xp, stream or None))


def bnn_layer_binw_realx(X: int, Wp: int, scale: int, bias: int, M: int, K: int, N: int, act: int, word_bits: int,
                         Y: int, stream: int = 0) -> int:
    return _check(_lib.bnn_layer_binw_realx(X, Wp, scale or None, bias or None, M, K, N, act, word_bits, Y,
                                            stream or None))


def bnn_layer_binw_binx(Xp: int, Wp: int, scale: int, bias: int, M: int, K: int, N: int, act: int, word_bits: int,
                        Y: int, stream: int = 0) -> int:
    return _check(_lib.bnn_layer_binw_binx(Xp, Wp, scale or None, bias or None, M, K, N, act, word_bits, Y,
                                           stream or None))


def bnn_layer_binw_binx01(Xp: int, Wp: int, scale: int, bias: int, M: int, K: int, N: int, act: int, word_bits: int,
                          Y: int, stream: int = 0) -> int:
    return _check(_lib.bnn_layer_binw_binx01(Xp, Wp, scale or None, bias or None, M, K, N, act, word_bits, Y,
                                             stream or None))


def bnn_layer_realw(X: int, W: int, bias: int, M: int, K: int, N: int, act: int, word_bits: int, Y: int,
                    stream: int = 0) -> int:
    return _check(_lib.bnn_layer_realw(X, W, bias or None, M, K, N, act, word_bits, Y, stream or None))


def bnn_unpack_activations(Xp: int, M: int, K: int, word_bits: int, zero_one: int, X: int, stream: int = 0) -> int:
    return _check(_lib.bnn_unpack_activations(Xp, M, K, word_bits, zero_one, X, stream or None))


def bnn_layer_binw_binx_arm(Xp: int, Wp: int, scale: int, bias: int, M: int, K: int, N: int, act: int,
                            word_bits: int, Y: int, arm: int, stream: int = 0) -> int:
    return _check(_lib.bnn_layer_binw_binx_arm(Xp, Wp, scale or None, bias or None, M, K, N, act, word_bits, Y, arm,
                                               stream or None))


# ---- training side (argument order as in include/bnn.h)

def bnn_pack_weights_transposed(W: int, N: int, K: int, word_bits: int, WpT: int, stream: int = 0) -> int:
    return _check(_lib.bnn_pack_weights_transposed(W, N, K, word_bits, WpT, stream or None))


def bnn_transpose_f32(A: int, R: int, C: int, out: int, stream: int = 0) -> int:
    return _check(_lib.bnn_transpose_f32(A, R, C, out, stream or None))


def bnn_softmax_xent_grad(logp: int, labels: int, M: int, N: int, g: int, stream: int = 0) -> int:
    return _check(_lib.bnn_softmax_xent_grad(logp, labels, M, N, g, stream or None))


def bnn_mask_grad(g_h: int, hhat: int, count: int, k: float, g_hhat: int, stream: int = 0) -> int:
    return _check(_lib.bnn_mask_grad(g_h, hhat, count, k, g_hhat, stream or None))


def bnn_sigmoid_grad(g_h: int, h: int, count: int, g_hhat: int, stream: int = 0) -> int:
    return _check(_lib.bnn_sigmoid_grad(g_h, h, count, g_hhat, stream or None))


def bnn_backward_input_binw(g_hhat: int, WpT: int, M: int, N: int, K: int, word_bits: int, g_h: int, stream: int = 0) -> int:
    return _check(_lib.bnn_backward_input_binw(g_hhat, WpT, M, N, K, word_bits, g_h, stream or None))


def bnn_backward_input_realw(g_hhat: int, Wt: int, M: int, N: int, K: int, g_h: int, stream: int = 0) -> int:
    return _check(_lib.bnn_backward_input_realw(g_hhat, Wt, M, N, K, g_h, stream or None))


def bnn_backward_weight(g_hhat_t: int, h_t: int, N: int, K: int, M: int, g_w: int, stream: int = 0) -> int:
    return _check(_lib.bnn_backward_weight(g_hhat_t, h_t, N, K, M, g_w, stream or None))


def bnn_backward_weight_binh(g_hhat_t: int, HpT: int, N: int, K: int, M: int, word_bits: int, g_w: int, stream: int = 0) -> int:
    return _check(_lib.bnn_backward_weight_binh(g_hhat_t, HpT, N, K, M, word_bits, g_w, stream or None))


def bnn_layer_binw_realx_i8_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(_lib.bnn_layer_binw_realx_i8_workspace_bytes(M, K, N))


def bnn_layer_binw_realx_i8(X: int, Wp: int, scale: int, bias: int, M: int, K: int, N: int, word_bits: int, Y: int,
                            workspace: int, workspace_bytes: int, stream: int = 0) -> int:
    return _check(_lib.bnn_layer_binw_realx_i8(X, Wp, scale or None, bias or None, M, K, N, word_bits, Y, workspace or None,
                                               workspace_bytes, stream or None))


def bnn_bias_grad(g_hhat: int, M: int, N: int, g_r: int, stream: int = 0) -> int:
    return _check(_lib.bnn_bias_grad(g_hhat, M, N, g_r, stream or None))


def bnn_update_clip(w: int, g: int, count: int, eta: float, clip: int, stream: int = 0) -> int:
    return _check(_lib.bnn_update_clip(w, g, count, eta, clip, stream or None))


def bnn_grad_norm_clip(g: int, count: int, alpha: float, workspace: int, norm_out: int, stream: int = 0) -> int:
    return _check(_lib.bnn_grad_norm_clip(g, count, alpha, workspace, norm_out, stream or None))


def bnn_subtract_log_prior(logp: int, log_prior: int, M: int, N: int, stream: int = 0) -> int:
    return _check(_lib.bnn_subtract_log_prior(logp, log_prior, M, N, stream or None))


def bnn_semi_stochastic_binarize(w: int, u: int, count: int, stream: int = 0) -> int:
    return _check(_lib.bnn_semi_stochastic_binarize(w, u, count, stream or None))


def make_layer_array(descs: Sequence[dict]):
    """HOST array of bnn_layer_desc from dicts with keys K, N, act, word_bits, x_is_binary, Wp, scale, bias and,
    optionally, w_is_real."""
    arr = (bnn_layer_desc * len(descs))()
    for i, d in enumerate(descs):
        arr[i].K, arr[i].N = d["K"], d["N"]
        arr[i].act, arr[i].word_bits = d["act"], d["word_bits"]
        arr[i].x_is_binary, arr[i].w_is_real = int(d["x_is_binary"]), int(d.get("w_is_real", 0))
        arr[i].Wp, arr[i].scale, arr[i].bias = d["Wp"] or None, d.get("scale") or None, d.get("bias") or None
    return arr


def bnn_forward_workspace_bytes(layers, n_layers: int, M: int) -> int:
    return int(_lib.bnn_forward_workspace_bytes(ctypes.cast(layers, c_void_p), n_layers, M))


BNN_FORWARD_STATIC_MAX_BYTES = 16 << 20


def bnn_forward_static(layers, n_layers: int, X: int, M: int, out: int, stream: int = 0) -> int:
    return _check(_lib.bnn_forward_static(ctypes.cast(layers, c_void_p), n_layers, X, M, out, stream or None))


def bnn_forward(layers, n_layers: int, X: int, M: int, out: int, workspace: int, workspace_bytes: int,
                stream: int = 0) -> int:
    return _check(_lib.bnn_forward(ctypes.cast(layers, c_void_p), n_layers, X, M, out, workspace or None,
                                   workspace_bytes, stream or None))
