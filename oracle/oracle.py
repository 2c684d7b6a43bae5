"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrappers over oracle/bnn_oracle.c plus the composition of those
steps into layers and into the whole forward pass, in the order the paper
gives them (Alg. 1 forward for binary weights, Alg. 2 forward for binary
activations, Sec. 2.3 for both).  Nothing here is imported by the product
package, and nothing here imports it.

Activation names follow the C ABI of the GPU library only in meaning, not in
code: "raw" (int32 product), "linear", "hardtanh", "sign" (packed bits out),
"logsoftmax".
"""
from __future__ import annotations

import ctypes
from ctypes import c_int, c_int64, c_void_p, c_float
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.orc_words_per_row.restype = c_int64
        lib.orc_words_per_row.argtypes = [c_int64, c_int]
        lib.orc_mean_abs.restype = c_float
        lib.orc_mean_abs.argtypes = [c_void_p, c_int64]
        lib.orc_sumsq_f64.restype = ctypes.c_double
        lib.orc_sumsq_f64.argtypes = [c_void_p, c_int64]
        for name, args in {
            "orc_pack_sign": [c_void_p, c_int64, c_int64, c_int, c_void_p],
            "orc_unpack_pm1": [c_void_p, c_int64, c_int64, c_int, c_void_p],
            "orc_dot_pm1": [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p],
            "orc_dot_xor": [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_void_p],
            "orc_dot_x01_wpm1": [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p],
            "orc_dot_and": [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_void_p],
            "orc_realx_acc": [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p],
            "orc_realw_acc": [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p],
            "orc_bits_to_real": [c_void_p, c_int64, c_int64, c_int, c_int, c_void_p],
            "orc_colsum_f32": [c_void_p, c_int64, c_int64, c_void_p],
            "orc_update_clip": [c_void_p, c_void_p, c_int64, c_float, c_int],
            "orc_affine_f32": [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_void_p],
            "orc_affine_f64": [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_void_p],
            "orc_i32_to_f32": [c_void_p, c_int64, c_void_p],
            "orc_hardtanh": [c_void_p, c_int64, c_void_p],
            "orc_sigmoid": [c_void_p, c_int64, c_void_p],
            "orc_log_softmax": [c_void_p, c_int64, c_int64, c_void_p, c_void_p],
        }.items():
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = args
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _word_dtype(word_bits: int):
    if word_bits not in (32, 64):
        raise ValueError("word_bits must be 32 or 64")
    return np.uint32 if word_bits == 32 else np.uint64


# ----------------------------------------------------------------------------- steps

def words_per_row(K: int, word_bits: int) -> int:
    return int(_L().orc_words_per_row(K, word_bits))


def pack_sign(x: np.ndarray, word_bits: int) -> np.ndarray:
    """Eq. 3 + storage reading: [rows, K] fp32 -> [rows, ceil(K/wb)] words, bit 1 <=> +1, LSB first."""
    x = _c(x, np.float32)
    rows, K = x.shape
    out = np.empty((rows, words_per_row(K, word_bits)), dtype=_word_dtype(word_bits))
    _L().orc_pack_sign(_p(x), rows, K, word_bits, _p(out))
    return out


def unpack_pm1(words: np.ndarray, K: int, word_bits: int) -> np.ndarray:
    """Packed rows -> [rows, K] int8 in {-1, +1}."""
    words = _c(words, _word_dtype(word_bits))
    rows = words.shape[0]
    assert words.shape[1] == words_per_row(K, word_bits)
    out = np.empty((rows, K), dtype=np.int8)
    _L().orc_unpack_pm1(_p(words), rows, K, word_bits, _p(out))
    return out


def mean_abs(w: np.ndarray) -> np.float32:
    """Per-layer scale: mean |w| over the real-valued weights (fp64 sum, rounded to fp32)."""
    w = _c(w, np.float32)
    return np.float32(_L().orc_mean_abs(_p(w), w.size))


def dot_pm1(a_pm1: np.ndarray, b_pm1: np.ndarray) -> np.ndarray:
    """Eq. 1 product for +-1 operands, plain definition: [M,K] x [N,K] -> int32 [M,N]."""
    a, b = _c(a_pm1, np.int8), _c(b_pm1, np.int8)
    M, K = a.shape
    N = b.shape[0]
    assert b.shape[1] == K
    out = np.empty((M, N), dtype=np.int32)
    _L().orc_dot_pm1(_p(a), _p(b), M, N, K, _p(out))
    return out


def dot_x01_wpm1(h01: np.ndarray, w_pm1: np.ndarray) -> np.ndarray:
    """Activations in {0, 1}, weights in {-1, +1} (Sec. 3.2, Tables 3-4), plain definition: [M,K] x [N,K] -> int32 [M,N]."""
    h, w = _c(h01, np.int8), _c(w_pm1, np.int8)
    M, K = h.shape
    N = w.shape[0]
    assert w.shape[1] == K
    out = np.empty((M, N), dtype=np.int32)
    _L().orc_dot_x01_wpm1(_p(h), _p(w), M, N, K, _p(out))
    return out


def dot_and(h_words: np.ndarray, w_words: np.ndarray, K: int, word_bits: int) -> np.ndarray:
    """The same product on packed rows: 2*popcount(h AND w) - popcount(h)."""
    dt = _word_dtype(word_bits)
    h, w = _c(h_words, dt), _c(w_words, dt)
    Kw = words_per_row(K, word_bits)
    assert h.shape[1] == Kw and w.shape[1] == Kw
    out = np.empty((h.shape[0], w.shape[0]), dtype=np.int32)
    _L().orc_dot_and(_p(h), _p(w), h.shape[0], w.shape[0], K, word_bits, _p(out))
    return out


def unpack_01(words: np.ndarray, K: int, word_bits: int) -> np.ndarray:
    """Packed rows -> [rows, K] int8 in {0, 1}: the stored bit itself."""
    return ((unpack_pm1(words, K, word_bits).astype(np.int16) + 1) // 2).astype(np.int8)


def dot_xor(a_words: np.ndarray, b_words: np.ndarray, K: int, word_bits: int) -> np.ndarray:
    """Sec. 2.3 form on packed rows: K - 2*popcount(a XOR b)."""
    dt = _word_dtype(word_bits)
    a, b = _c(a_words, dt), _c(b_words, dt)
    Kw = words_per_row(K, word_bits)
    assert a.shape[1] == Kw and b.shape[1] == Kw
    out = np.empty((a.shape[0], b.shape[0]), dtype=np.int32)
    _L().orc_dot_xor(_p(a), _p(b), a.shape[0], b.shape[0], K, word_bits, _p(out))
    return out


def realx_acc(x: np.ndarray, w_pm1: np.ndarray, want64: bool = True):
    """Alg. 1 product with real input: (acc32 canonical fp32 order, acc64 fp64 shadow)."""
    x, w = _c(x, np.float32), _c(w_pm1, np.int8)
    M, K = x.shape
    N = w.shape[0]
    assert w.shape[1] == K
    acc32 = np.empty((M, N), dtype=np.float32)
    acc64 = np.empty((M, N), dtype=np.float64) if want64 else None
    _L().orc_realx_acc(_p(x), _p(w), M, N, K, _p(acc32), _p(acc64))
    return acc32, acc64


def realw_acc(x: np.ndarray, w: np.ndarray, want64: bool = True):
    """Eq. 1 product of a real-weight layer: (acc32 in ascending k with one fma per step, acc64 fp64 shadow)."""
    x, w = _c(x, np.float32), _c(w, np.float32)
    M, K = x.shape
    N = w.shape[0]
    assert w.shape[1] == K
    acc32 = np.empty((M, N), dtype=np.float32)
    acc64 = np.empty((M, N), dtype=np.float64) if want64 else None
    _L().orc_realw_acc(_p(x), _p(w), M, N, K, _p(acc32), _p(acc64))
    return acc32, acc64


def bits_to_real(words: np.ndarray, K: int, word_bits: int, zero_one: bool) -> np.ndarray:
    """Stored bits of a binary layer as fp32 numbers: -1/+1 (Sign units) or 0/1 (Sec. 3.2)."""
    a = _c(words, _word_dtype(word_bits))
    out = np.empty((a.shape[0], K), dtype=np.float32)
    _L().orc_bits_to_real(_p(a), a.shape[0], K, word_bits, int(zero_one), _p(out))
    return out


def affine_f32(v: np.ndarray, scale: Optional[np.ndarray], bias: Optional[np.ndarray]) -> np.ndarray:
    """h^ = fmaf(scale[n], v[m,n], bias[n]) in fp32, one rounding."""
    v = _c(v, np.float32)
    M, N = v.shape
    s = None if scale is None else _c(scale, np.float32)
    b = None if bias is None else _c(bias, np.float32)
    out = np.empty((M, N), dtype=np.float32)
    _L().orc_affine_f32(_p(v), _p(s), _p(b), M, N, _p(out))
    return out


def affine_f64(v: np.ndarray, scale, bias) -> np.ndarray:
    v = _c(v, np.float64)
    M, N = v.shape
    s = None if scale is None else _c(scale, np.float32)
    b = None if bias is None else _c(bias, np.float32)
    out = np.empty((M, N), dtype=np.float64)
    _L().orc_affine_f64(_p(v), _p(s), _p(b), M, N, _p(out))
    return out


def i32_to_f32(dot: np.ndarray) -> np.ndarray:
    d = _c(dot, np.int32)
    out = np.empty(d.shape, dtype=np.float32)
    _L().orc_i32_to_f32(_p(d), d.size, _p(out))
    return out


def hardtanh(h: np.ndarray) -> np.ndarray:
    h = _c(h, np.float32)
    out = np.empty_like(h)
    _L().orc_hardtanh(_p(h), h.size, _p(out))
    return out


def sigmoid(h: np.ndarray) -> np.ndarray:
    """Sigmoid of the paper's real hidden layers (Sec. 3), fp64 from the fp32 pre-activation, rounded to fp32."""
    h = _c(h, np.float32)
    out = np.empty_like(h)
    _L().orc_sigmoid(_p(h), h.size, _p(out))
    return out


def log_softmax(z: np.ndarray):
    """Alg. 2 output layer as log-posteriors: returns (fp32 rounded, fp64)."""
    z = _c(z, np.float32)
    M, N = z.shape
    o32 = np.empty((M, N), dtype=np.float32)
    o64 = np.empty((M, N), dtype=np.float64)
    _L().orc_log_softmax(_p(z), M, N, _p(o32), _p(o64))
    return o32, o64


def subtract_log_prior(logp: np.ndarray, log_prior: np.ndarray) -> np.ndarray:
    """Scaled log-likelihoods for decoding with a hybrid system (the recipe the paper's systems follow, Sec. 3; the
    paper's own equations end at the Softmax): by Bayes' rule log p(x | s) = log P(s | x) - log P(s) + log p(x), so the
    log-posterior of every tied state minus the log of that state's prior, the frame's constant left out.
    out[m][n] = logp[m][n] - log_prior[n], one fp32 subtraction."""
    logp, log_prior = _c(logp, np.float32), _c(log_prior, np.float32)
    assert logp.ndim == 2 and log_prior.shape == (logp.shape[1],)
    return (logp - log_prior[None, :]).astype(np.float32)


# ----------------------------------------------------------------------------- layers

def _finish(hhat32: np.ndarray, act: str, word_bits: int):
    """h_l = f_l(h^_l)  (Eq. 2): the nonlinearity chosen for this layer."""
    if act == "linear":
        return hhat32
    if act == "hardtanh":
        return hardtanh(hhat32)
    if act == "sigmoid":
        return sigmoid(hhat32)
    if act in ("sign", "step01"):          # Alg. 2: h_l = Sign(h^_l), stored as bits along n; the (0, 1) step (Sec. 3.2)
        return pack_sign(hhat32, word_bits)  # stores the very same bit: 1 where h^_l > 0
    if act == "logsoftmax":                # Alg. 2: Softmax at l = L
        return log_softmax(hhat32)[0]
    raise ValueError(f"unknown activation {act!r}")


def layer_binw_realx(x: np.ndarray, w_words: np.ndarray, K: int, scale, bias, act: str, word_bits: int):
    """One layer with binary weights and real input (Alg. 1 forward): add/subtract product."""
    acc32, _ = realx_acc(x, unpack_pm1(w_words, K, word_bits), want64=False)
    return _finish(affine_f32(acc32, scale, bias), act, word_bits)


def layer_realw(x: np.ndarray, W: np.ndarray, bias, act: str, word_bits: int):
    """One layer with real-valued weights (Eq. 1-2; the input and Softmax layers of the paper's systems, Sec. 3.1)."""
    acc32, _ = realw_acc(x, W, want64=False)
    return _finish(affine_f32(acc32, None, bias), act, word_bits)


def layer_binw_binx(x_words: np.ndarray, w_words: np.ndarray, K: int, scale, bias, act: str, word_bits: int,
                    form: str = "definition"):
    """One layer with binary weights and binary input (Sec. 2.3).

    form = "definition": unpack to +-1 and take the plain integer product;
    form = "xor": K - 2*popcount(XOR) on the packed words (same values, pinned by tests).
    """
    if form == "definition":
        dot = dot_pm1(unpack_pm1(x_words, K, word_bits), unpack_pm1(w_words, K, word_bits))
    elif form == "xor":
        dot = dot_xor(x_words, w_words, K, word_bits)
    else:
        raise ValueError(form)
    if act == "raw":
        return dot
    return _finish(affine_f32(i32_to_f32(dot), scale, bias), act, word_bits)


def layer_binw_binx01(h_words: np.ndarray, w_words: np.ndarray, K: int, scale, bias, act: str, word_bits: int,
                      form: str = "definition"):
    """One layer with binary weights in {-1,+1} and binary input read as {0,1} (Sec. 3.2).

    form = "definition": unpack and take the plain integer product; form = "and" (or "xor", so that
    forward(form="xor") runs every binary layer on packed words): 2*popcount(AND) - popcount on the packed words
    (same values, pinned by tests).
    """
    if form == "definition":
        dot = dot_x01_wpm1(unpack_01(h_words, K, word_bits), unpack_pm1(w_words, K, word_bits))
    elif form in ("and", "xor"):
        dot = dot_and(h_words, w_words, K, word_bits)
    else:
        raise ValueError(form)
    if act == "raw":
        return dot
    return _finish(affine_f32(i32_to_f32(dot), scale, bias), act, word_bits)


@dataclass
class OracleLayer:
    K: int
    N: int
    act: str                    # "sign" | "step01" | "hardtanh" | "linear" | "logsoftmax"
    word_bits: int
    w_words: np.ndarray         # [N, ceil(K/wb)]
    scale: Optional[np.ndarray]  # [N] fp32 or None
    bias: Optional[np.ndarray]   # [N] fp32 or None
    w_real: Optional[np.ndarray] = None   # [N, K] fp32: the layer keeps real-valued weights (then w_words is None)


def make_layers(Ws: Sequence[np.ndarray], biases: Sequence[np.ndarray], hidden_act: str, word_bits: int,
                use_scale: bool = True, real_weight_layers: Sequence[int] = ()) -> List[OracleLayer]:
    """Alg. 1, first step of the forward loop: w^b_l = Sign(w_l), done once; scale_l = mean|w_l| broadcast over n.

    hidden_act: one activation name for every hidden layer, or a sequence with one name per hidden layer.
    real_weight_layers: indices of the layers that keep their real-valued weights (Sec. 3.1: input and Softmax layer).
    """
    layers = []
    for l, (W, r) in enumerate(zip(Ws, biases)):
        N, K = W.shape
        act = "logsoftmax" if l == len(Ws) - 1 else (hidden_act if isinstance(hidden_act, str) else hidden_act[l])
        if l in real_weight_layers:
            layers.append(OracleLayer(K, N, act, word_bits, None, None, np.ascontiguousarray(r, dtype=np.float32),
                                      np.ascontiguousarray(W, dtype=np.float32)))
            continue
        scale = np.full(N, mean_abs(W), dtype=np.float32) if use_scale else None
        layers.append(OracleLayer(K, N, act, word_bits, pack_sign(W, word_bits), scale,
                                  np.ascontiguousarray(r, dtype=np.float32)))
    return layers


def forward(layers: Sequence[OracleLayer], x: np.ndarray, form: str = "definition", keep: bool = False):
    """Whole forward pass (Alg. 2 forward with Alg. 1's binary weights): returns log-posteriors [M, N_L].

    The input of a layer is binary exactly when the previous layer's activation was Sign (read as -1/+1) or the (0, 1)
    step (act "step01": the same stored bits, read as 0/1 by the next layer).
    With keep=True also returns the list of every layer's output.
    """
    h = np.ascontiguousarray(x, dtype=np.float32)
    domain = "real"
    outs = []
    for ly in layers:
        act = ly.act
        if ly.w_real is not None:
            if domain != "real":   # the bits of a binary layer, as the numbers they stand for
                h = bits_to_real(h, ly.K, ly.word_bits, zero_one=(domain == "01"))
            h = layer_realw(h, ly.w_real, ly.bias, act, ly.word_bits)
        elif domain == "pm1":
            h = layer_binw_binx(h, ly.w_words, ly.K, ly.scale, ly.bias, act, ly.word_bits, form=form)
        elif domain == "01":
            h = layer_binw_binx01(h, ly.w_words, ly.K, ly.scale, ly.bias, act, ly.word_bits, form=form)
        else:
            h = layer_binw_realx(h, ly.w_words, ly.K, ly.scale, ly.bias, act, ly.word_bits)
        domain = {"sign": "pm1", "step01": "01"}.get(ly.act, "real")
        outs.append(h)
    return (h, outs) if keep else h
