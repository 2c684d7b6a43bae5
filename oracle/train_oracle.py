"""Training-side steps of the CPU oracle (TEST INFRASTRUCTURE ONLY): backward propagation and update of Alg. 1
(binary weights) and Alg. 2 (binary activations), gradient-norm clipping (Sec. 2.3) and the semi-stochastic
binarisation of Sec. 2.1.

Readings where the paper is silent:
  - the loss is the cross entropy of the Softmax output against one label per frame (Sec. 3), summed over the frames
    of the minibatch (no division by their number): g_{h^_L} = softmax(h^_L) - onehot(label);
  - every sum (over outputs n in g_h = g_{h^} w^b, over frames m in g_w = g_{h^} h and g_r) is taken in fp32 in
    ascending index with one accumulator per result, one fused multiply-add per step where there is a product;
  - p(|w|) of the semi-stochastic binarisation is never written out; it says only that |w| close to 1 gives a high
    probability and |w| close to 0 a small one, with w in [-1, +1] after clipping: p(|w|) = |w| is taken.  The uniform
    numbers in [0, 1) are an INPUT (a weight is set to its sign where u < |w|);
  - the gradient through a layer with a per-layer scale is not in the paper (no scale there): the backward products
    here are the paper's, without scale; a caller that uses one multiplies g_{h^} by it first.
"""
from __future__ import annotations

import ctypes
from ctypes import c_float, c_int, c_int64

import numpy as np

from . import oracle as O


def softmax_xent_grad(logp: np.ndarray, labels: np.ndarray) -> np.ndarray:
    """Alg. 1/2, gradient from the loss through the Softmax layer: g[m][n] = exp(logp[m][n]) - (n == label[m]),
    fp64 from the fp32 log-posteriors, rounded to fp32."""
    lp = np.ascontiguousarray(logp, dtype=np.float32).astype(np.float64)
    g = np.exp(lp)
    g[np.arange(lp.shape[0]), np.asarray(labels, dtype=np.int64)] -= 1.0
    return g.astype(np.float32)


def mask_grad(g_h: np.ndarray, hhat: np.ndarray, k: float) -> np.ndarray:
    """Sec. 2.2: g_{h^} = g_h (.) Mask(h^, k), Mask = 0 where |h^| > k, 1 otherwise (so NaN passes: not > k)."""
    g = np.ascontiguousarray(g_h, dtype=np.float32)
    hh = np.ascontiguousarray(hhat, dtype=np.float32)
    return np.where(np.abs(hh) > np.float32(k), np.float32(0.0), g).astype(np.float32)


def sigmoid_grad(g_h: np.ndarray, h: np.ndarray) -> np.ndarray:
    """Alg. 1 backward through a Sigmoid layer (the real hidden layers of Sec. 3): g_{h^} = g_h f'(h^) with
    f'(h^) = h (1 - h), h the layer's output; fp32, evaluated as g_h * (h * (1 - h)), every operation rounded."""
    g = np.ascontiguousarray(g_h, dtype=np.float32)
    hh = np.ascontiguousarray(h, dtype=np.float32)
    one_minus = (np.float32(1.0) - hh).astype(np.float32)
    return (g * (hh * one_minus).astype(np.float32)).astype(np.float32)


def backward_input_binw(g_hhat: np.ndarray, w_pm1: np.ndarray) -> np.ndarray:
    """Alg. 1 backward: g_{h_{l-1}} = g_{h^_l} w^b_l, [M][N] x [N][K] -> [M][K]; sum over n ascending (add/subtract)."""
    wt = np.ascontiguousarray(np.asarray(w_pm1, dtype=np.int8).T)          # [K][N]
    return O.realx_acc(g_hhat, wt, want64=False)[0]


def backward_input_realw(g_hhat: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Alg. 2 backward with real-valued weights: g_{h_{l-1}} = g_{h^_l} w_l; sum over n ascending, one fma per step."""
    wt = np.ascontiguousarray(np.asarray(W, dtype=np.float32).T)           # [K][N]
    return O.realw_acc(g_hhat, wt, want64=False)[0]


def backward_weight(g_hhat: np.ndarray, h_prev: np.ndarray) -> np.ndarray:
    """Alg. 1/2 backward: g_{w_l} = g_{h^_l}^T h_{l-1}, [N][M] x [M][K] -> [N][K]; sum over frames m ascending."""
    gt = np.ascontiguousarray(np.asarray(g_hhat, dtype=np.float32).T)      # [N][M]
    ht = np.ascontiguousarray(np.asarray(h_prev, dtype=np.float32).T)      # [K][M]
    return O.realw_acc(gt, ht, want64=False)[0]


def bias_grad(g_hhat: np.ndarray) -> np.ndarray:
    g = np.ascontiguousarray(g_hhat, dtype=np.float32)
    out = np.empty(g.shape[1], dtype=np.float32)
    O._L().orc_colsum_f32(O._p(g), g.shape[0], g.shape[1], O._p(out))
    return out


def update_clip(w: np.ndarray, g: np.ndarray, eta: float, clip: bool) -> np.ndarray:
    """Alg. 1 Update: Clip(w - eta g); clip=False: the plain update (Alg. 2, and the bias)."""
    out = np.array(w, dtype=np.float32, copy=True, order="C")
    gg = np.ascontiguousarray(g, dtype=np.float32)
    assert out.shape == gg.shape
    O._L().orc_update_clip(O._p(out), O._p(gg), out.size, c_float(eta), int(clip))
    return out


def grad_norm_clip(g: np.ndarray, alpha: float):
    """Sec. 2.3: if ||g||_2 > alpha then g <- (alpha / ||g||_2) g.  Returns (g', ||g||_2 as fp32)."""
    gg = np.ascontiguousarray(g, dtype=np.float32)
    norm = np.float32(np.sqrt(O._L().orc_sumsq_f64(O._p(gg), gg.size)))
    if norm > np.float32(alpha):
        factor = np.float32(np.float32(alpha) / norm)
        return (gg * factor).astype(np.float32), norm
    return gg.copy(), norm


def semi_stochastic_binarize(w: np.ndarray, u: np.ndarray) -> np.ndarray:
    """Sec. 2.1, Alg. 1 Update (optional step): w_ij <- Sign(w_ij) with probability p(|w_ij|) = |w_ij|, the draw u_ij
    in [0, 1) given: the weight is set to its sign where u_ij < |w_ij|."""
    ww = np.ascontiguousarray(w, dtype=np.float32)
    uu = np.ascontiguousarray(u, dtype=np.float32)
    sign = np.where(ww > 0, np.float32(1.0), np.float32(-1.0))
    return np.where(uu < np.abs(ww), sign, ww).astype(np.float32)
