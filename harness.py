"""Device-side harness shared by bench.py, the smoke run and the GPU tests: device buffers through PyTorch, every
computation through the C ABI (the binding marshals arguments, nothing else)."""
from __future__ import annotations

import numpy as np
import torch

import paper_1706_09453_amd as bnn

DEV = "cuda:0"


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def to_dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def words_to_host(t: torch.Tensor, word_bits: int) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(np.uint32 if word_bits == 32 else np.uint64)


def word_tensor(rows: int, K: int, word_bits: int) -> torch.Tensor:
    kw = bnn.bnn_packed_words(K, word_bits)
    # filled with a pattern so that unwritten words would be noticed
    return torch.full((rows, kw), -0x0123456, dtype=torch.int32 if word_bits == 32 else torch.int64, device=DEV)


def ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def pack_activations(X: torch.Tensor, word_bits: int) -> torch.Tensor:
    M, K = X.shape
    out = word_tensor(M, K, word_bits)
    bnn.bnn_pack_activations(ptr(X), M, K, word_bits, ptr(out), stream())
    return out


def pack_weights(W: torch.Tensor, word_bits: int, want_scale: bool = True):
    N, K = W.shape
    out = word_tensor(N, K, word_bits)
    sc = torch.full((1,), float("nan"), dtype=torch.float32, device=DEV) if want_scale else None
    bnn.bnn_pack_weights(ptr(W), N, K, word_bits, ptr(out), ptr(sc), stream())
    return out, sc


def out_tensor(M: int, N: int, act: int, word_bits: int) -> torch.Tensor:
    if act == bnn.BNN_ACT_SIGN:
        return word_tensor(M, N, word_bits)
    if act == bnn.BNN_ACT_RAW_I32:
        return torch.full((M, N), -77777, dtype=torch.int32, device=DEV)
    return torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)


def layer_realx(X, Wp, scale, bias, K, N, act, word_bits):
    M = X.shape[0]
    Y = out_tensor(M, N, act, word_bits)
    bnn.bnn_layer_binw_realx(ptr(X), ptr(Wp), ptr(scale), ptr(bias), M, K, N, act, word_bits, ptr(Y), stream())
    return Y


def layer_binx(Xp, Wp, scale, bias, K, N, act, word_bits, arm=bnn.BNN_ARM_AUTO):
    M = Xp.shape[0]
    Y = out_tensor(M, N, act, word_bits)
    bnn.bnn_layer_binw_binx_arm(ptr(Xp), ptr(Wp), ptr(scale), ptr(bias), M, K, N, act, word_bits, ptr(Y), arm, stream())
    return Y


def layer_binx01(Xp, Wp, scale, bias, K, N, act, word_bits):
    M = Xp.shape[0]
    Y = out_tensor(M, N, act, word_bits)
    bnn.bnn_layer_binw_binx01(ptr(Xp), ptr(Wp), ptr(scale), ptr(bias), M, K, N, act, word_bits, ptr(Y), stream())
    return Y


def layer_realw(X, W, bias, K, N, act, word_bits):
    M = X.shape[0]
    Y = out_tensor(M, N, act, word_bits)
    bnn.bnn_layer_realw(ptr(X), ptr(W), ptr(bias), M, K, N, act, word_bits, ptr(Y), stream())
    return Y


def unpack_activations(Xp, K, word_bits, zero_one):
    M = Xp.shape[0]
    X = torch.full((M, K), float("nan"), dtype=torch.float32, device=DEV)
    bnn.bnn_unpack_activations(ptr(Xp), M, K, word_bits, int(zero_one), ptr(X), stream())
    return X


class GpuModel:
    """Packed model on the GPU, prepared with bnn_pack_weights from real-valued weights (Alg. 1: w^b = Sign(w))."""

    def __init__(self, Ws, biases, hidden_act: str, word_bits: int, x_is_binary: bool = False, real_weight_layers=()):
        self.word_bits = word_bits
        self.keep = []           # device tensors referenced by the descriptors
        self.scales = []
        descs = []
        binary = int(x_is_binary)   # 0: real input, 1: bits read as -1/+1, 2: bits read as 0/1 ("step01" hidden layers)
        for l, (W, r) in enumerate(zip(Ws, biases)):
            N, K = W.shape
            Wd = to_dev(W.astype(np.float32))
            bias = to_dev(r.astype(np.float32))
            name = hidden_act if isinstance(hidden_act, str) else (hidden_act[l] if l < len(Ws) - 1 else None)
            act = bnn.BNN_ACT_LOGSOFTMAX if l == len(Ws) - 1 else bnn.ACT_BY_NAME[name]
            if l in real_weight_layers:                 # the layer keeps its real-valued weights, fp32 [N][K]
                self.keep += [Wd, bias]
                self.scales.append(None)
                descs.append(dict(K=K, N=N, act=act, word_bits=word_bits, x_is_binary=binary, w_is_real=1,
                                  Wp=ptr(Wd), scale=0, bias=ptr(bias)))
            else:
                Wp, sc = pack_weights(Wd, word_bits)
                scale = sc.expand(N).contiguous()       # broadcast the per-layer scalar to [N] (a copy, no arithmetic)
                self.keep += [Wp, scale, bias]
                self.scales.append(sc)
                descs.append(dict(K=K, N=N, act=act, word_bits=word_bits, x_is_binary=binary,
                                  Wp=ptr(Wp), scale=ptr(scale), bias=ptr(bias)))
            binary = (2 if name == "step01" else 1) if act == bnn.BNN_ACT_SIGN else 0
            del Wd
        self.descs = descs
        self.layers = bnn.make_layer_array(descs)
        self.n_layers = len(descs)
        self.N_out = descs[-1]["N"]
        self._ws = None
        self._ws_M = -1

    def workspace(self, M: int):
        if self._ws_M != M:
            nbytes = bnn.bnn_forward_workspace_bytes(self.layers, self.n_layers, M)
            self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)
            self._ws_bytes = nbytes
            self._ws_M = M
        return self._ws, self._ws_bytes

    def forward(self, X: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        M = X.shape[0]
        ws, nbytes = self.workspace(M)
        if out is None:
            out = torch.full((M, self.N_out), float("nan"), dtype=torch.float32, device=DEV)
        bnn.bnn_forward(self.layers, self.n_layers, ptr(X), M, ptr(out), ptr(ws), nbytes, stream())
        return out
