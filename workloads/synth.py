"""Counter-based synthetic tensors with the shapes of hybrid DNN acoustic-model workloads.

The paper's networks (Section 3: 40-dim filterbank features spliced over 11
frames, six hidden layers of 1024 or 2048 units, a Softmax layer over a few
thousand tied triphone states) are trained on speech corpora that are not
available here, so every tensor is synthetic: features ~ N(0,1), real-valued
"shadow" weights ~ U(-1,1) (to be binarised by whoever consumes them),
biases ~ N(0, 0.1^2), and fair random bits for the isolated GEMM sweep.

Every element is a pure function of (seed, tensor id, flat index) through a
SplitMix64-style hash, so any slice of any tensor can be regenerated anywhere
and both the CPU oracle and the GPU path are fed the very same bytes.
Nothing in this module belongs to the method itself.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)

TENSOR_W, TENSOR_BIAS, TENSOR_INPUT, TENSOR_ABITS, TENSOR_BBITS = 0, 1, 2, 3, 4


def _mix(z: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on uint64 arrays (wrapping arithmetic)."""
    z = (z ^ (z >> _U64(30))) * _M1
    z = (z ^ (z >> _U64(27))) * _M2
    return z ^ (z >> _U64(31))


def _stream(seed: int, tensor_id: int, start: int, count: int, lane: int = 0) -> np.ndarray:
    """uint64 hash of the counters (seed, tensor_id, lane, start..start+count-1)."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed * 0x1000003 + tensor_id * 0x10001 + lane * 0x101 + 1) & 0xFFFFFFFFFFFFFFFF],
                            dtype=_U64) * _GOLDEN)[0]
        idx = np.arange(start, start + count, dtype=_U64)
        return _mix(key + (idx + _U64(1)) * _GOLDEN)


def uniform_pm1(seed: int, tensor_id: int, count: int, start: int = 0) -> np.ndarray:
    """fp32 samples on the grid (2i+1)/2^24 - 1, i in [0, 2^24): uniform on (-1, 1), never 0."""
    i = (_stream(seed, tensor_id, start, count) >> _U64(40)).astype(np.int64)
    return ((2 * i + 1 - (1 << 24)).astype(np.float64) / float(1 << 24)).astype(np.float32)


def normal(seed: int, tensor_id: int, count: int, std: float = 1.0, start: int = 0) -> np.ndarray:
    """fp32 N(0, std^2) samples: Box-Muller in fp64 from two hashed uniforms, rounded to fp32."""
    a = _stream(seed, tensor_id, start, count, lane=0)
    b = _stream(seed, tensor_id, start, count, lane=1)
    u1 = ((a >> _U64(11)).astype(np.float64) + 1.0) / float(1 << 53)      # (0, 1]
    u2 = (b >> _U64(11)).astype(np.float64) / float(1 << 53)              # [0, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (z * std).astype(np.float32)


def random_words(seed: int, tensor_id: int, rows: int, words_per_row: int, start_row: int = 0) -> np.ndarray:
    """[rows, words_per_row] uint32 of fair random bits (every bit position is used)."""
    n = rows * words_per_row
    h = _stream(seed, tensor_id, start_row * words_per_row, n)
    return (h >> _U64(32)).astype(np.uint32).reshape(rows, words_per_row)


@dataclass(frozen=True)
class NetConfig:
    """One feedforward acoustic-model workload.

    dims = [K0, hidden..., N_out]; hidden_act is "sign" (binary activations in {-1, +1}), "step01" (binary
    activations in {0, 1}) or "hardtanh" (real activations); the last layer always ends in log-softmax.
    """
    cfg_id: int
    name: str
    dims: Tuple[int, ...]
    M: int
    hidden_act: object          # str, or a tuple of str with one name per hidden layer
    word_bits: int
    seed: int = 0
    real_weight_layers: Tuple[int, ...] = ()   # 0-based layers that keep real-valued weights (Sec. 3.1)

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1

    def layer_shape(self, l: int) -> Tuple[int, int]:
        """(K, N) of layer l (0-based)."""
        return self.dims[l], self.dims[l + 1]

    def hidden_act_of(self, l: int) -> str:
        """Activation of hidden layer l (0-based): hidden_act is one name for all of them or one name per layer."""
        return self.hidden_act if isinstance(self.hidden_act, str) else self.hidden_act[l]

    def macs_per_frame(self) -> int:
        return sum(self.dims[l] * self.dims[l + 1] for l in range(self.n_layers))

    def binbin_macs_per_frame(self) -> int:
        """MACs of the layers whose input is binary (the previous layer's activation is Sign or the (0, 1) step)."""
        return sum(self.dims[l] * self.dims[l + 1] for l in range(1, self.n_layers)
                   if self.hidden_act_of(l - 1) in ("sign", "step01") and l not in self.real_weight_layers)


@dataclass(frozen=True)
class GemmShape:
    M: int
    K: int
    N: int


CONFIGS = {
    1: NetConfig(1, "C1 tiny 440-3x512-1000 sign M=64", (440, 512, 512, 512, 1000), 64, "sign", 32),
    2: NetConfig(2, "C2 binW/realX 440-6x2048-3400 hardtanh M=4096",
                 (440,) + (2048,) * 6 + (3400,), 4096, "hardtanh", 32),
    3: NetConfig(3, "C3 binW/binX 440-6x2048-3400 sign M=4096",
                 (440,) + (2048,) * 6 + (3400,), 4096, "sign", 32),
    4: NetConfig(4, "C4 binW/binX 440-6x4096-4000 sign M=16384 w64",
                 (440,) + (4096,) * 6 + (4000,), 16384, "sign", 64),
    # the paper's own two network shapes (Sec. 3): 6 x 1024 units with 3307 tied states, 6 x 2048 units with 3972;
    # their output sizes are no multiple of 4, 32 or 128
    6: NetConfig(6, "C6 binW/binX 440-6x1024-3307 sign M=4096 (WSJ-shaped)",
                 (440,) + (1024,) * 6 + (3307,), 4096, "sign", 32),
    7: NetConfig(7, "C7 binW/binX 440-6x2048-3972 sign M=4096 (AMI-shaped)",
                 (440,) + (2048,) * 6 + (3972,), 4096, "sign", 32),
    # Config 3 with the hidden activations binarised to (0, 1) instead of (-1, +1) (Sec. 3.2, Tables 3 and 4)
    8: NetConfig(8, "C8 binW/binX(0,1) 440-6x2048-3400 step01 M=4096",
                 (440,) + (2048,) * 6 + (3400,), 4096, "step01", 32),
    # the topology the paper's binary-activation systems keep (Sec. 3.2, Table 2: sigma, b, b, b, b, sigma, delta):
    # Sigmoid in the first and last hidden layer, binary activations in between; binary weights in every layer here
    9: NetConfig(9, "C9 binW 440-6x2048-3400 (sigmoid,sign,sign,sign,sign,sigmoid) M=4096",
                 (440,) + (2048,) * 6 + (3400,), 4096, ("sigmoid", "sign", "sign", "sign", "sign", "sigmoid"), 32),
    # the same topology as the paper deploys it (Sec. 2.2 end, Sec. 3.1, Table 2 rows 1-3): the input layer and the
    # Softmax layer keep real-valued weights, only the intermediate hidden layers have binary weights
    10: NetConfig(10, "C10 realW in/out, binW between, 440-6x2048-3400 (sigmoid,sign,sign,sign,sign,sigmoid) M=4096",
                  (440,) + (2048,) * 6 + (3400,), 4096, ("sigmoid", "sign", "sign", "sign", "sign", "sigmoid"), 32,
                  real_weight_layers=(0, 6)),
}

GEMM_SWEEP: List[GemmShape] = [GemmShape(M, K, N)
                               for M in (4096, 65536) for K in (2048, 8192) for N in (2048, 8192)]


def get_config(cfg_id: int) -> NetConfig:
    return CONFIGS[cfg_id]


def _tid(cfg_id: int, layer: int, kind: int) -> int:
    return 100 * cfg_id + 10 * layer + kind


def make_net_params(cfg: NetConfig):
    """Real-valued weights [N,K] ~ U(-1,1) and biases [N] ~ N(0, 0.1^2) for every layer.

    A layer that keeps its real-valued weights gets them scaled by sqrt(3/K) (unit-variance pre-activations for
    unit-variance inputs, the range a trained layer works in); a binarised layer's scale is its mean |w| anyway.
    """
    Ws, bs = [], []
    for l in range(cfg.n_layers):
        K, N = cfg.layer_shape(l)
        W = uniform_pm1(cfg.seed, _tid(cfg.cfg_id, l + 1, TENSOR_W), N * K).reshape(N, K)
        if l in cfg.real_weight_layers:
            W = (W * np.float32(np.sqrt(3.0 / K))).astype(np.float32)
        Ws.append(W)
        bs.append(normal(cfg.seed, _tid(cfg.cfg_id, l + 1, TENSOR_BIAS), N, std=0.1))
    return Ws, bs


def make_frames(cfg: NetConfig, M: int | None = None, start: int = 0) -> np.ndarray:
    """Input frames [M, K0] ~ N(0,1); frames start..start+M-1 of the config's stream."""
    M = cfg.M if M is None else M
    K0 = cfg.dims[0]
    return normal(cfg.seed, _tid(cfg.cfg_id, 0, TENSOR_INPUT), M * K0, start=start * K0).reshape(M, K0)
