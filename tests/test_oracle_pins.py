"""Pins for the CPU oracle: every check compares it with something other than itself.

Sources of truth used here: hand-worked fixtures under tests/golden/ (derived from
the paper's Eq. 1-3 and Alg. 1-2 forward), numpy's matmul / sequential cumsum,
exact rational arithmetic, scipy's log-softmax, closed forms and invariants.
The paper prints no numeric example, so no value below comes from printed results.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

GOLD = os.path.join(os.path.dirname(__file__), "golden")
K_LIST = [1, 31, 32, 33, 63, 64, 65, 127, 129, 440, 2048]


def _rng(seed):
    return np.random.default_rng(seed)


def _pm1(rng, rows, K):
    return (rng.integers(0, 2, size=(rows, K)) * 2 - 1).astype(np.int8)


# ----------------------------------------------------------------------------- Eq. 3 + storage

def test_sign_pack_hand_cases(oracle):
    with open(os.path.join(GOLD, "sign_pack_cases.txt")) as f:
        lines = [ln for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(lines) >= 4
    for ln in lines:
        wb, vals, words = [s.strip() for s in ln.split("|")]
        wb = int(wb)
        x = np.array([float(v) for v in vals.split()], dtype=np.float32)[None, :]
        want = [int(w, 16) for w in words.split()]
        got = oracle.pack_sign(x, wb)
        assert got.shape == (1, len(want))
        assert [int(v) for v in got[0]] == want, ln


def test_sign_is_strictly_positive_test(oracle):
    # Eq. 3: only v > 0 maps to +1.
    x = np.array([[0.0, -0.0, np.nan, -np.nan, np.float32(1e-45), -np.float32(1e-45), np.inf, -np.inf]],
                 dtype=np.float32)
    assert int(oracle.pack_sign(x, 32)[0, 0]) == 0b01010000
    assert oracle.unpack_pm1(oracle.pack_sign(x, 32), 8, 32).tolist() == [[-1, -1, -1, -1, 1, -1, 1, -1]]


@pytest.mark.parametrize("K", K_LIST)
def test_pack_bit_positions_and_padding(oracle, K):
    rng = _rng(K)
    v = _pm1(rng, 5, K)
    x = v.astype(np.float32) * rng.uniform(0.1, 3.0, size=v.shape).astype(np.float32)
    for wb in (32, 64):
        words = oracle.pack_sign(x, wb)
        # independent decoding through numpy's bit unpacking of the little-endian bytes
        bits = np.unpackbits(words.view(np.uint8).reshape(5, -1), axis=1, bitorder="little")
        assert np.array_equal(bits[:, :K], (v > 0).astype(np.uint8))
        assert not bits[:, K:].any(), "pad bits must be 0"
        assert np.array_equal(oracle.unpack_pm1(words, K, wb), v)


def test_word32_and_word64_rows_are_byte_identical(oracle):
    rng = _rng(7)
    x = rng.standard_normal((6, 640)).astype(np.float32)      # 640 = 20 x 32 = 10 x 64
    b32 = oracle.pack_sign(x, 32).view(np.uint8)
    b64 = oracle.pack_sign(x, 64).view(np.uint8)
    assert np.array_equal(b32, b64)


def test_mean_abs(oracle):
    w = np.array([[0.5, -0.25, 1.0], [-0.75, 0.0, -0.5]], dtype=np.float32)
    assert oracle.mean_abs(w) == np.float32(0.5)
    rng = _rng(3)
    w = rng.uniform(-1, 1, size=(64, 129)).astype(np.float32)
    exact = sum(Fraction(abs(float(v))) for v in w.ravel()) / w.size
    got = Fraction(float(oracle.mean_abs(w)))
    assert abs(got - exact) <= Fraction(float(np.spacing(np.float32(float(exact))))), "within 1 ulp of the exact mean"
    assert abs(float(oracle.mean_abs(w)) - 0.5) < 0.02


# ----------------------------------------------------------------------------- +-1 products

@pytest.mark.parametrize("K", K_LIST)
def test_dot_pm1_vs_numpy_matmul(oracle, K):
    rng = _rng(100 + K)
    a, b = _pm1(rng, 7, K), _pm1(rng, 5, K)
    want = a.astype(np.float64) @ b.astype(np.float64).T          # library routine on +-1 floats (exact)
    got = oracle.dot_pm1(a, b)
    assert got.shape == (7, 5) and got.dtype == np.int32
    assert np.array_equal(got, want.astype(np.int32))
    want32 = a.astype(np.float32) @ b.astype(np.float32).T          # also exact in fp32 (|dot| < 2^24)
    assert np.array_equal(got, want32.astype(np.int32))


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("K", K_LIST)
def test_dot_xor_equals_definition(oracle, K, wb):
    rng = _rng(200 + K)
    a, b = _pm1(rng, 9, K), _pm1(rng, 6, K)
    aw, bw = oracle.pack_sign(a.astype(np.float32), wb), oracle.pack_sign(b.astype(np.float32), wb)
    got = oracle.dot_xor(aw, bw, K, wb)
    assert np.array_equal(got, (a.astype(np.int64) @ b.astype(np.int64).T).astype(np.int32))
    assert np.array_equal(got, oracle.dot_pm1(a, b))
    assert np.all(np.abs(got) <= K)
    assert np.all((got - K) % 2 == 0), "dot and K have the same parity"


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("K", [1, 33, 64, 440, 2048])
def test_dot_xor_closed_forms(oracle, K, wb):
    rng = _rng(300 + K)
    a = _pm1(rng, 4, K)
    aw = oracle.pack_sign(a.astype(np.float32), wb)
    nw = oracle.pack_sign((-a).astype(np.float32), wb)             # complement on the valid bits only
    assert np.array_equal(np.diag(oracle.dot_xor(aw, aw, K, wb)), np.full(4, K))
    assert np.array_equal(np.diag(oracle.dot_xor(aw, nw, K, wb)), np.full(4, -K))
    if K % 2 == 0:
        half = a.copy()
        half[:, : K // 2] *= -1                                      # differs in exactly K/2 places
        hw = oracle.pack_sign(half.astype(np.float32), wb)
        assert np.array_equal(np.diag(oracle.dot_xor(aw, hw, K, wb)), np.zeros(4))


def test_sign_symmetry(oracle):
    rng = _rng(5)
    K = 440
    a, b = _pm1(rng, 6, K), _pm1(rng, 8, K)
    base = oracle.dot_pm1(a, b)
    b2 = b.copy(); b2[3] *= -1
    d = oracle.dot_pm1(a, b2)
    assert np.array_equal(d[:, 3], -base[:, 3]) and np.array_equal(np.delete(d, 3, 1), np.delete(base, 3, 1))
    a2 = a.copy(); a2[2] *= -1
    d = oracle.dot_pm1(a2, b)
    assert np.array_equal(d[2], -base[2]) and np.array_equal(np.delete(d, 2, 0), np.delete(base, 2, 0))
    # the same in the bit domain
    for wb in (32, 64):
        aw, bw = oracle.pack_sign(a.astype(np.float32), wb), oracle.pack_sign(b.astype(np.float32), wb)
        b2w = oracle.pack_sign(b2.astype(np.float32), wb)
        assert np.array_equal(oracle.dot_xor(aw, b2w, K, wb)[:, 3], -oracle.dot_xor(aw, bw, K, wb)[:, 3])


def test_operands_are_not_transposed(oracle):
    # a is [M,K], b is [N,K], result [M,N]: a one-hot difference lands where the definition says.
    K = 40
    a = np.ones((3, K), np.int8); b = np.ones((4, K), np.int8)
    a[1, :10] = -1          # row 1 of a differs in 10 places -> dot[1, :] = K - 20
    b[2, :3] = -1           # row 2 of b has 3 places -> overlap with a[1]: 3 agree again
    got = oracle.dot_pm1(a, b)
    want = np.full((3, 4), K, np.int32)
    want[1, :] = K - 20
    want[:, 2] = K - 6
    want[1, 2] = K - 2 * 7
    assert np.array_equal(got, want)
    aw, bw = oracle.pack_sign(a.astype(np.float32), 32), oracle.pack_sign(b.astype(np.float32), 32)
    assert np.array_equal(oracle.dot_xor(aw, bw, K, 32), want)


def test_dot_statistics(oracle):
    rng = _rng(11)
    K = 2048
    d = oracle.dot_pm1(_pm1(rng, 64, K), _pm1(rng, 256, K)).astype(np.float64)
    assert abs(d.mean()) < 1.5 and abs(d.var() / K - 1.0) < 0.05


# ----------------------------------------------------------------------------- real input x binary weights

@pytest.mark.parametrize("K", [1, 2, 33, 440, 2048])
def test_realx_acc_vs_library_and_sequential_cumsum(oracle, K):
    rng = _rng(400 + K)
    x = rng.standard_normal((5, K)).astype(np.float32)
    w = _pm1(rng, 7, K)
    acc32, acc64 = oracle.realx_acc(x, w)
    # fp64 shadow == library GEMM up to fp64 rounding of a K-term sum
    want64 = x.astype(np.float64) @ w.astype(np.float64).T
    bound = K * np.finfo(np.float64).eps * (np.abs(x).astype(np.float64).sum(1, keepdims=True))
    assert np.all(np.abs(acc64 - want64) <= bound + 1e-300)
    # identity: sum_k x - 2 * sum_{w=-1} x
    alt = x.astype(np.float64).sum(1)[:, None] - 2.0 * (x.astype(np.float64) @ (w < 0).astype(np.float64).T)
    assert np.all(np.abs(acc64 - alt) <= 4 * bound + 1e-300)
    # canonical fp32 order == numpy's sequential fp32 cumulative sum of the signed terms
    for m in range(5):
        for n in range(7):
            terms = (x[m] * w[n].astype(np.float32)).astype(np.float32)       # exact: +-x
            assert acc32[m, n] == np.cumsum(terms, dtype=np.float32)[-1]
    # fp32 result stays within the classical bound of the exact sum
    u = 2.0 ** -24
    assert np.all(np.abs(acc32.astype(np.float64) - acc64) <= (K * u / (1 - K * u)) * np.abs(x).astype(np.float64).sum(1)[:, None])


def test_realx_order_is_ascending_k(oracle):
    # 2^24 + 1 + 1 ... : in ascending order every +1 is absorbed; in any other order it is not.
    K = 9
    x = np.array([[2.0 ** 24] + [1.0] * 8], dtype=np.float32)
    w = np.ones((1, K), np.int8)
    acc32, acc64 = oracle.realx_acc(x, w)
    assert acc32[0, 0] == np.float32(2.0 ** 24) and acc64[0, 0] == 2.0 ** 24 + 8
    acc32r, _ = oracle.realx_acc(x[:, ::-1].copy(), w)
    assert acc32r[0, 0] == np.float32(2.0 ** 24 + 8)
    # subtraction really subtracts
    w2 = np.array([[1, -1, -1, 1, 1, 1, 1, 1, 1]], np.int8)
    assert oracle.realx_acc(np.arange(1, 10, dtype=np.float32)[None], w2)[0][0, 0] == 1 - 2 - 3 + 4 + 5 + 6 + 7 + 8 + 9


def test_realx_special_cases(oracle):
    rng = _rng(17)
    K = 257
    x = rng.standard_normal((4, K)).astype(np.float32)
    ones = np.ones((1, K), np.int8)
    acc32, acc64 = oracle.realx_acc(x, ones)
    assert np.allclose(acc64[:, 0], x.astype(np.float64).sum(1), rtol=0, atol=1e-12)
    # x in {-1,+1}: equals the binary product exactly
    a, b = _pm1(rng, 6, K), _pm1(rng, 5, K)
    acc32, acc64 = oracle.realx_acc(a.astype(np.float32), b)
    assert np.array_equal(acc32, oracle.dot_pm1(a, b).astype(np.float32))
    assert np.array_equal(acc64, oracle.dot_pm1(a, b).astype(np.float64))


# ----------------------------------------------------------------------------- real input x real weights

@pytest.mark.parametrize("K", [1, 2, 33, 440, 2048])
def test_realw_acc_vs_library_gemm(oracle, K):
    rng = _rng(900 + K)
    x = rng.standard_normal((5, K)).astype(np.float32)
    w = (rng.standard_normal((7, K)) / math.sqrt(K)).astype(np.float32)
    acc32, acc64 = oracle.realw_acc(x, w)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    want64 = x64 @ w64.T                                # library GEMM, any order
    mag = np.abs(x64) @ np.abs(w64).T                   # sum_k |w x|
    assert np.all(np.abs(acc64 - want64) <= K * np.finfo(np.float64).eps * mag + 1e-300)
    u = 2.0 ** -24                                      # one rounding per step: the classical bound K u / (1 - K u)
    assert np.all(np.abs(acc32.astype(np.float64) - want64) <= (K * u / (1 - K * u)) * mag + 1e-300)
    # transposing the operands' roles must not matter: (x w^T)^T = w x^T
    accT, _ = oracle.realw_acc(w, x)
    assert np.array_equal(accT, acc32.T)                # products commute exactly, the order in k is the same


def test_realw_reduces_to_the_binary_weight_product(oracle):
    # every weight +1 or -1: each fused multiply-add is an exact add or subtract, i.e. Alg. 1's product, bit for bit
    rng = _rng(41)
    for K in (31, 440, 1000):
        x = rng.standard_normal((6, K)).astype(np.float32)
        w = _pm1(rng, 9, K)
        a32, a64 = oracle.realw_acc(x, w.astype(np.float32))
        b32, b64 = oracle.realx_acc(x, w)
        assert np.array_equal(a32, b32) and np.array_equal(a64, b64)


def test_realw_order_and_single_rounding(oracle):
    one = np.ones((1, 3), np.float32)
    # ascending k: 1e8 - 1e8 + 1 = 1, but 1 + 1e8 - 1e8 = 0 in fp32
    assert oracle.realw_acc(np.array([[1e8, -1e8, 1.0]], np.float32), one)[0][0, 0] == 1.0
    assert oracle.realw_acc(np.array([[1.0, 1e8, -1e8]], np.float32), one)[0][0, 0] == 0.0
    # one rounding per step: (1 + 2^-12)^2 - (1 + 2^-11) = 2^-24 exactly; a rounded product would give 0
    a = np.float32(1 + 2.0 ** -12)
    x = np.array([[-(1 + 2.0 ** -11), a]], np.float32)
    w = np.array([[1.0, a]], np.float32)
    acc32, acc64 = oracle.realw_acc(x, w)
    assert acc32[0, 0] == np.float32(2.0 ** -24) and acc64[0, 0] == 2.0 ** -24
    # exact small integers
    x = np.arange(1, 7, dtype=np.float32)[None]
    w = np.array([[2, -1, 0, 3, -2, 1]], np.float32)
    assert oracle.realw_acc(x, w)[0][0, 0] == 2 - 2 + 0 + 12 - 10 + 6


def test_bits_to_real(oracle):
    rng = _rng(5)
    for wb in (32, 64):
        for K in (1, 31, 33, 64, 65, 130):
            v = rng.standard_normal((3, K)).astype(np.float32)
            words = oracle.pack_sign(v, wb)
            assert np.array_equal(oracle.bits_to_real(words, K, wb, False), np.where(v > 0, 1.0, -1.0).astype(np.float32))
            assert np.array_equal(oracle.bits_to_real(words, K, wb, True), (v > 0).astype(np.float32))


def test_real_weight_network_vs_independent_numpy(oracle):
    # (sigmoid, sign, step01, sigmoid) hidden layers, real weights in the first, third and last layer, the rest binary
    import workloads
    cfg = workloads.NetConfig(11, "pin", (40, 64, 70, 48, 33, 21), 9, ("sigmoid", "sign", "step01", "sigmoid"), 32,
                              real_weight_layers=(0, 2, 4))
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg)
    layers = oracle.make_layers(Ws, bs, cfg.hidden_act, 32, real_weight_layers=cfg.real_weight_layers)
    got, outs = oracle.forward(layers, X, keep=True)
    # independent fp64 restatement; the binary layers' inputs are taken from the oracle's own bits so that a
    # pre-activation within rounding of zero cannot make the two diverge
    h = X.astype(np.float64)
    for l, (W, r) in enumerate(zip(Ws, bs)):
        W64 = W.astype(np.float64) if l in cfg.real_weight_layers else np.where(W > 0, 1.0, -1.0) * np.float64(np.float32(np.mean(np.abs(W), dtype=np.float64)))
        z = h @ W64.T + r.astype(np.float64)
        act = "logsoftmax" if l == len(Ws) - 1 else cfg.hidden_act[l]
        if act == "sigmoid":
            h = 1.0 / (1.0 + np.exp(-z))
            assert np.max(np.abs(outs[l] - h)) <= 2e-6
        elif act in ("sign", "step01"):
            bits = oracle.unpack_01(outs[l], W.shape[0], 32).astype(bool)
            clear = np.abs(z) > 1e-4
            assert np.array_equal(bits[clear], (z > 0)[clear]) and clear.mean() > 0.99
            h = np.where(bits, 1.0, -1.0 if act == "sign" else 0.0)
        else:
            want = z - scipy.special.logsumexp(z, axis=1, keepdims=True)
            assert np.max(np.abs(got - want)) <= 1e-5


# ----------------------------------------------------------------------------- affine step

def _nearest_f32(fr: Fraction) -> np.float32:
    """Correctly rounded (ties-to-even) fp32 of an exact rational, without any floating-point shortcut."""
    c = np.float32(float(fr))                       # a candidate within 1 ulp
    best = None
    for cand in (np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))):
        err = abs(Fraction(float(cand)) - fr)
        mant_even = (int(np.float32(cand).view(np.uint32)) & 1) == 0
        key = (err, 0 if mant_even else 1)
        if best is None or key < best[0]:
            best = (key, np.float32(cand))
    return best[1]


def test_affine_is_one_correctly_rounded_fma(oracle):
    rng = _rng(23)
    N = 64
    scale = rng.uniform(0.3, 0.7, N).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float32)
    dots = rng.integers(-2048, 2049, size=(8, N)).astype(np.int32)
    got = oracle.affine_f32(oracle.i32_to_f32(dots), scale, bias)
    n_differs_from_two_roundings = 0
    for m in range(8):
        for n in range(N):
            exact = Fraction(float(scale[n])) * int(dots[m, n]) + Fraction(float(bias[n]))
            assert got[m, n] == _nearest_f32(exact)
            two = np.float32(np.float32(scale[n] * np.float32(dots[m, n])) + bias[n])
            n_differs_from_two_roundings += int(two != got[m, n])
    assert n_differs_from_two_roundings > 0, "the sample must be able to tell an fma from mul-then-add"
    # NULL scale = 1, NULL bias = 0
    v = rng.standard_normal((3, N)).astype(np.float32)
    assert np.array_equal(oracle.affine_f32(v, None, None), v)
    assert np.array_equal(oracle.affine_f32(v, None, bias), (v.astype(np.float64) + bias).astype(np.float32))


def test_affine_f64_against_exact_rationals(oracle):
    # Eq. 1 carried in fp64: scale[n] * v[m][n] + bias[n] with the fp32 scale and bias widened exactly.  The exact
    # rational value is within two fp64 roundings (product, then sum) of what the function returns; a swapped scale and
    # bias, a transposed index (scale[m] for scale[n]) or a missing term is off by far more than that.
    rng = _rng(31)
    M, N = 5, 48
    scale = rng.uniform(0.3, 0.7, N).astype(np.float32)
    scale[::7] *= -1.0
    bias = (rng.standard_normal(N) * 3.0).astype(np.float32)
    v = rng.standard_normal((M, N)) * 200.0
    got = oracle.affine_f64(v, scale, bias)
    assert got.dtype == np.float64 and got.shape == (M, N)
    for m in range(M):
        for n in range(N):
            prod = Fraction(float(scale[n])) * Fraction(float(v[m, n]))
            exact = prod + Fraction(float(bias[n]))
            bound = (abs(prod) + abs(exact)) * Fraction(1, 2 ** 52)
            assert abs(Fraction(float(got[m, n])) - exact) <= bound, (m, n)
            swapped = Fraction(float(bias[n])) * Fraction(float(v[m, n])) + Fraction(float(scale[n]))
            assert abs(swapped - exact) > 1000 * bound, "the sample must tell scale from bias"
    # integer products (24-bit scale x |dot| <= 2048) are exact in fp64: one rounding, of the sum, is left
    dots = rng.integers(-2048, 2049, size=(M, N)).astype(np.float64)
    got = oracle.affine_f64(dots, scale, bias)
    for m in range(M):
        for n in range(N):
            exact = Fraction(float(scale[n])) * int(dots[m, n]) + Fraction(float(bias[n]))
            assert abs(Fraction(float(got[m, n])) - exact) <= abs(exact) * Fraction(1, 2 ** 53)
    # NULL scale = 1, NULL bias = 0
    assert np.array_equal(oracle.affine_f64(v, None, None), v)
    assert np.array_equal(oracle.affine_f64(v, None, bias), v + bias.astype(np.float64)[None, :])
    assert np.array_equal(oracle.affine_f64(v, scale, None), scale.astype(np.float64)[None, :] * v)
    # it is the fp64 companion of the fp32 affine step: the two agree to fp32 rounding on fp32 inputs
    v32 = v.astype(np.float32)
    h32 = oracle.affine_f32(v32, scale, bias)
    h64 = oracle.affine_f64(v32.astype(np.float64), scale, bias)
    assert np.array_equal(h32, h64.astype(np.float32)) or np.max(np.abs(h32 - h64)) <= 2e-5


def test_sign_bit_is_monotone_in_dot(oracle):
    # for fixed scale > 0 the bit (h^ > 0) switches once from 0 to 1 as dot grows; for scale < 0 once from 1 to 0
    K = 2048
    dots = np.arange(-K, K + 1, 2, dtype=np.int32)[:, None]
    rng = _rng(29)
    for s in (0.5, 0.4999, -0.5, 1.0):
        for b in rng.standard_normal(5) * 3:
            h = oracle.affine_f32(oracle.i32_to_f32(dots), np.array([s], np.float32), np.array([b], np.float32))
            bits = (h[:, 0] > 0).astype(int)
            assert (np.abs(np.diff(bits)).sum()) <= 1
            if s > 0:
                assert np.all(np.diff(bits) >= 0)
            else:
                assert np.all(np.diff(bits) <= 0)


def test_hardtanh(oracle):
    h = np.array([-3.0, -1.0, -0.5, 0.0, 0.25, 1.0, 1.5, np.inf, -np.inf], np.float32)
    assert oracle.hardtanh(h).tolist() == [-1.0, -1.0, -0.5, 0.0, 0.25, 1.0, 1.0, 1.0, -1.0]


# ----------------------------------------------------------------------------- log-softmax

def test_sigmoid_vs_scipy_and_identities(oracle):
    from scipy.special import expit
    rng = np.random.default_rng(9)
    v = np.concatenate([rng.standard_normal(1000) * 8, [0.0, -0.0, 1e-30, -1e-30, 88.0, -88.0, 104.0, -104.0, 1e30, -1e30]]).astype(np.float32)
    got = oracle.sigmoid(v)
    assert got.dtype == np.float32
    assert np.array_equal(got, expit(v.astype(np.float64)).astype(np.float32))     # library routine, same rounding
    assert oracle.sigmoid(np.zeros(1, np.float32))[0] == np.float32(0.5)
    assert np.allclose(got.astype(np.float64) + oracle.sigmoid(-v).astype(np.float64), 1.0, atol=2e-7)   # sigma(-v) = 1 - sigma(v)
    order = np.argsort(v, kind="stable")
    assert np.all(np.diff(got[order]) >= 0)                                         # monotone
    assert got.min() >= 0.0 and got.max() <= 1.0
    assert oracle.sigmoid(np.array([1e30], np.float32))[0] == 1.0 and oracle.sigmoid(np.array([-1e30], np.float32))[0] == 0.0


def test_log_softmax_vs_scipy_and_invariants(oracle):
    rng = _rng(31)
    for N in (2, 1000, 3307, 3400, 3972):
        z = (rng.standard_normal((4, N)) * 20).astype(np.float32)
        o32, o64 = oracle.log_softmax(z)
        want = scipy.special.log_softmax(z.astype(np.float64), axis=1)
        assert np.max(np.abs(o64 - want)) < 1e-11
        assert np.array_equal(o32, o64.astype(np.float32))
        assert np.allclose(np.exp(o64).sum(1), 1.0, atol=1e-12)
        assert np.array_equal(o64.argmax(1), z.argmax(1))
        # shift invariance (a power-of-two shift of power-of-two-spaced values keeps the fp32 inputs exact)
        zq = np.round(z * 8) / 8
        s32, s64 = oracle.log_softmax((zq + 64.0).astype(np.float32))
        assert np.max(np.abs(s64 - oracle.log_softmax(zq.astype(np.float32))[1])) < 1e-11
    eq = np.full((2, 3400), 1.75, np.float32)
    assert np.allclose(oracle.log_softmax(eq)[1], -math.log(3400), atol=1e-13)
    # huge spread does not overflow
    big = np.array([[1e4, 0.0, -1e4]], np.float32)
    assert np.allclose(oracle.log_softmax(big)[1][0], [0.0, -1e4, -2e4])


# ----------------------------------------------------------------------------- (0, 1) activations (Sec. 3.2)

def test_x01_hand_cases(oracle):
    with open(os.path.join(GOLD, "x01_hand_cases.txt")) as f:
        rows = [ln.split("|") for ln in f if ln.strip() and not ln.startswith("#")]
    for hs, ws, ds in rows:
        h = np.array([[int(v) for v in hs.split()]], np.int8)
        w = np.array([[int(v) for v in ws.split()]], np.int8)
        want = int(ds)
        assert oracle.dot_x01_wpm1(h, w)[0, 0] == want
        K = h.shape[1]
        for wb in (32, 64):
            hp = oracle.pack_sign(h.astype(np.float32), wb)           # bit 1 <=> h = 1 (h > 0)
            wp = oracle.pack_sign(w.astype(np.float32), wb)
            assert oracle.unpack_01(hp, K, wb).tolist() == h.tolist()
            assert oracle.dot_and(hp, wp, K, wb)[0, 0] == want


@pytest.mark.parametrize("K", [1, 31, 32, 33, 63, 64, 65, 440, 2048])
def test_x01_vs_numpy_and_packed_form(oracle, K):
    rng = np.random.default_rng(K)
    M, N = 7, 9
    h = rng.integers(0, 2, (M, K)).astype(np.int8)
    w = (2 * rng.integers(0, 2, (N, K)) - 1).astype(np.int8)
    want = h.astype(np.int64) @ w.astype(np.int64).T                   # library integer matmul
    assert np.array_equal(oracle.dot_x01_wpm1(h, w), want)
    # not transposed: a non-square case with distinct rows
    assert oracle.dot_x01_wpm1(h[:2], w[:5]).shape == (2, 5)
    for wb in (32, 64):
        hp, wp = oracle.pack_sign(h.astype(np.float32), wb), oracle.pack_sign(w.astype(np.float32), wb)
        assert np.array_equal(oracle.dot_and(hp, wp, K, wb), want)
        # relation to the -1/+1 product of the same bits: h = (a + 1) / 2  =>  h.w = (a.w + sum_k w_k) / 2
        a_dot = oracle.dot_xor(hp, wp, K, wb).astype(np.int64)
        assert np.array_equal(2 * want, a_dot + w.astype(np.int64).sum(1)[None, :])
    # closed forms: no active input -> 0; every input active -> the row sum of the weights; all weights +1 -> popcount(h)
    assert np.array_equal(oracle.dot_x01_wpm1(np.zeros((1, K), np.int8), w), np.zeros((1, N)))
    assert np.array_equal(oracle.dot_x01_wpm1(np.ones((1, K), np.int8), w)[0], w.astype(np.int64).sum(1))
    assert np.array_equal(oracle.dot_x01_wpm1(h, np.ones((1, K), np.int8))[:, 0], h.astype(np.int64).sum(1))
    # unlike the -1/+1 product it is NOT odd in the activations: complementing h gives (sum_k w_k) - dot
    assert np.array_equal(oracle.dot_x01_wpm1(1 - h, w), w.astype(np.int64).sum(1)[None, :] - want)


def test_x01_network_vs_independent_numpy(oracle):
    """A small network with (0, 1) hidden activations: the oracle's forward against plain numpy on unpacked values."""
    rng = np.random.default_rng(5)
    dims = (13, 40, 33, 17)
    Ws = [rng.uniform(-1, 1, (dims[i + 1], dims[i])).astype(np.float32) for i in range(3)]
    bs = [(0.1 * rng.standard_normal(dims[i + 1])).astype(np.float32) for i in range(3)]
    X = rng.standard_normal((6, 13)).astype(np.float32)
    for wb in (32, 64):
        layers = oracle.make_layers(Ws, bs, "step01", wb)
        out_def, keep = oracle.forward(layers, X, form="definition", keep=True)
        out_pk = oracle.forward(layers, X, form="xor")
        assert np.array_equal(out_def, out_pk)
        # plain numpy: layer 1 real input (ascending-k fp32 sum via cumsum), then {0,1} activations against +-1 weights
        S = [np.where(W > 0, 1.0, -1.0).astype(np.float32) for W in Ws]
        sc = [np.float32(np.abs(W.astype(np.float64)).mean()) for W in Ws]
        acc = np.stack([[np.cumsum((S[0][n] * x).astype(np.float32), dtype=np.float32)[-1] for n in range(dims[1])] for x in X])
        h = (np.float32(sc[0]) * acc.astype(np.float32) + bs[0] > 0)
        assert np.array_equal(oracle.unpack_01(keep[0], dims[1], wb), h.astype(np.int8))
        d2 = h.astype(np.int64) @ S[1].astype(np.int64).T
        z2 = (sc[1].astype(np.float64) * d2 + bs[1].astype(np.float64))
        h2 = z2 > 0
        clear = np.abs(z2) > 1e-4                                         # away from fp32 rounding of the affine step
        assert np.array_equal(oracle.unpack_01(keep[1], dims[2], wb)[clear], h2.astype(np.int8)[clear])


# ----------------------------------------------------------------------------- layers and network

def _load_hand():
    d = {}
    with open(os.path.join(GOLD, "hand_worked_network.txt")) as f:
        for ln in f:
            if ln.strip() and not ln.startswith("#"):
                name, *vals = ln.split()
                d[name] = [float(v) for v in vals]
    return d


def test_hand_worked_network(oracle):
    g = _load_hand()
    W1 = np.array(g["W1"], np.float32).reshape(2, 3); r1 = np.array(g["r1"], np.float32)
    W2 = np.array(g["W2"], np.float32).reshape(2, 2); r2 = np.array(g["r2"], np.float32)
    X = np.array(g["X"], np.float32).reshape(2, 3)
    for wb in (32, 64):
        layers = oracle.make_layers([W1, W2], [r1, r2], "sign", wb)
        assert [int(v) for v in layers[0].w_words[:, 0]] == [int(v) for v in g["W1_words"]]
        assert [int(v) for v in layers[1].w_words[:, 0]] == [int(v) for v in g["W2_words"]]
        assert float(layers[0].scale[0]) == g["scale1"][0] and float(layers[1].scale[0]) == g["scale2"][0]
        acc32, acc64 = oracle.realx_acc(X, oracle.unpack_pm1(layers[0].w_words, 3, wb))
        assert acc32.ravel().tolist() == g["acc1"] and acc64.ravel().tolist() == g["acc1"]
        assert oracle.affine_f32(acc32, layers[0].scale, layers[0].bias).ravel().tolist() == g["hhat1"]
        for form in ("definition", "xor"):
            out, keep = oracle.forward(layers, X, form=form, keep=True)
            assert [int(v) for v in keep[0][:, 0]] == [int(v) for v in g["h1_words"]]
            dot2 = oracle.layer_binw_binx(keep[0], layers[1].w_words, 2, None, None, "raw", wb, form=form)
            assert dot2.ravel().tolist() == g["dot2"]
            z = np.array(g["z"]).reshape(2, 2)
            lse = np.array([off + math.log1p(math.exp(-0.75)) for off in g["lse_offset"]])[:, None]
            assert np.max(np.abs(out.astype(np.float64) - (z - lse))) < 1e-7


def _independent_forward(Ws, bs, X, hidden_act):
    """A second, numpy-only statement of the same network, sharing nothing with oracle/.

    +-1 matrices as floats and library matmuls for the binary layers (exact in fp64),
    numpy's sequential fp32 cumsum for the real-input layer.
    """
    h = X.astype(np.float32)
    binary = False
    L = len(Ws)
    for l, (W, r) in enumerate(zip(Ws, bs)):
        Wb = np.where(W > 0, 1.0, -1.0)
        alpha = np.float32(np.abs(W.astype(np.float64)).sum() / W.size)
        if binary:
            acc = (h.astype(np.float64) @ Wb.T).astype(np.float32)                 # exact integers
        else:
            terms = h[:, None, :] * Wb[None, :, :].astype(np.float32)               # [M,N,K], exact +-x
            acc = np.cumsum(terms, axis=2, dtype=np.float32)[:, :, -1]
        # exact fma through fp64: scale*acc has <= 48 significant bits, so the fp64 product is exact; the
        # fp64 sum is then rounded once more to fp32 - double rounding can differ from a true fma only on
        # a tie of the fp64 sum, which the assertion below rules out for the inputs used.
        prod = alpha.astype(np.float64) * acc.astype(np.float64)
        s = prod + r.astype(np.float64)[None, :]
        hhat = s.astype(np.float32)
        if l == L - 1:
            z = hhat.astype(np.float64)
            return scipy.special.log_softmax(z, axis=1).astype(np.float32)
        if hidden_act == "sign":
            h = np.where(hhat > 0, 1.0, -1.0).astype(np.float32)
            binary = True
        else:
            h = np.clip(hhat, -1.0, 1.0)
            binary = False


@pytest.mark.parametrize("hidden_act", ["sign", "hardtanh"])
def test_small_network_vs_independent_numpy(oracle, hidden_act):
    import workloads
    cfg = workloads.NetConfig(9, "pin", (70, 96, 65, 50), 12, hidden_act, 32)
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg)
    want = _independent_forward(Ws, bs, X, hidden_act)
    for wb in (32, 64):
        layers = oracle.make_layers(Ws, bs, hidden_act, wb)
        for form in ("definition", "xor"):
            got = oracle.forward(layers, X, form=form)
            assert got.shape == want.shape
            if hidden_act == "sign":
                assert np.max(np.abs(got - want)) <= 1e-6
            else:
                assert np.max(np.abs(got - want)) <= 1e-4 * np.max(np.abs(want))


def test_config1_end_to_end_definition_vs_xor_and_numpy(oracle):
    """Config 1 (440 -> 3x512 -> 1000, 64 frames): brute-force definition, XOR form and numpy agree."""
    import workloads
    cfg = workloads.CONFIGS[1]
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg)
    layers = oracle.make_layers(Ws, bs, "sign", 32)
    a, ka = oracle.forward(layers, X, form="definition", keep=True)
    b, kb = oracle.forward(layers, X, form="xor", keep=True)
    for u, v in zip(ka, kb):
        assert np.array_equal(u, v)
    want = _independent_forward(Ws, bs, X, "sign")
    assert np.max(np.abs(a - want)) <= 1e-5
    assert np.allclose(np.exp(a.astype(np.float64)).sum(1), 1.0, atol=1e-5)
    # hidden bits are roughly balanced (bias is small against the spread of the pre-activations)
    for h in ka[:-1]:
        frac = np.unpackbits(h.view(np.uint8), bitorder="little").mean()
        assert 0.4 < frac < 0.6


def test_forward_flipping_a_weight_row_flips_that_hidden_unit(oracle):
    # bias 0 and scale 1: negating every weight of hidden unit j negates h^_j, hence flips its bit
    import workloads
    cfg = workloads.NetConfig(8, "flip", (33, 40, 10), 6, "sign", 32)
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg)
    zero = [np.zeros_like(b) for b in bs]
    l0 = oracle.make_layers(Ws, zero, "sign", 32, use_scale=False)
    _, k0 = oracle.forward(l0, X, keep=True)
    W2 = [w.copy() for w in Ws]
    W2[0][5] *= -1
    _, k1 = oracle.forward(oracle.make_layers(W2, zero, "sign", 32, use_scale=False), X, keep=True)
    h0 = oracle.unpack_pm1(k0[0], 40, 32); h1 = oracle.unpack_pm1(k1[0], 40, 32)
    assert np.array_equal(h1[:, 5], -h0[:, 5]) and np.array_equal(np.delete(h1, 5, 1), np.delete(h0, 5, 1))


def test_subtract_log_prior_bayes_rule_and_rounding(oracle):
    """Two tied states, two frames with known likelihoods and priors: posterior = likelihood x prior / evidence, so
    log-posterior minus log-prior is the log-likelihood up to one constant per frame (a wrong sign, or the prior taken
    along the frames, breaks this).  Then the arithmetic: dyadic values exactly, random values as the correctly rounded
    exact difference."""
    lik = np.array([[0.2, 0.6], [0.05, 0.01]])
    prior = np.array([0.75, 0.25])
    post = lik * prior / (lik * prior).sum(1, keepdims=True)
    out = oracle.subtract_log_prior(np.log(post).astype(np.float32), np.log(prior).astype(np.float32)).astype(np.float64)
    assert np.allclose(out[:, 0] - out[:, 1], np.log(lik[:, 0] / lik[:, 1]), atol=1e-6)
    assert np.array_equal(oracle.subtract_log_prior(np.array([[-0.5, -2.0], [0.0, -8.0]], np.float32), np.array([-1.0, -0.25], np.float32)),
                          np.array([[0.5, -1.75], [1.0, -7.75]], np.float32))
    rng = np.random.default_rng(3)
    a = -rng.uniform(0.01, 300, (7, 11)).astype(np.float32)
    b = -rng.uniform(0.5, 12, 11).astype(np.float32)
    got = oracle.subtract_log_prior(a, b)
    for m in range(7):
        for n in range(11):
            exact = Fraction(float(a[m, n])) - Fraction(float(b[n]))   # fits a double exactly: one rounding to fp32 below
            assert got[m, n] == np.float32(float(exact))
    assert np.array_equal(oracle.subtract_log_prior(a, np.zeros(11, np.float32)), a)
