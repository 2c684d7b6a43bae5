"""GPU parity: the HIP path behind the C ABI against the CPU oracle, element by element.

Bars: bit-exact for packed bits and int32 products (also for the real-input layer, whose fp32 order
of additions is fixed on both sides: ascending k, one accumulator); fp32 outputs within
max|gpu - oracle| <= 1e-4 * max|oracle| ("layer output scale" = L-infinity norm of the oracle tensor).
"""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-4


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


@pytest.fixture(scope="module")
def bnn():
    """The library with the small-batch (streaming) dispatch switched off, so that batches of a few frames exercise the
    large-batch kernels too; the streaming tests switch it on themselves."""
    import paper_1706_09453_amd as b
    b.bnn_set_option(b.BNN_OPT_STREAM_MAX_FRAMES, 0)
    yield b
    b.bnn_set_option(b.BNN_OPT_STREAM_MAX_FRAMES, 64)


class _streaming:
    """Batches of at most `frames` frames take the streaming kernels for the duration of a test."""

    def __init__(self, bnn, frames=64):
        self.bnn, self.frames = bnn, frames

    def __enter__(self):
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_STREAM_MAX_FRAMES, self.frames)

    def __exit__(self, *exc):
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_STREAM_MAX_FRAMES, 0)


def _close(got: np.ndarray, want: np.ndarray, what=""):
    scale = float(np.max(np.abs(want)))
    err = float(np.max(np.abs(got.astype(np.float64) - want.astype(np.float64))))
    assert np.isfinite(got).all(), what
    assert err <= TOL * scale, f"{what}: max abs err {err:g} > {TOL:g} * {scale:g}"


ARMS = ["valu", "mfma16", "mfma32", "mfma32wm2", "mfma32rot", "mfma32wm2rot", "mfma32xcd", "mfma_i8"]


class _arm:
    """Select the arithmetic arm (and the MFMA shape) of the binary product for the duration of a test."""

    def __init__(self, bnn, name):
        self.bnn, self.name = bnn, name

    def __enter__(self):
        b = self.bnn
        if self.name == "mfma_i8":
            return b.BNN_ARM_MFMA_I8
        if self.name != "valu":
            b.bnn_set_option(b.BNN_OPT_MFMA_SHAPE, 16 if self.name == "mfma16" else 32)
            b.bnn_set_option(b.BNN_OPT_MFMA32_WM, 2 if "wm2" in self.name else 4)
            b.bnn_set_option(b.BNN_OPT_MFMA32_PIPELINE, 2 if self.name.endswith("rot") else 0)
            b.bnn_set_option(b.BNN_OPT_MFMA32_XCD_ORDER, 1 if self.name.endswith("xcd") else 0)
        return b.BNN_ARM_VALU_XOR if self.name == "valu" else b.BNN_ARM_MFMA

    def __exit__(self, *exc):
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_MFMA_SHAPE, 0)
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_MFMA32_WM, 0)
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_MFMA32_PIPELINE, 0)
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_MFMA32_XCD_ORDER, 0)
        return False


def _rand_layer(seed, M, K, N):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.uniform(-1, 1, size=(N, K)).astype(np.float32)
    scale = rng.uniform(0.3, 0.7, N).astype(np.float32)
    scale[::7] *= -1.0                                   # negative scales reverse the threshold direction
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32)
    return X, W, scale, bias


# ----------------------------------------------------------------------------- pack

@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("rows,K", [(1, 1), (3, 31), (5, 32), (7, 33), (4, 63), (4, 64), (9, 65), (64, 440),
                                    (33, 2048), (2, 3307), (130, 1000)])
def test_pack_activations_bit_exact(G, oracle, rows, K, wb):
    rng = np.random.default_rng(rows * 1000 + K)
    X = rng.standard_normal((rows, K)).astype(np.float32)
    X.ravel()[:: 5] = 0.0
    X.ravel()[1:: 11] = -0.0
    if X.size > 8:
        X.ravel()[3] = np.nan; X.ravel()[4] = np.inf; X.ravel()[5] = -np.inf
        X.ravel()[6] = np.float32(1e-45); X.ravel()[7] = -np.float32(1e-45)
    got = G.words_to_host(G.pack_activations(G.to_dev(X), wb), wb)
    assert np.array_equal(got, oracle.pack_sign(X, wb))


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("N,K", [(1, 1), (5, 440), (64, 100), (512, 512), (1000, 513), (3400, 2048)])
def test_pack_weights_bits_and_scale(G, oracle, N, K, wb):
    W = workloads.uniform_pm1(3, 7000 + N, N * K).reshape(N, K)
    Wp, sc = G.pack_weights(G.to_dev(W), wb)
    assert np.array_equal(G.words_to_host(Wp, wb), oracle.pack_sign(W, wb))
    # weights on the 2^-24 grid: every partial sum of |w| is exact in fp64, so the mean is order-independent
    assert sc.cpu().numpy()[0] == oracle.mean_abs(W)
    # arbitrary floats: equal up to the last fp32 bit
    W2 = np.random.default_rng(N + K).standard_normal((N, K)).astype(np.float32)
    _, sc2 = G.pack_weights(G.to_dev(W2), wb)
    want = oracle.mean_abs(W2)
    assert abs(float(sc2.cpu().numpy()[0]) - float(want)) <= float(np.spacing(want))


# ----------------------------------------------------------------------------- binary x binary

BIN_SHAPES = [(1, 1, 1), (3, 31, 5), (70, 33, 65), (16, 64, 64), (130, 440, 200), (257, 512, 129), (64, 1000, 1000),
              (300, 2048, 512), (129, 1536, 3307), (65, 4096, 70), (128, 8192, 128), (70, 4608, 96)]


def _bin_operands(oracle, seed, M, K, N, wb):
    rng = np.random.default_rng(seed)
    a = (rng.integers(0, 2, (M, K)) * 2 - 1).astype(np.float32)
    b = (rng.integers(0, 2, (N, K)) * 2 - 1).astype(np.float32)
    return oracle.pack_sign(a, wb), oracle.pack_sign(b, wb)


@pytest.mark.parametrize("arm", ARMS)
@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("M,K,N", BIN_SHAPES)
def test_binx_raw_dot_bit_exact(G, bnn, oracle, M, K, N, wb, arm):
    aw, bw = _bin_operands(oracle, M + K + N, M, K, N, wb)
    with _arm(bnn, arm) as armv:
        got = G.layer_binx(G.to_dev(aw), G.to_dev(bw), None, None, K, N, bnn.BNN_ACT_RAW_I32, wb, armv).cpu().numpy()
    want = oracle.dot_xor(aw, bw, K, wb)
    if M * K * N <= 40_000_000:
        assert np.array_equal(want, oracle.dot_pm1(oracle.unpack_pm1(aw, K, wb), oracle.unpack_pm1(bw, K, wb)))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("arm", ARMS)
@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("act", ["sign", "linear", "hardtanh", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(3, 31, 5), (70, 33, 65), (130, 440, 200), (257, 512, 129), (200, 2048, 1000),
                                   (96, 1024, 3307)])
def test_binx_layer_acts(G, bnn, oracle, M, K, N, act, wb, arm):
    aw, bw = _bin_operands(oracle, 5 * M + K + N, M, K, N, wb)
    _, _, scale, bias = _rand_layer(M + N, 1, 1, N)
    if act in ("hardtanh", "sigmoid"):
        scale = scale / np.float32(np.sqrt(K))            # keep a good share of outputs inside (-1, 1)
    with _arm(bnn, arm) as armv:
        Y = G.layer_binx(G.to_dev(aw), G.to_dev(bw), G.to_dev(scale), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], wb, armv)
    want = oracle.layer_binw_binx(aw, bw, K, scale, bias, act, wb, form="xor")
    if act == "sign":
        assert np.array_equal(G.words_to_host(Y, wb), want)
    elif act in ("logsoftmax", "sigmoid"):
        _close(Y.cpu().numpy(), want, act)                 # fp32 exp on the GPU, fp64 in the oracle
    else:
        assert np.array_equal(Y.cpu().numpy(), want)       # one fma on an exact integer: identical bits
        if act == "hardtanh":
            inside = np.mean(np.abs(want) < 1.0)
            assert 0.05 < inside < 0.999


def test_binx_null_scale_bias(G, bnn, oracle):
    M, K, N, wb = 40, 96, 70, 32
    aw, bw = _bin_operands(oracle, 9, M, K, N, wb)
    for arm in ARMS:
        with _arm(bnn, arm) as armv:
            Y = G.layer_binx(G.to_dev(aw), G.to_dev(bw), None, None, K, N, bnn.BNN_ACT_SIGN, wb, armv)
        assert np.array_equal(G.words_to_host(Y, wb), oracle.layer_binw_binx(aw, bw, K, None, None, "sign", wb))


# ----------------------------------------------------------------------------- activations read as 0/1 (Sec. 3.2)

@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("act", ["raw", "sign", "linear", "hardtanh", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 31, 5), (70, 33, 65), (130, 440, 200), (257, 512, 129),
                                   (200, 2048, 1000), (96, 1024, 3307), (1100, 1024, 384), (4096, 2048, 256)])
def test_binx01_layer(G, bnn, oracle, M, K, N, act, wb):
    aw, bw = _bin_operands(oracle, 7 * M + K + N, M, K, N, wb)
    _, _, scale, bias = _rand_layer(M + N, 1, 1, N)
    if act in ("hardtanh", "sigmoid"):
        scale = scale / np.float32(np.sqrt(K))
    Y = G.layer_binx01(G.to_dev(aw), G.to_dev(bw), G.to_dev(scale), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], wb)
    want = oracle.layer_binw_binx01(aw, bw, K, scale, bias, act, wb, form="and")
    if M * K * N <= 40_000_000:
        assert np.array_equal(oracle.layer_binw_binx01(aw, bw, K, None, None, "raw", wb, form="definition"),
                              oracle.layer_binw_binx01(aw, bw, K, None, None, "raw", wb, form="and"))
    if act == "sign":
        assert np.array_equal(G.words_to_host(Y, wb), want)
    elif act in ("logsoftmax", "sigmoid"):
        _close(Y.cpu().numpy(), want, act)
    else:
        assert np.array_equal(Y.cpu().numpy(), want)     # exact integer, then one fma: identical bits


# ----------------------------------------------------------------------------- batches of a few frames (streaming)

@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("act", ["raw", "sign", "linear", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("x01", [False, True])
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (1, 2048, 2048), (2, 31, 5), (3, 440, 3307), (16, 2048, 300), (17, 33, 65),
                                   (33, 1024, 200), (64, 2048, 512)])
def test_streaming_binary_layer(G, bnn, oracle, M, K, N, act, x01, wb):
    """Default arm, at most 64 frames: the vector-ALU kernel with 1 or 2 frames per workgroup; same bits as ever."""
    aw, bw = _bin_operands(oracle, 11 * M + K + N, M, K, N, wb)
    _, _, scale, bias = _rand_layer(M + N, 1, 1, N)
    if act == "sigmoid":
        scale = scale / np.float32(np.sqrt(K))
    layer = G.layer_binx01 if x01 else G.layer_binx
    with _streaming(bnn):
        Y = layer(G.to_dev(aw), G.to_dev(bw), G.to_dev(scale), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], wb)
        torch.cuda.synchronize()
    if x01:
        want = oracle.layer_binw_binx01(aw, bw, K, scale, bias, act, wb, form="and")
    else:
        want = oracle.layer_binw_binx(aw, bw, K, scale, bias, act, wb, form="xor")
    if act == "sign":
        assert np.array_equal(G.words_to_host(Y, wb), want)
    elif act in ("logsoftmax", "sigmoid"):
        _close(Y.cpu().numpy(), want, act)
    else:
        assert np.array_equal(Y.cpu().numpy(), want)


@pytest.mark.parametrize("cfg_id", [1, 3, 8, 9, 10])
@pytest.mark.parametrize("M", [1, 4, 16, 40, 64])
def test_streaming_forward(G, bnn, oracle, cfg_id, M):
    """bnn_forward on a few frames at a time (every layer on the streaming kernels), all of them compared."""
    with _streaming(bnn):
        _net_parity(G, bnn, oracle, workloads.CONFIGS[cfg_id], M)


def test_streaming_forward_equals_large_batch_forward(G, bnn, oracle):
    """The same 48 frames through the streaming kernels (16 at a time) and through the large-batch kernels: the
    log-posteriors agree within the tolerance of the two log-Softmax kernels, their arg max exactly."""
    cfg = workloads.CONFIGS[3]
    Ws, bs = workloads.make_net_params(cfg)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits)
    X = G.to_dev(workloads.make_frames(cfg, 48))
    big = model.forward(X).cpu().numpy()
    with _streaming(bnn):
        small = np.concatenate([model.forward(X[i:i + 16].contiguous()).cpu().numpy() for i in range(0, 48, 16)])
    _close(small, big, "streaming vs batch")
    assert np.array_equal(small.argmax(1), big.argmax(1))


# ----------------------------------------------------------------------------- real x binary

@pytest.mark.parametrize("tm", [0, 1, 2, 4, 8, 16, 32])
@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("act", ["sign", "linear", "hardtanh", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 31, 5), (70, 33, 65), (64, 440, 512), (130, 440, 200),
                                   (37, 2048, 300), (50, 100, 3307)])
def test_realx_layer(G, bnn, oracle, M, K, N, act, wb, tm):
    """The vector-ALU kernel adds in ascending k, as the oracle's fp32 sum does: fp32 outputs are identical bits."""
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_TM, tm)
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 2)
    try:
        X, W, scale, bias = _rand_layer(M * 3 + K + N, M, K, N)
        if act in ("hardtanh", "sigmoid"):
            scale = scale / np.float32(np.sqrt(K))
        Wp = oracle.pack_sign(W, wb)
        Y = G.layer_realx(G.to_dev(X), G.to_dev(Wp), G.to_dev(scale), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], wb)
        want = oracle.layer_binw_realx(X, Wp, K, scale, bias, act, wb)
        if act == "sign":
            assert np.array_equal(G.words_to_host(Y, wb), want)
        elif act in ("logsoftmax", "sigmoid"):
            _close(Y.cpu().numpy(), want, act)
        else:
            got = Y.cpu().numpy()
            _close(got, want, act)
            assert np.array_equal(got, want), "same order of fp32 additions on both sides: identical bits"
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_TM, 0)
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("act", ["linear", "hardtanh", "logsoftmax", "sign", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(128, 16, 1), (130, 440, 200), (300, 33, 65), (257, 100, 3307), (256, 2048, 384),
                                   (1000, 2048, 2048), (513, 1023, 129)])
def test_realx_layer_matrix_cores(G, bnn, oracle, M, K, N, act, wb):
    """BNN_OPT_REALX_F32_MFMA = 1, 128 frames or more: fp32 outputs come from the fp32 matrix-core kernel, whose order
    of additions is its own: within the tolerance of the oracle's fp32 sum and of its fp64 shadow.  Sign outputs stay
    bit-exact (other kernel)."""
    X, W, scale, bias = _rand_layer(M * 5 + K + N, M, K, N)
    if act in ("hardtanh", "sigmoid"):
        scale = scale / np.float32(np.sqrt(K))
    Wp = oracle.pack_sign(W, wb)
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 1)
    try:
        Y = G.layer_realx(G.to_dev(X), G.to_dev(Wp), G.to_dev(scale), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], wb)
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)
    want = oracle.layer_binw_realx(X, Wp, K, scale, bias, act, wb)
    if act == "sign":
        assert np.array_equal(G.words_to_host(Y, wb), want)
        return
    got = Y.cpu().numpy()
    _close(got, want, act)
    if act in ("linear", "hardtanh"):
        _, acc64 = oracle.realx_acc(X, oracle.unpack_pm1(Wp, K, wb))
        z64 = oracle.affine_f64(acc64, scale, bias)
        _close(got, np.clip(z64, -1.0, 1.0) if act == "hardtanh" else z64, act + " fp64 shadow")
        # much closer than the tolerance: a few units in the last place of the largest partial sum
        assert float(np.max(np.abs(got.astype(np.float64) - z64 if act == "linear" else 0.0))) <= \
            2e-6 * float(np.max(np.abs(z64))) + 1e-30


# ----------------------------------------------------------------------------- real x real (layers that keep their weights)

def _rand_realw(seed, M, K, N):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.uniform(-1, 1, size=(N, K)) * np.sqrt(3.0 / K)).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32)
    return X, W, bias


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("act", ["sign", "linear", "hardtanh", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 31, 5), (70, 33, 65), (64, 440, 512), (130, 440, 200), (17, 16, 257),
                                   (37, 2048, 300), (50, 100, 3307), (33, 12, 70), (300, 452, 260)])
def test_realw_layer(G, bnn, oracle, M, K, N, act, wb):
    """Real-valued weights on the vector ALU: the same ascending-k chain of fused multiply-adds as the oracle's, so fp32
    outputs are identical bits (K a multiple of 4 takes the LDS-staged kernel, any other K the element-load one)."""
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 2)
    try:
        X, W, bias = _rand_realw(M * 7 + K + N, M, K, N)
        Y = G.layer_realw(G.to_dev(X), G.to_dev(W), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], wb)
        want = oracle.layer_realw(X, W, bias, act, wb)
        if act == "sign":
            assert np.array_equal(G.words_to_host(Y, wb), want)
        elif act in ("logsoftmax", "sigmoid"):
            _close(Y.cpu().numpy(), want, act)
        else:
            assert np.array_equal(Y.cpu().numpy(), want), "same order of fp32 operations on both sides: identical bits"
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)


@pytest.mark.parametrize("act", ["sign", "linear", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(1, 440, 2048), (2, 31, 5), (5, 16, 257), (16, 452, 260), (33, 2048, 300), (64, 100, 3307)])
def test_streaming_real_weight_layer(G, bnn, oracle, M, K, N, act):
    """At most 64 frames: the real-weight kernels with 2 frames per workgroup; the same ascending-k chain, identical bits."""
    X, W, bias = _rand_realw(M * 13 + K + N, M, K, N)
    with _streaming(bnn):
        Y = G.layer_realw(G.to_dev(X), G.to_dev(W), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], 32)
        torch.cuda.synchronize()
    want = oracle.layer_realw(X, W, bias, act, 32)
    if act == "sign":
        assert np.array_equal(G.words_to_host(Y, 32), want)
    elif act in ("logsoftmax", "sigmoid"):
        _close(Y.cpu().numpy(), want, act)
    else:
        assert np.array_equal(Y.cpu().numpy(), want)


def _one_layer_realw_forward(G, bnn, X, W, bias, K, N, act, arm, wb=32):
    """A one-layer network with real weights through bnn_forward; `arm` = BNN_OPT_REALW_VALU_LDS."""
    keep = [G.to_dev(W), G.to_dev(bias)]
    d = [dict(K=K, N=N, act=act, word_bits=wb, x_is_binary=False, w_is_real=True, Wp=G.ptr(keep[0]), scale=0, bias=G.ptr(keep[1]))]
    arr = bnn.make_layer_array(d)
    dX = G.to_dev(X)
    M = dX.shape[0]
    nbytes = bnn.bnn_forward_workspace_bytes(arr, 1, M)
    ws = torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=G.DEV)
    out = (G.word_tensor(M, N, wb) if act == bnn.BNN_ACT_SIGN
           else torch.full((M, N), float("nan"), dtype=torch.float32, device=G.DEV))
    bnn.bnn_set_option(bnn.BNN_OPT_REALW_VALU_LDS, arm)
    try:
        assert bnn.bnn_forward(arr, 1, G.ptr(dX), M, G.ptr(out), G.ptr(ws), nbytes, G.stream()) == bnn.BNN_OK
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALW_VALU_LDS, 1)
    return G.words_to_host(out, wb) if act == bnn.BNN_ACT_SIGN else out.cpu().numpy()


@pytest.mark.parametrize("act", ["sign", "linear", "hardtanh", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(512, 4, 1), (513, 12, 70), (600, 440, 300), (1030, 200, 513), (577, 64, 256),
                                   (2048, 452, 1025), (640, 2048, 257)])
def test_real_weight_layer_in_forward_register_fmas(G, bnn, oracle, M, K, N, act):
    """512 frames or more inside bnn_forward: the ascending-k chains of the real-weight layer (paper Sec. 3.1) from the
    kernel whose fmas take three register operands (frames through LDS, weights from a transposed copy): the oracle's
    chain, so identical bits, and identical to the other kernel's."""
    X, W, bias = _rand_realw(M * 5 + K + N, M, K, N)
    a = bnn.ACT_BY_NAME[act]
    got = _one_layer_realw_forward(G, bnn, X, W, bias, K, N, a, 1)
    old = _one_layer_realw_forward(G, bnn, X, W, bias, K, N, a, 0)
    want = oracle.layer_realw(X, W, bias, act, 32)
    assert np.array_equal(got.view(np.uint32), old.view(np.uint32))
    if act == "sigmoid":
        _close(got, want, act)
    else:
        assert np.array_equal(got, want)


def test_real_weight_layer_in_forward_register_fmas_special_values(G, bnn, oracle):
    """NaN, infinities, signed zeros, denormals and huge values in frames and weights: the same bits from both kernels
    (NaN payloads included), and rows without them as the oracle has them."""
    M, K, N = 700, 100, 330
    X, W, bias = _rand_realw(77, M, K, N)
    X[3, 17] = np.inf
    X[4, 50] = np.nan
    X[5] = 0.0
    X[6] = -0.0
    X[7] *= np.float32(1e-41)
    X[8, 99] = np.float32(3e38)
    X[9, 0] = -np.inf
    W[10, 3] = np.nan
    W[11] = -0.0
    W[12] *= np.float32(1e-40)
    W[13, 99] = np.float32(3e38)
    for act in ("linear", "sign", "sigmoid"):
        a = bnn.ACT_BY_NAME[act]
        got = _one_layer_realw_forward(G, bnn, X, W, bias, K, N, a, 1)
        old = _one_layer_realw_forward(G, bnn, X, W, bias, K, N, a, 0)
        assert np.array_equal(got.view(np.uint32), old.view(np.uint32)), act
        with np.errstate(all="ignore"):
            want = oracle.layer_realw(X, W, bias, act, 32)
        if act == "linear":
            assert np.array_equal(np.isnan(got), np.isnan(want))
            fin = ~np.isnan(want)
            assert np.array_equal(got[fin], want[fin])
        elif act == "sign":
            assert np.array_equal(got, want)


def test_realw_layer_with_pm1_weights_equals_binary_weight_layer(G, bnn, oracle):
    """Every weight +1 or -1 and no scale: the real-weight layer and the binary-weight layer give the same bits."""
    M, K, N = 70, 440, 300
    X, W, _, bias = _rand_layer(5, M, K, N)
    Wpm = np.where(W > 0, 1.0, -1.0).astype(np.float32)
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 2)
    try:
        a = G.layer_realw(G.to_dev(X), G.to_dev(Wpm), G.to_dev(bias), K, N, bnn.BNN_ACT_LINEAR, 32).cpu().numpy()
        b = G.layer_realx(G.to_dev(X), G.to_dev(oracle.pack_sign(W, 32)), None, G.to_dev(bias), K, N, bnn.BNN_ACT_LINEAR, 32).cpu().numpy()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("act", ["linear", "hardtanh", "logsoftmax", "sign", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(128, 16, 1), (130, 440, 200), (300, 33, 65), (257, 100, 3307), (256, 2048, 384),
                                   (1000, 2048, 2048), (513, 1023, 129)])
def test_realw_layer_matrix_cores(G, bnn, oracle, M, K, N, act):
    """BNN_OPT_REALX_F32_MFMA = 1, 128 frames or more: fp32 outputs come from the fp32 matrix-core kernel (its own order
    of additions): within the tolerance of the oracle's fp32 chain and of the fp64 value.  Sign bits stay exact."""
    X, W, bias = _rand_realw(M * 11 + K + N, M, K, N)
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 1)
    try:
        Y = G.layer_realw(G.to_dev(X), G.to_dev(W), G.to_dev(bias), K, N, bnn.ACT_BY_NAME[act], 32)
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)
    want = oracle.layer_realw(X, W, bias, act, 32)
    if act == "sign":
        assert np.array_equal(G.words_to_host(Y, 32), want)
        return
    got = Y.cpu().numpy()
    _close(got, want, act)
    if act in ("linear", "hardtanh"):
        _, acc64 = oracle.realw_acc(X, W)
        z64 = oracle.affine_f64(acc64, None, bias)
        _close(got, np.clip(z64, -1.0, 1.0) if act == "hardtanh" else z64, act + " fp64 value")
        if act == "linear":
            assert float(np.max(np.abs(got.astype(np.float64) - z64))) <= 2e-6 * float(np.max(np.abs(z64))) + 1e-30


def test_realw_logsoftmax_default_uses_matrix_cores_within_tolerance(G, bnn, oracle):
    """Default options, the paper's Softmax layer shape: log-posteriors within tolerance of the oracle's."""
    M, K, N = 300, 2048, 3400
    X, W, bias = _rand_realw(99, M, K, N)
    X = (1.0 / (1.0 + np.exp(-X))).astype(np.float32)      # the layer reads Sigmoid outputs (Table 2)
    got = G.layer_realw(G.to_dev(X), G.to_dev(W), G.to_dev(bias), K, N, bnn.BNN_ACT_LOGSOFTMAX, 32).cpu().numpy()
    _close(got, oracle.layer_realw(X, W, bias, "logsoftmax", 32), "logsoftmax")
    assert np.allclose(np.exp(got.astype(np.float64)).sum(1), 1.0, atol=1e-4)


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("M,K", [(1, 1), (5, 31), (7, 64), (33, 65), (64, 2048), (100, 3307)])
def test_unpack_activations(G, bnn, oracle, M, K, wb):
    rng = np.random.default_rng(M + K)
    words = oracle.pack_sign(rng.standard_normal((M, K)).astype(np.float32), wb)
    for zero_one in (False, True):
        got = G.unpack_activations(G.to_dev(words), K, wb, zero_one).cpu().numpy()
        assert np.array_equal(got, oracle.bits_to_real(words, K, wb, zero_one))


@pytest.mark.parametrize("wb", [32, 64])
def test_forward_real_weight_layers_after_binary_layers(G, bnn, oracle, wb):
    """Real-weight layers in every position: reading features, Sign bits, (0, 1) bits and Sigmoid outputs."""
    cfg = workloads.NetConfig(12, "mixed real/binary weights", (40, 96, 70, 130, 65, 50), 37,
                              ("sigmoid", "sign", "step01", "sigmoid"), wb, real_weight_layers=(0, 2, 3, 4))
    _net_parity(G, bnn, oracle, cfg, cfg.M, form="definition")
    cfg = workloads.NetConfig(13, "real weights after sign", (33, 64, 64, 21), 150, ("sign", "step01"), wb,
                              real_weight_layers=(1, 2))
    _net_parity(G, bnn, oracle, cfg, cfg.M, form="definition")


def test_realx_against_fp64_shadow(G, bnn, oracle):
    """The fp32 product also stays within the tolerance of the fp64 value of the same sum."""
    M, K, N, wb = 64, 440, 256, 32
    X, W, scale, bias = _rand_layer(77, M, K, N)
    Wp = oracle.pack_sign(W, wb)
    Y = G.layer_realx(G.to_dev(X), G.to_dev(Wp), G.to_dev(scale), G.to_dev(bias), K, N, bnn.BNN_ACT_LINEAR, wb)
    _, acc64 = oracle.realx_acc(X, oracle.unpack_pm1(Wp, K, wb))
    _close(Y.cpu().numpy(), oracle.affine_f64(acc64, scale, bias), "fp64 shadow")


# ----------------------------------------------------------------------------- first layer on the matrix cores

def _first_layer_bits(G, bnn, X, Wp, scale, bias, K, N, wb, use_mfma):
    """Real input -> Sign bits through bnn_forward with a one-layer network (the path bnn_forward takes for layer 1)."""
    keep = [G.to_dev(Wp), None if scale is None else G.to_dev(scale), None if bias is None else G.to_dev(bias)]
    d = [dict(K=K, N=N, act=bnn.BNN_ACT_SIGN, word_bits=wb, x_is_binary=False, Wp=G.ptr(keep[0]),
              scale=G.ptr(keep[1]), bias=G.ptr(keep[2]))]
    arr = bnn.make_layer_array(d)
    M = X.shape[0]
    nbytes = bnn.bnn_forward_workspace_bytes(arr, 1, M)
    ws = torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=G.DEV)
    out = G.word_tensor(M, N, wb)
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_SIGN_MFMA, int(use_mfma))   # 1: tiled product for 128 frames or more, 2: 16-frame workgroups
    dX = G.to_dev(X)
    try:
        bnn.bnn_forward(arr, 1, G.ptr(dX), M, G.ptr(out), G.ptr(ws), nbytes, G.stream())
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_SIGN_MFMA, 1)
    return G.words_to_host(out, wb)


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (3, 31, 5), (70, 33, 65), (64, 440, 512), (300, 440, 2048), (130, 64, 200),
                                   (37, 1023, 300), (50, 100, 3307), (257, 129, 129),
                                   # more than 512 inputs: the filter with K streamed in slabs
                                   (130, 513, 65), (300, 2048, 700), (64, 4096, 200), (33, 8192, 40), (17, 600, 1025),
                                   (1000, 2048, 2048),
                                   # 128 frames or more: the tiled product (128 x 256 tiles, ragged on both sides)
                                   (128, 8192, 300), (257, 1000, 513), (129, 577, 31), (640, 2048, 257), (1100, 3000, 96)])
def test_first_layer_mfma_filter_bit_exact(G, bnn, oracle, M, K, N, wb):
    X, W, scale, bias = _rand_layer(M * 7 + K + N, M, K, N)
    Wp = oracle.pack_sign(W, wb)
    want = oracle.layer_binw_realx(X, Wp, K, scale, bias, "sign", wb)
    for arm in (1, 2, 0):
        assert np.array_equal(_first_layer_bits(G, bnn, X, Wp, scale, bias, K, N, wb, arm), want), arm


def test_first_layer_mfma_filter_all_outputs_near_tie(G, bnn, oracle):
    """Every pre-activation within rounding of 0: all outputs go through the exact fix-up (queue and its overflow)."""
    M, K, N, wb = 300, 440, 200, 32
    rng = np.random.default_rng(5)
    x0 = rng.standard_normal((1, K)).astype(np.float32)
    X = np.repeat(x0, M, axis=0)
    X[1::2] *= np.float32(1.0 + 2.0 ** -20)                       # a second, slightly different frame
    W = rng.uniform(-1, 1, (N, K)).astype(np.float32)
    Wp = oracle.pack_sign(W, wb)
    scale = np.full(N, 0.5, np.float32)
    acc32, _ = oracle.realx_acc(x0, oracle.unpack_pm1(Wp, K, wb))
    bias = (-0.5 * acc32[0]).astype(np.float32)                     # h^ = 0.5 * acc - 0.5 * acc(frame 0): ties and near-ties
    bias[::3] = np.nextafter(bias[::3], np.float32(np.inf))
    bias[1::3] = np.nextafter(bias[1::3], np.float32(-np.inf))
    want = oracle.layer_binw_realx(X, Wp, K, scale, bias, "sign", wb)
    frac = np.unpackbits(want.view(np.uint8), bitorder="little").mean()
    assert 0.05 < frac < 0.95
    assert np.array_equal(_first_layer_bits(G, bnn, X, Wp, scale, bias, K, N, wb, True), want)


def test_slab_filter_sigmoid_inputs_and_near_ties(G, bnn, oracle):
    """The layer the paper's (sigma, b, ...) topology puts behind its first Sigmoid layer: 2048 inputs in (0, 1), Sign
    outputs.  Half of the biases are set so that the pre-activation of frame 0 is within rounding of 0: those outputs go
    through the exact sums (list, several passes of the term table, overflow), the others through the filter."""
    M, K, N, wb = 200, 2048, 1100, 32
    rng = np.random.default_rng(11)
    X = (1.0 / (1.0 + np.exp(-rng.standard_normal((M, K))))).astype(np.float32)
    X[1::2] = X[0] * np.float32(1.0 + 2.0 ** -21)                 # many frames nearly equal to frame 0
    W = rng.uniform(-1, 1, (N, K)).astype(np.float32)
    Wp = oracle.pack_sign(W, wb)
    scale = np.full(N, 0.25, np.float32)
    scale[::5] = -0.25
    acc32, _ = oracle.realx_acc(X[:1], oracle.unpack_pm1(Wp, K, wb))
    bias = (rng.standard_normal(N) * 3).astype(np.float32)
    bias[::2] = (-scale[::2] * acc32[0, ::2]).astype(np.float32)
    bias[::6] = np.nextafter(bias[::6], np.float32(np.inf))
    want = oracle.layer_binw_realx(X, Wp, K, scale, bias, "sign", wb)
    frac = np.unpackbits(want.view(np.uint8), bitorder="little").mean()
    assert 0.05 < frac < 0.95
    # the tiled product records what it cannot decide per frame and tile of 256 outputs (here about 110, far more than the
    # 31 a record holds, and 1240 for 16 frames where the second kernel takes 1024: the rest is summed by the lane that
    # finds it, in either kernel); the 16-frame kernel keeps its list in LDS
    for arm in (1, 2):
        assert np.array_equal(_first_layer_bits(G, bnn, X, Wp, scale, bias, K, N, wb, arm), want), arm


@pytest.mark.parametrize("M", [70, 200])
@pytest.mark.parametrize("K", [440, 1100])
def test_first_layer_mfma_filter_special_rows(G, bnn, oracle, K, M):
    N, wb = 130, 32
    X, W, scale, bias = _rand_layer(123, M, K, N)
    X[0] = 0.0
    X[1] *= np.float32(1e-41)          # subnormal row
    X[2] *= np.float32(1e-30)
    X[3] *= np.float32(1e30)
    X[4] *= np.float32(3e36)           # too large to quantise: goes to the exact path
    X[5, 17] = np.inf
    X[6, 100] = np.nan
    X[7, 3] = -np.inf
    X[8] = np.float32(1.0)
    X[9, :] = 0.0; X[9, 5] = np.float32(1e-45)
    X[10, ::2] *= np.float32(1e-20)    # wide dynamic range inside a row
    scale[5] = 0.0
    Wp = oracle.pack_sign(W, wb)
    with np.errstate(all="ignore"):
        want = oracle.layer_binw_realx(X, Wp, K, scale, bias, "sign", wb)
    for arm in (1, 2, 0):
        assert np.array_equal(_first_layer_bits(G, bnn, X, Wp, scale, bias, K, N, wb, arm), want), arm


def _one_layer_logsoftmax(G, bnn, X, Wp, scale, bias, K, N, wb, i8):
    """Real input, binary weights, log-posteriors, through bnn_forward with a one-layer network."""
    keep = [G.to_dev(Wp), G.to_dev(scale), G.to_dev(bias)]
    d = [dict(K=K, N=N, act=bnn.BNN_ACT_LOGSOFTMAX, word_bits=wb, x_is_binary=False, Wp=G.ptr(keep[0]),
              scale=G.ptr(keep[1]), bias=G.ptr(keep[2]))]
    arr = bnn.make_layer_array(d)
    M = X.shape[0]
    nbytes = bnn.bnn_forward_workspace_bytes(arr, 1, M)
    ws = torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=G.DEV)
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device=G.DEV)
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_I8_LOGSOFTMAX, int(i8))   # 1: tiled product, 2: 16-frame workgroups
    dX = G.to_dev(X)
    try:
        bnn.bnn_forward(arr, 1, G.ptr(dX), M, G.ptr(out), G.ptr(ws), nbytes, G.stream())
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_I8_LOGSOFTMAX, 1)
    return out.cpu().numpy()


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("kind", ["normal", "sigmoid", "wide"])
@pytest.mark.parametrize("M,K,N", [(128, 1, 1), (130, 440, 200), (300, 2048, 3400), (257, 1023, 129), (128, 8192, 65),
                                   (1000, 2048, 2048), (513, 600, 3307)])
def test_output_layer_real_inputs_int8_digit_planes(G, bnn, oracle, M, K, N, kind, wb):
    """The output layer of a network with real hidden activations (binary weights, real inputs, log-Softmax) on the
    int8 matrix cores from four digit planes: log-posteriors against the oracle's, ten times closer than the tolerance
    asks, and as close to the fp32 matrix-core kernel's."""
    rng = np.random.default_rng(M * 13 + K * 5 + N + wb)
    X = rng.standard_normal((M, K)).astype(np.float32)
    if kind == "sigmoid":
        X = (1.0 / (1.0 + np.exp(-X))).astype(np.float32)
    if kind == "wide":                                      # 12 orders of magnitude inside a frame, and tiny frames
        X *= np.exp(rng.uniform(-14, 14, (M, K))).astype(np.float32)
        X[::7] *= np.float32(1e-30)
    W = rng.uniform(-1, 1, (N, K)).astype(np.float32)
    Wp = oracle.pack_sign(W, wb)
    scale = np.full(N, 1.0 / np.sqrt(K), np.float32) * rng.uniform(0.5, 1.5, N).astype(np.float32)
    scale[::11] *= -1
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32)
    want = oracle.layer_binw_realx(X, Wp, K, scale, bias, "logsoftmax", wb)
    ref = _one_layer_logsoftmax(G, bnn, X, Wp, scale, bias, K, N, wb, 0)
    s = float(np.max(np.abs(want)))
    both = []
    for arm in (1, 2):
        got = _one_layer_logsoftmax(G, bnn, X, Wp, scale, bias, K, N, wb, arm)
        assert np.isfinite(got).all()
        assert float(np.max(np.abs(got.astype(np.float64) - want))) <= 1e-5 * s
        assert float(np.max(np.abs(got.astype(np.float64) - ref))) <= 1e-5 * s
        assert np.allclose(np.exp(got.astype(np.float64)).sum(1), 1.0, atol=1e-4)
        both.append(got)
    assert np.array_equal(both[0], both[1])                 # the same exact integer sums, the same roundings after them


def test_output_layer_int8_digit_planes_special_frames(G, bnn, oracle):
    """Frames the quantisation cannot take (NaN, Inf, values beyond 2^90) go through the fp32 sum in ascending k: their
    rows come out as the oracle's (NaN rows stay NaN), the other rows are untouched by them."""
    M, K, N, wb = 140, 700, 300, 32
    X, W, scale, bias = _rand_layer(321, M, K, N)
    scale = scale / np.float32(np.sqrt(K))
    X[3, 17] = np.inf
    X[4, 100] = np.nan
    X[5] *= np.float32(1e30)
    X[6] = 0.0
    X[7] *= np.float32(1e-41)
    Wp = oracle.pack_sign(W, wb)
    with np.errstate(all="ignore"):
        want = oracle.layer_binw_realx(X, Wp, K, scale, bias, "logsoftmax", wb)
    for arm in (1, 2):
        got = _one_layer_logsoftmax(G, bnn, X, Wp, scale, bias, K, N, wb, arm)
        fin = np.isfinite(want).all(axis=1)
        assert not fin[3] and not fin[4]
        assert np.array_equal(np.isnan(got), np.isnan(want))
        _close(got[fin], want[fin], "finite rows")


def _one_layer_realw_logsoftmax(G, bnn, X, W, bias, K, N, split, x_bits=None, wb=32):
    """Real weights, log-posteriors, through bnn_forward with a one-layer network; `x_bits` = packed input instead of X."""
    keep = [G.to_dev(W), G.to_dev(bias)]
    d = [dict(K=K, N=N, act=bnn.BNN_ACT_LOGSOFTMAX, word_bits=wb, x_is_binary=x_bits is not None, w_is_real=True,
              Wp=G.ptr(keep[0]), scale=0, bias=G.ptr(keep[1]))]
    arr = bnn.make_layer_array(d)
    dX = G.to_dev(X if x_bits is None else x_bits)
    M = dX.shape[0]
    nbytes = bnn.bnn_forward_workspace_bytes(arr, 1, M)
    ws = torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=G.DEV)
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device=G.DEV)
    bnn.bnn_set_option(bnn.BNN_OPT_REALW_SPLIT_LOGSOFTMAX, int(split))
    try:
        bnn.bnn_forward(arr, 1, G.ptr(dX), M, G.ptr(out), G.ptr(ws), nbytes, G.stream())
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALW_SPLIT_LOGSOFTMAX, 1)
    return out.cpu().numpy()


@pytest.mark.parametrize("kind", ["normal", "sigmoid", "wide"])
@pytest.mark.parametrize("M,K,N", [(128, 1, 1), (130, 440, 200), (300, 2048, 3400), (257, 1023, 129), (128, 8191, 65),
                                   (1000, 2048, 2048), (513, 600, 3307), (256, 32, 128), (640, 96, 384)])
def test_softmax_layer_real_weights_bf16_pieces(G, bnn, oracle, M, K, N, kind):
    """The Softmax layer with real weights and real inputs (paper Sec. 3.1, 4.3) on the bf16 matrix cores from three
    pieces per operand: log-posteriors against the oracle's, ten times closer than the tolerance asks, and as close to
    the fp32 matrix-core kernel's."""
    rng = np.random.default_rng(M * 17 + K * 3 + N)
    X = rng.standard_normal((M, K)).astype(np.float32)
    if kind == "sigmoid":
        X = (1.0 / (1.0 + np.exp(-X))).astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    if kind == "wide":                                      # 12 orders of magnitude inside a row, on both sides
        X *= np.exp(rng.uniform(-14, 14, (M, K))).astype(np.float32)
        W *= np.exp(rng.uniform(-14, 14, (N, K))).astype(np.float32)
        X[::7] *= np.float32(1e-30)
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32)
    want = oracle.layer_realw(X, W, bias, "logsoftmax", 32)
    ref = _one_layer_realw_logsoftmax(G, bnn, X, W, bias, K, N, 0)
    s = float(np.max(np.abs(want)))
    for waves in (1, 2):                                    # workgroups of four waves (default) and of eight
        got = _one_layer_realw_logsoftmax(G, bnn, X, W, bias, K, N, waves)
        assert np.isfinite(got).all()
        assert float(np.max(np.abs(got.astype(np.float64) - want))) <= 1e-5 * s
        assert float(np.max(np.abs(got.astype(np.float64) - ref))) <= 1e-5 * s
        assert np.allclose(np.exp(got.astype(np.float64)).sum(1), 1.0, atol=1e-4)


def test_softmax_layer_bf16_pieces_sum_within_its_bound(G, bnn, oracle):
    """The bound the kernel states for its sums, seen through the log-posteriors: out[m][a] - out[m][0] = z_a - z_0, and
    each z is within 2^-22 sum_k |x_k w_k| (the piece products left out) plus the rounding of about 800 fp32 additions
    (allowed here: 2^-18 of the row's largest |z|, twice what a random walk of that length gives) of the exact sum."""
    M, K, N = 256, 2048, 256
    rng = np.random.default_rng(5)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.standard_normal((N, K)).astype(np.float32)
    bias = np.zeros(N, np.float32)
    got = _one_layer_realw_logsoftmax(G, bnn, X, W, bias, K, N, True).astype(np.float64)
    _, z = oracle.realw_acc(X, W)
    mass = np.abs(X.astype(np.float64)) @ np.abs(W.astype(np.float64)).T
    bound = 2.0 ** -22 * mass + 2.0 ** -18 * np.abs(z).max(1, keepdims=True)
    assert np.all(np.abs((got - got[:, :1]) - (z - z[:, :1])) <= bound + bound[:, :1])


def test_softmax_layer_bf16_pieces_binary_inputs_and_special_values(G, bnn, oracle):
    """Packed binary inputs are unpacked in front of the split (their pieces are +-1, 0, 0: the products are exact);
    rows holding NaN or Inf come out NaN like the oracle's, values next to the largest finite float stay finite in the
    split, tiny rows keep their relative accuracy, and no row disturbs another."""
    M, K, N = 200, 777, 150
    rng = np.random.default_rng(8)
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32)
    xb = oracle.pack_sign(X, 32)
    want = oracle.layer_realw(oracle.unpack_pm1(xb, K, 32).astype(np.float32), W, bias, "logsoftmax", 32)
    got = _one_layer_realw_logsoftmax(G, bnn, None, W, bias, K, N, True, x_bits=xb)
    _close(got, want, "binary inputs")
    X[3, 17] = np.inf
    X[4, 100] = np.nan
    X[5] = 0.0
    X[6] *= np.float32(1e-41)
    X[7] *= np.float32(1e-30)
    X[8, :] = 0.0
    X[8, 5] = np.float32(3.4028234e38)       # rounds up to infinity as a bf16: must be cut instead
    W[9, 5] = np.float32(1e-38)
    with np.errstate(all="ignore"):
        want = oracle.layer_realw(X, W, bias, "logsoftmax", 32)
    got = _one_layer_realw_logsoftmax(G, bnn, X, W, bias, K, N, True)
    fin = np.isfinite(want).all(axis=1)
    assert not fin[3] and not fin[4]
    assert np.array_equal(np.isnan(got), np.isnan(want))
    _close(got[fin], want[fin], "finite rows")


# ----------------------------------------------------------------------------- whole network

def _net_parity(G, bnn, oracle, cfg, M, frames=None, form="xor", arm=None):
    """GPU forward on M frames of cfg; oracle on `frames` (indices) or on all of them."""
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg, M)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits, real_weight_layers=cfg.real_weight_layers)
    layers = oracle.make_layers(Ws, bs, cfg.hidden_act, cfg.word_bits, real_weight_layers=cfg.real_weight_layers)
    for ly, sc in zip(layers, model.scales):
        assert (sc is None and ly.scale is None) or sc.cpu().numpy()[0] == ly.scale[0]
    if arm is not None:
        bnn.bnn_set_option(bnn.BNN_OPT_BINX_ARM, arm)
    try:
        got = model.forward(G.to_dev(X))
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_BINX_ARM, bnn.BNN_ARM_MFMA)
    idx = np.arange(M) if frames is None else np.asarray(frames)
    want, keep = oracle.forward(layers, X[idx], form=form, keep=True)
    got_h = got[torch.from_numpy(idx).to(G.DEV)].cpu().numpy()
    _close(got_h, want, cfg.name)
    # The most likely state is the oracle's: its arg-max attains the GPU row's maximum (subtracting the row's constant
    # is monotone, so rounding can create a tie but not reverse an order), except where the oracle's two largest
    # log-posteriors are closer than the two sides may differ (each within TOL * scale of the other).
    best = want.argmax(1)
    attains = got_h[np.arange(len(best)), best] == got_h.max(1)
    top2 = np.partition(want, -2, axis=1)[:, -2:]
    near_tie = (top2[:, 1] - top2[:, 0]) <= 2 * TOL * float(np.max(np.abs(want)))
    assert np.all(attains | near_tie), f"{int((~(attains | near_tie)).sum())} frames with another most likely state"
    assert np.allclose(np.exp(got_h.astype(np.float64)).sum(1), 1.0, atol=1e-4)
    return model, layers, X, keep


@pytest.mark.parametrize("arm", ARMS)
def test_forward_config1_full(G, bnn, oracle, arm):
    cfg = workloads.CONFIGS[1]
    with _arm(bnn, arm) as armv:
        _net_parity(G, bnn, oracle, cfg, cfg.M, form="definition", arm=armv)


def test_forward_config1_layer_by_layer_bits(G, bnn, oracle):
    """Every hidden layer's packed output equals the oracle's, fed with the oracle's own previous bits."""
    cfg = workloads.CONFIGS[1]
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg)
    layers = oracle.make_layers(Ws, bs, "sign", 32)
    _, keep = oracle.forward(layers, X, form="definition", keep=True)
    h = G.to_dev(X)
    for l, ly in enumerate(layers[:-1]):
        args = (G.to_dev(ly.w_words), G.to_dev(ly.scale), G.to_dev(ly.bias), ly.K, ly.N, bnn.BNN_ACT_SIGN, 32)
        Y = G.layer_realx(h, *args) if l == 0 else G.layer_binx(h, *args)
        assert np.array_equal(G.words_to_host(Y, 32), keep[l]), f"layer {l + 1}"
        h = Y


@pytest.mark.parametrize("cfg_id,M", [(2, 96), (3, 300), (4, 200), (6, 1100), (7, 1030), (8, 300), (8, 1280), (9, 96), (9, 1100),
                                      (10, 96), (10, 1100)])
def test_forward_configs_reduced_batch_full_compare(G, bnn, oracle, cfg_id, M):
    cfg = workloads.CONFIGS[cfg_id]
    _net_parity(G, bnn, oracle, cfg, M)


def _hidden_bits_layer_by_layer(G, bnn, model, layers, X, keep, rows=None):
    """Every hidden layer's packed output at the full batch, through the per-layer entry points in the launch
    configuration of the batch, against the oracle's bits (all rows, or the rows the oracle computed)."""
    wb = model.word_bits
    h = G.to_dev(X)
    sel = None if rows is None else torch.from_numpy(np.asarray(rows)).to(G.DEV)
    for l, (ly, d) in enumerate(zip(layers[:-1], model.descs[:-1])):
        assert d["act"] == bnn.BNN_ACT_SIGN
        Y = G.word_tensor(X.shape[0], ly.N, wb)
        if l == 0:   # as bnn_forward runs its first layer: a one-layer network
            one = bnn.make_layer_array(model.descs[:1])
            bnn.bnn_forward(one, 1, G.ptr(h), X.shape[0], G.ptr(Y), 0, 0, G.stream())
        else:
            fn = bnn.bnn_layer_binw_binx01 if d["x_is_binary"] == 2 else bnn.bnn_layer_binw_binx
            fn(G.ptr(h), d["Wp"], d["scale"], d["bias"], X.shape[0], ly.K, ly.N, bnn.BNN_ACT_SIGN, wb, G.ptr(Y), G.stream())
        torch.cuda.synchronize()
        got = G.words_to_host(Y if sel is None else Y[sel], wb)
        assert np.array_equal(got, keep[l]), f"hidden layer {l + 1}: {int((got != keep[l]).sum())} words differ"
        h = Y


def test_forward_config3_full_batch_every_frame(G, bnn, oracle):
    """Config 3 at its full size (M = 4096, the launch configuration the benchmark times): every log-posterior of every
    frame against the oracle, and all six hidden bit tensors bit for bit."""
    cfg = workloads.CONFIGS[3]
    model, layers, X, keep = _net_parity(G, bnn, oracle, cfg, cfg.M)
    _hidden_bits_layer_by_layer(G, bnn, model, layers, X, keep)


@pytest.mark.parametrize("wb", [32, 64])
@pytest.mark.parametrize("M,K,N", [(4096, 2048, 2048), (300, 1024, 200), (777, 3072, 333), (130, 2048, 129), (1, 1024, 1),
                                   (520, 4096, 2050)])
def test_binx_sign_split_k(G, bnn, oracle, M, K, N, wb):
    """Sign layers with K split between the two halves of an 8-wave workgroup (BNN_OPT_MFMA32_SPLITK, a comparison arm):
    same bits, ragged shapes included."""
    aw, bw = _bin_operands(oracle, 7 * M + K + N, M, K, N, wb)
    _, _, scale, bias = _rand_layer(M + N + 3, 1, 1, N)
    bnn.bnn_set_option(bnn.BNN_OPT_MFMA_SHAPE, 32)
    bnn.bnn_set_option(bnn.BNN_OPT_MFMA32_WM, 4)
    bnn.bnn_set_option(bnn.BNN_OPT_MFMA32_SPLITK, 1)
    try:
        Y = G.layer_binx(G.to_dev(aw), G.to_dev(bw), G.to_dev(scale), G.to_dev(bias), K, N, bnn.BNN_ACT_SIGN, wb)
        torch.cuda.synchronize()
        bnn.bnn_set_option(bnn.BNN_OPT_MFMA32_SPLITK, 0)
        Y_off = G.layer_binx(G.to_dev(aw), G.to_dev(bw), G.to_dev(scale), G.to_dev(bias), K, N, bnn.BNN_ACT_SIGN, wb)
        torch.cuda.synchronize()
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_MFMA_SHAPE, 0)
        bnn.bnn_set_option(bnn.BNN_OPT_MFMA32_WM, 0)
        bnn.bnn_set_option(bnn.BNN_OPT_MFMA32_SPLITK, 0)
    want = oracle.layer_binw_binx(aw, bw, K, scale, bias, "sign", wb, form="xor")
    assert np.array_equal(G.words_to_host(Y, wb), want)
    assert np.array_equal(G.words_to_host(Y_off, wb), want)


class _cooperative:
    """BNN_OPT_COOPERATIVE for the duration of a test (the test process runs one stream at a time, as the option asks)."""

    def __init__(self, bnn):
        self.bnn = bnn

    def __enter__(self):
        self.before = self.bnn.bnn_cooperative_timeouts()
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_COOPERATIVE, 1)

    def __exit__(self, *exc):
        self.bnn.bnn_set_option(self.bnn.BNN_OPT_COOPERATIVE, 0)
        assert self.bnn.bnn_cooperative_timeouts() == self.before, "a bounded wait of a cooperative kernel ran out"


@pytest.mark.parametrize("x01", [False, True])
@pytest.mark.parametrize("M,K,N", [(4096, 2048, 3400), (4096, 512, 2048), (3333, 1024, 3307), (2100, 512, 4001),
                                   (2048, 2048, 8192), (257, 512, 129)])
def test_cooperative_logsoftmax_layer(G, bnn, oracle, M, K, N, x01):
    """The LOGSOFTMAX layer finished inside the product kernel (rows exchanged between workgroups through memory):
    every log-posterior against the oracle, ragged frames and outputs included; the last shapes are ones the
    cooperative kernel does not take (too many tiles to be resident at once, too few to use 128-row tiles), which
    must fall back to the two-kernel path unharmed."""
    aw, bw = _bin_operands(oracle, 3 * M + K + N, M, K, N, 32)
    _, _, scale, bias = _rand_layer(M + N + 1, 1, 1, N)
    scale = scale / np.float32(np.sqrt(K))                 # log-posteriors of a plausible spread
    dA, dB, dsc, dbi = (G.to_dev(a) for a in (aw, bw, scale, bias))
    fn = G.layer_binx01 if x01 else G.layer_binx
    with _cooperative(bnn):
        Y = fn(dA, dB, dsc, dbi, K, N, bnn.BNN_ACT_LOGSOFTMAX, 32)
        torch.cuda.synchronize()
        Y2 = fn(dA, dB, dsc, dbi, K, N, bnn.BNN_ACT_LOGSOFTMAX, 32)   # the hand-over area is reused: same result again
        torch.cuda.synchronize()
    got = Y.cpu().numpy()
    want = (oracle.layer_binw_binx01(aw, bw, K, scale, bias, "logsoftmax", 32, form="and") if x01 else
            oracle.layer_binw_binx(aw, bw, K, scale, bias, "logsoftmax", 32, form="xor"))
    _close(got, want, "cooperative logsoftmax")
    assert np.allclose(np.exp(got.astype(np.float64)).sum(1), 1.0, atol=1e-4)
    assert np.array_equal(got, Y2.cpu().numpy())
    plain = fn(dA, dB, dsc, dbi, K, N, bnn.BNN_ACT_LOGSOFTMAX, 32).cpu().numpy()
    _close(got, plain, "cooperative against the two-kernel path")


def test_cooperative_wait_runs_out_and_the_kernel_still_ends(G, bnn, oracle):
    """The bounded wait, forced to run out from the host (one poll instead of a million): the kernel ends on its own,
    the workgroups that gave up are counted, and the next call with the normal limit is right again."""
    M, K, N = 4096, 2048, 3400
    aw, bw = _bin_operands(oracle, 99, M, K, N, 32)
    _, _, scale, bias = _rand_layer(98, 1, 1, N)
    scale = scale / np.float32(np.sqrt(K))
    dA, dB, dsc, dbi = (G.to_dev(a) for a in (aw, bw, scale, bias))
    before = bnn.bnn_cooperative_timeouts()
    bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE, 1)
    bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE_SPIN, 1)
    try:
        G.layer_binx(dA, dB, dsc, dbi, K, N, bnn.BNN_ACT_LOGSOFTMAX, 32)
        torch.cuda.synchronize()                               # returns: every workgroup left its wait
        gave_up = bnn.bnn_cooperative_timeouts() - before
        assert gave_up > 0
        bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE_SPIN, 1 << 20)
        Y = G.layer_binx(dA, dB, dsc, dbi, K, N, bnn.BNN_ACT_LOGSOFTMAX, 32)
        torch.cuda.synchronize()
        assert bnn.bnn_cooperative_timeouts() - before == gave_up
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE_SPIN, 1 << 20)
        bnn.bnn_set_option(bnn.BNN_OPT_COOPERATIVE, 0)
    _close(Y.cpu().numpy(), oracle.layer_binw_binx(aw, bw, K, scale, bias, "logsoftmax", 32, form="xor"), "after a wait that ran out")


def test_forward_config3_full_batch_cooperative(G, bnn, oracle):
    """Config 3 at its full size with the cooperative output layer, the configuration the benchmark times: every
    log-posterior of every frame against the oracle."""
    cfg = workloads.CONFIGS[3]
    with _cooperative(bnn):
        _net_parity(G, bnn, oracle, cfg, cfg.M)


def _tile_class_frames(M, count, seed, tile=128):
    """`count` or more frames of a batch of M: the first and last tile whole, one frame of every `tile`-row tile with the
    position inside the tile running through all residues, and random ones."""
    tiles = M // tile
    per_tile = np.arange(tiles) * tile + (np.arange(tiles) * 37) % tile
    base = np.concatenate([np.arange(0, tile), np.arange(M - tile, M), per_tile])
    extra = np.random.default_rng(seed).integers(0, M, max(0, count - base.size))
    return np.unique(np.concatenate([base, extra]))


def test_forward_config2_full_batch_sampled_frames(G, bnn, oracle):
    cfg = workloads.CONFIGS[2]
    _net_parity(G, bnn, oracle, cfg, cfg.M, frames=_tile_class_frames(cfg.M, 320, 1))


def test_forward_config2_matrix_cores_layer_by_layer(G, bnn, oracle):
    """Config 2 at full batch with the fp32 matrix-core kernel in every layer.  Seven hard-tanh layers amplify fp32
    rounding differences (a different order of additions) beyond the end-to-end tolerance, so each layer is checked on
    its own: the oracle's layer, fed with the GPU's own previous activations, against the GPU's layer."""
    cfg = workloads.CONFIGS[2]
    Ws, bs = workloads.make_net_params(cfg)
    X = workloads.make_frames(cfg)
    layers = oracle.make_layers(Ws, bs, cfg.hidden_act, cfg.word_bits)
    idx = np.unique(np.concatenate([np.arange(0, 8), np.arange(cfg.M - 8, cfg.M),
                                    np.random.default_rng(3).integers(0, cfg.M, 48)]))
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 1)
    try:
        h = G.to_dev(X)
        for l, ly in enumerate(layers):
            Y = G.layer_realx(h, G.to_dev(ly.w_words), G.to_dev(ly.scale), G.to_dev(ly.bias), ly.K, ly.N,
                              bnn.ACT_BY_NAME[ly.act], cfg.word_bits)
            torch.cuda.synchronize()
            h_in = h[torch.from_numpy(idx).to(G.DEV)].cpu().numpy()
            want = oracle.layer_binw_realx(h_in, ly.w_words, ly.K, ly.scale, ly.bias, ly.act, cfg.word_bits)
            _close(Y[torch.from_numpy(idx).to(G.DEV)].cpu().numpy(), want, f"layer {l + 1}")
            h = Y
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)


def test_forward_config8_full_batch_sampled_frames(G, bnn, oracle):
    """(0, 1) hidden activations at the benchmark's size."""
    cfg = workloads.CONFIGS[8]
    frames = np.unique(np.concatenate([np.arange(0, 8), np.arange(cfg.M - 8, cfg.M),
                                       np.random.default_rng(4).integers(0, cfg.M, 48)]))
    _net_parity(G, bnn, oracle, cfg, cfg.M, frames=frames)


@pytest.mark.parametrize("cfg_id", [9, 10])
def test_forward_sigmoid_topologies_full_batch_sampled_frames(G, bnn, oracle, cfg_id):
    """(sigma, b, b, b, b, sigma, delta) at the benchmark's size, with binary (9) and real-valued (10) outer weights."""
    cfg = workloads.CONFIGS[cfg_id]
    frames = np.unique(np.concatenate([np.arange(0, 8), np.arange(cfg.M - 8, cfg.M),
                                       np.random.default_rng(6).integers(0, cfg.M, 32)]))
    _net_parity(G, bnn, oracle, cfg, cfg.M, frames=frames)


def test_forward_config4_full_batch_sampled_frames(G, bnn, oracle):
    """Config 4 at its full size (16384 frames, 64-bit words): 1200 or more frames, among them the first and the last
    128-row tile whole and a frame of every tile, for the log-posteriors and for every hidden layer's bits."""
    cfg = workloads.CONFIGS[4]
    frames = _tile_class_frames(cfg.M, 1200, 2)
    model, layers, X, keep = _net_parity(G, bnn, oracle, cfg, cfg.M, frames=frames)
    _hidden_bits_layer_by_layer(G, bnn, model, layers, X, keep, rows=frames)


# ----------------------------------------------------------------------------- isolated GEMM sweep (Config 5)

@pytest.mark.parametrize("arm", ARMS)
@pytest.mark.parametrize("shape", workloads.GEMM_SWEEP, ids=lambda s: f"M{s.M}_K{s.K}_N{s.N}")
def test_gemm_sweep_int32(G, bnn, oracle, shape, arm):
    M, K, N = shape.M, shape.K, shape.N
    A = workloads.random_words(0, 500 + workloads.TENSOR_ABITS, M, K // 32)
    B = workloads.random_words(0, 500 + workloads.TENSOR_BBITS, N, K // 32)
    with _arm(bnn, arm) as armv:
        Y = G.layer_binx(G.to_dev(A), G.to_dev(B), None, None, K, N, bnn.BNN_ACT_RAW_I32, 32, armv)
    torch.cuda.synchronize()
    if M <= 4096:
        rows = np.arange(M)
    else:   # the oracle computes sampled rows one by one: first and last tiles, a row of every 128-row tile, random rows
        tiles = np.arange(M // 128)
        rows = np.unique(np.concatenate([np.arange(0, 160), np.arange(M - 160, M), tiles * 128 + (tiles * 37) % 128,
                                         np.random.default_rng(M + K + N).integers(0, M, 300)]))
    got = Y[torch.from_numpy(rows).to(G.DEV)].cpu().numpy()
    want = oracle.dot_xor(A[rows], B, K, 32)
    assert np.array_equal(got, want)
    # properties that hold at any size, on the whole output, evaluated on the GPU tensor
    assert int(Y.abs().max()) <= K
    assert int((Y & 1).max()) == (K & 1) and int((Y & 1).min()) == (K & 1)
    del Y
    torch.cuda.empty_cache()


# ----------------------------------------------------------------------------- edges

def test_forward_in_a_captured_graph_replays_identically(G, bnn, oracle):
    """bnn_forward only enqueues kernels on the caller's stream: it can be captured and replayed; every replay, with
    eager work and synchronisations in between, gives the eager result bit for bit."""
    cfg = workloads.CONFIGS[1]
    Ws, bs = workloads.make_net_params(cfg)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits)
    X = G.to_dev(workloads.make_frames(cfg, 200))
    out = torch.empty((200, model.N_out), dtype=torch.float32, device=G.DEV)
    model.forward(X, out)
    torch.cuda.synchronize()
    ref = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        model.forward(X, out)                      # warm-up on a side stream, as graph capture wants
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.forward(X, out)
    for _ in range(4):
        out.fill_(float("nan"))                    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
        assert torch.equal(model.forward(X), ref)  # and eager again


def test_zero_frames_is_a_noop(G, bnn):
    assert bnn.bnn_layer_binw_binx(0, 0, 0, 0, 0, 64, 64, bnn.BNN_ACT_SIGN, 32, 0, G.stream()) == 0
    assert bnn.bnn_layer_binw_realx(0, 0, 0, 0, 0, 64, 64, bnn.BNN_ACT_SIGN, 32, 0, G.stream()) == 0
    assert bnn.bnn_pack_activations(0, 0, 64, 32, 0, G.stream()) == 0


def test_forward_twice_same_result_and_other_stream(G, bnn, oracle):
    cfg = workloads.CONFIGS[1]
    Ws, bs = workloads.make_net_params(cfg)
    X = G.to_dev(workloads.make_frames(cfg))
    model = G.GpuModel(Ws, bs, "sign", 32)
    a = model.forward(X).clone()
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        b = model.forward(X)
    s.synchronize()
    assert torch.equal(a, b)


def test_forward_several_batches_in_flight_on_four_streams(G, bnn, oracle):
    """Config 3 at its full size with four batches in flight on four streams (the way the benchmark issues its steps):
    each stream has its own frames, output and workspace, the packed model is shared; every output equals the one the
    same frames give alone on one stream, bit for bit, over three rounds."""
    cfg = workloads.CONFIGS[3]
    Ws, bs = workloads.make_net_params(cfg)
    model = G.GpuModel(Ws, bs, cfg.hidden_act, cfg.word_bits)
    M, S = cfg.M, 4
    rng = np.random.default_rng(77)
    Xh = [workloads.make_frames(cfg)] + [rng.standard_normal((M, cfg.dims[0])).astype(np.float32) for _ in range(S - 1)]
    Xs = [G.to_dev(x) for x in Xh]
    alone = [model.forward(x).clone() for x in Xs]
    torch.cuda.synchronize()
    nbytes = bnn.bnn_forward_workspace_bytes(model.layers, model.n_layers, M)
    streams = [torch.cuda.Stream() for _ in range(S)]
    outs = [torch.full((M, model.N_out), float("nan"), dtype=torch.float32, device=G.DEV) for _ in range(S)]
    wss = [torch.empty(max(nbytes, 256), dtype=torch.uint8, device=G.DEV) for _ in range(S)]
    torch.cuda.synchronize()
    for _ in range(3):
        for j in range(S):
            bnn.bnn_forward(model.layers, model.n_layers, Xs[j].data_ptr(), M, outs[j].data_ptr(), wss[j].data_ptr(), nbytes,
                            streams[j].cuda_stream)
    torch.cuda.synchronize()
    for j in range(S):
        assert torch.equal(outs[j], alone[j]), f"stream {j}"


# ----------------------------------------------------------------------------- seeded random shapes, every layer kind

def _random_shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        M = int(rng.choice([1, 2, 3, 15, 16, 17, 63, 64, 65, 127, 129, 200, 300]))
        K = int(rng.choice([4, 8, 12, 60, 64, 68, 100, 252, 256, 260, 440, 1000, 1024, 1028, 37, 129]))
        N = int(rng.choice([1, 31, 32, 33, 63, 64, 65, 255, 256, 257, 1000, 1025]))
        out.append((M, K, N))
    return out


@pytest.fixture()
def bnn_defaults(bnn):
    """The library as a caller finds it: every option at its default, the small-batch dispatch (64 frames) included."""
    bnn.bnn_set_option(bnn.BNN_OPT_STREAM_MAX_FRAMES, 64)
    yield bnn
    bnn.bnn_set_option(bnn.BNN_OPT_STREAM_MAX_FRAMES, 0)


@pytest.mark.parametrize("act", ["sign", "linear", "logsoftmax", "sigmoid"])
@pytest.mark.parametrize("M,K,N", [(1, 440, 2048), (40, 2048, 300), (64, 440, 512), (65, 33, 65), (130, 440, 200),
                                   (300, 2048, 2048), (257, 512, 3307)])
def test_layers_with_every_option_at_its_default(G, bnn_defaults, oracle, M, K, N, act):
    """One pass over the four layer kinds through whatever kernels the default dispatch picks, on both sides of the
    small-batch boundary.  Sign bits and the binary layers' fp32 outputs are exact; fp32 outputs of the real-input
    layers may come from the matrix-core kernel (its own order of additions) and are held to the tolerance."""
    bnn = bnn_defaults
    X, W, scale, bias = _rand_layer(M * 17 + K * 3 + N, M, K, N)
    Wr = (W * np.float32(np.sqrt(3.0 / K))).astype(np.float32)
    Wp, aw = oracle.pack_sign(W, 32), oracle.pack_sign(X, 32)
    dX, dWp, dWr, dsc, dbi, daw = (G.to_dev(a) for a in (X, Wp, Wr, scale, bias, aw))
    a = bnn.ACT_BY_NAME[act]
    got = [G.layer_realx(dX, dWp, dsc, dbi, K, N, a, 32), G.layer_realw(dX, dWr, dbi, K, N, a, 32),
           G.layer_binx(daw, dWp, dsc, dbi, K, N, a, 32), G.layer_binx01(daw, dWp, dsc, dbi, K, N, a, 32)]
    torch.cuda.synchronize()
    want = [oracle.layer_binw_realx(X, Wp, K, scale, bias, act, 32), oracle.layer_realw(X, Wr, bias, act, 32),
            oracle.layer_binw_binx(aw, Wp, K, scale, bias, act, 32, form="xor"),
            oracle.layer_binw_binx01(aw, Wp, K, scale, bias, act, 32, form="and")]
    for i, (g_, w_) in enumerate(zip(got, want)):
        kind = ("realx", "realw", "binx", "binx01")[i]
        if act == "sign":
            assert np.array_equal(G.words_to_host(g_, 32), w_), kind
        elif act == "linear" and i >= 2:
            assert np.array_equal(g_.cpu().numpy(), w_), kind      # one fma on an exact integer
        else:
            _close(g_.cpu().numpy(), w_, f"{kind} {act}")


@pytest.mark.parametrize("stream_frames", [0, 64])
@pytest.mark.parametrize("M,K,N", _random_shapes(2024, 40))
def test_random_shapes_all_layer_kinds(G, bnn, oracle, M, K, N, stream_frames):
    """Binary-weight and real-weight layers on real input, binary layers in both readings, Sign and fp32 outputs, with
    the small-batch dispatch off and on; every kernel here keeps the oracle's order, so fp32 outputs are identical bits."""
    X, W, scale, bias = _rand_layer(M * 31 + K * 7 + N, M, K, N)
    Wr = (W * np.float32(np.sqrt(3.0 / K))).astype(np.float32)
    Wp = oracle.pack_sign(W, 32)
    aw = oracle.pack_sign(X, 32)
    dX, dWp, dWr, dsc, dbi, daw = (G.to_dev(a) for a in (X, Wp, Wr, scale, bias, aw))
    bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 2)
    try:
        with _streaming(bnn, stream_frames):
            for act in ("sign", "linear"):
                a = bnn.ACT_BY_NAME[act]
                got = [G.layer_realx(dX, dWp, dsc, dbi, K, N, a, 32), G.layer_realw(dX, dWr, dbi, K, N, a, 32),
                       G.layer_binx(daw, dWp, dsc, dbi, K, N, a, 32), G.layer_binx01(daw, dWp, dsc, dbi, K, N, a, 32)]
                torch.cuda.synchronize()
                want = [oracle.layer_binw_realx(X, Wp, K, scale, bias, act, 32), oracle.layer_realw(X, Wr, bias, act, 32),
                        oracle.layer_binw_binx(aw, Wp, K, scale, bias, act, 32, form="xor"),
                        oracle.layer_binw_binx01(aw, Wp, K, scale, bias, act, 32, form="and")]
                for i, (g_, w_) in enumerate(zip(got, want)):
                    g_ = G.words_to_host(g_, 32) if act == "sign" else g_.cpu().numpy()
                    assert np.array_equal(g_, w_), (act, i)
    finally:
        bnn.bnn_set_option(bnn.BNN_OPT_REALX_F32_MFMA, 0)


@pytest.mark.parametrize("M,N", [(1, 1), (3, 5), (70, 3307), (300, 3400), (4096, 3972)])
def test_subtract_log_prior(G, bnn, oracle, M, N):
    """Log-posteriors minus log-priors (scaled log-likelihoods for hybrid decoding): one fp32 subtraction per element,
    identical bits; NaN and infinities pass through as the arithmetic has them."""
    rng = np.random.default_rng(M + N)
    z = (rng.standard_normal((M, N)) * 4).astype(np.float32)
    logp, _ = oracle.log_softmax(z)
    counts = rng.integers(1, 1000, N).astype(np.float64)
    log_prior = np.log(counts / counts.sum()).astype(np.float32)
    if M > 2:
        logp[1, 0] = -np.inf
        logp[2, N - 1] = np.nan
    d = G.to_dev(logp.copy())
    bnn.bnn_subtract_log_prior(G.ptr(d), G.ptr(G.to_dev(log_prior)), M, N, G.stream())
    torch.cuda.synchronize()
    with np.errstate(all="ignore"):
        want = oracle.subtract_log_prior(logp, log_prior)
    assert np.array_equal(d.cpu().numpy().view(np.uint32), want.view(np.uint32))
