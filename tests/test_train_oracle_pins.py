"""Pins for the training-side oracle (Alg. 1 and Alg. 2 backward and update, Sec. 2.1-2.3): every check compares it
with something other than itself - finite differences of an independent fp64 forward pass, numpy products, closed
forms, hand-worked cases."""
import numpy as np
import pytest
import scipy.special


@pytest.fixture(scope="module")
def T():
    from oracle import train_oracle
    return train_oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _loss64(Ws, rs, X, labels):
    """Independent fp64 forward pass: Sigmoid hidden layers, Softmax output, summed cross entropy."""
    h = X.astype(np.float64)
    for l, (W, r) in enumerate(zip(Ws, rs)):
        z = h @ W.astype(np.float64).T + r.astype(np.float64)
        h = scipy.special.expit(z) if l < len(Ws) - 1 else z
    logp = h - scipy.special.logsumexp(h, axis=1, keepdims=True)
    return -logp[np.arange(len(labels)), labels].sum()


def test_backward_of_a_real_network_matches_finite_differences(oracle, T):
    """Alg. 2's backward loop with real weights and Sigmoid hidden units against central differences of the loss."""
    rng = _rng(1)
    dims, M = (6, 5, 4, 3), 7
    Ws = [(rng.standard_normal((n, k)) * 0.7).astype(np.float32) for k, n in zip(dims[:-1], dims[1:])]
    rs = [(rng.standard_normal(n) * 0.3).astype(np.float32) for n in dims[1:]]
    X = rng.standard_normal((M, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], M)
    # forward with the oracle, keeping every layer's output
    layers = oracle.make_layers(Ws, rs, "sigmoid", 32, real_weight_layers=(0, 1, 2))
    logp, outs = oracle.forward(layers, X, keep=True)
    hs = [X] + outs[:-1]
    g_hhat = T.softmax_xent_grad(logp, labels)
    gW, gr = [None] * 3, [None] * 3
    for l in (2, 1, 0):
        gW[l] = T.backward_weight(g_hhat, hs[l])
        gr[l] = T.bias_grad(g_hhat)
        if l > 0:
            g_h = T.backward_input_realw(g_hhat, Ws[l])
            g_hhat = T.sigmoid_grad(g_h, hs[l])                    # through the Sigmoid of layer l
    eps = 1e-4
    for l in range(3):
        for (n, k) in [(0, 0), (1, 2), (dims[l + 1] - 1, dims[l] - 1)]:
            Wp = [w.astype(np.float64).copy() for w in Ws]
            Wm = [w.astype(np.float64).copy() for w in Ws]
            Wp[l][n, k] += eps
            Wm[l][n, k] -= eps
            fd = (_loss64(Wp, rs, X, labels) - _loss64(Wm, rs, X, labels)) / (2 * eps)
            assert abs(gW[l][n, k] - fd) <= 2e-4 * max(1.0, abs(fd)), (l, n, k)
        rp = [r.astype(np.float64).copy() for r in rs]
        rm = [r.astype(np.float64).copy() for r in rs]
        rp[l][1] += eps
        rm[l][1] -= eps
        fd = (_loss64(Ws, rp, X, labels) - _loss64(Ws, rm, X, labels)) / (2 * eps)
        assert abs(gr[l][1] - fd) <= 2e-4 * max(1.0, abs(fd))


def test_softmax_xent_grad_closed_forms(T):
    z = _rng(2).standard_normal((5, 9))
    logp = (z - scipy.special.logsumexp(z, axis=1, keepdims=True)).astype(np.float32)
    labels = np.array([0, 8, 3, 3, 5])
    g = T.softmax_xent_grad(logp, labels)
    assert np.allclose(g.sum(1), 0.0, atol=1e-6)                                   # softmax sums to 1, one-hot to 1
    want = scipy.special.softmax(z, axis=1)
    want[np.arange(5), labels] -= 1.0
    assert np.max(np.abs(g - want)) <= 1e-6
    assert np.all(g[np.arange(5), labels] < 0) and np.all(np.delete(g[0], 0) > 0)


def test_backward_products_vs_numpy_and_each_other(oracle, T):
    rng = _rng(3)
    M, N, K = 9, 13, 21
    g = rng.standard_normal((M, N)).astype(np.float32)
    Wb = (rng.integers(0, 2, (N, K)) * 2 - 1).astype(np.int8)
    h = rng.standard_normal((M, K)).astype(np.float32)
    gi = T.backward_input_binw(g, Wb)
    assert gi.shape == (M, K)
    assert np.max(np.abs(gi - g.astype(np.float64) @ Wb.astype(np.float64))) <= 1e-5
    # binary weights as real numbers: the same chain of exact adds and subtracts, bit for bit
    assert np.array_equal(gi, T.backward_input_realw(g, Wb.astype(np.float32)))
    gw = T.backward_weight(g, h)
    assert gw.shape == (N, K)
    assert np.max(np.abs(gw - g.astype(np.float64).T @ h.astype(np.float64))) <= 1e-5
    # one frame: the weight gradient is the outer product, exactly (a single product, rounded once)
    g1, h1 = g[:1], h[:1]
    assert np.array_equal(T.backward_weight(g1, h1), (g1.T.astype(np.float64) * h1.astype(np.float64)).astype(np.float32))
    # order of the sums: ascending n, ascending m (2^24 absorbs the ones that follow it, not those before it)
    big = np.array([[2.0 ** 24] + [1.0] * 8], dtype=np.float32)
    ones = np.ones((9, 1), np.int8)
    assert T.backward_input_binw(big, ones)[0, 0] == np.float32(2.0 ** 24)
    assert T.backward_input_binw(big[:, ::-1].copy(), ones)[0, 0] == np.float32(2.0 ** 24 + 8)
    assert T.bias_grad(big.T.copy())[0] == np.float32(2.0 ** 24)
    assert T.bias_grad(big.T[::-1].copy())[0] == np.float32(2.0 ** 24 + 8)
    assert T.backward_weight(big.T.copy(), np.ones((9, 1), np.float32))[0, 0] == np.float32(2.0 ** 24)


def test_mask_grad_hand_cases(T):
    g = np.array([1.5, -2.0, 3.0, 4.0, -5.0, 6.0], np.float32)
    hh = np.array([0.0, 1.0, -1.0, 1.0000001, -3.0, np.nan], np.float32)
    # |h^| = k passes (Mask is 0 only where |h^| > k); NaN is not > k
    assert np.array_equal(T.mask_grad(g, hh, 1.0), np.array([1.5, -2.0, 3.0, 0.0, 0.0, 6.0], np.float32))
    assert np.array_equal(T.mask_grad(g, hh, 3.0)[:5], g[:5])
    rng = _rng(4)
    a, b = rng.standard_normal(1000).astype(np.float32), (rng.standard_normal(1000) * 2).astype(np.float32)
    for k in (0.5, 1.0, 2.0, 3.0):
        assert np.array_equal(T.mask_grad(a, b, k), a * (np.abs(b) <= np.float32(k)))


def test_sigmoid_grad(T):
    h = np.array([0.5, 0.25, 1.0, 0.0, 0.75], np.float32)
    g = np.array([4.0, -16.0, 3.0, 3.0, 1.0], np.float32)
    assert np.array_equal(T.sigmoid_grad(g, h), np.array([1.0, -3.0, 0.0, 0.0, 0.1875], np.float32))
    # against the derivative of scipy's expit by central differences
    z = np.linspace(-6, 6, 49)
    fd = (scipy.special.expit(z + 1e-6) - scipy.special.expit(z - 1e-6)) / 2e-6
    got = T.sigmoid_grad(np.ones_like(z, dtype=np.float32), scipy.special.expit(z).astype(np.float32))
    assert np.max(np.abs(got - fd)) <= 1e-6


def test_update_clip(T):
    w = np.array([0.5, 0.99, -0.99, 0.0, 1.0, -1.0], np.float32)
    g = np.array([1.0, -1.0, 1.0, 0.0, -4.0, 4.0], np.float32)
    got = T.update_clip(w, g, 0.25, True)
    assert np.array_equal(got, np.array([0.25, 1.0, -1.0, 0.0, 1.0, -1.0], np.float32))
    assert np.array_equal(T.update_clip(w, g, 0.25, False), np.array([0.25, 1.24, -1.24, 0.0, 2.0, -2.0], np.float32))
    # w - eta g is one fused multiply-add: (1 + 2^-12)^2 - (1 + 2^-11) = 2^-24; a rounded product would give 0
    a = np.float32(1 + 2.0 ** -12)
    assert T.update_clip(np.array([-(1 + 2.0 ** -11)], np.float32), np.array([a], np.float32), float(-a), False)[0] == np.float32(2.0 ** -24)
    assert T.update_clip(w, g, 0.0, True).tobytes() == w.tobytes()


def test_grad_norm_clip(T):
    g = np.ones((30, 30), np.float32)                   # ||g|| = 30
    out, norm = T.grad_norm_clip(g, 15.0)
    assert norm == np.float32(30.0) and np.array_equal(out, np.full((30, 30), 0.5, np.float32))
    out, norm = T.grad_norm_clip(g, 30.0)                # not above the threshold: untouched
    assert np.array_equal(out, g)
    rng = _rng(5)
    g = rng.standard_normal((64, 50)).astype(np.float32)
    out, norm = T.grad_norm_clip(g, 15.0)
    assert abs(float(norm) - np.linalg.norm(g.astype(np.float64))) <= 1e-5
    assert abs(np.linalg.norm(out.astype(np.float64)) - 15.0) <= 1e-4
    assert np.max(np.abs(out / g - 15.0 / np.linalg.norm(g.astype(np.float64)))) <= 1e-6   # same direction


def test_semi_stochastic_binarize(T):
    w = np.array([0.9, 0.9, -0.9, -0.2, 0.0, 1.0, -1.0, 0.5], np.float32)
    u = np.array([0.5, 0.95, 0.1, 0.5, 0.0, 0.999, 0.0, 0.5], np.float32)
    # set to the sign where u < |w|; w = 0 and |w| <= u stay
    assert np.array_equal(T.semi_stochastic_binarize(w, u), np.array([1.0, 0.9, -1.0, -0.2, 0.0, 1.0, -1.0, 0.5], np.float32))
    rng = _rng(6)
    w = rng.uniform(-1, 1, 200000).astype(np.float32)
    out = T.semi_stochastic_binarize(w, rng.uniform(0, 1, w.size).astype(np.float32))
    locked = np.abs(out) == 1.0
    assert abs(locked.mean() - 0.5) < 0.01                     # E p(|w|) = E |w| = 1/2 for w ~ U(-1, 1)
    assert np.array_equal(np.sign(out), np.sign(w)) and np.array_equal(out[~locked], w[~locked])
    # a weight near +-1 is locked far more often than one near 0
    assert locked[np.abs(w) > 0.9].mean() > 0.9 and locked[np.abs(w) < 0.1].mean() < 0.1


def test_alg1_training_reduces_the_loss_of_a_binary_weight_network(oracle, T):
    """Alg. 1 end to end with the oracle's own steps: binary weights in every layer, Sigmoid hidden units, clipped
    updates of the real-valued weights.  Twenty minibatch steps on a fixed synthetic task lower the cross entropy:
    a wrong sign or a transposed operand anywhere in the backward pass or the update would raise it instead."""
    rng = _rng(11)
    dims, M, eta = (12, 16, 16, 4), 64, 0.01
    X = rng.standard_normal((M, dims[0])).astype(np.float32)
    teacher = rng.standard_normal((dims[0], dims[-1]))
    labels = np.argmax(X @ teacher, axis=1)
    Ws = [rng.uniform(-1, 1, (n, k)).astype(np.float32) for k, n in zip(dims[:-1], dims[1:])]
    rs = [np.zeros(n, np.float32) for n in dims[1:]]

    def forward(Ws, rs):
        hs, h = [X], X
        for l, (W, r) in enumerate(zip(Ws, rs)):
            Wb = np.where(W > 0, 1, -1).astype(np.int8)                       # w^b = Sign(w)
            hhat = oracle.affine_f32(oracle.realx_acc(h, Wb, want64=False)[0], np.full(len(r), 0.25, np.float32), r)
            h = oracle.sigmoid(hhat) if l < len(Ws) - 1 else oracle.log_softmax(hhat)[0]
            hs.append(h)
        return hs

    losses = []
    for step in range(20):
        hs = forward(Ws, rs)
        losses.append(-float(hs[-1][np.arange(M), labels].sum()))
        g = T.softmax_xent_grad(hs[-1], labels)
        for l in (2, 1, 0):
            g = g * np.float32(0.25)                                          # the constant scale of this toy network
            gW, gr = T.backward_weight(g, hs[l]), T.bias_grad(g)
            if l > 0:
                g = T.sigmoid_grad(T.backward_input_binw(g, np.where(Ws[l] > 0, 1, -1).astype(np.int8)), hs[l])
            Ws[l] = T.update_clip(Ws[l], T.grad_norm_clip(gW, 15.0)[0], eta, True)
            rs[l] = T.update_clip(rs[l], gr, eta, False)
        assert all(np.abs(W).max() <= 1.0 for W in Ws)
    assert losses[-1] < 0.95 * losses[0] and min(losses) < 0.95 * losses[0], losses
    assert sum(b < a for a, b in zip(losses[:-1], losses[1:])) >= 12, losses   # most steps lower it (weights flip in jumps)
