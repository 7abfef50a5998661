"""Pins for the CPU oracle: every function is checked against something other than itself.

* brute-force dense masked products written here as plain Python loops (tiny shapes),
* a library GEMM for the density-1 special case,
* the adjoint identity between the forward and the transposed product,
* fp64 central finite differences of the mean cross-entropy,
* closed forms (uniform softmax, geometric momentum series),
* the bit-identical sparsity pattern invariant.
"""
import hashlib
import math

import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl


def _dense(layer, values=None):
    W = np.zeros((layer.rows, layer.cols), dtype=np.float64)
    M = np.zeros((layer.rows, layer.cols), dtype=bool)
    vals = layer.values if values is None else values
    for i in range(layer.rows):
        for p in range(layer.indptr[i], layer.indptr[i + 1]):
            W[i, layer.indices[p]] = vals[p]
            M[i, layer.indices[p]] = True
    return W, M


def _tiny_layer(rows, cols, density, seed, relu=False):
    nnz = wl.round_half_up(density * rows * cols)
    indptr, indices = wl.uniform_pattern(rows, cols, nnz, seed)
    rng = np.random.default_rng(seed + 77)
    values = rng.standard_normal(nnz).astype(np.float32)
    bias = rng.standard_normal(rows).astype(np.float32)
    return wl.SparseLayerData(rows, cols, indptr, indices, values, bias, relu)


TINY = [(7, 5, 0.0), (7, 5, 0.3), (7, 5, 1.0), (4, 9, 0.5), (1, 1, 1.0), (3, 6, 0.15)]


@pytest.mark.parametrize("rows,cols,density", TINY)
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_forward_matches_dense_masked_loops(oracle, rows, cols, density, dtype):
    B = 3
    lay = _tiny_layer(rows, cols, density, seed=11)
    W, M = _dense(lay)
    X = np.random.default_rng(5).standard_normal((cols, B)).astype(dtype)
    for relu in (False, True):
        Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, X, relu, dtype)
        for i in range(rows):
            for c in range(B):
                z = float(lay.bias[i]); s = abs(float(lay.bias[i]))
                for j in range(cols):
                    if M[i, j]:
                        z += W[i, j] * float(X[j, c]); s += abs(W[i, j] * float(X[j, c]))
                if relu:
                    z = max(z, 0.0)
                assert Y[i, c] == pytest.approx(z, rel=2e-6 if dtype == np.float32 else 1e-14, abs=1e-30)
                assert S[i, c] == pytest.approx(s, rel=1e-14)
    # without bias
    Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, None, X, False, dtype)
    assert np.allclose(Y, W @ X.astype(np.float64), rtol=1e-5 if dtype == np.float32 else 1e-13, atol=1e-6 if dtype == np.float32 else 1e-14)


@pytest.mark.parametrize("rows,cols,density", TINY)
def test_transposed_matches_dense_masked_loops(oracle, rows, cols, density):
    B = 4
    lay = _tiny_layer(rows, cols, density, seed=13)
    W, M = _dense(lay)
    dZ = np.random.default_rng(6).standard_normal((rows, B))
    dX, S = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, lay.values, dZ, np.float64)
    for j in range(cols):
        for c in range(B):
            z = 0.0; s = 0.0
            for i in range(rows):
                if M[i, j]:
                    z += W[i, j] * dZ[i, c]; s += abs(W[i, j] * dZ[i, c])
            assert dX[j, c] == pytest.approx(z, rel=1e-13, abs=1e-300)
            assert S[j, c] == pytest.approx(s, rel=1e-13, abs=1e-300)


@pytest.mark.parametrize("rows,cols,density", TINY)
def test_sddmm_matches_dense_masked_loops(oracle, rows, cols, density):
    B = 5
    lay = _tiny_layer(rows, cols, density, seed=17)
    _, M = _dense(lay)
    rng = np.random.default_rng(8)
    dZ = rng.standard_normal((rows, B)); X = rng.standard_normal((cols, B))
    g, Sg, db, Sdb = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dZ, X, np.float64)
    # dense product dZ X^T restricted to the mask, loops written out
    G = np.zeros((rows, cols)); SG = np.zeros((rows, cols))
    for i in range(rows):
        for j in range(cols):
            if M[i, j]:
                for c in range(B):
                    G[i, j] += dZ[i, c] * X[j, c]; SG[i, j] += abs(dZ[i, c] * X[j, c])
    p = 0
    for i in range(rows):
        for j in range(cols):
            if M[i, j]:
                assert g[p] == pytest.approx(G[i, j], rel=1e-13); assert Sg[p] == pytest.approx(SG[i, j], rel=1e-13)
                p += 1
        assert db[i] == pytest.approx(sum(dZ[i, c] for c in range(B)), rel=1e-13)
        assert Sdb[i] == pytest.approx(sum(abs(dZ[i, c]) for c in range(B)), rel=1e-13)
    assert p == lay.nnz


def test_density_one_equals_library_gemm(oracle):
    rows, cols, B = 96, 130, 37
    lay = _tiny_layer(rows, cols, 1.0, seed=19)
    W = lay.values.reshape(rows, cols).astype(np.float64)       # every entry stored, row-major
    rng = np.random.default_rng(3)
    X = rng.standard_normal((cols, B)); dZ = rng.standard_normal((rows, B))
    v64 = lay.values.astype(np.float64)
    Y, _ = oracle.spmm(rows, cols, lay.indptr, lay.indices, v64, lay.bias.astype(np.float64), X, False, np.float64)
    assert np.allclose(Y, W @ X + lay.bias[:, None].astype(np.float64), rtol=1e-12, atol=1e-12)
    dX, _ = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, v64, dZ, np.float64)
    assert np.allclose(dX, W.T @ dZ, rtol=1e-12, atol=1e-12)
    g, _, db, _ = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dZ, X, np.float64)
    assert np.allclose(g.reshape(rows, cols), dZ @ X.T, rtol=1e-12, atol=1e-12)
    assert np.allclose(db, dZ.sum(axis=1), rtol=1e-12, atol=1e-12)


def test_adjoint_identity_full_size(oracle):
    """<W X, U> = <X, W^T U> on the first layer of the paper's MLP at 99 % sparsity."""
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=0.99)
    lay = mlp.layers[0]
    rng = np.random.default_rng(21)
    X = rng.standard_normal((lay.cols, 100)); U = rng.standard_normal((lay.rows, 100))
    v = lay.values.astype(np.float64)
    Y, _ = oracle.spmm(lay.rows, lay.cols, lay.indptr, lay.indices, v, None, X, False, np.float64)
    Xt, _ = oracle.spmm_t(lay.rows, lay.cols, lay.indptr, lay.indices, v, U, np.float64)
    lhs, rhs = float((Y * U).sum()), float((X * Xt).sum())
    assert lhs == pytest.approx(rhs, rel=1e-11)


def test_sddmm_identity_full_size(oracle):
    """sum_p g[p] t[p] = <dZ, T X> for random t on the same pattern."""
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=0.99)
    lay = mlp.layers[1]
    rng = np.random.default_rng(23)
    X = rng.standard_normal((lay.cols, 100)); dZ = rng.standard_normal((lay.rows, 100))
    t = rng.standard_normal(lay.nnz)
    g, _, _, _ = oracle.sddmm(lay.rows, lay.cols, lay.indptr, lay.indices, dZ, X, np.float64)
    TX, _ = oracle.spmm(lay.rows, lay.cols, lay.indptr, lay.indices, t, None, X, False, np.float64)
    assert float(g @ t) == pytest.approx(float((dZ * TX).sum()), rel=1e-11)


def test_relu_backward_is_strict(oracle):
    A = np.array([[0.0, 1.0, -1.0, 1e-30]]); dA = np.array([[5.0, 6.0, 7.0, 8.0]])
    assert oracle.relu_backward(dA, A, np.float64).tolist() == [[0.0, 6.0, 0.0, 8.0]]
    # forward ReLU clamps at zero
    Y, _ = oracle.spmm(1, 1, [0, 1], [0], [-2.0], [0.0], np.array([[1.0, -1.0]]), True, np.float64)
    assert Y.tolist() == [[0.0, 2.0]]


def test_softmax_ce_uniform_closed_form(oracle):
    """All logits equal -> loss = ln(classes), dZ = (1/classes - onehot)/B."""
    C, B = 10, 100
    labels = np.random.default_rng(1).integers(0, C, size=B)
    for shift in (0.0, 3.5, -1000.0, 1000.0):
        Z = np.full((C, B), shift)
        loss, _, dZ, SdZ = oracle.softmax_ce(Z, labels, np.float64)
        assert loss == pytest.approx(math.log(10.0), rel=1e-12)
        hot = np.zeros((C, B)); hot[labels, np.arange(B)] = 1.0
        assert np.allclose(dZ, (0.1 - hot) / B, rtol=1e-12, atol=1e-15)
        assert np.allclose(SdZ, (0.1 + hot) / B, rtol=1e-12)


def test_softmax_ce_two_class_closed_form_and_gradient(oracle):
    # two classes: loss = log(1 + exp(-(z_t - z_other)))
    Z = np.array([[2.0, -1.0, 0.3], [0.5, 4.0, 0.3]]); labels = np.array([0, 0, 1])
    loss, _, dZ, _ = oracle.softmax_ce(Z, labels, np.float64)
    expect = np.mean([math.log1p(math.exp(-1.5)), math.log1p(math.exp(5.0)), math.log(2.0)])
    assert loss == pytest.approx(expect, rel=1e-13)
    assert np.allclose(dZ.sum(axis=0), 0.0, atol=1e-16)          # columns of the gradient sum to zero
    h = 1e-6
    for i in range(2):
        for c in range(3):
            Zp, Zm = Z.copy(), Z.copy(); Zp[i, c] += h; Zm[i, c] -= h
            fd = (oracle.softmax_ce(Zp, labels, np.float64)[0] - oracle.softmax_ce(Zm, labels, np.float64)[0]) / (2 * h)
            assert dZ[i, c] == pytest.approx(fd, rel=1e-7, abs=1e-10)


def test_softmax_ce_shift_invariance_large_logits(oracle):
    rng = np.random.default_rng(4)
    Z = rng.standard_normal((10, 7)) * 5; labels = rng.integers(0, 10, size=7)
    l0, _, d0, _ = oracle.softmax_ce(Z, labels, np.float64)
    l1, _, d1, _ = oracle.softmax_ce(Z + 700.0, labels, np.float64)
    assert l1 == pytest.approx(l0, rel=1e-10) and np.allclose(d0, d1, rtol=1e-9, atol=1e-15)


def test_momentum_closed_forms(oracle):
    rng = np.random.default_rng(9)
    n = 50
    w0, v0, g = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    # lr = 0: v_t = mu^t v_0, w_t = w_0 + v_0 mu (1 - mu^t)/(1 - mu)
    mu, T = 0.9, 12
    w, v = w0.copy(), v0.copy()
    for _ in range(T):
        w, v, _, _ = oracle.momentum(w, v, g, 0.0, mu, dtype=np.float64)
    assert np.allclose(v, mu ** T * v0, rtol=1e-12)
    assert np.allclose(w, w0 + v0 * mu * (1 - mu ** T) / (1 - mu), rtol=1e-12, atol=1e-13)
    # mu = 0: plain gradient descent
    w, v, _, _ = oracle.momentum(w0, v0, g, 0.05, 0.0, dtype=np.float64)
    assert np.allclose(w, w0 - 0.05 * g, rtol=1e-14) and np.allclose(v, -0.05 * g, rtol=1e-14)
    # constant gradient from rest: v_t = -lr g (1 - mu^t)/(1 - mu)
    w, v = w0.copy(), np.zeros(n)
    lr = 0.01
    for _ in range(T):
        w, v, Sw, Sv = oracle.momentum(w, v, g, lr, mu, dtype=np.float64)
    assert np.allclose(v, -lr * g * (1 - mu ** T) / (1 - mu), rtol=1e-12)
    t = np.arange(1, T + 1)
    assert np.allclose(w, w0 - lr * g * ((1 - mu ** t) / (1 - mu)).sum(), rtol=1e-12, atol=1e-13)
    assert np.all(Sv >= np.abs(v) * (1 - 1e-12)) and np.all(Sw >= np.abs(w) * (1 - 1e-12))
    # inputs untouched
    assert np.array_equal(w0, np.random.default_rng(9).standard_normal(n))


def test_momentum_f32_rounds_velocity_before_adding(oracle):
    w = np.array([1.0], dtype=np.float32); v = np.array([0.0], dtype=np.float32)
    g = np.array([1.0 / 3.0], dtype=np.float32)
    w1, v1, _, _ = oracle.momentum(w, v, g, 0.01, 0.9, dtype=np.float32)
    lr32 = np.float32(0.01)
    v_expect = np.float32(-(float(lr32) * float(g[0])))
    assert v1[0] == v_expect and w1[0] == np.float32(float(w[0]) + float(v_expect))


def _tiny_mlp(bias_std=0.3):
    return wl.make_mlp((7, 5, 4, 3), layer_nnz=(14, 9, 8), pattern_seed=40, value_seed=50, bias_std=bias_std)


def test_finite_difference_gradients_tiny_mlp(oracle):
    """fp64 central differences of the mean CE loss w.r.t. every stored weight and bias."""
    mlp = _tiny_mlp()
    rng = np.random.default_rng(31)
    B = 3
    X = rng.standard_normal((7, B)); labels = rng.integers(0, 3, size=B)
    state = oracle.new_state(mlp.layers, np.float64)
    out = oracle.mlp_step(state, X, labels, 0.0, 0.0, np.float64, update=False)
    assert out["loss"] == pytest.approx(oracle.mlp_loss(state, X, labels), rel=1e-14)
    h = 1e-6
    checked = 0
    for l, st in enumerate(state):
        for name, grad in (("values", out["g"][l]), ("bias", out["db"][l])):
            arr = st[name]
            for k in range(arr.shape[0]):
                keep = arr[k]
                arr[k] = keep + h; lp = oracle.mlp_loss(state, X, labels)
                arr[k] = keep - h; lm = oracle.mlp_loss(state, X, labels)
                arr[k] = keep
                fd = (lp - lm) / (2 * h)
                assert grad[k] == pytest.approx(fd, rel=2e-6, abs=2e-9), (l, name, k)
                checked += 1
    assert checked == 14 + 9 + 8 + 5 + 4 + 3
    # input gradient of layer 2 and 3 (dA of the previous hidden layer) by differences on A
    # is covered through the chain: a wrong transposed product would break layer-1/2 gradients.


def test_relu_mask_override_changes_backward_only(oracle):
    mlp = _tiny_mlp()
    rng = np.random.default_rng(33)
    X = rng.standard_normal((7, 4)); labels = rng.integers(0, 3, size=4)
    s0 = oracle.new_state(mlp.layers, np.float64)
    base = oracle.mlp_step(s0, X, labels, 0.1, 0.9, np.float64, update=False)
    masks = [base["A"][0] > 0, base["A"][1] > 0, None]
    same = oracle.mlp_step(s0, X, labels, 0.1, 0.9, np.float64, update=False, relu_masks=masks)
    assert all(np.array_equal(a, b) for a, b in zip(base["g"], same["g"]))
    masks[0] = np.ones_like(masks[0])
    other = oracle.mlp_step(s0, X, labels, 0.1, 0.9, np.float64, update=False, relu_masks=masks)
    assert other["loss"] == base["loss"] and not np.array_equal(other["g"][0], base["g"][0])


def _digest(*arrays):
    h = hashlib.sha256()
    for a in arrays:
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()


def test_training_reduces_loss_and_pattern_is_bit_identical(oracle):
    mlp = wl.make_mlp((48, 32, 16, 10), sparsity=0.7, pattern_seed=60, value_seed=70)
    Xs, Ts = wl.make_batches(48, 10, 20, 1, seed=80)
    state = oracle.new_state(mlp.layers, np.float32)
    before = [_digest(l.indptr, l.indices) for l in mlp.layers]
    losses = []
    for _ in range(30):
        losses.append(oracle.mlp_step(state, Xs[0], Ts[0], 0.05, 0.9, np.float32)["loss"])
        assert [_digest(st["indptr"], st["indices"]) for st in state] == before
    assert losses[-1] < 0.5 * losses[0]            # same batch repeated: the loss must fall
    assert all(st["values"].shape == (l.nnz,) for st, l in zip(state, mlp.layers))


def test_first_step_loss_near_ln10_with_zero_weights(oracle):
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=0.99)
    Xs, Ts = wl.make_batches(3072, 10, 100, 1, seed=3000)
    state = oracle.new_state(mlp.layers, np.float32)
    for st in state:
        st["values"][:] = 0
    out = oracle.mlp_step(state, Xs[0], Ts[0], 0.01, 0.9, np.float32)
    assert out["loss"] == pytest.approx(math.log(10.0), rel=1e-6)
    # with all-zero weights only the last layer's biases receive a gradient
    assert all(not g.any() for g in out["g"])
    assert out["db"][2].any() and not out["db"][0].any()


def test_f32_storage_close_to_f64(oracle):
    mlp = wl.make_mlp((64, 48, 32, 10), sparsity=0.8, pattern_seed=61, value_seed=71, bias_std=0.1)
    Xs, Ts = wl.make_batches(64, 10, 16, 1, seed=81)
    s32 = oracle.new_state(mlp.layers, np.float32); s64 = oracle.new_state(mlp.layers, np.float64)
    o32 = oracle.mlp_step(s32, Xs[0], Ts[0], 0.01, 0.9, np.float32)
    o64 = oracle.mlp_step(s64, Xs[0], Ts[0], 0.01, 0.9, np.float64)
    assert o32["loss"] == pytest.approx(o64["loss"], rel=1e-6)
    for l in range(3):
        assert np.all(np.abs(o32["g"][l] - o64["g"][l]) <= 2e-6 * o64["Sg"][l] + 1e-12)
        assert np.all(np.abs(s32[l]["values"] - s64[l]["values"]) <= 1e-6 * o64["Sw"][l])


def test_oracle_threads_do_not_change_results(oracle):
    mlp = wl.make_mlp((64, 48, 32, 10), sparsity=0.8, pattern_seed=62, value_seed=72)
    Xs, Ts = wl.make_batches(64, 10, 33, 1, seed=82)
    n = oracle.num_threads()
    outs = []
    for t in (1, max(2, n)):
        oracle.set_num_threads(t)
        st = oracle.new_state(mlp.layers, np.float32)
        o = oracle.mlp_step(st, Xs[0], Ts[0], 0.01, 0.9, np.float32)
        outs.append((o, st))
    oracle.set_num_threads(n)
    for l in range(3):
        assert np.array_equal(outs[0][1][l]["values"], outs[1][1][l]["values"])
        assert np.array_equal(outs[0][0]["dZ"][l], outs[1][0]["dZ"][l])


@pytest.mark.parametrize("nesterov", [False, True])
def test_momentum_matches_library_sgd(oracle, nesterov):
    """torch.optim.SGD (momentum 0.9, no dampening, no weight decay; Nesterov or not) on the CPU, constant
    learning rate: its buffer is -velocity/lr, its weights must follow the oracle's step for step."""
    import torch
    rng = np.random.default_rng(41)
    n, lr, mu, T = 64, 0.03, 0.9, 15
    w0 = rng.standard_normal(n)
    grads = rng.standard_normal((T, n))
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, nesterov=nesterov)
    w, v = w0.copy(), np.zeros(n)
    for t in range(T):
        p.grad = torch.tensor(grads[t], dtype=torch.float64)
        opt.step()
        w, v, _, _ = oracle.momentum(w, v, grads[t], lr, mu, dtype=np.float64, nesterov=nesterov)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-13), t
        assert np.allclose(v, -lr * opt.state[p]["momentum_buffer"].numpy(), rtol=1e-12, atol=1e-14), t


def test_nesterov_closed_forms(oracle):
    rng = np.random.default_rng(43)
    n = 20
    w0, v0, g = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    # mu = 0: both variants are plain gradient descent
    a = oracle.momentum(w0, v0, g, 0.05, 0.0, dtype=np.float64, nesterov=True)
    b = oracle.momentum(w0, v0, g, 0.05, 0.0, dtype=np.float64, nesterov=False)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # one step from rest: v = -lr g, w = w0 - (1 + mu) lr g
    w, v, Sw, Sv = oracle.momentum(w0, np.zeros(n), g, 0.1, 0.9, dtype=np.float64, nesterov=True)
    assert np.allclose(v, -0.1 * g, rtol=1e-14) and np.allclose(w, w0 - 1.9 * 0.1 * g, rtol=1e-13, atol=1e-15)
    assert np.allclose(Sw, np.abs(w0) + 1.9 * 0.1 * np.abs(g), rtol=1e-13)
    # the velocity itself is the same in both variants
    w2, v2, _, _ = oracle.momentum(w0, v0, g, 0.1, 0.9, dtype=np.float64, nesterov=False)
    w3, v3, _, _ = oracle.momentum(w0, v0, g, 0.1, 0.9, dtype=np.float64, nesterov=True)
    assert np.array_equal(v2, v3) and np.allclose(w3 - w2, 0.9 * v3 - 0.1 * g - v3, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("nesterov", [False, True])
def test_training_loop_matches_masked_dense_autograd(oracle, nesterov):
    """The whole loop (feedforward, loss gradient / batch size, backpropagate from the step's initial weights,
    optimize weights AND biases) against an independent implementation: a masked dense MLP in torch (CPU, fp64),
    gradients by autograd, torch.optim.SGD with momentum -- the masked reference the paper compares with
    (Section 5).  Constant learning rate, so torch's v = mu v + g ; w -= lr v is the same iteration."""
    import torch
    mlp = _tiny_mlp()
    rng = np.random.default_rng(77)
    B, steps, lr, mu = 5, 4, 0.1, 0.9
    Xs = rng.standard_normal((steps, 7, B)); Ts = rng.integers(0, 3, size=(steps, B))
    state = oracle.new_state(mlp.layers, np.float64)
    Ws, Ms, bs = [], [], []
    for lay in mlp.layers:
        W, M = _dense(lay)
        Ws.append(torch.nn.Parameter(torch.tensor(W))); Ms.append(torch.tensor(M)); bs.append(torch.nn.Parameter(torch.tensor(lay.bias, dtype=torch.float64)))
    opt = torch.optim.SGD(Ws + bs, lr=lr, momentum=mu, nesterov=nesterov)
    for t in range(steps):
        out = oracle.mlp_step(state, Xs[t], Ts[t], lr, mu, np.float64, nesterov=nesterov)
        a = torch.tensor(Xs[t])
        for l in range(3):
            a = (Ws[l] * Ms[l]) @ a + bs[l][:, None]
            if l < 2:
                a = torch.relu(a)
        loss = torch.nn.functional.cross_entropy(a.T, torch.tensor(Ts[t]), reduction="mean")
        opt.zero_grad(); loss.backward(); opt.step()
        assert out["loss"] == pytest.approx(float(loss), rel=1e-12)
        for l, lay in enumerate(mlp.layers):
            W = Ws[l].detach().numpy()
            got = np.array([W[i, lay.indices[p]] for i in range(lay.rows) for p in range(lay.indptr[i], lay.indptr[i + 1])])
            np.testing.assert_allclose(state[l]["values"], got, rtol=1e-10, atol=1e-13, err_msg=f"values[{l}] after step {t}")
            np.testing.assert_allclose(state[l]["bias"], bs[l].detach().numpy(), rtol=1e-10, atol=1e-13, err_msg=f"bias[{l}] after step {t}")


# ---- the normalisers S = sum of |terms| that set every tolerance of the parity tests ------------------
# Each one is recomputed here from loops written out in the test, on inputs with non-zero velocity and
# mixed signs, and compared exactly (to fp64 rounding of a different summation order).

def test_loss_normaliser_is_mean_of_abs_lse_plus_abs_target_logit(oracle):
    rng = np.random.default_rng(91)
    C, B = 7, 9
    Z = rng.standard_normal((C, B)) * 4.0 - 1.0      # logits of both signs, some lse negative
    Z[:, 0] -= 9.0                                   # a column whose log-sum-exp is negative
    labels = rng.integers(0, C, size=B)
    loss, S_loss, dZ, SdZ = oracle.softmax_ce(Z, labels, np.float64)
    s = 0.0; l = 0.0
    for c in range(B):
        m = max(Z[i, c] for i in range(C))
        lse = m + math.log(sum(math.exp(Z[i, c] - m) for i in range(C)))
        l += lse - Z[labels[c], c]
        s += abs(lse) + abs(Z[labels[c], c])
        for i in range(C):
            p = math.exp(Z[i, c] - lse); hot = 1.0 if i == labels[c] else 0.0
            assert SdZ[i, c] == pytest.approx((p + hot) / B, rel=1e-13)
            assert dZ[i, c] == pytest.approx((p - hot) / B, rel=1e-12, abs=1e-17)
    assert any(max(Z[:, c]) + math.log(np.exp(Z[:, c] - max(Z[:, c])).sum()) < 0 for c in range(B))
    assert loss == pytest.approx(l / B, rel=1e-13)
    assert S_loss == pytest.approx(s / B, rel=1e-13)
    assert S_loss > abs(loss)                        # |lse| + |z_t| dominates |lse - z_t|


@pytest.mark.parametrize("with_Sg", [False, True])
@pytest.mark.parametrize("lr", [0.05, -0.05])
def test_momentum_normalisers_plain(oracle, with_Sg, lr):
    """Sv = mu |v| + |lr| Sg and Sw = |w| + Sv, with Sg = |g| when no normaliser of g is handed in."""
    rng = np.random.default_rng(92)
    n, mu = 40, 0.9
    w0, v0, g = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    Sg = np.abs(g) * (1.0 + rng.random(n) * 3.0) if with_Sg else None    # Sg >= |g|, as a sum of |terms| is
    w, v, Sw, Sv = oracle.momentum(w0, v0, g, lr, mu, Sg=Sg, dtype=np.float64)
    for k in range(n):
        sg = abs(lr) * (Sg[k] if with_Sg else abs(g[k]))
        sv = mu * abs(v0[k]) + sg
        assert Sv[k] == pytest.approx(sv, rel=1e-14)
        assert Sw[k] == pytest.approx(abs(w0[k]) + sv, rel=1e-14)
        assert v[k] == pytest.approx(mu * v0[k] - lr * g[k], rel=1e-13, abs=1e-16)
        assert w[k] == pytest.approx(w0[k] + mu * v0[k] - lr * g[k], rel=1e-13, abs=1e-16)
    # the normalisers are those of the starting point: they do not follow the new velocity
    assert not np.allclose(Sv, np.abs(v))


@pytest.mark.parametrize("with_Sg", [False, True])
def test_momentum_normalisers_nesterov_with_velocity(oracle, with_Sg):
    """Nesterov, expanded: w' = w + mu^2 v - (1 + mu) lr g, so Sw = |w| + mu^2 |v| + (1 + mu) lr Sg; Sv as plain."""
    rng = np.random.default_rng(93)
    n, mu, lr = 40, 0.8, 0.07
    w0, v0, g = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n)
    Sg = np.abs(g) * (1.0 + rng.random(n) * 3.0) if with_Sg else None
    w, v, Sw, Sv = oracle.momentum(w0, v0, g, lr, mu, Sg=Sg, dtype=np.float64, nesterov=True)
    for k in range(n):
        sg = lr * (Sg[k] if with_Sg else abs(g[k]))
        assert Sv[k] == pytest.approx(mu * abs(v0[k]) + sg, rel=1e-14)
        assert Sw[k] == pytest.approx(abs(w0[k]) + mu * mu * abs(v0[k]) + (1.0 + mu) * sg, rel=1e-14)
        assert w[k] == pytest.approx(w0[k] + mu * mu * v0[k] - (1.0 + mu) * lr * g[k], rel=1e-13, abs=1e-16)


@pytest.mark.parametrize("nesterov", [False, True])
def test_step_normalisers_follow_the_gradient_normalisers(oracle, nesterov):
    """The normalisers a whole step reports for the new weights, velocities and biases are built from the
    step's own Sg / Sdb (sums over the batch of |dZ x|, |dZ|) and from the state the step started with."""
    mlp = _tiny_mlp()
    rng = np.random.default_rng(94)
    B, lr, mu = 6, 0.2, 0.9
    state = oracle.new_state(mlp.layers, np.float64)
    for t in range(2):      # the second step starts with non-zero velocities
        X = rng.standard_normal((7, B)); labels = rng.integers(0, 3, size=B)
        before = [{k: np.array(st[k]) for k in ("values", "bias", "vel_w", "vel_b")} for st in state]
        out = oracle.mlp_step(state, X, labels, lr, mu, np.float64, nesterov=nesterov)
        for l, lay in enumerate(mlp.layers):
            inp = X if l == 0 else out["A"][l - 1]
            p = 0
            for i in range(lay.rows):
                sdb = sum(abs(out["dZ"][l][i, c]) for c in range(B))
                assert out["Sdb"][l][i] == pytest.approx(sdb, rel=1e-13)
                svb = mu * abs(before[l]["vel_b"][i]) + lr * sdb
                assert out["Sbv"][l][i] == pytest.approx(svb, rel=1e-13)
                swb = abs(before[l]["bias"][i]) + (mu * svb + lr * sdb if nesterov else svb)
                assert out["Sbw"][l][i] == pytest.approx(swb, rel=1e-13)
                for q in range(lay.indptr[i], lay.indptr[i + 1]):
                    sg = sum(abs(out["dZ"][l][i, c] * inp[lay.indices[q], c]) for c in range(B))
                    assert out["Sg"][l][q] == pytest.approx(sg, rel=1e-13)
                    sv = mu * abs(before[l]["vel_w"][q]) + lr * sg
                    assert out["Sv"][l][q] == pytest.approx(sv, rel=1e-13)
                    sw = abs(before[l]["values"][q]) + (mu * sv + lr * sg if nesterov else sv)
                    assert out["Sw"][l][q] == pytest.approx(sw, rel=1e-13)
                    p += 1
            assert p == lay.nnz
        if t == 1:
            assert all(np.abs(b["vel_w"]).max() > 0 for b in before)
