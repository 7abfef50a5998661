"""mlp_train_step against the oracle.

Strict gate ("stage parity"): every kernel of a step is checked at 1e-5 * S against the oracle
applied to the GPU's own inputs of that stage (read back from the workspace), so rounding does
not compound from stage to stage and a ReLU unit within rounding of zero cannot flip a mask:
the mask is taken from the GPU's activations on both sides.  Free-running runs (GPU and oracle
each on their own trajectory) are checked with the tie rule and a looser, stated tolerance.
"""
import hashlib

import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl
from test_gpu_parity import close, raw_i32, TOL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2407_17437_amd import binding
    return binding


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    return torch


@pytest.fixture(scope="module", autouse=True)
def sparse_route_only(nb):
    """These tests are about the sparse kernels: layers are bound with the automatic choice of the dense route
    switched off (tests/test_gpu_dense.py and the full-size tests run with the library's default)."""
    nb.nerva_set_dense_threshold(2.0)
    yield
    nb.nerva_set_dense_threshold(0.4)


def snapshot(M):
    return [dict(values=l.values.cpu().numpy().copy(), bias=l.bias.cpu().numpy().copy(),
                 vel_w=l.velocity.cpu().numpy().copy(), vel_b=l.bias_velocity.cpu().numpy().copy())
            for l in M.layers]


def stage_parity(nb, torch, oracle, M, mlp, before, X, labels, batch, lr, mu, unfused, nesterov=False):
    """Compare one finished GPU step, stage by stage, with the oracle fed the GPU's inputs."""
    L = len(M.layers)
    A = [M.view("A", l, batch).cpu().numpy() for l in range(L)]
    dZ = [M.view("dZ", l, batch).cpu().numpy() for l in range(L)]
    worst = 0.0
    for l, lay in enumerate(mlp.layers):
        inp = X if l == 0 else A[l - 1]
        Y, S = oracle.spmm(lay.rows, lay.cols, lay.indptr, lay.indices, before[l]["values"], before[l]["bias"],
                           inp, lay.relu)
        worst = max(worst, close(A[l], Y, S, what=f"A[{l}]"))
    loss, S_loss, dZL, SdZL = oracle.softmax_ce(A[L - 1], labels)
    worst = max(worst, close(dZ[L - 1], dZL, SdZL, what="dZ[last]"))
    assert abs(float(M.loss.item()) - loss) <= TOL * S_loss, (float(M.loss.item()), loss)
    for l in range(L - 1, -1, -1):
        lay = mlp.layers[l]
        if l > 0:
            dA, SdA = oracle.spmm_t(lay.rows, lay.cols, lay.indptr, lay.indices, before[l]["values"], dZ[l])
            ref = np.where(A[l - 1] > 0, dA, 0).astype(np.float32)
            worst = max(worst, close(dZ[l - 1], ref, SdA, what=f"dZ[{l - 1}]"))
        inp = X if l == 0 else A[l - 1]
        g, Sg, db, Sdb = oracle.sddmm(lay.rows, lay.cols, lay.indptr, lay.indices, dZ[l], inp)
        if unfused:
            worst = max(worst, close(M.view("g", l, batch).cpu().numpy(), g, Sg, what=f"g[{l}]"))
            worst = max(worst, close(M.view("db", l, batch).cpu().numpy(), db, Sdb, what=f"db[{l}]"))
        w, v, Sw, Sv = oracle.momentum(before[l]["values"], before[l]["vel_w"], g, lr, mu, Sg, nesterov=nesterov)
        worst = max(worst, close(M.layers[l].velocity.cpu().numpy(), v, Sv, what=f"velocity[{l}]"))
        worst = max(worst, close(M.layers[l].values.cpu().numpy(), w, Sw, what=f"values[{l}]"))
        b, bv, Sb, Sbv = oracle.momentum(before[l]["bias"], before[l]["vel_b"], db, lr, mu, Sdb, nesterov=nesterov)
        worst = max(worst, close(M.layers[l].bias_velocity.cpu().numpy(), bv, Sbv, what=f"bias_velocity[{l}]"))
        worst = max(worst, close(M.layers[l].bias.cpu().numpy(), b, Sb, what=f"bias[{l}]"))
    return worst


CASES = [
    # sizes, kwargs, batch, steps
    ((7, 5, 4, 3), dict(layer_nnz=(14, 9, 8), bias_std=0.3), 3, 3),
    ((48, 32, 16, 10), dict(sparsity=0.7, bias_std=0.1), 20, 3),
    ((100, 300, 50, 10), dict(sparsity=0.9), 100, 2),
    ((64, 40, 10), dict(sparsity=0.5), 260, 2),
    ((40, 30, 20, 10), dict(sparsity=0.999), 16, 2),          # almost every row empty
    ((6000, 300, 10), dict(sparsity=0.98, bias_std=0.1), 200, 2),  # first layer's input beyond an L2: tiled SDDMM + update
    ((100, 300, 10), dict(layer_nnz=(6000, 3000), bias_std=0.1), 64, 2),  # output layer stores every entry: streaming kernels, fused update
]


@pytest.mark.parametrize("sizes,kw,batch,steps", CASES)
@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("separate_head", [False, True])
def test_stage_parity_small(nb, torch_mod, oracle, sizes, kw, batch, steps, unfused, separate_head):
    """Every stage of a step against the oracle, with the output layer's forward product, loss
    and transposed product in one launch (the default for small output layers) and as three."""
    torch = torch_mod
    mlp = wl.make_mlp(sizes, pattern_seed=100, value_seed=200, **kw)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, steps, seed=300)
    flags = (nb.NERVA_MLP_UNFUSED if unfused else 0) | (nb.NERVA_MLP_SEPARATE_HEAD if separate_head else 0)
    M = nb.MLP(mlp, batch, flags)
    for t in range(steps):
        before = snapshot(M)
        Xd = nb.to_dense(Xs[t]); lab = torch.as_tensor(Ts[t]).cuda()
        M.train_step(Xd, lab, batch, 0.05, 0.9)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, unfused)
    M.close()


def test_stage_parity_staged_products(nb, torch_mod, oracle):
    """A batch of 512 on layers with ~200 entries per row: the forward products of both hidden layers and the
    transposed product of the second (with the ReLU mask of the first applied as it is stored) take the
    staged kernel; two steps, so that the second uses weights and mirror values the first one updated."""
    torch = torch_mod
    sizes, batch = (600, 2048, 2048, 10), 512
    mlp = wl.make_mlp(sizes, sparsity=0.9, bias_std=0.1, pattern_seed=101, value_seed=201)
    for l, (rows, cols) in enumerate([(2048, 600), (2048, 2048)]):
        lay = mlp.layers[l]
        assert nb.nerva_plan_staged_host(rows, cols, lay.indptr, lay.indices, batch)[0].shape[0] >= 32
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 2, seed=301)
    M = nb.MLP(mlp, batch)
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, False)
    M.close()


def test_stage_parity_power_law_layer(nb, torch_mod, oracle):
    """A hidden layer with power-law rows at batch 1024: its forward product and its SDDMM + update stage the long
    rows through LDS and serve the thousands of short rows with the other kernels, in the training step's own
    launches (fused update in the common finish pass); two steps, every stage against the oracle."""
    torch = torch_mod
    n, batch = 6144, 1024
    mlp = wl.make_mlp((n, n, 10), sparsity=0.97, bias_std=0.1, pattern_seed=102, value_seed=202)
    lens = wl.zipf_row_nnz(n, n, n * n * 3 // 100, 1.2, seed=19)
    indptr, indices = wl.pattern_from_row_nnz(lens, n, seed=20)
    prng = np.random.default_rng(21)
    mlp.layers[0] = wl.SparseLayerData(n, n, indptr, indices, (prng.standard_normal(int(indptr[-1])) * 0.02).astype(np.float32),
                                       (prng.standard_normal(n) * 0.1).astype(np.float32), True)
    assert nb.nerva_plan_staged_host(n, n, indptr, indices, batch, nb.NERVA_PACK_MAX_LEN + 1)[0].shape[0] == 16
    Xs, Ts = wl.make_batches(n, 10, batch, 2, seed=302)
    M = nb.MLP(mlp, batch)
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, False)
    M.close()


def _digest(*arrays):
    h = hashlib.sha256()
    for a in arrays:
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()


def test_config1_ten_steps(nb, torch_mod, oracle):
    """3072-1024-512-10 at 99 % sparsity, batch 100, 10 momentum-SGD steps (lr 0.01, momentum 0.9):
    stage parity at every step, a free-running oracle beside it, pattern and mirror bit-identical."""
    torch = torch_mod
    batch, steps, lr, mu = 100, 10, 0.01, 0.9
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=0.99)
    Xs, Ts = wl.make_batches(3072, 10, batch, steps, seed=3000)
    M = nb.MLP(mlp, batch)
    M2 = nb.MLP(mlp, batch, nb.NERVA_MLP_UNFUSED)
    free = oracle.new_state(mlp.layers, np.float32)
    pat0 = [_digest(l.indptr.cpu().numpy(), l.indices.cpu().numpy()) for l in M.layers]
    assert pat0 == [_digest(l.indptr, l.indices) for l in mlp.layers]
    mir0 = []
    for l in M.layers:
        ip, ix, _, pm = nb.sparse_linear_mirror(l.handle)
        mir0.append(_digest(raw_i32(nb, torch, ip, l.cols + 1), raw_i32(nb, torch, ix, l.nnz), raw_i32(nb, torch, pm, l.nnz)))
    worst = 0.0
    for t in range(steps):
        before = snapshot(M)
        Xd = nb.to_dense(Xs[t]); lab = torch.as_tensor(Ts[t]).cuda()
        M.train_step(Xd, lab, batch, lr, mu)
        M2.train_step(Xd, lab, batch, lr, mu)
        torch.cuda.synchronize()
        worst = max(worst, stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False))
        # free-running oracle with the tie rule: where the two ReLU masks differ, the oracle's
        # pre-activation must be within rounding of zero, and the oracle then takes the GPU's mask
        probe = oracle.mlp_forward(free, Xs[t], np.float32, want_S=True)
        masks = []
        for l in range(2):
            ga = M.view("A", l, batch).cpu().numpy()
            gm = ga > 0
            diff = gm != (probe[0][l] > 0)
            if diff.any():
                # one side has the unit at zero, the other barely above it
                assert np.all(np.abs(ga[diff] - probe[0][l][diff]) <= 1e-4 * probe[1][l][diff]), \
                    f"step {t} layer {l}: ReLU masks differ away from zero"
            masks.append(gm)
        masks.append(None)
        out = oracle.mlp_step(free, Xs[t], Ts[t], lr, mu, np.float32, relu_masks=masks)
        gl = float(M.loss.item())
        # Free-running tolerance: per-stage rounding (<= 1e-5 S, a few 1e-7 in practice) is carried through
        # three layers and t momentum steps; 1e-4 relative leaves an order of magnitude of room.
        assert abs(gl - out["loss"]) <= 1e-4 * abs(out["loss"]), (t, gl, out["loss"])
        assert 1.5 < gl < 4.0
        # the pattern and the mirror's index arrays are bit-identical after every update
        assert [_digest(l.indptr.cpu().numpy(), l.indices.cpu().numpy()) for l in M.layers] == pat0
    for li, l in enumerate(M.layers):
        ip, ix, vt, pm = nb.sparse_linear_mirror(l.handle)
        assert _digest(raw_i32(nb, torch, ip, l.cols + 1), raw_i32(nb, torch, ix, l.nnz), raw_i32(nb, torch, pm, l.nnz)) == mir0[li]
        w_gpu = l.values.cpu().numpy()
        scale = np.abs(free[li]["values"]) + np.abs(free[li]["vel_w"]) + 1e-3
        assert np.all(np.abs(w_gpu - free[li]["values"]) <= 1e-4 * scale), li
        # fused and unfused pipelines run the same arithmetic: bit-identical state
        assert torch.equal(l.values, M2.layers[li].values) and torch.equal(l.velocity, M2.layers[li].velocity)
        assert torch.equal(l.bias, M2.layers[li].bias)
        # the mirror's values follow the update (layer 0's mirror is never read and may lag)
        if li > 0:
            from test_gpu_parity import raw_f32
            perm = raw_i32(nb, torch, pm, l.nnz)
            assert np.array_equal(raw_f32(nb, torch, vt, l.nnz), w_gpu[perm])
    print(f"worst stage error / (1e-5 S) over {steps} steps: {worst / 1.0:.3f}")
    M.close(); M2.close()


def test_step_is_bit_reproducible(nb, torch_mod):
    torch = torch_mod
    mlp = wl.make_mlp((256, 128, 64, 10), sparsity=0.8)
    Xs, Ts = wl.make_batches(256, 10, 100, 4, seed=11)
    states = []
    for _ in range(2):
        M = nb.MLP(mlp, 100)
        for t in range(4):
            M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), 100, 0.05, 0.9)
        torch.cuda.synchronize()
        states.append([(l.values.clone(), l.velocity.clone(), l.bias.clone()) for l in M.layers] + [M.loss.clone()])
        M.close()
    for a, b in zip(states[0][:-1], states[1][:-1]):
        assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert torch.equal(states[0][-1], states[1][-1])


def test_mlp_forward_and_errors(nb, torch_mod, oracle):
    torch = torch_mod
    mlp = wl.make_mlp((64, 32, 10), sparsity=0.6, bias_std=0.2)
    Xs, _ = wl.make_batches(64, 10, 50, 1, seed=12)
    M = nb.MLP(mlp, 50)
    logits = M.forward(nb.to_dense(Xs[0]), 50)
    torch.cuda.synchronize()
    st = oracle.new_state(mlp.layers)
    A, S = oracle.mlp_forward(st, Xs[0], np.float32, want_S=True)
    # two chained layers: compare the last against the oracle fed the GPU's hidden activations
    hidden = M.view("A", 0, 50).cpu().numpy()
    close(hidden, A[0], S[0], what="hidden")
    Y, S1 = oracle.spmm(10, 32, mlp.layers[1].indptr, mlp.layers[1].indices, mlp.layers[1].values, mlp.layers[1].bias, hidden, False)
    close(logits.cpu().numpy(), Y, S1, what="logits")
    X = nb.to_dense(Xs[0])
    lab = torch.zeros(50, dtype=torch.int32, device="cuda")
    with pytest.raises(nb.NervaError) as e:
        M.train_step(X, lab, 51, 0.1, 0.9)                        # ldx (64) >= 51 but above max_batch
    assert e.value.code == nb.NERVA_ERR_SHAPE
    small = torch.empty(16, device="cuda")
    with pytest.raises(nb.NervaError) as e:
        nb.mlp_train_step(M.handle, X, 64, lab, 50, 0.1, 0.9, small, M.loss)
    assert e.value.code == nb.NERVA_ERR_WORKSPACE
    # layers that do not chain
    a = nb.SparseLinear(mlp.layers[0]); b = nb.SparseLinear(mlp.layers[0])
    with pytest.raises(nb.NervaError) as e:
        nb.mlp_create([a.handle, b.handle], [a.velocity, b.velocity], [a.bias_velocity, b.bias_velocity], 8)
    assert e.value.code in (nb.NERVA_ERR_SHAPE, nb.NERVA_ERR_ARGUMENT)
    a.close(); b.close(); M.close()


def test_step_profiler_slots(nb, torch_mod):
    """Per-launch event timing: one slot per launch in launch order, and it does not change results."""
    torch = torch_mod
    mlp = wl.make_mlp((256, 128, 64, 10), sparsity=0.8)
    Xs, Ts = wl.make_batches(256, 10, 100, 3, seed=13)
    ref = nb.MLP(mlp, 100); M = nb.MLP(mlp, 100)
    nb.mlp_profile_enable(M.handle, 2)
    for t in range(3):                                   # the third step is past max_steps: not recorded
        for m in (ref, M):
            m.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), 100, 0.05, 0.9)
    torch.cuda.synchronize()
    steps, slots = nb.mlp_profile_read(M.handle)
    assert steps == 2
    names = [n for n, _ in slots]
    assert names == ["spmm_forward[0]", "spmm_forward[1]", "spmm_forward+softmax_ce+spmm_transposed[2]",
                     "spmm_transposed+sddmm_update[1]", "sddmm_update+sddmm_update[0]"]
    assert all(0.0 < ms < 50.0 for _, ms in slots)
    nb.mlp_profile_enable(M.handle, 0)
    assert nb.mlp_profile_read(M.handle) == (0, [])
    for a, b in zip(ref.layers, M.layers):
        assert torch.equal(a.values, b.values) and torch.equal(a.velocity, b.velocity)
    ref.close(); M.close()
    # the same network with the output layer's three launches kept apart
    S = nb.MLP(mlp, 100, nb.NERVA_MLP_SEPARATE_HEAD)
    nb.mlp_profile_enable(S.handle, 1)
    S.train_step(nb.to_dense(Xs[0]), torch.as_tensor(Ts[0]).cuda(), 100, 0.05, 0.9)
    torch.cuda.synchronize()
    steps, slots = nb.mlp_profile_read(S.handle)
    assert steps == 1
    assert [n for n, _ in slots] == ["spmm_forward[0]", "spmm_forward[1]", "spmm_forward[2]", "softmax_ce[2]",
                                     "spmm_transposed[2]", "spmm_transposed+sddmm_update[1]",
                                     "sddmm_update+sddmm_update[0]"]
    S.close()


def test_head_loss_is_reproducible(nb, torch_mod):
    """The fused head leaves one loss per column and a later launch of the step takes their mean in
    a fixed order: many steps in a row give the same losses on two identical runs, also with a
    batch that is not a multiple of the four columns a work-group owns."""
    torch = torch_mod
    for batch in (100, 37, 3):
        mlp = wl.make_mlp((96, 64, 10), sparsity=0.7, bias_std=0.1)
        Xs, Ts = wl.make_batches(96, 10, batch, 12, seed=21)
        runs = []
        for _ in range(2):
            M = nb.MLP(mlp, batch)
            losses = []
            for t in range(12):
                M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
                losses.append(float(M.loss.item()))
            runs.append((losses, [l.values.clone() for l in M.layers]))
            M.close()
        assert runs[0][0] == runs[1][0]
        assert all(torch.equal(a, b) for a, b in zip(runs[0][1], runs[1][1]))
        assert all(np.isfinite(x) and x > 0 for x in runs[0][0])


@pytest.mark.parametrize("unfused", [False, True])
def test_stage_parity_nesterov(nb, torch_mod, oracle, unfused):
    """Nesterov momentum (the optimiser of the paper's experiments) with a learning rate that follows the
    paper's step decay: the rate is an argument of every step."""
    from paper_2407_17437_amd import schedule
    torch = torch_mod
    sizes, batch, mu = (100, 300, 50, 10), 100, 0.9
    mlp = wl.make_mlp(sizes, sparsity=0.9, pattern_seed=110, value_seed=210, bias_std=0.1)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 4, seed=310)
    flags = nb.NERVA_MLP_NESTEROV | (nb.NERVA_MLP_UNFUSED if unfused else 0)
    M = nb.MLP(mlp, batch, flags)
    plain = nb.MLP(mlp, batch)
    lr0 = schedule.initial_learning_rate(0.1)
    for t in range(4):
        lr = schedule.learning_rate(t, 4, lr0)                   # 0.03, 0.03, 0.003, 0.0003
        before = snapshot(M)
        Xd = nb.to_dense(Xs[t]); lab = torch.as_tensor(Ts[t]).cuda()
        M.train_step(Xd, lab, batch, lr, mu)
        plain.train_step(Xd, lab, batch, lr, mu)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, unfused, nesterov=True)
    assert not torch.equal(M.layers[0].values, plain.layers[0].values)     # the variant is really a different update
    M.close(); plain.close()


@pytest.mark.parametrize("batch,ld", [(1, 1), (1, 32), (3, 4)])
def test_mlp_forward_single_examples(nb, torch_mod, oracle, batch, ld):
    """Inference on one (or a few) examples (Section 5.4 measures batch-1 inference)."""
    torch = torch_mod
    mlp = wl.make_mlp((3072, 1024, 512, 10), sparsity=0.95, bias_std=0.1)
    Xs, _ = wl.make_batches(3072, 10, batch, 1, seed=14)
    M = nb.MLP(mlp, 32)
    logits = M.forward(nb.to_dense(Xs[0], ld=ld), batch)
    torch.cuda.synchronize()
    st = oracle.new_state(mlp.layers)
    prev = Xs[0]
    for l, lay in enumerate(mlp.layers):                       # every layer against the oracle fed the GPU's input
        Y, S = oracle.spmm(lay.rows, lay.cols, lay.indptr, lay.indices, lay.values, lay.bias, prev, lay.relu)
        got = M.view("A", l, batch).cpu().numpy()
        close(got, Y, S, what=f"A[{l}] batch {batch}")
        prev = got
    assert logits.shape == (10, batch)
    M.close()


def test_layer_trained_as_first_layer_then_chained_further_up(nb, torch_mod, oracle):
    """A training step leaves the mirror's values of an MLP's first layer alone (nothing reads them).  The same
    layer object chained at a later position of another MLP must backpropagate through its CURRENT weights: the
    library remembers that the mirror is behind and refreshes it before the first product that reads it."""
    torch = torch_mod
    batch, lr, mu = 64, 0.05, 0.9
    first = wl.make_mlp((40, 48, 10), sparsity=0.6, bias_std=0.1, pattern_seed=110, value_seed=210)
    M1 = nb.MLP(first, batch)
    Xs, Ts = wl.make_batches(40, 10, batch, 3, seed=310)
    for t in range(3):       # three steps: layer 0's weights move away from the mirror's copy
        M1.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, lr, mu)
    torch.cuda.synchronize()
    shared = M1.layers[0]                                       # 48 x 40, ReLU
    w_now = shared.values.cpu().numpy().copy()
    _, _, vt_addr, perm_addr = nb.sparse_linear_mirror(shared.handle)
    from test_gpu_parity import raw_f32
    perm = raw_i32(nb, torch, perm_addr, shared.nnz)
    assert not np.array_equal(raw_f32(nb, torch, vt_addr, shared.nnz), w_now[perm])      # the mirror is behind
    # a second MLP: a new 40-wide input layer below, the shared layer in the middle, a new output layer on top
    below = wl.make_mlp((30, 40, 10), sparsity=0.5, bias_std=0.1, pattern_seed=111, value_seed=211).layers[0]
    top = wl.make_mlp((40, 48, 10), sparsity=0.5, bias_std=0.1, pattern_seed=112, value_seed=212).layers[1]
    L0 = nb.SparseLinear(below, batch); L2 = nb.SparseLinear(top, batch)
    handle = nb.mlp_create([L0.handle, shared.handle, L2.handle], [L0.velocity, shared.velocity, L2.velocity],
                           [L0.bias_velocity, shared.bias_velocity, L2.bias_velocity], batch)
    nbytes = nb.mlp_workspace_bytes(handle, batch)
    ws = torch.full((nbytes // 4,), float("nan"), device="cuda"); loss = torch.zeros(1, device="cuda")
    lay = nb.mlp_workspace_layout(handle, batch, 3)
    X2, T2 = wl.make_batches(30, 10, batch, 1, seed=311)
    Xd = nb.to_dense(X2[0])
    nb.mlp_train_step(handle, Xd, Xd.stride(0), torch.as_tensor(T2[0]).cuda(), batch, lr, mu, ws, loss)
    torch.cuda.synchronize()
    ld = lay[0]
    dZ1 = ws[lay[1 + 4 * 1 + 1] // 4:][:48 * ld].view(48, ld)[:, :batch].cpu().numpy()
    dZ0 = ws[lay[1 + 4 * 0 + 1] // 4:][:40 * ld].view(40, ld)[:, :batch].cpu().numpy()
    A0 = ws[lay[1 + 4 * 0 + 0] // 4:][:40 * ld].view(40, ld)[:, :batch].cpu().numpy()
    d = first.layers[0]
    dA, SdA = oracle.spmm_t(d.rows, d.cols, d.indptr, d.indices, w_now, dZ1)
    close(dZ0, np.where(A0 > 0, dA, 0).astype(np.float32), SdA, what="dZ below the shared layer (current weights)")
    # and afterwards the mirror follows the weights again (the layer sits above the first one now)
    assert np.array_equal(raw_f32(nb, torch, vt_addr, shared.nnz), shared.values.cpu().numpy()[perm])
    nb.mlp_destroy(handle)
    L0.close(); L2.close(); M1.close()


@pytest.mark.parametrize("sizes,sparsity,batch,unfused", [
    ((100, 2100, 8600, 10), 0.992, 256, False),     # 64-column tiles (16 lanes per mirror row): a 128-column tile of dZ would exceed an L2
    ((100, 2100, 5200, 10), 0.985, 200, False),     # 128-column tiles, ragged last tile
    ((100, 2100, 5200, 10), 0.985, 200, True),      # gradients stored, separate momentum kernels
    ((100, 2304, 2304, 2304, 10), 0.98, 512, False),  # 128-column tiles (32 lanes per mirror row), two hidden layers fused in a row
])
def test_stage_parity_backward_on_one_gather_stream(nb, torch_mod, oracle, sizes, sparsity, batch, unfused):
    """Hidden layers whose mirror has only short rows and whose backward operand does not fit an L2: the transposed
    product and the SDDMM + update of the layer run as one launch that gathers every row of dZ once for both
    (Section 4: A = S^T B and S = A B^T); every stage of two steps against the oracle."""
    torch = torch_mod
    mlp = wl.make_mlp(sizes, sparsity=sparsity, bias_std=0.1, pattern_seed=130, value_seed=230)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 2, seed=330)
    M = nb.MLP(mlp, batch, nb.NERVA_MLP_UNFUSED if unfused else 0)
    nb.mlp_profile_enable(M.handle, 1)
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        if t == 0:
            names = [n for n, _ in nb.mlp_profile_read(M.handle)[1]]
            nb.mlp_profile_enable(M.handle, 0)
            if not unfused:
                assert sum(n.startswith("backward_fused") for n in names) == len(sizes) - 3, names
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, unfused)
    M.close()


@pytest.mark.parametrize("batch,unfused", [(256, False), (192, False), (1024, False), (256, True), (40, False), (66, False)])
def test_stage_parity_backward_of_a_saturated_output_layer(nb, torch_mod, oracle, batch, unfused):
    """An output layer that stores every entry (Erdos-Renyi split of a small global density: the 10-row layer
    saturates, as in the wide MLP) and is too large for the fused head: its transposed product, SDDMM and update run
    as one streaming launch that reads the layer's input once (Section 4: A = S^T B and S = A B^T); every stage of
    two steps against the oracle, and the same state, to rounding, as the pipeline of separate kernels."""
    torch = torch_mod
    sizes = (96, 1500, 1200, 10)
    nnz = [int(0.05 * 1500 * 96), int(0.03 * 1200 * 1500), 10 * 1200]
    mlp = wl.make_mlp(sizes, layer_nnz=nnz, bias_std=0.1, pattern_seed=140, value_seed=240)
    assert mlp.layers[2].nnz == 10 * 1200
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 2, seed=340)
    M = nb.MLP(mlp, batch, nb.NERVA_MLP_UNFUSED if unfused else 0)
    nb.mlp_profile_enable(M.handle, 1)
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        if t == 0:
            names = [n for n, _ in nb.mlp_profile_read(M.handle)[1]]
            nb.mlp_profile_enable(M.handle, 0)
            streaming = not unfused and batch >= 64 and batch % 4 == 0      # (narrow or ragged batches take the ordinary kernels)
            assert ("backward_full[2]" in names) == streaming, names
            assert ("spmm_forward+softmax_ce[2]" in names) == streaming, names   # loss gradient formed by the product's finish pass
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, unfused)
    if not unfused:
        # the pipeline of separate kernels from the same start.  Its transposed product adds a row's terms in another
        # order (lane groups first), so the two states agree to rounding, not bit for bit
        mlp2 = wl.make_mlp(sizes, layer_nnz=nnz, bias_std=0.1, pattern_seed=140, value_seed=240)
        M2 = nb.MLP(mlp2, batch, nb.NERVA_MLP_UNFUSED)
        for t in range(2):
            M2.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        for a, b in zip(M.layers, M2.layers):
            for u, v in ((a.values, b.values), (a.velocity, b.velocity), (a.bias, b.bias)):
                u, v = u.cpu().numpy(), v.cpu().numpy()
                assert np.all(np.abs(u - v) <= 1e-5 * (np.abs(v) + 1e-2))
        M2.close()
    M.close()


@pytest.mark.parametrize("static", [False, True])
@pytest.mark.parametrize("sizes,kw,batch", [
    ((3072, 1024, 512, 10), dict(sparsity=0.95), 100),                          # fused head, paired launches
    ((96, 1500, 1200, 10), dict(layer_nnz=(7200, 54000, 12000)), 256),           # column tiles, partial buffers, streaming output layer
])
def test_training_steps_replayed_from_a_hip_graph(nb, torch_mod, sizes, kw, batch, static):
    """A training step only enqueues kernels, so it can be captured: three steps (three batches) recorded into one HIP
    graph, replayed three times with eager work of the same process and synchronisations in between; after every
    replay the weights, momentum buffers and the loss equal, bit for bit, those of a twin trained by plain launches."""
    torch = torch_mod
    lr, mu = 0.05, 0.9
    mlp = wl.make_mlp(sizes, pattern_seed=150, value_seed=250, bias_std=0.1, **kw)
    G = nb.MLP(mlp, batch); E = nb.MLP(mlp, batch)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 3, seed=350)
    Xd = [nb.to_dense(x) for x in Xs]; Td = [torch.as_tensor(t).cuda() for t in Ts]
    loss_g = torch.zeros(1, device="cuda")

    def step(M, k, loss):
        if static:
            nb.mlp_train_step_static(M.handle, Xd[k], Xd[k].stride(0), Td[k], batch, lr, mu, loss)
        else:
            nb.mlp_train_step(M.handle, Xd[k], Xd[k].stride(0), Td[k], batch, lr, mu, M.workspace, loss)

    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for k in range(3):
            step(G, k, loss_g)
    # (capture has run nothing: both twins are still at the start)
    other = torch.zeros(1 << 20, device="cuda")
    for r in range(3):
        g.replay()
        other.add_(1.0)                                   # eager work of the process between the replays
        for k in range(3):
            step(E, k, E.loss)
        torch.cuda.synchronize()
        assert float(other.sum().item()) == (r + 1) * other.numel()
        for a, b in zip(G.layers, E.layers):
            assert torch.equal(a.values, b.values) and torch.equal(a.velocity, b.velocity), f"replay {r}"
            assert torch.equal(a.bias, b.bias) and torch.equal(a.bias_velocity, b.bias_velocity), f"replay {r}"
        assert float(loss_g.item()) == float(E.loss.item()) and np.isfinite(float(loss_g.item()))
    del g
    G.close(); E.close()


def _random_case(seed):
    """A seeded draw of a network and a batch: depths 2-4, widths from a few to 1500, per-layer densities from 2 %
    to full (a layer may also be empty), batches from 1 to 512 including odd ones, every pipeline flag."""
    rng = np.random.default_rng(7000 + seed)
    depth = int(rng.integers(2, 5))
    widths = [int(rng.choice([7, 33, 64, 120, 300, 700, 1500])) for _ in range(depth)] + [int(rng.choice([3, 10, 16, 40]))]
    dens = [float(rng.choice([0.0, 0.02, 0.1, 0.3, 0.6, 1.0], p=[0.05, 0.25, 0.25, 0.2, 0.15, 0.1])) for _ in range(depth)]
    nnz = [int(round(d * widths[l] * widths[l + 1])) for l, d in enumerate(dens)]
    batch = int(rng.choice([1, 3, 8, 33, 64, 100, 132, 256, 512]))
    return tuple(widths), nnz, batch, bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2))


@pytest.mark.parametrize("seed", range(40))
def test_stage_parity_random_networks(nb, torch_mod, oracle, seed):
    """Which kernels serve a step depends on shapes, densities, the batch and the flags (packed, tiled, paired, fused
    backward passes, streaming kernels for saturated layers, the head, the dense route): random draws of all of these,
    every stage of two steps against the oracle."""
    torch = torch_mod
    sizes, nnz, batch, unfused, separate_head, nesterov, dense_route = _random_case(seed)
    mlp = wl.make_mlp(sizes, layer_nnz=nnz, bias_std=0.1, pattern_seed=160 + seed, value_seed=260 + seed)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 2, seed=360 + seed)
    flags = (nb.NERVA_MLP_UNFUSED if unfused else 0) | (nb.NERVA_MLP_SEPARATE_HEAD if separate_head else 0) | \
            (nb.NERVA_MLP_NESTEROV if nesterov else 0)
    print(f"case {seed}: sizes {sizes} nnz {nnz} batch {batch} unfused {unfused} separate_head {separate_head} "
          f"nesterov {nesterov} dense_route {dense_route}", flush=True)
    nb.nerva_set_dense_threshold(0.4 if dense_route else 2.0)
    try:
        M = nb.MLP(mlp, batch, flags)
    finally:
        nb.nerva_set_dense_threshold(2.0)
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, unfused, nesterov=nesterov)
    M.close()
