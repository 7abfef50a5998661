"""Topology updates between steps (dynamic sparse training hook): sparse_linear_rebind + mlp_rebind_velocity.

The pattern of a layer is replaced by another canonical CSR of the same shape; afterwards every
product of the layer, its mirror and a training step through it must match the oracle on the new
pattern to the usual bar (index structure bit-exact, fp32 within 1e-5 * S).  The prune-and-grow
rule used to make new patterns (drop the k entries of smallest magnitude, grow k entries at
unused positions with weight and momentum 0; Mocanu et al.'s SET step, which Section 2 of the
paper refers to) lives here, in the test: the library only rebuilds what depends on the pattern.
"""
import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl
from test_gpu_parity import close, raw_i32, layer_case
from test_gpu_mlp_step import snapshot, stage_parity

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


def prune_and_grow(rows, cols, indptr, indices, values, velocity, k, seed):
    """New canonical CSR with the k smallest-magnitude entries removed and k new positions added
    (value 0, velocity 0); surviving entries keep value and velocity."""
    rng = np.random.default_rng(seed)
    nnz = int(indptr[-1])
    row_of = np.repeat(np.arange(rows), np.diff(indptr))
    keep = np.ones(nnz, dtype=bool)
    keep[np.argsort(np.abs(values), kind="stable")[:k]] = False
    lin = row_of[keep].astype(np.int64) * cols + indices[keep]
    taken = set((row_of.astype(np.int64) * cols + indices).tolist())
    grown = []
    while len(grown) < k:
        c = int(rng.integers(0, rows * cols))
        if c not in taken:
            taken.add(c)
            grown.append(c)
    all_lin = np.concatenate([lin, np.array(grown, dtype=np.int64)])
    all_val = np.concatenate([values[keep], np.zeros(k, dtype=np.float32)])
    all_vel = np.concatenate([velocity[keep], np.zeros(k, dtype=np.float32)])
    order = np.argsort(all_lin, kind="stable")
    all_lin, all_val, all_vel = all_lin[order], all_val[order], all_vel[order]
    new_rows = (all_lin // cols).astype(np.int64)
    new_indptr = np.zeros(rows + 1, dtype=np.int32)
    np.add.at(new_indptr, new_rows + 1, 1)
    new_indptr = np.cumsum(new_indptr).astype(np.int32)
    return new_indptr, (all_lin % cols).astype(np.int32), all_val.astype(np.float32), all_vel.astype(np.float32)


def check_layer(nb, torch, oracle, L, lay, batch):
    rng = np.random.default_rng(batch + lay.nnz)
    X = rng.standard_normal((lay.cols, batch)).astype(np.float32)
    dY = rng.standard_normal((lay.rows, batch)).astype(np.float32)
    Xd = nb.to_dense(X); Yd = nb.dense(lay.rows, batch); dYd = nb.to_dense(dY); dXd = nb.dense(lay.cols, batch)
    g = torch.full((max(lay.nnz, 1),), float("nan"), device="cuda")[:lay.nnz]
    db = torch.full((lay.rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, None, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(lay.rows, lay.cols, lay.indptr, lay.indices, lay.values, lay.bias, X, False)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    dX, SdX = oracle.spmm_t(lay.rows, lay.cols, lay.indptr, lay.indices, lay.values, dY)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    gr, Sg, dbr, Sdb = oracle.sddmm(lay.rows, lay.cols, lay.indptr, lay.indices, dY, X)
    close(g.cpu().numpy(), gr, Sg, what="dvalues"); close(db.cpu().numpy(), dbr, Sdb, what="dbias")
    # the mirror is the canonical CSR of the transposed pattern, bit for bit
    ip, ix, _, pm = nb.sparse_linear_mirror(L.handle)
    row_of = np.repeat(np.arange(lay.rows), np.diff(lay.indptr))
    order = np.argsort(lay.indices, kind="stable")
    want_indptr_t = np.concatenate([[0], np.cumsum(np.bincount(lay.indices, minlength=lay.cols))]).astype(np.int32)
    assert np.array_equal(raw_i32(nb, torch, ip, lay.cols + 1), want_indptr_t)
    assert np.array_equal(raw_i32(nb, torch, ix, lay.nnz), row_of[order].astype(np.int32))
    assert np.array_equal(raw_i32(nb, torch, pm, lay.nnz), order.astype(np.int32))


@pytest.mark.parametrize("rows,cols,density,new_density,batch", [
    (33, 65, 0.2, 0.3, 100),          # nnz grows
    (130, 257, 0.05, 0.02, 64),       # nnz shrinks
    (2500, 300, 0.02, 0.03, 100),     # packed short rows before and after
    (12, 4096, 0.9, 0.1, 100),        # huge rows become ordinary ones
    (50, 40, 0.3, 0.0, 8),            # everything pruned
    (4096, 700, 0.1, 0.15, 256),      # staged products and staged SDDMM before and after
])
def test_layer_rebind(nb, torch_mod, oracle, rows, cols, density, new_density, batch):
    torch = torch_mod
    a = layer_case(rows, cols, density, seed=rows + cols, relu=False)
    b = layer_case(rows, cols, new_density, seed=rows + cols + 77, relu=False)
    b.bias = a.bias                                        # the bias array stays bound
    L = nb.SparseLinear(a, max_batch=batch)
    check_layer(nb, torch, oracle, L, a, batch)
    L.rebind(b.indptr, b.indices, b.values)
    assert L.nnz == b.nnz
    check_layer(nb, torch, oracle, L, b, batch)
    L.rebind(a.indptr, a.indices, a.values)                # and back
    check_layer(nb, torch, oracle, L, a, batch)
    L.close()


def test_mlp_forward_after_a_rebind_that_changes_nnz(nb, torch_mod, oracle):
    """The workspace layout depends on every layer's nnz: after a rebind to a larger pattern the binding asks
    for the layout (and the size) again, and the forward pass through all layers matches the oracle."""
    torch = torch_mod
    sizes, batch = (48, 64, 10), 32
    mlp = wl.make_mlp(sizes, sparsity=0.4, bias_std=0.1, pattern_seed=61, value_seed=62)
    X = np.random.default_rng(63).standard_normal((sizes[0], batch)).astype(np.float32)
    M = nb.MLP(mlp, batch)
    for density in (0.9, 0.1):
        lay = mlp.layers[0]
        new = layer_case(lay.rows, lay.cols, density, seed=64, relu=True)
        M.rebind_layer(0, new.indptr, new.indices, new.values)
        out = M.forward(nb.to_dense(X), batch).cpu().numpy()
        torch.cuda.synchronize()
        A0 = M.view("A", 0, batch).cpu().numpy()
        ref0, S0 = oracle.spmm(lay.rows, lay.cols, new.indptr, new.indices, new.values, M.layers[0].bias.cpu().numpy(), X, True)
        close(A0, ref0, S0, what="A[0]")
        l1 = mlp.layers[1]
        ref1, S1 = oracle.spmm(l1.rows, l1.cols, l1.indptr, l1.indices, l1.values, l1.bias, A0, False)
        close(out, ref1, S1, what="logits")
    M.close()


def test_rebind_rejects_bad_pattern_and_keeps_the_old_one(nb, torch_mod, oracle):
    torch = torch_mod
    a = layer_case(40, 30, 0.3, seed=5, relu=False)
    L = nb.SparseLinear(a, max_batch=16)
    bad = a.indices.copy()
    row = int(np.argmax(np.diff(a.indptr) >= 2)); p = a.indptr[row]
    bad[p], bad[p + 1] = bad[p + 1], bad[p]                # columns no longer ascending
    with pytest.raises(nb.NervaError) as e:
        L.rebind(a.indptr, bad, a.values)
    assert e.value.code == nb.NERVA_ERR_CSR
    short = a.indptr.copy(); short[-1] -= 1                 # indptr[rows] != nnz
    with pytest.raises(nb.NervaError):
        nb.sparse_linear_rebind(L.handle, a.nnz, torch.as_tensor(short).cuda(), L.indices, L.values)
    with pytest.raises(nb.NervaError) as e:
        nb.sparse_linear_rebind(L.handle, a.nnz, None, L.indices, L.values)
    assert e.value.code == nb.NERVA_ERR_ARGUMENT
    check_layer(nb, torch, oracle, L, a, 16)               # still the old pattern, still correct
    L.close()


@pytest.mark.parametrize("nesterov", [False, True])
def test_training_across_topology_updates(nb, torch_mod, oracle, nesterov):
    """Steps, a prune-and-grow update of two layers, more steps: stage parity at every step, and the
    momentum of surviving entries carries over (velocity of grown entries starts at 0)."""
    torch = torch_mod
    sizes, batch, lr, mu = (96, 64, 32, 10), 20, 0.05, 0.9
    mlp = wl.make_mlp(sizes, sparsity=0.8, bias_std=0.1, pattern_seed=11, value_seed=12)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 6, seed=13)
    M = nb.MLP(mlp, batch, nb.NERVA_MLP_NESTEROV if nesterov else 0)

    def steps(ts):
        for t in ts:
            before = snapshot(M)
            M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, lr, mu)
            torch.cuda.synchronize()
            stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False, nesterov=nesterov)

    steps(range(0, 2))
    for round_, ts in enumerate([range(2, 4), range(4, 6)]):
        for l in (0, 2):
            lay, dev = mlp.layers[l], M.layers[l]
            k = max(1, lay.nnz // 5)
            ip, ix, val, vel = prune_and_grow(lay.rows, lay.cols, lay.indptr, lay.indices,
                                              dev.values.cpu().numpy(), dev.velocity.cpu().numpy(), k, seed=100 + 10 * round_ + l)
            assert int(ip[-1]) == lay.nnz and not np.array_equal(ix, lay.indices)
            M.rebind_layer(l, ip, ix, val, vel)
            mlp.layers[l] = wl.SparseLayerData(lay.rows, lay.cols, ip, ix, val, dev.bias.cpu().numpy(), lay.relu)
            assert torch.equal(M.layers[l].velocity.cpu(), torch.as_tensor(vel))
        steps(ts)
    M.close()
