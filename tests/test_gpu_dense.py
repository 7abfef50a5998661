"""The density-adaptive route: products of a dense-enabled layer run as fp32 MFMA products on zero-filled
dense copies of the weights; everything else (SDDMM on the pattern, momentum, values[]) stays sparse.

Same bar as the sparse route: every result against the oracle within 1e-5 * S, element by element.
"""
import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl
from test_gpu_parity import close, layer_case
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


# (rows, cols, density, batch, ld): tiles with ragged edges in M, N and K, odd K, any leading dimension
DENSE_SHAPES = [
    (64, 96, 0.5, 37, None),
    (300, 200, 0.5, 100, None),
    (130, 257, 1.0, 64, None),       # odd K: the last MFMA step is half empty
    (33, 65, 0.7, 100, 101),         # odd leading dimension
    (10, 512, 0.6, 16, None),        # narrowest batch that takes the dense route
    (1024, 3072, 0.5, 100, None),    # first layer of the paper's MLP at 50 % sparsity
    (40, 30, 0.0, 32, None),         # empty pattern: the copies are all zero
    (96, 128, 0.5, 300, None),
]


@pytest.mark.parametrize("rows,cols,density,batch,ld", DENSE_SHAPES)
@pytest.mark.parametrize("relu", [False, True])
def test_dense_forward_and_backward_parity(nb, torch_mod, oracle, rows, cols, density, batch, ld, relu):
    torch = torch_mod
    lay = layer_case(rows, cols, density, seed=rows + 2 * cols, relu=relu)
    rng = np.random.default_rng(batch + 3)
    X = rng.standard_normal((cols, batch)).astype(np.float32)
    dY = rng.standard_normal((rows, batch)).astype(np.float32)
    L = nb.SparseLinear(lay, max_batch=batch)
    nb.sparse_linear_enable_dense(L.handle)
    nb.sparse_linear_enable_dense(L.handle)                 # idempotent
    Xd = nb.to_dense(X, ld=ld); Yd = nb.dense(rows, batch, ld=ld); dYd = nb.to_dense(dY, ld=ld)
    dXd = nb.dense(cols, batch, ld=ld)
    g = torch.full((max(lay.nnz, 1),), float("nan"), device="cuda")[:lay.nnz]
    db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, X, relu)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    full = Yd._base if Yd._base is not None else Yd
    assert torch.isnan(full.view(rows, -1)[:, batch:]).all()     # padding columns were not written
    dZ = oracle.relu_backward(dY, Yd.cpu().numpy()) if relu else dY
    dX, SdX = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, lay.values, dZ)
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dZ, X)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    close(g.cpu().numpy(), gr, Sg, what="dvalues"); close(db.cpu().numpy(), dbr, Sdb, what="dbias")
    # the caller changes values[]: a stand-alone product sees the change
    L.values.mul_(-0.5)
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    torch.cuda.synchronize()
    Y2, S2 = oracle.spmm(rows, cols, lay.indptr, lay.indices, (-0.5 * lay.values).astype(np.float32), lay.bias, X, relu)
    close(Yd.cpu().numpy(), Y2, S2, what="Y after the caller changed values")
    L.close()


@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("nesterov", [False, True])
def test_dense_route_in_training_steps(nb, torch_mod, oracle, unfused, nesterov):
    """Every layer of density >= 1/2 on the dense route: stage parity over several steps, so the dense
    copies must follow every update of values[]."""
    torch = torch_mod
    sizes, batch, lr, mu = (100, 300, 50, 10), 100, 0.05, 0.9
    mlp = wl.make_mlp(sizes, sparsity=0.5, bias_std=0.1, pattern_seed=41, value_seed=42)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 4, seed=43)
    flags = (nb.NERVA_MLP_UNFUSED if unfused else 0) | (nb.NERVA_MLP_NESTEROV if nesterov else 0)
    M = nb.MLP(mlp, batch, flags, dense_from_density=0.5)
    for t in range(4):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, lr, mu)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, unfused, nesterov=nesterov)
    # launch names say which route ran
    nb.mlp_profile_enable(M.handle, 1)
    M.train_step(nb.to_dense(Xs[0]), torch.as_tensor(Ts[0]).cuda(), batch, lr, mu)
    torch.cuda.synchronize()
    names = [n for n, _ in nb.mlp_profile_read(M.handle)[1]]
    assert "dense_forward[0]" in names and "dense_forward[1]" in names and "dense_transposed[1]" in names
    M.close()


def test_mixed_routes_and_large_output_layer(nb, torch_mod, oracle):
    """Only the output layer dense, and too large for the fused head, so that its forward and transposed
    products are launches of their own, both on the dense route; the first layer stays sparse."""
    torch = torch_mod
    sizes, batch, lr, mu = (64, 96, 40), 48, 0.05, 0.9
    mlp = wl.make_mlp(sizes, layer_nnz=(600, 3000), bias_std=0.1, pattern_seed=51, value_seed=52)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 3, seed=53)
    M = nb.MLP(mlp, batch, nb.NERVA_MLP_SEPARATE_HEAD)
    nb.sparse_linear_enable_dense(M.layers[1].handle)
    for t in range(3):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, lr, mu)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False)
    M.close()


def test_sync_values_and_rebind_keep_the_dense_copies_right(nb, torch_mod, oracle):
    torch = torch_mod
    sizes, batch = (48, 64, 10), 32
    mlp = wl.make_mlp(sizes, sparsity=0.4, bias_std=0.1, pattern_seed=61, value_seed=62)
    X = np.random.default_rng(63).standard_normal((sizes[0], batch)).astype(np.float32)
    M = nb.MLP(mlp, batch, dense_from_density=0.5)

    def check():
        out = M.forward(nb.to_dense(X), batch).cpu().numpy()
        torch.cuda.synchronize()
        inp = X
        for l, lay in enumerate(mlp.layers):
            inp_next, S = oracle.spmm(lay.rows, lay.cols, lay.indptr, lay.indices, M.layers[l].values.cpu().numpy(),
                                      M.layers[l].bias.cpu().numpy(), inp, lay.relu)
            if l + 1 < len(mlp.layers):
                # feed the GPU's own hidden activation forward so that rounding does not compound
                got = M.view("A", l, batch).cpu().numpy()
                close(got, inp_next, S, what=f"A[{l}]")
                inp = got
            else:
                close(out, inp_next, S, what="logits")

    check()
    # the caller rewrites the weights in place: without the sync the dense copies would be stale
    for l in M.layers:
        l.values.mul_(1.5)
        nb.sparse_linear_sync_values(l.handle)
    check()
    # a new pattern for layer 0: the fresh copies hold the new entries and nothing of the old ones
    lay = mlp.layers[0]
    new = layer_case(lay.rows, lay.cols, 0.55, seed=64, relu=True)
    M.rebind_layer(0, new.indptr, new.indices, new.values)
    mlp.layers[0] = wl.SparseLayerData(lay.rows, lay.cols, new.indptr, new.indices, new.values,
                                        M.layers[0].bias.cpu().numpy(), True)
    check()
    M.close()


def test_the_library_chooses_the_route_by_density(nb, torch_mod, oracle):
    """Bound with the library's default, a layer of at least 40 % density (and at least 64 x 64) takes the dense route by
    itself, a sparser one does not; on the dense route the SDDMM + update of a training step runs through the dense
    gradient.  Stage parity on both networks; the pattern arrays stay bit-identical on either route."""
    torch = torch_mod
    sizes, batch, lr, mu = (300, 200, 100, 10), 100, 0.05, 0.9
    for sparsity, want_dense in [(0.5, True), (0.9, False)]:
        mlp = wl.make_mlp(sizes, sparsity=sparsity, bias_std=0.1, pattern_seed=71, value_seed=72)
        Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 3, seed=73)
        M = nb.MLP(mlp, batch)
        nb.mlp_profile_enable(M.handle, 1)
        for t in range(3):
            before = snapshot(M)
            M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, lr, mu)
            torch.cuda.synchronize()
            if t == 0:
                names = [n for n, _ in nb.mlp_profile_read(M.handle)[1]]
                nb.mlp_profile_enable(M.handle, 0)
                assert ("dense_forward[0]" in names) == want_dense and ("dense_sddmm_update[0]" in names) == want_dense, names
                assert ("dense_transposed[1]" in names) == want_dense and ("dense_sddmm_update[1]" in names) == want_dense, names
            stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False)
        for l, lay in zip(M.layers, mlp.layers):
            assert np.array_equal(l.indptr.cpu().numpy(), lay.indptr) and np.array_equal(l.indices.cpu().numpy(), lay.indices)
        M.close()


@pytest.mark.parametrize("sizes,batch", [((130, 257, 70, 10), 37), ((64, 96, 200, 10), 300), ((100, 300, 64, 10), 16)])
def test_dense_route_training_on_ragged_shapes(nb, torch_mod, oracle, sizes, batch):
    """Ragged tiles in every dimension of the three dense products (rows, columns, batch not multiples of 16 / 64),
    a batch beyond one column tile, and the narrowest batch that takes the route; Nesterov momentum."""
    torch = torch_mod
    mlp = wl.make_mlp(sizes, sparsity=0.4, bias_std=0.1, pattern_seed=81, value_seed=82)
    Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 2, seed=83)
    M = nb.MLP(mlp, batch, nb.NERVA_MLP_NESTEROV)
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, 0.05, 0.9)
        torch.cuda.synchronize()
        stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, 0.05, 0.9, False, nesterov=True)
    M.close()
