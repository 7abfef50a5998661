"""Parity at the full sizes of the benchmark configurations, in the launch shapes bench.py uses.

Where the oracle cannot finish the whole result in seconds, a seeded sample of output rows (or of
stored entries) is computed one by one by the oracle on the corresponding sub-pattern and compared
at the same 1e-5 * S bar; properties that hold at any size (bit-identical pattern, reproducibility)
are checked on everything.
"""
import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl
from test_gpu_parity import close, TOL
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


def sub_rows(lay, rows_sel):
    """CSR of the selected rows only (same column space)."""
    counts = np.diff(lay.indptr)[rows_sel]
    indptr = np.zeros(len(rows_sel) + 1, dtype=np.int32)
    np.cumsum(counts, out=indptr[1:])
    pos = np.concatenate([np.arange(lay.indptr[r], lay.indptr[r + 1]) for r in rows_sel]) if len(rows_sel) else np.zeros(0, int)
    return indptr, lay.indices[pos], pos


def sub_cols_transposed(lay, cols_sel):
    """CSR of W^T restricted to the selected columns of W: row k lists the rows of W that store (.., cols_sel[k])."""
    row_of = np.repeat(np.arange(lay.rows, dtype=np.int32), np.diff(lay.indptr))
    indptr = [0]; idx = []; pos = []
    for j in cols_sel:
        hit = np.nonzero(lay.indices == j)[0]          # ascending position = ascending row
        idx.append(row_of[hit]); pos.append(hit); indptr.append(indptr[-1] + len(hit))
    return (np.asarray(indptr, dtype=np.int32), np.concatenate(idx).astype(np.int32) if idx else np.zeros(0, np.int32),
            np.concatenate(pos) if pos else np.zeros(0, int))


def test_config2_step_stage_parity(nb, torch_mod, oracle):
    """The bench configuration: 3072-1024-512-10 at 90 % sparsity, batch 100, fused step, pooled batches."""
    torch = torch_mod
    batch, lr, mu = 100, 0.01, 0.9
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=0.9)
    Xs, Ts = wl.make_batches(3072, 10, batch, 3, seed=3000)
    ld = nb.padded_ld(batch)
    Xd = torch.full((3, 3072, ld), float("nan"), device="cuda")
    Xd[:, :, :batch] = torch.as_tensor(Xs).cuda()
    Td = torch.as_tensor(Ts).cuda()
    M = nb.MLP(mlp, batch)
    worst = 0.0
    for t in range(3):
        before = snapshot(M)
        nb.mlp_train_step(M.handle, Xd[t].data_ptr(), ld, Td[t].data_ptr(), batch, lr, mu, M.workspace, M.loss)
        torch.cuda.synchronize()
        worst = max(worst, stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False))
    for l, lay in zip(M.layers, mlp.layers):
        assert np.array_equal(l.indptr.cpu().numpy(), lay.indptr) and np.array_equal(l.indices.cpu().numpy(), lay.indices)
    print(f"config 2: worst stage error = {worst:.3f} x (1e-5 S)")
    M.close()


def test_config4_step_sampled(nb, torch_mod, oracle):
    """3072-8192-8192-10, global density 1 % split by Erdos-Renyi (dense last layer), batch 1024: one fused
    step; every stage checked on sampled rows / entries against the oracle fed the GPU's stage inputs."""
    torch = torch_mod
    batch, lr, mu = 1024, 0.01, 0.9
    mlp = wl.make_mlp(wl.WIDE_MLP, er_density=0.01)
    assert [l.nnz for l in mlp.layers] == [342893, 498753, 81920]
    Xs, Ts = wl.make_batches(3072, 10, batch, 1, seed=3000)
    X = Xs[0]
    M = nb.MLP(mlp, batch)
    before = snapshot(M)
    M.train_step(nb.to_dense(X), torch.as_tensor(Ts[0]).cuda(), batch, lr, mu)
    torch.cuda.synchronize()
    L = 3
    A = [M.view("A", l, batch).cpu().numpy() for l in range(L)]
    dZ = [M.view("dZ", l, batch).cpu().numpy() for l in range(L)]
    rng = np.random.default_rng(4)
    for l, lay in enumerate(mlp.layers):
        inp = X if l == 0 else A[l - 1]
        sel = np.sort(rng.choice(lay.rows, size=min(lay.rows, 96), replace=False))
        ip, ix, pos = sub_rows(lay, sel)
        # forward rows
        Y, S = oracle.spmm(len(sel), lay.cols, ip, ix, before[l]["values"][pos], before[l]["bias"][sel], inp, lay.relu)
        close(A[l][sel], Y, S, what=f"A[{l}] sampled rows")
        # gradient of the sampled rows' entries and the momentum step on them
        g, Sg, db, Sdb = oracle.sddmm(len(sel), lay.cols, ip, ix, dZ[l][sel], inp)
        w, v, Sw, Sv = oracle.momentum(before[l]["values"][pos], before[l]["vel_w"][pos], g, lr, mu, Sg)
        close(M.layers[l].velocity.cpu().numpy()[pos], v, Sv, what=f"velocity[{l}] sampled")
        close(M.layers[l].values.cpu().numpy()[pos], w, Sw, what=f"values[{l}] sampled")
        b, bv, Sb, Sbv = oracle.momentum(before[l]["bias"][sel], before[l]["vel_b"][sel], db, lr, mu, Sdb)
        close(M.layers[l].bias.cpu().numpy()[sel], b, Sb, what=f"bias[{l}] sampled")
        # transposed product: sampled rows of dZ_{l-1}
        if l > 0:
            csel = np.sort(rng.choice(lay.cols, size=64, replace=False))
            tp, tx, tpos = sub_cols_transposed(lay, csel)
            dA, SdA = oracle.spmm(len(csel), lay.rows, tp, tx, before[l]["values"][tpos], None, dZ[l], False)
            ref = np.where(A[l - 1][csel] > 0, dA, 0).astype(np.float32)
            close(dZ[l - 1][csel], ref, SdA, what=f"dZ[{l - 1}] sampled rows")
    loss, S_loss, dZL, SdZL = oracle.softmax_ce(A[L - 1], Ts[0])
    close(dZ[L - 1], dZL, SdZL, what="dZ[last]")
    assert abs(float(M.loss.item()) - loss) <= TOL * S_loss
    # entries that were not sampled changed too, and nothing is NaN
    for l in range(L):
        w = M.layers[l].values.cpu().numpy()
        assert np.all(np.isfinite(w)) and np.count_nonzero(w != before[l]["values"]) > 0.5 * len(w)
    M.close()


@pytest.mark.parametrize("density,batch", [(0.001, 1024), (0.01, 128), (0.1, 128), (0.1, 1024)])
def test_config5_kernels_sampled(nb, torch_mod, oracle, density, batch):
    """16384 x 16384 with power-law row lengths (rank^-1.2): forward, transposed and sampled products
    alone, checked on sampled rows / columns / entries, the heaviest rows included."""
    z = wl.make_zipf_matrix(16384, density, seed=11)
    rn = np.diff(z.indptr)
    assert rn.max() == 16384 and rn.sum() == z.nnz               # full rows exist: the huge-row path is exercised
    _config5_case(nb, torch_mod, oracle, z, batch)


def test_config5_uniform_rows_sampled(nb, torch_mod, oracle):
    """The same size with uniform rows at 1 % and batch 1024: a 64 MiB operand and short segments, the case in which
    the products and the SDDMM are staged through LDS because of the operand's size."""
    n = 16384
    nnz = wl.round_half_up(0.01 * n * n)
    indptr, indices = wl.uniform_pattern(n, n, nnz, seed=11)
    prng = np.random.default_rng(12)
    z = wl.SparseLayerData(n, n, indptr, indices, prng.standard_normal(nnz, dtype=np.float32),
                           (prng.standard_normal(n) * 0.5).astype(np.float32), False)
    assert nb.nerva_plan_staged_host(n, n, indptr, indices, 1024)[0].shape[0] >= 32
    _config5_case(nb, torch_mod, oracle, z, 1024)


def _config5_case(nb, torch, oracle, z, batch):
    n = z.rows
    rn = np.diff(z.indptr)
    rng = np.random.default_rng(batch)
    X = rng.standard_normal((n, batch), dtype=np.float32)
    dY = rng.standard_normal((n, batch), dtype=np.float32)
    Lh = nb.SparseLinear(z, max_batch=batch)
    Xd = nb.to_dense(X); Yd = nb.dense(n, batch); dYd = nb.to_dense(dY); dXd = nb.dense(n, batch)
    g = torch.full((z.nnz,), float("nan"), device="cuda"); db = torch.full((n,), float("nan"), device="cuda")
    nb.sparse_linear_forward(Lh.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(Lh.handle, Xd, None, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy(); dX = dXd.cpu().numpy(); gh = g.cpu().numpy(); dbh = db.cpu().numpy()
    assert np.all(np.isfinite(Y)) and np.all(np.isfinite(dX)) and np.all(np.isfinite(gh)) and np.all(np.isfinite(dbh))
    # rows: the 4 longest, the empty ones among a random draw, and random ones (bounded oracle work)
    order = np.argsort(-rn)
    sel = np.unique(np.concatenate([order[:4], rng.choice(n, size=40, replace=False)]))
    ip, ix, pos = sub_rows(z, sel)
    Yr, S = oracle.spmm(len(sel), n, ip, ix, z.values[pos], z.bias[sel], X, False)
    close(Y[sel], Yr, S, what="Y sampled rows")
    gr, Sg, dbr, Sdb = oracle.sddmm(len(sel), n, ip, ix, dY[sel], X)
    close(gh[pos], gr, Sg, what="dvalues sampled rows")
    close(dbh[sel], dbr, Sdb, what="dbias sampled rows")
    empty = np.nonzero(rn == 0)[0]
    if len(empty):
        assert np.array_equal(Y[empty], np.broadcast_to(z.bias[empty, None], Y[empty].shape))   # empty rows give exactly the bias
    csel = np.sort(rng.choice(n, size=24, replace=False))
    tp, tx, tpos = sub_cols_transposed(z, csel)
    dXr, SdX = oracle.spmm(len(csel), n, tp, tx, z.values[tpos], None, dY, False)
    close(dX[csel], dXr, SdX, what="dX sampled rows")
    # run again: bit-identical (no atomics, fixed summation order)
    Y2 = nb.dense(n, batch); g2 = torch.empty_like(g); db2 = torch.empty_like(db); dX2 = nb.dense(n, batch)
    nb.sparse_linear_forward(Lh.handle, Xd, Y2, batch)
    nb.sparse_linear_backward(Lh.handle, Xd, None, dYd, dX2, g2, db2, batch)
    torch.cuda.synchronize()
    assert torch.equal(Y2, Yd) and torch.equal(g2, g) and torch.equal(db2, db) and torch.equal(dX2, dXd)
    Lh.close()


def test_operand_beyond_4gib(nb, torch_mod, oracle):
    """A gathered operand that spans more than 4 GiB (2^20 + 5 rows with a leading dimension of 1024 floats):
    the kernels that address the operand with 32-bit byte offsets must step aside for the ones with 64-bit row
    bases.  The oracle works on the referenced operand rows only (same sums, compacted column indices)."""
    torch = torch_mod
    rows, cols, batch, ld, per_row = 64, (1 << 20) + 5, 100, 1024, 12
    rng = np.random.default_rng(2024)
    indptr = np.arange(0, rows * per_row + 1, per_row, dtype=np.int32)
    indices = np.empty(rows * per_row, dtype=np.int32)
    for i in range(rows):
        c = rng.choice(cols - 1, size=per_row - 1, replace=False)
        indices[i * per_row:(i + 1) * per_row] = np.sort(np.concatenate([c, [cols - 1]]))   # every row reaches the far end
    values = rng.standard_normal(rows * per_row).astype(np.float32)
    bias = rng.standard_normal(rows).astype(np.float32)
    lay = wl.SparseLayerData(rows, cols, indptr, indices, values, bias, False)
    L = nb.SparseLinear(lay, max_batch=batch)
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    Xd = torch.randn((cols, ld), generator=g, device="cuda", dtype=torch.float32)
    assert Xd.numel() * 4 > (1 << 32)
    dY = rng.standard_normal((rows, batch)).astype(np.float32)
    Yd = nb.dense(rows, batch); dYd = nb.to_dense(dY)
    gv = torch.full((lay.nnz,), float("nan"), device="cuda"); db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)                      # the tensor's row stride (1024) is ldx
    nb.sparse_linear_backward(L.handle, Xd, None, dYd, None, gv, db, batch)
    torch.cuda.synchronize()
    used, compact = np.unique(indices, return_inverse=True)
    Xs = Xd[torch.as_tensor(used, dtype=torch.int64, device="cuda"), :batch].cpu().numpy()
    Y, S = oracle.spmm(rows, len(used), indptr, compact.astype(np.int32), values, bias, Xs, False)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, len(used), indptr, compact.astype(np.int32), dY, Xs)
    close(gv.cpu().numpy(), gr, Sg, what="dvalues"); close(db.cpu().numpy(), dbr, Sdb, what="dbias")
    L.close()
