"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: index structure bit-exact; fp32 values within 1e-5 of the oracle, normalised by the sum
of the absolute values of the terms of each result (S, returned by the oracle).  Elements
whose S is zero (empty rows) must match exactly.
"""
import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-5


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


def close(got, ref, S, tol=TOL, what=""):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    bound = tol * np.asarray(S, dtype=np.float64)
    bad = err > bound
    if bad.any():
        k = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {err.size} elements off; worst at {k}: "
                             f"gpu={got[k]!r} oracle={ref[k]!r} err={err[k]:.3e} allowed={bound[k]:.3e}")
    return float((err / np.maximum(bound / tol, 1e-300)).max()) if err.size else 0.0


def raw_i32(nb, torch, addr, n):
    """Copy n int32 from a raw device address (bit copy through the library's copy kernel)."""
    out = torch.empty(max(n, 1), dtype=torch.float32, device="cuda")
    if n:
        nb._check(nb.lib.nerva_copy_f32(out.data_ptr(), addr, n, None))
    torch.cuda.synchronize()
    return out[:n].view(torch.int32).cpu().numpy()


def raw_f32(nb, torch, addr, n):
    out = torch.empty(max(n, 1), dtype=torch.float32, device="cuda")
    if n:
        nb._check(nb.lib.nerva_copy_f32(out.data_ptr(), addr, n, None))
    torch.cuda.synchronize()
    return out[:n].cpu().numpy()


def layer_case(rows, cols, density, seed, relu=False, bias=True):
    nnz = wl.round_half_up(density * rows * cols)
    indptr, indices = wl.uniform_pattern(rows, cols, nnz, seed)
    rng = np.random.default_rng(seed + 1)
    values = wl.init_values(indptr, seed + 2)
    b = (rng.standard_normal(rows) * 0.5).astype(np.float32) if bias else np.zeros(rows, dtype=np.float32)
    return wl.SparseLayerData(rows, cols, indptr, indices, values, b, relu)


# (rows, cols, density, batch, ld or None): several tiles, ragged tails, empty rows, every kernel variant
SHAPES = [
    (7, 5, 0.3, 3, None),            # tiny, batch not a multiple of 4
    (33, 65, 0.2, 100, None),        # the paper's batch size
    (130, 257, 0.05, 64, None),
    (64, 96, 1.0, 37, None),         # fully dense pattern
    (50, 40, 0.0, 8, None),          # empty matrix
    (300, 200, 0.5, 100, 101),       # odd leading dimension -> scalar kernels
    (200, 300, 0.1, 256, None),
    (96, 128, 0.3, 300, None),       # two tiles per lane
    (128, 512, 0.2, 1024, None),     # four tiles per lane
    (40, 64, 0.3, 1100, None),       # beyond one column tile
    (1024, 3072, 0.01, 100, None),   # first layer of the paper's MLP at 99 % sparsity
    (10, 512, 0.1, 100, None),       # its last layer
    (10, 2048, 1.0, 1024, None),     # dense rows cut over several work-groups (huge rows), wide batch
    (12, 4096, 0.9, 100, None),      # huge rows at the paper's batch size
    (6, 3000, 1.0, 37, 41),          # huge rows through the scalar kernels
    (300, 200, 0.3, 1, 1),           # one example, stored as a plain vector: lanes across the row's entries
    (1024, 3072, 0.1, 1, None),      # batch-1 inference on the first layer of the paper's MLP
    (64, 4096, 0.9, 2, None),        # few columns and huge rows
    (33, 65, 0.2, 4, 5),
    (33, 65, 0.2, 3, None),
    # more than 2048 rows of at most 128 entries: the packed path (one row per lane group)
    (2500, 300, 0.02, 100, None),    # 6 entries per row, some rows empty
    (3000, 200, 0.1, 37, None),      # 4 rows per gather instruction, ragged batch
    (2100, 5000, 0.01, 128, None),   # the mirror (5000 short rows) is packed too
    (2400, 1000, 0.125, 64, None),   # rows around the 128-entry limit: packed and ordinary rows in one grid
    (2200, 3000, 0.005, 300, None),  # operand beyond an L2: packed rows inside column tiles
    (300, 2500, 0.02, 100, None),    # short rows only in the mirror
    # every entry stored and few rows: the operand is streamed once for all rows
    (16, 700, 1.0, 300, None),       # 16 rows, ragged slices and columns
    (3, 1000, 1.0, 64, None),
    (10, 8192, 1.0, 256, None),      # the wide MLP's saturated output layer, a quarter of its batch
    # wide batch, several entries per operand row and row range: operand blocks staged in LDS
    (2048, 1100, 0.3, 512, None),    # segments of ~150 entries, ragged last column block; the mirror is not staged
    (4096, 4200, 0.08, 256, None),   # both directions staged, 64 row ranges
    (3072, 12300, 0.012, 1024, None),  # a 50 MB operand: staged although its segments are short (~6 entries)
    (4096, 700, 0.1, 216, None),     # last tile ragged (24 of 64 columns)
    (4096, 600, 0.1, 704, None),     # 11 tiles: eight XCD-aligned, three dealt plainly
    # operands beyond an L2: column tiles in the products and per-tile partial sums in the SDDMM
    (300, 6000, 0.02, 200, None),    # 64-column tiles, ragged last tile
    (320, 12000, 0.02, 360, None),   # 32-column tiles (240 entries per row, a 17 MB operand)
]


@pytest.mark.parametrize("rows,cols,density,batch,ld", SHAPES)
@pytest.mark.parametrize("relu", [False, True])
def test_forward_parity(nb, torch_mod, oracle, rows, cols, density, batch, ld, relu):
    torch = torch_mod
    lay = layer_case(rows, cols, density, seed=rows + cols, relu=relu)
    X = np.random.default_rng(batch).standard_normal((cols, batch)).astype(np.float32)
    L = nb.SparseLinear(lay, max_batch=batch)
    Xd = nb.to_dense(X, ld=ld); Yd = nb.dense(rows, batch, ld=ld)
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, X, relu)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    # padding columns of the output were not written
    full = Yd._base if Yd._base is not None else Yd
    assert torch.isnan(full.view(rows, -1)[:, batch:]).all()
    L.close()


@pytest.mark.parametrize("rows,cols,density,batch,ld", SHAPES)
@pytest.mark.parametrize("relu", [False, True])
def test_backward_parity(nb, torch_mod, oracle, rows, cols, density, batch, ld, relu):
    torch = torch_mod
    lay = layer_case(rows, cols, density, seed=rows * 3 + cols, relu=relu)
    rng = np.random.default_rng(batch + 1)
    X = rng.standard_normal((cols, batch)).astype(np.float32)
    dY = rng.standard_normal((rows, batch)).astype(np.float32)
    L = nb.SparseLinear(lay, max_batch=batch)
    Xd = nb.to_dense(X, ld=ld); Yd = nb.dense(rows, batch, ld=ld); dYd = nb.to_dense(dY, ld=ld)
    dXd = nb.dense(cols, batch, ld=ld)
    g = torch.full((max(lay.nnz, 1),), float("nan"), device="cuda")[:lay.nnz]
    db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    dZ = oracle.relu_backward(dY, Y) if relu else dY            # mask from the GPU's own output
    dX, SdX = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, lay.values, dZ)
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dZ, X)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    close(g.cpu().numpy(), gr, Sg, what="dvalues")
    close(db.cpu().numpy(), dbr, Sdb, what="dbias")
    # pieces can be asked for separately
    db2 = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_backward(L.handle, None, Yd, dYd, None, None, db2, batch)
    torch.cuda.synchronize()
    close(db2.cpu().numpy(), dbr, Sdb, what="dbias alone")     # (with the products it may be summed per column tile)
    L.close()


def test_backward_sees_changed_values(nb, torch_mod, oracle):
    """values[] changed behind the library's back: dX must use the new values."""
    torch = torch_mod
    lay = layer_case(64, 48, 0.3, seed=9)
    rng = np.random.default_rng(2)
    dY = rng.standard_normal((64, 20)).astype(np.float32)
    L = nb.SparseLinear(lay)
    dYd = nb.to_dense(dY); dXd = nb.dense(48, 20)
    new_vals = rng.standard_normal(lay.nnz).astype(np.float32)
    L.values.copy_(torch.as_tensor(new_vals))
    nb.sparse_linear_backward(L.handle, None, None, dYd, dXd, None, None, 20)
    torch.cuda.synchronize()
    dX, S = oracle.spmm_t(64, 48, lay.indptr, lay.indices, new_vals, dY)
    close(dXd.cpu().numpy(), dX, S, what="dX after external update")
    L.close()


@pytest.mark.parametrize("rows,cols,density", [(7, 5, 0.3), (130, 257, 0.05), (64, 96, 1.0), (50, 40, 0.0),
                                               (1024, 3072, 0.01)])
def test_mirror_is_the_transposed_pattern_bit_exact(nb, torch_mod, rows, cols, density):
    torch = torch_mod
    lay = layer_case(rows, cols, density, seed=5)
    L = nb.SparseLinear(lay)
    ip_t, ix_t, v_t, perm = nb.sparse_linear_mirror(L.handle)
    indptr_t = raw_i32(nb, torch, ip_t, cols + 1)
    indices_t = raw_i32(nb, torch, ix_t, lay.nnz)
    perm_h = raw_i32(nb, torch, perm, lay.nnz)
    values_t = raw_f32(nb, torch, v_t, lay.nnz)
    # expected: stable sort of the stored entries by column (rows ascending inside a column)
    row_of = np.repeat(np.arange(rows, dtype=np.int32), np.diff(lay.indptr))
    order = np.argsort(lay.indices, kind="stable")
    exp_indptr = np.zeros(cols + 1, dtype=np.int32)
    np.cumsum(np.bincount(lay.indices, minlength=cols), out=exp_indptr[1:])
    assert np.array_equal(indptr_t, exp_indptr)
    assert np.array_equal(indices_t, row_of[order])
    assert np.array_equal(perm_h, order.astype(np.int32))
    assert np.array_equal(values_t, lay.values[order])
    # the caller's pattern arrays are untouched
    assert np.array_equal(L.indptr.cpu().numpy(), lay.indptr) and np.array_equal(L.indices.cpu().numpy(), lay.indices)
    L.close()


def _mirror_check(nb, torch, rows, cols, indptr, indices):
    nnz = int(indptr[-1])
    lay = wl.SparseLayerData(rows, cols, np.asarray(indptr, np.int32), np.asarray(indices, np.int32),
                             np.arange(1, nnz + 1, dtype=np.float32), np.zeros(rows, np.float32), False)
    L = nb.SparseLinear(lay, max_batch=64)
    ip_t, ix_t, v_t, perm = nb.sparse_linear_mirror(L.handle)
    row_of = np.repeat(np.arange(rows, dtype=np.int32), np.diff(lay.indptr))
    order = np.argsort(lay.indices, kind="stable")
    exp_indptr = np.zeros(cols + 1, dtype=np.int32)
    np.cumsum(np.bincount(lay.indices, minlength=cols), out=exp_indptr[1:])
    assert np.array_equal(raw_i32(nb, torch, ip_t, cols + 1), exp_indptr)
    assert np.array_equal(raw_i32(nb, torch, ix_t, nnz), row_of[order])
    assert np.array_equal(raw_i32(nb, torch, perm, nnz), order.astype(np.int32))
    assert np.array_equal(raw_f32(nb, torch, v_t, nnz), lay.values[order])
    L.close()


def test_mirror_build_on_awkward_patterns(nb, torch_mod):
    """The mirror is built on the device by a counting sort over row tiles: patterns that stress it -- every row
    in one column (all tiles meet in one counter column), one row holding every column, rows far longer than a tile's
    share next to thousands of rows with one entry, trailing and leading empty rows, a power-law matrix of 300 k
    entries cut into hundreds of tiles -- each compared bit for bit with a stable sort by column."""
    torch = torch_mod
    rows, cols = 5000, 37
    _mirror_check(nb, torch, rows, cols, np.arange(rows + 1), np.full(rows, 11))                       # one column
    _mirror_check(nb, torch, 3, 9000, [0, 0, 9000, 9000], np.arange(9000))                            # one full row, two empty
    lens = np.ones(6000, dtype=np.int64); lens[[5, 3000, 5999]] = 4000; lens[:3] = 0; lens[-2:] = [0, 4000][::-1]
    ip, ix = wl.pattern_from_row_nnz(lens, 4000, seed=3)
    _mirror_check(nb, torch, 6000, 4000, ip, ix)
    z = wl.make_zipf_matrix(4096, 0.02, seed=7)
    _mirror_check(nb, torch, 4096, 4096, z.indptr, z.indices)
    _mirror_check(nb, torch, 40, 30, np.zeros(41, np.int32), np.zeros(0, np.int32))                    # empty


def test_invalid_patterns_are_rejected_by_the_device_side_check(nb, torch_mod):
    """Every way a pattern can fail to be canonical CSR, found by the kernels that check it where it lives; nothing
    outside the arrays is read (the row pointers are checked before they are used as positions)."""
    torch = torch_mod
    lay = layer_case(40, 30, 0.3, seed=6)
    rows, cols, nnz = 40, 30, lay.nnz

    def rejected(indptr, indices, word):
        bad = wl.SparseLayerData(rows, cols, np.asarray(indptr, np.int32), np.asarray(indices, np.int32), lay.values, lay.bias, False)
        with pytest.raises(nb.NervaError) as e:
            nb.SparseLinear(bad)
        assert e.value.code == nb.NERVA_ERR_CSR and word in str(e.value), str(e.value)

    ip = lay.indptr.copy(); ip[0] = 1
    rejected(ip, lay.indices, "indptr[0]")
    ip = lay.indptr.copy(); ip[7], ip[8] = ip[8] + 1, ip[7]
    rejected(ip, lay.indices, "decreases")
    ip = lay.indptr.copy(); ip[20] = 10 ** 9                         # far beyond nnz: must not be used as a position
    rejected(ip, lay.indices, "indptr")
    ip = lay.indptr.copy(); ip[20] = -5
    rejected(ip, lay.indices, "indptr")
    ix = lay.indices.copy(); ix[17] = cols
    rejected(lay.indptr, ix, "out of range")
    ix = lay.indices.copy(); ix[17] = -1
    rejected(lay.indptr, ix, "out of range")
    row = int(np.argmax(np.diff(lay.indptr) >= 2)); p = int(lay.indptr[row])
    ix = lay.indices.copy(); ix[p + 1] = ix[p]
    rejected(lay.indptr, ix, "ascending")
    ix = lay.indices.copy(); ix[p], ix[p + 1] = ix[p + 1], ix[p]
    rejected(lay.indptr, ix, "ascending")
    L = nb.SparseLinear(lay)                                         # the untouched pattern is accepted
    L.close()


def test_invalid_pattern_is_rejected_on_create(nb, torch_mod):
    torch = torch_mod
    lay = layer_case(16, 16, 0.3, seed=3)
    bad = lay.indices.copy(); bad[1] = bad[0]
    lay_bad = wl.SparseLayerData(16, 16, lay.indptr, bad, lay.values, lay.bias, False)
    with pytest.raises(nb.NervaError) as e:
        nb.SparseLinear(lay_bad)
    assert e.value.code == nb.NERVA_ERR_CSR


def test_shape_errors(nb, torch_mod):
    lay = layer_case(16, 12, 0.3, seed=4)
    L = nb.SparseLinear(lay)
    X = nb.dense(12, 8); Y = nb.dense(16, 8)
    with pytest.raises(nb.NervaError) as e:
        nb.sparse_linear_forward(L.handle, X, Y, 64)       # batch larger than the leading dimension
    assert e.value.code == nb.NERVA_ERR_SHAPE
    with pytest.raises(nb.NervaError) as e:
        nb.sparse_linear_forward(L.handle, X, Y, 0)
    assert e.value.code == nb.NERVA_ERR_ARGUMENT
    L.close()
    L = nb.SparseLinear(lay, max_batch=4)
    with pytest.raises(nb.NervaError) as e:
        nb.sparse_linear_forward(L.handle, X, Y, 8)         # beyond the batch the layer was created for
    assert e.value.code == nb.NERVA_ERR_SHAPE
    L.close()


@pytest.mark.parametrize("n", [0, 1, 3, 4, 1000, 1027, 314573])
@pytest.mark.parametrize("offset", [0, 1])
@pytest.mark.parametrize("nesterov", [False, True])
def test_sgd_update_parity(nb, torch_mod, oracle, n, offset, nesterov):
    torch = torch_mod
    rng = np.random.default_rng(n + offset)
    w, v, g = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    pad = lambda a: torch.as_tensor(np.concatenate([np.zeros(offset, np.float32), a])).cuda()[offset:]
    wd, vd, gd = pad(w), pad(v), pad(g)     # offset 1: not 16-byte aligned -> scalar kernel
    (nb.sgd_update_values_nesterov if nesterov else nb.sgd_update_values)(wd, vd, gd, n, 0.01, 0.9)
    torch.cuda.synchronize()
    wr, vr, Sw, Sv = oracle.momentum(w, v, g, 0.01, 0.9, nesterov=nesterov)
    close(vd.cpu().numpy(), vr, Sv, what="velocity")
    close(wd.cpu().numpy(), wr, Sw, what="values")
    assert np.array_equal(gd.cpu().numpy(), g)


@pytest.mark.parametrize("classes,batch", [(10, 100), (10, 1), (3, 7), (10, 1024), (100, 2500)])
def test_softmax_ce_parity(nb, torch_mod, oracle, classes, batch):
    torch = torch_mod
    rng = np.random.default_rng(classes + batch)
    Z = (rng.standard_normal((classes, batch)) * 3).astype(np.float32)
    labels = rng.integers(0, classes, size=batch).astype(np.int32)
    Zd = nb.to_dense(Z); dZd = nb.dense(classes, batch)
    loss = torch.zeros(1, device="cuda"); lab = torch.as_tensor(labels).cuda()
    nb.softmax_cross_entropy(Zd, lab, classes, batch, dZd, loss)
    torch.cuda.synchronize()
    lr, Sl, dZr, SdZ = oracle.softmax_ce(Z, labels)
    close(dZd.cpu().numpy(), dZr, SdZ, what="dZ")
    assert abs(float(loss.item()) - lr) <= TOL * Sl
    # uniform logits: ln(classes)
    Zd.zero_()
    nb.softmax_cross_entropy(Zd, lab, classes, batch, dZd, loss)
    assert abs(float(loss.item()) - np.log(classes)) < 1e-6 * np.log(max(classes, 2)) + 1e-7


def test_zipf_matrix_packed_rows(nb, torch_mod, oracle):
    """Power-law rows on a matrix large enough for the packed path: a few full rows (huge), a long
    tail of rows with one or no entry; forward, transposed and SDDMM at batches that take the
    grouped, the tiled and the wide kernels."""
    torch = torch_mod
    n = 4096
    z = wl.make_zipf_matrix(n, 0.004, seed=9)
    short, ns, waves, _ = nb.nerva_plan_short_rows_host(n, z.indptr)
    assert ns >= nb.NERVA_PACK_MIN_ROWS and len(waves) >= 1
    for batch in (100, 7, 512):
        rng = np.random.default_rng(batch)
        X = rng.standard_normal((n, batch)).astype(np.float32)
        dY = rng.standard_normal((n, batch)).astype(np.float32)
        L = nb.SparseLinear(z, max_batch=batch)
        Xd = nb.to_dense(X); Yd = nb.dense(n, batch); dYd = nb.to_dense(dY); dXd = nb.dense(n, batch)
        g = torch.empty(z.nnz, device="cuda"); db = torch.empty(n, device="cuda")
        nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
        nb.sparse_linear_backward(L.handle, Xd, None, dYd, dXd, g, db, batch)
        torch.cuda.synchronize()
        Y, S = oracle.spmm(n, n, z.indptr, z.indices, z.values, z.bias, X, False)
        close(Yd.cpu().numpy(), Y, S, what="Y")
        dX, SdX = oracle.spmm_t(n, n, z.indptr, z.indices, z.values, dY)
        close(dXd.cpu().numpy(), dX, SdX, what="dX")
        gr, Sg, dbr, Sdb = oracle.sddmm(n, n, z.indptr, z.indices, dY, X)
        close(g.cpu().numpy(), gr, Sg, what="g"); close(db.cpu().numpy(), dbr, Sdb, what="db")
        L.close()


def test_zipf_matrix_staged_products(nb, torch_mod, oracle):
    """Power-law rows on the staged products and the staged SDDMM: full rows (a segment of 512 entries in every column block) next
    to rows with a single entry and empty rows (bias only), in both directions, with and without ReLU mask."""
    torch = torch_mod
    n, batch = 4096, 1024
    lens = wl.zipf_row_nnz(n, n, n * n // 10, 1.2, seed=19)
    lens[np.arange(5, n, 37)] = 0                              # empty rows and rows with one entry, scattered
    lens[np.arange(11, n, 41)] = 1
    indptr, indices = wl.pattern_from_row_nnz(lens, n, seed=20)
    prng = np.random.default_rng(21)
    z = wl.SparseLayerData(n, n, indptr, indices, prng.standard_normal(int(indptr[-1])).astype(np.float32),
                           (prng.standard_normal(n) * 0.5).astype(np.float32), False)
    slot_rows, ends = nb.nerva_plan_staged_host(n, n, z.indptr, z.indices, batch)
    assert ends.shape[0] >= 16 and ends.shape[1] == 9 and (lens == n).any()
    rng = np.random.default_rng(batch)
    X = rng.standard_normal((n, batch)).astype(np.float32)
    dY = rng.standard_normal((n, batch)).astype(np.float32)
    for relu in (False, True):
        lay = wl.SparseLayerData(n, n, z.indptr, z.indices, z.values, z.bias, relu)
        L = nb.SparseLinear(lay, max_batch=batch)
        Xd = nb.to_dense(X); Yd = nb.dense(n, batch); dYd = nb.to_dense(dY); dXd = nb.dense(n, batch)
        g = torch.full((lay.nnz,), float("nan"), device="cuda"); db = torch.full((n,), float("nan"), device="cuda")
        nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
        nb.sparse_linear_backward(L.handle, Xd, Yd if relu else None, dYd, dXd, g, db, batch)
        torch.cuda.synchronize()
        Y, S = oracle.spmm(n, n, z.indptr, z.indices, z.values, z.bias, X, relu)
        close(Yd.cpu().numpy(), Y, S, what="Y")
        dZ = oracle.relu_backward(dY, Y) if relu else dY
        dX, SdX = oracle.spmm_t(n, n, z.indptr, z.indices, z.values, dZ)
        close(dXd.cpu().numpy(), dX, SdX, what="dX")
        gr, Sg, dbr, Sdb = oracle.sddmm(n, n, z.indptr, z.indices, dZ, X)
        close(g.cpu().numpy(), gr, Sg, what="g"); close(db.cpu().numpy(), dbr, Sdb, what="db")
        L.close()


@pytest.mark.parametrize("rows,cols,lens_kind,batch", [
    (7, 5, "uniform", 128),          # fewer rows than one group of four, one column block, one range
    (33, 65, "uniform", 132),        # third tile holds 4 of 64 columns
    (130, 1025, "uniform", 256),     # a column block of a single operand row
    (64, 96, "full", 128),           # every entry stored
    (50, 700, "empty_heavy", 128),   # most rows empty
    (1300, 40, "uniform", 192),      # several ranges, rows cut by the 512-row limit
    (600, 3000, "zipf", 320),        # full rows next to empty ones: segments of 512 entries and of none side by side
])
def test_staged_kernels_on_awkward_shapes(nb, torch_mod, oracle, rows, cols, lens_kind, batch):
    """The staged products and the staged SDDMM where the library would not choose them: the partition mode that
    prefers them runs them on any matrix at batches of 128 or more, which reaches their edge cases (few rows,
    ragged tiles and blocks, empty rows and segments, very long segments)."""
    torch = torch_mod
    rng = np.random.default_rng(rows * 7 + cols)
    if lens_kind == "uniform":
        lens = rng.binomial(cols, 0.2, size=rows)
    elif lens_kind == "full":
        lens = np.full(rows, cols)
    elif lens_kind == "empty_heavy":
        lens = np.where(rng.random(rows) < 0.8, 0, rng.integers(1, cols + 1, size=rows))
    else:
        lens = np.minimum(cols, (cols * rng.permutation(np.arange(1, rows + 1)) ** -1.2).astype(np.int64))
    indptr, indices = wl.pattern_from_row_nnz(lens.astype(np.int64), cols, seed=rows + cols)
    nnz = int(indptr[-1])
    lay = wl.SparseLayerData(rows, cols, indptr, indices, rng.standard_normal(nnz).astype(np.float32),
                             (rng.standard_normal(rows) * 0.5).astype(np.float32), True)
    X = rng.standard_normal((cols, batch)).astype(np.float32)
    dY = rng.standard_normal((rows, batch)).astype(np.float32)
    nb.nerva_set_partition_mode(nb.NERVA_PARTITION_PREFER_STAGED)
    try:
        assert nb.nerva_plan_staged_host(rows, cols, indptr, indices, batch)[0].shape[0] >= 1
        L = nb.SparseLinear(lay, max_batch=batch)
    finally:
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_BALANCED)
    Xd = nb.to_dense(X); Yd = nb.dense(rows, batch); dYd = nb.to_dense(dY); dXd = nb.dense(cols, batch)
    g = torch.full((max(nnz, 1),), float("nan"), device="cuda")[:nnz]; db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(rows, cols, indptr, indices, lay.values, lay.bias, X, True)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    dZ = oracle.relu_backward(dY, Yd.cpu().numpy())
    dX, SdX = oracle.spmm_t(rows, cols, indptr, indices, lay.values, dZ)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, indptr, indices, dZ, X)
    close(g.cpu().numpy(), gr, Sg, what="g"); close(db.cpu().numpy(), dbr, Sdb, what="db")
    full = Yd._base if Yd._base is not None else Yd
    assert torch.isnan(full.view(rows, -1)[:, batch:]).all()     # padding columns of the output were not written
    L.close()


def test_power_law_rows_staged_and_ordinary_kernels_together(nb, torch_mod, oracle):
    """The same split on an operand small enough to stay untiled (600 rows x 1024 columns): without column tiles the
    packed path does not run, so the short rows of the forward product go through the wide kernel on a partition of
    their own, next to the staged long rows; the SDDMM splits likewise; the mirror (600 long rows) is not staged."""
    torch = torch_mod
    rows, cols, batch = 8192, 600, 1024
    lens = wl.zipf_row_nnz(rows, cols, rows * cols * 12 // 100, 1.2, seed=31)
    lens[np.arange(3, rows, 61)] = 0
    indptr, indices = wl.pattern_from_row_nnz(lens, cols, seed=32)
    assert (lens <= nb.NERVA_PACK_MAX_LEN).sum() >= nb.NERVA_PACK_MIN_ROWS
    assert nb.nerva_plan_staged_host(rows, cols, indptr, indices, batch, nb.NERVA_PACK_MAX_LEN + 1)[0].shape[0] >= 8
    prng = np.random.default_rng(33)
    lay = wl.SparseLayerData(rows, cols, indptr, indices, prng.standard_normal(int(indptr[-1])).astype(np.float32),
                             (prng.standard_normal(rows) * 0.5).astype(np.float32), True)
    X = prng.standard_normal((cols, batch)).astype(np.float32)
    dY = prng.standard_normal((rows, batch)).astype(np.float32)
    L = nb.SparseLinear(lay, max_batch=batch)
    Xd = nb.to_dense(X); Yd = nb.dense(rows, batch); dYd = nb.to_dense(dY); dXd = nb.dense(cols, batch)
    g = torch.full((lay.nnz,), float("nan"), device="cuda"); db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(rows, cols, indptr, indices, lay.values, lay.bias, X, True)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    dZ = oracle.relu_backward(dY, Yd.cpu().numpy())
    dX, SdX = oracle.spmm_t(rows, cols, indptr, indices, lay.values, dZ)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, indptr, indices, dZ, X)
    close(g.cpu().numpy(), gr, Sg, what="g"); close(db.cpu().numpy(), dbr, Sdb, what="db")
    L.close()


def test_power_law_rows_staged_and_packed_together(nb, torch_mod, oracle):
    """Power-law rows with thousands of short rows next to a thousand long ones: the forward product stages the
    rows of more than 128 entries through LDS and serves the others with the packed kernel, two launches writing
    disjoint rows; with bias, ReLU, empty rows, and the operand mask of the stand-alone backward pass."""
    torch = torch_mod
    n, batch = 6144, 1024
    lens = wl.zipf_row_nnz(n, n, n * n * 3 // 100, 1.2, seed=19)
    lens[np.arange(7, n, 53)] = 0
    indptr, indices = wl.pattern_from_row_nnz(lens, n, seed=20)
    short, ns, _, _ = nb.nerva_plan_short_rows_host(n, indptr)
    assert ns >= nb.NERVA_PACK_MIN_ROWS and (lens > nb.NERVA_PACK_MAX_LEN).sum() >= 1000
    assert nb.nerva_plan_staged_host(n, n, indptr, indices, batch, nb.NERVA_PACK_MAX_LEN + 1)[0].shape[0] == 16
    prng = np.random.default_rng(21)
    lay = wl.SparseLayerData(n, n, indptr, indices, prng.standard_normal(int(indptr[-1])).astype(np.float32),
                             (prng.standard_normal(n) * 0.5).astype(np.float32), True)
    X = prng.standard_normal((n, batch)).astype(np.float32)
    dY = prng.standard_normal((n, batch)).astype(np.float32)
    L = nb.SparseLinear(lay, max_batch=batch)
    Xd = nb.to_dense(X); Yd = nb.dense(n, batch); dYd = nb.to_dense(dY); dXd = nb.dense(n, batch)
    g = torch.full((lay.nnz,), float("nan"), device="cuda"); db = torch.full((n,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(n, n, indptr, indices, lay.values, lay.bias, X, True)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    dZ = oracle.relu_backward(dY, Yd.cpu().numpy())
    dX, SdX = oracle.spmm_t(n, n, indptr, indices, lay.values, dZ)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    gr, Sg, dbr, Sdb = oracle.sddmm(n, n, indptr, indices, dZ, X)
    close(g.cpu().numpy(), gr, Sg, what="g"); close(db.cpu().numpy(), dbr, Sdb, what="db")
    L.close()


def test_staged_layer_at_smaller_batches(nb, torch_mod, oracle):
    """A layer bound for batch 1024 (row ranges chosen for 16 column tiles) run at smaller batches: 512 and 320 still
    take the staged kernels with fewer tiles, 128 and 100 fall back to the other kernels; same results to the bar."""
    torch = torch_mod
    rows, cols = 4096, 2100
    lay = layer_case(rows, cols, 0.06, seed=77, relu=True)
    assert nb.nerva_plan_staged_host(rows, cols, lay.indptr, lay.indices, 1024)[0].shape[0] >= 16
    L = nb.SparseLinear(lay, max_batch=1024)
    for batch in (1024, 512, 320, 128, 100):
        rng = np.random.default_rng(batch)
        X = rng.standard_normal((cols, batch)).astype(np.float32)
        dY = rng.standard_normal((rows, batch)).astype(np.float32)
        Xd = nb.to_dense(X); Yd = nb.dense(rows, batch); dYd = nb.to_dense(dY); dXd = nb.dense(cols, batch)
        g = torch.full((lay.nnz,), float("nan"), device="cuda"); db = torch.full((rows,), float("nan"), device="cuda")
        nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
        nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
        torch.cuda.synchronize()
        Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, X, True)
        close(Yd.cpu().numpy(), Y, S, what=f"Y at batch {batch}")
        dZ = oracle.relu_backward(dY, Yd.cpu().numpy())
        dX, SdX = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, lay.values, dZ)
        close(dXd.cpu().numpy(), dX, SdX, what=f"dX at batch {batch}")
        gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dZ, X)
        close(g.cpu().numpy(), gr, Sg, what=f"g at batch {batch}"); close(db.cpu().numpy(), dbr, Sdb, what=f"db at batch {batch}")
    L.close()


def test_zipf_matrix_all_row_classes(nb, torch_mod, oracle):
    """Power-law rows (one full row, many empty ones): every share count of the row partition."""
    torch = torch_mod
    z = wl.make_zipf_matrix(1024, 0.02, seed=5)
    _, blocks, huge, nh, _ = nb.nerva_plan_rows_host(1024, z.indptr)
    assert len(set((blocks[nh:, 0] & 0xFF).tolist())) >= 3 and len(huge) >= 1
    for batch in (128, 100):
        rng = np.random.default_rng(batch)
        X = rng.standard_normal((1024, batch)).astype(np.float32)
        dY = rng.standard_normal((1024, batch)).astype(np.float32)
        L = nb.SparseLinear(z)
        Xd = nb.to_dense(X); Yd = nb.dense(1024, batch); dYd = nb.to_dense(dY); dXd = nb.dense(1024, batch)
        g = torch.empty(z.nnz, device="cuda"); db = torch.empty(1024, device="cuda")
        nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
        nb.sparse_linear_backward(L.handle, Xd, None, dYd, dXd, g, db, batch)
        torch.cuda.synchronize()
        Y, S = oracle.spmm(1024, 1024, z.indptr, z.indices, z.values, z.bias, X, False)
        close(Yd.cpu().numpy(), Y, S, what="Y")
        dX, SdX = oracle.spmm_t(1024, 1024, z.indptr, z.indices, z.values, dY)
        close(dXd.cpu().numpy(), dX, SdX, what="dX")
        gr, Sg, dbr, Sdb = oracle.sddmm(1024, 1024, z.indptr, z.indices, dY, X)
        close(g.cpu().numpy(), gr, Sg, what="g"); close(db.cpu().numpy(), dbr, Sdb, what="db")
        L.close()


def _random_case(k):
    """Seeded draw of a layer shape, a row-length distribution, a batch and a leading dimension, spread over the
    regimes that select different kernels (lanes across entries, grouped, wide, column tiles, packed short rows,
    huge rows, scalar paths for odd leading dimensions)."""
    rng = np.random.default_rng(9000 + k)
    rows = int(rng.choice([1, 3, 17, 64, 200, 1000, 2500, 5000]))
    cols = int(rng.choice([1, 5, 33, 128, 700, 3000, 9000]))
    kind = rng.choice(["uniform", "zipf", "dense_rows", "empty_heavy"])
    if kind == "uniform":
        lens = rng.binomial(cols, rng.choice([0.002, 0.02, 0.2, 0.7]), size=rows)
    elif kind == "zipf":
        lens = np.minimum(cols, (cols * rng.permutation(np.arange(1, rows + 1)) ** -1.2).astype(np.int64))
    elif kind == "dense_rows":
        lens = np.where(rng.random(rows) < 0.05, cols, rng.integers(0, min(cols, 8) + 1, size=rows))
    else:
        lens = np.where(rng.random(rows) < 0.9, 0, rng.integers(0, min(cols, 300) + 1, size=rows))
    if lens.sum() > 3_000_000:
        lens = (lens * (3_000_000 / lens.sum())).astype(np.int64)
    batch = int(rng.choice([1, 2, 4, 5, 16, 31, 64, 100, 128, 129, 256, 500, 1024]))
    ld = None if rng.random() < 0.7 else batch + int(rng.integers(0, 9))
    return rows, cols, lens.astype(np.int64), batch, ld, bool(rng.random() < 0.5)


@pytest.mark.parametrize("k", range(48))
def test_random_shapes_all_three_products(nb, torch_mod, oracle, k):
    _random_shape_parity(nb, torch_mod, oracle, k, prefer_staged=False)


@pytest.mark.parametrize("k", range(100, 124))
def test_random_shapes_staged_kernels(nb, torch_mod, oracle, k):
    """The same draw at batches the staged kernels accept, bound in the partition mode that prefers them: whatever
    the shape and the row lengths, the staged products and the staged SDDMM (or, for an empty matrix, the others)."""
    _random_shape_parity(nb, torch_mod, oracle, k, prefer_staged=True)


@pytest.mark.parametrize("rows,cols,kind,batch", [
    (2500, 20000, "uniform", 1024),   # forward and SDDMM gather a 20000-row operand: 64- and 128-column tiles beyond an L2
    (2500, 20000, "zipf", 512),
    (20000, 2500, "uniform", 1024),   # the transposed product gathers it
    (20000, 2500, "zipf", 640),       # ... with a few hot operand rows: 128-column tiles
    (2500, 14000, "uniform", 200),    # batches below 512: 64-column tiles from about 128 entries per row on
    (14000, 2500, "uniform", 132),
])
def test_wide_tiles_on_operands_beyond_an_l2(nb, torch_mod, oracle, rows, cols, kind, batch):
    """Operands of more rows than a column tile can keep L2-resident are tiled all the same at wide batches (the tile
    cuts the rows in flight); all three products on such operands, in both orientations, against the oracle."""
    torch = torch_mod
    rng = np.random.default_rng(rows + cols + batch)
    if kind == "uniform":
        lens = rng.binomial(cols, 150.0 / cols, size=rows)
    else:
        lens = np.minimum(cols, (4 * cols * rng.permutation(np.arange(1, rows + 1)) ** -1.2).astype(np.int64))
    indptr, indices = wl.pattern_from_row_nnz(lens.astype(np.int64), cols, seed=rows + batch)
    lay = wl.SparseLayerData(rows, cols, indptr, indices, rng.standard_normal(int(indptr[-1])).astype(np.float32),
                             rng.standard_normal(rows).astype(np.float32), False)
    X = rng.standard_normal((cols, batch)).astype(np.float32)
    dY = rng.standard_normal((rows, batch)).astype(np.float32)
    L = nb.SparseLinear(lay, max_batch=batch)
    Xd = nb.to_dense(X); Yd = nb.dense(rows, batch); dYd = nb.to_dense(dY); dXd = nb.dense(cols, batch)
    g = torch.full((lay.nnz,), float("nan"), device="cuda"); db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, None, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, X, False)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    dX, SdX = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, lay.values, dY)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dY, X)
    close(g.cpu().numpy(), gr, Sg, what="dvalues"); close(db.cpu().numpy(), dbr, Sdb, what="dbias")
    L.close()


def _random_shape_parity(nb, torch_mod, oracle, k, prefer_staged):
    torch = torch_mod
    rows, cols, lens, batch, ld, relu = _random_case(k)
    if prefer_staged:
        batch = int(np.random.default_rng(k).choice([128, 132, 192, 256, 320, 1024]))
        ld = None
    indptr, indices = wl.pattern_from_row_nnz(lens, cols, seed=9100 + k)
    rng = np.random.default_rng(9200 + k)
    lay = wl.SparseLayerData(rows, cols, indptr, indices, rng.standard_normal(int(indptr[-1])).astype(np.float32),
                             rng.standard_normal(rows).astype(np.float32), relu)
    if lay.nnz * batch > 400_000_000:                        # keep the oracle's share of the run short
        batch = max(1, 400_000_000 // max(lay.nnz, 1))
        ld = None
    X = rng.standard_normal((cols, batch)).astype(np.float32)
    dY = rng.standard_normal((rows, batch)).astype(np.float32)
    if prefer_staged:
        batch -= batch % 4                                     # (a cut batch must stay a multiple of 4)
        X, dY = X[:, :batch], dY[:, :batch]
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_PREFER_STAGED)
    try:
        L = nb.SparseLinear(lay, max_batch=batch)
    finally:
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_BALANCED)
    Xd = nb.to_dense(X, ld=ld); Yd = nb.dense(rows, batch, ld=ld); dYd = nb.to_dense(dY, ld=ld); dXd = nb.dense(cols, batch, ld=ld)
    g = torch.full((max(lay.nnz, 1),), float("nan"), device="cuda")[:lay.nnz]
    db = torch.full((rows,), float("nan"), device="cuda")
    nb.sparse_linear_forward(L.handle, Xd, Yd, batch)
    nb.sparse_linear_backward(L.handle, Xd, Yd, dYd, dXd, g, db, batch)
    torch.cuda.synchronize()
    Y, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, X, relu)
    close(Yd.cpu().numpy(), Y, S, what="Y")
    dZ = oracle.relu_backward(dY, Yd.cpu().numpy()) if relu else dY
    dX, SdX = oracle.spmm_t(rows, cols, lay.indptr, lay.indices, lay.values, dZ)
    close(dXd.cpu().numpy(), dX, SdX, what="dX")
    gr, Sg, dbr, Sdb = oracle.sddmm(rows, cols, lay.indptr, lay.indices, dZ, X)
    close(g.cpu().numpy(), gr, Sg, what="dvalues"); close(db.cpu().numpy(), dbr, Sdb, what="dbias")
    L.close()


def test_staged_product_keeps_a_non_finite_operand_row_to_the_rows_that_read_it(nb, torch_mod, oracle):
    """Definition of A = S B (Section 4): output row i depends on operand row j only if (i, j) is stored.  An operand
    row of Inf must therefore reach exactly the output rows that reference it, also in the staged product, whose
    lanes without an entry of their own ride along with weight 0: they gather a zero row, not an operand row.  The
    rows chosen are the first of a column block of 512, where such a lane would otherwise read."""
    torch = torch_mod
    rows, cols, batch = 2048, 1100, 512
    lay = layer_case(rows, cols, 0.3, seed=rows + cols)
    assert nb.nerva_plan_staged_host(rows, cols, lay.indptr, lay.indices, batch)[0].shape[0] > 0     # the staged kernel runs
    rng = np.random.default_rng(5)
    X = rng.standard_normal((cols, batch)).astype(np.float32)
    for j in (0, 512, 1024):
        X[j, :] = np.inf
    L = nb.SparseLinear(lay, max_batch=batch)
    Yd = nb.dense(rows, batch)
    nb.sparse_linear_forward(L.handle, nb.to_dense(X), Yd, batch)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    row_of = np.repeat(np.arange(rows), np.diff(lay.indptr))
    touched = np.zeros(rows, dtype=bool)
    touched[row_of[np.isin(lay.indices, (0, 512, 1024))]] = True
    assert 0.2 * rows < touched.sum() < 0.9 * rows
    Xf = X.copy(); Xf[[0, 512, 1024], :] = 0.0                   # for the untouched rows these operand rows do not exist
    Yr, S = oracle.spmm(rows, cols, lay.indptr, lay.indices, lay.values, lay.bias, Xf, False)
    assert np.all(np.isfinite(Y[~touched])), "an operand row of Inf reached output rows that do not reference it"
    close(Y[~touched], Yr[~touched], S[~touched], what="rows that do not reference the Inf rows")
    assert not np.isfinite(Y[touched]).all(axis=1).any()          # and every row that does reference one shows it
    L.close()
