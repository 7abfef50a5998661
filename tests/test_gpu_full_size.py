"""Parity at the full sizes of the benchmark configurations, in the launch shapes bench.py uses.

Where the oracle cannot finish the whole result in seconds (the 16384 x 16384 matrices), output rows
drawn from every class of the library's static partitions (read from the partitions themselves) are
computed one by one by the oracle on the corresponding sub-pattern and compared at the same
1e-5 * S bar; everything else is compared whole.  Properties that hold at any size (bit-identical pattern, reproducibility)
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


def test_config4_step_whole(nb, torch_mod, oracle):
    """3072-8192-8192-10, global density 1 % split by Erdos-Renyi (dense last layer), batch 1024, the launch
    configuration bench.py times: two fused steps, EVERY element of every stage (activations, loss gradient,
    transposed products, velocities, weights, biases) against the oracle fed the GPU's stage inputs.  The
    second step runs on the weights and the mirror values that the first one updated."""
    torch = torch_mod
    batch, lr, mu = 1024, 0.01, 0.9
    mlp = wl.make_mlp(wl.WIDE_MLP, er_density=0.01)
    assert [l.nnz for l in mlp.layers] == [342893, 498753, 81920]
    Xs, Ts = wl.make_batches(3072, 10, batch, 2, seed=3000)
    M = nb.MLP(mlp, batch)
    digest = [(l.indptr.cpu().numpy().tobytes(), l.indices.cpu().numpy().tobytes()) for l in M.layers]
    worst = 0.0
    for t in range(2):
        before = snapshot(M)
        M.train_step(nb.to_dense(Xs[t]), torch.as_tensor(Ts[t]).cuda(), batch, lr, mu)
        torch.cuda.synchronize()
        worst = max(worst, stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False))
        print(f"config 4 step {t}: worst stage error so far = {worst:.3f} x (1e-5 S)", flush=True)
        for l in range(3):
            w = M.layers[l].values.cpu().numpy()
            assert np.all(np.isfinite(w)) and np.count_nonzero(w != before[l]["values"]) > 0.5 * len(w)
    assert digest == [(l.indptr.cpu().numpy().tobytes(), l.indices.cpu().numpy().tobytes()) for l in M.layers]
    M.close()


@pytest.mark.parametrize("sparsity", [0.5, 0.999])
def test_sweep_ends_step_stage_parity(nb, torch_mod, oracle, sparsity):
    """The two ends of the sparsity sweep on 3072-1024-512-10 at batch 100 (Section 5.1 / 5.3): 50 % (1.57 M
    stored entries in the first layer, other partition targets than at 90 %) and 99.9 % (an output layer with
    5 stored entries in 10 rows, most rows of every layer empty or of a single entry); two fused steps each."""
    torch = torch_mod
    batch, lr, mu = 100, 0.01, 0.9
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=sparsity)
    if sparsity == 0.999:
        assert [l.nnz for l in mlp.layers] == [3146, 524, 5]
    Xs, Ts = wl.make_batches(3072, 10, batch, 2, seed=3000)
    ld = nb.padded_ld(batch)
    Xd = torch.full((2, 3072, ld), float("nan"), device="cuda")
    Xd[:, :, :batch] = torch.as_tensor(Xs).cuda()
    Td = torch.as_tensor(Ts).cuda()
    M = nb.MLP(mlp, batch)
    worst = 0.0
    for t in range(2):
        before = snapshot(M)
        nb.mlp_train_step(M.handle, Xd[t].data_ptr(), ld, Td[t].data_ptr(), batch, lr, mu, M.workspace, M.loss)
        torch.cuda.synchronize()
        worst = max(worst, stage_parity(nb, torch, oracle, M, mlp, before, Xs[t], Ts[t], batch, lr, mu, False))
    for l, lay in zip(M.layers, mlp.layers):
        assert np.array_equal(l.indptr.cpu().numpy(), lay.indptr) and np.array_equal(l.indices.cpu().numpy(), lay.indices)
    print(f"sweep end {sparsity}: worst stage error = {worst:.3f} x (1e-5 S)")
    M.close()


def transposed_csr(lay):
    """Canonical CSR of W^T (stable counting sort by column) and, per mirror entry, its CSR position."""
    perm = np.argsort(lay.indices, kind="stable")
    row_of = np.repeat(np.arange(lay.rows, dtype=np.int32), np.diff(lay.indptr))
    indptr_t = np.zeros(lay.cols + 1, dtype=np.int32)
    np.cumsum(np.bincount(lay.indices, minlength=lay.cols), out=indptr_t[1:])
    return indptr_t, row_of[perm].astype(np.int32), perm


def partition_sample(nb, rows, cols, indptr, indices, batch, rng, budget_entries):
    """Rows that between them touch every class of the library's static partitions of this matrix, read from
    the partitions themselves: every lg class of the ordinary rows (first, last and a random row of the class),
    huge rows (all of the first eight, then random ones), the packed table's longest and shortest rows, rows of
    1 and of 128 entries, an empty row, and from the staged plan a row split over a wave's four lane rows and the
    first and last slot of the first, a middle and the last range; then random rows while the budget lasts.
    Returns {row: reason}."""
    rn = np.diff(indptr)
    picked = {}

    def take(r, why):
        r = int(r)
        if 0 <= r < rows and r not in picked:
            picked[r] = why

    order, blocks, huge, n_huge_blocks, waves = nb.nerva_plan_rows_host(rows, indptr)
    for k, h in enumerate(huge):
        if k < 8:
            take(h[0], f"huge row ({h[2]} shares)")
    if len(huge) > 8:
        for h in huge[rng.choice(np.arange(8, len(huge)), size=min(8, len(huge) - 8), replace=False)]:
            take(h[0], "huge row (random)")
    ordinary = blocks[n_huge_blocks:]
    for lg in np.unique(ordinary[:, 0] & 0xFF) if len(ordinary) else []:
        cls = ordinary[(ordinary[:, 0] & 0xFF) == lg]
        first = int(cls[0, 1]); last = int(cls[-1, 1]) + int(cls[-1, 0] >> 8) - 1
        take(order[first], f"lg {lg} first"); take(order[last], f"lg {lg} last")
        take(order[rng.integers(first, last + 1)], f"lg {lg} random")
    short, n_short, long_waves, _ = nb.nerva_plan_short_rows_host(rows, indptr)
    if n_short:
        take(short[0, 0], "packed: longest"); take(short[n_short - 1, 0], "packed: shortest")
        take(short[n_short // 2, 0], "packed: middle")
        lw = long_waves.reshape(-1, 4)
        lw = lw[lw[:, 0] >= 0]
        if len(lw):
            take(lw[0, 0], "beside the packed rows: first"); take(lw[-1, 0], "beside the packed rows: last")
    for length in (0, 1, 2, 127, 128, 129):
        hit = np.nonzero(rn == length)[0]
        if len(hit):
            take(hit[rng.integers(len(hit))], f"{length} entries")
    # the staged plan as the library binds it: of the long rows only where the rows differ widely in length
    partial = 0 < n_short < rows and int(rn.max()) * rows > 4 * int(indptr[-1])
    slot_rows, ends = nb.nerva_plan_staged_host(rows, cols, indptr, indices, batch, nb.NERVA_PACK_MAX_LEN + 1 if partial else 0)
    if partial and slot_rows.shape[0] == 0:
        slot_rows, ends = nb.nerva_plan_staged_host(rows, cols, indptr, indices, batch, 0)
    n_ranges = slot_rows.shape[0]
    if n_ranges:
        quad = np.nonzero((slot_rows >= 0) & ((slot_rows & nb.NERVA_STAGE_QUAD) != 0))
        if len(quad[0]):
            k = rng.integers(len(quad[0]))
            take(slot_rows[quad[0][k], quad[1][k]] & ~nb.NERVA_STAGE_QUAD, "staged: split over four lane rows")
        for q in sorted({0, n_ranges // 2, n_ranges - 1}):
            used = np.nonzero(slot_rows[q] >= 0)[0]
            if len(used):
                take(slot_rows[q, used[0]] & ~nb.NERVA_STAGE_QUAD, f"staged range {q}: first slot")
                take(slot_rows[q, used[-1]] & ~nb.NERVA_STAGE_QUAD, f"staged range {q}: last slot")
    spent = int(sum(rn[r] for r in picked))
    for r in rng.permutation(rows)[:64]:
        if spent + rn[r] > budget_entries:
            continue
        if int(r) not in picked:
            take(r, "random"); spent += int(rn[r])
    return picked


@pytest.mark.parametrize("density,batch", [(0.001, 1024), (0.001, 128), (0.01, 128), (0.01, 1024), (0.1, 128), (0.1, 1024)])
def test_config5_kernels_sampled(nb, torch_mod, oracle, density, batch):
    """16384 x 16384 with power-law row lengths (rank^-1.2): forward, transposed and sampled products
    alone, checked on rows / columns / entries drawn from every class of the static partitions."""
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
    budget = (3 << 30) // (8 * batch)          # stored entries the oracle walks per direction: seconds of work
    # forward product and SDDMM: rows of W, one or more from every class of W's partitions
    picked = partition_sample(nb, n, n, z.indptr, z.indices, batch, rng, budget)
    reasons = sorted(set(picked.values()))
    assert any(r.startswith("lg ") for r in reasons) and (rn.max() < n or any(r.startswith("huge row") for r in reasons)), reasons
    sel = np.array(sorted(picked), dtype=np.int64)
    ip, ix, pos = sub_rows(z, sel)
    Yr, S = oracle.spmm(len(sel), n, ip, ix, z.values[pos], z.bias[sel], X, False)
    close(Y[sel], Yr, S, what=f"Y rows {reasons}")
    gr, Sg, dbr, Sdb = oracle.sddmm(len(sel), n, ip, ix, dY[sel], X)
    close(gh[pos], gr, Sg, what="dvalues sampled rows")
    close(dbh[sel], dbr, Sdb, what="dbias sampled rows")
    empty = np.nonzero(rn == 0)[0]
    if len(empty):
        assert np.array_equal(Y[empty], np.broadcast_to(z.bias[empty, None], Y[empty].shape))   # empty rows give exactly the bias
    # transposed product: rows of W^T (columns of W), one or more from every class of the mirror's partitions
    indptr_t, indices_t, perm = transposed_csr(z)
    picked_t = partition_sample(nb, n, n, indptr_t, indices_t, batch, rng, budget)
    csel = np.array(sorted(picked_t), dtype=np.int64)
    counts = np.diff(indptr_t)[csel]
    tp = np.zeros(len(csel) + 1, dtype=np.int32); np.cumsum(counts, out=tp[1:])
    tpos = np.concatenate([np.arange(indptr_t[j], indptr_t[j + 1]) for j in csel]) if len(csel) else np.zeros(0, int)
    dXr, SdX = oracle.spmm(len(csel), n, tp, indices_t[tpos], z.values[perm[tpos]], None, dY, False)
    close(dX[csel], dXr, SdX, what=f"dX rows {sorted(set(picked_t.values()))}")
    print(f"n={n} nnz={z.nnz} batch={batch}: {len(sel)} rows ({int(rn[sel].sum())} entries) and {len(csel)} columns "
          f"({int(counts.sum())} entries) checked; classes {reasons}", flush=True)
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
