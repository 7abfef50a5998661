"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates CSR patterns, plans the row partition, and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nb():
    from paper_2407_17437_amd import binding
    return binding


def test_header_symbols_are_exported(nb):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b([a-z_0-9]+)\s*\(", header)) - {"defined"}
    assert declared == set(nb.EXPORTS), declared ^ set(nb.EXPORTS)
    for name in declared:
        assert hasattr(nb.lib, name), name
    assert "gfx950" in nb.build_info()


def test_library_is_newer_than_its_sources(nb):
    csrc = os.path.join(ROOT, "paper_2407_17437_amd", "csrc")
    srcs = [os.path.join(csrc, f) for f in os.listdir(csrc)] + [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    stale = [s for s in srcs if os.path.getmtime(s) > os.path.getmtime(nb.LIB_PATH)]
    assert not stale, f"rebuild the library: {stale} changed after it was built"


def test_validate_csr_accepts_generated_patterns(nb):
    for rows, cols, nnz in [(5, 7, 0), (5, 7, 35), (64, 33, 500)]:
        indptr, indices = wl.uniform_pattern(rows, cols, nnz, seed=1)
        assert nb.nerva_validate_csr_host(rows, cols, nnz, indptr, indices) == nb.NERVA_OK


def test_validate_csr_rejects_broken_patterns(nb):
    indptr, indices = wl.uniform_pattern(6, 9, 20, seed=2)
    ok = lambda ip, ix, nnz=20, cols=9: nb.nerva_validate_csr_host(6, cols, nnz, ip, ix)
    assert ok(indptr, indices) == 0
    bad = indptr.copy(); bad[0] = 1
    assert ok(bad, indices) == nb.NERVA_ERR_CSR and "indptr[0]" in nb.last_error()
    bad = indptr.copy(); bad[3], bad[4] = bad[4] + 1, bad[3]
    assert ok(bad, indices) == nb.NERVA_ERR_CSR
    bad = indptr.copy(); bad[-1] = 19
    assert ok(bad, indices) == nb.NERVA_ERR_CSR
    bad = indices.copy(); bad[5] = 9
    assert ok(indptr, bad) == nb.NERVA_ERR_CSR and "out of range" in nb.last_error()
    bad = indices.copy(); bad[5] = -1
    assert ok(indptr, bad) == nb.NERVA_ERR_CSR
    # duplicate / unsorted inside a row
    row = int(np.argmax(np.diff(indptr) >= 2)); p = indptr[row]
    bad = indices.copy(); bad[p + 1] = bad[p]
    assert ok(indptr, bad) == nb.NERVA_ERR_CSR and "ascending" in nb.last_error()
    bad = indices.copy(); bad[p], bad[p + 1] = bad[p + 1], bad[p]
    assert ok(indptr, bad) == nb.NERVA_ERR_CSR
    assert ok(indptr, indices, nnz=21) == nb.NERVA_ERR_CSR
    assert nb.lib.nerva_validate_csr_host(6, 9, 20, None, None) == nb.NERVA_ERR_ARGUMENT
    assert nb.lib.nerva_validate_csr_host(-1, 9, 0, indptr.ctypes.data, None) == nb.NERVA_ERR_ARGUMENT


def _check_plan(nb, indptr, rows):
    order, blocks, huge, n_huge_blocks, waves = nb.nerva_plan_rows_host(rows, indptr)
    W = nb.NERVA_WAVES_PER_BLOCK
    # per-wave table: the shares of every row tile its entries exactly once, in order, in multiples of 4
    seen = {}
    for b in range(len(blocks)):
        for w in range(W):
            row, s0, s1, fl = waves[b, w].tolist()
            if row < 0:
                assert s0 == s1
                continue
            assert indptr[row] <= s0 <= s1 <= indptr[row + 1]
            end = blocks[b, 3] if blocks[b, 0] & nb.NERVA_HUGE_FLAG else indptr[row + 1]
            assert (s1 - s0) % 4 == 0 or s1 == end
            assert ((fl >> 9) & 1) == (1 if blocks[b, 0] & nb.NERVA_HUGE_FLAG else 0)
            seen.setdefault(row, []).append((b, w, s0, s1, (fl >> 8) & 1))
    assert sorted(seen) == list(range(rows))
    for row, shares in seen.items():
        pos = int(indptr[row])
        for k, (b, w, s0, s1, lead) in enumerate(shares):       # table order = entry order
            assert s0 == pos or s0 == s1 == int(indptr[row + 1])
            pos = max(pos, s1)
            assert lead == (1 if k == 0 else 0)                  # exactly one owner per row: its first share
        assert pos == int(indptr[row + 1])
    nnz = int(indptr[-1])
    target = min(64, max(8, nnz // 4096))             # entries per wave aimed at for ordinary rows
    cap = min(64, max(8, nnz // 16384)) * W          # huge rows are cut finer
    row_nnz = np.diff(indptr)
    huge_ids = huge[:, 0].tolist()
    assert sorted(order.tolist() + huge_ids) == list(range(rows))           # every row exactly once
    assert set(huge_ids) == set(np.nonzero(row_nnz > 4 * cap)[0].tolist())    # huge = far beyond one work-group
    # huge work-groups come first and tile each huge row's entries exactly, in order
    assert all(b[0] & nb.NERVA_HUGE_FLAG for b in blocks[:n_huge_blocks])
    assert not any(b[0] & nb.NERVA_HUGE_FLAG for b in blocks[n_huge_blocks:])
    for r, first, parts, _ in huge.tolist():
        pos = int(indptr[r])
        for q in range(parts):
            info, row, b, e = blocks[first + q].tolist()
            assert row == r and (info & ~nb.NERVA_HUGE_FLAG) == q and b == pos and b < e <= b + 2 * cap
            pos = e
        assert pos == int(indptr[r + 1])
        assert parts == -(-int(row_nnz[r]) // (2 * cap))
    covered = 0
    prev_lg = 99
    max_lg = W.bit_length() - 1
    rows_in_class, promoted = [0] * (max_lg + 1), [0] * (max_lg + 1)
    for info, f, _, _ in blocks[n_huge_blocks:].tolist():
        lg, n = info & 0xFF, info >> 8
        assert 1 <= n <= (W >> lg) and f == covered
        assert lg <= prev_lg                                       # heavy rows are served first
        prev_lg = lg
        for r in order[f:f + n]:
            k = int(row_nnz[r])
            assert -(-k // (1 << lg)) <= (target if (1 << lg) < W else 4 * target)   # a full work-group may run 4x over
            rows_in_class[lg] += 1
            if lg > 0 and -(-k // (1 << (lg - 1))) <= target:     # more waves than its length asks for:
                promoted[lg] += 1                                  # handed up by a class that could not fill a work-group
        covered += n
    assert covered == len(order)
    natural = [0] * (max_lg + 1)                                   # the classes by length alone
    for r in order.tolist():
        k, lg = int(row_nnz[r]), 0
        while lg < max_lg and -(-k // (1 << lg)) > target:
            lg += 1
        natural[lg] += 1
    assert len(blocks) - n_huge_blocks <= sum(-(-natural[lg] // (W >> lg)) for lg in range(max_lg + 1))
    for lg in range(max_lg):
        assert promoted[lg + 1] <= sum((W >> l) - 1 for l in range(lg + 1))
        if promoted[lg + 1]:                                       # a class hands up a whole left-over work-group or nothing
            assert rows_in_class[lg] % (W >> lg) == 0
    assert promoted[0] == 0
    # inside one class the rows come longest first, ties in row order
    lg_of_slot = np.concatenate([np.full(info >> 8, info & 0xFF) for info in blocks[n_huge_blocks:, 0].tolist()] or [np.zeros(0, int)])
    key = list(zip((-lg_of_slot).tolist(), (-row_nnz[order]).tolist(), order.tolist()))
    assert key == sorted(key)
    return order, blocks, huge, n_huge_blocks


def test_row_split_mode(nb):
    """The measurement aid: plain row splitting gives every row exactly one wave and nothing else."""
    lens = np.array([0, 5, 70000, 300, 1] * 500)
    indptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    nb.nerva_set_partition_mode(nb.NERVA_PARTITION_ROW_SPLIT)
    try:
        order, blocks, huge, nh, waves = nb.nerva_plan_rows_host(len(lens), indptr)
        assert nh == 0 and len(huge) == 0 and sorted(order.tolist()) == list(range(len(lens)))
        recs = waves.reshape(-1, 4)
        recs = recs[recs[:, 0] >= 0]
        assert len(recs) == len(lens)
        assert np.array_equal(recs[:, 1], indptr[recs[:, 0]]) and np.array_equal(recs[:, 2], indptr[recs[:, 0] + 1])
        assert nb.nerva_plan_short_rows_host(len(lens), indptr)[1] == 0
    finally:
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_BALANCED)
    with pytest.raises(nb.NervaError):
        nb.nerva_set_partition_mode(7)
    _, _, huge, nh, _ = nb.nerva_plan_rows_host(len(lens), indptr)
    assert nh > 0                                                    # back to the balanced partition


def test_short_row_partition(nb):
    """Second partition: short rows longest first, each exactly once; the other rows tiled by the
    long partition; none at all below the row-count threshold."""
    W = nb.NERVA_WAVES_PER_BLOCK
    rng = np.random.default_rng(5)
    for rows, lens in [(5000, rng.integers(0, 40, 5000)),
                       (4096, np.where(rng.random(4096) < 0.1, rng.integers(129, 3000, 4096), rng.integers(0, 129, 4096))),
                       (3000, np.full(3000, 128))]:
        indptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        short, ns, waves, n_long_huge = nb.nerva_plan_short_rows_host(rows, indptr)
        is_short = lens <= nb.NERVA_PACK_MAX_LEN
        assert ns == int(is_short.sum()) and len(short) == (ns + 63) // 64 * 64
        got = short[:ns]
        assert sorted(got[:, 0].tolist()) == np.nonzero(is_short)[0].tolist()
        assert np.array_equal(got[:, 1], indptr[got[:, 0]]) and np.array_equal(got[:, 2], lens[got[:, 0]])
        key = list(zip((-got[:, 2]).tolist(), got[:, 0].tolist()))
        assert key == sorted(key)                                   # longest first, ties in row order
        assert (short[ns:] == np.array([-1, 0, 0, 0])).all() and (got[:, 3] == 0).all()
        seen = {}
        for b in range(len(waves)):
            for w in range(W):
                row, s0, s1, fl = waves[b, w].tolist()
                if row >= 0:
                    seen.setdefault(row, []).append((s0, s1))
        assert sorted(seen) == np.nonzero(~is_short)[0].tolist()
        for row, shares in seen.items():
            pos = int(indptr[row])
            for s0, s1 in shares:
                assert s0 == pos or s0 == s1
                pos = max(pos, s1)
            assert pos == int(indptr[row + 1])
        # the huge work-groups of the long partition are those of the full one, in the same slots
        _, blocks, _, nh, full_waves = nb.nerva_plan_rows_host(rows, indptr)
        assert n_long_huge == nh and np.array_equal(waves[:nh], full_waves[:nh])
    # too few short rows, or an empty matrix: no second partition
    indptr = np.concatenate([[0], np.cumsum(np.full(2047, 3))]).astype(np.int32)
    assert nb.nerva_plan_short_rows_host(2047, indptr)[1] == 0
    assert nb.nerva_plan_short_rows_host(4000, np.zeros(4001, dtype=np.int32))[1] == 0


def test_staged_ranges_and_segment_bounds(nb):
    """Third form: ranges of consecutive rows (at most 512 each), every row in exactly one slot, longest first
    inside a range, and per slot the positions that cut its row at the multiples of 512 in the column indices."""
    R, RR = nb.NERVA_STAGE_ROWS, nb.NERVA_STAGE_RANGE_ROWS
    cases = [(700, 1300, wl.uniform_pattern(700, 1300, 700 * 1300 // 5, seed=3), 256),
             (2048, 512, wl.uniform_pattern(2048, 512, 2048 * 512 // 10, seed=4), 1024),
             (5000, 900, wl.uniform_pattern(5000, 900, 5000 * 900 // 4, seed=8), 2048),
             (640, 2100, wl.pattern_from_row_nnz(wl.zipf_row_nnz(640, 2100, 640 * 2100 // 8, 1.2, seed=5), 2100, seed=6), 128)]
    for rows, cols, (indptr, indices), max_batch in cases:
        slot_rows, ends = nb.nerva_plan_staged_host(rows, cols, indptr, indices, max_batch)
        ranges, nb1, _ = ends.shape
        n_tiles = -(-max_batch // nb.NERVA_STAGE_COLS)
        assert nb1 - 1 == -(-cols // R)
        assert ranges >= max(-(-rows // RR), min(256 // n_tiles, rows // 64)) and ranges <= 256 // n_tiles + -(-rows // RR)
        lens = np.diff(indptr)
        seen = np.zeros(rows, dtype=np.int32)
        first = []
        n_quads = 0
        for q in range(ranges):
            used = slot_rows[q] >= 0
            n = int(used.sum())
            assert n >= 1 and used[:n].all() and (ends[q][:, ~used] == 0).all()
            quad = (slot_rows[q, :n] & nb.NERVA_STAGE_QUAD) != 0
            r = slot_rows[q, :n] & ~nb.NERVA_STAGE_QUAD
            nq = int(quad.sum())
            assert nq % 4 == 0 and quad[:nq].all()                              # split rows first, four slots each
            assert (r[:nq].reshape(-1, 4) == r[:nq:4, None]).all()
            n_quads += nq // 4
            e = ends[q][:, :n]
            assert (e[:, :nq].reshape(nb1, -1, 4) == e[:, :nq:4, None]).all()    # ... holding the same bounds
            keep = np.ones(n, dtype=bool); keep[:nq] = (np.arange(nq) % 4 == 0)
            r, e = r[keep], e[:, keep]
            seen[r] += 1
            assert r.max() - r.min() == len(r) - 1                              # consecutive rows
            first.append(int(r.min()))
            key = list(zip((-lens[r]).tolist(), r.tolist()))
            assert key == sorted(key)                                           # longest first, ties in row order
            assert (lens[r[:nq // 4]] >= 256).all()
            assert np.array_equal(e[0], indptr[r]) and np.array_equal(e[-1], indptr[r + 1]) and (np.diff(e, axis=0) >= 0).all()
            for s in range(0, len(r), max(1, len(r) // 7)):                     # the cut positions, on a sample of slots
                row_cols = indices[indptr[r[s]]:indptr[r[s] + 1]]
                want = indptr[r[s]] + np.searchsorted(row_cols, np.arange(nb1) * R)
                assert np.array_equal(e[:, s], want)
        assert (n_quads > 0) == (rows == 640)                                    # only the power-law case has rows that long
        assert (seen == 1).all() and first == sorted(first)
    indptr, indices = cases[0][2]
    assert nb.nerva_plan_staged_host(700, 1300, indptr, indices, 127)[0].shape[0] == 0      # batch too narrow
    ip, ix = wl.uniform_pattern(700, 1300, 700 * 13, seed=7)
    assert nb.nerva_plan_staged_host(700, 1300, ip, ix, 256)[0].shape[0] == 0                # too few entries per staged row
    assert nb.nerva_plan_staged_host(50, 40, np.zeros(51, dtype=np.int32), np.zeros(0, dtype=np.int32), 256)[0].shape[0] == 0


def test_staged_plan_of_the_long_rows_only(nb):
    """With min_entries the plan covers exactly the rows that long, each once, ranges still in row order."""
    rows = cols = 6144
    lens = wl.zipf_row_nnz(rows, cols, rows * cols * 3 // 100, 1.2, seed=19)
    indptr, indices = wl.pattern_from_row_nnz(lens, cols, seed=20)
    m = nb.NERVA_PACK_MAX_LEN + 1
    slot_rows, ends = nb.nerva_plan_staged_host(rows, cols, indptr, indices, 1024, m)
    assert slot_rows.shape[0] == 16                                              # 256 work-groups at 16 column tiles
    got = slot_rows[slot_rows >= 0] & ~nb.NERVA_STAGE_QUAD
    quad = (slot_rows[slot_rows >= 0] & nb.NERVA_STAGE_QUAD) != 0
    want = np.nonzero(lens >= m)[0]
    assert np.array_equal(np.unique(got), want) and len(got) == len(want) + 3 * int(quad.sum()) // 4
    lo = [int((r[r >= 0] & ~nb.NERVA_STAGE_QUAD).min()) for r in slot_rows]
    hi = [int((r[r >= 0] & ~nb.NERVA_STAGE_QUAD).max()) for r in slot_rows]
    assert all(h < l for h, l in zip(hi[:-1], lo[1:]))                           # ranges are runs of the covered rows
    for q, s in [(0, 0), (7, 3), (15, 1)]:
        r = int(slot_rows[q, s] & ~nb.NERVA_STAGE_QUAD)
        assert ends[q, 0, s] == indptr[r] and ends[q, -1, s] == indptr[r + 1]


def test_row_plan_uniform_and_skewed(nb):
    mlp = wl.make_mlp(wl.CIFAR_MLP, sparsity=0.9)
    for lay in mlp.layers:
        _check_plan(nb, lay.indptr, lay.rows)
    # layer 1 at 90 %: 307 entries per row on average, 64 per wave aimed at -> 8 waves per row (a few
    # rows of at most 256 entries take 4), two rows per work-group, none huge
    _, blocks, huge, nh, _ = nb.nerva_plan_rows_host(1024, mlp.layers[0].indptr)
    lgs = (blocks[:, 0] & 0xFF).tolist()
    assert 512 <= len(blocks) <= 520 and set(lgs) <= {2, 3} and lgs.count(3) >= 500 and nh == 0 and len(huge) == 0
    z = wl.make_zipf_matrix(1024, 0.02, seed=5)
    order, blocks, huge, nh = _check_plan(nb, z.indptr, 1024)
    assert len(set((blocks[nh:, 0] & 0xFF).tolist())) >= 3         # several row classes in one matrix
    assert len(huge) >= 1 and nh >= 2                              # and rows cut over several work-groups
    # the dense last layer of the wide MLP: every row is huge
    dense = np.arange(0, 11 * 8192, 8192, dtype=np.int32)
    order, blocks, huge, nh = _check_plan(nb, dense, 10)
    assert len(order) == 0 and len(huge) == 10 and nh == len(blocks) == 320
    empty = np.zeros(11, dtype=np.int32)
    order, blocks, huge, nh = _check_plan(nb, empty, 10)
    assert len(blocks) == 1 and blocks[0, 0] == (10 << 8) and nh == 0


def test_argument_errors_come_before_any_device_work(nb):
    lib = nb.lib
    h = ctypes.c_void_p()
    assert lib.sparse_linear_create(None, 4, 4, 0, None, None, None, None, 0, 8, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sparse_linear_create(ctypes.addressof(h), 0, 4, 0, None, None, None, None, 0, 8, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sparse_linear_create(ctypes.addressof(h), 4, 4, 3, None, None, None, None, 0, 8, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sparse_linear_forward(None, None, 4, None, 4, 4, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sparse_linear_backward(None, None, 0, None, 0, None, 0, None, 0, None, None, 4, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sgd_update_values(None, None, None, 5, 0.1, 0.9, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sgd_update_values(None, None, None, -1, 0.1, 0.9, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.sgd_update_values(None, None, None, 0, 0.1, 0.9, None) == nb.NERVA_OK       # empty update is a no-op
    assert lib.softmax_cross_entropy(None, 4, None, 10, 4, None, 4, None, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.mlp_create(ctypes.addressof(h), 0, None, None, None, 4, 0) == nb.NERVA_ERR_ARGUMENT
    assert lib.mlp_train_step(None, None, 4, None, 4, 0.1, 0.9, None, 0, None, None) == nb.NERVA_ERR_ARGUMENT
    assert lib.mlp_workspace_bytes(None, 4) == 0
    assert lib.nerva_copy_f32(None, None, 3, None) == nb.NERVA_ERR_ARGUMENT
    assert nb.last_error() != ""
    lib.sparse_linear_destroy(None)
    lib.mlp_destroy(None)


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    import importlib
    from paper_2407_17437_amd import binding
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError, match="no fallback"):
        binding._load()
