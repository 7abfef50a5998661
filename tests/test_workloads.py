"""Pins for the synthetic-workload generators against the values the paper prints."""
import json
import os

import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
SIZES = tuple(GOLD["mlp_sizes"]["value"])


def _is_canonical(indptr, indices, rows, cols):
    assert indptr.dtype == np.int32 and indices.dtype == np.int32
    assert indptr.shape == (rows + 1,) and indptr[0] == 0 and indptr[-1] == len(indices)
    assert np.all(np.diff(indptr) >= 0)
    for i in range(rows):
        seg = indices[indptr[i]:indptr[i + 1]]
        assert np.all(np.diff(seg) > 0)
        if len(seg):
            assert 0 <= seg[0] and seg[-1] < cols


def test_dense_parameter_count():
    weights = sum(a * b for a, b in zip(SIZES[:-1], SIZES[1:]))
    biases = sum(SIZES[1:])
    assert weights + biases == GOLD["dense_parameters"]["value"]


def test_parameter_count_at_999_sparsity():
    # stored weights at global density 0.001 plus the dense, unsparsified biases (Section 3)
    nnz = wl.er_layer_nnz(SIZES, 0.001)
    assert sum(nnz) + sum(SIZES[1:]) == GOLD["parameters_at_sparsity_0.999"]["value"]
    assert sum(wl.uniform_layer_nnz(SIZES, 0.999)) + sum(SIZES[1:]) == GOLD["parameters_at_sparsity_0.999"]["value"]


def test_er_densities_match_printed_example():
    d, eps = wl.er_layer_densities(SIZES, 0.01)
    printed = GOLD["er_layer_densities_at_sparsity_0.99"]["value"]
    # The printed example is rounded loosely: 0.00778 / 0.017496 / 0.609 here against
    # 0.008 / 0.018 / 0.6 in print, i.e. agreement to 0.6 units of the last printed digit.
    assert abs(float(d[0]) - printed[0]) < 6e-4 and abs(float(d[1]) - printed[1]) < 6e-4
    assert abs(float(d[2]) - printed[2]) < 0.05
    assert round(1 - float(d[2]), 1) == GOLD["last_layer_sparsity_at_0.99"]["value"]
    # larger layers are sparser
    assert d[0] < d[1] < d[2]
    nnz = wl.er_layer_nnz(SIZES, 0.01)
    total = sum(a * b for a, b in zip(SIZES[:-1], SIZES[1:]))
    assert sum(nnz) == wl.round_half_up(0.01 * total)


def test_er_saturates_small_layers():
    d, _ = wl.er_layer_densities(wl.WIDE_MLP, 0.01)
    assert d[2] == 1.0 and 0 < d[1] < d[0] < 1
    nnz = wl.er_layer_nnz(wl.WIDE_MLP, 0.01)
    assert nnz[2] == 10 * 8192
    total = sum(a * b for a, b in zip(wl.WIDE_MLP[:-1], wl.WIDE_MLP[1:]))
    assert sum(nnz) == wl.round_half_up(0.01 * total)
    # every density of the paper's Table 1 is reachable
    for dens in (1, 0.5, 0.2, 0.1, 0.05, 0.01, 0.005, 0.001):
        dd, _ = wl.er_layer_densities(SIZES, dens)
        assert np.all(dd <= 1.0) and np.all(dd > 0)
        assert sum(wl.er_layer_nnz(SIZES, dens)) == wl.round_half_up(dens * 3675136)


def test_storage_model_close_to_table3():
    """values + column indices (8 B per stored weight) + row pointers + dense biases."""
    for key, printed in GOLD["model_size_bytes_by_density"]["value"].items():
        dens = float(key)
        if dens == 1.0:
            size = 4 * GOLD["dense_parameters"]["value"]
        else:
            nnz = wl.er_layer_nnz(SIZES, dens)
            size = sum(8 * n + 4 * (r + 1) + 4 * r for n, r in zip(nnz, SIZES[1:]))
        assert abs(size - printed) / printed < 0.15, (dens, size, printed)


@pytest.mark.parametrize("rows,cols,nnz", [(5, 7, 0), (5, 7, 35), (5, 7, 11), (64, 33, 500), (1, 1, 1)])
def test_uniform_pattern_is_canonical_and_seeded(rows, cols, nnz):
    a = wl.uniform_pattern(rows, cols, nnz, seed=5)
    b = wl.uniform_pattern(rows, cols, nnz, seed=5)
    _is_canonical(a[0], a[1], rows, cols)
    assert a[0][-1] == nnz
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    if 0 < nnz < rows * cols and nnz > 5:
        c = wl.uniform_pattern(rows, cols, nnz, seed=6)
        assert not (np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1]))


def test_layer_nnz_table():
    assert wl.uniform_layer_nnz(SIZES, 0.99) == [31457, 5243, 51]
    assert wl.uniform_layer_nnz(SIZES, 0.9) == [314573, 52429, 512]
    assert wl.uniform_layer_nnz(SIZES, 0.5) == [1572864, 262144, 2560]


def test_empty_rows_are_legal():
    mlp = wl.make_mlp(SIZES, sparsity=0.999)
    last = mlp.layers[2]
    assert last.nnz == 5 and np.sum(np.diff(last.indptr) == 0) >= 5
    assert not last.relu and mlp.layers[0].relu and mlp.layers[1].relu


def test_zipf_rows():
    rn = wl.zipf_row_nnz(2048, 2048, wl.round_half_up(0.01 * 2048 * 2048), 1.2, seed=3)
    assert rn.sum() == wl.round_half_up(0.01 * 2048 * 2048) and rn.max() <= 2048 and rn.min() >= 0
    srt = np.sort(rn)[::-1].astype(np.float64)
    # power law on the unsaturated part: log-log slope close to -1.2
    sel = (srt < 2048) & (srt > 8)
    r = np.nonzero(sel)[0] + 1
    slope = np.polyfit(np.log(r), np.log(srt[sel]), 1)[0]
    assert -1.3 < slope < -1.1
    indptr, indices = wl.pattern_from_row_nnz(rn, 2048, seed=4)
    _is_canonical(indptr, indices, 2048, 2048)
    assert np.array_equal(np.diff(indptr), rn)


def test_init_values_scale():
    mlp = wl.make_mlp((512, 256, 10), sparsity=0.9)
    lay = mlp.layers[0]
    rn = np.diff(lay.indptr)
    # per-row variance ~ 2 / row_nnz  =>  sum over the row of w^2 ~ 2
    ssq = np.add.reduceat(lay.values.astype(np.float64) ** 2, lay.indptr[:-1][rn > 0])
    assert 1.6 < ssq.mean() < 2.4
    assert lay.values.dtype == np.float32 and not lay.bias.any()


def test_batches_shape_and_labels():
    X, T = wl.make_batches(3072, 10, 100, 3, seed=3000)
    assert X.shape == (3, 3072, 100) and X.dtype == np.float32
    assert T.shape == (3, 100) and T.dtype == np.int32 and T.min() >= 0 and T.max() <= 9
    assert abs(float(X.mean())) < 0.01 and abs(float(X.std()) - 1) < 0.01


def test_learning_rate_schedule_matches_table1_and_decay_rule():
    from paper_2407_17437_amd import schedule
    for dens, lr in GOLD["initial_learning_rate_by_density"]["value"].items():
        assert schedule.initial_learning_rate(float(dens)) == lr
    assert schedule.initial_learning_rate(0.02) == 0.1 and schedule.initial_learning_rate(0.3) == 0.01
    rule = GOLD["lr_decay"]["value"]
    E = rule["epochs"]
    lrs = [schedule.learning_rate(e, E, 0.1) for e in range(E)]
    assert lrs[0] == 0.1 and lrs[49] == 0.1                      # unchanged through the first half
    assert lrs[50] == pytest.approx(0.01) and lrs[74] == pytest.approx(0.01)
    assert lrs[75] == pytest.approx(0.001) and lrs[99] == pytest.approx(0.001)
    assert sorted(set(round(x, 12) for x in lrs), reverse=True) == [0.1, 0.01, 0.001]
    with pytest.raises(ValueError):
        schedule.learning_rate(100, 100, 0.1)
