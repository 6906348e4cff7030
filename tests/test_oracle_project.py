"""Pins of the projection oracle (oracle/pconv_project_oracle.c): the Euclidean projection of dense
3x3 weights onto "every kernel masked by one pattern of the table, at most `keep` kernels kept"
(the step an ADMM pruner for PCONV needs; paper, "Accuracy Analysis").  Parity with the paper's own
assignments is unpinned (the paper prints none)."""
import itertools

import numpy as np
import pytest

import oracle
from pconv_inputs import PATTERN_TABLE


def masked(w, table, pid, conn):
    bits = ((table[pid][..., None] >> np.arange(9)) & 1).reshape(pid.shape + (3, 3))
    return w.astype(np.float64) * bits * conn[..., None, None]


def dist2(w, z):
    return float(((w.astype(np.float64) - z) ** 2).sum())


@pytest.mark.parametrize("seed,f,c,keep", [(0, 2, 2, 2), (1, 1, 4, 3), (2, 3, 1, 1), (3, 2, 2, 4), (4, 2, 2, 0)])
def test_projection_is_the_closest_feasible_point_by_exhaustive_search(seed, f, c, keep):
    """Every choice of a pattern per kernel and of `keep` kernels out of F*C: none is closer to W."""
    rng = np.random.default_rng(seed)
    table = PATTERN_TABLE[[0, 2, 5]]
    w = rng.standard_normal((f, c, 3, 3)).astype(np.float32)
    pid, conn = oracle.project(w, table, keep)
    assert int(conn.sum()) == keep
    got = dist2(w, masked(w, table, pid, conn))
    best = np.inf
    kernels = list(itertools.product(range(f), range(c)))
    for chosen in itertools.combinations(range(f * c), keep):
        cn = np.zeros((f, c), np.uint8)
        for k in chosen:
            cn[kernels[k]] = 1
        for pats in itertools.product(range(len(table)), repeat=keep):
            pp = np.zeros((f, c), np.int64)
            for k, p in zip(chosen, pats):
                pp[kernels[k]] = p
            best = min(best, dist2(w, masked(w, table, pp, cn)))
    assert got <= best * (1 + 1e-12) + 1e-300
    # any weight tensor with fewer kept kernels is no closer either (kept energy is non-negative)
    assert got <= dist2(w, np.zeros_like(w, dtype=np.float64)) + 1e-12


def test_one_dense_mask_keeps_the_largest_kernels_by_norm():
    rng = np.random.default_rng(7)
    w = rng.standard_normal((6, 5, 3, 3)).astype(np.float32)
    pid, conn = oracle.project(w, np.array([0x1FF], np.uint16), 11)
    assert not pid.any()
    norms = (w.astype(np.float64) ** 2).sum(axis=(2, 3)).ravel()
    top = set(np.argsort(-norms, kind="stable")[:11].tolist())
    assert set(np.flatnonzero(conn.ravel()).tolist()) == top


def test_keep_all_keep_none_and_pattern_choice_per_kernel():
    rng = np.random.default_rng(8)
    table = PATTERN_TABLE[:8]
    w = rng.standard_normal((4, 7, 3, 3)).astype(np.float32)
    pid_all, conn_all = oracle.project(w, table, 28)
    assert conn_all.all()
    pid_none, conn_none = oracle.project(w, table, 0)
    assert not conn_none.any() and np.array_equal(pid_all, pid_none)
    # the chosen pattern keeps at least as much energy as any other pattern of the table
    sq = w.astype(np.float64).reshape(4, 7, 9) ** 2
    for p, mask in enumerate(table):
        bits = (int(mask) >> np.arange(9)) & 1
        e_p = (sq * bits).sum(-1)
        e_best = np.take_along_axis(np.stack([(sq * ((int(m) >> np.arange(9)) & 1)).sum(-1) for m in table], -1),
                                    pid_all[..., None].astype(np.int64), -1)[..., 0]
        assert (e_best >= e_p - 1e-15).all()


def test_ties_go_to_the_smaller_index():
    w = np.zeros((1, 3, 3, 3), np.float32)
    w[0, :, 1, 1] = 2.0                      # three identical kernels: centre tap only
    pid, conn = oracle.project(w, PATTERN_TABLE[:4], 2)
    assert pid.tolist() == [[0, 0, 0]]       # every pattern keeps the centre: the first wins
    assert conn.tolist() == [[1, 1, 0]]


def test_a_weight_already_in_pconv_form_is_a_fixed_point():
    """Projecting weights that already satisfy the constraints returns their own masks."""
    from pconv_inputs import LayerSpec, make_layer
    L = make_layer(LayerSpec("p", 1, 24, 20, 8, 8, num_patterns=8, pattern_dist="uniform"), 5)
    wm = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"]).astype(np.float32)
    keep = int(L["conn"].sum())
    pid, conn = oracle.project(wm, L["table"], keep)
    assert np.array_equal(conn, (L["conn"] != 0).astype(np.uint8))
    kept = conn.astype(bool)
    # (two masks of the table may both contain all four kept taps only if they are equal: they are not)
    assert np.array_equal(pid[kept], L["pattern_id"][kept])
