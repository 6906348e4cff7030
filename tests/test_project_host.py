"""pconv_project (the library's host-side projection onto the PCONV constraints) against the
oracle's: both decide on double sums over the taps in ascending order, so pattern ids and the kept
set must agree exactly.  No GPU needed."""
import numpy as np
import pytest

import oracle
import paper_1909_05073_amd as P
from pconv_inputs import PATTERN_TABLE


@pytest.mark.parametrize("seed,f,c,np_,keep_div", [(1, 16, 16, 4, 2.0), (2, 64, 48, 8, 3.6), (3, 130, 70, 12, 8.0),
                                                    (4, 7, 300, 8, 2.5), (5, 33, 1, 16, 1.0)])
def test_project_matches_the_oracle_exactly(seed, f, c, np_, keep_div):
    rng = np.random.default_rng(seed)
    table = np.concatenate([PATTERN_TABLE, np.array([0x1FF, 0x145, 0x010, 0x007], np.uint16)])[:np_]
    w = rng.standard_normal((f, c, 3, 3)).astype(np.float32)
    w[rng.random((f, c)) < 0.1] = 0.0                      # whole zero kernels: ties on energy 0
    w[0, 0] = w[-1, -1]                                     # two equal kernels: a tie between kernels
    keep = int(round(f * c / keep_div))
    pid, conn = P.pconv_project(w, table, keep)
    rp, rc = oracle.project(w, table, keep)
    assert np.array_equal(pid, rp)
    assert np.array_equal(conn, rc)
    assert int(conn.sum()) == keep


def test_projected_layer_packs_and_round_trips():
    """project -> pack (host stages) -> export: the packed layer holds exactly the projected weights."""
    rng = np.random.default_rng(9)
    f, c = 40, 24
    table = PATTERN_TABLE[:8]
    w = rng.standard_normal((f, c, 3, 3)).astype(np.float32)
    pid, conn = P.pconv_project(w, table, 300)
    h = P.pconv_pack(w, pid, conn, table, "f32", host_only=True)
    got = P.pconv_debug_export(h)
    ref = oracle.pack(w, pid, conn, table)
    for k in ("perm", "row_ptr", "pat_cnt", "cin", "vals"):
        assert got[k].tobytes() == ref[k].tobytes(), k
    assert h.info().kept_kernels == 300
    h.free()


def test_project_rejects_bad_arguments():
    w = np.zeros((2, 2, 3, 3), np.float32)
    with pytest.raises(P.PconvError) as e:
        P.pconv_project(w, np.array([0], np.uint16), 1)
    assert e.value.status == P.INVALID_ARG
    with pytest.raises(P.PconvError):
        P.pconv_project(w, PATTERN_TABLE[:4], 5)
    with pytest.raises(P.PconvError):
        P.pconv_project(w, PATTERN_TABLE[:4], -1)
