"""The comparator accepts exact results and near-tie swaps, and rejects real errors."""
import numpy as np
import pytest

from compare import check_probes, check_topk

SCORES = {10: 0.9, 11: 0.8, 12: 0.80001, 13: 0.5, 14: 0.1}


def _score_of(q, ids):
    return np.array([SCORES[int(i)] for i in ids], np.float64)


def _ref():
    return np.array([[10, 12, 11]], np.int64), np.array([[0.9, 0.80001, 0.8]])


def test_topk_exact_and_near_tie_swap():
    ri, rs = _ref()
    st = check_topk(ri.copy(), rs.astype(np.float32), ri, rs, _score_of, "ip", 1e-4, 0.02)
    assert st["exact_id_rows"] == 1.0
    gi = np.array([[10, 11, 12]], np.int64)             # near-tie swapped: fine
    gs = np.array([[0.9, 0.80001, 0.8]], np.float32)
    st = check_topk(gi, gs, ri, rs, _score_of, "ip", 1e-4, 0.02)
    assert st["exact_id_rows"] == 0.0 and st["id_set_overlap"] == 1.0 and st["n_under_floor"] == 0
    st = check_topk(ri.copy(), rs.astype(np.float32), ri, rs, _score_of, "ip", 1e-4, 0.85)
    assert st["n_under_floor"] == 2                      # 0.80001 and 0.8 are judged against 0.85, not against themselves


def test_topk_rejects_wrong_id_score_order_dups_padding():
    ri, rs = _ref()
    with pytest.raises(AssertionError):                 # clearly worse id
        check_topk(np.array([[10, 12, 13]]), np.array([[0.9, 0.80001, 0.8]], np.float32), ri, rs,
                   _score_of, "ip", 1e-4, 0.02)
    with pytest.raises(AssertionError):                 # score error
        check_topk(ri.copy(), np.array([[0.9, 0.81, 0.8]], np.float32), ri, rs, _score_of, "ip",
                   1e-4, 0.02)
    with pytest.raises(AssertionError):                 # duplicates
        check_topk(np.array([[10, 12, 12]]), rs.astype(np.float32), ri, rs, _score_of, "ip", 1e-4, 0.02)
    with pytest.raises(AssertionError):                 # padding where results exist
        check_topk(np.array([[10, 12, -1]]), np.array([[0.9, 0.80001, -np.inf]], np.float32), ri, rs,
                   _score_of, "ip", 1e-4, 0.02)
    # L2 direction and padding accepted when the oracle pads too
    ri2 = np.array([[14, 13, -1]])
    rs2 = np.array([[0.1, 0.5, np.inf]])
    check_topk(ri2.copy(), rs2.astype(np.float32), ri2, rs2, _score_of, "l2", 1e-4, 0.02)
    with pytest.raises(AssertionError):                 # descending order is wrong for L2
        check_topk(np.array([[13, 14, -1]]), np.array([[0.5, 0.1, np.inf]], np.float32), ri2, rs2,
                   _score_of, "l2", 1e-4, 0.02)


def test_probes():
    rp = np.array([[10, 12, 11]], np.int32)
    rs = np.array([[0.9, 0.80001, 0.8]])
    st = check_probes(rp.copy(), None, rp, rs, _score_of, "ip", 1e-4, 0.02)
    assert st == {"exact_order_rate": 1.0, "exact_set_rate": 1.0, "n_under_floor": 0}
    st = check_probes(np.array([[10, 11, 12]], np.int32), None, rp, rs, _score_of, "ip", 1e-4, 0.02)
    assert st == {"exact_order_rate": 0.0, "exact_set_rate": 1.0, "n_under_floor": 0}
    # a boundary score smaller than the floor is counted: the tolerance there is absolute
    st = check_probes(rp.copy(), None, rp, rs, _score_of, "ip", 1e-4, 0.85)
    assert st["n_under_floor"] == 2
    with pytest.raises(AssertionError):                 # 13 is no near-tie of the boundary
        check_probes(np.array([[10, 12, 13]], np.int32), None, rp, rs, _score_of, "ip", 1e-4, 0.02)
    with pytest.raises(AssertionError):                 # out of order beyond tolerance
        check_probes(np.array([[12, 10, 11]], np.int32), None, rp, rs, _score_of, "ip", 1e-4, 0.02)
    with pytest.raises(AssertionError):                 # wrong coarse scores
        check_probes(rp.copy(), np.array([[0.9, 0.7, 0.8]]), rp, rs, _score_of, "ip", 1e-4, 0.02)
