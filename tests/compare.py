"""Tolerance-aware comparison of a search result with the oracle's.

Bar: probe lists and top-k ids identical except at score ties or near-ties inside
the tolerance; scores within TAU relative (1e-4 for float32 storage, 2e-3 for
16-bit storage).  "Relative" is taken against max(|oracle score|, FLOOR * scale)
where scale is the magnitude of the operands (|q||x| for inner product,
|q|^2 + |x|^2 for squared L2) and FLOOR = 0.02 at d = 768 (floor_for(d) otherwise; callers
pass floor * magnitude as `scale`): a score that is itself the result of cancellation
(a distance near zero, an inner product of near-orthogonal vectors) cannot be
relative-accurate to itself in any float32 arithmetic.
"""
import numpy as np

TAU = {"f32": 1e-4, "f16": 2e-3, "bf16": 2e-3}
FLOOR = 0.02


def floor_for(d):
    """Rounding one operand to a t-bit significand perturbs a d-term dot product by about
    2^-t |q||x| / sqrt(d) (independent components), whatever the size of the result; the floor
    below which errors are judged absolutely scales the same way: 0.02 at d = 768."""
    return 0.02 * (768.0 / d) ** 0.5


def _tol(s_ref, scale, tau):
    return tau * np.maximum(np.abs(s_ref), scale)


def _is_ip(metric):
    return metric in (0, "ip")


def _worse_by(a, b, metric):
    """How much worse score a is than score b (positive = worse)."""
    return (b - a) if _is_ip(metric) else (a - b)


def check_probes(got_probe, got_scores, ref_probe, ref_scores, score_of, metric, tau, scale):
    """got_*: [nq,nprobe] from the path under test; ref_*: the oracle's, best-first.
    score_of(q, centroid_ids) -> oracle coarse scores (float64) for those centroids.
    Returns stats; raises AssertionError when a difference is not a near-tie."""
    nq, nprobe = ref_probe.shape
    exact_rows = 0
    exact_sets = 0
    under = 0               # comparisons in which the absolute floor, not the score itself, set the tolerance
    for q in range(nq):
        g, r = got_probe[q], ref_probe[q]
        assert len(set(g.tolist())) == nprobe, f"query {q}: duplicate probe"
        if np.array_equal(g, r):
            exact_rows += 1
            exact_sets += 1
        else:
            sc = scale[q] if np.ndim(scale) else scale
            bound = ref_scores[q, -1]
            tol = float(_tol(bound, sc, tau))
            extra = np.setdiff1d(g, r)
            missing = np.setdiff1d(r, g)
            if len(extra) == 0:
                exact_sets += 1
            else:
                s_extra = score_of(q, extra)
                assert np.all(_worse_by(s_extra, bound, metric) <= tol), \
                    f"query {q}: probe {extra} not a near-tie of the boundary"
                s_missing = ref_scores[q, np.isin(r, missing)]
                assert np.all(_worse_by(bound, s_missing, metric) <= tol), \
                    f"query {q}: missed probe {missing} is clearly better than the boundary"
            # order: any swap must be between near-equal scores
            s_g = score_of(q, g)
            d = _worse_by(s_g[:-1], s_g[1:], metric)          # >0 where an earlier one is worse
            assert np.all(d <= 2 * tol), f"query {q}: probes out of order"
        sc = scale[q] if np.ndim(scale) else scale
        under += int((np.abs(ref_scores[q]) < sc).sum())
        if got_scores is not None:
            s_g = score_of(q, g)
            assert np.all(np.abs(got_scores[q] - s_g) <= _tol(s_g, sc, tau)), \
                f"query {q}: coarse scores off by {np.abs(got_scores[q] - s_g).max()}"
    return {"exact_order_rate": exact_rows / max(nq, 1), "exact_set_rate": exact_sets / max(nq, 1),
            "n_under_floor": under}


def check_topk(got_ids, got_scores, ref_ids, ref_scores, score_of, metric, tau, scale):
    """Compare [nq,k] results with the oracle's for the same probe lists.
    score_of(q, ids) -> oracle scores (float64) of those labels for query q.
    Returns stats; raises AssertionError on a difference that is not a near-tie."""
    nq, k = ref_ids.shape
    exact = 0
    max_rel = 0.0
    under = 0               # comparisons in which the absolute floor, not the score itself, set the tolerance
    same = total = 0        # ids shared with the oracle / ids the oracle reports
    for q in range(nq):
        g_i, g_s = got_ids[q], got_scores[q].astype(np.float64)
        r_i, r_s = ref_ids[q], ref_scores[q]
        sc = scale[q] if np.ndim(scale) else scale
        nvalid = int((r_i >= 0).sum())
        assert int((g_i >= 0).sum()) == nvalid, f"query {q}: {int((g_i >= 0).sum())} results, want {nvalid}"
        assert np.all(g_i[nvalid:] == -1) and np.array_equal(g_s[nvalid:], r_s[nvalid:]), \
            f"query {q}: padding"
        if nvalid == 0:
            exact += 1
            continue
        g_i, g_s, r_i, r_s = g_i[:nvalid], g_s[:nvalid], r_i[:nvalid], r_s[:nvalid]
        assert len(set(g_i.tolist())) == nvalid, f"query {q}: duplicate ids"
        tol = _tol(r_s, sc, tau)
        under += int((np.abs(r_s) < sc).sum())
        total += nvalid
        same += int(np.isin(g_i, r_i).sum())
        err = np.abs(g_s - r_s)
        assert np.all(err <= tol), f"query {q}: rank-wise score error {err.max()} > tol"
        max_rel = max(max_rel, float((err / np.maximum(np.abs(r_s), sc)).max()))
        # best-first up to rounding
        assert np.all(_worse_by(g_s[:-1], g_s[1:], metric) <= 0), f"query {q}: not sorted"
        if np.array_equal(g_i, r_i):
            exact += 1
            continue
        diff = g_i != r_i
        s_true = score_of(q, g_i[diff])
        assert np.all(np.abs(g_s[diff] - s_true) <= _tol(s_true, sc, tau)), \
            f"query {q}: reported score does not belong to the reported id"
        kth_tol = float(_tol(r_s[-1], sc, tau))
        assert np.all(_worse_by(s_true, r_s[-1], metric) <= kth_tol), \
            f"query {q}: id {g_i[diff]} is worse than the oracle's k-th by more than the tolerance"
        missing = np.setdiff1d(r_i, g_i)
        if len(missing):
            s_miss = r_s[np.isin(r_i, missing)]
            assert np.all(_worse_by(r_s[-1], s_miss, metric) <= kth_tol) or \
                np.all(_worse_by(g_s[-1], s_miss, metric) <= kth_tol), \
                f"query {q}: oracle id {missing} clearly inside the top-k is missing"
    return {"exact_id_rows": exact / max(nq, 1), "id_set_overlap": same / max(total, 1), "max_rel_err": max_rel,
            "n_under_floor": under}
