"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no worked search, so the pins are: a hand-worked integer example
(tests/golden), a dense float64 matmul + stable sort (library routine for the
special case "no index"), exact conversion tables for the 16-bit storage types,
and invariants that the definition in Section 2.2 of the paper fixes.
"""
import os

import numpy as np
import pytest
import torch

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
RNG = np.random.default_rng(12345)


def _store(x, dtype):
    """Round float32 data to a storage dtype; returns (array for the oracle, float64 values)."""
    if dtype == "f32":
        a = x.astype(np.float32)
        return a, a.astype(np.float64)
    if dtype == "f16":
        a = x.astype(np.float16)
        return a, a.astype(np.float64)
    t = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16).copy()
    return bits, t.to(torch.float64).numpy()


def _random_index(n, d, nlist, dtype="f32", dup=False):
    x = RNG.standard_normal((n, d)).astype(np.float32)
    if dup:
        x[n // 2:] = x[: n - n // 2]          # every vector twice
    cent = RNG.standard_normal((nlist, d)).astype(np.float32)
    sizes = RNG.multinomial(n, np.ones(nlist) / nlist)
    sizes[0] += sizes[-1]
    sizes[-1] = 0                              # one empty list
    off = np.zeros(nlist + 1, np.int64)
    off[1:] = np.cumsum(sizes)
    ids = RNG.permutation(n).astype(np.int64) + 1000
    stored, vals = _store(x, dtype)
    return cent, off, stored, vals, ids


def _dense_reference(q, vals, ids, k, metric):
    """float64 matmul + lexsort: the textbook definition through library routines."""
    q64 = q.astype(np.float64)
    if metric == oracle.IP:
        s = q64 @ vals.T
        key = -s
    else:
        s = ((q64[:, None, :] - vals[None, :, :]) ** 2).sum(-1)
        key = s
    out_i = np.empty((q.shape[0], k), np.int64)
    out_s = np.empty((q.shape[0], k), np.float64)
    for r in range(q.shape[0]):
        order = np.lexsort((ids, key[r]))[:k]
        out_i[r] = ids[order]
        out_s[r] = s[r, order]
    return out_i, out_s


# ---------------------------------------------------------------- golden example
def _golden_cases():
    cases = []
    with open(os.path.join(HERE, "golden", "tiny_ivf_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, probe, ids, scores = [p.split() for p in line.split("|")]
            cases.append((head[0], int(head[1]), int(head[2]), [int(v) for v in probe],
                          [int(v) for v in ids], [float(v) for v in scores]))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: f"{c[0]}-p{c[1]}-k{c[2]}")
def test_hand_worked_example(case):
    metric, nprobe, k, probe_exp, ids_exp, scores_exp = case
    cent = np.array([[4, 0], [0, 4], [-4, 0]], np.float32)
    vec = np.array([[3, 0], [5, 1], [4, -2], [0, 3], [1, 5], [-3, 0], [-5, -1]], np.float32)
    off = np.array([0, 3, 5, 7], np.int64)
    ids = np.array([10, 11, 12, 20, 21, 30, 31], np.int64)
    q = np.array([[2, 1]], np.float32)
    m = oracle.IP if metric == "ip" else oracle.L2
    for dtype in ("f32", "f16", "bf16"):       # small integers are exact in all three
        stored, _ = _store(vec, dtype)
        probe, out_i, out_s = oracle.ivf_search(q, cent, off, stored, dtype, ids, nprobe, k, m)
        assert probe[0].tolist() == probe_exp
        assert out_i[0].tolist() == ids_exp
        assert out_s[0].tolist() == scores_exp


# ---------------------------------------------------------------- storage conversions
def test_half_conversion_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16).reshape(-1, 1)
    q = np.ones((1, 1), np.float32)
    got = oracle.pair_scores(q, h, "f16", oracle.IP, np.zeros(65536, np.int64), np.arange(65536))
    want = h[:, 0].astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])      # (-0 + 0 = +0 in the accumulator: sign of zero not compared)


def test_bf16_conversion_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(-1, 1)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()[:, 0]
    q = np.ones((1, 1), np.float32)
    got = oracle.pair_scores(q, bits, "bf16", oracle.IP, np.zeros(65536, np.int64), np.arange(65536))
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])


# ---------------------------------------------------------------- brute force vs library
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_bruteforce_matches_dense_float64(dtype, metric):
    n, d, k = 700, 24, 9
    _, _, stored, vals, ids = _random_index(n, d, 5, dtype)
    q = RNG.standard_normal((13, d)).astype(np.float32)
    got_i, got_s = oracle.bruteforce(q, stored, dtype, ids, k, metric)
    ref_i, ref_s = _dense_reference(q, vals, ids, k, metric)
    assert np.array_equal(got_i, ref_i)
    np.testing.assert_allclose(got_s, ref_s, rtol=1e-12, atol=1e-12)


def test_transposed_or_swapped_operands_would_fail():
    """A non-square, non-symmetric case: scores of query i against row j differ from j against i."""
    d = 3
    vec = np.array([[1, 2, 3], [0, 1, 0], [2, 0, 0], [0, 0, 5]], np.float32)
    q = np.array([[1, 0, 0], [0, 1, 1]], np.float32)
    ids = np.arange(4, dtype=np.int64)
    got_i, got_s = oracle.bruteforce(q, vec, "f32", ids, 4, oracle.IP)
    assert got_i.tolist() == [[2, 0, 1, 3], [0, 3, 1, 2]]
    assert got_s.tolist() == [[2, 1, 0, 0], [5, 5, 1, 0]]
    got_i, got_s = oracle.bruteforce(q, vec, "f32", ids, 4, oracle.L2)
    # q0=(1,0,0): d2 = [0+4+9, 1+1, 1, 1+25] = [13,2,1,26]; q1=(0,1,1): [1+1+4, 0+0+1, 4+1+1, 1+16] = [6,1,6,17]
    assert got_i.tolist() == [[2, 1, 0, 3], [1, 0, 2, 3]]
    assert got_s.tolist() == [[1, 2, 13, 26], [1, 6, 6, 17]]
    assert d == vec.shape[1]


# ---------------------------------------------------------------- IVF == brute force at nprobe = nlist
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_full_probe_equals_bruteforce(dtype, metric):
    n, d, nlist, k = 900, 16, 11, 12
    cent, off, stored, _, ids = _random_index(n, d, nlist, dtype, dup=True)
    q = RNG.standard_normal((17, d)).astype(np.float32)
    probe, got_i, got_s = oracle.ivf_search(q, cent, off, stored, dtype, ids, nlist, k, metric)
    bf_i, bf_s = oracle.bruteforce(q, stored, dtype, ids, k, metric)
    assert np.array_equal(got_i, bf_i)
    assert np.array_equal(got_s, bf_s)          # bitwise: same sums in the same order
    assert np.array_equal(np.sort(probe, 1), np.tile(np.arange(nlist), (17, 1)))


# ---------------------------------------------------------------- score function identities
def test_ip_l2_identity_and_scaling():
    n, d = 300, 40
    _, _, stored, vals, ids = _random_index(n, d, 3, "f32")
    q = RNG.standard_normal((7, d)).astype(np.float32)
    qi = np.repeat(np.arange(7), n)
    ri = np.tile(np.arange(n), 7)
    ip = oracle.pair_scores(q, stored, "f32", oracle.IP, qi, ri).reshape(7, n)
    l2 = oracle.pair_scores(q, stored, "f32", oracle.L2, qi, ri).reshape(7, n)
    qn = (q.astype(np.float64) ** 2).sum(1)[:, None]
    xn = (vals ** 2).sum(1)[None, :]
    np.testing.assert_allclose(ip, (qn + xn - l2) / 2, rtol=0, atol=1e-12 * (qn + xn).max())
    # unit vectors: ip = 1 - l2/2
    xu = (vals / np.sqrt(xn.T)).astype(np.float32)
    qu = (q / np.sqrt(qn)).astype(np.float32)
    ipu = oracle.pair_scores(qu, xu, "f32", oracle.IP, qi, ri)
    l2u = oracle.pair_scores(qu, xu, "f32", oracle.L2, qi, ri)
    np.testing.assert_allclose(ipu, 1 - l2u / 2, atol=5e-7)   # float32 normalisation error only
    # scaling the query by a power of two scales IP scores exactly and keeps the ids
    i1, s1 = oracle.bruteforce(q, stored, "f32", ids, 5, oracle.IP)
    i2, s2 = oracle.bruteforce(q * 4, stored, "f32", ids, 5, oracle.IP)
    assert np.array_equal(i1, i2) and np.array_equal(s1 * 4, s2)
    # L2 to itself is exactly zero and wins
    i3, s3 = oracle.bruteforce(stored[:5], stored, "f32", ids, 1, oracle.L2)
    assert np.array_equal(i3[:, 0], ids[:5]) and np.all(s3 == 0)


def test_database_permutation_invariance():
    n, d, nlist, k = 800, 20, 9, 10
    cent, off, stored, _, ids = _random_index(n, d, nlist, "f16")
    q = RNG.standard_normal((9, d)).astype(np.float32)
    p0, i0, s0 = oracle.ivf_search(q, cent, off, stored, "f16", ids, 4, k, oracle.L2)
    # permute the lists, and the rows inside every list, consistently
    lperm = RNG.permutation(nlist)
    rows = []
    for l in lperm:
        r = np.arange(off[l], off[l + 1])
        rows.append(RNG.permutation(r))
    rows = np.concatenate(rows)
    sizes = (off[1:] - off[:-1])[lperm]
    off2 = np.zeros(nlist + 1, np.int64)
    off2[1:] = np.cumsum(sizes)
    p1, i1, s1 = oracle.ivf_search(q, cent[lperm], off2, stored[rows], "f16", ids[rows], 4, k,
                                   oracle.L2)
    assert np.array_equal(i0, i1) and np.array_equal(s0, s1)
    assert np.array_equal(lperm[p1], p0)


# ---------------------------------------------------------------- probe selection
@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_probe_selection_properties(metric):
    n, d, nlist, k = 1200, 12, 14, 8
    cent, off, stored, vals, ids = _random_index(n, d, nlist, "f32")
    cent[5] = cent[2]                        # two identical centroids: lower index first
    q = RNG.standard_normal((11, d)).astype(np.float32)
    q64, c64 = q.astype(np.float64), cent.astype(np.float64)
    full = q64 @ c64.T if metric == oracle.IP else ((q64[:, None] - c64[None]) ** 2).sum(-1)
    best = full.argmax(1) if metric == oracle.IP else full.argmin(1)
    prev_probe, prev_kth = None, None
    for nprobe in range(1, nlist + 1):
        probe, sc = oracle.coarse(q, cent, nprobe, metric)
        if nprobe == 1:
            assert np.array_equal(probe[:, 0], best)        # argmax / argmin (first on ties)
        else:
            assert np.array_equal(probe[:, :-1], prev_probe)  # prefix property
        srt = -sc if metric == oracle.IP else sc
        assert np.all(np.diff(srt, axis=1) >= 0)
        np.testing.assert_allclose(sc, np.take_along_axis(full, probe.astype(np.int64), 1),
                                   rtol=1e-13, atol=1e-13)
        for r in range(q.shape[0]):                          # 2 before 5 whenever both appear
            row = probe[r].tolist()
            if 2 in row and 5 in row:
                assert row.index(5) == row.index(2) + 1
            else:
                assert 5 not in row or 2 in row
        _, out_i, out_s = oracle.ivf_search(q, cent, off, stored, "f32", ids, nprobe, k, metric)
        kth = out_s[:, -1]
        if prev_kth is not None:                             # k-th score never gets worse
            assert np.all(kth >= prev_kth) if metric == oracle.IP else np.all(kth <= prev_kth)
        prev_probe, prev_kth = probe, kth
        # candidate set: every id comes from a probed list, no duplicates
        row_of = {int(v): i for i, v in enumerate(ids)}
        for r in range(q.shape[0]):
            got = [int(v) for v in out_i[r] if v >= 0]
            assert len(set(got)) == len(got)
            avail = sum(off[l + 1] - off[l] for l in probe[r])
            assert len(got) == min(k, avail)
            for v in got:
                row = row_of[v]
                l = np.searchsorted(off, row, side="right") - 1
                assert l in probe[r]


# ---------------------------------------------------------------- ties and padding
def test_ties_lowest_id_and_padding():
    d = 4
    base = np.array([[1, 0, 0, 0], [0, 1, 0, 0], [0.5, 0.5, 0, 0]], np.float32)
    vec = np.concatenate([base, base, base])         # 9 rows, each vector three times
    ids = np.array([50, 7, 30, 2, 90, 31, 60, 8, 29], np.int64)
    off = np.array([0, 4, 4, 9], np.int64)           # list1 empty
    cent = np.array([[1, 0, 0, 0], [0, 0, 1, 0], [0, 1, 0, 0]], np.float32)
    q = np.array([[1, 0, 0, 0]], np.float32)
    i, s = oracle.bruteforce(q, vec, "f32", ids, 9, oracle.IP)
    assert i[0].tolist() == [2, 50, 60, 29, 30, 31, 7, 8, 90]
    assert s[0].tolist() == [1, 1, 1, .5, .5, .5, 0, 0, 0]
    # probing list0 only (rows 0..3: ids 50,7,30,2) with k=6: four results and padding
    _, i, s = oracle.ivf_search(q, cent, off, vec, "f32", ids, 1, 6, oracle.IP)
    assert i[0].tolist() == [2, 50, 30, 7, -1, -1]
    assert s[0].tolist() == [1, 1, .5, 0, -np.inf, -np.inf]
    # nprobe=2 picks centroid 0 then (tie between c1 and c2 at 0) centroid 1, which is empty
    p, i, s = oracle.ivf_search(q, cent, off, vec, "f32", ids, 2, 6, oracle.L2)
    assert p[0].tolist() == [0, 1]
    assert i[0].tolist() == [2, 50, 30, 7, -1, -1]
    assert s[0].tolist() == [0, 0, .5, 2, np.inf, np.inf]
    # skipped probe slots (negative list numbers) are ignored by the staged entry
    probe = np.array([[-1, 2, -1]], np.int32)
    i, s = oracle.scan(q, off, vec, "f32", ids, probe, 3, oracle.IP)
    assert i[0].tolist() == [60, 29, 31] and s[0].tolist() == [1, .5, .5]


def test_argument_errors():
    q = np.zeros((1, 2), np.float32)
    c = np.zeros((3, 2), np.float32)
    with pytest.raises(RuntimeError):
        oracle.coarse(q, c, 4, oracle.IP)            # nprobe > nlist
    with pytest.raises(RuntimeError):
        oracle.coarse(q, c, 1, 7)                    # unknown metric


def test_merge_of_two_partial_scans_is_the_scan_of_the_union():
    """Carrying a result across sub-stages: scanning two disjoint halves of the probe lists and
    merging equals scanning all of them (ids exactly, scores bitwise), also when a half finds
    fewer than k candidates."""
    rng = np.random.default_rng(77)
    n, d, nlist, nq = 900, 24, 30, 40
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[100:140] = x[60:100]                                   # equal scores across lists
    off = np.sort(np.concatenate([[0, n], rng.integers(0, n + 1, nlist - 1)])).astype(np.int64)
    ids = rng.permutation(n).astype(np.int64) * 5 + 3
    q = rng.standard_normal((nq, d)).astype(np.float32)
    probe = np.stack([rng.permutation(nlist)[:12] for _ in range(nq)]).astype(np.int32)
    probe[3, 7:] = -1
    for metric in (oracle.IP, oracle.L2):
        for k in (1, 7, 64):
            whole_i, whole_s = oracle.scan(q, off, x, "f32", ids, probe, k, metric)
            a_i, a_s = oracle.scan(q, off, x, "f32", ids, probe[:, :5], k, metric)
            b_i, b_s = oracle.scan(q, off, x, "f32", ids, probe[:, 5:], k, metric)
            m_i, m_s = oracle.merge_topk(a_i, a_s, b_i, b_s, k, metric)
            assert np.array_equal(m_i, whole_i)
            assert np.array_equal(m_s, whole_s)


# ---------------------------------------------------------------- reuse of the previous retrieval (Section 4.3)
def test_topk_of_rows_reduces_to_scan_and_to_bruteforce():
    """The k best of a set of rows: over the rows of the probed lists it is the scan, over all
    rows the exhaustive search (both are the C routines pinned above); rows named twice, -1 and
    rows past the end change nothing."""
    rng = np.random.default_rng(5)
    n, d, nlist, nq = 700, 20, 25, 30
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[50:80] = x[10:40]                                      # equal scores, decided by id
    off = np.sort(np.concatenate([[0, n], rng.integers(0, n + 1, nlist - 1)])).astype(np.int64)
    ids = rng.permutation(n).astype(np.int64) * 3 + 1
    q = rng.standard_normal((nq, d)).astype(np.float32)
    probe = np.stack([rng.permutation(nlist)[:9] for _ in range(nq)]).astype(np.int32)
    rows = [np.concatenate([np.arange(off[l], off[l + 1]) for l in probe[i]]) for i in range(nq)]
    noisy = [np.concatenate([r, r[::3], [-1, -7, n, n + 5]]) for r in rows]
    for metric in (oracle.IP, oracle.L2):
        for k in (1, 10, 200):
            s_i, s_s = oracle.scan(q, off, x, "f32", ids, probe, k, metric)
            t_i, t_s, t_r = oracle.topk_of_rows(q, x, "f32", ids, rows, k, metric)
            assert np.array_equal(t_i, s_i) and np.allclose(t_s, s_s, rtol=0, atol=1e-12)
            assert np.array_equal(ids[t_r[t_r >= 0]], t_i[t_i >= 0])
            u_i, u_s, _ = oracle.topk_of_rows(q, x, "f32", ids, noisy, k, metric)
            assert np.array_equal(u_i, s_i) and np.array_equal(u_s, t_s)
            b_i, b_s = oracle.bruteforce(q, x, "f32", ids, k, metric)
            a_i, a_s, _ = oracle.topk_of_rows(q, x, "f32", ids, [np.arange(n)] * nq, k, metric)
            assert np.array_equal(a_i, b_i) and np.allclose(a_s, b_s, rtol=0, atol=1e-12)
    e_i, e_s, e_r = oracle.topk_of_rows(q[:1], x, "f32", ids, [[-1]], 3, oracle.L2)
    assert (e_i == -1).all() and np.isinf(e_s).all() and (e_r == -1).all()


def test_lists_of_rows_against_a_walk_over_the_lists():
    off = np.array([0, 0, 4, 4, 4, 9, 10, 10], np.int64)      # empty lists at both ends and inside
    want = {}
    for l in range(len(off) - 1):
        for r in range(off[l], off[l + 1]):
            want[r] = l
    rows = np.array([-3, -1] + list(range(0, 12)), np.int64)
    got = oracle.lists_of_rows(rows, off)
    assert got.tolist() == [want.get(int(r), -1) for r in rows]


def test_reorder_probes_worked_example_and_invariants():
    """The three groups of Section 4.3 on an example worked by hand (tests/golden), and on
    random inputs: the output is the input rearranged, groups in order, given order kept inside
    each group (checked with numpy set operations, not with the oracle's own loops)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "reorder_worked_example.txt")
    vals = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            key, _, rest = line.partition(":")
            vals[key.strip()] = np.array([int(t) for t in rest.split()], np.int32)
    got = oracle.reorder_probes(vals["probe"][None], vals["prev"][None], vals["hot"][None])
    assert got[0].tolist() == vals["order"].tolist()
    # no history at all: nothing moves (except absent entries, which go last)
    assert oracle.reorder_probes(vals["probe"][None], None, None)[0].tolist() == \
        [int(x) for x in vals["probe"] if x >= 0] + [-1] * int((vals["probe"] < 0).sum())

    rng = np.random.default_rng(8)
    nq, nlist = 50, 90
    probe = np.stack([rng.permutation(nlist)[:40] for _ in range(nq)]).astype(np.int32)
    probe[rng.random(probe.shape) < 0.1] = -1
    prev = np.stack([rng.permutation(nlist)[:30] for _ in range(nq)]).astype(np.int32)
    prev[rng.random(prev.shape) < 0.1] = -1
    hot = rng.integers(-1, nlist, (nq, 7)).astype(np.int32)    # with repeats
    out = oracle.reorder_probes(probe, prev, hot)
    for i in range(nq):
        assert sorted(out[i].tolist()) == sorted(probe[i].tolist())
        group = np.where(out[i] < 0, 3, np.where(np.isin(out[i], hot[i][hot[i] >= 0]), 0,
                                                 np.where(np.isin(out[i], prev[i][prev[i] >= 0]), 1, 2)))
        assert (np.diff(group) >= 0).all()
        pos = {int(l): j for j, l in enumerate(probe[i]) if l >= 0}
        for gno in range(3):
            members = [pos[int(l)] for l in out[i][group == gno]]
            assert members == sorted(members)


def test_hot_lists_worked_example():
    """Counts 5 0 9 5 0 9 1: the two lists with 9 first (lower number first), then the two with
    5, then 1, then the never-probed ones in list order (worked by hand)."""
    hits = [5, 0, 9, 5, 0, 9, 1]
    assert oracle.hot_lists(hits, 7).tolist() == [2, 5, 0, 3, 6, 1, 4]
    assert oracle.hot_lists(hits, 3).tolist() == [2, 5, 0]



def test_split_probes_worked_example_and_invariants():
    """Partial residency (Section 4.4): a probe row split by hand (lists 3, 8 and 20 resident of 0..24: the row
    8 5 20 -1 3 30 11 gives 8 20 3 here and 5 11 elsewhere; 30 is no list at all), and on random inputs: the two parts
    are disjoint, together they are the valid entries of the row, each keeps the given order, the first holds
    exactly the resident ones (numpy set operations, not the oracle's own loops)."""
    resident = np.zeros(25, bool)
    resident[[3, 8, 20]] = True
    res, mis = oracle.split_probes(np.array([[8, 5, 20, -1, 3, 30, 11]], np.int32), resident)
    assert res[0].tolist() == [8, 20, 3, -1, -1, -1, -1] and mis[0].tolist() == [5, 11, -1, -1, -1, -1, -1]
    rng = np.random.default_rng(4)
    nlist = 60
    resident = rng.random(nlist) < 0.4
    probe = np.stack([rng.permutation(nlist + 6)[:25] - 3 for _ in range(40)]).astype(np.int32)    # some outside 0..nlist-1
    res, mis = oracle.split_probes(probe, resident)
    for i in range(probe.shape[0]):
        valid = probe[i][(probe[i] >= 0) & (probe[i] < nlist)]
        r, m = res[i][res[i] >= 0], mis[i][mis[i] >= 0]
        assert len(r) + len(m) == len(valid) and not np.intersect1d(r, m).size
        assert np.array_equal(r, valid[resident[valid]]) and np.array_equal(m, valid[~resident[valid]])
        assert (res[i][len(r):] == -1).all() and (mis[i][len(m):] == -1).all()


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The oracle's C code built with -fsanitize=address,undefined (host code only) and run on small inputs that
    reach its corners (oracle/sanitize_main.c): any out-of-bounds access, use after free or undefined arithmetic
    stops the run with a report."""
    import subprocess
    src = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "sanitize_main.c")
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe, src, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "oracle sanitize ok" in r.stdout, r.stdout + r.stderr
