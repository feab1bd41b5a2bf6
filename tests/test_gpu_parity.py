"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs (copied, not regenerated).  Tolerances: 1e-4 relative for float32 storage,
2e-3 for 16-bit storage (see compare.py for what "relative" is taken against); ids and probe
lists identical except at near-ties inside that tolerance."""
import os
import time

import numpy as np
import pytest
import torch

import oracle
import synth
from compare import TAU, check_probes, check_topk, floor_for

pytestmark = pytest.mark.gpu
METRIC = {"ip": oracle.IP, "l2": oracle.L2}


def _hr():
    import paper_2507_09138_amd as hr
    return hr


class Host:
    """Host copies of an index for the oracle."""

    def __init__(self, index):
        self.cfg = index.cfg
        self.cent = synth.to_numpy(index.centroids)
        self.off = synth.to_numpy(index.list_offsets)
        self.vec = synth.to_numpy(index.list_vectors)
        self.ids = synth.to_numpy(index.list_ids)
        self.row_of = {}
        self._inv = None

    def rows_of(self, ids):
        if self._inv is None:
            order = np.argsort(self.ids, kind="stable")
            self._sorted_ids = self.ids[order]
            self._inv = order
        pos = np.searchsorted(self._sorted_ids, ids)
        assert np.array_equal(self._sorted_ids[pos], ids)
        return self._inv[pos]

    def xnorm(self):
        n = min(4096, self.vec.shape[0])
        sel = np.linspace(0, self.vec.shape[0] - 1, n).astype(np.int64)
        v = self.vec[sel]
        if self.cfg.dtype == "bf16":
            v = (v.astype(np.uint32) << 16).view(np.float32)
        return float(np.sqrt((v.astype(np.float64) ** 2).sum(1)).mean())


def _scale(q, xn, metric):
    """floor * operand magnitude per query: below it score errors are judged absolutely"""
    qn = np.sqrt((q.astype(np.float64) ** 2).sum(1))
    return floor_for(q.shape[1]) * (qn * xn if metric == "ip" else qn ** 2 + xn ** 2)


def compare_all(index, queries, nprobe, k, metric, sample=None, label="", row_tables=False, host=None,
                floor_free=False, also_with_row_tables=False):
    """coarse vs oracle; scan (with the GPU's probe lists) vs oracle; search == coarse + scan.
    floor_free: no comparison may have been judged under the absolute floor of the comparator (the workload shapes:
    their scores are far above it, so the tolerance there is purely relative).  also_with_row_tables: the same
    queries through an index loaded with the derived row tables (HR_LOAD_ROW_TABLES), against the same oracle results
    (the coarse step does not depend on the tables, so the probe lists must be the same bits)."""
    hr = _hr()
    cfg = index.cfg
    tau = TAU[cfg.dtype]
    host = host or Host(index)
    ix = hr.IvfIndex(index.centroids, index.list_offsets, index.list_vectors, index.list_ids, row_tables=row_tables)
    q_dev = queries
    t0 = time.time()
    probe_g, pscore_g = ix.coarse(q_dev, nprobe, metric)
    ids_s, sc_s = ix.scan(q_dev, probe_g, k, metric)
    ids_f, sc_f = ix.search(q_dev, nprobe, k, metric)
    torch.cuda.synchronize()
    t_gpu = time.time() - t0
    st = ix.stats(q_dev.shape[0], nprobe, k)
    ix.close()
    probe_g, pscore_g = probe_g.cpu().numpy(), pscore_g.cpu().numpy()
    ids_s, sc_s = ids_s.cpu().numpy(), sc_s.cpu().numpy()
    ids_f, sc_f = ids_f.cpu().numpy(), sc_f.cpu().numpy()
    # the one-call path and the two staged calls are the same kernels: identical bits
    assert np.array_equal(ids_f, ids_s) and np.array_equal(sc_f, sc_s), "search != coarse+scan"
    q = synth.to_numpy(q_dev)
    sel = np.arange(q.shape[0]) if sample is None else np.asarray(sample)
    qs = np.ascontiguousarray(q[sel])
    m = METRIC[metric]
    cn = float(np.sqrt((host.cent.astype(np.float64) ** 2).sum(1)).mean())
    t0 = time.time()
    probe_o, pscore_o = oracle.coarse(qs, host.cent, nprobe, m)
    st_p = check_probes(probe_g[sel], pscore_g[sel], probe_o, pscore_o,
                        lambda i, c: oracle.pair_scores(qs, host.cent, "f32", m, np.full(len(c), i), c),
                        metric, TAU["f32"], _scale(qs, cn, metric))
    ids_o, sc_o = oracle.scan(qs, host.off, host.vec, cfg.dtype, host.ids,
                              np.ascontiguousarray(probe_g[sel]), k, m)
    score_of = lambda i, ids: oracle.pair_scores(qs, host.vec, cfg.dtype, m, np.full(len(ids), i), host.rows_of(ids))
    scale = _scale(qs, host.xnorm(), metric)
    st_k = check_topk(ids_s[sel], sc_s[sel], ids_o, sc_o, score_of, metric, tau, scale)
    # end to end against the unstaged oracle: how often is everything identical.  (Where the GPU's probe set is the
    # oracle's, the oracle's whole search is its scan of the GPU's probe lists: same candidates, same order; only
    # the other queries are searched again.)
    ids_e = ids_o.copy()
    other = np.nonzero((np.sort(probe_g[sel], 1) != np.sort(probe_o, 1)).any(1))[0]
    if len(other):
        _, ids_x, _ = oracle.ivf_search(np.ascontiguousarray(qs[other]), host.cent, host.off, host.vec, cfg.dtype, host.ids,
                                        nprobe, k, m)
        ids_e[other] = ids_x
    e2e = float((ids_e == ids_f[sel]).all(1).mean())
    t_or = time.time() - t0
    print(f"[parity {label or cfg.name}] nq={len(sel)} probes: {st_p} topk: {st_k} end-to-end exact rows: {e2e:.4f} "
          f"stats: {st} gpu {t_gpu:.2f}s oracle {t_or:.1f}s", flush=True)
    if floor_free:
        assert st_k["n_under_floor"] == 0, "a top-k comparison was judged under the absolute floor"
        assert st_p["n_under_floor"] == 0 or floor_free == "topk", "a probe comparison was judged under the absolute floor"
    if also_with_row_tables:
        ix = hr.IvfIndex(index.centroids, index.list_offsets, index.list_vectors, index.list_ids, row_tables=True)
        probe_n, _ = ix.coarse(q_dev, nprobe, metric)
        ids_n, sc_n = ix.scan(q_dev, probe_n, k, metric)
        torch.cuda.synchronize()
        ix.close()
        assert np.array_equal(probe_n.cpu().numpy(), probe_g), "probe lists depend on the row tables"
        st_n = check_topk(ids_n.cpu().numpy()[sel], sc_n.cpu().numpy()[sel], ids_o, sc_o, score_of, metric, tau, scale)
        print(f"[parity {label or cfg.name}, with row tables] topk: {st_n}", flush=True)
        if floor_free:
            assert st_n["n_under_floor"] == 0
        return st_p, st_k, e2e, st_n
    return st_p, st_k, e2e


def _random_index(n, d, nlist, dtype, seed, dup=1, empty=True, device="cuda"):
    """Unclustered random data: candidates everywhere, many insertions, ragged lists."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    base = torch.randn(n // dup, d, generator=g)
    x = base.repeat(dup, 1)[torch.randperm(n // dup * dup, generator=g)]
    n = x.shape[0]
    cent = torch.randn(nlist, d, generator=g)
    cuts = torch.sort(torch.randint(0, n + 1, (nlist - 1,), generator=g)).values
    off = torch.cat([torch.zeros(1, dtype=torch.int64), cuts, torch.tensor([n])])
    if empty and nlist > 2:
        off[2] = off[1]                      # list 1 is empty
    ids = torch.randperm(n, generator=g) * 3 + 7
    cfg = synth.Config("rand", n, d, nlist, "uniform", 0, False, dtype, "ip", 0, "uniform", 0, 0, 0)
    return synth.Index(cfg, cent.to(device), off, x.to(synth.TORCH_DTYPE[dtype]).to(device), ids.to(device),
                       torch.arange(nlist))


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_random_small(dtype, metric):
    print(f"case random_small {dtype} {metric}", flush=True)
    idx = _random_index(6000, 128, 37, dtype, seed=11)
    g = torch.Generator(device="cpu").manual_seed(5)
    q = torch.randn(150, 128, generator=g).cuda()
    compare_all(idx, q, nprobe=9, k=10, metric=metric)


@pytest.mark.parametrize("d", [64, 256, 512, 1024])
def test_dimensions(d):
    print(f"case dimensions d={d}", flush=True)
    idx = _random_index(3000, d, 19, "f16", seed=d)
    g = torch.Generator(device="cpu").manual_seed(6)
    q = torch.randn(70, d, generator=g).cuda()
    compare_all(idx, q, nprobe=5, k=7, metric="ip")
    idx = _random_index(3000, d, 19, "f32", seed=d + 1)
    compare_all(idx, q, nprobe=5, k=7, metric="l2")


@pytest.mark.parametrize("nprobe,k", [(1, 1), (37, 128), (37, 3), (2, 100)])
def test_extreme_k_and_nprobe(nprobe, k):
    print(f"case extreme nprobe={nprobe} k={k}", flush=True)
    idx = _random_index(5000, 64, 37, "f16", seed=23)
    g = torch.Generator(device="cpu").manual_seed(7)
    q = torch.randn(65, 64, generator=g).cuda()
    compare_all(idx, q, nprobe=nprobe, k=k, metric="ip")       # k > candidates for some: padding
    idx = _random_index(5000, 64, 37, "bf16", seed=24)
    compare_all(idx, q, nprobe=nprobe, k=k, metric="l2")


def test_nprobe_max_many_lists():
    print("case nprobe=128 over 300 lists", flush=True)
    idx = _random_index(20000, 64, 300, "f16", seed=29)
    g = torch.Generator(device="cpu").manual_seed(8)
    q = torch.randn(33, 64, generator=g).cuda()
    compare_all(idx, q, nprobe=128, k=20, metric="ip")


@pytest.mark.parametrize("nlist", [5000, 20000])
def test_many_short_lists(nlist):
    """More lists than the grouping kernel's one workgroup has threads: 5 and 20 lists per thread (the second
    beyond what a thread keeps in registers), many of them empty or shorter than k."""
    print(f"case {nlist} lists of 2.5 rows on average", flush=True)
    idx = _random_index(nlist * 5 // 2, 64, nlist, "f16", seed=41)
    g = torch.Generator(device="cpu").manual_seed(11)
    q = torch.randn(70, 64, generator=g).cuda()
    compare_all(idx, q, nprobe=200, k=10, metric="ip")
    compare_all(idx, q, nprobe=17, k=3, metric="l2")


def test_nprobe_512_paper_range():
    """The paper probes 128 to 512 clusters with k = 1 (Section 6.1): nprobe 512 over 700 lists."""
    print("case nprobe=512 over 700 lists, k=1", flush=True)
    idx = _random_index(30000, 64, 700, "f16", seed=37)
    g = torch.Generator(device="cpu").manual_seed(10)
    q = torch.randn(21, 64, generator=g).cuda()
    compare_all(idx, q, nprobe=512, k=1, metric="l2")
    compare_all(idx, q, nprobe=256, k=5, metric="ip")


def test_duplicates_lowest_id_wins_exactly():
    """Every vector is stored four times: equal scores; the ids must be the oracle's exactly."""
    print("case duplicates", flush=True)
    hr = _hr()
    idx = _random_index(4000, 64, 5, "f32", seed=31, dup=4, empty=False)
    g = torch.Generator(device="cpu").manual_seed(9)
    q = torch.randn(120, 64, generator=g).cuda()
    host = Host(idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    for metric in ("ip", "l2"):
        for k in (2, 6, 11):
            ids, sc = ix.search(q, 5, k, metric)
            _, ids_o, sc_o = oracle.ivf_search(synth.to_numpy(q), host.cent, host.off, host.vec, "f32", host.ids,
                                               5, k, METRIC[metric])
            assert np.array_equal(ids.cpu().numpy(), ids_o), f"{metric} k={k}"
            np.testing.assert_allclose(sc.cpu().numpy(), sc_o, rtol=1e-4, atol=1e-4)
    ix.close()


def test_coarse_duplicate_centroids_lower_index_first():
    """Every centroid appears three times: equal coarse scores; the probe lists must be the
    oracle's exactly (lower centroid index first), for odd table sizes and nprobe up to nlist."""
    print("case duplicate centroids", flush=True)
    hr = _hr()
    g = torch.Generator(device="cpu").manual_seed(41)
    for nbase, d, nprobes in ((7, 64, (1, 5, 21)), (67, 128, (3, 64, 128)), (43, 256, (129 - 1, 2))):
        base = torch.randn(nbase, d, generator=g)
        cent = base.repeat(3, 1)[torch.randperm(3 * nbase, generator=g)].contiguous()
        nlist = cent.shape[0]
        n = nlist * 5
        x = torch.randn(n, d, generator=g)
        off = torch.arange(0, n + 1, 5, dtype=torch.int64)
        ids = torch.arange(n, dtype=torch.int64)
        q = torch.randn(77, d, generator=g)
        ix = hr.IvfIndex(cent.cuda(), off, x.cuda(), ids.cuda())
        for metric in ("ip", "l2"):
            for nprobe in nprobes:
                nprobe = min(nprobe, nlist)
                probe, score = ix.coarse(q.cuda(), nprobe, metric)
                probe_o, score_o = oracle.coarse(q.numpy(), cent.numpy(), nprobe, METRIC[metric])
                assert np.array_equal(probe.cpu().numpy(), probe_o), f"nlist={nlist} {metric} nprobe={nprobe}"
                np.testing.assert_allclose(score.cpu().numpy(), score_o, rtol=1e-4, atol=1e-4)
        ix.close()


def test_coarse_in_chunks_of_queries():
    """More queries than one chunk of the coarse key table holds (512 MiB / (4 nlist) = 32768 at
    nlist = 4096): every chunk, and the ragged last one, against the oracle."""
    print("case coarse chunks", flush=True)
    hr = _hr()
    g = torch.Generator(device="cpu").manual_seed(43)
    nlist, d, nq = 4096, 64, 32768 + 32768 + 333
    cent = torch.randn(nlist, d, generator=g)
    x = torch.randn(nlist, d, generator=g).to(torch.float16)
    off = torch.arange(0, nlist + 1, dtype=torch.int64)
    ids = torch.arange(nlist, dtype=torch.int64)
    q = torch.randn(nq, d, generator=g)
    ix = hr.IvfIndex(cent.cuda(), off, x.cuda(), ids.cuda())
    probe, score = ix.coarse(q.cuda(), 16, "ip")
    probe, score = probe.cpu().numpy(), score.cpu().numpy()
    sel = np.concatenate([np.arange(0, 40), np.arange(32740, 32800), np.arange(65510, 65560), np.arange(nq - 40, nq)])
    qs = np.ascontiguousarray(q.numpy()[sel])
    probe_o, score_o = oracle.coarse(qs, cent.numpy(), 16, oracle.IP)
    cn = float(np.sqrt((cent.numpy().astype(np.float64) ** 2).sum(1)).mean())
    st = check_probes(probe[sel], score[sel], probe_o, score_o,
                      lambda i, c: oracle.pair_scores(qs, cent.numpy(), "f32", oracle.IP, np.full(len(c), i), c),
                      "ip", TAU["f32"], _scale(qs, cn, "ip"))
    print(f"[parity coarse chunks] {st}", flush=True)
    ix.close()


@pytest.mark.parametrize("dtype,metric", [("f16", "ip"), ("f32", "l2"), ("bf16", "l2")])
def test_scan_in_steps_with_carried_result(dtype, metric):
    """A retrieval split into sub-stages: the probe lists of every query are searched in four
    steps (ragged: some places empty), the result carried from step to step.  The final result
    must be that of one scan over all the lists: against the oracle's scan of the union, and,
    for the inner product (a carried score is the key itself), bit for bit against the GPU's own
    one-call scan.  A step that leaves fewer than k candidates carries empty places."""
    print(f"case steps {dtype} {metric}", flush=True)
    hr = _hr()
    idx = _random_index(24000, 128, 60, dtype, seed=51)
    host = Host(idx)
    g = torch.Generator(device="cpu").manual_seed(12)
    nq, nprobe, k = 150, 24, 40
    q = torch.randn(nq, 128, generator=g).cuda()
    probe = torch.stack([torch.randperm(60, generator=g)[:nprobe] for _ in range(nq)]).to(torch.int32)
    probe[5, 3:] = -1                       # three lists in all for this query
    probe[6, :] = -1                        # none at all
    probe[7, 1::2] = -1                     # holes
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    state = ix.new_state(nq, k)
    for s0 in range(0, nprobe, 6):
        ix.scan_step(q, probe[:, s0:s0 + 6].cuda(), state, metric)
    ids_st, sc_st = state[0].cpu().numpy(), state[1].cpu().numpy()
    ids_1, sc_1 = ix.scan(q, probe.cuda(), k, metric)
    ids_1, sc_1 = ids_1.cpu().numpy(), sc_1.cpu().numpy()
    qn = synth.to_numpy(q)
    m = METRIC[metric]
    ids_o, sc_o = oracle.scan(qn, host.off, host.vec, dtype, host.ids, probe.numpy(), k, m)
    st = check_topk(ids_st, sc_st, ids_o, sc_o,
                    lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, m, np.full(len(ids), i), host.rows_of(ids)),
                    metric, TAU[dtype], _scale(qn, host.xnorm(), metric))
    print(f"[parity steps {dtype} {metric}] {st} same as one call: {float((ids_st == ids_1).all(1).mean()):.4f}", flush=True)
    assert (ids_st[6] == -1).all() and (ids_1[6] == -1).all()
    if metric == "ip":
        assert np.array_equal(ids_st, ids_1) and np.array_equal(sc_st, sc_1)
    else:
        assert (ids_st == ids_1).all(1).mean() > 0.98
    ix.close()


def test_list_access_counters():
    """Per-list access frequency (what a cache of hot clusters is driven by): after some calls
    the counters equal the histogram of all probe lists used, exactly; empty places are not
    counted; a reset starts again from zero."""
    print("case access counters", flush=True)
    hr = _hr()
    idx = _random_index(9000, 64, 40, "f16", seed=61)
    g = torch.Generator(device="cpu").manual_seed(14)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    assert int(ix.list_hits().sum()) == 0
    want = np.zeros(40, np.int64)
    for nq, nprobe in ((50, 7), (130, 12)):
        q = torch.randn(nq, 64, generator=g).cuda()
        probe, _ = ix.coarse(q, nprobe, "ip")            # (the coarse step alone counts nothing)
        ix.search(q, nprobe, 5, "ip")
        want += np.bincount(probe.cpu().numpy().ravel(), minlength=40)
    pr = torch.stack([torch.randperm(40, generator=g)[:6] for _ in range(33)]).to(torch.int32)
    pr[4, 2:] = -1
    q = torch.randn(33, 64, generator=g).cuda()
    ix.scan(q, pr.cuda(), 3, "l2")
    want += np.bincount(pr.numpy()[pr.numpy() >= 0], minlength=40)
    got = ix.list_hits(reset=True).cpu().numpy()
    assert np.array_equal(got, want), (got, want)
    assert int(ix.list_hits().sum()) == 0
    ix.close()


def test_variable_length_probe_lists_and_empty_batch():
    print("case variable-length probes", flush=True)
    hr = _hr()
    idx = _random_index(5000, 64, 23, "f16", seed=37)
    host = Host(idx)
    g = torch.Generator(device="cpu").manual_seed(10)
    q = torch.randn(90, 64, generator=g).cuda()
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    probe = torch.stack([torch.randperm(23, generator=g)[:8] for _ in range(90)]).to(torch.int32)
    drop = torch.rand(90, 8, generator=g) < 0.4
    probe[drop] = -1
    probe[3] = -1                                 # a query with nothing to search
    probe[4, 0] = 1000                            # out of range = skipped
    ids, sc = ix.scan(q, probe.cuda(), 10, "ip")
    ids_o, sc_o = oracle.scan(synth.to_numpy(q), host.off, host.vec, "f16", host.ids, probe.numpy(), 10, oracle.IP)
    qn = synth.to_numpy(q)
    check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o,
               lambda i, v: oracle.pair_scores(qn, host.vec, "f16", oracle.IP, np.full(len(v), i), host.rows_of(v)),
               "ip", TAU["f16"], _scale(qn, host.xnorm(), "ip"))
    assert (ids[3] == -1).all() and torch.isinf(sc[3]).all()
    # nq = 0 is a no-op
    e_ids, e_sc = ix.search(q[:0], 4, 5, "ip")
    assert e_ids.shape == (0, 5)
    ix.close()


def test_errors_and_determinism():
    print("case errors + determinism", flush=True)
    hr = _hr()
    idx = _random_index(3000, 64, 11, "f16", seed=41)
    g = torch.Generator(device="cpu").manual_seed(12)
    q = torch.randn(40, 64, generator=g).cuda()
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    ids = torch.full((40, 5), 12345, dtype=torch.int64, device="cuda")
    sc = torch.zeros(40, 5, device="cuda")
    ws = ix.workspace(40, 4, 5)
    for args, code in [((12, 5), -1), ((0, 5), -1), ((4, 0), -1), ((4, hr.HR_K_MAX + 1), -1)]:
        with pytest.raises(hr.HrError) as e:
            hr.hr_ivf_search(ix.handle, q, 40, args[0], args[1], 0, ids, sc, ws, ws.numel())
        assert e.value.code == code
    with pytest.raises(hr.HrError) as e:
        hr.hr_ivf_search(ix.handle, q, 40, 4, 5, 0, ids, sc, ws, 1024)
    assert e.value.code == -3
    with pytest.raises(hr.HrError) as e:
        hr.hr_ivf_search(ix.handle, q, 40, 4, 5, 7, ids, sc, ws, ws.numel())
    assert e.value.code == -1
    torch.cuda.synchronize()
    assert (ids == 12345).all()                   # nothing was enqueued
    a = ix.search(q, 4, 5, "l2")
    b = ix.search(q, 4, 5, "l2")
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    h = ix.handle
    ix.close()
    with pytest.raises(hr.HrError) as e:
        hr.hr_ivf_free(h)
    assert e.value.code == -2


# ---------------------------------------------------------------- the five workload shapes
# Floors asserted below on the share of rows with identical ids / of identical id sets are the rates of earlier runs
# less a margin: a drop in id agreement that stays inside the score tolerance would otherwise pass unnoticed.
def _run_config(name, sample=None, **kw):
    scale = {a: b for a, b in kw.items() if a not in ("also_with_row_tables", "floor_free")}
    cfg = synth.CONFIGS[name]
    if scale:
        cfg = synth.scaled(cfg, **scale)
    print(f"case config {name} {scale or 'full size'}", flush=True)
    idx = synth.make_index(cfg, "cuda")
    host = Host(idx)
    rounds = synth.make_queries(cfg, idx)
    out = []
    for r, q in enumerate(rounds):
        sel = None
        if sample is not None:
            gs = np.random.default_rng(99 + r)
            sel = np.sort(gs.choice(q.shape[0], size=min(sample, q.shape[0]), replace=False))
        out.append(compare_all(idx, q, cfg.nprobe, cfg.k, cfg.metric, sample=sel, host=host, floor_free=kw.get("floor_free", True),
                               also_with_row_tables=kw.get("also_with_row_tables", False),
                               label=f"{name} round {r}" if len(rounds) > 1 else name))
    return out


def test_config1_tiny_fp32_full():
    (st_p, st_k, e2e, st_t), = _run_config("C1", also_with_row_tables=True)
    assert st_p["exact_set_rate"] >= 0.98 and st_k["exact_id_rows"] >= 0.98 and st_t["exact_id_rows"] >= 0.98


def test_config2_medium_fp32_full_size():
    (st_p, st_k, e2e, st_t), = _run_config("C2", also_with_row_tables=True)
    assert st_p["exact_set_rate"] >= 0.98 and st_k["exact_id_rows"] >= 0.98 and st_t["exact_id_rows"] >= 0.98


def test_config3_skewed_fp16_scaled():
    (st_p, st_k, e2e), = _run_config("C3", N=262144, nlist=256, nq=1024, nprobe=32)
    assert st_p["exact_set_rate"] >= 0.95 and st_k["id_set_overlap"] >= 0.99


def test_config3_skewed_fp16_full_size_sampled():
    (st_p, st_k, e2e), = _run_config("C3", sample=768)
    assert st_p["exact_set_rate"] >= 0.95 and st_k["exact_id_rows"] >= 0.5 and st_k["id_set_overlap"] >= 0.99


def test_config4_iterative_fp16_scaled_rounds():
    out = _run_config("C4", N=262144, nlist=256, nq=128, nprobe=16)
    assert len(out) == 8


def test_config4_iterative_fp16_full_size_sampled():
    """The multi-hop workload at its stated size: the index of the skewed workload (same bytes), eight rounds of 512
    drifting queries, nprobe 32, every round one batch; 128 sampled queries of every round against the oracle."""
    out = _run_config("C4", sample=128)
    assert len(out) == 8
    for st_p, st_k, e2e in out:
        assert st_p["exact_set_rate"] >= 0.95 and st_k["exact_id_rows"] >= 0.5 and st_k["id_set_overlap"] >= 0.99


def test_config5_large_bf16_l2_scaled():
    (st_p, st_k, e2e, st_n), = _run_config("C5", N=524288, nlist=512, nq=512, nprobe=64, also_with_row_tables=True)
    assert st_k["id_set_overlap"] >= 0.9995 and st_k["exact_id_rows"] >= 0.7 and st_n["id_set_overlap"] >= 0.998


@pytest.mark.skipif(os.environ.get("HR_SKIP_C5_FULL") == "1", reason="HR_SKIP_C5_FULL=1")
def test_config5_large_bf16_l2_full_size_sampled():
    """Consecutive neighbour distances of this workload differ by 2.8e-4 of their value in the median.  As loaded by
    default (bfloat16 rows times the query in bfloat16 hi + lo parts, error ~5e-6) the 100 ids are the oracle's in the
    oracle's order in most rows and the id sets agree to 99.99 %.  With the binary16 row table the query is rounded to
    binary16 once (error ~1.7e-4, inside the 2e-3 tolerance but the size of those gaps): neighbours swap places in
    nearly every row, and what must hold is that the set of ids is the oracle's (99.9 %; floor 99.8 %)."""
    (st_p, st_k, e2e, st_n), = _run_config("C5", sample=512, also_with_row_tables=True)
    assert st_p["exact_set_rate"] >= 0.95
    assert st_k["id_set_overlap"] >= 0.9995 and st_k["exact_id_rows"] >= 0.7 and st_n["id_set_overlap"] >= 0.998


def test_paper_shape_scaled():
    """d = 1024, nprobe 128, top-1, a small batch (the paper's own parameters, Section 6.1) on a small index"""
    # (128 of 512 lists: the last centroids chosen are nearly orthogonal to the query, their scores are a cancellation
    # and are judged under the comparator's absolute floor; at full size, 128 of 4096, they are not)
    (st_p, st_k, e2e), = _run_config("P1", N=1 << 20, nlist=512, nq=96, floor_free="topk")
    assert st_k["exact_id_rows"] >= 0.98


@pytest.mark.skipif(os.environ.get("HR_SKIP_P1_FULL") == "1", reason="HR_SKIP_P1_FULL=1 (77 GB index, 80 GB of host memory)")
def test_paper_shape_full_size_sampled():
    (st_p, st_k, e2e), = _run_config("P1", sample=96)
    assert st_k["exact_id_rows"] >= 0.95


# ---------------------------------------------------------------- reuse of the previous retrieval (Section 4.3)
def test_reorder_probes_exact():
    """Integer work: identical to the oracle, at the size limits and with absent entries."""
    hr = _hr()
    rng = np.random.default_rng(31)
    for nq, nlist, np_, pp, nh in [(70, 900, 512, 512, 128), (33, 40, 5, 0, 3), (9, 64, 64, 17, 0), (5, 10, 3, 0, 0),
                                   (130, 200, 37, 64, 20)]:
        print(f"case reorder nq={nq} nprobe={np_} nprev={pp} nhot={nh}", flush=True)
        probe = np.stack([rng.permutation(nlist)[:np_] for _ in range(nq)]).astype(np.int32)
        probe[rng.random(probe.shape) < 0.08] = -1
        prev = np.stack([rng.permutation(nlist)[:pp] for _ in range(nq)]).astype(np.int32) if pp else None
        if prev is not None:
            prev[rng.random(prev.shape) < 0.08] = -1
        hot = rng.integers(-1, nlist, (nq, nh)).astype(np.int32) if nh else None
        got = hr.reorder_probes(torch.from_numpy(probe).cuda(),
                                torch.from_numpy(prev).cuda() if prev is not None else None,
                                torch.from_numpy(hot).cuda() if hot is not None else None).cpu().numpy()
        assert np.array_equal(got, oracle.reorder_probes(probe, prev, hot))


def test_lists_of_rows_exact():
    hr = _hr()
    idx = _random_index(5000, 64, 37, "f16", seed=3)          # (with empty lists)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    rows = np.concatenate([np.arange(-3, 5003), np.random.default_rng(1).integers(0, 5000, 999)]).astype(np.int32)
    got = ix.lists_of_rows(torch.from_numpy(rows).cuda()).cpu().numpy()
    assert np.array_equal(got, oracle.lists_of_rows(rows, synth.to_numpy(idx.list_offsets)))
    ix.close()


@pytest.mark.parametrize("dtype,metric", [("f16", "ip"), ("f16", "l2"), ("bf16", "l2"), ("f32", "ip"), ("f32", "l2")])
def test_rescore_of_cached_rows(dtype, metric):
    """The local cache: k best of m given rows per query against the oracle's top-k of those rows
    (rows named twice, absent and out-of-range rows; fewer rows than k; m and k at their limits)."""
    print(f"case rescore {dtype} {metric}", flush=True)
    hr = _hr()
    n, d = 9000, 256
    idx = _random_index(n, d, 20, dtype, seed=17, dup=3)
    host = Host(idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    rng = np.random.default_rng(23)
    m_ = METRIC[metric]
    for nq, m, k in [(101, 20, 10), (40, 5, 10), (37, 128, 128), (64, 64, 1)]:
        q = torch.randn(nq, d, generator=torch.Generator().manual_seed(nq)).cuda()
        rows = rng.integers(0, n, (nq, m)).astype(np.int32)
        rows[rng.random(rows.shape) < 0.1] = -1
        rows[0, :] = -1                                   # nothing cached for this query
        if m > 3:
            rows[1, 1] = rows[1, 0]; rows[1, 3] = rows[1, 0]; rows[2, 2] = n + 4
        ids_g, sc_g, rows_g = [t.cpu().numpy() for t in ix.rescore(q, torch.from_numpy(rows).cuda(), k, metric)]
        qn = synth.to_numpy(q)
        ids_o, sc_o, rows_o = oracle.topk_of_rows(qn, host.vec, dtype, host.ids, list(rows), k, m_)
        st = check_topk(ids_g, sc_g, ids_o, sc_o,
                        lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, m_, np.full(len(ids), i), host.rows_of(ids)),
                        metric, TAU[dtype], _scale(qn, host.xnorm(), metric))
        print(f"[parity rescore {dtype} {metric} m={m} k={k}] {st}", flush=True)
        assert (ids_g[0] == -1).all() and (rows_g[0] == -1).all()
        assert ((ids_g >= 0) == (ids_o >= 0)).all()        # same number of entries per query
        have = ids_g >= 0
        assert np.array_equal(host.ids[rows_g[have]], ids_g[have])      # rows and ids name the same vectors
        for i in range(nq):                                # every row reported once
            r = rows_g[i][rows_g[i] >= 0]
            assert len(np.unique(r)) == len(r)
    ix.close()


def test_scan_step_rows_carries_rows():
    """The carried result with row numbers: same ids and scores as without, rows name the vectors."""
    hr = _hr()
    idx = _random_index(20000, 128, 50, "f16", seed=29)
    host = Host(idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    g = torch.Generator().manual_seed(4)
    nq, nprobe, k = 90, 20, 30
    q = torch.randn(nq, 128, generator=g).cuda()
    probe = torch.stack([torch.randperm(50, generator=g)[:nprobe] for _ in range(nq)]).to(torch.int32)
    probe[3, 2:] = -1
    a = ix.new_state(nq, k)
    b = ix.new_state_rows(nq, k)
    for s0 in range(0, nprobe, 5):
        ix.scan_step(q, probe[:, s0:s0 + 5].cuda(), a, "ip")
        ix.scan_step_rows(q, probe[:, s0:s0 + 5].cuda(), b, "ip")
    ids_a, sc_a = a[0].cpu().numpy(), a[1].cpu().numpy()
    ids_b, sc_b, rows_b = b[0].cpu().numpy(), b[1].cpu().numpy(), b[2].cpu().numpy()
    assert np.array_equal(ids_a, ids_b) and np.array_equal(sc_a, sc_b)
    have = ids_b >= 0
    assert ((rows_b >= 0) == have).all()
    assert np.array_equal(host.ids[rows_b[have]], ids_b[have])
    ix.close()


@pytest.mark.parametrize("dtype,metric", [("f16", "ip"), ("bf16", "l2"), ("f32", "l2")])
def test_retrieval_started_from_the_cache_of_the_previous_one(dtype, metric):
    """Two consecutive retrievals of the same requests (the second query drifted a little): the
    second starts from the 20 cached rows of the first, searches its lists in the order of
    Section 4.3, in sub-stages; rows the cache already gave are found again by the scan and
    must not be reported twice.  Expected: the oracle's k best over the union of the cached
    rows and the rows of all probed lists."""
    print(f"case cache {dtype} {metric}", flush=True)
    hr = _hr()
    cfg = synth.scaled(synth.CONFIGS["C4"], N=60000, nlist=96, nq=120, nprobe=16, k=10, rounds=2, dtype=dtype,
                       metric=metric, d=128)
    idx = synth.make_index(cfg, "cuda")
    v, v2 = synth.make_queries(cfg, idx)
    host = Host(idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    nq, k, big = cfg.nq, cfg.k, 20
    # first retrieval, keeping the 20 best with their rows
    probe1, _ = ix.coarse(v, cfg.nprobe, metric)
    st1 = ix.new_state_rows(nq, big)
    ix.scan_step_rows(v, probe1, st1, metric)
    cache = st1[2].clone()
    hot = ix.lists_of_rows(st1[2][:, :k])                      # H_v: where the k best of v were
    # second retrieval
    probe2, _ = ix.coarse(v2, cfg.nprobe, metric)
    order = hr.reorder_probes(probe2, probe1, hot)
    assert np.array_equal(order.cpu().numpy(),
                          oracle.reorder_probes(probe2.cpu().numpy(), probe1.cpu().numpy(), hot.cpu().numpy()))
    st2 = ix.rescore(v2, cache, k, metric)
    for s0 in range(0, cfg.nprobe, 4):
        ix.scan_step_rows(v2, order[:, s0:s0 + 4].contiguous(), st2, metric)
    ids_g, sc_g, rows_g = [t.cpu().numpy() for t in st2]
    qn = synth.to_numpy(v2)
    p2 = probe2.cpu().numpy()
    cache_h = cache.cpu().numpy()
    union = [np.concatenate([cache_h[i]] + [np.arange(host.off[l], host.off[l + 1]) for l in p2[i]]) for i in range(nq)]
    m_ = METRIC[metric]
    ids_o, sc_o, _ = oracle.topk_of_rows(qn, host.vec, dtype, host.ids, union, k, m_)
    st = check_topk(ids_g, sc_g, ids_o, sc_o,
                    lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, m_, np.full(len(ids), i), host.rows_of(ids)),
                    metric, TAU[dtype], _scale(qn, host.xnorm(), metric))
    inside = float(np.mean([np.isin(ids_o[i], st1[0][i].cpu().numpy()).all() for i in range(nq)]))
    print(f"[parity cache {dtype} {metric}] {st}; results of v' all inside the 20 cached of v: {inside:.2f}", flush=True)
    for i in range(nq):
        assert len(np.unique(ids_g[i])) == k                # k distinct vectors
    assert np.array_equal(host.ids[rows_g], ids_g)
    ix.close()


def test_search_captured_in_a_hip_graph_replays_identically():
    """The search only enqueues kernels (no allocation, no host synchronisation, no memset
    nodes), so a caller can capture it in a HIP graph and replay it for launch-bound small
    batches.  Replayed several times with new queries in the same buffers and eager work in
    between; every replay must give the bits of the eager call."""
    hr = _hr()
    idx = _random_index(30000, 128, 64, "f16", seed=61)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    nq, nprobe, k = 48, 8, 10
    gen = torch.Generator().manual_seed(9)
    batches = [torch.randn(nq, 128, generator=gen).cuda() for _ in range(4)]
    q = batches[0].clone()
    ids = torch.empty(nq, k, dtype=torch.int64, device="cuda")
    scores = torch.empty(nq, k, dtype=torch.float32, device="cuda")
    ws = ix.workspace(nq, nprobe, k)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        hr.hr_ivf_search(ix.handle, q, nq, nprobe, k, hr.HR_METRIC_IP, ids, scores, ws, ws.numel())    # warm-up, eager
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        hr.hr_ivf_search(ix.handle, q, nq, nprobe, k, hr.HR_METRIC_IP, ids, scores, ws, ws.numel())
    for r, b in enumerate(batches):
        want_ids, want_scores = ix.search(b, nprobe, k, "ip")              # eager, own buffers
        torch.cuda.synchronize()
        q.copy_(b)
        ids.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids, want_ids) and torch.equal(scores, want_scores), f"replay {r}"
    ix.close()


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_float32_lists_with_and_without_row_tables(metric):
    """float32 lists are split on the fly into binary16 hi and lo parts, or, when the caller asked for
    row tables at load, scanned from tables of those parts: the same products in the same order, so
    the results must be the same bits; the on-the-fly path is checked against the oracle as well."""
    print(f"case f32 row tables {metric}", flush=True)
    hr = _hr()
    idx = _random_index(40000, 256, 48, "f32", seed=71, dup=2)
    host = Host(idx)
    a = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=True)
    b = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=False)
    q = torch.randn(300, 256, generator=torch.Generator().manual_seed(2)).cuda()
    m = METRIC[metric]
    for nprobe, k in [(12, 10), (7, 100)]:
        ids_a, sc_a = a.search(q, nprobe, k, metric)
        ids_b, sc_b = b.search(q, nprobe, k, metric)
        assert torch.equal(ids_a, ids_b) and torch.equal(sc_a, sc_b)
        probe, _ = b.coarse(q, nprobe, metric)
        qn = synth.to_numpy(q)
        ids_o, sc_o = oracle.scan(qn, host.off, host.vec, "f32", host.ids, probe.cpu().numpy(), k, m)
        st = check_topk(ids_b.cpu().numpy(), sc_b.cpu().numpy(), ids_o, sc_o,
                        lambda i, ids: oracle.pair_scores(qn, host.vec, "f32", m, np.full(len(ids), i), host.rows_of(ids)),
                        metric, TAU["f32"], _scale(qn, host.xnorm(), metric))
        print(f"[parity f32 on the fly {metric} nprobe={nprobe} k={k}] {st}", flush=True)
    a.close()
    b.close()


def test_hot_lists_by_access_counters():
    """The most frequently probed lists, exactly as the oracle orders the counters (many lists
    tie at zero and at small counts)."""
    hr = _hr()
    idx = _random_index(20000, 64, 700, "f16", seed=5)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    g = torch.Generator().manual_seed(3)
    for nq, nprobe in ((40, 9), (111, 5)):
        ix.search(torch.randn(nq, 64, generator=g).cuda(), nprobe, 4, "ip")
    hits = ix.list_hits().cpu().numpy()
    assert (hits == 0).sum() > 50 and hits.max() > 1
    for gc in (1, 10, 256, 257, 700):
        assert np.array_equal(ix.hot_lists(gc).cpu().numpy(), oracle.hot_lists(hits, gc))
    with pytest.raises(hr.HrError):
        ix.hot_lists(701)
    ix.close()


@pytest.mark.parametrize("dtype,metric,tables", [("f32", "l2", True), ("f32", "ip", False), ("f16", "l2", False),
                                                 ("bf16", "ip", True), ("bf16", "l2", False)])
def test_refresh_rows_after_vectors_replaced_in_place(dtype, metric, tables):
    """A cluster's vectors replaced in place (what an asynchronous load of another cluster into its
    slot does): after hr_ivf_refresh_rows the index answers for the new bytes: against the oracle on
    a host copy of the new data, and bit for bit like an index loaded from it (squared norms and
    the row tables are derived again)."""
    hr = _hr()
    idx = _random_index(16000, 128, 30, dtype, seed=9)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=tables)
    q = torch.randn(64, 128, generator=torch.Generator().manual_seed(1)).cuda()
    before = ix.search(q, 30, 10, metric)
    off = idx.list_offsets
    lst = int(torch.argmax(off[1:] - off[:-1]))
    r0, r1 = int(off[lst]), int(off[lst + 1])
    # (longer vectors win inner products, shorter ones are nearer: either way the new rows enter the results)
    new = (torch.randn(r1 - r0, 128, generator=torch.Generator().manual_seed(2)) * (3.0 if metric == "ip" else 0.3)).to(idx.list_vectors.dtype)
    idx.list_vectors[r0:r1] = new.cuda()
    ix.refresh_rows(r0, r1)
    ix.refresh_rows(r0, r0)                                   # empty range: nothing to do
    probe, _ = ix.coarse(q, 30, metric)
    got = ix.scan(q, probe, 10, metric)
    host = Host(idx)                                          # (copied after the replacement: the new bytes)
    qn = synth.to_numpy(q)
    m = METRIC[metric]
    ids_o, sc_o = oracle.scan(qn, host.off, host.vec, dtype, host.ids, probe.cpu().numpy(), 10, m)
    st = check_topk(got[0].cpu().numpy(), got[1].cpu().numpy(), ids_o, sc_o,
                    lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, m, np.full(len(ids), i), host.rows_of(ids)),
                    metric, TAU[dtype], _scale(qn, host.xnorm(), metric))
    print(f"[parity refresh {dtype} {metric} tables={tables}] {st}", flush=True)
    in_new = np.isin(ids_o, host.ids[r0:r1]).mean()
    assert in_new > 0.2                                       # (the replaced rows do matter)
    fresh = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=tables)
    want = fresh.search(q, 30, 10, metric)
    got = ix.search(q, 30, 10, metric)
    assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
    assert not torch.equal(before[0], want[0])
    with pytest.raises(hr.HrError):
        ix.refresh_rows(5, idx.list_vectors.shape[0] + 1)
    if dtype == "bf16" and tables:
        # a new value beyond binary16 cannot go into the table: the call says so
        idx.list_vectors[r0 + 3, 5] = 1.0e6
        with pytest.raises(hr.HrError) as e:
            ix.refresh_rows(r0, r1)
        assert e.value.code == -5
        idx.list_vectors[r0 + 3, 5] = 1.0
        ix.refresh_rows(r0, r1)                                # replaced again: fine
    ix.close()
    fresh.close()


@pytest.mark.parametrize("dtype,metric", [("f16", "ip"), ("bf16", "l2"), ("f32", "ip")])
def test_partial_residency_hot_lists_resident_then_one_swapped_in(dtype, metric):
    """Section 4.4: only the gc most frequently probed lists are kept in place.  A first batch fills the access
    counters; the gc hottest lists (hr_ivf_hot_lists) are marked resident, all others not.  Then, for a second batch:
    the split of its probe lists into lists served here and lists to be served elsewhere is the oracle's exactly;
    the scan of the first part is the oracle's scan of those lists; a scan handed the whole probe lists drops the
    others by itself (same bits); the dropped probes still count as accesses.  Finally one missing list is swapped
    in (new vectors copied into its rows by the caller, hr_ivf_refresh_rows, flag set) and the search is compared
    with the oracle on the new bytes."""
    print(f"case residency {dtype} {metric}", flush=True)
    hr = _hr()
    cfg = synth.scaled(synth.CONFIGS["C3"], N=120000, nlist=96, nq=400, nprobe=12, k=10, dtype=dtype, metric=metric, d=128,
                       normalize=metric == "ip")
    idx = synth.make_index(cfg, "cuda")
    q1 = synth.make_queries(cfg, idx)[0]
    q2 = synth.make_queries(synth.scaled(cfg, seed=cfg.seed + 77), idx)[0]
    host = Host(idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    m = METRIC[metric]
    ix.search(q1, cfg.nprobe, cfg.k, metric)
    gc = 30
    hot = ix.hot_lists(gc)
    assert np.array_equal(hot.cpu().numpy(), oracle.hot_lists(ix.list_hits(reset=True).cpu().numpy(), gc))
    ix.set_resident(None, False)
    ix.set_resident(hot, True)
    resident = np.zeros(cfg.nlist, bool)
    resident[hot.cpu().numpy()] = True
    # the second batch
    probe, _ = ix.coarse(q2, cfg.nprobe, metric)
    res, mis = ix.split_probes(probe)
    res_o, mis_o = oracle.split_probes(probe.cpu().numpy(), resident)
    assert np.array_equal(res.cpu().numpy(), res_o) and np.array_equal(mis.cpu().numpy(), mis_o)
    assert (mis_o >= 0).any() and (res_o >= 0).any()
    ids_r, sc_r = ix.scan(q2, res, cfg.k, metric)
    qn = synth.to_numpy(q2)
    score_of = lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, m, np.full(len(ids), i), host.rows_of(ids))
    scale = _scale(qn, host.xnorm(), metric)
    ids_o, sc_o = oracle.scan(qn, host.off, host.vec, dtype, host.ids, res_o, cfg.k, m)
    st = check_topk(ids_r.cpu().numpy(), sc_r.cpu().numpy(), ids_o, sc_o, score_of, metric, TAU[dtype], scale)
    print(f"[parity residency {dtype} {metric}] resident part: {st}; probes served here: {(res_o >= 0).mean():.2f}", flush=True)
    ids_w, sc_w = ix.scan(q2, probe, cfg.k, metric)                # the whole probe lists: the others are dropped
    assert torch.equal(ids_w, ids_r) and torch.equal(sc_w, sc_r)
    # accesses: missing ones counted by the split and again by the scan that dropped them, resident ones by both scans
    want = 2 * np.bincount(probe.cpu().numpy().ravel(), minlength=cfg.nlist)
    assert np.array_equal(ix.list_hits(reset=True).cpu().numpy(), want)
    # swap one missing list in: other vectors into its rows, norms and tables derived again, flag set
    lst = int(mis_o[mis_o >= 0][0])
    r0, r1 = int(host.off[lst]), int(host.off[lst + 1])
    new = idx.centroids[lst][None, :] + 0.02 * torch.randn(r1 - r0, cfg.d, generator=torch.Generator().manual_seed(3)).cuda()
    idx.list_vectors[r0:r1] = new.to(idx.list_vectors.dtype)
    ix.refresh_rows(r0, r1)
    ix.set_resident(torch.tensor([lst], dtype=torch.int32, device="cuda"), True)
    resident[lst] = True
    host = Host(idx)                                               # (the new bytes)
    res2, mis2 = ix.split_probes(probe)
    res2_o, mis2_o = oracle.split_probes(probe.cpu().numpy(), resident)
    assert np.array_equal(res2.cpu().numpy(), res2_o) and np.array_equal(mis2.cpu().numpy(), mis2_o)
    ids_2, sc_2 = ix.scan(q2, res2, cfg.k, metric)
    score_of = lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, m, np.full(len(ids), i), host.rows_of(ids))
    ids_o2, sc_o2 = oracle.scan(qn, host.off, host.vec, dtype, host.ids, res2_o, cfg.k, m)
    st2 = check_topk(ids_2.cpu().numpy(), sc_2.cpu().numpy(), ids_o2, sc_o2, score_of, metric, TAU[dtype], _scale(qn, host.xnorm(), metric))
    got_new = np.isin(ids_o2, host.ids[r0:r1]).any(1).mean()
    print(f"[parity residency {dtype} {metric}] after the swap: {st2}; queries with a result from the new rows: {got_new:.2f}", flush=True)
    assert got_new > 0
    # everything resident again: the plain search
    ix.set_resident(None, True)
    compare_ids, _ = ix.search(q2, cfg.nprobe, cfg.k, metric)
    _, ids_all, _ = oracle.ivf_search(qn, host.cent, host.off, host.vec, dtype, host.ids, cfg.nprobe, cfg.k, m)
    assert (compare_ids.cpu().numpy() == ids_all).all(1).mean() > 0.8
    ix.close()


@pytest.mark.parametrize("dtype,metric,k,tables", [("f16", "ip", 10, False), ("bf16", "l2", 100, False), ("f32", "l2", 30, True),
                                                   ("f32", "ip", 5, False), ("bf16", "ip", 64, True)])
def test_no_kernel_writes_outside_its_workspace_region(dtype, metric, k, tables):
    """Guard words: the workspace is filled with a pattern, a search, a coarse call, a scan and a step-wise scan run in
    it, and the pattern must survive in every byte that lies outside the regions the library says it uses (behind
    every region there is a gap for exactly this), and in the bytes beyond the size it asked for.  The regions are
    sized on the host from worst-case bounds and indexed on the device, where an overrun would otherwise be silent."""
    hr = _hr()
    print(f"case guards {dtype} {metric} k={k}", flush=True)
    cfg = synth.scaled(synth.CONFIGS["C3"], N=150000, nlist=200, nq=700, nprobe=24, k=k, dtype=dtype, metric=metric, d=128,
                       normalize=metric == "ip")
    idx = synth.make_index(cfg, "cuda")
    q = synth.make_queries(cfg, idx)[0]
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=tables)
    m = hr.HR_METRIC_IP if metric == "ip" else hr.HR_METRIC_L2
    for nq, nprobe in ((700, 24), (33, 200), (1, 1)):
        need = hr.hr_ivf_workspace_bytes(ix.handle, nq, nprobe, k)
        regions = hr.hr_ivf_workspace_layout(ix.handle, nq, nprobe, k)
        assert regions and all(o % 256 == 0 for o, _ in regions) and max(o + n for o, n in regions) <= need
        tail = 1 << 16
        ws = torch.full((need + tail,), 0xA5, dtype=torch.uint8, device="cuda")
        qq = q[:nq].contiguous()
        ids = torch.empty(nq, k, dtype=torch.int64, device="cuda")
        sc = torch.empty(nq, k, dtype=torch.float32, device="cuda")
        probe = torch.empty(nq, nprobe, dtype=torch.int32, device="cuda")
        hr.hr_ivf_search(ix.handle, qq, nq, nprobe, k, m, ids, sc, ws, need)
        hr.hr_ivf_coarse(ix.handle, qq, nq, nprobe, m, probe, None, ws, need)
        hr.hr_ivf_scan(ix.handle, qq, nq, probe, nprobe, k, m, ids, sc, ws, need)
        ids.fill_(-1)
        hr.hr_ivf_scan_step(ix.handle, qq, nq, probe, nprobe, k, m, ids, sc, ws, need)
        torch.cuda.synchronize()
        outside = torch.ones(need + tail, dtype=torch.bool, device="cuda")
        for o, n in regions:
            outside[o:o + n] = False
        bad = (ws != 0xA5) & outside
        assert not bool(bad.any()), f"nq={nq} nprobe={nprobe}: byte {int(bad.nonzero()[0])} outside every region was written"
        assert int(outside[:need].sum()) >= 256 * len(regions)
    ix.close()


def test_negative_labels_are_refused_at_load():
    """A negative id marks an empty place in results, so a label may not be negative."""
    hr = _hr()
    idx = _random_index(3000, 64, 7, "f16", seed=3)
    idx.list_ids[1234] = -5
    with pytest.raises(hr.HrError) as e:
        hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    assert e.value.code == -1 and "negative label" in str(e.value)


def test_scan_takes_more_places_than_there_are_lists():
    """hr_ivf_scan takes probe rows of up to HR_NPROBE_MAX places whatever the number of lists (the
    other places empty), and hr_ivf_workspace_bytes sizes a workspace for that shape."""
    hr = _hr()
    idx = _random_index(4000, 64, 6, "f16", seed=13)
    host = Host(idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    assert hr.hr_ivf_workspace_bytes(ix.handle, 20, 40, 5) > 0
    assert hr.hr_ivf_workspace_bytes(ix.handle, 20, hr.HR_NPROBE_MAX + 1, 5) == 0
    q = torch.randn(20, 64, generator=torch.Generator().manual_seed(2)).cuda()
    probe = torch.full((20, 40), -1, dtype=torch.int32)
    probe[:, 7] = 2
    probe[:, 33] = 5
    ids, sc = ix.scan(q, probe.cuda(), 5, "ip")
    qn = synth.to_numpy(q)
    ids_o, sc_o = oracle.scan(qn, host.off, host.vec, "f16", host.ids, probe.numpy(), 5, oracle.IP)
    check_topk(ids.cpu().numpy(), sc.cpu().numpy(), ids_o, sc_o,
               lambda i, v: oracle.pair_scores(qn, host.vec, "f16", oracle.IP, np.full(len(v), i), host.rows_of(v)),
               "ip", TAU["f16"], _scale(qn, host.xnorm(), "ip"))
    with pytest.raises(hr.HrError):
        ix.search(q, 7, 5, "ip")                               # the whole search still wants nprobe <= nlist
    ix.close()



def test_seeded_sweep_of_small_configurations():
    """Forty seeded draws of (N, d, lists, storage, metric, batch, nprobe, k) from the corners of
    the supported ranges (one row, one list, one query, k at the buffer-size boundaries 24/25,
    64/65 and at its maximum, nprobe up to 300), each through coarse, scan and search against
    the oracle; every other draw with row tables."""
    rng = np.random.default_rng(1)
    for c in range(40):
        d = int(rng.choice([64, 128, 256, 512, 768, 1024]))
        dtype = str(rng.choice(["f32", "f16", "bf16"]))
        metric = str(rng.choice(["ip", "l2"]))
        nlist = int(rng.choice([1, 2, 7, 33, 150, 600]))
        n = int(rng.choice([1, 15, 17, 300, 5000, 40000]))
        nq = int(rng.choice([1, 2, 17, 129, 700]))
        nprobe = int(min(nlist, rng.choice([1, 2, 9, 64, 300])))
        k = int(rng.choice([1, 2, 10, 24, 25, 64, 65, 100, 128]))
        print(f"case sweep {c}: n={n} d={d} nlist={nlist} {dtype} {metric} nq={nq} nprobe={nprobe} k={k}", flush=True)
        idx = _random_index(n, d, nlist, dtype, seed=1000 + c)
        q = torch.randn(nq, d, generator=torch.Generator().manual_seed(c)).cuda()
        compare_all(idx, q, nprobe=nprobe, k=k, metric=metric, row_tables=bool(c & 1))


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_bfloat16_lists_with_the_binary16_table(metric):
    """bfloat16 lists are scanned as bfloat16 with the query in bfloat16 hi and lo parts, or, when the
    caller asked for row tables at load, from a binary16 copy (query rounded to binary16, one MFMA
    column per query).  The second way is checked here (the first is what every other bfloat16 test
    runs), on random data with k on both sides of the buffer-size boundary and on the scaled large
    workload."""
    print(f"case bf16 with table {metric}", flush=True)
    idx = _random_index(30000, 256, 40, "bf16", seed=83, dup=2)
    q = torch.randn(200, 256, generator=torch.Generator().manual_seed(5)).cuda()
    compare_all(idx, q, nprobe=9, k=10, metric=metric, row_tables=True)
    compare_all(idx, q, nprobe=9, k=100, metric=metric, row_tables=True)
    if metric == "l2":
        cfg = synth.scaled(synth.CONFIGS["C5"], N=262144, nlist=256, nq=256, nprobe=32)
        ci = synth.make_index(cfg, "cuda")
        compare_all(ci, synth.make_queries(cfg, ci)[0], cfg.nprobe, cfg.k, cfg.metric, row_tables=True, label="C5 scaled, with table")


def test_bfloat16_values_beyond_binary16_keep_the_bfloat16_scan():
    """A value above 65504 cannot go into the binary16 table: the load notices and the lists are
    scanned as bfloat16 (results against the oracle as usual)."""
    idx = _random_index(6000, 64, 12, "bf16", seed=19)
    idx.list_vectors[1234, 7] = 1.0e6
    idx.list_vectors[77, 0] = -3.0e5
    q = torch.randn(50, 64, generator=torch.Generator().manual_seed(8)).cuda()
    compare_all(idx, q, nprobe=12, k=5, metric="ip", row_tables=True)



def test_two_searches_in_flight_on_two_streams():
    """Two calls on the same index, each with its own stream, workspace and outputs, enqueued
    back to back so that they overlap on the device: both must give what they give alone."""
    hr = _hr()
    idx = _random_index(60000, 128, 64, "f16", seed=41)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    gen = torch.Generator().manual_seed(6)
    qa, qb = torch.randn(700, 128, generator=gen).cuda(), torch.randn(500, 128, generator=gen).cuda()
    want_a = ix.search(qa, 16, 10, "ip")
    want_b = ix.search(qb, 24, 20, "l2")
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    out = []
    for q, nprobe, k in ((qa, 16, 10), (qb, 24, 20)):
        nbytes = hr.hr_ivf_workspace_bytes(ix.handle, q.shape[0], nprobe, k)
        out.append((torch.empty(q.shape[0], k, dtype=torch.int64, device="cuda"),
                    torch.empty(q.shape[0], k, dtype=torch.float32, device="cuda"),
                    torch.empty(nbytes, dtype=torch.uint8, device="cuda")))
    for _ in range(3):
        for t in out:
            t[0].fill_(-9)
        torch.cuda.synchronize()
        hr.hr_ivf_search(ix.handle, qa, 700, 16, 10, hr.HR_METRIC_IP, out[0][0], out[0][1], out[0][2], out[0][2].numel(), stream=sa)
        hr.hr_ivf_search(ix.handle, qb, 500, 24, 20, hr.HR_METRIC_L2, out[1][0], out[1][1], out[1][2], out[1][2].numel(), stream=sb)
        torch.cuda.synchronize()
        assert torch.equal(out[0][0], want_a[0]) and torch.equal(out[0][1], want_a[1])
        assert torch.equal(out[1][0], want_b[0]) and torch.equal(out[1][1], want_b[1])
    ix.close()


def test_coarse_selection_when_the_one_pass_way_does_not_apply():
    """The nprobe best centroids are normally found in one pass from a sampled lower bound; two
    rows built so that this cannot work (more keys at the bound than the collection holds; a
    bound above the nprobe-th key) must come out of the full radix select, exact as ever."""
    hr = _hr()
    g = torch.Generator(device="cpu").manual_seed(77)
    d = 64
    v = torch.randn(d, generator=g)
    v = v / v.norm()

    def run(cent, nprobe):
        nlist = cent.shape[0]
        off = torch.arange(0, nlist + 1, dtype=torch.int64)
        x = torch.randn(nlist, d, generator=g).to(torch.float16)
        ix = hr.IvfIndex(cent.cuda(), off, x.cuda(), torch.arange(nlist, dtype=torch.int64).cuda())
        q = (v[None, :] + 0.01 * torch.randn(40, d, generator=g)).contiguous()
        probe, score = ix.coarse(q.cuda(), nprobe, "ip")
        probe, score = probe.cpu().numpy(), score.cpu().numpy()
        probe_o, score_o = oracle.coarse(q.numpy(), cent.numpy(), nprobe, oracle.IP)
        cn = float(np.sqrt((cent.numpy().astype(np.float64) ** 2).sum(1)).mean())
        st = check_probes(probe, score, probe_o, score_o,
                          lambda i, c: oracle.pair_scores(q.numpy(), cent.numpy(), "f32", oracle.IP, np.full(len(c), i), c),
                          "ip", TAU["f32"], _scale(q.numpy(), cn, "ip"))
        ix.close()
        return probe, probe_o, st

    # 2000 copies of the best centroid among 3000: far more equal keys at the top than the 1024 collected
    cent = 0.05 * torch.randn(3000, d, generator=g)
    copies = torch.randperm(3000, generator=g)[:2000]
    cent[copies] = v * 2.0
    probe, probe_o, st = run(cent, 100)
    lowest = np.sort(copies.numpy())[:100]
    assert (probe == lowest[None, :]).all() and np.array_equal(probe, probe_o)       # equal keys: lower index first
    # 50 outstanding centroids, all on sampled positions (every 4th of 2048): the sampled bound lands among them,
    # fewer than nprobe = 64 keys reach it
    cent = 0.05 * torch.randn(2048, d, generator=g)
    top = torch.arange(0, 200, 4)
    cent[top] = v[None, :] * (2.0 + 0.01 * torch.arange(50, dtype=torch.float32)[:, None])
    probe, probe_o, st = run(cent, 64)
    assert np.array_equal(np.sort(probe[:, :50], axis=1), np.broadcast_to(top.numpy(), (40, 50)))
    assert np.array_equal(probe[:, :50], probe_o[:, :50])
    print(f"[parity coarse fallback] {st}", flush=True)


def test_seeded_sweep_of_stepwise_retrievals_started_from_cached_rows():
    """Twenty-four seeded draws of storage type, metric, sizes, k, cache size and sub-stage width:
    a carried result started from random cached rows (absent, repeated, inside and outside the
    probed lists), then the probe lists (with holes) searched a few at a time; expected: the
    oracle's k best over the union of the cached rows and the rows of the probed lists, every
    vector once, rows and ids naming the same vectors.  Half of the draws load without row tables."""
    hr = _hr()
    rng = np.random.default_rng(3)
    for c in range(24):
        d = int(rng.choice([64, 128, 256]))
        dtype = str(rng.choice(["f32", "f16", "bf16"]))
        metric = str(rng.choice(["ip", "l2"]))
        nlist = int(rng.choice([5, 33, 150]))
        n = int(rng.choice([300, 5000, 30000]))
        nq = int(rng.choice([1, 17, 200]))
        nprobe = int(min(nlist, rng.choice([2, 9, 40])))
        k = int(rng.choice([1, 10, 25, 100]))
        m = int(rng.choice([1, 20, 128]))
        step = int(rng.choice([1, 3, 8]))
        print(f"case steps sweep {c}: n={n} d={d} nlist={nlist} {dtype} {metric} nq={nq} nprobe={nprobe} k={k} m={m} step={step}", flush=True)
        idx = _random_index(n, d, nlist, dtype, seed=2000 + c)
        host = Host(idx)
        ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=bool(rng.integers(0, 2)))
        q = torch.randn(nq, d, generator=torch.Generator().manual_seed(c)).cuda()
        cache = rng.integers(-1, idx.list_vectors.shape[0], (nq, m)).astype(np.int32)
        probe = np.stack([rng.permutation(nlist)[:nprobe] for _ in range(nq)]).astype(np.int32)
        probe[rng.random(probe.shape) < 0.1] = -1
        state = ix.rescore(q, torch.from_numpy(cache).cuda(), k, metric)
        pd = torch.from_numpy(probe).cuda()
        for s0 in range(0, nprobe, step):
            ix.scan_step_rows(q, pd[:, s0:s0 + step].contiguous(), state, metric)
        ids_g, sc_g, rows_g = [t.cpu().numpy() for t in state]
        qn = synth.to_numpy(q)
        union = [np.concatenate([cache[i]] + [np.arange(host.off[l], host.off[l + 1]) for l in probe[i] if l >= 0])
                 for i in range(nq)]
        mm = METRIC[metric]
        ids_o, sc_o, _ = oracle.topk_of_rows(qn, host.vec, dtype, host.ids, union, k, mm)
        check_topk(ids_g, sc_g, ids_o, sc_o,
                   lambda i, ids: oracle.pair_scores(qn, host.vec, dtype, mm, np.full(len(ids), i), host.rows_of(ids)),
                   metric, TAU[dtype], _scale(qn, host.xnorm(), metric))
        have = ids_g >= 0
        assert np.array_equal(host.ids[rows_g[have]], ids_g[have])
        assert ((ids_g >= 0) == (ids_o >= 0)).all()
        for i in range(nq):
            r = rows_g[i][rows_g[i] >= 0]
            assert len(np.unique(r)) == len(r)
        ix.close()
