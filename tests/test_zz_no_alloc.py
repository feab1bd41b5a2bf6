"""hr_ivf_search_static (the entry point that allocates nothing: its scratch memory is a fixed array inside the
library) against hr_ivf_search with a workspace, through the C ABI: same bits, on two calls in a row, the second
with a smaller batch (the array keeps what the first call left), and against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from compare import TAU, check_topk

pytestmark = pytest.mark.gpu


def _both(hr, ix, q, nprobe, k, metric):
    nq = q.shape[0]
    m = hr.HR_METRIC_IP if metric == "ip" else hr.HR_METRIC_L2
    want = ix.search(q, nprobe, k, metric)
    ids = torch.full((nq, k), -7, dtype=torch.int64, device=q.device)
    scores = torch.zeros(nq, k, dtype=torch.float32, device=q.device)
    torch.cuda.synchronize()
    hr.hr_ivf_search_static(ix.handle, q, nq, nprobe, k, m, ids, scores)
    torch.cuda.synchronize()
    return want, (ids, scores)


@pytest.mark.parametrize("dtype,metric,k", [("f16", "ip", 10), ("bf16", "l2", 100), ("f32", "l2", 30)])
def test_static_scratch_search_matches_the_workspace_search(dtype, metric, k):
    import paper_2507_09138_amd as hr
    print(f"case static scratch {dtype} {metric} k={k}", flush=True)
    cfg = synth.scaled(synth.CONFIGS["C3"], N=100000, nlist=128, nq=300, nprobe=12, k=k, dtype=dtype, metric=metric, d=256,
                       normalize=metric == "ip")
    idx = synth.make_index(cfg, "cuda")
    q = synth.make_queries(cfg, idx)[0]
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    # two calls in a row; the second is smaller and finds the first one's leftovers in the array
    for n, nprobe in ((300, 12), (41, 5)):
        want, got = _both(hr, ix, q[:n].contiguous(), nprobe, k, metric)
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1]), f"nq={n}"
    # and against the oracle (the small batch)
    qs = synth.to_numpy(q[:41])
    m = oracle.IP if metric == "ip" else oracle.L2
    vec, ids_h = synth.to_numpy(idx.list_vectors), synth.to_numpy(idx.list_ids)
    probe, _ = ix.coarse(q[:41].contiguous(), 5, metric)
    ids_o, sc_o = oracle.scan(qs, synth.to_numpy(idx.list_offsets), vec, dtype, ids_h, probe.cpu().numpy(), k, m)
    row_of = {int(v): i for i, v in enumerate(ids_h)}
    xn = float(np.sqrt((idx.list_vectors[:2048].float().cpu().numpy().astype(np.float64) ** 2).sum(1)).mean())
    qn = np.sqrt((qs.astype(np.float64) ** 2).sum(1))
    scale = 0.02 * (768.0 / 256) ** 0.5 * (qn * xn if metric == "ip" else qn ** 2 + xn ** 2)
    st = check_topk(got[0].cpu().numpy(), got[1].cpu().numpy(), ids_o, sc_o,
                    lambda i, ids: oracle.pair_scores(qs, vec, dtype, m, np.full(len(ids), i), np.array([row_of[int(v)] for v in ids])),
                    metric, TAU[dtype], scale)
    print(f"[parity static scratch {dtype} {metric}] {st}", flush=True)
    ix.close()


def test_static_scratch_refuses_what_does_not_fit_and_allocates_nothing():
    import paper_2507_09138_amd as hr
    cfg = synth.scaled(synth.CONFIGS["C3"], N=50000, nlist=64, nq=64, nprobe=8, d=128)
    idx = synth.make_index(cfg, "cuda")
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids)
    q = synth.make_queries(cfg, idx)[0]
    ids = torch.full((64, 10), -7, dtype=torch.int64, device="cuda")
    scores = torch.zeros(64, 10, device="cuda")
    big = torch.zeros(1 << 17, 128, device="cuda")
    big_ids = torch.empty(1 << 17, 100, dtype=torch.int64, device="cuda")
    big_sc = torch.empty(1 << 17, 100, device="cuda")
    with pytest.raises(hr.HrError) as e:                   # 131072 queries x 64 lists, k = 100: far beyond 64 MiB
        hr.hr_ivf_search_static(ix.handle, big, 1 << 17, 64, 100, 0, big_ids, big_sc)
    assert e.value.code == -3 and "static array" in str(e.value)
    with pytest.raises(hr.HrError) as e:
        hr.hr_ivf_search_static(ix.handle, q, 64, 8, 0, 0, ids, scores)
    assert e.value.code == -1
    torch.cuda.synchronize()
    assert (ids == -7).all()                               # nothing was enqueued by the refused calls
    # device memory in use does not move over a series of calls (nothing allocated, nothing freed)
    hr.hr_ivf_search_static(ix.handle, q, 64, 8, 10, 0, ids, scores)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(20):
        hr.hr_ivf_search_static(ix.handle, q, 64, 8, 10, 0, ids, scores)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0
    want = ix.search(q, 8, 10, "ip")
    assert torch.equal(ids, want[0]) and torch.equal(scores, want[1])
    ix.close()
