"""The synthetic workloads have the shape the configs describe (closed forms of the recipe)."""
import numpy as np
import torch

import synth


def test_list_sizes_sum_and_shape():
    for name, cfg in synth.CONFIGS.items():
        s = synth.list_sizes(cfg)
        assert s.sum() == cfg.N and s.min() >= 1 and len(s) == cfg.nlist
        assert np.all(np.diff(s) <= 0)
    s3 = synth.list_sizes(synth.CONFIGS["C3"])
    assert (s3.min(), int(np.median(s3)), s3.max()) == (72, 153, 673054)
    s1 = synth.list_sizes(synth.CONFIGS["C1"])
    assert (s1.min(), s1.max()) == (42, 10701)
    s5 = synth.list_sizes(synth.CONFIGS["C5"])
    assert (s5.min(), s5.max()) == (76, 2028826)
    # top 20 % of the lists hold most of the vectors (access skew, Section 3.3 of the paper)
    assert s3[: len(s3) // 5].sum() / s3.sum() > 0.69


def test_closed_forms_of_the_recipe():
    cfg = synth.scaled(synth.CONFIGS["C3"], N=8192, nlist=16, nq=256, dtype="f32")
    idx = synth.make_index(cfg)
    q = synth.make_queries(cfg, idx)[0]
    off = idx.list_offsets
    assert off[0] == 0 and off[-1] == cfg.N
    assert sorted(idx.list_ids.tolist()) == list(range(cfg.N))
    x = idx.list_vectors.double()
    assert torch.allclose(x.norm(dim=1), torch.ones(cfg.N, dtype=torch.float64), atol=1e-6)
    l = int(torch.argmax(off[1:] - off[:-1]))
    rows = x[off[l]: off[l + 1]]
    c = idx.centroids[l].double()
    sig2 = cfg.noise ** 2
    assert abs(float((rows @ c).mean()) - 1 / (1 + sig2) ** 0.5) < 3e-3      # 0.9578
    g = rows[:200] @ rows[200:400].T
    assert abs(float(g.mean()) - 1 / (1 + sig2)) < 3e-3                      # 0.9174
    other = x[off[(l + 1) % cfg.nlist]: off[(l + 1) % cfg.nlist + 1]]
    if len(other):
        assert abs(float((rows[:100] @ other[:100].T).mean())) < 0.1
    # queries sit on their centroid the same way
    best = (q.double() @ idx.centroids.double().T).max(1).values
    assert abs(float(best.mean()) - 1 / (1 + sig2) ** 0.5) < 3e-3


def test_unnormalised_l2_config_and_rounds():
    cfg = synth.scaled(synth.CONFIGS["C5"], N=4096, nlist=8, nq=64)
    idx = synth.make_index(cfg)
    assert idx.list_vectors.dtype == torch.bfloat16
    off = idx.list_offsets
    l = int(torch.argmax(off[1:] - off[:-1]))
    rows = idx.list_vectors[off[l]: off[l + 1]].double()
    d2 = torch.cdist(rows[:100], rows[100:200]) ** 2
    assert abs(float(d2.mean()) - 2 * cfg.noise ** 2) < 0.02                 # 0.18
    cfg4 = synth.scaled(synth.CONFIGS["C4"], N=4096, nlist=8, nq=32)
    idx4 = synth.make_index(cfg4)
    rounds = synth.make_queries(cfg4, idx4)
    assert len(rounds) == 8
    step = (rounds[1] - rounds[0]).norm(dim=1).mean()
    assert 0.03 < float(step) < 0.07                                          # drift 0.05
    # same seed, same bytes
    again = synth.make_index(cfg4)
    assert torch.equal(again.list_vectors, idx4.list_vectors) and torch.equal(again.list_ids, idx4.list_ids)
    bits = synth.to_numpy(idx.list_vectors)
    assert bits.dtype == np.uint16 and bits.shape == (cfg.N, cfg.d)
