"""Benchmark of the batched IVF search hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--nq N] [--nprobe P] [--no-cpu-baseline]

One step = one hr_ivf_search call (coarse scoring, top-nprobe, grouping by list, cluster-major
scan, per-query merge) over one batch of synthetic queries, index and queries resident in HBM.
Prints one JSON line: queries/s, plus the roofline of the list-scan kernel (algorithmic bytes
of the probed lists / its average duration, measured with HIP events around its launches) and
the CPU oracle timed on a bounded sample of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
F16_MFMA_PEAK_TFLOPS = 2500.0      # dense binary16 / bfloat16 MFMA
F32_PEAK_TFLOPS = 157.3            # float32 (vector or MFMA): what float32 storage is priced against
ESIZE = {"f32": 4, "f16": 2, "bf16": 2}


def mfma_peak(cfg, ix):
    """float32 lists are a float32 contraction to the caller (that it runs as three binary16 products per element on
    the matrix pipes is this library's choice): its 2 d flops per (query, row) pair are priced against the float32
    peak; 16-bit lists against the dense 16-bit MFMA peak."""
    return F32_PEAK_TFLOPS if cfg.dtype == "f32" else F16_MFMA_PEAK_TFLOPS


def operand_name(cfg, ix):
    """The type the list scan multiplies in (accumulation is float32 throughout)."""
    if cfg.dtype == "f32":
        return "f16x2"                              # binary16 hi + scaled lo parts of both operands
    if cfg.dtype == "bf16":
        return "f16" if ix.row_tables else "bf16"   # binary16 row table asked for at load, else bfloat16 rows x (hi, lo) query
    return "f16"


def traffic_from_profiles(cfg, row_tables):
    """HBM bytes per list-scan launch (read + written) as the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised under
    profiles/ measured them for this workload (counters cannot be read from inside this process): the number after
    `hbm_bytes_per_scan_launch:` in profiles/k_scan_<storage>_<workload>[_row_tables].txt, or None when there is no
    such summary (other batch sizes than the workload's own are not looked up at all)."""
    name = f"k_scan_{cfg.dtype}_{cfg.name}{'_row_tables' if row_tables and cfg.dtype != 'f16' else ''}.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.strip().startswith("hbm_bytes_per_scan_launch:"):
            return float(line.split(":", 1)[1].split()[0]), "profiles/" + name
    return None, None


def cpu_info():
    model, phys = "unknown", set()
    try:
        pid = cid = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name") and model == "unknown":
                model = line.split(":", 1)[1].strip()
            elif line.startswith("physical id"):
                pid = line.split(":", 1)[1].strip()
            elif line.startswith("core id"):
                cid = line.split(":", 1)[1].strip()
            elif not line.strip():
                if pid is not None and cid is not None:
                    phys.add((pid, cid))
                pid = cid = None
    except OSError:
        pass
    return model, len(phys) or None, os.cpu_count()


def cpu_baseline(cfg, idx, q, gpu_ids, gpu_scores, target_s=20.0):
    """The oracle as it stands, on the host cores, on a sample of the batch sized for about target_s seconds; next to
    it the same on one thread (a smaller sample), how the timed GPU result compares with the oracle's on that sample,
    and the recall of the search against the oracle's exhaustive search on a few queries."""
    import numpy as np
    import oracle
    import synth
    cent = synth.to_numpy(idx.centroids)
    off = synth.to_numpy(idx.list_offsets)
    vec = synth.to_numpy(idx.list_vectors)
    ids = synth.to_numpy(idx.list_ids)
    qh = synth.to_numpy(q)
    m = oracle.IP if cfg.metric == "ip" else oracle.L2
    threads = oracle.num_threads()
    rng = np.random.default_rng(7)
    order = rng.permutation(qh.shape[0])
    n0 = min(len(order), max(threads, 8))
    t0 = time.time()
    oracle.ivf_search(np.ascontiguousarray(qh[order[:n0]]), cent, off, vec, cfg.dtype, ids, cfg.nprobe, cfg.k, m)
    t_pilot = time.time() - t0          # also pages the index in; only sizes the timed sample
    n1 = int(min(len(order) - n0, target_s / max(t_pilot / n0, 1e-9)))
    n1 -= n1 % threads if n1 > threads else 0
    if n1 > 0:
        sel = order[n0:n0 + n1]
        t0 = time.time()
        _, ids_o, sc_o = oracle.ivf_search(np.ascontiguousarray(qh[sel]), cent, off, vec, cfg.dtype, ids, cfg.nprobe, cfg.k, m)
        total_t, total_n = time.time() - t0, n1
    else:
        sel = order[:n0]
        _, ids_o, sc_o = oracle.ivf_search(np.ascontiguousarray(qh[sel]), cent, off, vec, cfg.dtype, ids, cfg.nprobe, cfg.k, m)
        total_t, total_n = t_pilot, n0
    rate = total_n / total_t
    # one thread: about 5 s worth of the same queries
    n_one = int(max(1, min(len(sel), 5.0 * rate / max(threads, 1))))
    oracle.set_threads(1)
    t0 = time.time()
    oracle.ivf_search(np.ascontiguousarray(qh[sel[:n_one]]), cent, off, vec, cfg.dtype, ids, cfg.nprobe, cfg.k, m)
    t_one = time.time() - t0
    oracle.set_threads(threads)
    # the GPU's result for the sampled queries against the oracle's (whole search, the oracle's own probe lists)
    g_i, g_s = gpu_ids[sel], gpu_scores[sel].astype(np.float64)
    finite = np.isfinite(sc_o) & (np.abs(sc_o) > 0)
    rel = np.abs(g_s - sc_o)[finite] / np.abs(sc_o[finite])
    overlap = float(np.mean([np.isin(g_i[i], ids_o[i]).mean() for i in range(len(sel))]))
    # recall of the approximate search (both sides) against the exhaustive search, on a few queries
    nb = int(min(16, len(sel)))
    t0 = time.time()
    ids_b, _ = oracle.bruteforce(np.ascontiguousarray(qh[sel[:nb]]), vec, cfg.dtype, ids, cfg.k, m)
    t_b = time.time() - t0
    rec_gpu = float(np.mean([np.isin(ids_b[i], g_i[i]).mean() for i in range(nb)]))
    rec_or = float(np.mean([np.isin(ids_b[i], ids_o[i]).mean() for i in range(nb)]))
    model, phys, logical = cpu_info()
    return {"value": rate, "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": f"{total_n} randomly chosen queries of the batch (full index, nprobe={cfg.nprobe}, "
                      f"k={cfg.k}), {total_t:.1f} s after a {n0}-query pilot",
            "cpu_model": model, "physical_cores": phys, "logical_cpus": logical,
            "one_thread": {"value": n_one / t_one, "unit": "queries/s", "sample": f"the first {n_one} of those queries, {t_one:.1f} s"},
            "gpu_vs_oracle_on_sample": {"queries": int(len(sel)), "rows_with_identical_ids": float((g_i == ids_o).all(1).mean()),
                                        "id_set_overlap": overlap, "max_rel_score_err": float(rel.max()) if rel.size else 0.0},
            "recall_at_k_vs_exhaustive": {"queries": nb, "k": cfg.k, "gpu": rec_gpu, "oracle": rec_or,
                                          "exhaustive_search_s": round(t_b, 1)}}


def bench_width_split(args, cfg, hr, ix, idx, rounds, metric):
    """The list scan on a part of the probe lists only: the lists that at least `--wide-only W` queries of the batch
    probe (the wide buckets: a dense [rows x d] . [d x queries] contraction, bound by the matrix pipes), or the lists
    that fewer than `--narrow-only W` probe (bound by the row stream from HBM).  One step = one hr_ivf_scan call with
    the other places of the probe lists emptied; the scan kernel is timed by the library's events."""
    import torch
    nq = cfg.nq
    q = rounds[0]
    probe, _ = ix.coarse(q, cfg.nprobe, cfg.metric)
    w = torch.bincount(probe.flatten().long(), minlength=cfg.nlist)
    wide = args.wide_only > 0
    W = args.wide_only if wide else args.narrow_only
    keep_list = (w >= W) if wide else ((w < W) & (w > 0))
    part = torch.where(keep_list[probe.long()], probe, torch.full_like(probe, -1)).contiguous()
    ids = torch.empty(nq, cfg.k, dtype=torch.int64, device="cuda")
    scores = torch.empty(nq, cfg.k, dtype=torch.float32, device="cuda")
    ws = ix.workspace(nq, cfg.nprobe, cfg.k)

    def step():
        hr.hr_ivf_scan(ix.handle, q, nq, part, cfg.nprobe, cfg.k, metric, ids, scores, ws, ws.numel())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    hr.hr_ivf_profile_begin(ix.handle, args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    n_timed, scan_ms = hr.hr_ivf_profile_end(ix.handle)
    st = ix.stats(nq, cfg.nprobe, cfg.k)
    lens = (idx.list_offsets[1:] - idx.list_offsets[:-1])
    wk = (w.cpu() * keep_list.cpu())
    rows = int(lens[keep_list.cpu()].sum())
    pair_rows = int((wk * lens).sum())
    assert rows == st["rows_streamed"], (rows, st)
    nbytes = rows * cfg.d * ESIZE[cfg.dtype]
    flops = 2.0 * cfg.d * pair_rows
    tf = flops / (scan_ms * 1e-3) / 1e12
    gbs = nbytes / (scan_ms * 1e-3) / 1e9
    peak = mfma_peak(cfg, ix)
    ix.close()
    roof = ({"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak} if wide else
            {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS})
    roof.update({"kernel": "k_scan (list scan)", "traffic": None, "scan_ms_avg": scan_ms, "launches_timed": n_timed,
                 "algorithmic_bytes_per_launch": nbytes, "algorithmic_flops_per_launch": flops,
                 "hbm_gbs": gbs, "mfma_tflops": tf})
    print(json.dumps({"metric": "list scan on the %s buckets only" % ("wide" if wide else "narrow"),
                      "value": tf if wide else gbs, "unit": roof["unit"], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": ms, "higher_is_better": True, "data": "synthetic", "dtype": operand_name(cfg, ix),
                      "config": {"workload": f"{cfg.name}: lists probed by {'at least' if wide else 'fewer than'} {W} of the "
                                             f"{nq} queries (nprobe={cfg.nprobe}, k={cfg.k}, {cfg.dtype} storage, {cfg.metric})",
                                 "lists": int(keep_list.sum()), "widest_bucket": int(wk.max()), "pairs": st["pairs"],
                                 "scan_items": st["items"], "seg_rows": st["seg_rows"]},
                      "roofline": roof}))


def bench_substages(args, cfg, hr, ix, rounds, metric):
    """Step-wise retrieval: per step one coarse call, then the probe lists searched in `substages`
    slices with hr_ivf_scan_step, the per-query result carried from slice to slice."""
    import torch
    nq, S = cfg.nq, args.substages
    per = (cfg.nprobe + S - 1) // S
    probe = torch.empty(nq, cfg.nprobe, dtype=torch.int32, device="cuda")
    slices = [torch.empty(nq, min(per, cfg.nprobe - j), dtype=torch.int32, device="cuda") for j in range(0, cfg.nprobe, per)]
    ids = torch.empty(nq, cfg.k, dtype=torch.int64, device="cuda")
    scores = torch.empty(nq, cfg.k, dtype=torch.float32, device="cuda")
    ws_c = ix.workspace(nq, cfg.nprobe, cfg.k)
    ws_s = ix.workspace(nq, per, cfg.k)

    def step(i):
        q = rounds[i % len(rounds)]
        hr.hr_ivf_coarse(ix.handle, q, nq, cfg.nprobe, metric, probe, None, ws_c, ws_c.numel())
        ids.fill_(-1)
        for j, sl in enumerate(slices):
            sl.copy_(probe[:, j * per:j * per + sl.shape[1]])
            hr.hr_ivf_scan_step(ix.handle, q, nq, sl, sl.shape[1], cfg.k, metric, ids, scores, ws_s, ws_s.numel())

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    ref_ids, _ = ix.search(rounds[(args.steps - 1) % len(rounds)], cfg.nprobe, cfg.k, cfg.metric)
    same = float((ref_ids == ids).all(1).float().mean())
    ix.close()
    print(json.dumps({"metric": "queries/sec batched IVF top-k search, step-wise", "value": nq / (ms * 1e-3),
                      "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                      "higher_is_better": True, "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: nq={nq}, nprobe={cfg.nprobe} in {len(slices)} sub-stages of "
                                             f"{per} lists, k={cfg.k}", "rows_identical_to_one_call": same}}))


def bench_reuse(args, cfg, hr, ix, rounds, metric):
    """Consecutive retrievals of the same requests (the rounds of the workload: every query drifts a
    little from round to round).  Each retrieval searches its probe lists in `reuse` sub-stages with a
    carried top-20.  Two ways: lists in rank order from an empty result; or started from the 20 cached
    rows of the previous round, lists in the order hot / probed before / rest.  Reported: after how
    many sub-stages the final top-k is in place on average (the search could have stopped there), and
    the time of a whole retrieval."""
    import torch
    nq, S, k, big = cfg.nq, args.reuse, cfg.k, max(20, cfg.k)
    per = (cfg.nprobe + S - 1) // S
    nst = (cfg.nprobe + per - 1) // per
    R = len(rounds)

    def retrieval(q, prev, use, record):
        """prev = (probe, state) of the previous round or None; returns (probe, state, ids after every sub-stage)"""
        probe, _ = ix.coarse(q, cfg.nprobe, cfg.metric)
        if use and prev is not None:
            hot = ix.lists_of_rows(prev[1][2][:, :k])
            order = hr.reorder_probes(probe, prev[0], hot)
            state = ix.rescore(q, prev[1][2], big, cfg.metric)
        else:
            order = probe
            state = ix.new_state_rows(nq, big)
        seen = [state[0][:, :k].clone()] if record else None          # (before any list: what the cache alone gives)
        for j in range(nst):
            ix.scan_step_rows(q, order[:, j * per:(j + 1) * per].contiguous(), state, cfg.metric)
            if record:
                seen.append(state[0][:, :k].clone())
        return probe, state, seen

    out = {}
    for use in (False, True):
        # how early the final result is in place (untimed pass)
        prev, stages = None, []
        for r in range(R):
            probe, state, seen = retrieval(rounds[r], prev, use, True)
            if r > 0:
                final = seen[-1]
                first = torch.full((nq,), nst, dtype=torch.int64, device="cuda")
                for j in range(nst, -1, -1):
                    first = torch.where((seen[j] == final).all(1), torch.full_like(first, j), first)
                # (sub-stages are counted from 1; 0 = the cached rows already were the answer)
                stages.append(first.float().mean().item())
            prev = (probe, state)
        # time of whole retrievals, rounds 1..R-1
        def one_pass():
            prev = None
            for r in range(R):
                probe, state, _ = retrieval(rounds[r], prev, use, False)
                prev = (probe, state)
        for _ in range(max(1, args.warmup // 2)):
            one_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_pass()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / (args.steps * R) * 1e3
        out["reuse" if use else "plain"] = {"substages_until_final_mean": sum(stages) / len(stages), "ms_per_retrieval": ms}
    ix.close()
    a, b = out["plain"]["substages_until_final_mean"], out["reuse"]["substages_until_final_mean"]
    print(json.dumps({"metric": "sub-stages until the final top-k is in place (of %d)" % nst, "value": b, "unit": "sub-stages",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: nq={nq}, nprobe={cfg.nprobe} in {nst} sub-stages of {per} lists, "
                                             f"k={k}, top-{big} carried and cached, {R} rounds, noise {cfg.noise}, drift {cfg.drift}"},
                      "plain_order": out["plain"], "cache_and_reordering": out["reuse"], "reduction": 1.0 - b / a if a > 0 else 0.0}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--nq", type=int, default=0, help="batch size instead of the workload's own")
    ap.add_argument("--nprobe", type=int, default=0, help="lists probed per query instead of the workload's own")
    ap.add_argument("--substages", type=int, default=0,
                    help="extra mode: one step = coarse + this many hr_ivf_scan_step calls over slices of the probe "
                         "lists, result carried along (the step-wise interface); prints its own JSON line")
    ap.add_argument("--reuse", type=int, default=0,
                    help="extra mode (workloads with several rounds, e.g. C4): retrievals in this many sub-stages, with and "
                         "without the cache of the previous round and the reordering of the probe lists; prints its own JSON line")
    ap.add_argument("--graph", action="store_true",
                    help="replay the search from a captured HIP graph (one graph per round of the workload) instead of "
                         "enqueueing its kernels every step: for launch-bound small batches")
    ap.add_argument("--wide-only", type=int, default=0,
                    help="extra mode: the list scan over the lists that at least this many queries of the batch probe; "
                         "reports flops / time against the MFMA peak; prints its own JSON line")
    ap.add_argument("--narrow-only", type=int, default=0,
                    help="extra mode: the list scan over the lists that fewer than this many queries probe; reports bytes / "
                         "time against the HBM peak; prints its own JSON line")
    ap.add_argument("--row-tables", action="store_true",
                    help="load float32 / bfloat16 lists with HR_LOAD_ROW_TABLES (binary16 row tables: as many bytes again)")
    ap.add_argument("--flush-mb", type=int, default=0,
                    help="write this many MB of scratch between the timed calls (512 evicts the last-level cache, for batches "
                         "small enough to stay in it); each call is then timed by its own pair of events")
    ap.add_argument("--noise", type=float, default=0.0, help="spread of vectors and queries around their centroid instead of the workload's own")
    ap.add_argument("--drift", type=float, default=0.0, help="step of a query from round to round instead of the workload's own")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    import paper_2507_09138_amd as hr
    import synth

    cfg = synth.CONFIGS[args.workload]
    if args.nq > 0:
        cfg = synth.scaled(cfg, nq=args.nq)
    if args.nprobe > 0:
        cfg = synth.scaled(cfg, nprobe=args.nprobe)
    if args.noise > 0:
        cfg = synth.scaled(cfg, noise=args.noise)
    if args.drift > 0:
        cfg = synth.scaled(cfg, drift=args.drift)
    torch.cuda.set_device(0)
    idx = synth.make_index(cfg, "cuda")
    rounds = synth.make_queries(cfg, idx)
    ix = hr.IvfIndex(idx.centroids, idx.list_offsets, idx.list_vectors, idx.list_ids, row_tables=args.row_tables)
    nq = cfg.nq
    metric = hr.HR_METRIC_IP if cfg.metric == "ip" else hr.HR_METRIC_L2
    ids = torch.empty(nq, cfg.k, dtype=torch.int64, device="cuda")
    scores = torch.empty(nq, cfg.k, dtype=torch.float32, device="cuda")
    ws = ix.workspace(nq, cfg.nprobe, cfg.k)

    if args.wide_only > 0 or args.narrow_only > 0:
        return bench_width_split(args, cfg, hr, ix, idx, rounds, metric)
    if args.substages > 0:
        return bench_substages(args, cfg, hr, ix, rounds, metric)
    if args.reuse > 0:
        return bench_reuse(args, cfg, hr, ix, rounds, metric)

    def step(i):
        q = rounds[i % len(rounds)]
        hr.hr_ivf_search(ix.handle, q, nq, cfg.nprobe, cfg.k, metric, ids, scores, ws, ws.numel())

    if args.graph:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.synchronize()
        graphs = []
        for r in range(len(rounds)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                step(r)
            graphs.append(g)
        eager_step = step

        def step(i):
            graphs[i % len(graphs)].replay()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    hr.hr_ivf_profile_begin(ix.handle, args.steps)
    if args.flush_mb > 0:
        scratch = torch.empty(args.flush_mb << 20, dtype=torch.uint8, device="cuda")
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for i in range(args.steps):
            scratch.fill_(i & 255)
            evs[i][0].record()
            step(i)
            evs[i][1].record()
        torch.cuda.synchronize()
        dt = sum(a.elapsed_time(b) for a, b in evs) * 1e-3
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    n_timed, scan_ms = hr.hr_ivf_profile_end(ix.handle)
    if args.graph:
        # (the library records its events when it enqueues the kernel; a replayed graph enqueues
        # nothing, so the list scan is timed in a pass of eager calls after the timed region)
        hr.hr_ivf_profile_begin(ix.handle, args.steps)
        for i in range(args.steps):
            eager_step(i)
        torch.cuda.synchronize()
        n_timed, scan_ms = hr.hr_ivf_profile_end(ix.handle)
    ms_per_step = dt / args.steps * 1e3
    st = ix.stats(nq, cfg.nprobe, cfg.k)

    # work of the last step, from its probe lists (host arithmetic on the coarse output)
    probe, _ = ix.coarse(rounds[(args.steps - 1) % len(rounds)], cfg.nprobe, cfg.metric)
    w = torch.bincount(probe.flatten().long(), minlength=cfg.nlist).cpu()
    lens = idx.list_offsets[1:] - idx.list_offsets[:-1]
    pair_rows = int((w * lens).sum())
    rows_streamed = int(lens[w > 0].sum())
    assert rows_streamed == st["rows_streamed"], (rows_streamed, st)
    scan_bytes = rows_streamed * cfg.d * ESIZE[cfg.dtype]
    scan_flops = 2.0 * cfg.d * pair_rows
    # flops the matrix pipes execute for them: a wave's MFMA covers 16 columns = 16 queries (binary16 operands) or 8
    # queries in hi and lo parts (bfloat16 rows as stored; float32 rows, which also come as two planes), whether or
    # not all of them belong to the bucket (the 16-row padding of a segment's last block is not counted)
    gran, mult = (16, 1) if operand_name(cfg, ix) == "f16" else ((8, 2) if cfg.dtype == "bf16" else (8, 4))
    executed_rows = int((((w + gran - 1) // gran) * gran * lens).sum()) * mult
    achieved = scan_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0

    own_shape = args.nq == 0 and args.nprobe == 0 and args.noise == 0 and args.drift == 0
    traffic, traffic_src = traffic_from_profiles(cfg, args.row_tables) if own_shape else (None, None)
    out = {
        "metric": "queries/sec batched IVF top-k search", "value": nq / (ms_per_step * 1e-3),
        "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": operand_name(cfg, ix),      # MFMA operand type; float32 accumulation
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={cfg.N}, d={cfg.d}, nlist={cfg.nlist}, nq={nq}, "
                               f"nprobe={cfg.nprobe}, k={cfg.k}, {cfg.dtype} storage, {cfg.metric}",
                   "row_tables": bool(args.row_tables and cfg.dtype != "f16"), "rounds": cfg.rounds, "launch": "hip graph replay" if args.graph else "eager", "cache_flushed_between_calls_mb": args.flush_mb, "scan_items": st["items"], "seg_rows": st["seg_rows"],
                   "pairs": st["pairs"], "workspace_mb": round(ws.numel() / 2**20, 1)},
        "roofline": {"bound": "hbm", "kernel": "k_scan (list scan)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_src, "scan_ms_avg": scan_ms, "launches_timed": n_timed,
                     "algorithmic_bytes_per_launch": scan_bytes,
                     "mfma_tflops": scan_flops / (scan_ms * 1e-3) / 1e12 if scan_ms > 0 else 0.0,
                     "mfma_frac": (scan_flops / (scan_ms * 1e-3) / 1e12 / mfma_peak(cfg, ix)) if scan_ms > 0 else 0.0,
                     "mfma_peak_tflops": mfma_peak(cfg, ix),
                     "mfma_flops_executed_over_algorithmic": executed_rows / max(pair_rows, 1)},
    }
    if len(rounds) > 1:
        # every round of the workload timed as a call of its own (three passes over the rounds, after the timed region)
        per = [[] for _ in rounds]
        for _ in range(3):
            for r in range(len(rounds)):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                (eager_step if args.graph else step)(r)
                e1.record()
                torch.cuda.synchronize()
                per[r].append(e0.elapsed_time(e1))
        out["config"]["per_round_ms"] = [round(min(x), 4) for x in per]
    if not args.no_cpu_baseline:
        # (the result of the last timed step, for the comparison with the oracle on the sampled queries)
        last = (args.steps - 1) % len(rounds)
        out["cpu_baseline"] = cpu_baseline(cfg, idx, rounds[last], ids.cpu().numpy(), scores.cpu().numpy())
    ix.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
