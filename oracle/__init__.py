"""CPU oracle for batched IVF-Flat search.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``ivf_oracle.c`` (plain C, double accumulation,
query-major; see the header of that file for the conventions and the passages
of the paper it follows).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It imports
nothing from the HIP package and the HIP package imports nothing from here.

Arrays are numpy.  Stored vectors are passed as ``float32``, ``float16`` or, for
bfloat16, as the ``uint16`` bit patterns together with ``dtype="bf16"``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivf_oracle.c")
_LIB = os.path.join(_HERE, "libivf_oracle.so")

IP, L2 = 0, 1
_DTYPES = {"f32": 0, "f16": 1, "bf16": 2}

_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math so that the
    summation order is the one written in the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        p = c.c_void_p
        lib.oracle_num_threads.restype = c.c_int
        lib.oracle_set_threads.argtypes = [c.c_int]
        lib.oracle_coarse.argtypes = [p, c.c_int64, p, c.c_int64, c.c_int, c.c_int, c.c_int, p, p]
        lib.oracle_scan.argtypes = [p, c.c_int64, c.c_int, p, c.c_int64, p, c.c_int, p, p,
                                    c.c_int, c.c_int, c.c_int, p, p]
        lib.oracle_ivf_search.argtypes = [p, c.c_int64, c.c_int, p, p, c.c_int64, p, c.c_int, p,
                                          c.c_int, c.c_int, c.c_int, p, p, p]
        lib.oracle_bruteforce.argtypes = [p, c.c_int64, c.c_int, p, c.c_int, p, c.c_int64,
                                          c.c_int, c.c_int, p, p]
        lib.oracle_pair_scores.argtypes = [p, c.c_int, p, c.c_int, c.c_int, p, p, c.c_int64, p]
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def set_threads(n):
    """Threads the query loops use from now on (timing on one core); results do not depend on it."""
    _load().oracle_set_threads(int(n))


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _as(a, dt):
    a = np.ascontiguousarray(a)
    if a.dtype != dt:
        raise TypeError(f"expected {dt}, got {a.dtype}")
    return a


def _vectors(vectors, dtype):
    code = _DTYPES[dtype]
    want = {0: np.float32, 1: np.float16, 2: np.uint16}[code]
    return _as(vectors, want), code


def _check(rc, name):
    if rc != 0:
        raise RuntimeError(f"{name} failed with code {rc}")


def coarse(queries, centroids, nprobe, metric):
    """Returns (probe_ids [nq,nprobe] int32 best-first, scores [nq,nprobe] float64)."""
    q = _as(queries, np.float32)
    c = _as(centroids, np.float32)
    nq, d = q.shape
    nlist = c.shape[0]
    assert c.shape[1] == d
    probe = np.empty((nq, nprobe), np.int32)
    sc = np.empty((nq, nprobe), np.float64)
    _check(_load().oracle_coarse(_ptr(q), nq, _ptr(c), nlist, d, metric, nprobe, _ptr(probe),
                                 _ptr(sc)), "oracle_coarse")
    return probe, sc


def scan(queries, offsets, vectors, dtype, ids, probe, k, metric):
    """Fine step with given probe lists.  Returns (ids [nq,k] int64, scores [nq,k] float64)."""
    q = _as(queries, np.float32)
    off = _as(offsets, np.int64)
    v, code = _vectors(vectors, dtype)
    lab = _as(ids, np.int64)
    pr = _as(probe, np.int32)
    nq, d = q.shape
    assert pr.shape[0] == nq and v.shape[1] == d and lab.shape[0] == v.shape[0]
    assert off[0] == 0 and off[-1] == v.shape[0]
    out_i = np.empty((nq, k), np.int64)
    out_s = np.empty((nq, k), np.float64)
    _check(_load().oracle_scan(_ptr(q), nq, d, _ptr(off), off.shape[0] - 1, _ptr(v), code,
                               _ptr(lab), _ptr(pr), pr.shape[1], k, metric, _ptr(out_i),
                               _ptr(out_s)), "oracle_scan")
    return out_i, out_s


def merge_topk(ids_a, scores_a, ids_b, scores_b, k, metric):
    """Carrying a result from one sub-stage of a retrieval to the next (Section 4.2 of the paper:
    a request's clusters are searched in several sub-stages): the k best of two partial results
    over disjoint sets of lists, in the order used everywhere (score best first, then id
    ascending); places with id -1 are empty.  Plain numpy, query by query."""
    nq = ids_a.shape[0]
    out_i = np.full((nq, k), -1, np.int64)
    out_s = np.full((nq, k), np.inf if metric == L2 else -np.inf, np.float64)
    for q in range(nq):
        ids = np.concatenate([ids_a[q], ids_b[q]]).astype(np.int64)
        sc = np.concatenate([scores_a[q], scores_b[q]]).astype(np.float64)
        keep = ids >= 0
        ids, sc = ids[keep], sc[keep]
        order = np.lexsort((ids, sc if metric == L2 else -sc))[:k]
        out_i[q, :len(order)] = ids[order]
        out_s[q, :len(order)] = sc[order]
    return out_i, out_s


def topk_of_rows(queries, vectors, dtype, ids, rows, k, metric):
    """The k best of a given set of rows per query, in the order used everywhere (score best
    first, then id ascending).  ``rows[q]`` is any sequence of row numbers; numbers < 0 or past
    the end mean "no row" and a row named twice counts once.  This is what searching a local
    cache of earlier results for a new query amounts to (Section 4.3 of the paper), and, over
    the union of such rows and the rows of probed lists, what a retrieval started from that
    cache must end with.  Returns (ids [nq,k] int64, scores [nq,k] float64, rows [nq,k] int64);
    empty places: -1, -inf (inner product) or +inf (L2), -1."""
    nq = len(rows)
    n = np.asarray(vectors).shape[0]
    out_i = np.full((nq, k), -1, np.int64)
    out_s = np.full((nq, k), np.inf if metric == L2 else -np.inf, np.float64)
    out_r = np.full((nq, k), -1, np.int64)
    for q in range(nq):
        r = np.unique(np.asarray(rows[q], np.int64))
        r = r[(r >= 0) & (r < n)]
        if r.size == 0:
            continue
        sc = pair_scores(queries, vectors, dtype, metric, np.full(r.size, q), r)
        lab = np.asarray(ids)[r].astype(np.int64) if ids is not None else r
        order = np.lexsort((lab, sc if metric == L2 else -sc))[:k]
        out_i[q, :order.size] = lab[order]
        out_s[q, :order.size] = sc[order]
        out_r[q, :order.size] = r[order]
    return out_i, out_s, out_r


def lists_of_rows(rows, offsets):
    """The list each row belongs to: the l with offsets[l] <= row < offsets[l+1]; -1 for rows
    outside the index.  (H_v of Section 4.3: the clusters that held the results of v.)"""
    rows = np.asarray(rows, np.int64)
    off = np.asarray(offsets, np.int64)
    out = np.searchsorted(off, rows, side="right") - 1
    out[(rows < 0) | (rows >= off[-1])] = -1
    return out.astype(np.int64)


def reorder_probes(probe, prev, hot):
    """Search order of the new probe lists C' (Section 4.3 of the paper): first the lists of C'
    that are in H_v (``hot``), then those in (C - H_v) (``prev`` without ``hot``), then the
    remaining ones; inside each group the given order stays.  Entries < 0 are "no list": they
    go last, and are ignored in ``prev`` and ``hot``.  Plain Python, query by query."""
    probe = np.asarray(probe)
    out = np.empty_like(probe)
    for q in range(probe.shape[0]):
        h = set(int(x) for x in (hot[q] if hot is not None else []) if x >= 0)
        c = set(int(x) for x in (prev[q] if prev is not None else []) if x >= 0)
        row = [int(x) for x in probe[q]]
        first = [l for l in row if l >= 0 and l in h]
        second = [l for l in row if l >= 0 and l not in h and l in c]
        rest = [l for l in row if l >= 0 and l not in h and l not in c]
        absent = [l for l in row if l < 0]
        out[q] = first + second + rest + absent
    return out


def hot_lists(hits, gc):
    """The gc most frequently probed lists (Section 4.4 of the paper: the clusters accessed most
    often are the ones a partial index cache keeps), most frequent first, equal counts by
    ascending list number."""
    hits = np.asarray(hits, np.int64)
    return np.lexsort((np.arange(hits.size), -hits))[:gc].astype(np.int64)


def split_probes(probe, resident):
    """Partial residency (Section 4.4 of the paper: only some clusters are kept where the search runs; the others
    are searched elsewhere): every row of ``probe`` split into the lists that are resident (``resident[l]`` true) and
    the others, each part in the given order and padded with -1; entries outside 0..nlist-1 go to neither.  Plain
    Python, row by row."""
    probe = np.asarray(probe)
    nlist = len(resident)
    res = np.full_like(probe, -1)
    mis = np.full_like(probe, -1)
    for q in range(probe.shape[0]):
        a = [int(l) for l in probe[q] if 0 <= l < nlist and resident[l]]
        b = [int(l) for l in probe[q] if 0 <= l < nlist and not resident[l]]
        res[q, :len(a)] = a
        mis[q, :len(b)] = b
    return res, mis


def ivf_search(queries, centroids, offsets, vectors, dtype, ids, nprobe, k, metric):
    """Whole search.  Returns (probe_ids, ids, scores)."""
    q = _as(queries, np.float32)
    c = _as(centroids, np.float32)
    off = _as(offsets, np.int64)
    v, code = _vectors(vectors, dtype)
    lab = _as(ids, np.int64)
    nq, d = q.shape
    nlist = c.shape[0]
    assert off.shape[0] == nlist + 1 and off[0] == 0 and off[-1] == v.shape[0]
    probe = np.empty((nq, nprobe), np.int32)
    out_i = np.empty((nq, k), np.int64)
    out_s = np.empty((nq, k), np.float64)
    _check(_load().oracle_ivf_search(_ptr(q), nq, d, _ptr(c), _ptr(off), nlist, _ptr(v), code,
                                     _ptr(lab), nprobe, k, metric, _ptr(probe), _ptr(out_i),
                                     _ptr(out_s)), "oracle_ivf_search")
    return probe, out_i, out_s


def bruteforce(queries, vectors, dtype, ids, k, metric):
    """Exact search over all rows.  Returns (ids [nq,k], scores [nq,k] float64)."""
    q = _as(queries, np.float32)
    v, code = _vectors(vectors, dtype)
    lab = _as(ids, np.int64)
    nq, d = q.shape
    out_i = np.empty((nq, k), np.int64)
    out_s = np.empty((nq, k), np.float64)
    _check(_load().oracle_bruteforce(_ptr(q), nq, d, _ptr(v), code, _ptr(lab), v.shape[0], k,
                                     metric, _ptr(out_i), _ptr(out_s)), "oracle_bruteforce")
    return out_i, out_s


def pair_scores(queries, vectors, dtype, metric, qidx, ridx):
    """Scores of chosen (query, row) pairs, float64."""
    q = _as(queries, np.float32)
    v, code = _vectors(vectors, dtype)
    qi = _as(np.asarray(qidx, np.int64), np.int64)
    ri = _as(np.asarray(ridx, np.int64), np.int64)
    out = np.empty(qi.shape[0], np.float64)
    _check(_load().oracle_pair_scores(_ptr(q), q.shape[1], _ptr(v), code, metric, _ptr(qi),
                                      _ptr(ri), qi.shape[0], _ptr(out)), "oracle_pair_scores")
    return out
