"""ctypes binding with the same names as the C entry points of hr_ivf.h.

The low-level functions take raw addresses / torch tensors and return the C return code's
meaning as an exception (HrError) when it is not HR_OK.  ``IvfIndex`` is a small convenience
wrapper that keeps the borrowed tensors alive and owns a workspace tensor.

The library must have been built (``python -m paper_2507_09138_amd.build``); there is no
fallback: if ``libhr_ivf.so`` is missing, importing this module raises.
"""
import ctypes
import os

import torch

HR_METRIC_IP, HR_METRIC_L2 = 0, 1
HR_F32, HR_F16, HR_BF16 = 0, 1, 2
HR_K_MAX, HR_NPROBE_MAX = 128, 512
HR_LOAD_ROW_TABLES = 0x100
HR_STATIC_SCRATCH_BYTES = 64 << 20
_ERR = {-1: "HR_ERR_ARG", -2: "HR_ERR_HANDLE", -3: "HR_ERR_WORKSPACE", -4: "HR_ERR_HIP",
        -5: "HR_ERR_UNSUPPORTED"}
_DTYPE = {torch.float32: HR_F32, torch.float16: HR_F16, torch.bfloat16: HR_BF16}
_METRIC = {"ip": HR_METRIC_IP, "l2": HR_METRIC_L2, 0: 0, 1: 1}

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libhr_ivf.so")


class HrError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{_ERR.get(code, code)}: {msg}")
        self.code = code


def _load_lib():
    if not os.path.exists(lib_path):
        raise ImportError(f"{lib_path} not built; run `python -m paper_2507_09138_amd.build`")
    L = ctypes.CDLL(lib_path)
    c, p = ctypes, ctypes.c_void_p
    L.hr_ivf_load.argtypes = [p, p, p, p, c.c_int64, c.c_int64, c.c_int32, c.c_int32, p, c.POINTER(p)]
    L.hr_ivf_free.argtypes = [p]
    L.hr_ivf_workspace_bytes.argtypes = [p, c.c_int64, c.c_int32, c.c_int32]
    L.hr_ivf_workspace_bytes.restype = c.c_size_t
    L.hr_ivf_search.argtypes = [p, p, c.c_int64, c.c_int32, c.c_int32, c.c_int32, p, p, p, c.c_size_t, p]
    L.hr_ivf_search_static.argtypes = [p, p, c.c_int64, c.c_int32, c.c_int32, c.c_int32, p, p, p]
    L.hr_ivf_coarse.argtypes = [p, p, c.c_int64, c.c_int32, c.c_int32, p, p, p, c.c_size_t, p]
    L.hr_ivf_scan.argtypes = [p, p, c.c_int64, p, c.c_int32, c.c_int32, c.c_int32, p, p, p, c.c_size_t, p]
    L.hr_ivf_list_hits.argtypes = [p, p, c.c_int32, p]
    L.hr_ivf_hot_lists.argtypes = [p, c.c_int32, p, p]
    L.hr_ivf_set_resident.argtypes = [p, p, c.c_int64, c.c_int32, p]
    L.hr_ivf_split_probes.argtypes = [p, p, c.c_int64, c.c_int32, p, p, p]
    L.hr_ivf_refresh_rows.argtypes = [p, c.c_int64, c.c_int64, p]
    L.hr_ivf_scan_step.argtypes = [p, p, c.c_int64, p, c.c_int32, c.c_int32, c.c_int32, p, p, p, c.c_size_t, p]
    L.hr_ivf_scan_step_rows.argtypes = [p, p, c.c_int64, p, c.c_int32, c.c_int32, c.c_int32, p, p, p, p, c.c_size_t, p]
    L.hr_ivf_rescore.argtypes = [p, p, c.c_int64, p, c.c_int32, c.c_int32, c.c_int32, p, p, p, p]
    L.hr_ivf_lists_of_rows.argtypes = [p, p, c.c_int64, p, p]
    L.hr_ivf_reorder_probes.argtypes = [p, c.c_int64, c.c_int32, p, c.c_int32, p, c.c_int32, p, p]
    L.hr_ivf_workspace_layout.argtypes = [p, c.c_int64, c.c_int32, c.c_int32, c.POINTER(c.c_int64), c.c_int32, c.POINTER(c.c_int32)]
    L.hr_ivf_stats.argtypes = [p, p, c.c_size_t, c.c_int64, c.c_int32, c.c_int32, c.POINTER(c.c_int64)]
    L.hr_ivf_profile_begin.argtypes = [p, c.c_int32]
    L.hr_ivf_profile_end.argtypes = [p, c.POINTER(c.c_int32), c.POINTER(c.c_double)]
    L.hr_last_error.restype = c.c_char_p
    L.hr_version.restype = c.c_char_p
    return L


lib = _load_lib()


def hr_last_error():
    return lib.hr_last_error().decode()


def hr_version():
    return lib.hr_version().decode()


def _check(rc):
    if rc != 0:
        raise HrError(rc, hr_last_error())


def _addr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def hr_ivf_load(centroids, list_offsets, list_vectors, list_ids, nlist, N, d, dtype, stream=None):
    """list_offsets: host int64 tensor; the others device tensors (or raw addresses)."""
    h = ctypes.c_void_p()
    _check(lib.hr_ivf_load(_addr(centroids), _addr(list_offsets), _addr(list_vectors),
                           _addr(list_ids), nlist, N, d, dtype, _stream(stream), ctypes.byref(h)))
    return h


def hr_ivf_free(handle):
    _check(lib.hr_ivf_free(handle))


def hr_ivf_workspace_bytes(handle, nq, nprobe, k):
    return int(lib.hr_ivf_workspace_bytes(handle, nq, nprobe, k))


def hr_ivf_search(handle, queries, nq, nprobe, k, metric, out_ids, out_scores, workspace,
                  workspace_bytes, stream=None):
    _check(lib.hr_ivf_search(handle, _addr(queries), nq, nprobe, k, metric, _addr(out_ids),
                             _addr(out_scores), _addr(workspace), workspace_bytes, _stream(stream)))


def hr_ivf_search_static(handle, queries, nq, nprobe, k, metric, out_ids, out_scores, stream=None):
    _check(lib.hr_ivf_search_static(handle, _addr(queries), nq, nprobe, k, metric, _addr(out_ids),
                                    _addr(out_scores), _stream(stream)))


def hr_ivf_coarse(handle, queries, nq, nprobe, metric, out_probe_ids, out_probe_scores, workspace,
                  workspace_bytes, stream=None):
    _check(lib.hr_ivf_coarse(handle, _addr(queries), nq, nprobe, metric, _addr(out_probe_ids),
                             _addr(out_probe_scores), _addr(workspace), workspace_bytes,
                             _stream(stream)))


def hr_ivf_scan(handle, queries, nq, probe_ids, nprobe, k, metric, out_ids, out_scores, workspace,
                workspace_bytes, stream=None):
    _check(lib.hr_ivf_scan(handle, _addr(queries), nq, _addr(probe_ids), nprobe, k, metric,
                           _addr(out_ids), _addr(out_scores), _addr(workspace), workspace_bytes,
                           _stream(stream)))


def hr_ivf_scan_step(handle, queries, nq, probe_ids, nprobe, k, metric, io_ids, io_scores, workspace,
                     workspace_bytes, stream=None):
    _check(lib.hr_ivf_scan_step(handle, _addr(queries), nq, _addr(probe_ids), nprobe, k, metric,
                                _addr(io_ids), _addr(io_scores), _addr(workspace), workspace_bytes,
                                _stream(stream)))


def hr_ivf_scan_step_rows(handle, queries, nq, probe_ids, nprobe, k, metric, io_ids, io_scores, io_rows, workspace,
                          workspace_bytes, stream=None):
    _check(lib.hr_ivf_scan_step_rows(handle, _addr(queries), nq, _addr(probe_ids), nprobe, k, metric,
                                     _addr(io_ids), _addr(io_scores), _addr(io_rows), _addr(workspace),
                                     workspace_bytes, _stream(stream)))


def hr_ivf_rescore(handle, queries, nq, rows, m, k, metric, out_ids, out_scores, out_rows, stream=None):
    _check(lib.hr_ivf_rescore(handle, _addr(queries), nq, _addr(rows), m, k, metric, _addr(out_ids),
                              _addr(out_scores), _addr(out_rows), _stream(stream)))


def hr_ivf_lists_of_rows(handle, rows, n, out_lists, stream=None):
    _check(lib.hr_ivf_lists_of_rows(handle, _addr(rows), n, _addr(out_lists), _stream(stream)))


def hr_ivf_reorder_probes(probe, nq, nprobe, prev, nprev, hot, nhot, out_probe, stream=None):
    _check(lib.hr_ivf_reorder_probes(_addr(probe), nq, nprobe, _addr(prev) if prev is not None else None, nprev,
                                     _addr(hot) if hot is not None else None, nhot, _addr(out_probe),
                                     _stream(stream)))


def hr_ivf_list_hits(handle, out_hits, reset=False, stream=None):
    _check(lib.hr_ivf_list_hits(handle, _addr(out_hits), 1 if reset else 0, _stream(stream)))


def hr_ivf_hot_lists(handle, gc, out_lists, stream=None):
    _check(lib.hr_ivf_hot_lists(handle, gc, _addr(out_lists), _stream(stream)))


def hr_ivf_set_resident(handle, lists, n, resident, stream=None):
    _check(lib.hr_ivf_set_resident(handle, _addr(lists), n, 1 if resident else 0, _stream(stream)))


def hr_ivf_split_probes(handle, probe_ids, nq, nprobe, out_resident, out_missing, stream=None):
    _check(lib.hr_ivf_split_probes(handle, _addr(probe_ids), nq, nprobe, _addr(out_resident), _addr(out_missing),
                                   _stream(stream)))


def hr_ivf_refresh_rows(handle, row_begin, row_end, stream=None):
    _check(lib.hr_ivf_refresh_rows(handle, row_begin, row_end, _stream(stream)))


def hr_ivf_workspace_layout(handle, nq, nprobe, k):
    """[(offset, bytes)] of the regions of a workspace for this batch shape."""
    out = (ctypes.c_int64 * 64)()
    n = ctypes.c_int32()
    _check(lib.hr_ivf_workspace_layout(handle, nq, nprobe, k, out, 32, ctypes.byref(n)))
    return [(out[2 * i], out[2 * i + 1]) for i in range(min(n.value, 32))]


def hr_ivf_stats(handle, workspace, workspace_bytes, nq, nprobe, k):
    out = (ctypes.c_int64 * 4)()
    _check(lib.hr_ivf_stats(handle, _addr(workspace), workspace_bytes, nq, nprobe, k, out))
    return {"items": out[0], "seg_rows": out[1], "rows_streamed": out[2], "pairs": out[3]}


def hr_ivf_profile_begin(handle, max_calls):
    _check(lib.hr_ivf_profile_begin(handle, max_calls))


def hr_ivf_profile_end(handle):
    n = ctypes.c_int32()
    ms = ctypes.c_double()
    _check(lib.hr_ivf_profile_end(handle, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value


def _want(t, name, dtype, shape, device):
    """The kernels read raw addresses: a tensor of another type, shape or device would be read out of bounds.
    shape entries that are None are free.  Raises HrError(HR_ERR_ARG) before anything reaches the library."""
    if not isinstance(t, torch.Tensor):
        raise HrError(-1, f"{name} must be a torch tensor")
    if t.device != device:
        raise HrError(-1, f"{name} is on {t.device}, the index is on {device}")
    if t.dtype != dtype:
        raise HrError(-1, f"{name} has dtype {t.dtype}, want {dtype}")
    if t.dim() != len(shape) or any(w is not None and int(g) != int(w) for g, w in zip(t.shape, shape)):
        raise HrError(-1, f"{name} has shape {tuple(t.shape)}, want {tuple('*' if w is None else w for w in shape)}")
    return t.contiguous()


def _want_int(t, name, shape, device):
    """Integer tensors of list or row numbers: any integer type is converted to int32 on the way."""
    if not isinstance(t, torch.Tensor) or t.dtype not in (torch.int32, torch.int64, torch.int16, torch.int8, torch.uint8):
        raise HrError(-1, f"{name} must be an integer tensor")
    return _want(t.to(torch.int32), name, torch.int32, shape, device)


def _want_range(v, name, lo, hi):
    if not (lo <= int(v) <= hi):
        raise HrError(-1, f"{name}={int(v)} must be in {lo}..{hi}")
    return int(v)


class IvfIndex:
    """Keeps the borrowed tensors alive, owns the handle and a growable workspace tensor."""

    def __init__(self, centroids, list_offsets, list_vectors, list_ids, row_tables=False):
        """row_tables: also keep float32 / bfloat16 rows as binary16 tables (as many bytes again) that the scan
        reads instead: HR_LOAD_ROW_TABLES of hr_ivf_load."""
        for t, name in ((centroids, "centroids"), (list_vectors, "list_vectors"), (list_ids, "list_ids")):
            if not isinstance(t, torch.Tensor) or not t.is_cuda:
                raise HrError(-1, f"{name} must be a device tensor")
        if list_vectors.dtype not in _DTYPE:
            raise HrError(-1, f"list_vectors has dtype {list_vectors.dtype}, want float32, float16 or bfloat16")
        self.device = centroids.device
        _want(centroids, "centroids", torch.float32, (None, None), self.device)
        _want(list_vectors, "list_vectors", list_vectors.dtype, (None, centroids.shape[1]), self.device)
        _want(list_ids, "list_ids", torch.int64, (list_vectors.shape[0],), self.device)
        if not isinstance(list_offsets, torch.Tensor) or list_offsets.dim() != 1 or list_offsets.numel() != centroids.shape[0] + 1:
            raise HrError(-1, "list_offsets must be a tensor of nlist + 1 entries")
        self.centroids = centroids.contiguous()
        self.list_offsets = list_offsets.to("cpu", torch.int64).contiguous()
        self.list_vectors = list_vectors.contiguous()
        self.list_ids = list_ids.contiguous()
        self.nlist, self.d = self.centroids.shape
        self.N = self.list_vectors.shape[0]
        self.dtype = _DTYPE[self.list_vectors.dtype]
        self.row_tables = bool(row_tables)
        self.handle = hr_ivf_load(self.centroids, self.list_offsets, self.list_vectors,
                                  self.list_ids, self.nlist, self.N, self.d,
                                  self.dtype | (HR_LOAD_ROW_TABLES if row_tables else 0))
        self._ws = None

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            hr_ivf_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, nq, nprobe, k):
        need = hr_ivf_workspace_bytes(self.handle, nq, nprobe, k)
        if need == 0 and nq > 0:
            raise HrError(-1, hr_last_error())
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.centroids.device)
        return self._ws

    def _queries(self, queries, nq=None):
        return _want(queries, "queries", torch.float32, (nq, self.d), self.device)

    def _state(self, state, nq, rows):
        """A carried result (ids, scores[, rows]) of nq queries; returns it with k."""
        if len(state) != (3 if rows else 2):
            raise HrError(-1, "state must be (ids, scores, rows)" if rows else "state must be (ids, scores)")
        ids = state[0]
        if not isinstance(ids, torch.Tensor) or ids.dim() != 2:
            raise HrError(-1, "state ids must be a [nq, k] tensor")
        k = _want_range(ids.shape[1], "k", 1, HR_K_MAX)
        for t, name, dt in zip(state, ("state ids", "state scores", "state rows"), (torch.int64, torch.float32, torch.int32)):
            _want(t, name, dt, (nq, k), self.device)
            if not t.is_contiguous():
                raise HrError(-1, f"{name} must be contiguous (it is updated in place)")
        return k

    def search(self, queries, nprobe, k, metric="ip"):
        q = self._queries(queries)
        nq = q.shape[0]
        ids = torch.empty(nq, k, dtype=torch.int64, device=q.device)
        scores = torch.empty(nq, k, dtype=torch.float32, device=q.device)
        ws = self.workspace(nq, nprobe, k)
        hr_ivf_search(self.handle, q, nq, nprobe, k, _METRIC[metric], ids, scores, ws, ws.numel())
        return ids, scores

    def coarse(self, queries, nprobe, metric="ip"):
        q = self._queries(queries)
        nq = q.shape[0]
        probe = torch.empty(nq, nprobe, dtype=torch.int32, device=q.device)
        scores = torch.empty(nq, nprobe, dtype=torch.float32, device=q.device)
        ws = self.workspace(nq, nprobe, 1)
        hr_ivf_coarse(self.handle, q, nq, nprobe, _METRIC[metric], probe, scores, ws, ws.numel())
        return probe, scores

    def scan(self, queries, probe_ids, k, metric="ip"):
        q = self._queries(queries)
        pr = _want_int(probe_ids, "probe_ids", (q.shape[0], None), self.device)
        nq, nprobe = pr.shape
        ids = torch.empty(nq, k, dtype=torch.int64, device=q.device)
        scores = torch.empty(nq, k, dtype=torch.float32, device=q.device)
        ws = self.workspace(nq, nprobe, k)
        hr_ivf_scan(self.handle, q, nq, pr, nprobe, k, _METRIC[metric], ids, scores, ws, ws.numel())
        return ids, scores

    def new_state(self, nq, k):
        """An empty carried result for scan_step: ids -1."""
        return (torch.full((nq, k), -1, dtype=torch.int64, device=self.device),
                torch.zeros(nq, k, dtype=torch.float32, device=self.device))

    def new_state_rows(self, nq, k):
        """An empty carried result with row numbers, for scan_step_rows."""
        return self.new_state(nq, k) + (torch.full((nq, k), -1, dtype=torch.int32, device=self.device),)

    def scan_step(self, queries, probe_ids, state, metric="ip"):
        """One sub-stage: merges the lists in probe_ids into the carried result (ids, scores), in place."""
        q = self._queries(queries)
        pr = _want_int(probe_ids, "probe_ids", (q.shape[0], None), self.device)
        nq, nprobe = pr.shape
        k = self._state(state, nq, False)
        ids, scores = state
        ws = self.workspace(nq, nprobe, k)
        hr_ivf_scan_step(self.handle, q, nq, pr, nprobe, k, _METRIC[metric], ids, scores, ws, ws.numel())
        return ids, scores

    def scan_step_rows(self, queries, probe_ids, state, metric="ip"):
        """scan_step on a carried result (ids, scores, rows) that also holds the row number of every entry."""
        q = self._queries(queries)
        pr = _want_int(probe_ids, "probe_ids", (q.shape[0], None), self.device)
        nq, nprobe = pr.shape
        k = self._state(state, nq, True)
        ids, scores, rows = state
        ws = self.workspace(nq, nprobe, k)
        hr_ivf_scan_step_rows(self.handle, q, nq, pr, nprobe, k, _METRIC[metric], ids, scores, rows, ws, ws.numel())
        return ids, scores, rows

    def rescore(self, queries, rows, k, metric="ip"):
        """The k best of the given rows [nq, m] for the queries: a carried result (ids, scores, rows)."""
        q = self._queries(queries)
        r = _want_int(rows, "rows", (q.shape[0], None), self.device)
        nq, m = r.shape
        _want_range(m, "m", 1, HR_K_MAX)
        _want_range(k, "k", 1, HR_K_MAX)
        ids = torch.empty(nq, k, dtype=torch.int64, device=q.device)
        scores = torch.empty(nq, k, dtype=torch.float32, device=q.device)
        out_rows = torch.empty(nq, k, dtype=torch.int32, device=q.device)
        hr_ivf_rescore(self.handle, q, nq, r, m, k, _METRIC[metric], ids, scores, out_rows)
        return ids, scores, out_rows

    def lists_of_rows(self, rows):
        if not isinstance(rows, torch.Tensor):
            raise HrError(-1, "rows must be a torch tensor")
        r = _want_int(rows, "rows", tuple(rows.shape), self.device)
        out = torch.empty_like(r)
        hr_ivf_lists_of_rows(self.handle, r, r.numel(), out)
        return out

    def list_hits(self, reset=False):
        """Probes per list since load / the last reset: int64 [nlist] on the device."""
        out = torch.empty(self.nlist, dtype=torch.int64, device=self.device)
        hr_ivf_list_hits(self.handle, out, reset)
        return out

    def hot_lists(self, gc):
        """The gc most frequently probed lists, most frequent first: int32 [gc] on the device."""
        out = torch.empty(_want_range(gc, "gc", 1, self.nlist), dtype=torch.int32, device=self.device)
        hr_ivf_hot_lists(self.handle, gc, out)
        return out

    def set_resident(self, lists, resident):
        """Mark the given lists (int tensor on the device, or None: all lists) as in place / not in place."""
        if lists is None:
            hr_ivf_set_resident(self.handle, None, 0, resident)
        else:
            ls = _want_int(lists, "lists", (None,), self.device)
            hr_ivf_set_resident(self.handle, ls, ls.numel(), resident)

    def split_probes(self, probe_ids):
        """(lists in place, lists not in place) of every row of probe_ids [nq, nprobe], each -1-padded."""
        pr = _want_int(probe_ids, "probe_ids", (None, None), self.device)
        _want_range(pr.shape[1], "nprobe", 1, HR_NPROBE_MAX)
        res, mis = torch.empty_like(pr), torch.empty_like(pr)
        hr_ivf_split_probes(self.handle, pr, pr.shape[0], pr.shape[1], res, mis)
        return res, mis

    def refresh_rows(self, row_begin, row_end):
        """After the vectors of these rows were replaced in place: recompute what is derived from them."""
        hr_ivf_refresh_rows(self.handle, row_begin, row_end)

    def stats(self, nq, nprobe, k):
        ws = self.workspace(nq, nprobe, k)
        return hr_ivf_stats(self.handle, ws, ws.numel(), nq, nprobe, k)


def reorder_probes(probe, prev=None, hot=None):
    """Search order of the probe lists [nq, nprobe]: lists in hot first, then those in prev, then the rest."""
    if not isinstance(probe, torch.Tensor) or not probe.is_cuda:
        raise HrError(-1, "probe must be a device tensor")
    pr = _want_int(probe, "probe", (None, None), probe.device)
    nq, nprobe = pr.shape
    _want_range(nprobe, "nprobe", 1, HR_NPROBE_MAX)
    pv = _want_int(prev, "prev", (nq, None), probe.device) if prev is not None else None
    ht = _want_int(hot, "hot", (nq, None), probe.device) if hot is not None else None
    if pv is not None:
        _want_range(pv.shape[1], "nprev", 0, HR_NPROBE_MAX)
    if ht is not None:
        _want_range(ht.shape[1], "nhot", 0, HR_K_MAX)
    out = torch.empty_like(pr)
    hr_ivf_reorder_probes(pr, nq, nprobe, pv, pv.shape[1] if pv is not None else 0, ht,
                          ht.shape[1] if ht is not None else 0, out)
    return out
