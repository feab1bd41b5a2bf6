"""The C-ABI library loads, exports every symbol the header declares, and validates arguments
on the host (no GPU needed for any of this)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hr():
    import paper_2507_09138_amd as hr
    if not os.path.exists(hr.lib_path):
        from paper_2507_09138_amd import build
        build.build()
    return hr


def test_every_declared_symbol_is_exported(hr):
    text = open(os.path.join(ROOT, "include", "hr_ivf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(hr_[a-z0-9_]+)\s*\(", text))
    assert {"hr_ivf_load", "hr_ivf_search", "hr_ivf_coarse", "hr_ivf_scan", "hr_ivf_scan_step", "hr_ivf_free",
            "hr_ivf_workspace_bytes", "hr_last_error"} <= names
    for n in names:
        assert hasattr(hr.lib, n), n
    assert hr.hr_version().startswith("hr_ivf")


def test_header_constants_match_binding(hr):
    text = open(os.path.join(ROOT, "include", "hr_ivf.h")).read()
    assert int(re.search(r"#define HR_K_MAX (\d+)", text).group(1)) == hr.HR_K_MAX
    assert int(re.search(r"#define HR_NPROBE_MAX (\d+)", text).group(1)) == hr.HR_NPROBE_MAX
    assert int(re.search(r"#define HR_LOAD_ROW_TABLES (0x[0-9a-f]+)", text).group(1), 16) == hr.HR_LOAD_ROW_TABLES


def test_load_argument_validation_on_host(hr):
    h = ctypes.c_void_p()
    P = ctypes.c_void_p
    off = np.array([0, 3, 5], np.int64)
    bad = np.array([0, 6, 5], np.int64)
    fake = P(4096)                                  # never dereferenced: validation fails first

    def load(cent=fake, offs=off, vec=fake, ids=fake, nlist=2, N=5, d=768, dtype=0):
        return hr.lib.hr_ivf_load(cent, P(offs.ctypes.data) if offs is not None else None, vec, ids,
                                  nlist, N, d, dtype, None, ctypes.byref(h))

    assert load(cent=None) == -1
    assert load(offs=None) == -1
    assert load(vec=None) == -1
    assert load(nlist=0) == -1
    assert load(N=-1) == -1
    assert load(N=1 << 31) == -1
    assert load(dtype=3) == -1
    assert load(dtype=3 | hr.HR_LOAD_ROW_TABLES) == -1
    assert load(d=0) == -1
    assert load(d=100) == -5 and "d=100" in hr.hr_last_error()
    assert load(offs=bad) == -1 and "decreases" in hr.hr_last_error()
    assert load(N=4) == -1
    assert h.value is None
    assert hr.lib.hr_ivf_load(fake, P(off.ctypes.data), fake, fake, 2, 5, 768, 0, None, None) == -1


def test_null_handle_is_rejected(hr):
    assert hr.lib.hr_ivf_free(None) == -2
    assert hr.lib.hr_ivf_workspace_bytes(None, 10, 4, 4) == 0
    assert hr.lib.hr_ivf_search(None, None, 1, 1, 1, 0, None, None, None, 0, None) == -2
    assert hr.lib.hr_ivf_coarse(None, None, 1, 1, 0, None, None, None, 0, None) == -2
    assert hr.lib.hr_ivf_scan(None, None, 1, None, 1, 1, 0, None, None, None, 0, None) == -2
    assert hr.lib.hr_ivf_scan_step(None, None, 1, None, 1, 1, 0, None, None, None, 0, None) == -2
    assert hr.lib.hr_ivf_scan_step_rows(None, None, 1, None, 1, 1, 0, None, None, None, None, 0, None) == -2
    assert hr.lib.hr_ivf_rescore(None, None, 1, None, 1, 1, 0, None, None, None, None) == -2
    assert hr.lib.hr_ivf_lists_of_rows(None, None, 1, None, None) == -2
    assert hr.lib.hr_ivf_hot_lists(None, 1, None, None) == -2
    assert hr.lib.hr_ivf_refresh_rows(None, 0, 0, None) == -2
    assert hr.lib.hr_ivf_set_resident(None, None, 0, 1, None) == -2
    assert hr.lib.hr_ivf_workspace_layout(None, 1, 1, 1, None, 0, None) == -2
    assert hr.lib.hr_ivf_split_probes(None, None, 1, 1, None, None, None) == -2
    assert hr.lib.hr_ivf_search_static(None, None, 1, 1, 1, 0, None, None, None) == -2
    bogus = (ctypes.c_uint64 * 64)()                 # memory that is not an index
    assert hr.lib.hr_ivf_free(ctypes.cast(bogus, ctypes.c_void_p)) == -2


def test_reorder_argument_validation_on_host(hr):
    P = ctypes.c_void_p
    fake, other = P(4096), P(8192)                  # never dereferenced: validation fails first
    f = hr.lib.hr_ivf_reorder_probes
    assert f(fake, 4, 0, None, 0, None, 0, other, None) == -1
    assert f(fake, 4, hr.HR_NPROBE_MAX + 1, None, 0, None, 0, other, None) == -1
    assert f(fake, 4, 8, fake, hr.HR_NPROBE_MAX + 1, None, 0, other, None) == -1
    assert f(fake, 4, 8, None, 0, fake, hr.HR_K_MAX + 1, other, None) == -1
    assert f(None, 4, 8, None, 0, None, 0, other, None) == -1
    assert f(fake, 4, 8, None, 0, None, 0, fake, None) == -1 and "must not be probe" in hr.hr_last_error()
    assert f(fake, 0, 8, None, 0, None, 0, other, None) == 0      # empty batch: nothing to do



def test_binding_rejects_tensors_the_kernels_would_read_out_of_bounds(hr):
    """The binding hands raw addresses to the kernels; a tensor on the host, of another type or of another shape
    must be refused before that (no GPU needed: the checks run first)."""
    import torch
    from paper_2507_09138_amd import binding as b
    cpu = torch.device("cpu")
    ok = torch.zeros(5, 64)
    assert b._want(ok, "queries", torch.float32, (None, 64), cpu).shape == (5, 64)
    for bad in (torch.zeros(5, 64, dtype=torch.float16), torch.zeros(5, 64, dtype=torch.float64), torch.zeros(5, 32),
                torch.zeros(64), ok.numpy()):
        with pytest.raises(hr.HrError) as e:
            b._want(bad, "queries", torch.float32, (None, 64), cpu)
        assert e.value.code == -1
    with pytest.raises(hr.HrError):                                  # wrong device
        b._want(ok, "queries", torch.float32, (None, 64), torch.device("cuda:0"))
    with pytest.raises(hr.HrError):                                  # float list numbers
        b._want_int(torch.zeros(5, 3), "probe_ids", (5, None), cpu)
    with pytest.raises(hr.HrError):                                  # rows of another batch size
        b._want_int(torch.zeros(4, 3, dtype=torch.int64), "probe_ids", (5, None), cpu)
    assert b._want_int(torch.zeros(5, 3, dtype=torch.int64), "probe_ids", (5, None), cpu).dtype == torch.int32
    # an index object without a library handle: every method must refuse host tensors before calling the library
    ix = b.IvfIndex.__new__(b.IvfIndex)
    ix.handle, ix.d, ix.nlist, ix.device, ix._ws = None, 64, 10, torch.device("cuda:0"), None
    probe = torch.zeros(5, 3, dtype=torch.int32)
    state = (torch.zeros(5, 4, dtype=torch.int64), torch.zeros(5, 4), torch.zeros(5, 4, dtype=torch.int32))
    for call in (lambda: ix.search(ok, 3, 4), lambda: ix.coarse(ok, 3), lambda: ix.scan(ok, probe, 4),
                 lambda: ix.scan_step(ok, probe, state[:2]), lambda: ix.scan_step_rows(ok, probe, state),
                 lambda: ix.rescore(ok, probe, 4), lambda: ix.lists_of_rows(probe), lambda: b.reorder_probes(probe),
                 lambda: b.IvfIndex(ok, torch.zeros(6, dtype=torch.int64), ok, torch.zeros(5, dtype=torch.int64))):
        with pytest.raises(hr.HrError) as e:
            call()
        assert e.value.code == -1
    ix.handle = None                                                  # (nothing to free)
