"""CPU-side checks of the C-ABI library: it loads, exports every function the header declares,
and its host-only logic (the packing planner, argument validation) agrees with the oracle.  No
compute call is made; calls that need a GPU must fail with an error, not crash."""
import ctypes
import itertools
import os
import re

import pytest

import oracle
import paper_2303_02868_amd as apm
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "apm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(apm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert len(names) >= 20 and "apm_page_adamw_step" in names and "apm_step_delayed" in names
    lib = apm.lib()
    raw = ctypes.CDLL(apm.LIB_PATH)
    for n in names:
        assert getattr(raw, n) is not None, n
    assert sorted(apm.EXPORTS) == names            # the binding covers the same set
    for n in names:
        assert callable(getattr(apm, n)), f"binding lacks {n}"
    assert lib.apm_last_error() is not None


def segs_of(plan):
    return [(s.tensor, s.tensor_off, s.page, s.page_off, s.n) for s in plan.segments]


def test_planner_matches_oracle_on_boundary_sizes_and_workloads():
    E = 64
    sizes = [0, 1, 7, 8, E - 1, E, E + 1, 2 * E, 2 * E + 3, 3 * E - 8]
    for numels in itertools.product(sizes, repeat=3):
        got = apm.apm_pack_plan(E, list(numels))
        want = oracle.plan_pack(list(numels), E)
        assert got.segments == segs_of(want) and got.n_pages == want.n_pages
        assert got.fragmentation == pytest.approx(want.fragmentation, abs=1e-15)
    for name, (factory, Ep) in synth.WORKLOADS.items():
        numels = [t.numel for t in factory()]
        got = apm.apm_pack_plan(Ep, numels)
        want = oracle.plan_pack(numels, Ep)
        assert got.segments == segs_of(want), name
        assert got.n_pages == want.n_pages


def test_planner_argument_errors():
    L = apm.lib()
    n_segs = ctypes.c_int64(0)
    arr = (ctypes.c_int64 * 2)(10, -1)
    assert L.apm_pack_plan(64, arr, 2, None, ctypes.byref(n_segs), None, None) == apm.APM_EINVAL
    assert "negative" in apm.apm_last_error()
    arr = (ctypes.c_int64 * 2)(10, 200)
    assert L.apm_pack_plan(63, arr, 2, None, ctypes.byref(n_segs), None, None) == apm.APM_EINVAL
    assert L.apm_pack_plan(64, arr, 2, None, None, None, None) == apm.APM_EINVAL
    # too small a segment buffer: the needed count comes back
    segs = (apm.apm_segment * 2)()
    n_segs = ctypes.c_int64(2)
    assert L.apm_pack_plan(64, arr, 2, segs, ctypes.byref(n_segs), None, None) == apm.APM_ENOMEM
    assert n_segs.value == 5


def test_gpu_calls_fail_cleanly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(apm.ApmError) as e:
        apm.apm_pool_create(apm.APM_DEV_GPU, 1024, 4)
    assert e.value.code == apm.APM_EDEVICE
    L = apm.lib()
    assert L.apm_pool_destroy(None) == apm.APM_OK
    assert L.apm_pool_pages_in_use(None) == 0
    assert L.apm_streamer_destroy(None) == apm.APM_OK
    hy = apm.make_hyper()
    assert L.apm_page_adamw_step(None, None, 0, 1, ctypes.byref(hy), None, None, None) == apm.APM_EINVAL
    assert L.apm_step_delayed(None, None, 0, None, ctypes.byref(hy), None) == apm.APM_EINVAL
    bad = apm.apm_pool_desc()
    out = ctypes.c_void_p()
    assert L.apm_pool_create(ctypes.byref(out), ctypes.byref(bad)) == apm.APM_EINVAL   # page_elems 0
    assert out.value is None
