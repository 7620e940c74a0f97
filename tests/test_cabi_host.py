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


def test_fixed_scratch_of_the_allocation_free_step_is_a_symbol_the_runtime_can_look_up(tmp_path):
    """apm_page_adamw_step_noalloc asks the runtime for the device address of a static device
    array by its symbol.  The runtime finds symbols of the code object's dynamic symbol table only,
    and aborts the process on one it cannot find, so the array must be emitted there (the compiler
    does that for a static device variable host code refers to, unless attributes get in the
    way).  Checked on the device code of that source file, compiled here."""
    import shutil
    import subprocess
    hipcc = "/opt/rocm/bin/hipcc"
    bundler = "/opt/rocm/llvm/bin/clang-offload-bundler"
    readelf = "/opt/rocm/llvm/bin/llvm-readelf"
    for tool in (hipcc, bundler, readelf):
        if not os.path.exists(tool):
            pytest.skip(f"{tool} not present")
    src = os.path.join(ROOT, "paper_2303_02868_amd", "csrc", "apm_noalloc.hip")
    obj, elf = str(tmp_path / "dev.o"), str(tmp_path / "dev.elf")
    subprocess.run([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "-c",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(src), src, "-o", obj],
                   check=True, capture_output=True)
    subprocess.run([bundler, "--unbundle", "--type=o", f"--input={obj}", f"--output={elf}",
                    "--targets=hipv4-amdgcn-amd-amdhsa--gfx950"], check=True, capture_output=True)
    out = subprocess.run([readelf, "--dyn-syms", elf], check=True, capture_output=True, text=True).stdout
    rows = [l.split() for l in out.splitlines() if l.split()[-1:] and l.split()[-1].endswith("scratch")]
    assert rows, "the scratch array is not in the code object's dynamic symbol table:\n" + out
    assert rows[0][3] == "OBJECT" and rows[0][4] == "GLOBAL" and int(rows[0][2]) == apm.apm_noalloc_scratch_bytes()


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


def test_planner_reproduces_the_hand_worked_layout_with_two_handovers(golden_dir):
    # the library's planner against the layout worked on paper, not against the oracle's planner:
    # a misreading of the packing rule shared by the two planners would not get past this
    from test_oracle_packer import read_worked_layout
    E, numels, segs, pages, total = read_worked_layout(os.path.join(golden_dir, "packer_worked_layout_two_handovers.txt"))
    res = apm.apm_pack_plan(E, numels)
    assert res.segments == segs
    assert res.n_pages == len(pages)
    assert abs(res.fragmentation - (1 - total / (len(pages) * E))) < 1e-15


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


# ---- the scheduler planner (host-only, Alg. 1 phase 1): bit-exact against the oracle ------------

def _oracle_schedule(layers, last_access, page_bytes, memory):
    from oracle import scheduler as sch
    model = [sch.Layer(list(pl), sz) for pl, sz in layers]
    traces = ({p: i for i, l in enumerate(model) for p in l.page_list} if last_access is None
              else {p: la for p, la in enumerate(last_access)})
    S = sch.schedule(model, traces, memory, page_bytes)
    return [(apm.APM_TASK_MOVE_TO_GPU if t.operation == sch.MOVE_TO_GPU else apm.APM_TASK_COMPUTE,
             t.target, t.trigger_id) for t in S]


@pytest.mark.parametrize("reuse", [False, True])
def test_schedule_plan_equals_oracle_on_random_traces(reuse):
    import random
    from oracle import scheduler as sch
    rng = random.Random(11 + reuse)
    n_ok = n_oom = 0
    for _ in range(400):
        n_layers = rng.randint(1, 9)
        ids = list(range(rng.randint(0, 24)))
        rng.shuffle(ids)                                   # page ids need not be in layer order
        cuts = sorted(rng.randint(0, len(ids)) for _ in range(n_layers - 1))
        lists = [ids[a:b] for a, b in zip([0] + cuts, cuts + [len(ids)])]
        layers = [(pl, rng.randint(0, 9)) for pl in lists]
        own_of = {p: i for i, (pl, _) in enumerate(layers) for p in pl}
        last = None
        if reuse:
            own = {p: i for i, (pl, _) in enumerate(layers) for p in pl}
            last = [rng.randint(own[p], n_layers - 1) if rng.random() < 0.3 else own[p] for p in range(len(ids))]
        page_bytes, memory = rng.choice([1, 4]), rng.randint(0, 60)
        try:
            want = _oracle_schedule(layers, last, page_bytes, memory)
        except sch.OutOfMemory:
            with pytest.raises(apm.ApmError) as e:
                apm.apm_schedule_plan(layers, last, page_bytes, memory)
            assert e.value.code == apm.APM_ENOMEM
            n_oom += 1
            continue
        got, peak = apm.apm_schedule_plan(layers, last, page_bytes, memory)
        assert got == want
        assert peak <= memory
        # and against what the algorithm guarantees, checked on the library's task list alone
        import schedule_properties as props
        la = last if last is not None else [own_of[p] for p in range(len(ids))]
        tuples = [(props.MOVE if op == apm.APM_TASK_MOVE_TO_GPU else props.COMPUTE, t, g) for op, t, g in got]
        assert props.check(tuples, layers, dict(enumerate(la)), memory, page_bytes) == peak
        n_ok += 1
    assert n_ok > 80 and n_oom > 80


def test_schedule_plan_on_a_model_sized_trace_and_its_errors():
    from oracle import scheduler as sch
    # the 1.3 B shape, one "layer" per transformer block: 1449 pages of 12 MiB (p, m, v)
    f, E = synth.WORKLOADS["gpt_1p3b"]
    plan = oracle.plan_pack([t.numel for t in f()], E)
    n = plan.n_pages
    per = -(-n // 26)
    layers = [(list(range(a, min(a + per, n))), 0) for a in range(0, n, per)]
    page_bytes = 12 * E
    got, peak = apm.apm_schedule_plan(layers, None, page_bytes, 192 * page_bytes)
    assert got == _oracle_schedule(layers, None, page_bytes, 192 * page_bytes)
    assert peak <= 192 * page_bytes and len(got) == n + len(layers)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_schedule_plan(layers, None, page_bytes, (per - 1) * page_bytes)
    assert e.value.code == apm.APM_ENOMEM and "layer 0" in str(e.value)
    with pytest.raises(apm.ApmError) as e:                      # a page in two layers
        apm.apm_schedule_plan([([0, 1], 0), ([1], 0)], None, 1, 10)
    assert e.value.code == apm.APM_EINVAL
    with pytest.raises(apm.ApmError) as e:                      # last access before the first
        apm.apm_schedule_plan([([0], 0), ([1], 0)], [0, 0], 1, 10)
    assert e.value.code == apm.APM_EINVAL
    assert apm.apm_schedule_plan([], None, 1, 0) == ([], 0)


def test_file_pool_files_sizes_flags_and_refusals(tmp_path):
    # a FILE pool needs no GPU: one file per stored class, full size, zeros; reopening keeps contents
    E, n = 2048, 5
    prefix = str(tmp_path / "state")
    pool = apm.apm_file_pool_create(prefix, E, n, state_mask=apm.FP32_STATES | (1 << apm.APM_P16))
    for suffix, eb in ((".p32", 4), (".m32", 4), (".v32", 4), (".p16", 2)):
        assert os.path.getsize(prefix + suffix) == n * E * eb
    assert not os.path.exists(prefix + ".g16")
    assert open(prefix + ".m32", "rb").read() == bytes(n * E * 4)
    assert apm.apm_pool_state_ptr(pool, apm.APM_P32) is None
    with pytest.raises(apm.ApmError) as e:
        apm.apm_pack_tensors(pool, apm.APM_P32, apm.make_tensors([10], apm.APM_F32), 1)
    assert e.value.code == apm.APM_EDEVICE
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_copy_async(pool, 0, pool, 1, 1, apm.APM_P32)
    assert e.value.code in (apm.APM_EDEVICE, apm.APM_EINVAL)
    pool.destroy()
    with open(prefix + ".p32", "r+b") as f:
        f.write(b"\x01\x02\x03\x04")
    again = apm.apm_file_pool_create(prefix, E, n, flags=apm.APM_POOL_NO_ZERO)
    again.destroy()
    assert open(prefix + ".p32", "rb").read(4) == b"\x01\x02\x03\x04"
    fresh = apm.apm_file_pool_create(prefix, E, n)
    fresh.destroy()
    assert open(prefix + ".p32", "rb").read(4) == bytes(4)
    with pytest.raises(apm.ApmError) as e:                      # 8-element pages of 32 bytes cannot be unbuffered
        apm.apm_file_pool_create(prefix, 8, n, flags=apm.APM_POOL_FILE_DIRECT)
    assert e.value.code == apm.APM_EINVAL
    with pytest.raises(apm.ApmError) as e:
        apm.apm_file_pool_create(str(tmp_path / "no_such_dir" / "x"), E, n)
    assert e.value.code == apm.APM_EDEVICE


def test_header_is_plain_c_and_callable_from_a_c_program(tmp_path):
    # include/apm.h under a strict C99 compiler, linked against the built library; the program
    # calls the two host-only planners
    import subprocess
    src = tmp_path / "cabi.c"
    src.write_text(r'''
#include <stdio.h>
#include "apm.h"
int main(void) {
    int64_t numels[3] = {3000000, 17, 1048576};
    apm_segment segs[16];
    int64_t n_segs = 16, n_pages = 0, n_tasks = 8, peak = 0;
    double frag = 0;
    int64_t offsets[3] = {0, 2, 3}, pages[3] = {0, 1, 2}, sizes[2] = {0, 0};
    apm_task tasks[8];
    int rc = apm_pack_plan(1048576, numels, 3, segs, &n_segs, &n_pages, &frag);
    if (rc != APM_OK) return 1;
    printf("%lld %lld %.9f\n", (long long)n_segs, (long long)n_pages, frag);
    rc = apm_schedule_plan(offsets, pages, sizes, 2, NULL, 3, 4, 8, tasks, &n_tasks, &peak);
    if (rc != APM_OK) return 2;
    printf("%lld %lld", (long long)n_tasks, (long long)peak);
    for (int k = 0; k < (int)n_tasks; ++k) printf(" %d:%lld@%d", tasks[k].op, (long long)tasks[k].target, tasks[k].trigger_id);
    printf("\n%s|\n", apm_last_error());
    return 0;
}
''')
    exe = tmp_path / "cabi"
    libdir = os.path.dirname(apm.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), apm.LIB_PATH, f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines()
    plan = oracle.plan_pack([3000000, 17, 1048576], 1048576)
    assert out[0] == f"{len(plan.segments)} {plan.n_pages} {plan.fragmentation:.9f}"
    # two pages fit: the move of page 2 is taken off for layer 0 and put back right after its compute
    assert out[1] == "5 8 0:0@0 0:1@0 1:0@0 0:2@0 1:1@1"
    assert out[2] == "|"
