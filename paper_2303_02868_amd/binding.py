"""Thin ctypes binding of libapm.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels; nothing here computes.  The library must
have been built (python -m paper_2303_02868_amd.build); loading fails loudly otherwise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
# APM_LIBRARY selects another build of the same library (e.g. one compiled with different tunables).
LIB_PATH = os.environ.get("APM_LIBRARY") or os.path.join(_PKG, "libapm.so")

APM_OK, APM_EINVAL, APM_ENOMEM, APM_ERANGE, APM_EDEVICE, APM_ESTATE = 0, -1, -2, -3, -4, -5
APM_DEV_GPU, APM_DEV_HOST, APM_DEV_FILE = 0, 1, 2
APM_F32, APM_BF16 = 0, 1
APM_P32, APM_M32, APM_V32, APM_G16, APM_P16, APM_N_STATES = 0, 1, 2, 3, 4, 5
APM_SKIP_NONE, APM_SKIP_UNTOUCHED = 0, 1
APM_POOL_NO_ZERO = 1
APM_POOL_FILE_DIRECT = 2
APM_STREAM_STAGED, APM_STREAM_DIRECT, APM_STREAM_STAGED_DMA = 0, 1, 2
APM_K_REDUCE, APM_K_UPDATE, APM_K_SEGCOPY, APM_N_KERNEL_CLASSES = 0, 1, 2, 3
ALL_STATES = 0b11111
FP32_STATES = 0b00111
B16_STATES = 0b11000

EXPORTS = [
    "apm_last_error", "apm_pack_plan", "apm_pool_create", "apm_pool_destroy",
    "apm_pool_pages_in_use", "apm_pool_page_info", "apm_pool_state_ptr", "apm_pool_set_layout",
    "apm_pack_tensors", "apm_unpack", "apm_page_adamw_step", "apm_page_adamw_step_fused",
    "apm_page_copy_async",
    "apm_schedule_plan", "apm_file_pool_create", "apm_tiered_create", "apm_tiered_destroy", "apm_tiered_io_bytes", "apm_tiered_set_range", "apm_streamer_set_page_count", "apm_tiered_step", "apm_tiered_step_delayed", "apm_streamer_step_scheduled", "apm_streamer_step_delayed", "apm_streamer_create", "apm_streamer_destroy", "apm_streamer_step", "apm_streamer_copy_only", "apm_streamer_set_cache", "apm_cache_pages_that_fit", "apm_streamer_set_host_first_page", "apm_streamer_set_mode", "apm_streamer_get_mode", "apm_streamer_probe_rates", "apm_step_delayed",
    "apm_delayed_applied", "apm_delayed_set_outputs", "apm_delayed_grad_buffer", "apm_delayed_accumulate", "apm_pool_set_timing", "apm_pool_read_timing",
    "apm_page_adamw_step_noalloc", "apm_noalloc_scratch_bytes", "apm_noalloc_max_pages",
    "apm_streamer_overlap_report",
    "apm_streamer_set_host_write_through",
]


class apm_pool_desc(C.Structure):
    _fields_ = [("device", C.c_int32), ("hip_device", C.c_int32), ("page_elems", C.c_int64),
                ("n_pages", C.c_int64), ("state_mask", C.c_uint32), ("flags", C.c_uint32),
                ("base", C.c_void_p * APM_N_STATES)]


class apm_tensor(C.Structure):
    _fields_ = [("id", C.c_int64), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("numel", C.c_int64), ("data", C.c_void_p)]


class apm_segment(C.Structure):
    _fields_ = [("tensor", C.c_int64), ("tensor_off", C.c_int64), ("page", C.c_int64),
                ("page_off", C.c_int64), ("n", C.c_int64)]

    def astuple(self):
        return (self.tensor, self.tensor_off, self.page, self.page_off, self.n)


class apm_page_info(C.Structure):
    _fields_ = [("total_elems", C.c_int64), ("used_elems", C.c_int64),
                ("available_elems", C.c_int64), ("device", C.c_int32), ("n_tensors", C.c_int32),
                ("tensor_id", C.c_int64 * 2), ("tensor_elems", C.c_int64 * 2)]


class apm_task(C.Structure):
    _fields_ = [("op", C.c_int32), ("trigger_id", C.c_int32), ("target", C.c_int64)]


APM_TASK_MOVE_TO_GPU, APM_TASK_COMPUTE = 0, 1


class apm_hyper(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("max_grad_norm", C.c_double),
                ("skip_mode", C.c_int32), ("reserved", C.c_int32)]


class ApmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"apm error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2303_02868_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
    P = C.POINTER
    L.apm_last_error.restype = C.c_char_p
    L.apm_last_error.argtypes = []
    L.apm_pack_plan.argtypes = [i64, P(i64), i64, P(apm_segment), P(i64), P(i64), P(C.c_double)]
    L.apm_pool_create.argtypes = [P(vp), P(apm_pool_desc)]
    L.apm_pool_destroy.argtypes = [vp]
    L.apm_pool_pages_in_use.argtypes = [vp]
    L.apm_pool_pages_in_use.restype = i64
    L.apm_pool_page_info.argtypes = [vp, i64, P(apm_page_info)]
    L.apm_pool_state_ptr.argtypes = [vp, i32, i64]
    L.apm_pool_state_ptr.restype = vp
    L.apm_pool_set_layout.argtypes = [vp, P(apm_tensor), i64, P(apm_segment), P(i64), P(i64),
                                      P(C.c_double), vp]
    L.apm_pack_tensors.argtypes = [vp, i32, P(apm_tensor), i64, P(apm_segment), P(i64), P(i64),
                                   P(C.c_double), vp]
    L.apm_unpack.argtypes = [vp, i32, P(apm_tensor), i64, vp]
    L.apm_page_adamw_step.argtypes = [vp, P(i64), i64, i64, P(apm_hyper), vp, vp, vp]
    L.apm_page_adamw_step_fused.argtypes = [vp, P(i64), i64, i64, P(apm_hyper), P(apm_tensor),
                                            P(apm_tensor), i64, vp, vp, vp]
    L.apm_page_copy_async.argtypes = [vp, i64, vp, i64, i64, i32, vp]
    L.apm_page_adamw_step_noalloc.argtypes = [vp, i64, i64, P(apm_hyper), vp, vp, vp]
    L.apm_noalloc_scratch_bytes.argtypes = []
    L.apm_noalloc_scratch_bytes.restype = C.c_size_t
    L.apm_noalloc_max_pages.argtypes = [i64]
    L.apm_noalloc_max_pages.restype = i64
    L.apm_schedule_plan.argtypes = [P(i64), P(i64), P(i64), i64, P(i64), i64, i64, i64, P(apm_task), P(i64), P(i64)]
    L.apm_streamer_step_scheduled.argtypes = [vp, P(apm_task), i64, P(i64), i64, P(i64), i64, P(apm_hyper), vp, vp, vp]
    L.apm_streamer_step_delayed.argtypes = [vp, vp, P(apm_hyper), vp]
    L.apm_file_pool_create.argtypes = [P(vp), C.c_char_p, i32, i64, i64, C.c_uint32, C.c_uint32]
    L.apm_tiered_create.argtypes = [P(vp), vp, vp, i64, i32, i32]
    L.apm_tiered_destroy.argtypes = [vp]
    L.apm_tiered_step.argtypes = [vp, i64, P(apm_hyper), vp, vp, vp]
    L.apm_tiered_io_bytes.argtypes = [vp, P(i64), P(i64)]
    L.apm_tiered_set_range.argtypes = [vp, i64, i64]
    L.apm_streamer_set_page_count.argtypes = [vp, i64]
    L.apm_tiered_step_delayed.argtypes = [vp, vp, P(apm_hyper), vp]
    L.apm_streamer_create.argtypes = [P(vp), vp, vp, i64, i32]
    L.apm_streamer_destroy.argtypes = [vp]
    L.apm_streamer_step.argtypes = [vp, i64, P(apm_hyper), vp, vp, vp]
    L.apm_streamer_copy_only.argtypes = [vp, i32, vp]
    L.apm_streamer_set_cache.argtypes = [vp, vp, i64]
    L.apm_streamer_set_host_first_page.argtypes = [vp, i64]
    L.apm_cache_pages_that_fit.argtypes = [i32, i64, i64, C.c_size_t, P(i64)]
    L.apm_streamer_set_mode.argtypes = [vp, i32, i32, i32]
    L.apm_streamer_get_mode.argtypes = [vp]
    L.apm_streamer_probe_rates.argtypes = [vp, P(C.c_double), P(C.c_double), P(C.c_double)]
    L.apm_streamer_overlap_report.argtypes = [vp, P(C.c_int), P(C.c_int)]
    L.apm_streamer_set_host_write_through.argtypes = [vp, C.c_int]
    L.apm_step_delayed.argtypes = [vp, P(i64), i64, vp, P(apm_hyper), vp]
    L.apm_delayed_accumulate.argtypes = [vp, P(i64), i64, vp, vp]
    L.apm_delayed_grad_buffer.argtypes = [vp, vp]
    L.apm_delayed_grad_buffer.restype = vp
    L.apm_delayed_applied.argtypes = [vp]
    L.apm_delayed_applied.restype = i64
    L.apm_delayed_set_outputs.argtypes = [vp, vp, vp]
    L.apm_pool_set_timing.argtypes = [vp, i32]
    L.apm_pool_read_timing.argtypes = [vp, P(C.c_double), P(i64)]
    for name in EXPORTS:
        getattr(L, name)              # every declared entry point must be exported
    _lib = L
    return L


def apm_last_error() -> str:
    return lib().apm_last_error().decode()


def _check(rc: int) -> None:
    if rc != APM_OK:
        raise ApmError(rc, apm_last_error())


def _ptr(x) -> Optional[int]:
    """Raw address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(type(x))


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None          # torch.cuda.Stream


def _i64_array(xs: Optional[Sequence[int]]):
    if xs is None:
        return None, 0
    arr = (C.c_int64 * len(xs))(*[int(x) for x in xs])
    return arr, len(xs)


def make_hyper(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=0.0,
               skip_mode=APM_SKIP_NONE) -> apm_hyper:
    return apm_hyper(lr, beta1, beta2, eps, weight_decay, max_grad_norm, skip_mode, 0)


def make_tensors(numels: Sequence[int], dtype: int, datas: Optional[Sequence] = None,
                 ids: Optional[Sequence[int]] = None):
    n = len(numels)
    arr = (apm_tensor * max(n, 1))()
    for i in range(n):
        arr[i].id = i if ids is None else int(ids[i])
        arr[i].dtype = dtype
        arr[i].numel = int(numels[i])
        arr[i].data = None if datas is None else _ptr(datas[i])
    return arr


class PlanResult:
    def __init__(self, segs, n_pages, fragmentation):
        self.segments = segs              # list of (tensor, tensor_off, page, page_off, n)
        self.n_pages = n_pages
        self.fragmentation = fragmentation


def apm_pack_plan(page_elems: int, numels: Sequence[int]) -> PlanResult:
    L = lib()
    arr, n = _i64_array(numels)
    n_segs, n_pages, frag = C.c_int64(0), C.c_int64(0), C.c_double(0)
    _check(L.apm_pack_plan(page_elems, arr, n, None, C.byref(n_segs), C.byref(n_pages), C.byref(frag)))
    segs = (apm_segment * max(1, n_segs.value))()
    cap = C.c_int64(n_segs.value)
    _check(L.apm_pack_plan(page_elems, arr, n, segs, C.byref(cap), C.byref(n_pages), C.byref(frag)))
    return PlanResult([segs[i].astuple() for i in range(cap.value)], n_pages.value, frag.value)


class Pool:
    """Owner of an apm_pool handle."""

    def __init__(self, handle: int, desc: apm_pool_desc, keepalive=None):
        self.handle = handle
        self.desc = desc
        self._keepalive = keepalive

    def destroy(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().apm_pool_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def apm_pool_create(device: int, page_elems: int, n_pages: int, state_mask: int = ALL_STATES,
                    flags: int = 0, hip_device: int = 0, base: Optional[dict] = None) -> Pool:
    """base: {state: torch tensor | address} of caller-owned regions (kept alive by the Pool)."""
    d = apm_pool_desc()
    d.device, d.hip_device, d.page_elems, d.n_pages = device, hip_device, page_elems, n_pages
    d.state_mask, d.flags = state_mask, flags
    for s in range(APM_N_STATES):
        d.base[s] = _ptr(base.get(s)) if base else None
    out = C.c_void_p()
    _check(lib().apm_pool_create(C.byref(out), C.byref(d)))
    return Pool(out.value, d, keepalive=base)


def apm_pool_destroy(pool: Pool) -> None:
    pool.destroy()


def apm_pool_pages_in_use(pool: Pool) -> int:
    return lib().apm_pool_pages_in_use(pool.handle)


def apm_pool_page_info(pool: Pool, page: int) -> apm_page_info:
    info = apm_page_info()
    _check(lib().apm_pool_page_info(pool.handle, page, C.byref(info)))
    return info


def apm_pool_state_ptr(pool: Pool, state: int, page: int = 0) -> Optional[int]:
    return lib().apm_pool_state_ptr(pool.handle, state, page)


def apm_pool_set_layout(pool: Pool, tensors, n: int, stream=None) -> PlanResult:
    L = lib()
    cap = 2 * pool.desc.n_pages + 2
    segs = (apm_segment * cap)()
    n_segs, n_pages, frag = C.c_int64(cap), C.c_int64(0), C.c_double(0)
    _check(L.apm_pool_set_layout(pool.handle, tensors, n, segs, C.byref(n_segs), C.byref(n_pages),
                                 C.byref(frag), _stream(stream)))
    return PlanResult([segs[i].astuple() for i in range(n_segs.value)], n_pages.value, frag.value)


def apm_pack_tensors(pool: Pool, state: int, tensors, n: int, stream=None) -> PlanResult:
    L = lib()
    cap = 2 * pool.desc.n_pages + 2
    segs = (apm_segment * cap)()
    n_segs, n_pages, frag = C.c_int64(cap), C.c_int64(0), C.c_double(0)
    _check(L.apm_pack_tensors(pool.handle, state, tensors, n, segs, C.byref(n_segs),
                              C.byref(n_pages), C.byref(frag), _stream(stream)))
    return PlanResult([segs[i].astuple() for i in range(n_segs.value)], n_pages.value, frag.value)


def apm_unpack(pool: Pool, state: int, tensors, n: int, stream=None) -> None:
    _check(lib().apm_unpack(pool.handle, state, tensors, n, _stream(stream)))


def apm_page_adamw_step(pool: Pool, pages: Optional[Sequence[int]], n_pages: int, step: int,
                        hyper: apm_hyper, grad_norm=None, skip_mask=None, stream=None) -> None:
    arr, _ = _i64_array(pages)
    _check(lib().apm_page_adamw_step(pool.handle, arr, n_pages, step, C.byref(hyper),
                                     _ptr(grad_norm), _ptr(skip_mask), _stream(stream)))


def apm_page_adamw_step_fused(pool: Pool, pages: Optional[Sequence[int]], n_pages: int, step: int,
                              hyper: apm_hyper, grad_tensors, p16_tensors, n_tensors: int,
                              grad_norm=None, skip_mask=None, stream=None) -> None:
    arr, _ = _i64_array(pages)
    _check(lib().apm_page_adamw_step_fused(pool.handle, arr, n_pages, step, C.byref(hyper),
                                           grad_tensors, p16_tensors, n_tensors, _ptr(grad_norm),
                                           _ptr(skip_mask), _stream(stream)))


def apm_page_adamw_step_noalloc(pool: Pool, n_pages: int, step: int, hyper: apm_hyper,
                                grad_norm=None, skip_mask=None, stream=None) -> None:
    _check(lib().apm_page_adamw_step_noalloc(pool.handle, n_pages, step, C.byref(hyper),
                                             _ptr(grad_norm), _ptr(skip_mask), _stream(stream)))


def apm_noalloc_scratch_bytes() -> int:
    return lib().apm_noalloc_scratch_bytes()


def apm_noalloc_max_pages(page_elems: int) -> int:
    return lib().apm_noalloc_max_pages(page_elems)


def apm_page_copy_async(dst: Pool, dst_page: int, src: Pool, src_page: int, n_pages: int,
                        state: int, stream=None) -> None:
    _check(lib().apm_page_copy_async(dst.handle, dst_page, src.handle, src_page, n_pages, state,
                                     _stream(stream)))


def apm_file_pool_create(path_prefix: str, page_elems: int, n_pages: int, state_mask: int = FP32_STATES,
                         flags: int = 0, hip_device: int = 0) -> Pool:
    d = apm_pool_desc()
    d.device, d.hip_device, d.page_elems, d.n_pages = APM_DEV_FILE, hip_device, page_elems, n_pages
    d.state_mask, d.flags = state_mask, flags
    out = C.c_void_p()
    _check(lib().apm_file_pool_create(C.byref(out), path_prefix.encode(), hip_device, page_elems, n_pages,
                                      state_mask, flags))
    return Pool(out.value, d)


class Tiered:
    def __init__(self, handle, file: Pool, dev: Pool):
        self.handle, self.file, self.dev = handle, file, dev

    def destroy(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().apm_tiered_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def apm_tiered_create(file: Pool, dev: Pool, batch_pages: int, n_slots: int, io_threads: int) -> Tiered:
    out = C.c_void_p()
    _check(lib().apm_tiered_create(C.byref(out), file.handle, dev.handle, batch_pages, n_slots, io_threads))
    return Tiered(out.value, file, dev)


def apm_tiered_destroy(t: Tiered) -> None:
    t.destroy()


def apm_tiered_set_range(t: Tiered, first_page: int, n_pages: int = -1) -> None:
    _check(lib().apm_tiered_set_range(t.handle, first_page, n_pages))


def apm_streamer_set_page_count(s: "Streamer", n_pages: int) -> None:
    _check(lib().apm_streamer_set_page_count(s.handle, n_pages))


def apm_tiered_io_bytes(t: Tiered):
    """(bytes read, bytes written) queued since creation."""
    r, w = C.c_int64(0), C.c_int64(0)
    _check(lib().apm_tiered_io_bytes(t.handle, C.byref(r), C.byref(w)))
    return r.value, w.value


def apm_tiered_step(t: Tiered, step: int, hyper: apm_hyper, grad_norm=None, skip_mask=None, stream=None) -> None:
    _check(lib().apm_tiered_step(t.handle, step, C.byref(hyper), _ptr(grad_norm), _ptr(skip_mask), _stream(stream)))


def apm_tiered_step_delayed(t: Tiered, new_g16, hyper: apm_hyper, stream=None) -> None:
    _check(lib().apm_tiered_step_delayed(t.handle, _ptr(new_g16), C.byref(hyper), _stream(stream)))


class Streamer:
    def __init__(self, handle, host: Pool, dev: Pool):
        self.handle, self.host, self.dev = handle, host, dev

    def destroy(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().apm_streamer_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def apm_schedule_plan(layers: Sequence, last_access: Optional[Sequence[int]], page_bytes: int,
                      gpu_memory_bytes: int):
    """layers: sequence of (page_list, bytes).  Returns ([(op, target, trigger_id), ...], peak_bytes)."""
    offsets, pages, sizes = [0], [], []
    for page_list, nbytes in layers:
        pages.extend(int(p) for p in page_list)
        offsets.append(len(pages))
        sizes.append(int(nbytes))
    off_a, _ = _i64_array(offsets)
    pg_a, n_pages = _i64_array(pages)
    sz_a, n_layers = _i64_array(sizes)
    la_a = _i64_array(last_access)[0] if last_access is not None else None
    cap = n_pages + n_layers
    tasks = (apm_task * max(1, cap))()
    n_tasks, peak = C.c_int64(cap), C.c_int64(0)
    _check(lib().apm_schedule_plan(off_a, pg_a, sz_a, n_layers, la_a, n_pages, page_bytes, gpu_memory_bytes,
                                   tasks, C.byref(n_tasks), C.byref(peak)))
    return [(tasks[i].op, tasks[i].target, tasks[i].trigger_id) for i in range(n_tasks.value)], peak.value


def apm_streamer_create(host: Pool, dev: Pool, batch_pages: int, n_slots: int) -> Streamer:
    out = C.c_void_p()
    _check(lib().apm_streamer_create(C.byref(out), host.handle, dev.handle, batch_pages, n_slots))
    return Streamer(out.value, host, dev)


def apm_streamer_destroy(s: Streamer) -> None:
    s.destroy()


def apm_streamer_step(s: Streamer, step: int, hyper: apm_hyper, grad_norm=None, skip_mask=None,
                      stream=None) -> None:
    _check(lib().apm_streamer_step(s.handle, step, C.byref(hyper), _ptr(grad_norm),
                                   _ptr(skip_mask), _stream(stream)))


def apm_streamer_step_scheduled(s: Streamer, tasks: Sequence, layer_first_page: Sequence[int], step: int,
                                hyper: apm_hyper, grad_norm=None, skip_mask=None, stream=None,
                                last_access: Optional[Sequence[int]] = None) -> None:
    """tasks: [(op, target, trigger_id), ...] as apm_schedule_plan returns them."""
    arr = (apm_task * max(1, len(tasks)))()
    for i, (op, target, trig) in enumerate(tasks):
        arr[i].op, arr[i].target, arr[i].trigger_id = op, target, trig
    lf, n1 = _i64_array(layer_first_page)
    la = _i64_array(last_access)[0] if last_access is not None else None
    _check(lib().apm_streamer_step_scheduled(s.handle, arr, len(tasks), lf, n1 - 1, la, step, C.byref(hyper),
                                             _ptr(grad_norm), _ptr(skip_mask), _stream(stream)))


def apm_streamer_set_host_write_through(s: Streamer, on: bool) -> None:
    _check(lib().apm_streamer_set_host_write_through(s.handle, int(bool(on))))


def apm_streamer_overlap_report(s: Streamer):
    """(update stream, pipeline streams): 1 runs beside the producer stream, 0 does not, -1 not measured."""
    a, b = C.c_int(-1), C.c_int(-1)
    _check(lib().apm_streamer_overlap_report(s.handle, C.byref(a), C.byref(b)))
    return a.value, b.value


def apm_streamer_step_delayed(s: Streamer, new_g16, hyper: apm_hyper, stream=None) -> None:
    _check(lib().apm_streamer_step_delayed(s.handle, _ptr(new_g16), C.byref(hyper), _stream(stream)))


def apm_streamer_set_cache(s: Streamer, cache: Optional[Pool], n_resident: int) -> None:
    _check(lib().apm_streamer_set_cache(s.handle, cache.handle if cache else None, n_resident))
    s.cache = cache


def apm_cache_pages_that_fit(page_elems: int, n_pages: int, reserve_bytes: int = 0, hip_device: int = 0) -> int:
    out = C.c_int64(0)
    _check(lib().apm_cache_pages_that_fit(hip_device, page_elems, n_pages, reserve_bytes, C.byref(out)))
    return out.value


def apm_streamer_set_host_first_page(s: Streamer, first_model_page: int) -> None:
    _check(lib().apm_streamer_set_host_first_page(s.handle, first_model_page))


def apm_streamer_set_mode(s: Streamer, mode: int, direct_wavefronts: int = 0,
                          wavefronts_per_workgroup: int = 0) -> None:
    _check(lib().apm_streamer_set_mode(s.handle, mode, direct_wavefronts, wavefronts_per_workgroup))


def apm_streamer_get_mode(s: Streamer) -> int:
    m = lib().apm_streamer_get_mode(s.handle)
    _check(min(m, 0))
    return m


def apm_streamer_probe_rates(s: Streamer):
    """(copy-in alone, copy-out alone, each way when both run) in GB/s, from creation."""
    a, b, c = C.c_double(), C.c_double(), C.c_double()
    _check(lib().apm_streamer_probe_rates(s.handle, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def apm_streamer_copy_only(s: Streamer, directions: int, stream=None) -> None:
    _check(lib().apm_streamer_copy_only(s.handle, directions, _stream(stream)))


def apm_step_delayed(pool: Pool, pages: Optional[Sequence[int]], n_pages: int, new_g16,
                     hyper: apm_hyper, stream=None) -> None:
    arr, _ = _i64_array(pages)
    _check(lib().apm_step_delayed(pool.handle, arr, n_pages, _ptr(new_g16), C.byref(hyper),
                                  _stream(stream)))


def apm_delayed_accumulate(pool: Pool, pages: Optional[Sequence[int]], n_pages: int, g16, stream=None) -> None:
    arr, _ = _i64_array(pages)
    _check(lib().apm_delayed_accumulate(pool.handle, arr, n_pages, _ptr(g16), _stream(stream)))


def apm_delayed_grad_buffer(pool: Pool, stream=None) -> int:
    p = lib().apm_delayed_grad_buffer(pool.handle, _stream(stream))
    if not p:
        raise ApmError(APM_EDEVICE, apm_last_error())
    return p


def apm_delayed_applied(pool: Pool) -> int:
    return lib().apm_delayed_applied(pool.handle)


def apm_delayed_set_outputs(pool: Pool, grad_norm=None, skip_mask=None) -> None:
    _check(lib().apm_delayed_set_outputs(pool.handle, _ptr(grad_norm), _ptr(skip_mask)))


def apm_pool_set_timing(pool: Pool, enable: bool) -> None:
    _check(lib().apm_pool_set_timing(pool.handle, int(enable)))


def apm_pool_read_timing(pool: Pool):
    """({class: total ms}, {class: launches}) since the last read."""
    ms = (C.c_double * APM_N_KERNEL_CLASSES)()
    n = (C.c_int64 * APM_N_KERNEL_CLASSES)()
    _check(lib().apm_pool_read_timing(pool.handle, ms, n))
    return list(ms), list(n)
