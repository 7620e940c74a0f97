#!/usr/bin/env python3
"""Benchmark of the page-AdamW hot path on one MI355X.  Prints ONE JSON line.

Resident leg (the headline `value`): a step is one pass of the whole path over one batch of
synthetic gradients,
  per-page grad reduce -> fused page AdamW, both reading g16 from the gradient tensors, p16
  written to the parameter tensors (`--unfused`: separate pack g16 / unpack p16 kernels),
with the pool and the packing plan set up once (the method pre-allocates them) and every input
resident in HBM before the timed region.

Streamed leg (reported under "streamed"): the fp32 master / momentum / variance pages live in
pinned host memory.  Measured: the direct mode (the update kernel reads and writes the host pages
across PCIe itself), the staged mode (pages pass through HBM staging slots; copy-in, update and
copy-out on three streams) with its copy-only pipeline, the schedule-driven mode ("scheduled"),
mixed residency, and the one-step-stale update beside a matrix-product producer ("lock_free").
The PCIe rates are held against plain pinned copies measured in the same run.

`--file-tier DIR` runs only the third-tier leg (fp32 state in files under DIR).
"""
from __future__ import annotations

import argparse
import json
import statistics
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
BYTES_UPDATE = 28               # per element: read p,m,v (12) + g (2); write p,m,v (12) + p16 (2)
BYTES_REDUCE = 2                # per element: read g
BYTES_SEGCOPY_B16 = 4           # per element: read 2 + write 2
DEV = "cuda:0"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt_1p3b",
                    choices=["cfg1_8pages", "flat_1024pages", "gpt2_small_124m", "gpt_1p3b", "moe_8x64", "gpt_13b"])
    ap.add_argument("--clip", type=float, default=None,
                    help="per-page max grad norm (default: 1.0 for gpt_1p3b, else off)")
    ap.add_argument("--update-only", action="store_true", help="time reduce+update only (no pack/unpack)")
    ap.add_argument("--unfused", action="store_true",
                    help="headline step = separate pack g16 / unpack p16 kernels instead of the fused gather/scatter")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-pages", type=int, default=192, help="pages of the workload the oracle is timed on")
    ap.add_argument("--cpu-steps", type=int, default=10)
    ap.add_argument("--no-streamed", action="store_true", help="skip the host-streamed leg")
    ap.add_argument("--streamed-only", action="store_true", help="run only the host-streamed leg (gpt_13b: always)")
    ap.add_argument("--stream-steps", type=int, default=3)
    ap.add_argument("--page-sweep", action="store_true",
                    help="run only the page-size sweep (update kernel, direct and page-granular staged streaming)")
    ap.add_argument("--full-shape", action="store_true",
                    help="run only the 13 B shape at its full 40 layers: what cannot be pinned is cached in HBM")
    ap.add_argument("--file-tier", default=None, metavar="DIR",
                    help="run only the file-tier leg, with the fp32 state in files under DIR")
    ap.add_argument("--io-threads", type=int, default=8)
    ap.add_argument("--sched-layers", type=float, default=3.0,
                    help="GPU memory of the scheduled streaming leg, in units of the largest block")
    ap.add_argument("--direct-wavefronts", type=int, default=0,
                    help="wavefronts of the direct streaming mode's kernel (0 = library default)")
    ap.add_argument("--lockfree-sweep", action="store_true",
                    help="lock_free leg: sweep wavefronts x workgroup packing of the PCIe-crossing kernel")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the compact legs of the other configurations (124 M, 13 B, MoE) and the flat reference")
    ap.add_argument("--batch-pages", type=int, default=16,
                    help="pages per staging slot of the streamer (16: the fastest of 8 / 16 / 32 / 64 measured)")
    ap.add_argument("--tier-batch-pages", type=int, default=32, help="pages per window slot of the file tier")
    ap.add_argument("--slots", type=int, default=3)
    return ap.parse_args()


class Workload:
    def __init__(self, name, layers=None):
        import synth
        self.name = name
        factory, self.E = synth.WORKLOADS[name]
        self.layers = layers
        # layers: a reduced depth of the 13 B shape, used when the box cannot pin the full state
        self.specs = factory() if layers is None else synth.gpt_tensor_list(layers, 5120, 20480, 50257, 2048)
        self.numels = [t.numel for t in self.specs]
        self.n_t = len(self.specs)
        self.off = synth.tensor_offsets(self.specs)
        self.total = int(self.off[-1])

    def gen(self, stream, bf16, sigma, active=None):
        import torch
        import synth
        out = torch.zeros(self.total, dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
        fn = synth.normal_bf16 if bf16 else synth.normal_f32
        chunk = 1 << 26
        # consecutive active tensors are generated as one range
        i = 0
        while i < self.n_t:
            if active is not None and not active[i]:
                i += 1
                continue
            j = i
            while j + 1 < self.n_t and (active is None or active[j + 1]):
                j += 1
            a0, a1 = int(self.off[i]), int(self.off[j + 1])
            for a in range(a0, a1, chunk):
                m = min(chunk, a1 - a)
                out[a:a + m] = fn(0, stream, a, m, sigma, device=DEV)
            i = j + 1
        return out

    def tensors(self, flat):
        import torch
        import paper_2303_02868_amd as apm
        dt = apm.APM_BF16 if flat.dtype == torch.bfloat16 else apm.APM_F32
        return apm.make_tensors(self.numels, dt, [flat.data_ptr() + int(self.off[i]) * flat.element_size()
                                                  for i in range(self.n_t)])


def resident_leg(args, wl, pool, hyper, n_pages, fused, steps, warmup, first_step=1):
    import torch
    import paper_2303_02868_amd as apm
    import synth
    moe = wl.name == "moe_8x64"
    grads = []
    for k in range(2):          # two gradient sets, alternated (values do not affect timing)
        act = synth.moe_active_tensors(wl.specs, k + 1, 0, 64, 8) if moe else None
        grads.append(wl.gen(1001 + k, True, 1e-3, act))
    g_tensors = [wl.tensors(g) for g in grads]
    p16_flat = torch.zeros(wl.total, dtype=torch.bfloat16, device=DEV)
    p16_tensors = wl.tensors(p16_flat)
    if args.update_only:
        apm.apm_pack_tensors(pool, apm.APM_G16, g_tensors[0], wl.n_t)
    stream = torch.cuda.current_stream()

    def step(t):
        if args.update_only:
            apm.apm_page_adamw_step(pool, None, n_pages, t, hyper, None, None, stream)
        elif fused:
            apm.apm_page_adamw_step_fused(pool, None, n_pages, t, hyper, g_tensors[t & 1], p16_tensors,
                                          wl.n_t, None, None, stream)
        else:
            apm.apm_pack_tensors(pool, apm.APM_G16, g_tensors[t & 1], wl.n_t, stream)
            apm.apm_page_adamw_step(pool, None, n_pages, t, hyper, None, None, stream)
            apm.apm_unpack(pool, apm.APM_P16, p16_tensors, wl.n_t, stream)

    t_step = first_step
    for _ in range(warmup):
        step(t_step)
        t_step += 1
    torch.cuda.synchronize()
    apm.apm_pool_set_timing(pool, True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step(t_step)
        t_step += 1
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms, launches = apm.apm_pool_read_timing(pool)
    apm.apm_pool_set_timing(pool, False)
    del grads, p16_flat

    if moe:     # skipped pages are not credited
        act_elems = [int(sum(n for n, a in zip(wl.numels, synth.moe_active_tensors(wl.specs, k + 1, 0, 64, 8)) if a))
                     for k in range(2)]
        elems_update = sum(act_elems) / 2.0
    else:
        elems_update = float(wl.total)

    def avg(cls):
        return ms[cls] / launches[cls] if launches[cls] else None

    upd_ms, red_ms, seg_ms = avg(apm.APM_K_UPDATE), avg(apm.APM_K_REDUCE), avg(apm.APM_K_SEGCOPY)
    achieved = elems_update * BYTES_UPDATE / (upd_ms * 1e-3) / 1e9
    kernels = {"adamw_update": {"avg_ms": upd_ms, "launches": launches[apm.APM_K_UPDATE],
                                "GBps": achieved, "bytes_per_elem": BYTES_UPDATE}}
    if red_ms:
        kernels["grad_reduce"] = {"avg_ms": red_ms, "launches": launches[apm.APM_K_REDUCE],
                                  "GBps": wl.total * BYTES_REDUCE / (red_ms * 1e-3) / 1e9,
                                  "bytes_per_elem": BYTES_REDUCE}
    if seg_ms:
        kernels["seg_copy_bf16"] = {"avg_ms": seg_ms, "launches": launches[apm.APM_K_SEGCOPY],
                                    "GBps": wl.total * BYTES_SEGCOPY_B16 / (seg_ms * 1e-3) / 1e9,
                                    "bytes_per_elem": BYTES_SEGCOPY_B16}
    return {"wall": wall, "elems_update": elems_update, "kernels": kernels, "achieved": achieved,
            "upd_ms": upd_ms, "next_step": t_step}


def delayed_leg(args, wl, pool, hyper, n_pages, first_step):
    """Synchronous vs one-step-stale stepping with the same producer (packing the step's gradient
    tensors into page layout): wall time of `steps` steps each.  Both are HBM-bound here, so the
    overlap the delayed form allows cannot shorten the run; it shows that decoupling costs nothing."""
    import torch
    import paper_2303_02868_amd as apm
    import synth
    moe = wl.name == "moe_8x64"
    grads = [wl.gen(1001 + k, True, 1e-3, synth.moe_active_tensors(wl.specs, k + 1, 0, 64, 8) if moe else None)
             for k in range(2)]
    g_tensors = [wl.tensors(g) for g in grads]
    stream = torch.cuda.current_stream()
    steps = max(4, args.steps // 2)
    t = first_step

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        apm.apm_pack_tensors(pool, apm.APM_G16, g_tensors[k & 1], wl.n_t, stream)
        apm.apm_page_adamw_step(pool, None, n_pages, t, hyper, None, None, stream)
        t += 1
    torch.cuda.synchronize()
    t_sync = (time.perf_counter() - t0) / steps

    halves = {}
    def produce(k):
        ptr = apm.apm_delayed_grad_buffer(pool, stream)
        if ptr not in halves:
            halves[ptr] = apm.apm_pool_create(apm.APM_DEV_GPU, wl.E, n_pages, state_mask=1 << apm.APM_G16,
                                              flags=apm.APM_POOL_NO_ZERO, base={apm.APM_G16: ptr})
        apm.apm_pack_tensors(halves[ptr], apm.APM_G16, g_tensors[k & 1], wl.n_t, stream)
        return ptr
    for k in range(2):      # create both alias pools and warm up
        apm.apm_step_delayed(pool, None, n_pages, produce(k), hyper, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        apm.apm_step_delayed(pool, None, n_pages, produce(k), hyper, stream)
    apm.apm_step_delayed(pool, None, n_pages, None, hyper, stream)      # flush
    torch.cuda.synchronize()
    t_del = (time.perf_counter() - t0) / steps
    for h in halves.values():
        h.destroy()
    return {"steps": steps, "sync_ms_per_step": t_sync * 1e3, "delayed_ms_per_step": t_del * 1e3,
            "producer": "apm_pack_tensors of the step's bf16 gradient tensors into page layout",
            "applied_updates": apm.apm_delayed_applied(pool)}


def moe_active_list_leg(args, wl, pool, hyper, plan, first_step):
    """The MoE step when the caller already knows which experts received tokens and lists only
    their pages (plus the dense ones), against the default of listing every page and letting the
    device find the all-zero ones."""
    import torch
    import paper_2303_02868_amd as apm
    import synth
    stream = torch.cuda.current_stream()
    lists, g_tensors, keep = [], [], []
    for k in range(2):
        act = synth.moe_active_tensors(wl.specs, k + 1, 0, 64, 8)
        pages = sorted({pg for (t, _, pg, _, _) in plan.segments if act[t]})
        lists.append(pages)
        g = wl.gen(1001 + k, True, 1e-3, act)
        keep.append(g)
        g_tensors.append(wl.tensors(g))
    p16_flat = torch.zeros(wl.total, dtype=torch.bfloat16, device=DEV)
    p16_tensors = wl.tensors(p16_flat)
    steps = max(4, args.steps // 2)
    t = first_step
    for k in range(2):
        apm.apm_page_adamw_step_fused(pool, lists[k], len(lists[k]), t, hyper, g_tensors[k], p16_tensors,
                                      wl.n_t, None, None, stream)
        t += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        apm.apm_page_adamw_step_fused(pool, lists[k & 1], len(lists[k & 1]), t, hyper, g_tensors[k & 1],
                                      p16_tensors, wl.n_t, None, None, stream)
        t += 1
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    active = sum(sum(n for n, a in zip(wl.numels, synth.moe_active_tensors(wl.specs, k + 1, 0, 64, 8)) if a)
                 for k in range(2)) / 2.0
    return {"ms_per_step": dt * 1e3, "listed_pages": [len(x) for x in lists],
            "useful_params_per_s": active / dt}


def d2d_copy_ceiling():
    import torch
    n_copy = 1 << 29
    src = torch.empty(n_copy, dtype=torch.float32, device=DEV)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 10 * 2 * n_copy * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def pcie_raw(host, devp, n_pages, E, state):
    """Plain pinned copies through apm_page_copy_async: H2D alone, D2H alone, both at once.
    Returns GB/s per direction."""
    import torch
    import paper_2303_02868_amd as apm
    run = min(256, n_pages // 2)            # pages per copy (1 GiB at E = 1 Mi)
    reps = max(2, min(8, (n_pages // 2) // run))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    nbytes = reps * run * E * 4
    half = n_pages // 2

    def go(h2d, d2h):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(reps):
            if h2d:
                apm.apm_page_copy_async(devp, (r * run) % (half - run + 1), host, (r * run) % (half - run + 1), run, state, s1)
            if d2h:
                apm.apm_page_copy_async(host, half + (r * run) % (half - run + 1), devp, half + (r * run) % (half - run + 1), run, state, s2)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    go(True, True)
    th = go(True, False)
    td = go(False, True)
    tb = go(True, True)
    return {"h2d_GBps": nbytes / th / 1e9, "d2h_GBps": nbytes / td / 1e9,
            "duplex_each_GBps": nbytes / tb / 1e9, "copy_bytes": run * E * 4}


def note(msg):
    """Progress on stderr (stdout carries the one JSON line): long legs say where they are."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


PCIE_GEN5_X16_RAW_GBPS = 64.0   # 32 GT/s x 16 lanes, 128b/130b: raw rate per direction


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2] if len(xs) % 2 else 0.5 * (xs[len(xs) // 2 - 1] + xs[len(xs) // 2])


def time_streamer(args, streamer, hyper, first_step, n_pages, E, raw, total_params):
    """The three streaming modes -- direct (the update kernel reads and writes the host pages),
    staged (slot ring moved by the library's duplex copy kernel) and staged_dma (slot ring moved by
    the runtime's asynchronous copies) -- timed step by step (median and min), each staged mode
    with its copy-only pipeline.  Every mode is credited with the parameters' 12 B each way only
    (padding that page copies move as well is not credited) and held against named denominators:
    plain pinned copies measured in the same run (one direction alone, both at once) and the raw
    Gen5 x16 rate.  `update_hidden` is computed for every mode: T_step <= 1.02 x the time plain
    copies of the same bytes take with both directions busy (the slower of the one-way and duplex
    raw rates)."""
    import torch
    import paper_2303_02868_amd as apm
    stream = torch.cuda.current_stream()

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    t = [first_step]

    def full():
        apm.apm_streamer_step(streamer, t[0], hyper, None, None, stream)
        t[0] += 1

    each_way = total_params * 12                    # credited: the parameters' fp32 state
    moved_pages = n_pages * E * 12                  # what whole-page copies move
    if raw:
        t_raw = each_way / 1e9 / min(raw["duplex_each_GBps"], raw["h2d_GBps"], raw["d2h_GBps"])
    out_modes = {}
    for name, mode in (("direct", apm.APM_STREAM_DIRECT), ("staged", apm.APM_STREAM_STAGED),
                       ("staged_dma", apm.APM_STREAM_STAGED_DMA)):
        apm.apm_streamer_set_mode(streamer, mode, args.direct_wavefronts)
        note(f"streamed step, mode {name}")
        full()                                      # warm-up
        walls, boths = [], []
        for _ in range(args.stream_steps):
            if mode != apm.APM_STREAM_DIRECT:       # interleaved with the steps: the link is shared
                boths.append(timed(lambda: apm.apm_streamer_copy_only(streamer, 3, stream)))
            walls.append(timed(full))
        wall = _median(walls)
        r = {"ms_per_step": wall * 1e3, "ms_per_step_min": min(walls) * 1e3,
             "ms_per_step_all": [w * 1e3 for w in walls],
             "pcie_GBps_each_way": each_way / wall / 1e9, "bytes_credited_each_way": each_way,
             # the update kernel and the library's copy kernel move used extents only; the runtime's
             # copies move whole pages
             "bytes_moved_each_way": moved_pages if mode == apm.APM_STREAM_STAGED_DMA else each_way}
        if mode == apm.APM_STREAM_DIRECT:
            r["wavefronts"] = args.direct_wavefronts or "library default (48)"
            r["hbm_staging_bytes"] = 0
        else:
            t_h2d = timed(lambda: apm.apm_streamer_copy_only(streamer, 1, stream))
            t_d2h = timed(lambda: apm.apm_streamer_copy_only(streamer, 2, stream))
            t_both = _median(boths)
            r.update({"batch_pages": min(args.batch_pages, n_pages), "slots": args.slots,
                      "copy_only_pipeline": {"both_ms": t_both * 1e3, "both_ms_all": [x * 1e3 for x in boths],
                                             "h2d_only_ms": t_h2d * 1e3, "d2h_only_ms": t_d2h * 1e3,
                                             "both_GBps_each_way_moved": r["bytes_moved_each_way"] / t_both / 1e9},
                      "step_over_own_copy_only_pipeline": wall / max(t_both, t_h2d, t_d2h)})
            if mode == apm.APM_STREAM_STAGED_DMA:
                r["stream_calibration_GBps"] = dict(zip(("h2d", "d2h", "duplex_each_way"),
                                                        apm.apm_streamer_probe_rates(streamer)))
        if raw:
            r["frac_of_raw_duplex_copies"] = r["pcie_GBps_each_way"] / raw["duplex_each_GBps"]
            r["frac_of_raw_one_way_copy"] = r["pcie_GBps_each_way"] / min(raw["h2d_GBps"], raw["d2h_GBps"])
            r["update_hidden"] = bool(wall <= 1.02 * t_raw)
            r["step_over_raw_copy_time"] = wall / t_raw
        r["frac_of_gen5_x16_raw_64GBps"] = r["pcie_GBps_each_way"] / PCIE_GEN5_X16_RAW_GBPS
        out_modes[name] = r

    best_mode = min(out_modes, key=lambda k: out_modes[k]["ms_per_step"])
    best = out_modes[best_mode]
    out = {"mode": best_mode, "ms_per_step": best["ms_per_step"], "params_per_s": total_params / (best["ms_per_step"] * 1e-3),
           "pcie_GBps_each_way": best["pcie_GBps_each_way"], "bytes_each_way": each_way,
           "host_pinned_GB": moved_pages / 1e9,
           "timing": "median of --stream-steps single steps, each bracketed by device synchronisation",
           "update_hidden": best.get("update_hidden"),
           "update_hidden_criterion": "median step time <= 1.02 x time of plain pinned copies of the credited bytes "
                                      "at the slowest of the raw rates below (h2d alone, d2h alone, each way with both busy)",
           "frac_of_raw_duplex_copies": best.get("frac_of_raw_duplex_copies"),
           "frac_of_raw_one_way_copy": best.get("frac_of_raw_one_way_copy"),
           "frac_of_gen5_x16_raw_64GBps": best["frac_of_gen5_x16_raw_64GBps"]}
    out.update(out_modes)
    if raw:
        out["raw_pinned_copy"] = dict(raw)
        # the runtime overlaps its two copy directions in some processes and not in others; when
        # it does not, the denominators above are weak and the fractions flatter the modes
        out["raw_pinned_copy"]["duplex_degraded"] = bool(raw["duplex_each_GBps"] < 0.75 * min(raw["h2d_GBps"], raw["d2h_GBps"])
                                                       or min(raw["h2d_GBps"], raw["d2h_GBps"]) < 45.0)
    apm.apm_streamer_set_mode(streamer, {"direct": apm.APM_STREAM_DIRECT, "staged": apm.APM_STREAM_STAGED,
                                         "staged_dma": apm.APM_STREAM_STAGED_DMA}[best_mode], args.direct_wavefronts)
    return out


def _mode_const(name):
    import paper_2303_02868_amd as apm
    return {"direct": apm.APM_STREAM_DIRECT, "staged": apm.APM_STREAM_STAGED,
            "staged_dma": apm.APM_STREAM_STAGED_DMA}[name]


def layer_bounds(wl):
    """Page ranges of the model's blocks (a page belongs to the block of its first tenant)."""
    import paper_2303_02868_amd as apm
    plan = apm.apm_pack_plan(wl.E, wl.numels)
    first = {}
    for tensor, _, page, _, _ in plan.segments:
        first.setdefault(page, tensor)
    bounds, prev = [0], None
    for page in range(plan.n_pages):
        blk = (wl.specs[first[page]].layer, wl.specs[first[page]].expert)
        if prev is not None and blk != prev:
            bounds.append(page)
        prev = blk
    bounds.append(plan.n_pages)
    return bounds


def scheduled_leg(args, wl, host, dev_pool, hyper, n_pages, first_step):
    """The streamed step with its page movement planned by the life-time based scheduler for a GPU
    memory of --sched-layers times the largest block."""
    import torch
    import paper_2303_02868_amd as apm
    E = wl.E
    bounds = layer_bounds(wl)
    largest = max(b - a for a, b in zip(bounds, bounds[1:]))
    budget = min(n_pages, int(args.sched_layers * largest))
    page_bytes = 12 * E
    t0 = time.perf_counter()
    tasks, peak = apm.apm_schedule_plan([(range(a, b), 0) for a, b in zip(bounds, bounds[1:])], None,
                                        page_bytes, budget * page_bytes)
    t_plan = time.perf_counter() - t0
    streamer = apm.apm_streamer_create(host, dev_pool, (budget + 1) // 2, 2)
    stream = torch.cuda.current_stream()
    note("schedule-driven step")
    apm.apm_streamer_step_scheduled(streamer, tasks, bounds, first_step, hyper, None, None, stream)
    ts = []
    for k in range(args.stream_steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        apm.apm_streamer_step_scheduled(streamer, tasks, bounds, first_step + 1 + k, hyper, None, None, stream)
        torch.cuda.synchronize()
        ts.append(time.perf_counter() - t0)
    streamer.destroy()
    each_way = wl.total * 12          # credited: the parameters' 12 B each way (the copy kernels move no padding)
    med = statistics.median(ts)
    return {"blocks": len(bounds) - 1, "largest_block_pages": largest, "gpu_memory_pages": budget,
            "planned_peak_pages": peak // page_bytes,
            "pages_moved_before_first_compute": next(i for i, t in enumerate(tasks) if t[0] == apm.APM_TASK_COMPUTE),
            "mover": "the library's copy kernel; a layer's write-back and the movements that are due share a launch",
            "plan_ms": t_plan * 1e3, "ms_per_step": med * 1e3, "ms_per_step_all": [t * 1e3 for t in ts],
            "pcie_GBps_each_way": each_way / med / 1e9, "bytes_credited_each_way": each_way}


def one_way_traffic_beside_a_producer(streamer, iters):
    """Why the overlap is incomplete: an elementwise producer (gelu over 2^28 bf16 values, many short
    HBM-bound kernels) timed alone and beside the staged pipeline's page traffic in one direction
    only, then both (the copy-only pipeline: no update kernels).  Pages arriving (PCIe reads) barely
    disturb it; pages leaving (a kernel's writes to host memory) stretch it."""
    import torch
    import paper_2303_02868_amd as apm
    side = _stream_beside_the_current_one()
    x = torch.randn(1 << 28, device=DEV, dtype=torch.bfloat16)
    one = lambda: torch.nn.functional.gelu(x)
    apm.apm_streamer_set_mode(streamer, apm.APM_STREAM_STAGED, 0, 0)

    def timed(fn):
        ts = []
        for _ in range(iters):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return statistics.median(ts)

    for _ in range(10):
        one()
    per = timed(lambda: [one() for _ in range(50)]) / 50
    reps = max(1, int(0.65 / per))           # about twice one pass of the pages: the traffic ends inside it

    def prod():
        for _ in range(reps):
            one()

    t_p = timed(prod)
    out = {"producer": f"{reps} gelu calls over 2^28 bf16 values", "producer_alone_ms": t_p * 1e3}
    note("elementwise producer beside one-way page traffic")
    for d, name, wt in ((1, "host_to_device_only", False), (2, "device_to_host_only", False), (3, "both_directions", False),
                        (2, "device_to_host_only_written_through", True), (3, "both_directions_written_through", True)):
        apm.apm_streamer_set_host_write_through(streamer, wt)
        apm.apm_streamer_copy_only(streamer, d, side)
        t_c = timed(lambda: apm.apm_streamer_copy_only(streamer, d, side))

        def together():
            apm.apm_streamer_copy_only(streamer, d, side)
            prod()

        t_b = timed(together)
        out[name] = {"traffic_alone_ms": t_c * 1e3, "together_ms": t_b * 1e3,
                     "producer_stretched_by_ms": (t_b - t_p) * 1e3}
    apm.apm_streamer_set_host_write_through(streamer, False)
    del x
    return out


def _stream_beside_the_current_one():
    """A side stream whose work runs beside the current stream's.  Streams that the runtime maps
    onto one hardware queue run their work in order -- an event wait on one holds up the kernels of
    the other -- so candidates are tried with a pair of short sleeps until one overlaps."""
    import torch
    cycles = 2_000_000

    def both(side):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(side):
            torch.cuda._sleep(cycles)
        torch.cuda._sleep(cycles)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    torch.cuda._sleep(cycles)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    torch.cuda._sleep(cycles)
    torch.cuda.synchronize()
    one = time.perf_counter() - t0
    kept = []
    for _ in range(6):
        side = torch.cuda.Stream()
        kept.append(side)               # rejected ones stay alive: a freed queue slot would be handed out again
        both(side)
        if min(both(side), both(side)) < 1.6 * one:
            return side
    return kept[-1]


def lockfree_leg(args, streamer, dev_pool, hyper, update_ms):
    """Alg. 2's point on one GPU: the update of host-resident state runs beside the producer of the
    next gradient instead of after it.  The producer here is a stand-in for forward/backward (which
    this build does not have): dense bf16 matrix products through the BLAS library, sized to take
    about as long as one streamed update.  Synchronous: products, then apm_streamer_step.
    One-step-stale: apm_streamer_step_delayed (applies the previous gradient on the update stream),
    then the products.  Measured for four ways of streaming.  The library's large matrix products
    are a hard neighbour: they run 1.65-1.85x slower beside ANY second kernel, even one idle
    thread spinning on one CU (attention and elementwise kernels do not care), so the two
    kernel-driven ways are measured beside an attention producer as well (causal scaled-dot-product
    attention, 8 x 32 heads x 2048 x 128, through the framework's fused kernel)."""
    import torch
    import paper_2303_02868_amd as apm
    stream = torch.cuda.current_stream()
    g16 = apm.apm_pool_state_ptr(dev_pool, apm.APM_G16)
    iters = max(3, args.stream_steps)
    step = [1000]

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters

    def update_only():
        apm.apm_streamer_step(streamer, step[0], hyper, None, None, stream)
        step[0] += 1

    def measure(kind, ways):
        if kind == "attention":
            q = torch.randn(8, 32, 2048, 128, device=DEV, dtype=torch.bfloat16)
            one = lambda: torch.nn.functional.scaled_dot_product_attention(q, q, q, is_causal=True)
            what, flops = "causal attention calls (8 x 32 heads x 2048 x 128)", 2.0 * 8 * 32 * 2048 * 2048 * 128
        else:
            n = 8192
            a = torch.randn(n, n, device=DEV, dtype=torch.bfloat16)
            b = torch.randn(n, n, device=DEV, dtype=torch.bfloat16)
            c = torch.empty(n, n, device=DEV, dtype=torch.bfloat16)
            one = lambda: torch.matmul(a, b, out=c)
            what, flops = f"bf16 {n}^3 matrix products", 2.0 * n ** 3

        def products(reps):
            for _ in range(reps):
                one()

        products(10)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        products(50)
        torch.cuda.synchronize()
        per = (time.perf_counter() - t0) / 50
        reps = max(1, int(round(update_ms * 1e-3 / per)))
        t_compute = timed(lambda: products(reps))

        def sync_iter():
            products(reps)
            update_only()

        def delayed_iter():
            apm.apm_streamer_step_delayed(streamer, g16, hyper, stream)
            products(reps)

        out = {"producer": f"{reps} {what} per iteration (stand-in for forward/backward)",
               "producer_TFLOPs_alone": flops * reps / t_compute / 1e12, "producer_ms": t_compute * 1e3}
        for name, mode, waves, per_wg in ways:
            apm.apm_streamer_set_mode(streamer, mode, waves, per_wg)
            apm.apm_streamer_set_host_write_through(streamer, name.endswith("written_through"))
            note(f"one-step-stale beside {kind}: {name}")
            update_only()
            t_update = timed(update_only)
            t_sync = timed(sync_iter)
            apm.apm_streamer_step_delayed(streamer, g16, hyper, stream)      # fill the pipeline
            t_delayed = timed(delayed_iter)
            apm.apm_streamer_step_delayed(streamer, None, hyper, stream)     # flush
            torch.cuda.synchronize()
            out[name] = {"update_ms": t_update * 1e3, "synchronous_ms_per_iter": t_sync * 1e3,
                         "one_step_stale_ms_per_iter": t_delayed * 1e3, "speedup": t_sync / t_delayed,
                         "hidden_fraction_of_the_shorter": (t_sync - t_delayed) / min(t_compute, t_update),
                         "over_ideal_max_of_the_two": t_delayed / max(t_compute, t_update),
                         "streams_run_beside_the_producer": dict(zip(("update_stream", "pipeline_streams"),
                                                                     apm.apm_streamer_overlap_report(streamer)))}
        apm.apm_streamer_set_host_write_through(streamer, False)
        best = min((k for k in out if isinstance(out[k], dict)), key=lambda k: out[k]["one_step_stale_ms_per_iter"])
        out["best"] = {"way": best, **out[best]}
        return out

    kernel_ways = [("direct_128_wavefronts_on_8_CUs", apm.APM_STREAM_DIRECT, 128, 16),
                   ("staged_128_wavefronts_on_8_CUs", apm.APM_STREAM_STAGED, 128, 16)]
    ways = [("direct_64_wavefronts_on_64_CUs", apm.APM_STREAM_DIRECT, 64, 1)] + kernel_ways + \
           [("staged_dma", apm.APM_STREAM_STAGED_DMA, 0, 0)]
    if args.lockfree_sweep:     # wavefronts x workgroup packing of the kernel that crosses PCIe
        ways = [(f"{m}_{w}_wavefronts_{p}_per_workgroup", c, w, p)
                for m, c in (("direct", apm.APM_STREAM_DIRECT), ("staged", apm.APM_STREAM_STAGED))
                for w, p in ((48, 1), (64, 8), (80, 16), (96, 16), (128, 16), (160, 16), (256, 16))]
        ways.append(("staged_dma", apm.APM_STREAM_STAGED_DMA, 0, 0))
    wt_way = [("direct_128_wavefronts_on_8_CUs_host_stores_written_through", apm.APM_STREAM_DIRECT, 128, 16)]
    out = measure("matmul", ways + wt_way)
    out["beside_attention"] = measure("attention", kernel_ways[:1] + wt_way)
    out["elementwise_producer_beside_page_traffic_one_way"] = one_way_traffic_beside_a_producer(streamer, 2)
    return out


def file_tier_leg(args, wl, hyper, n_pages):
    """fp32 state in files under --file-tier DIR, streamed through a pinned window (buffered and
    unbuffered I/O), and the one-step-stale form beside a matrix-product producer."""
    import torch
    import paper_2303_02868_amd as apm
    E = wl.E
    import synth
    dev_pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages, state_mask=apm.B16_STATES)
    # MoE: the experts of one step's draw have a gradient; skipped pages then need no file I/O
    act = synth.moe_active_tensors(wl.specs, 1, 0, 64, 8) if wl.name == "moe_8x64" else None
    apm.apm_pack_tensors(dev_pool, apm.APM_G16, wl.tensors(wl.gen(1001, True, 1e-3, act)), wl.n_t)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=1 << apm.APM_P32)
    tmp = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages, state_mask=1 << apm.APM_P32)
    apm.apm_pack_tensors(tmp, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    apm.apm_page_copy_async(host, 0, tmp, 0, n_pages, apm.APM_P32)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    each_way = n_pages * E * 12
    out = {"dir": args.file_tier, "bytes_each_way": each_way, "batch_pages": min(args.tier_batch_pages, n_pages),
           "slots": args.slots, "io_threads": args.io_threads}
    for name, flags in (("buffered", 0), ("unbuffered", apm.APM_POOL_FILE_DIRECT)):
        prefix = os.path.join(args.file_tier, f"apm_bench_{os.getpid()}_{name}")
        filep = apm.apm_file_pool_create(prefix, E, n_pages, flags=flags)
        t0 = time.perf_counter()
        apm.apm_page_copy_async(filep, 0, host, 0, n_pages, apm.APM_P32)
        t_init = time.perf_counter() - t0
        tier = apm.apm_tiered_create(filep, dev_pool, min(args.tier_batch_pages, n_pages), args.slots, args.io_threads)
        apm.apm_tiered_step(tier, 1, hyper, None, None, stream)
        ts = []
        for k in range(args.stream_steps):
            t0 = time.perf_counter()
            apm.apm_tiered_step(tier, 2 + k, hyper, None, None, stream)
            ts.append(time.perf_counter() - t0)
        rd, wr = apm.apm_tiered_io_bytes(tier)
        per_step = rd / (1 + args.stream_steps)          # bytes read (= written) per step
        res = {"write_p32_GBps": n_pages * E * 4 / t_init / 1e9, "ms_per_step": min(ts) * 1e3,
               "ms_per_step_all": [t * 1e3 for t in ts], "io_bytes_each_way_per_step": per_step,
               "io_GBps_each_way": per_step / min(ts) / 1e9, "params_per_s": wl.total / min(ts)}
        if name == "unbuffered":
            # Alg. 2: products (stand-in for forward/backward) sized to one update, then the update;
            # against the update running on the library's updater thread beside the products
            n = 8192
            a = torch.randn(n, n, device=DEV, dtype=torch.bfloat16)
            b = torch.randn(n, n, device=DEV, dtype=torch.bfloat16)
            c = torch.empty(n, n, device=DEV, dtype=torch.bfloat16)
            for _ in range(10):
                torch.matmul(a, b, out=c)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(50):
                torch.matmul(a, b, out=c)
            torch.cuda.synchronize()
            reps = max(1, int(round(min(ts) / ((time.perf_counter() - t0) / 50))))
            g16 = apm.apm_pool_state_ptr(dev_pool, apm.APM_G16)

            def products():
                for _ in range(reps):
                    torch.matmul(a, b, out=c)
                torch.cuda.synchronize()          # the producer's gradient is complete

            iters = 3
            t0 = time.perf_counter()
            for k in range(iters):
                products()
                apm.apm_tiered_step(tier, 10 + k, hyper, None, None, stream)
            t_sync = (time.perf_counter() - t0) / iters
            apm.apm_tiered_step_delayed(tier, g16, hyper, stream)
            t0 = time.perf_counter()
            for k in range(iters):
                apm.apm_tiered_step_delayed(tier, g16, hyper, stream)
                products()
            t_stale = (time.perf_counter() - t0) / iters
            apm.apm_tiered_step_delayed(tier, None, hyper, stream)
            res["lock_free"] = {"producer": f"{reps} bf16 {n}^3 matrix products per iteration",
                                "synchronous_ms_per_iter": t_sync * 1e3, "one_step_stale_ms_per_iter": t_stale * 1e3,
                                "speedup": t_sync / t_stale}
        tier.destroy()
        filep.destroy()
        for suffix in (".p32", ".m32", ".v32"):
            os.remove(prefix + suffix)
        out[name] = res
    for p in (tmp, host, dev_pool):
        p.destroy()
    return out


def streamed_leg(args, wl, dev_pool, hyper, n_pages, first_step):
    """fp32 state in pinned host pages; dev_pool supplies G16/P16 and the layout."""
    import torch
    import paper_2303_02868_amd as apm
    E = wl.E
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
    has_fp32 = bool(dev_pool.desc.state_mask & 1)
    stage_src = dev_pool
    if has_fp32:
        for st in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
            apm.apm_page_copy_async(host, 0, dev_pool, 0, n_pages, st)
        torch.cuda.synchronize()
    raw = None
    if has_fp32:
        raw = pcie_raw(host, dev_pool, n_pages, E, apm.APM_M32)
        for st in (apm.APM_P32, apm.APM_M32, apm.APM_V32):     # restore what the raw copies overwrote
            apm.apm_page_copy_async(dev_pool, 0, host, 0, n_pages, st)
        torch.cuda.synchronize()
    streamer = apm.apm_streamer_create(host, dev_pool, min(args.batch_pages, n_pages), args.slots)
    out = time_streamer(args, streamer, hyper, first_step, n_pages, E, raw, wl.total)
    out["scheduled"] = scheduled_leg(args, wl, host, dev_pool, hyper, n_pages, first_step + 50)
    out["lock_free"] = lockfree_leg(args, streamer, dev_pool, hyper, out["ms_per_step"])
    apm.apm_streamer_set_mode(streamer, _mode_const(out["mode"]), args.direct_wavefronts)
    if has_fp32:
        # mixed residency: half of the pages keep their fp32 state in HBM (the pool's own fp32
        # classes serve as the cache), the other half is streamed
        R = n_pages // 2
        apm.apm_streamer_set_cache(streamer, dev_pool, R)
        stream = torch.cuda.current_stream()
        apm.apm_streamer_step(streamer, first_step + 100, hyper, None, None, stream)
        ts = []
        for k in range(args.stream_steps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            apm.apm_streamer_step(streamer, first_step + 101 + k, hyper, None, None, stream)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        out["mixed_residency"] = {"resident_pages": R, "streamed_pages": n_pages - R, "mode": out["mode"],
                                  "ms_per_step": min(ts) * 1e3, "params_per_s": wl.total / min(ts)}
    streamer.destroy()
    host.destroy()
    return out


def flat_reference_leg(args):
    """1024 completely full pages (one tensor, no fragmentation) in the same process as the
    headline: the update kernel on full pages, in the page-class form (g16 and p16 are page
    classes) and in the fused form (g16 read from / p16 written to tensors), both with clipping."""
    import torch
    import paper_2303_02868_amd as apm
    wl = Workload("flat_1024pages")
    plan = apm.apm_pack_plan(wl.E, wl.numels)
    pool = apm.apm_pool_create(apm.APM_DEV_GPU, wl.E, plan.n_pages)
    apm.apm_pack_tensors(pool, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    torch.cuda.synchronize()
    hyper = apm.make_hyper(max_grad_norm=1.0)
    out = {"params": wl.total, "pages": plan.n_pages, "clip": 1.0}
    steps = max(5, args.steps // 2)
    t = 1
    for name, upd_only in (("page_class", True), ("fused", False)):
        a2 = argparse.Namespace(**vars(args))
        a2.update_only = upd_only
        r = resident_leg(a2, wl, pool, hyper, plan.n_pages, not upd_only, steps, 2, t)
        t = r["next_step"]
        out[name] = {"ms_per_step": r["wall"] * 1e3 / steps, "params_per_s": wl.total * steps / r["wall"],
                     "update_kernel_ms": r["upd_ms"], "update_kernel_GBps": r["achieved"],
                     "update_kernel_frac_of_peak": r["achieved"] / HBM_PEAK_GBPS,
                     "reduce_kernel_ms": r["kernels"].get("grad_reduce", {}).get("avg_ms")}
    pool.destroy()
    return out


def oracle_sample_timing(wl, plan, clip, skip, active=None, max_pages=48, steps=2):
    """The oracle (reduce + AdamW in double) timed on every k-th page of a configuration, with the
    pages' real used extents and -- for the MoE shape -- real mix of pages with and without
    gradient; the per-step time of the whole configuration is EXTRAPOLATED linearly from it."""
    import numpy as np
    import torch
    import oracle
    import synth
    E = wl.E
    used_all = plan_used(plan, plan.n_pages)
    every = max(1, plan.n_pages // max_pages)
    sample = list(range(0, plan.n_pages, every))
    used = [used_all[p] for p in sample]
    threads = min(16, os.cpu_count() or 1)
    rng_p = synth.normal_f32(0, 1, 0, len(sample) * E, 0.02, device=DEV).cpu().numpy().reshape(len(sample), E)
    g = synth.normal_bf16(0, 1001, 0, len(sample) * E, 1e-3, device=DEV).view(torch.int16).cpu().numpy().view(np.uint16).reshape(len(sample), E).copy()
    live = np.ones(len(sample), dtype=bool)
    if active is not None:      # pages none of whose tenants received a gradient are all zero
        page_live = np.zeros(plan.n_pages, dtype=bool)
        for tensor, _, page, _, _ in plan.segments:
            if active[tensor]:
                page_live[page] = True
        live = page_live[sample]
        g[~live] = 0
    st = oracle.PagedAdamWState(rng_p, used)
    h = oracle.Hyper(max_grad_norm=clip, skip_mode=int(skip))
    st.step(g, 1, h, threads=threads)
    t0 = time.perf_counter()
    for k in range(steps):
        st.step(g, 2 + k, h, threads=threads)
    dt = (time.perf_counter() - t0) / steps
    elems = float(sum(used))
    return {"kind": "oracle", "sampled_pages": len(sample), "every": every, "sampled_params": elems,
            "pages_with_gradient_in_sample": int(live.sum()), "cores": threads,
            "params_per_s": elems / dt,
            "ms_per_step_extrapolated": dt * 1e3 * (wl.total / elems) if elems else None,
            "note": "extrapolated linearly from the sampled pages (pages are independent)"}


def configs_leg(args):
    """Compact legs for the configurations the headline is not quoted on: the 124 M shape resident,
    the 13 B shape with its fp32 state in pinned host memory (at the depth the box can pin, and at
    its full 40 layers with the head cached in HBM), and the MoE shape (synchronous against
    one-step-stale, and with the caller listing the active pages).  Each with the oracle timed on a
    sample of its pages."""
    import torch
    import paper_2303_02868_amd as apm
    import synth
    out = {"cfg1_8pages": "correctness only: 59 MB moved per step is cache-resident and launch-bound (tests)"}

    # ---- cfg 2: GPT-2-small shape, resident ---------------------------------------------------
    wl = Workload("gpt2_small_124m")
    plan = apm.apm_pack_plan(wl.E, wl.numels)
    pool = apm.apm_pool_create(apm.APM_DEV_GPU, wl.E, plan.n_pages)
    apm.apm_pack_tensors(pool, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    torch.cuda.synchronize()
    hyper = apm.make_hyper()
    a2 = argparse.Namespace(**vars(args))
    a2.update_only = False
    r = resident_leg(a2, wl, pool, hyper, plan.n_pages, True, args.steps, args.warmup)
    out["cfg2_gpt2_small_124m"] = {
        "params": wl.total, "pages": plan.n_pages, "fragmentation": plan.fragmentation,
        "step": "fused AdamW reading g16 from / writing p16 to the tensors, no clipping",
        "ms_per_step": r["wall"] * 1e3 / args.steps, "params_per_s": wl.total * args.steps / r["wall"],
        "update_kernel_ms": r["upd_ms"], "update_kernel_GBps": r["achieved"],
        "update_kernel_frac_of_peak": r["achieved"] / HBM_PEAK_GBPS,
        "oracle": oracle_sample_timing(wl, plan, 0.0, 0, max_pages=plan.n_pages, steps=3)}
    pool.destroy()

    # ---- cfg 5: MoE shape, device-side skip; synchronous vs one-step-stale; active-page list ----
    wl = Workload("moe_8x64")
    plan = apm.apm_pack_plan(wl.E, wl.numels)
    pool = apm.apm_pool_create(apm.APM_DEV_GPU, wl.E, plan.n_pages)
    apm.apm_pack_tensors(pool, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    torch.cuda.synchronize()
    hyper = apm.make_hyper(skip_mode=apm.APM_SKIP_UNTOUCHED)
    steps = max(6, args.steps // 2)
    r = resident_leg(a2, wl, pool, hyper, plan.n_pages, True, steps, 2)
    act = synth.moe_active_tensors(wl.specs, 1, 0, 64, 8)
    c5 = {"params": wl.total, "pages": plan.n_pages, "fragmentation": plan.fragmentation,
          "active_params_per_step": r["elems_update"],
          "step": "grad reduce (finds the pages without gradient on the device) + fused AdamW, 1/8 of the expert pages active",
          "sync_fused": {"ms_per_step": r["wall"] * 1e3 / steps, "useful_params_per_s": r["elems_update"] * steps / r["wall"],
                         "update_kernel_ms": r["upd_ms"], "update_kernel_GBps_useful": r["achieved"],
                         "reduce_kernel_ms": r["kernels"].get("grad_reduce", {}).get("avg_ms")}}
    d = delayed_leg(a2, wl, pool, hyper, plan.n_pages, r["next_step"])
    c5["sync_vs_one_step_stale"] = d
    c5["sync_vs_one_step_stale"]["useful_params_per_s_sync"] = r["elems_update"] / (d["sync_ms_per_step"] * 1e-3)
    c5["sync_vs_one_step_stale"]["useful_params_per_s_delayed"] = r["elems_update"] / (d["delayed_ms_per_step"] * 1e-3)
    c5["caller_lists_active_pages"] = moe_active_list_leg(a2, wl, pool, hyper, plan, r["next_step"] + 100)
    c5["oracle"] = oracle_sample_timing(wl, plan, 0.0, 1, active=act, max_pages=64, steps=2)
    out["cfg5_moe_8x64"] = c5
    pool.destroy()
    torch.cuda.empty_cache()

    # ---- cfg 4: 13 B shape, fp32 state in pinned host memory ----------------------------------
    note("13 B shape, state in host memory")
    out["cfg4_gpt_13b"] = cfg4_leg(args)
    return out


def cfg4_leg(args):
    """One pinned host pool, as large as the box allows, serves two runs: (a) the 13 B shape at the
    depth whose whole fp32 state fits in it; (b) the full 40-layer shape with the head of the model
    cached in HBM and the tail in the host pool."""
    import torch
    import paper_2303_02868_amd as apm
    E = 1 << 20
    hyper = apm.make_hyper()
    stream = torch.cuda.current_stream()
    host = wl = plan = None
    for layers in (40, 32, 24, 16, 12, 8, 4):
        wl = Workload("gpt_13b", layers)
        plan = apm.apm_pack_plan(E, wl.numels)
        try:
            host = apm.apm_pool_create(apm.APM_DEV_HOST, E, plan.n_pages, state_mask=apm.FP32_STATES)
            break
        except apm.ApmError as e:
            if e.code != apm.APM_ENOMEM:
                raise
    n_host = plan.n_pages
    out = {"host_pool_pages": n_host, "host_pinned_GB": n_host * E * 12 / 1e9}

    def steps_of(streamer, first, n):
        apm.apm_streamer_step(streamer, first, hyper, None, None, stream)
        ts = []
        for k in range(n):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            apm.apm_streamer_step(streamer, first + 1 + k, hyper, None, None, stream)
            torch.cuda.synchronize()
            ts.append(time.perf_counter() - t0)
        return ts

    # (a) everything in host memory, reduced depth
    dev_pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_host, state_mask=apm.B16_STATES)
    apm.apm_pack_tensors(dev_pool, apm.APM_G16, wl.tensors(wl.gen(1001, True, 1e-3)), wl.n_t)
    tmp = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_host, state_mask=1 << apm.APM_P32)
    apm.apm_pack_tensors(tmp, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    apm.apm_page_copy_async(host, 0, tmp, 0, n_host, apm.APM_P32)
    torch.cuda.synchronize()
    streamer = apm.apm_streamer_create(host, dev_pool, min(args.batch_pages, n_host), args.slots)
    a = {"layers": wl.layers, "layers_of_full_shape": 40, "params": wl.total, "pages": n_host,
         "fragmentation": plan.fragmentation, "state": "fp32 p/m/v all in pinned host pages, bf16 g/p16 in HBM"}
    for name in ("direct", "staged"):
        apm.apm_streamer_set_mode(streamer, _mode_const(name), args.direct_wavefronts)
        ts = steps_of(streamer, 1 if name == "direct" else 20, 2)
        a[name] = {"ms_per_step": _median(ts) * 1e3, "ms_per_step_all": [x * 1e3 for x in ts],
                   "params_per_s": wl.total / _median(ts),
                   "pcie_GBps_each_way": wl.total * 12 / _median(ts) / 1e9,
                   "frac_of_gen5_x16_raw_64GBps": wl.total * 12 / _median(ts) / 1e9 / PCIE_GEN5_X16_RAW_GBPS}
    a["oracle"] = oracle_sample_timing(wl, plan, 0.0, 0, max_pages=40, steps=2)
    out["all_state_in_host_memory"] = a
    streamer.destroy()
    dev_pool.destroy()
    tmp.destroy()
    torch.cuda.empty_cache()

    # (b) the full shape: the head's fp32 state cached in HBM, the tail in the same host pool
    wl = Workload("gpt_13b", 40)
    plan = apm.apm_pack_plan(E, wl.numels)
    N = plan.n_pages
    n_tail = min(n_host, N)
    R = N - n_tail
    dev_pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, N, state_mask=apm.B16_STATES)
    apm.apm_pack_tensors(dev_pool, apm.APM_G16, wl.tensors(wl.gen(1001, True, 1e-3)), wl.n_t)
    p32 = torch.zeros((N, E), dtype=torch.float32, device=DEV)
    init = apm.apm_pool_create(apm.APM_DEV_GPU, E, N, state_mask=1 << apm.APM_P32, flags=apm.APM_POOL_NO_ZERO,
                               base={apm.APM_P32: p32})
    apm.apm_pack_tensors(init, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    apm.apm_page_copy_async(host, 0, init, R, n_tail, apm.APM_P32)
    torch.cuda.synchronize()
    mv = {s_: torch.zeros((max(R, 1), E), dtype=torch.float32, device=DEV) for s_ in (apm.APM_M32, apm.APM_V32)}
    cache = apm.apm_pool_create(apm.APM_DEV_GPU, E, max(R, 1), state_mask=apm.FP32_STATES,
                                flags=apm.APM_POOL_NO_ZERO, base={apm.APM_P32: p32, **mv})
    streamer = apm.apm_streamer_create(host, dev_pool, min(args.batch_pages, N), args.slots)
    apm.apm_streamer_set_cache(streamer, cache if R else None, R)
    apm.apm_streamer_set_host_first_page(streamer, R)
    ts = steps_of(streamer, 1, 2)
    used_tail = sum(plan_used(plan, N)[R:])
    out["full_40_layers_head_cached_in_hbm"] = {
        "params": wl.total, "pages": N, "fragmentation": plan.fragmentation, "resident_pages": R,
        "host_pages": n_tail, "hbm_cache_GB": R * E * 12 / 1e9, "mode": "direct",
        "ms_per_step": _median(ts) * 1e3, "ms_per_step_all": [x * 1e3 for x in ts],
        "params_per_s": wl.total / _median(ts),
        "pcie_GBps_each_way_host_part": used_tail * 12 / _median(ts) / 1e9,
        "oracle": oracle_sample_timing(wl, plan, 0.0, 0, max_pages=40, steps=2)}
    streamer.destroy()
    for p_ in (cache, init, dev_pool, host):
        p_.destroy()
    del p32, mv
    torch.cuda.empty_cache()
    return out


def cpu_baseline(args, E, n_pages, clip, skip):
    import numpy as np
    import torch
    import oracle
    import synth
    n_cpu = min(args.cpu_pages, n_pages)
    threads = min(16, os.cpu_count() or 1)
    used = np.full(n_cpu, E, dtype=np.int64)
    p_rows = synth.normal_f32(0, 1, 0, n_cpu * E, 0.02, device=DEV).cpu().numpy().reshape(n_cpu, E)
    g_rows = synth.normal_bf16(0, 1001, 0, n_cpu * E, 1e-3, device=DEV).view(torch.int16).cpu().numpy().view(np.uint16).reshape(n_cpu, E)
    st = oracle.PagedAdamWState(p_rows, used)
    h = oracle.Hyper(max_grad_norm=clip, skip_mode=int(skip))
    st.step(g_rows, 1, h, threads=threads)          # warm the pages
    c0 = time.perf_counter()
    for k in range(args.cpu_steps):
        st.step(g_rows, 2 + k, h, threads=threads)
    cw = time.perf_counter() - c0
    n_one = min(24, n_cpu)                           # the same oracle on one thread
    one = oracle.PagedAdamWState(p_rows[:n_one], used[:n_one])
    one.step(g_rows[:n_one], 1, h)
    c1 = time.perf_counter()
    one.step(g_rows[:n_one], 2, h)
    c1 = time.perf_counter() - c1
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": n_cpu * E * args.cpu_steps / cw, "unit": "params/s", "cores": threads,
            "kind": "oracle", "single_thread_value": n_one * E / c1, "cpu_model": model,
            "host_cpus": os.cpu_count(),
            "sample": f"{n_cpu} full pages x {args.cpu_steps} steps of the same update (reduce + AdamW "
                      f"in double), pages split over {threads} threads, {cw:.2f} s wall"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2303_02868_amd as apm

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = Workload(args.workload)
    E = wl.E
    clip = args.clip if args.clip is not None else (1.0 if args.workload == "gpt_1p3b" else 0.0)
    skip = apm.APM_SKIP_UNTOUCHED if args.workload == "moe_8x64" else apm.APM_SKIP_NONE
    hyper = apm.make_hyper(max_grad_norm=clip, skip_mode=skip)
    plan = apm.apm_pack_plan(E, wl.numels)
    n_pages = plan.n_pages
    streamed_only = args.streamed_only or args.workload == "gpt_13b"

    out = {"metric": "page AdamW params/s", "value": None, "unit": "params/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": args.workload, "params": wl.total, "pages": n_pages, "page_elems": E,
                      "fragmentation": plan.fragmentation, "clip": clip, "skip_mode": skip}}

    if args.page_sweep:
        out["page_sweep"] = page_sweep_leg(args)
        out["config"] = {"workload": "one tensor of 2^30 elements, page size swept"}
        out["steps"], out["warmup"] = 10, 2
        best = max(out["page_sweep"], key=lambda r: r["resident_update_GBps"])
        out["value"] = best["resident_update_GBps"] * 1e9 / BYTES_UPDATE
        out["ms_per_step"] = (1 << 30) / out["value"] * 1e3
        print(json.dumps(out))
        return
    if args.full_shape:
        fs = full_shape_leg(args, hyper)
        out["full_shape"] = fs
        out["value"], out["ms_per_step"] = fs["params_per_s"], fs["ms_per_step"]
        out["steps"], out["warmup"] = args.stream_steps, 1
        out["config"].update({"workload": "gpt_13b", "params": fs["params"], "pages": fs["pages"],
                              "fragmentation": fs["fragmentation"],
                              "step": "reduce + AdamW: cached pages in HBM, host pages across PCIe (direct mode)",
                              "state": "fp32 p/m/v: head cached in HBM, tail in pinned host pages; bf16 g/p16 in HBM"})
        print(json.dumps(out))
        return
    if args.file_tier:
        out["file_tier"] = file_tier_leg(args, wl, hyper, n_pages)
        out["value"] = out["file_tier"]["unbuffered"]["params_per_s"]
        out["ms_per_step"] = out["file_tier"]["unbuffered"]["ms_per_step"]
        out["steps"], out["warmup"] = args.stream_steps, 1
        out["config"]["step"] = "files -> pinned window -> AdamW kernel across PCIe -> files (unbuffered I/O)"
        out["config"]["state"] = "fp32 p/m/v in files, bf16 g/p16 resident in HBM"
        print(json.dumps(out))
        return
    if not streamed_only:
        pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages)
        p_flat = wl.gen(1, False, 0.02)
        apm.apm_pack_tensors(pool, apm.APM_P32, wl.tensors(p_flat), wl.n_t)
        torch.cuda.synchronize()
        del p_flat
        fused = not args.unfused and not args.update_only
        r = resident_leg(args, wl, pool, hyper, n_pages, fused, args.steps, args.warmup)
        out["value"] = r["elems_update"] * args.steps / r["wall"]
        out["ms_per_step"] = r["wall"] * 1e3 / args.steps
        out["config"]["step"] = ("reduce+update on resident pages" if args.update_only else
                                 "grad reduce + fused AdamW, both reading g16 from the tensors; p16 written to "
                                 "the tensors (pack/unpack fused into the kernels)" if fused else
                                 "pack_g16 + reduce + update + unpack_p16 (separate kernels)")
        if fused:   # the same step with separate pack / unpack kernels, for comparison
            r2 = resident_leg(args, wl, pool, hyper, n_pages, False, max(3, args.steps // 4), 1, r["next_step"])
            out["unfused_step"] = {"ms_per_step": r2["wall"] * 1e3 / max(3, args.steps // 4),
                                   "kernels": r2["kernels"]}
            r["next_step"] = r2["next_step"]
        out["config"]["state"] = "fp32 p/m/v + bf16 g/p16 resident in HBM"
        traffic = None
        pmc = os.path.join(ROOT, "profiles", f"adamw_update_{args.workload}_pmc.txt")
        if os.path.exists(pmc):
            for line in open(pmc):
                if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                    traffic = float(line.split("=", 1)[1])
        out["hbm_GBps_update_kernel"] = r["achieved"]
        out["hbm_frac_of_peak"] = r["achieved"] / HBM_PEAK_GBPS
        out["roofline"] = {"bound": "hbm", "kernel": "apm_adamw_kernel", "achieved": r["achieved"],
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": r["achieved"] / HBM_PEAK_GBPS,
                           "traffic": traffic,
                           "algorithmic_bytes_per_launch": r["elems_update"] * BYTES_UPDATE,
                           "avg_launch_ms": r["upd_ms"]}
        out["kernels"] = r["kernels"]
        out["d2d_copy_GBps"] = d2d_copy_ceiling()
        seg = out.get("unfused_step", {}).get("kernels", {}).get("seg_copy_bf16")
        if seg:   # this library's plain copy kernel in the same run: the practical ceiling beside the 8 TB/s
            out["roofline"]["plain_copy_kernel_GBps"] = seg["GBps"]
        if args.workload == "moe_8x64" and not args.update_only:
            out["delayed"] = delayed_leg(args, wl, pool, hyper, n_pages, r["next_step"])
            out["active_page_list"] = moe_active_list_leg(args, wl, pool, hyper, plan, r["next_step"] + 100)
        if not args.no_streamed:
            apm.apm_pack_tensors(pool, apm.APM_G16, wl.tensors(wl.gen(1001, True, 1e-3)), wl.n_t)
            note("streamed legs")
            out["streamed"] = streamed_leg(args, wl, pool, hyper, n_pages, r["next_step"])
        pool.destroy()
        torch.cuda.empty_cache()
        default_run = args.workload == "gpt_1p3b" and not (args.update_only or args.unfused or args.no_configs or
                                                            args.no_streamed)
        if default_run:
            note("full-page reference")
            out["flat_1024pages"] = flat_reference_leg(args)
            note("the other configurations")
            out["configs"] = configs_leg(args)
    else:
        # fp32 state never resident: the GPU pool holds G16/P16 only.  If the box cannot pin the
        # whole fp32 state, the depth of the 13 B shape shrinks until it fits (stated in the output).
        if args.workload == "gpt_13b":
            for layers in (40, 32, 24, 16, 8, 4):
                wl = Workload(args.workload, layers)
                plan = apm.apm_pack_plan(E, wl.numels)
                n_pages = plan.n_pages
                try:
                    probe = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES,
                                                flags=apm.APM_POOL_NO_ZERO)
                except apm.ApmError as e:
                    if e.code != apm.APM_ENOMEM:
                        raise
                    continue
                probe.destroy()
                break
            out["config"].update({"params": wl.total, "pages": n_pages, "layers_used": layers,
                                  "layers_of_full_shape": 40, "fragmentation": plan.fragmentation})
        dev_pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages, state_mask=apm.B16_STATES)
        apm.apm_pack_tensors(dev_pool, apm.APM_G16, wl.tensors(wl.gen(1001, True, 1e-3)), wl.n_t)
        torch.cuda.synchronize()
        note("streamed legs (state initialised in host memory)")
        s = streamed_leg_host_init(args, wl, dev_pool, hyper, n_pages)
        out["streamed"] = s
        out["value"] = s["params_per_s"]
        out["ms_per_step"] = s["ms_per_step"]
        out["steps"] = args.stream_steps
        out["warmup"] = 1
        out["config"]["step"] = ("grad reduce + AdamW kernel reading and writing p,m,v in pinned host pages across PCIe"
                                 if s["mode"] == "direct" else "copy-in p,m,v -> reduce+update -> copy-out p,m,v through HBM staging slots")
        out["config"]["state"] = "fp32 p/m/v in pinned host pages, bf16 g/p16 resident in HBM"
        dev_pool.destroy()

    if not args.no_cpu_baseline:
        note("oracle on the host cores")
        out["cpu_baseline"] = cpu_baseline(args, E, n_pages, clip, skip)
    print(json.dumps(out))


def streamed_leg_host_init(args, wl, dev_pool, hyper, n_pages):
    """Streamed leg for a model whose fp32 state is only ever host-resident (13 B parameters)."""
    import torch
    import paper_2303_02868_amd as apm
    E = wl.E
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
    # Master parameters: pack into a P32-only GPU pool and move the pages to the host.  That pool
    # stays alive until the end: on this platform, releasing a multi-GB device allocation lowered
    # device-to-host copy throughput (57 -> 30 GB/s) for the rest of the process.
    tmp = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages, state_mask=1 << apm.APM_P32)
    p_flat = wl.gen(1, False, 0.02)
    apm.apm_pack_tensors(tmp, apm.APM_P32, wl.tensors(p_flat), wl.n_t)
    apm.apm_page_copy_async(host, 0, tmp, 0, n_pages, apm.APM_P32)
    torch.cuda.synchronize()
    # raw PCIe: both pools hold the same P32 pages, so copying them either way changes nothing
    raw = pcie_raw(host, tmp, n_pages, E, apm.APM_P32)
    streamer = apm.apm_streamer_create(host, dev_pool, min(args.batch_pages, n_pages), args.slots)
    out = time_streamer(args, streamer, hyper, 1, n_pages, E, raw, wl.total)
    out["lock_free"] = lockfree_leg(args, streamer, dev_pool, hyper, out["ms_per_step"])
    streamer.destroy()
    out["scheduled"] = scheduled_leg(args, wl, host, dev_pool, hyper, n_pages, 50)
    host.destroy()
    tmp.destroy()
    return out


def page_sweep_leg(args):
    """Page size against throughput (Sec. 4.1 "Optimal Page Size" asks which page size keeps the
    transfer path busy): one tensor of 2^30 elements in pages of 2^14 .. 2^24 elements; the
    resident update kernel, the direct streamed step, and the staged step moving one page per copy."""
    import torch
    import paper_2303_02868_amd as apm
    total = 1 << 30
    hyper = apm.make_hyper()
    g = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    g.normal_(0, 1e-3)
    stream = torch.cuda.current_stream()
    rows = []
    for log_e in (14, 16, 18, 20, 22, 24):
        E = 1 << log_e
        n = total // E
        t16 = apm.make_tensors([total], apm.APM_BF16, [g])
        pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n)
        apm.apm_pack_tensors(pool, apm.APM_G16, t16, 1)
        for t in range(1, 3):
            apm.apm_page_adamw_step(pool, None, n, t, hyper, None, None, stream)
        torch.cuda.synchronize()
        apm.apm_pool_set_timing(pool, True)
        for t in range(3, 13):
            apm.apm_page_adamw_step(pool, None, n, t, hyper, None, None, stream)
        torch.cuda.synchronize()
        ms, launches = apm.apm_pool_read_timing(pool)
        upd = ms[apm.APM_K_UPDATE] / launches[apm.APM_K_UPDATE]
        row = {"page_elems": E, "fp32_page_bytes": 4 * E, "pages": n,
               "resident_update_GBps": total * BYTES_UPDATE / (upd * 1e-3) / 1e9}
        host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n, state_mask=apm.FP32_STATES)
        for st in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
            apm.apm_page_copy_async(host, 0, pool, 0, n, st)
        torch.cuda.synchronize()
        streamer = apm.apm_streamer_create(host, pool, 1, 4)
        for name, mode in (("direct", apm.APM_STREAM_DIRECT), ("staged_one_page_per_copy", apm.APM_STREAM_STAGED)):
            if mode == apm.APM_STREAM_STAGED and n > 16384:
                row[name + "_GBps_each_way"] = None      # hundreds of thousands of tiny copies: not timed
                continue
            apm.apm_streamer_set_mode(streamer, mode)
            apm.apm_streamer_step(streamer, 20, hyper, None, None, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            apm.apm_streamer_step(streamer, 21, hyper, None, None, stream)
            torch.cuda.synchronize()
            row[name + "_GBps_each_way"] = total * 12 / (time.perf_counter() - t0) / 1e9
        streamer.destroy()
        host.destroy()
        pool.destroy()
        if args.file_tier:
            row.update(file_tier_page_row(args, g, E, hyper, stream))
        rows.append(row)
    return rows


def file_tier_page_row(args, g, E, hyper, stream):
    """The file tier moving one page per batch (2^28 elements, 1 GiB per class): the page is then the
    unit of I/O, as it is the unit of the paper's SSD transfers."""
    import torch
    import paper_2303_02868_amd as apm
    total = 1 << 28
    n = total // E
    pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n, state_mask=apm.B16_STATES)
    apm.apm_pack_tensors(pool, apm.APM_G16, apm.make_tensors([total], apm.APM_BF16, [g]), 1)
    torch.cuda.synchronize()
    out = {}
    for name, flags in (("buffered", 0), ("unbuffered", apm.APM_POOL_FILE_DIRECT)):
        if flags and 4 * E % 4096:
            continue
        prefix = os.path.join(args.file_tier, f"apm_sweep_{os.getpid()}_{E}_{name}")
        filep = apm.apm_file_pool_create(prefix, E, n, flags=flags)     # zero-filled (sparse) files
        tier = apm.apm_tiered_create(filep, pool, 1, 8, args.io_threads)
        apm.apm_tiered_step(tier, 1, hyper, None, None, stream)          # writes every page once
        t0 = time.perf_counter()
        apm.apm_tiered_step(tier, 2, hyper, None, None, stream)
        out[f"file_{name}_one_page_per_batch_GBps_each_way"] = total * 12 / (time.perf_counter() - t0) / 1e9
        tier.destroy()
        filep.destroy()
        for suffix in (".p32", ".m32", ".v32"):
            os.remove(prefix + suffix)
    pool.destroy()
    return out


def full_shape_leg(args, hyper):
    """The 13 B shape at its full 40 layers: the host pool holds as much of the model's tail as the
    box can pin, the head's fp32 state is cached in HBM (Sec. 4.2's cache of optimizer states)."""
    import torch
    import paper_2303_02868_amd as apm
    wl = Workload("gpt_13b", 40)
    E = wl.E
    plan = apm.apm_pack_plan(E, wl.numels)
    N = plan.n_pages
    host = None
    for frac in (1.0, 0.45, 0.4, 0.3, 0.2, 0.1):
        n_host = int(N * frac)
        try:
            host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_host, state_mask=apm.FP32_STATES)
            break
        except apm.ApmError as e:
            if e.code != apm.APM_ENOMEM:
                raise
    R = N - n_host
    dev_pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, N, state_mask=apm.B16_STATES)
    apm.apm_pack_tensors(dev_pool, apm.APM_G16, wl.tensors(wl.gen(1001, True, 1e-3)), wl.n_t)
    p32 = torch.zeros((N, E), dtype=torch.float32, device=DEV)
    init = apm.apm_pool_create(apm.APM_DEV_GPU, E, N, state_mask=1 << apm.APM_P32, flags=apm.APM_POOL_NO_ZERO,
                               base={apm.APM_P32: p32})
    apm.apm_pack_tensors(init, apm.APM_P32, wl.tensors(wl.gen(1, False, 0.02)), wl.n_t)
    apm.apm_page_copy_async(host, 0, init, R, n_host, apm.APM_P32)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    mv = {s_: torch.zeros((max(R, 1), E), dtype=torch.float32, device=DEV) for s_ in (apm.APM_M32, apm.APM_V32)}
    cache = apm.apm_pool_create(apm.APM_DEV_GPU, E, max(R, 1), state_mask=apm.FP32_STATES,
                                flags=apm.APM_POOL_NO_ZERO, base={apm.APM_P32: p32, **mv})
    streamer = apm.apm_streamer_create(host, dev_pool, min(args.batch_pages, N), args.slots)
    apm.apm_streamer_set_cache(streamer, cache if R else None, R)
    apm.apm_streamer_set_host_first_page(streamer, R)
    stream = torch.cuda.current_stream()
    apm.apm_streamer_step(streamer, 1, hyper, None, None, stream)
    ts = []
    for k in range(args.stream_steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        apm.apm_streamer_step(streamer, 2 + k, hyper, None, None, stream)
        torch.cuda.synchronize()
        ts.append(time.perf_counter() - t0)
    used_host = sum(plan_used(plan, N)[R:])
    out = {"params": wl.total, "pages": N, "layers": 40, "fragmentation": plan.fragmentation, "resident_pages": R, "host_pages": n_host,
           "host_pinned_GB": n_host * E * 12 / 1e9, "hbm_cache_GB": R * E * 12 / 1e9, "mode": "direct",
           "ms_per_step": min(ts) * 1e3, "ms_per_step_all": [t * 1e3 for t in ts],
           "params_per_s": wl.total / min(ts), "pcie_GBps_each_way": used_host * 12 / min(ts) / 1e9}
    streamer.destroy()
    for p in (cache, init, host, dev_pool):
        p.destroy()
    return out


def plan_used(plan, n_pages):
    """Used elements per page of a packing plan."""
    used = [0] * n_pages
    for _, _, page, page_off, n in plan.segments:
        used[page] = max(used[page], page_off + n)
    return used


if __name__ == "__main__":
    main()
