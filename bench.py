#!/usr/bin/env python3
"""Benchmark of the page-AdamW hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients:
  pack g16 (tensors -> pages)  ->  per-page grad reduce  ->  fused page AdamW  ->  unpack p16
(the pool and the packing plan are set up once, as the method pre-allocates them).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt_1p3b",
                    choices=["cfg1_8pages", "gpt2_small_124m", "gpt_1p3b", "moe_8x64"])
    ap.add_argument("--clip", type=float, default=None, help="per-page max grad norm (default: 1.0 for gpt_1p3b, else off)")
    ap.add_argument("--update-only", action="store_true", help="time reduce+update only (no pack/unpack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-pages", type=int, default=192, help="pages of the workload the oracle is timed on")
    ap.add_argument("--cpu-steps", type=int, default=2)
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2303_02868_amd as apm
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    factory, E = synth.WORKLOADS[args.workload]
    specs = factory()
    numels = [t.numel for t in specs]
    n_t = len(specs)
    off = synth.tensor_offsets(specs)
    total = int(off[-1])
    clip = args.clip if args.clip is not None else (1.0 if args.workload == "gpt_1p3b" else 0.0)
    skip = apm.APM_SKIP_UNTOUCHED if args.workload == "moe_8x64" else apm.APM_SKIP_NONE
    hyper = apm.make_hyper(max_grad_norm=clip, skip_mode=skip)

    plan = apm.apm_pack_plan(E, numels)
    n_pages = plan.n_pages
    pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages)

    def gen(stream, bf16, sigma, active=None):
        out = torch.zeros(total, dtype=torch.bfloat16 if bf16 else torch.float32, device=dev)
        fn = synth.normal_bf16 if bf16 else synth.normal_f32
        chunk = 1 << 26
        for i in range(n_t):
            if active is not None and not active[i]:
                continue
            a0, n = int(off[i]), numels[i]
            for a in range(a0, a0 + n, chunk):
                m = min(chunk, a0 + n - a)
                out[a:a + m] = fn(0, stream, a, m, sigma, device=dev)
        return out

    def tensors(flat):
        dt = apm.APM_BF16 if flat.dtype == torch.bfloat16 else apm.APM_F32
        return apm.make_tensors(numels, dt, [flat.data_ptr() + int(off[i]) * flat.element_size()
                                             for i in range(n_t)])

    p_flat = gen(1, False, 0.02)
    apm.apm_pack_tensors(pool, apm.APM_P32, tensors(p_flat), n_t)
    torch.cuda.synchronize()
    del p_flat
    # two gradient sets, alternated (values do not affect timing; they keep the state finite)
    grads = []
    for k in range(2):
        act = synth.moe_active_tensors(specs, k + 1, 0, 64, 8) if args.workload == "moe_8x64" else None
        grads.append(gen(1001 + k, True, 1e-3, act))
    g_tensors = [tensors(g) for g in grads]
    p16_flat = torch.zeros(total, dtype=torch.bfloat16, device=dev)
    p16_tensors = tensors(p16_flat)
    if args.update_only:
        apm.apm_pack_tensors(pool, apm.APM_G16, g_tensors[0], n_t)
    stream = torch.cuda.current_stream()

    def step(t):
        if not args.update_only:
            apm.apm_pack_tensors(pool, apm.APM_G16, g_tensors[t & 1], n_t, stream)
        apm.apm_page_adamw_step(pool, None, n_pages, t, hyper, None, None, stream)
        if not args.update_only:
            apm.apm_unpack(pool, apm.APM_P16, p16_tensors, n_t, stream)

    t_step = 1
    for _ in range(args.warmup):
        step(t_step)
        t_step += 1
    torch.cuda.synchronize()
    apm.apm_pool_set_timing(pool, True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(t_step)
        t_step += 1
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms, launches = apm.apm_pool_read_timing(pool)
    apm.apm_pool_set_timing(pool, False)

    # active elements per step (skipped pages are not credited)
    if args.workload == "moe_8x64":
        act_elems = [int(sum(n for n, a in zip(numels, synth.moe_active_tensors(specs, k + 1, 0, 64, 8)) if a))
                     for k in range(2)]
        elems_update = sum(act_elems) / 2.0
    else:
        elems_update = float(total)
    ms_per_step = wall * 1e3 / args.steps
    value = elems_update * args.steps / wall

    def avg(cls):
        return ms[cls] / launches[cls] if launches[cls] else None

    upd_ms = avg(apm.APM_K_UPDATE)
    red_ms = avg(apm.APM_K_REDUCE)
    seg_ms = avg(apm.APM_K_SEGCOPY)
    achieved = elems_update * BYTES_UPDATE / (upd_ms * 1e-3) / 1e9
    kernels = {"adamw_update": {"avg_ms": upd_ms, "launches": launches[apm.APM_K_UPDATE],
                                "GBps": achieved, "bytes_per_elem": BYTES_UPDATE}}
    if red_ms:
        kernels["grad_reduce"] = {"avg_ms": red_ms, "launches": launches[apm.APM_K_REDUCE],
                                  "GBps": total * BYTES_REDUCE / (red_ms * 1e-3) / 1e9,
                                  "bytes_per_elem": BYTES_REDUCE}
    if seg_ms:
        kernels["seg_copy_bf16"] = {"avg_ms": seg_ms, "launches": launches[apm.APM_K_SEGCOPY],
                                    "GBps": total * BYTES_SEGCOPY_B16 / (seg_ms * 1e-3) / 1e9,
                                    "bytes_per_elem": BYTES_SEGCOPY_B16}

    # practical ceiling: a plain device-to-device copy of 2 GiB (read + write counted)
    n_copy = 1 << 29
    src = torch.empty(n_copy, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 10 * 2 * n_copy * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    traffic = None
    pmc = os.path.join(ROOT, "profiles", f"adamw_update_{args.workload}_pmc.txt")
    if os.path.exists(pmc):
        for line in open(pmc):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                traffic = float(line.split("=", 1)[1])

    out = {
        "metric": "page AdamW params/s", "value": value, "unit": "params/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "params": total, "pages": n_pages, "page_elems": E,
                   "fragmentation": plan.fragmentation, "clip": clip, "skip_mode": skip,
                   "step": "reduce+update" if args.update_only else "pack_g16+reduce+update+unpack_p16",
                   "state": "fp32 p/m/v + bf16 g/p16 resident in HBM"},
        "hbm_GBps_update_kernel": achieved, "hbm_frac_of_peak": achieved / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": "apm_adamw_kernel", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "algorithmic_bytes_per_launch": elems_update * BYTES_UPDATE,
                     "avg_launch_ms": upd_ms},
        "kernels": kernels,
        "d2d_copy_GBps": copy_gbps,
    }

    if not args.no_cpu_baseline:
        import oracle
        n_cpu = min(args.cpu_pages, n_pages)
        threads = min(16, os.cpu_count() or 1)
        used = np.full(n_cpu, E, dtype=np.int64)
        p_rows = synth.normal_f32(0, 1, 0, n_cpu * E, 0.02, device=dev).cpu().numpy().reshape(n_cpu, E)
        g_rows = synth.normal_bf16(0, 1001, 0, n_cpu * E, 1e-3, device=dev).view(torch.int16).cpu().numpy().view(np.uint16).reshape(n_cpu, E)
        st = oracle.PagedAdamWState(p_rows, used)
        h = oracle.Hyper(max_grad_norm=clip, skip_mode=int(skip))
        st.step(g_rows, 1, h, threads=threads)          # warm the pages
        c0 = time.perf_counter()
        for k in range(args.cpu_steps):
            st.step(g_rows, 2 + k, h, threads=threads)
        cw = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": n_cpu * E * args.cpu_steps / cw, "unit": "params/s",
                               "cores": threads, "kind": "oracle",
                               "sample": f"{n_cpu} full pages x {args.cpu_steps} steps of the same update "
                                         f"(reduce + AdamW in double), pages split over {threads} threads, "
                                         f"{cw:.2f} s wall"}
    pool.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
