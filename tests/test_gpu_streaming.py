"""Page copies and the streamed (host-resident fp32 state) update: copies are bit-exact, and the
streamed step is bit-identical to the resident step."""
import ctypes
import os

import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2303_02868_amd as apm
    from gpu_helpers import DEV, DevicePool, Model, bf16_bits, check_state_close, check_p16, to_hyper


def host_view(pool, state, n_pages, E):
    """numpy view of a library-allocated pinned host region."""
    ptr = apm.apm_pool_state_ptr(pool, state, 0)
    buf = (ctypes.c_float * (n_pages * E)).from_address(ptr)
    return np.frombuffer(buf, dtype=np.float32).reshape(n_pages, E)


def set_mode(streamer, mode):
    """"staged" | "direct" | "direct:<wavefronts>[:<per workgroup>]" (a small odd count makes every
    wavefront stride over many pages and slices)."""
    if mode.endswith("+wt"):        # stores to the host pool written through at system scope
        apm.apm_streamer_set_host_write_through(streamer, True)
        mode = mode[:-3]
    if mode.startswith("direct"):
        parts = mode.split(":")
        n = int(parts[1]) if len(parts) > 1 else 0
        per = int(parts[2]) if len(parts) > 2 else 0
        apm.apm_streamer_set_mode(streamer, apm.APM_STREAM_DIRECT, n, per)
        assert apm.apm_streamer_get_mode(streamer) == apm.APM_STREAM_DIRECT
    else:
        # "staged[:<wavefronts>]": the library's duplex copy kernel moves the batches;
        # "staged_dma": the runtime's asynchronous copies do
        assert apm.apm_streamer_get_mode(streamer) == apm.APM_STREAM_DIRECT   # pinned pool: the default
        parts = mode.split(":")
        want = apm.APM_STREAM_STAGED_DMA if parts[0] == "staged_dma" else apm.APM_STREAM_STAGED
        apm.apm_streamer_set_mode(streamer, want, int(parts[1]) if len(parts) > 1 else 0)
        assert apm.apm_streamer_get_mode(streamer) == want


def test_page_copy_roundtrip_bit_exact():
    E, n = 8192, 10
    dp = DevicePool(n, E)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n, state_mask=apm.FP32_STATES)
    x = synth.normal_f32(1, 5, 0, n * E, 1.0, device=DEV).view(n, E)
    dp.reg[apm.APM_M32].copy_(x)
    apm.apm_page_copy_async(host, 2, dp.pool, 3, 5, apm.APM_M32)           # D2H pages 3..7 -> 2..6
    torch.cuda.synchronize()
    hv = host_view(host, apm.APM_M32, n, E)
    assert np.array_equal(hv[2:7].view(np.uint32), x[3:8].cpu().numpy().view(np.uint32))
    assert not hv[:2].any() and not hv[7:].any()
    apm.apm_page_copy_async(dp.pool, 0, host, 2, 5, apm.APM_M32)  # H2D back
    torch.cuda.synchronize()
    assert torch.equal(dp.reg[apm.APM_M32][0:5], x[3:8])
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_copy_async(dp.pool, 8, host, 0, 3, apm.APM_M32)
    assert e.value.code == apm.APM_ERANGE
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_copy_async(host, 0, dp.pool, 0, 1, apm.APM_G16)
    assert e.value.code == apm.APM_ERANGE
    host.destroy()
    dp.destroy()


@pytest.mark.parametrize("batch,slots,clip,mode", [(4, 2, 0.0, "staged"), (7, 3, 1.0, "staged"), (64, 2, 1.0, "staged"),
                                                   (5, 4, 1.0, "staged:7"), (200, 3, 0.0, "staged"),
                                                   (5, 3, 1.0, "staged:9+wt"), (4, 2, 1.0, "direct:37:16+wt"),
                                                   (4, 2, 0.0, "staged_dma"), (7, 3, 1.0, "staged_dma"),
                                                   (4, 2, 0.0, "direct"), (4, 2, 1.0, "direct:7"), (4, 2, 1.0, "direct:37:16"),
                                                   (4, 2, 0.0, "direct:128:8")])
def test_streamed_equals_resident_bit_exact(batch, slots, clip, mode):
    # a GPT-2-small-sized model: resident run vs. fp32 state in pinned host pages streamed through
    # `slots` staging slots of `batch` pages
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=1)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    h = oracle.Hyper(max_grad_norm=clip)
    hy = to_hyper(h)
    steps = 3
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)

    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    # initial master parameters reach the host pool by page copies from the resident pool
    apm.apm_page_copy_async(host, 0, res.pool, 0, n_pages, apm.APM_P32)
    st = apm.apm_streamer_create(host, dev.pool, batch, slots)
    set_mode(st, mode)
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_s = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, steps + 1):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, None)
        apm.apm_streamer_step(st, t, hy, norm_s, None)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s)
    for s in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        hv = host_view(host, s, n_pages, E)
        assert np.array_equal(hv.view(np.uint32), res.reg[s].cpu().numpy().view(np.uint32)), f"state {s}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    st.destroy()
    host.destroy()
    dev.destroy()
    res.destroy()


@pytest.mark.parametrize("frac,mode,short_host", [(0.0, "staged", False), (0.35, "staged", False), (1.0, "staged", False),
                                                  (0.35, "direct", False), (1.0, "direct", False),
                                                  (0.35, "direct", True), (0.35, "staged", True),
                                                  (0.35, "staged_dma", False)])
def test_mixed_residency_equals_resident_bit_exact(frac, mode, short_host):
    # the first R pages keep their fp32 state in an HBM cache pool, the rest is streamed;
    # short_host: the host pool holds only the pages from H0 = R - 3 on (a model whose fp32 state
    # exceeds what can be pinned), its page j being model page H0 + j
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=2)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    R = int(round(frac * n_pages))
    hy = to_hyper(oracle.Hyper(max_grad_norm=1.0))
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    H0 = R - 3 if short_host else 0
    n_host = n_pages - H0
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_host, state_mask=apm.FP32_STATES)
    cache = DevicePool(max(R, 1), E, states=(apm.APM_P32, apm.APM_M32, apm.APM_V32))
    apm.apm_page_copy_async(host, 0, res.pool, H0, n_host, apm.APM_P32)
    if R:
        apm.apm_page_copy_async(cache.pool, 0, res.pool, 0, R, apm.APM_P32)
        # the host copy of the cached pages is stale from now on: poison it to prove it is unused
        hv = host_view(host, apm.APM_P32, n_host, E)
        torch.cuda.synchronize()
        hv[:R - H0] = np.nan
    st = apm.apm_streamer_create(host, dev.pool, 16, 3)
    apm.apm_streamer_set_cache(st, cache.pool if R else None, R)
    if short_host:
        with pytest.raises(apm.ApmError) as e:      # without the offset the host pool is too small
            apm.apm_streamer_step(st, 1, hy)
        assert e.value.code == apm.APM_ESTATE
        apm.apm_streamer_set_host_first_page(st, H0)
    set_mode(st, mode)
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_s = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, None)
        apm.apm_streamer_step(st, t, hy, norm_s, None)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s)
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        want = res.reg[s_].cpu().numpy().view(np.uint32)
        if R:
            assert np.array_equal(cache.reg[s_][:R].cpu().numpy().view(np.uint32), want[:R]), f"cached state {s_}"
        hv = host_view(host, s_, n_host, E)
        assert np.array_equal(hv[R - H0:].view(np.uint32), want[R:]), f"streamed state {s_}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    st.destroy()
    host.destroy()
    cache.destroy()
    dev.destroy()
    res.destroy()


def test_cfg4_gpt13b_shape_streamed_sampled_oracle():
    # GPT-13B-shaped layers (d = 5120, ffn = 20480); fp32 state only ever lives in pinned host pages.
    # The box decides how much can be pinned: the layer count shrinks until the host pool fits (the
    # full 40 layers need ~158 GB pinned), which changes the page count but not the path.
    from gpu_helpers import HOST_THREADS
    E = 1 << 20
    host = None
    for layers in (40, 32, 24, 16, 8, 4):
        specs = synth.gpt_tensor_list(layers, 5120, 20480, 50257, 2048)
        plan = oracle.plan_pack([t.numel for t in specs], E)
        try:
            host = apm.apm_pool_create(apm.APM_DEV_HOST, E, plan.n_pages, state_mask=apm.FP32_STATES)
            break
        except apm.ApmError as e:
            assert e.code == apm.APM_ENOMEM
            print(f"cfg4: {layers} layers ({plan.n_pages} pages) cannot be pinned: {e}", flush=True)
    assert host is not None
    model = Model(specs, E, seed=0)
    n_pages, n_t = plan.n_pages, len(specs)
    print(f"cfg4: {layers} layers, {model.total} params, {n_pages} pages, "
          f"{n_pages * E * 12 / 2**30:.1f} GiB pinned", flush=True)
    sample = sorted(set(range(0, n_pages, 257)) | {0, n_pages - 1}
                    | {k for k, p in enumerate(plan.pages) if p.used < E})
    used = [plan.pages[p].used for p in sample]
    h = oracle.Hyper(max_grad_norm=1.0)
    hy = to_hyper(h)

    tmp = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages, state_mask=1 << apm.APM_P32)
    apm.apm_pack_tensors(tmp, apm.APM_P32, model.tensors(model.p_flat), n_t)
    apm.apm_page_copy_async(host, 0, tmp, 0, n_pages, apm.APM_P32)
    torch.cuda.synchronize()
    st = oracle.PagedAdamWState(model.host_pages(model.p_flat, sample).view(np.float32), used)

    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, apm.make_tensors(model.numels, apm.APM_BF16), n_t)
    streamer = apm.apm_streamer_create(host, dev.pool, 32, 3)
    norm_d = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        # the middle step crosses PCIe from inside the update kernel, the others through staging
        apm.apm_streamer_set_mode(streamer, apm.APM_STREAM_DIRECT if t == 2 else apm.APM_STREAM_STAGED)
        apm.apm_streamer_step(streamer, t, hy, norm_d, None)
        norms, _ = st.step(model.host_pages(g, sample), t, h, threads=HOST_THREADS)
        torch.cuda.synchronize()
        got = norm_d.cpu().numpy()[sample]
        assert np.all(np.abs(got - norms) <= 1e-6 * np.abs(norms))
        del g
    rows = {}
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        rows[s_] = host_view(host, s_, n_pages, E)[sample]
    worst = {k: check_state_close(k, rows[s_], ref, used)
             for k, s_, ref in (("p", apm.APM_P32, st.p), ("m", apm.APM_M32, st.m), ("v", apm.APM_V32, st.v))}
    print(f"cfg4 worst rel err {worst}", flush=True)
    check_p16(dev.rows_b16(apm.APM_P16, sample), rows[apm.APM_P32], st.p16, used)
    streamer.destroy()
    host.destroy()
    dev.destroy()
    tmp.destroy()


def test_cfg4_gpt13b_full_shape_with_what_cannot_be_pinned_cached_in_hbm():
    # The full 40-layer 13 B shape (12 578 pages, 154 GB of fp32 state).  The box pins about 64 GiB,
    # so the host pool holds the tail of the model (as many pages as can be pinned) and the head's
    # fp32 state is cached in HBM (the paper's GPU cache of optimizer states, Sec. 4.2); the host
    # pool's page j is model page R + j.  Sampled pages of both parts are checked against the oracle.
    from gpu_helpers import HOST_THREADS
    E = 1 << 20
    specs = synth.gpt_tensor_list(40, 5120, 20480, 50257, 2048)
    plan = oracle.plan_pack([t.numel for t in specs], E)
    n_pages, n_t = plan.n_pages, len(specs)
    assert n_pages == 12578
    host = None
    for frac in (1.0, 0.45, 0.4, 0.3, 0.2, 0.1):
        n_host = int(n_pages * frac)
        try:
            host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_host, state_mask=apm.FP32_STATES)
            break
        except apm.ApmError as e:
            assert e.code == apm.APM_ENOMEM
            print(f"cfg4 full: {n_host} pages ({n_host * E * 12 / 2**30:.0f} GiB) cannot be pinned", flush=True)
    assert host is not None
    R = n_pages - n_host
    print(f"cfg4 full: {n_pages} pages, {n_host} in pinned host memory ({n_host * E * 12 / 2**30:.1f} GiB), "
          f"{R} cached in HBM", flush=True)
    model = Model(specs, E, seed=0)
    sample = sorted(set(range(0, n_pages, 257)) | {0, R - 1, R, n_pages - 1} - {-1}
                    | {k for k, p in enumerate(plan.pages) if p.used < E})
    sample = [p for p in sample if 0 <= p < n_pages]
    used = [plan.pages[p].used for p in sample]
    h = oracle.Hyper(max_grad_norm=1.0)
    hy = to_hyper(h)

    init = DevicePool(n_pages, E, states=(apm.APM_P32,))       # the cache's P32 class is its head
    apm.apm_pack_tensors(init.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    apm.apm_page_copy_async(host, 0, init.pool, R, n_host, apm.APM_P32)
    torch.cuda.synchronize()
    st = oracle.PagedAdamWState(model.host_pages(model.p_flat, sample).view(np.float32), used)
    model.p_flat = None                                         # 51 GB back to the allocator
    torch.cuda.empty_cache()
    cache_mv = {s_: torch.zeros((max(R, 1), E), dtype=torch.float32, device=DEV) for s_ in (apm.APM_M32, apm.APM_V32)}
    cache = apm.apm_pool_create(apm.APM_DEV_GPU, E, max(R, 1), state_mask=apm.FP32_STATES,
                                flags=apm.APM_POOL_NO_ZERO,      # P32 holds the packed parameters already
                                base={apm.APM_P32: init.reg[apm.APM_P32], **cache_mv})
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, apm.make_tensors(model.numels, apm.APM_BF16), n_t)
    streamer = apm.apm_streamer_create(host, dev.pool, 32, 3)
    apm.apm_streamer_set_cache(streamer, cache if R else None, R)
    apm.apm_streamer_set_host_first_page(streamer, R)
    norm_d = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 3):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_streamer_set_mode(streamer, apm.APM_STREAM_DIRECT if t == 1 else apm.APM_STREAM_STAGED)
        apm.apm_streamer_step(streamer, t, hy, norm_d, None)
        norms, _ = st.step(model.host_pages(g, sample), t, h, threads=HOST_THREADS)
        torch.cuda.synchronize()
        got = norm_d.cpu().numpy()[sample]
        assert np.all(np.abs(got - norms) <= 1e-6 * np.abs(norms))
        del g
    rows = {}
    cached = [p for p in sample if p < R]
    streamed = [p - R for p in sample if p >= R]
    idx = torch.as_tensor(cached, device=DEV, dtype=torch.long)
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        head = (init.reg[s_] if s_ == apm.APM_P32 else cache_mv[s_])[idx].cpu().numpy() if cached else np.zeros((0, E), np.float32)
        tail = host_view(host, s_, n_host, E)[streamed]
        rows[s_] = np.concatenate([head, tail], axis=0)
    worst = {k: check_state_close(k, rows[s_], ref, used)
             for k, s_, ref in (("p", apm.APM_P32, st.p), ("m", apm.APM_M32, st.m), ("v", apm.APM_V32, st.v))}
    print(f"cfg4 full worst rel err {worst}", flush=True)
    check_p16(dev.rows_b16(apm.APM_P16, sample), rows[apm.APM_P32], st.p16, used)
    streamer.destroy()
    cache.destroy()
    host.destroy()
    dev.destroy()
    init.destroy()


def test_cache_size_from_free_memory():
    E = 1 << 20
    free_b, total_b = torch.cuda.mem_get_info()
    n_all = apm.apm_cache_pages_that_fit(E, 10 ** 9)
    assert 0.9 * free_b / (12 * E) - 1 <= n_all <= total_b / (12 * E)
    assert apm.apm_cache_pages_that_fit(E, 100) == 100
    assert apm.apm_cache_pages_that_fit(E, 10 ** 9, reserve_bytes=total_b) == 0
    half = apm.apm_cache_pages_that_fit(E, 10 ** 9, reserve_bytes=free_b // 2)
    assert abs(half - n_all / 2) <= 0.1 * n_all + 2


def layer_ranges(model):
    """First page of every transformer block (plus the embedding / final blocks): a page belongs
    to the block of its first tenant.  Returns the n_layers + 1 boundaries."""
    first_tensor = {}
    for s in model.plan.segments:
        first_tensor.setdefault(s.page, s.tensor)
    bounds, prev = [0], None
    for page in range(model.plan.n_pages):
        blk = model.specs[first_tensor[page]].layer
        if prev is not None and blk != prev:
            bounds.append(page)
        prev = blk
    bounds.append(model.plan.n_pages)
    return bounds


@pytest.mark.parametrize("budget_layers,mover", [(1.0, "kernel"), (2.5, "kernel"), (100.0, "kernel"), (2.5, "dma")])
def test_scheduled_step_equals_resident_bit_exact(budget_layers, mover):
    # the page movement follows the life-time based schedule (Alg. 1 phase 1) planned for a GPU
    # memory of `budget_layers` times the largest layer; results must not depend on it
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=4)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    bounds = layer_ranges(model)
    assert len(bounds) - 1 >= 12
    largest = max(b - a for a, b in zip(bounds, bounds[1:]))
    slots = min(n_pages, int(budget_layers * largest))
    page_bytes = 12 * E
    layers = [(range(a, b), 0) for a, b in zip(bounds, bounds[1:])]
    tasks, peak = apm.apm_schedule_plan(layers, None, page_bytes, slots * page_bytes)
    assert peak <= slots * page_bytes
    moves_at_start = next(i for i, t in enumerate(tasks) if t[0] == apm.APM_TASK_COMPUTE)
    assert moves_at_start <= slots and (budget_layers < 50 or moves_at_start == n_pages)

    hy = to_hyper(oracle.Hyper(max_grad_norm=1.0))
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    apm.apm_page_copy_async(host, 0, res.pool, 0, n_pages, apm.APM_P32)
    st = apm.apm_streamer_create(host, dev.pool, (slots + 1) // 2, 2)   # staging: at least the planned slots
    if mover == "dma":          # pages moved by the runtime's copies instead of the library's copy kernel
        apm.apm_streamer_set_mode(st, apm.APM_STREAM_STAGED_DMA)
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_s = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, None)
        apm.apm_streamer_step_scheduled(st, tasks, bounds, t, hy, norm_s, None)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s)
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        hv = host_view(host, s_, n_pages, E)
        assert np.array_equal(hv.view(np.uint32), res.reg[s_].cpu().numpy().view(np.uint32)), f"state {s_}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))

    # unsound schedules are refused before anything runs
    with pytest.raises(apm.ApmError) as e:      # a layer computes before its last page arrived
        bad = [t for t in tasks if not (t[0] == apm.APM_TASK_MOVE_TO_GPU and t[1] == bounds[1] - 1)]
        apm.apm_streamer_step_scheduled(st, bad, bounds, 4, hy)
    assert e.value.code == apm.APM_ESTATE
    with pytest.raises(apm.ApmError) as e:      # everything moved up front into too few slots
        if budget_layers > 50:
            raise apm.ApmError(apm.APM_ENOMEM, "n/a: every page has a slot")
        greedy = [(apm.APM_TASK_MOVE_TO_GPU, p, 0) for p in range(n_pages)] + [(apm.APM_TASK_COMPUTE, i, i) for i in range(len(bounds) - 1)]
        apm.apm_streamer_step_scheduled(st, greedy, bounds, 4, hy)
    assert e.value.code == apm.APM_ENOMEM
    st.destroy()
    host.destroy()
    dev.destroy()
    res.destroy()


@pytest.mark.parametrize("E", [8, 520, 1024, 2048, 5120])
@pytest.mark.parametrize("waves", [3, 200])
def test_copy_kernel_movers_on_small_and_odd_page_sizes(E, waves):
    # The copy kernel works on 4 KiB items: pages that are not a whole number of items (8 and 520
    # elements: it then moves whole runs without the page table), pages of exactly one item, of
    # two, and of five; fewer wavefronts than items per page and more wavefronts than items in a
    # run; tensors that leave pages full, nearly empty (a tiny tensor alone) and ending mid-item.
    # The ring and the schedule-driven step alternate on one host pool; both must match the
    # resident update bit for bit, unused tails included.
    numels = [3 * E + 8, 8, E, 2 * E - 8, 16, E // 2, 5 * E + 24, 8, 8, 4 * E, 24, max(8, E - 8)]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=9)
    n_pages, n_t = model.plan.n_pages, len(specs)
    hy = to_hyper(oracle.Hyper(max_grad_norm=1.0))
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    apm.apm_page_copy_async(host, 0, res.pool, 0, n_pages, apm.APM_P32)
    st = apm.apm_streamer_create(host, dev.pool, 5, 3)
    set_mode(st, f"staged:{waves}" + ("+wt" if waves == 200 else ""))
    per = 4
    bounds = list(range(0, n_pages, per)) + [n_pages]
    bounds = sorted(bounds + [bounds[1], bounds[3], n_pages])       # three layers without pages, one of them last
    layers = [(range(a, b), 0) for a, b in zip(bounds, bounds[1:])]
    tasks, _ = apm.apm_schedule_plan(layers, None, 12 * E, 11 * 12 * E)     # 11 of the 15 slots
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_s = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 5):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, None)
        if t % 2:
            apm.apm_streamer_step(st, t, hy, norm_s, None)
        else:
            apm.apm_streamer_step_scheduled(st, tasks, bounds, t, hy, norm_s, None)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s), f"step {t}"
        for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
            hv = host_view(host, s_, n_pages, E)
            assert np.array_equal(hv.view(np.uint32), res.reg[s_].cpu().numpy().view(np.uint32)), f"step {t} state {s_}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    st.destroy()
    host.destroy()
    dev.destroy()
    res.destroy()


def test_scheduled_step_with_a_trace_that_keeps_pages_beyond_their_own_layer():
    # Alg. 1's input is the trace: the layer after which a page's GPU memory is free again.  Here
    # the first page of every layer but the last is accessed again by the layer two further on (and
    # one page by the last layer), so the planner must keep those pages resident and defer others;
    # the executor holds their slots until that later layer has computed, honours the trigger ids,
    # and the result must still equal the resident update bit for bit.
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=14)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    bounds = layer_ranges(model)
    n_layers = len(bounds) - 1
    own = [i for i in range(n_layers) for _ in range(bounds[i], bounds[i + 1])]
    last_access = list(own)
    for i in range(n_layers - 1):
        last_access[bounds[i]] = min(i + 2, n_layers - 1)
    last_access[bounds[1] + 1] = n_layers - 1
    largest = max(b - a for a, b in zip(bounds, bounds[1:]))
    slots = 2 * largest + 6
    page_bytes = 12 * E
    layers = [(range(a, b), 0) for a, b in zip(bounds, bounds[1:])]
    tasks, peak = apm.apm_schedule_plan(layers, last_access, page_bytes, slots * page_bytes)
    assert peak <= slots * page_bytes
    plain, _ = apm.apm_schedule_plan(layers, None, page_bytes, slots * page_bytes)
    assert tasks != plain                                        # the trace changed the schedule
    assert any(t[0] == apm.APM_TASK_MOVE_TO_GPU and t[2] > 0 for t in tasks)   # some movements are triggered later

    hy = to_hyper(oracle.Hyper(max_grad_norm=1.0))
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    apm.apm_page_copy_async(host, 0, res.pool, 0, n_pages, apm.APM_P32)
    st = apm.apm_streamer_create(host, dev.pool, (slots + 1) // 2, 2)
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_s = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, None)
        apm.apm_streamer_step_scheduled(st, tasks, bounds, t, hy, norm_s, None, last_access=last_access)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s)
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        hv = host_view(host, s_, n_pages, E)
        assert np.array_equal(hv.view(np.uint32), res.reg[s_].cpu().numpy().view(np.uint32)), f"state {s_}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))

    def code(fn):
        with pytest.raises(apm.ApmError) as e:
            fn()
        return e.value.code
    # the schedule planned without the trace frees slots too early for it: refused, nothing runs
    assert code(lambda: apm.apm_streamer_step_scheduled(st, plain, bounds, 4, hy, last_access=last_access)) == apm.APM_ENOMEM
    # a movement triggered by a layer that computes after it in the list could never be issued
    k = next(i for i, t in enumerate(tasks) if t[0] == apm.APM_TASK_MOVE_TO_GPU)
    late = list(tasks)
    late[k] = (late[k][0], late[k][1], 1)
    assert code(lambda: apm.apm_streamer_step_scheduled(st, late, bounds, 4, hy, last_access=last_access)) == apm.APM_EINVAL
    early = list(last_access)
    early[bounds[3]] = 2                                         # before the page's own layer
    assert code(lambda: apm.apm_streamer_step_scheduled(st, tasks, bounds, 4, hy, last_access=early)) == apm.APM_EINVAL
    torch.cuda.synchronize()
    st.destroy()
    host.destroy()
    dev.destroy()
    res.destroy()


@pytest.mark.parametrize("mode", ["direct", "staged"])
def test_streamer_delayed_calls_plus_flush_equal_synchronous_steps(mode):
    # Alg. 2 with the fp32 state in host memory: N one-step-stale calls + flush must leave exactly
    # the state of N synchronous streamed steps, and the applied counter must run one behind
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=6)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    # a learning-rate schedule: gradient t must meet lr_t although call t+1 enqueues its update
    hys = [to_hyper(oracle.Hyper(max_grad_norm=1.0, lr=1e-4 * t, weight_decay=0.01 * (t % 2))) for t in range(6)]
    hy = hys[0]
    init = DevicePool(n_pages, E, states=(apm.APM_P32,))
    apm.apm_pack_tensors(init.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    sides = []
    for _ in range(2):
        dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
        apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
        host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
        apm.apm_page_copy_async(host, 0, init.pool, 0, n_pages, apm.APM_P32)
        st = apm.apm_streamer_create(host, dev.pool, 16, 3)
        set_mode(st, mode)
        sides.append((dev, host, st))
    (dev_a, host_a, st_a), (dev_b, host_b, st_b) = sides
    produce = DevicePool(n_pages, E, states=(apm.APM_G16,))       # the producer's own gradient pages
    apm.apm_pool_set_layout(produce.pool, model.tensors(model.p_flat), n_t)
    norm_a = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_b = torch.full((n_pages,), -1.0, dtype=torch.float32, device=DEV)
    apm.apm_delayed_set_outputs(dev_b.pool, norm_b, None)
    steps = 4
    for t in range(1, steps + 1):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(dev_a.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_streamer_step(st_a, t, hys[t], norm_a, None)
        apm.apm_pack_tensors(produce.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_streamer_step_delayed(st_b, produce.reg[apm.APM_G16], hys[t])
        assert apm.apm_delayed_applied(dev_b.pool) == t - 1
        torch.cuda.synchronize()
    apm.apm_streamer_step_delayed(st_b, None, hy)
    torch.cuda.synchronize()
    assert apm.apm_delayed_applied(dev_b.pool) == steps
    assert torch.equal(norm_a, norm_b)
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        a = host_view(host_a, s_, n_pages, E).view(np.uint32)
        b = host_view(host_b, s_, n_pages, E).view(np.uint32)
        assert np.array_equal(a, b), f"state {s_}"
    assert torch.equal(dev_a.reg[apm.APM_P16].view(torch.int16), dev_b.reg[apm.APM_P16].view(torch.int16))
    assert not dev_b.reg[apm.APM_G16].view(torch.int16).any()     # the pool's own G16 class was never used
    for dev, host, st in sides:
        st.destroy()
        host.destroy()
        dev.destroy()
    produce.destroy()
    init.destroy()


def needs_unbuffered_io(tmp_path):
    """Skips when the directory's file system refuses O_DIRECT (a memory file system does)."""
    probe = str(tmp_path / "o_direct_probe")
    try:
        os.close(os.open(probe, os.O_RDWR | os.O_CREAT | os.O_DIRECT, 0o600))
    except OSError as e:
        pytest.skip(f"no unbuffered I/O in {tmp_path}: {e}")
    os.remove(probe)


def file_rows(prefix, suffix, n_pages, E):
    return np.fromfile(prefix + suffix, dtype=np.uint32).reshape(n_pages, E)


@pytest.mark.parametrize("batch,slots,threads,flags", [(5, 2, 3, 0), (16, 3, 8, "direct"), (300, 2, 4, 0)])
def test_file_tier_step_equals_resident_bit_exact(tmp_path, batch, slots, threads, flags):
    # fp32 state in files, a pinned window as the only staging; results must equal the resident path
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=8)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    hy = to_hyper(oracle.Hyper(max_grad_norm=1.0))
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    prefix = str(tmp_path / "state")
    fl = apm.APM_POOL_FILE_DIRECT if flags == "direct" else 0
    if fl:
        needs_unbuffered_io(tmp_path)
    filep = apm.apm_file_pool_create(prefix, E, n_pages, flags=fl)
    # initial master parameters reach the files through a host pool
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=1 << apm.APM_P32)
    apm.apm_page_copy_async(host, 0, res.pool, 0, n_pages, apm.APM_P32)
    apm.apm_page_copy_async(filep, 0, host, 0, n_pages, apm.APM_P32)
    tier = apm.apm_tiered_create(filep, dev.pool, min(batch, n_pages), slots, threads)
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_s = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, None)
        apm.apm_tiered_step(tier, t, hy, norm_s, None)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s)
    tier.destroy()
    filep.destroy()
    for s_, suffix in ((apm.APM_P32, ".p32"), (apm.APM_M32, ".m32"), (apm.APM_V32, ".v32")):
        want = res.reg[s_].cpu().numpy().view(np.uint32)
        assert np.array_equal(file_rows(prefix, suffix, n_pages, E), want), f"state {s_}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    # the read-back path: file -> host pool
    filep = apm.apm_file_pool_create(prefix, E, n_pages, flags=apm.APM_POOL_NO_ZERO)
    apm.apm_page_copy_async(host, 3, filep, 3, n_pages - 3, apm.APM_P32)
    assert np.array_equal(host_view(host, apm.APM_P32, n_pages, E)[3:].view(np.uint32),
                          res.reg[apm.APM_P32][3:].cpu().numpy().view(np.uint32))
    filep.destroy()
    host.destroy()
    dev.destroy()
    res.destroy()


@pytest.mark.parametrize("with_mask,stale", [(True, False), (False, False), (False, True)])
def test_file_tier_moves_only_the_pages_that_received_a_gradient(tmp_path, with_mask, stale):
    # MoE-like: per step a few "experts" have a gradient; with APM_SKIP_UNTOUCHED the other pages are
    # neither read nor written, and the files still end bit-identical to the resident update
    E = 16384
    specs = [synth.TensorSpec(0, "dense", 2 * E + 100)]
    for x in range(10):
        specs += [synth.TensorSpec(1 + 2 * x, f"w1_{x}", 3 * E), synth.TensorSpec(2 + 2 * x, f"b_{x}", 64)]
    rng = np.random.default_rng(5)
    draws = {t: rng.permutation(10)[:3] for t in range(1, 6)}

    def active(step):
        a = np.zeros(len(specs), dtype=bool)
        a[0] = True
        for x in draws[step]:
            a[1 + 2 * x] = a[2 + 2 * x] = True
        return a

    model = Model(specs, E, seed=12, active_fn=active)
    n_pages, n_t = model.plan.n_pages, len(specs)
    hy = to_hyper(oracle.Hyper(max_grad_norm=0.05, skip_mode=1))
    res = DevicePool(n_pages, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    prefix = str(tmp_path / "state")
    filep = apm.apm_file_pool_create(prefix, E, n_pages)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=1 << apm.APM_P32)
    apm.apm_page_copy_async(host, 0, res.pool, 0, n_pages, apm.APM_P32)
    apm.apm_page_copy_async(filep, 0, host, 0, n_pages, apm.APM_P32)
    tier = apm.apm_tiered_create(filep, dev.pool, 4, 3, 4)
    norm_r = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    skip_r = torch.zeros(n_pages, dtype=torch.uint8, device=DEV)
    norm_s = torch.full((n_pages,), -1.0, dtype=torch.float32, device=DEV)
    skip_s = torch.full((n_pages,), 9, dtype=torch.uint8, device=DEV) if with_mask else None
    produce = DevicePool(n_pages, E, states=(apm.APM_G16,))
    apm.apm_pool_set_layout(produce.pool, model.tensors(model.p_flat), n_t)
    if stale:
        apm.apm_delayed_set_outputs(dev.pool, norm_s, skip_s)
    moved_pages = 0
    for t in range(1, 6):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, n_pages, t, hy, norm_r, skip_r)
        if stale:
            apm.apm_pack_tensors(produce.pool, apm.APM_G16, model.tensors(g), n_t)
            apm.apm_tiered_step_delayed(tier, produce.reg[apm.APM_G16], hy)
        else:
            apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
            apm.apm_tiered_step(tier, t, hy, norm_s, skip_s)
        torch.cuda.synchronize()
        n_active = int((skip_r == 0).sum())
        assert 0 < n_active < n_pages
        moved_pages += n_active
        if not stale:
            assert torch.equal(norm_r, norm_s)
            if with_mask:
                assert torch.equal(skip_r, skip_s)
    if stale:
        apm.apm_tiered_step_delayed(tier, None, hy)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s)
    rd, wr = apm.apm_tiered_io_bytes(tier)
    assert rd == wr == moved_pages * 12 * E, (rd, wr, moved_pages)
    tier.destroy()
    filep.destroy()
    for s_, suffix in ((apm.APM_P32, ".p32"), (apm.APM_M32, ".m32"), (apm.APM_V32, ".v32")):
        assert np.array_equal(file_rows(prefix, suffix, n_pages, E), res.reg[s_].cpu().numpy().view(np.uint32)), suffix
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    for x in (produce, host, dev, res):
        x.destroy()


def test_file_tier_delayed_calls_plus_flush_equal_synchronous_steps(tmp_path):
    # Alg. 2 with its two actors as host threads: the updater thread works through the files while
    # the caller hands over the next gradient
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    model = Model(f(), E, seed=9)
    n_pages, n_t = model.plan.n_pages, len(model.specs)
    hys = [to_hyper(oracle.Hyper(max_grad_norm=1.0, lr=1e-4 * t, weight_decay=0.01 * (t % 2))) for t in range(6)]
    hy = hys[0]
    init = DevicePool(n_pages, E, states=(apm.APM_P32,))
    apm.apm_pack_tensors(init.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=1 << apm.APM_P32)
    apm.apm_page_copy_async(host, 0, init.pool, 0, n_pages, apm.APM_P32)
    sides = []
    for name in ("sync", "stale"):
        dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
        apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
        prefix = str(tmp_path / name)
        filep = apm.apm_file_pool_create(prefix, E, n_pages)
        apm.apm_page_copy_async(filep, 0, host, 0, n_pages, apm.APM_P32)
        sides.append((dev, filep, apm.apm_tiered_create(filep, dev.pool, 16, 3, 6), prefix))
    (dev_a, file_a, tier_a, pre_a), (dev_b, file_b, tier_b, pre_b) = sides
    produce = DevicePool(n_pages, E, states=(apm.APM_G16,))
    apm.apm_pool_set_layout(produce.pool, model.tensors(model.p_flat), n_t)
    norm_a = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    norm_b = torch.full((n_pages,), -1.0, dtype=torch.float32, device=DEV)
    apm.apm_delayed_set_outputs(dev_b.pool, norm_b, None)
    steps = 4
    for t in range(1, steps + 1):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(dev_a.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_tiered_step(tier_a, t, hys[t], norm_a, None)
        apm.apm_pack_tensors(produce.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_tiered_step_delayed(tier_b, produce.reg[apm.APM_G16], hys[t])
        assert apm.apm_delayed_applied(dev_b.pool) == t - 1
    with pytest.raises(apm.ApmError) as e:          # the ping-pong halves are not handed out here
        apm.apm_tiered_step_delayed(tier_b, apm.apm_delayed_grad_buffer(dev_b.pool), hy)
    assert e.value.code == apm.APM_EINVAL
    apm.apm_tiered_step_delayed(tier_b, None, hy)
    torch.cuda.synchronize()
    assert apm.apm_delayed_applied(dev_b.pool) == steps
    assert torch.equal(norm_a, norm_b)
    for dev, filep, tier, prefix in sides:
        tier.destroy()
        filep.destroy()
    for suffix in (".p32", ".m32", ".v32"):
        assert np.array_equal(file_rows(pre_a, suffix, n_pages, E), file_rows(pre_b, suffix, n_pages, E)), suffix
    assert torch.equal(dev_a.reg[apm.APM_P16].view(torch.int16), dev_b.reg[apm.APM_P16].view(torch.int16))
    for dev, *_ in sides:
        dev.destroy()
    produce.destroy()
    host.destroy()
    init.destroy()


def test_file_tier_reports_a_failed_read_and_drains(tmp_path):
    # a state file cut short behind the pool's back: reads beyond its end fail; the step must
    # come back with an error (no hang, every queued batch accounted for) and work again afterwards
    E = 4096
    specs = [synth.TensorSpec(0, "a", 40 * E)]
    model = Model(specs, E, seed=1)
    n_pages = model.plan.n_pages
    dev = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), 1)
    prefix = str(tmp_path / "cut")
    filep = apm.apm_file_pool_create(prefix, E, n_pages)
    tier = apm.apm_tiered_create(filep, dev.pool, 4, 2, 3)
    hy = to_hyper(oracle.Hyper())
    apm.apm_tiered_step(tier, 1, hy)
    os.truncate(prefix + ".m32", 10 * E * 4)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_tiered_step(tier, 2, hy)
    assert e.value.code == apm.APM_EDEVICE and "I/O" in str(e.value)
    with pytest.raises(apm.ApmError) as e:          # the background form reports it on the next call
        apm.apm_tiered_step_delayed(tier, dev.reg[apm.APM_G16], hy)
        apm.apm_tiered_step_delayed(tier, dev.reg[apm.APM_G16], hy)
        apm.apm_tiered_step_delayed(tier, None, hy)
    assert e.value.code == apm.APM_EDEVICE
    os.truncate(prefix + ".m32", n_pages * E * 4)
    apm.apm_tiered_step(tier, 3, hy)
    torch.cuda.synchronize()
    tier.destroy()
    filep.destroy()
    dev.destroy()


def test_streamer_and_tier_argument_errors(tmp_path):
    E, n = 4096, 6
    dev = DevicePool(n, E, states=(apm.APM_G16, apm.APM_P16))
    x = torch.zeros(n * E, dtype=torch.bfloat16, device=DEV)
    apm.apm_pool_set_layout(dev.pool, apm.make_tensors([n * E], apm.APM_BF16, [x]), 1)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n, state_mask=apm.FP32_STATES)
    hy = to_hyper(oracle.Hyper())

    def code(fn):
        with pytest.raises(apm.ApmError) as e:
            fn()
        return e.value.code

    assert code(lambda: apm.apm_streamer_create(host, dev.pool, 0, 2)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_create(host, dev.pool, 2, 1)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_create(dev.pool, dev.pool, 2, 2)) == apm.APM_EDEVICE
    st = apm.apm_streamer_create(host, dev.pool, 2, 2)
    assert apm.apm_streamer_get_mode(st) == apm.APM_STREAM_DIRECT
    assert apm.apm_streamer_probe_rates(st) == (0.0, 0.0, 0.0)            # staged set-up has not run
    assert code(lambda: apm.apm_streamer_copy_only(st, 3)) == apm.APM_ESTATE   # a staged-mode measurement
    assert code(lambda: apm.apm_streamer_set_mode(st, 7)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_set_mode(st, apm.APM_STREAM_DIRECT, -1)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_set_mode(st, apm.APM_STREAM_DIRECT, 8, 17)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_set_host_first_page(st, n + 1)) == apm.APM_ERANGE
    apm.apm_streamer_set_host_first_page(st, 2)
    assert code(lambda: apm.apm_streamer_step(st, 1, hy)) == apm.APM_ESTATE     # pages 0, 1 are nowhere
    apm.apm_streamer_set_host_first_page(st, 0)
    assert code(lambda: apm.apm_streamer_step(st, 0, hy)) == apm.APM_EINVAL     # step numbers start at 1
    apm.apm_streamer_step(st, 1, hy)
    assert code(lambda: apm.apm_streamer_step_scheduled(st, [(apm.APM_TASK_COMPUTE, 0, 0)], [0, n], 2, hy)) == apm.APM_ESTATE
    assert code(lambda: apm.apm_streamer_step_scheduled(st, [(9, 0, 0)], [0, n], 2, hy)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_step_scheduled(st, [], [0, n - 1], 2, hy)) == apm.APM_EINVAL
    apm.apm_streamer_set_page_count(st, 3)                    # a page range: not with a schedule
    tasks = [(apm.APM_TASK_MOVE_TO_GPU, 0, p) for p in range(n)] + [(apm.APM_TASK_COMPUTE, 0, 0)]
    assert code(lambda: apm.apm_streamer_step_scheduled(st, tasks, [0, n], 2, hy)) == apm.APM_ESTATE
    apm.apm_streamer_step(st, 2, hy)                          # pages [0, 3) only
    apm.apm_streamer_set_page_count(st, -1)
    torch.cuda.synchronize()
    st.destroy()

    filep = apm.apm_file_pool_create(str(tmp_path / "s"), E, n)
    assert code(lambda: apm.apm_tiered_create(host, dev.pool, 2, 2, 2)) == apm.APM_EDEVICE   # not a FILE pool
    assert code(lambda: apm.apm_tiered_create(filep, dev.pool, 2, 1, 2)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_tiered_create(filep, dev.pool, 2, 2, 0)) == apm.APM_EINVAL
    assert code(lambda: apm.apm_streamer_create(filep, dev.pool, 2, 2)) == apm.APM_EDEVICE
    assert code(lambda: apm.apm_page_copy_async(filep, 0, dev.pool, 0, 1, apm.APM_P16)) in (apm.APM_ERANGE, apm.APM_EDEVICE)
    tier = apm.apm_tiered_create(filep, dev.pool, 4, 2, 2)
    assert code(lambda: apm.apm_tiered_step(tier, 0, hy)) == apm.APM_EINVAL
    apm.apm_tiered_step(tier, 1, hy)
    assert code(lambda: apm.apm_tiered_set_range(tier, -1)) == apm.APM_ERANGE
    assert code(lambda: apm.apm_tiered_set_range(tier, n + 1)) == apm.APM_ERANGE
    rd0, wr0 = apm.apm_tiered_io_bytes(tier)
    apm.apm_tiered_set_range(tier, n)                         # an empty range: a step that moves nothing
    apm.apm_tiered_step(tier, 2, hy)
    assert apm.apm_tiered_io_bytes(tier) == (rd0, wr0) == (n * 12 * E, n * 12 * E)
    apm.apm_tiered_set_range(tier, 2, 3)
    apm.apm_tiered_step(tier, 2, hy)
    assert apm.apm_tiered_io_bytes(tier) == ((n + 3) * 12 * E, (n + 3) * 12 * E)
    tier.destroy()
    filep.destroy()
    host.destroy()
    dev.destroy()


@pytest.mark.parametrize("form", ["resident", "fused", "delayed", "direct", "staged"])
def test_calls_on_a_side_stream_are_ordered_by_that_stream(form):
    # Everything (input generation, pack, steps, unpack) is enqueued on one non-default stream with
    # no synchronisation in between: a call that put part of its work on another stream, or joined
    # the caller's stream too early, would read gradients that are still being generated.
    E = 65536
    specs = [synth.TensorSpec(0, "a", 40 * E + 12), synth.TensorSpec(1, "b", 300), synth.TensorSpec(2, "c", 23 * E),
             synth.TensorSpec(3, "d", 7), synth.TensorSpec(4, "e", 9 * E + 1000)]
    model = Model(specs, E, seed=31, align_elems=8)
    n_pages, n_t = model.plan.n_pages, len(specs)
    hy = to_hyper(oracle.Hyper(max_grad_norm=0.05))
    steps = 3

    def run(side):
        s = torch.cuda.Stream() if side else torch.cuda.current_stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            streamed = form in ("direct", "staged")
            dp = DevicePool(n_pages, E, states=(apm.APM_G16, apm.APM_P16) if streamed else (0, 1, 2, 3, 4))
            torch.cuda.synchronize()
            host = st = None
            if streamed:
                tmp = DevicePool(n_pages, E, states=(apm.APM_P32,))
                torch.cuda.synchronize()
                apm.apm_pack_tensors(tmp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t, stream=s)
                apm.apm_pool_set_layout(dp.pool, model.tensors(model.p_flat), n_t, stream=s)
                host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n_pages, state_mask=apm.FP32_STATES)
                apm.apm_page_copy_async(host, 0, tmp.pool, 0, n_pages, apm.APM_P32, stream=s)
                st = apm.apm_streamer_create(host, dp.pool, 8, 3)
                set_mode(st, form)
            else:
                apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t, stream=s)
            norm = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
            q_flat = torch.zeros(model.total, dtype=torch.bfloat16, device=DEV)
            keep = []
            for t in range(1, steps + 1):
                if side and hasattr(torch.cuda, "_sleep"):
                    torch.cuda._sleep(50_000_000)            # a bounded spin (tens of ms) ahead of the inputs
                g = model.grad_flat(t)                       # many kernels on s
                keep.append(g)
                if form == "fused":
                    apm.apm_page_adamw_step_fused(dp.pool, None, n_pages, t, hy, model.tensors(g),
                                                  model.tensors(q_flat), n_t, norm, None, stream=s)
                    continue
                apm.apm_pack_tensors(dp.pool, apm.APM_G16, model.tensors(g), n_t, stream=s)
                if form == "resident":
                    apm.apm_page_adamw_step(dp.pool, list(reversed(range(n_pages))), n_pages, t, hy, norm, None, stream=s)
                elif form == "delayed":
                    apm.apm_step_delayed(dp.pool, None, n_pages, dp.reg[apm.APM_G16], hy, stream=s)
                else:
                    apm.apm_streamer_step(st, t, hy, norm, None, stream=s)
            if form == "delayed":
                apm.apm_step_delayed(dp.pool, None, n_pages, None, hy, stream=s)
            if form != "fused":
                apm.apm_unpack(dp.pool, apm.APM_P16, model.tensors(q_flat), n_t, stream=s)
            s.synchronize()
            torch.cuda.synchronize()
            if streamed:
                out = [host_view(host, c, n_pages, E).view(np.uint32).copy() for c in (apm.APM_P32, apm.APM_M32, apm.APM_V32)]
                st.destroy()
                host.destroy()
                tmp.destroy()
            else:
                out = [dp.reg[c].cpu().numpy().view(np.uint32) for c in (apm.APM_P32, apm.APM_M32, apm.APM_V32)]
            out.append(bf16_bits(q_flat))
            if form != "delayed":
                out.append(norm.cpu().numpy().view(np.uint32))
            dp.destroy()
        return out

    want = run(False)
    got = run(True)
    for k, (a, b) in enumerate(zip(want, got)):
        assert np.array_equal(a, b), f"output {k} differs between the default stream and a side stream"
    assert want[0].any() and want[3].any()


@pytest.mark.parametrize("where", ["host", "file"])
def test_accumulated_gradients_with_the_state_off_the_gpu(tmp_path, where):
    # Alg. 2 in full: the buffering side sums several micro-gradients while the updating side works
    # on states that live in pinned host memory or in files; equal to synchronous resident steps
    # on the pre-summed gradients (bf16 sums: fp32 add, nearest even)
    E = 16384
    numels = [3 * E + 5, 100, 2 * E, 9000, E, 5 * E + 77]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=13, sigma_g=5e-3)
    n, n_t = model.plan.n_pages, len(specs)
    hy = to_hyper(oracle.Hyper(max_grad_norm=0.5))
    res = DevicePool(n, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(n, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, n, state_mask=apm.FP32_STATES)
    apm.apm_page_copy_async(host, 0, res.pool, 0, n, apm.APM_P32)
    torch.cuda.synchronize()
    filep = tier = st = None
    if where == "file":
        prefix = str(tmp_path / "state")
        filep = apm.apm_file_pool_create(prefix, E, n)
        apm.apm_page_copy_async(filep, 0, host, 0, n, apm.APM_P32)
        tier = apm.apm_tiered_create(filep, dev.pool, 3, 2, 3)
        hand_over = lambda g: apm.apm_tiered_step_delayed(tier, g, hy)
    else:
        st = apm.apm_streamer_create(host, dev.pool, 4, 2)
        hand_over = lambda g: apm.apm_streamer_step_delayed(st, g, hy)
    stage = DevicePool(n, E, states=(apm.APM_G16,))
    apm.apm_pool_set_layout(stage.pool, model.tensors(model.p_flat), n_t)
    for t in range(1, 4):
        gs = [model.grad_flat(10 * t + k) for k in range(3)]
        total = (gs[0] + gs[1]) + gs[2]
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(total), n_t)
        apm.apm_page_adamw_step(res.pool, None, n, t, hy)
        apm.apm_pack_tensors(stage.pool, apm.APM_G16, model.tensors(gs[0]), n_t)
        hand_over(stage.reg[apm.APM_G16])
        for k in (1, 2):
            apm.apm_pack_tensors(stage.pool, apm.APM_G16, model.tensors(gs[k]), n_t)
            apm.apm_delayed_accumulate(dev.pool, None, n, stage.reg[apm.APM_G16])
        torch.cuda.synchronize()
    hand_over(None)
    torch.cuda.synchronize()
    assert apm.apm_delayed_applied(dev.pool) == 3
    if where == "file":
        tier.destroy()
        filep.destroy()
        got = [file_rows(prefix, suffix, n, E) for suffix in (".p32", ".m32", ".v32")]
    else:
        st.destroy()
        got = [host_view(host, c, n, E).view(np.uint32) for c in (apm.APM_P32, apm.APM_M32, apm.APM_V32)]
    for c, g in zip((apm.APM_P32, apm.APM_M32, apm.APM_V32), got):
        assert np.array_equal(g, res.reg[c].cpu().numpy().view(np.uint32)), f"state {c}"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    for x in (stage, host, dev, res):
        x.destroy()


@pytest.mark.parametrize("mode,skip", [("direct", 0), ("staged", 0), ("direct", 1)])
def test_three_levels_hbm_cache_host_memory_and_files_in_one_step(tmp_path, mode, skip):
    # the leading pages' fp32 state cached in HBM, the next in pinned host memory, the rest in
    # files: a streamer step over [0, H) and a tier step over [H, N) on the same GPU pool
    f, E = synth.WORKLOADS["gpt2_small_124m"]
    specs = f()
    zero = {i for i, t in enumerate(specs) if skip and i % 3 == 1}
    model = Model(specs, E, seed=14, active_fn=(lambda t: np.array([i not in zero for i in range(len(specs))])) if skip else None)
    N, n_t = model.plan.n_pages, len(specs)
    R, H = N // 4, (2 * N) // 3
    hy = to_hyper(oracle.Hyper(max_grad_norm=1.0, skip_mode=skip))
    res = DevicePool(N, E)
    apm.apm_pack_tensors(res.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    dev = DevicePool(N, E, states=(apm.APM_G16, apm.APM_P16))
    apm.apm_pool_set_layout(dev.pool, model.tensors(model.p_flat), n_t)
    cache = DevicePool(R, E, states=(apm.APM_P32, apm.APM_M32, apm.APM_V32))
    apm.apm_page_copy_async(cache.pool, 0, res.pool, 0, R, apm.APM_P32)
    host = apm.apm_pool_create(apm.APM_DEV_HOST, E, H - R, state_mask=apm.FP32_STATES)     # model pages [R, H)
    apm.apm_page_copy_async(host, 0, res.pool, R, H - R, apm.APM_P32)
    bounce = apm.apm_pool_create(apm.APM_DEV_HOST, E, N - H, state_mask=1 << apm.APM_P32)
    apm.apm_page_copy_async(bounce, 0, res.pool, H, N - H, apm.APM_P32)
    prefix = str(tmp_path / "state")
    filep = apm.apm_file_pool_create(prefix, E, N)                                       # file page = model page
    apm.apm_page_copy_async(filep, H, bounce, 0, N - H, apm.APM_P32)
    st = apm.apm_streamer_create(host, dev.pool, 16, 3)
    set_mode(st, mode)
    apm.apm_streamer_set_cache(st, cache.pool, R)
    apm.apm_streamer_set_host_first_page(st, R)
    apm.apm_streamer_set_page_count(st, H)
    tier = apm.apm_tiered_create(filep, dev.pool, 8, 3, 4)
    apm.apm_tiered_set_range(tier, H)
    norm_r = torch.zeros(N, dtype=torch.float32, device=DEV)
    skip_r = torch.zeros(N, dtype=torch.uint8, device=DEV)
    norm_s = torch.full((N,), -1.0, dtype=torch.float32, device=DEV)
    skip_s = torch.full((N,), 9, dtype=torch.uint8, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(res.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(dev.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(res.pool, None, N, t, hy, norm_r, skip_r)
        apm.apm_streamer_step(st, t, hy, norm_s, skip_s)
        apm.apm_tiered_step(tier, t, hy, norm_s, skip_s)
        torch.cuda.synchronize()
        assert torch.equal(norm_r, norm_s) and torch.equal(skip_r, skip_s)
    if skip:
        assert 0 < int(skip_r[H:].sum()) < N - H
        rd, wr = apm.apm_tiered_io_bytes(tier)
        assert rd == wr == 3 * int((skip_r[H:] == 0).sum()) * 12 * E
    tier.destroy()
    filep.destroy()
    st.destroy()
    for c, suffix in ((apm.APM_P32, ".p32"), (apm.APM_M32, ".m32"), (apm.APM_V32, ".v32")):
        want = res.reg[c].cpu().numpy().view(np.uint32)
        assert np.array_equal(cache.reg[c].cpu().numpy().view(np.uint32), want[:R]), f"cache {c}"
        assert np.array_equal(host_view(host, c, H - R, E).view(np.uint32), want[R:H]), f"host {c}"
        assert np.array_equal(file_rows(prefix, suffix, N, E)[H:], want[H:]), f"file {c}"
        assert not file_rows(prefix, suffix, N, E)[:H].any(), "file pages below the range were written"
    assert torch.equal(dev.reg[apm.APM_P16].view(torch.int16), res.reg[apm.APM_P16].view(torch.int16))
    for x in (bounce, host, cache, dev, res):
        x.destroy()
