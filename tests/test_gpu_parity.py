"""Parity of the HIP path (through the C ABI) against the oracle on the five configurations and on
edge cases.  Floating-point gate: |gpu - oracle| <= max(1e-6 |oracle|, 1e-9) for p32, m32, v32
after the last step; packing, masks, p16-vs-own-master and copies are bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2303_02868_amd as apm
    from gpu_helpers import (DEV, HOST_THREADS, DevicePool, Model, bf16_bits, check_p16,
                             check_state_close, run_resident, to_hyper, unpack_all)


def specs_of(name):
    f, E = synth.WORKLOADS[name]
    return f(), E


def log(msg):
    print(msg, flush=True)


def test_synth_device_backend_matches_host():
    a = synth.normal_f32(0, 1, 123456789, 1 << 16, 0.02)
    b = synth.normal_f32(0, 1, 123456789, 1 << 16, 0.02, device=DEV).cpu().numpy()
    assert a.tobytes() == b.tobytes()
    g = synth.normal_bf16(0, 1001, 5, 1 << 16, 1e-3)
    assert g.tobytes() == bf16_bits(synth.normal_bf16(0, 1001, 5, 1 << 16, 1e-3, device=DEV)).tobytes()


def test_cfg1_eight_pages_one_step_and_closed_form():
    specs, E = specs_of("cfg1_8pages")
    model = Model(specs, E, seed=0)
    h = oracle.Hyper()
    dp, st, worst = run_resident(model, 1, h)
    log(f"cfg1 worst rel err {worst}")
    # first-step closed form, element by element: p' = p - lr g/(|g|+eps) - lr wd p
    p0 = model.p_flat.cpu().numpy().astype(np.float64)
    g = oracle.bf16_bits_to_f64(bf16_bits(model.grad_flat(1)))
    want = p0 - h.lr * g / (np.abs(g) + h.eps) - h.lr * h.weight_decay * p0
    got = dp.reg[apm.APM_P32].cpu().numpy().reshape(-1).astype(np.float64)
    err = np.abs(got - want)
    assert np.all(err <= np.maximum(1e-6 * np.abs(want), 1e-9))
    dp.destroy()


def test_cfg2_gpt2_small_ten_steps_full_oracle_and_unpack():
    specs, E = specs_of("gpt2_small_124m")
    model = Model(specs, E, seed=0)
    dp, st, worst = run_resident(model, 10, oracle.Hyper())
    log(f"cfg2 pages {model.plan.n_pages} frag {model.plan.fragmentation:.4f} worst rel err {worst}")
    assert worst["v"] < 2e-6
    # unpack is the inverse of pack: tensor-space result == the pages gathered by the oracle plan
    for state in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        flat = unpack_all(model, dp, state)
        if state == apm.APM_P16:
            pages = bf16_bits(dp.reg[state])
            host = bf16_bits(flat)
        else:
            pages = dp.reg[state].cpu().numpy().view(np.uint32)
            host = flat.cpu().numpy().view(np.uint32)
        want = oracle.unpack(model.plan, pages, model.numels)
        for i, w in enumerate(want):
            a = int(model.off[i])
            assert np.array_equal(host[a:a + w.size], w), f"unpack state {state} tensor {i}"
    dp.destroy()


def sampled_pages(plan, every):
    """Every `every`-th page, the first and last, and every page that is not completely full."""
    s = set(range(0, plan.n_pages, every)) | {0, plan.n_pages - 1}
    s |= {k for k, p in enumerate(plan.pages) if p.used < plan.page_elems}
    return sorted(s)


@pytest.mark.parametrize("stepper", ["sync", "fused"])
def test_cfg3_gpt_1p3b_clipped_ten_steps_sampled_oracle(stepper):
    # "fused" is the launch configuration bench.py times: gradients read from the tensors, bf16
    # parameters written to the tensors, no G16 / P16 page traffic
    specs, E = specs_of("gpt_1p3b")
    model = Model(specs, E, seed=0)
    sample = sampled_pages(model.plan, 16)
    log(f"cfg3 pages {model.plan.n_pages}, oracle on {len(sample)} pages")
    h = oracle.Hyper(max_grad_norm=1.0)
    dp, st, worst = run_resident(model, 10, h, sample=sample, stepper=stepper)
    log(f"cfg3 worst rel err {worst}")
    assert worst["v"] < 2e-6
    dp.destroy()


def test_cfg5_moe_skip_sync_and_delayed_sampled_oracle():
    # 20 steps; per step 8 of 64 experts per layer receive a gradient, every other expert page is
    # skipped.  A synchronous pool (checked against the oracle on sampled pages) and a delayed pool
    # run side by side on the same gradients; after the flush they must agree bit for bit.
    f, E = synth.WORKLOADS["moe_8x64"]
    specs = f()
    steps = 20
    act = lambda t: synth.moe_active_tensors(specs, t, 0, 64, 8)
    h = oracle.Hyper(skip_mode=1)
    hy = to_hyper(h)
    model = Model(specs, E, seed=0, active_fn=act)
    plan, n_t = model.plan, len(specs)
    n_pages = plan.n_pages
    sample = sampled_pages(plan, 64)
    used = [plan.pages[p].used for p in sample]
    log(f"cfg5 pages {n_pages}, oracle on {len(sample)} pages")
    a = DevicePool(n_pages, E)
    b = DevicePool(n_pages, E, states=(apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16))
    for dp in (a, b):
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    st = oracle.PagedAdamWState(model.host_pages(model.p_flat, sample).view(np.float32), used)
    skip_d = torch.zeros(n_pages, dtype=torch.uint8, device=DEV)
    norm_d = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    n_skipped = 0
    touched = np.zeros(len(sample), dtype=bool)
    for t in range(1, steps + 1):
        g_flat = model.grad_flat(t)
        apm.apm_pack_tensors(a.pool, apm.APM_G16, model.tensors(g_flat), n_t)
        apm.apm_page_adamw_step(a.pool, None, n_pages, t, hy, norm_d, skip_d)
        apm.apm_step_delayed(b.pool, None, n_pages, a.reg[apm.APM_G16], hy)
        assert apm.apm_delayed_applied(b.pool) == t - 1
        norms, skips = st.step(model.host_pages(g_flat, sample), t, h, threads=HOST_THREADS)
        torch.cuda.synchronize()
        sk = skip_d.cpu().numpy()
        assert np.array_equal(sk[sample], skips)
        nrm = norm_d.cpu().numpy()[sample]
        assert np.all(np.abs(nrm - norms) <= 1e-6 * np.abs(norms))
        n_skipped += int(sk.sum())
        touched |= skips == 0
        del g_flat
    # 56 of 64 experts x 2 matrices x 4 pages x 8 layers are skipped every step
    assert n_skipped == steps * 8 * 56 * 2 * 4
    apm.apm_step_delayed(b.pool, None, n_pages, None, hy)          # flush
    torch.cuda.synchronize()
    assert apm.apm_delayed_applied(b.pool) == steps
    worst = {k: check_state_close(k, a.rows_f32(s_, sample), ref, used)
             for k, s_, ref in (("p", apm.APM_P32, st.p), ("m", apm.APM_M32, st.m), ("v", apm.APM_V32, st.v))}
    log(f"cfg5 worst rel err {worst}")
    check_p16(a.rows_b16(apm.APM_P16, sample), a.rows_f32(apm.APM_P32, sample), st.p16, used, touched)
    assert not touched.all() and touched.any()
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        assert torch.equal(a.reg[s_].view(torch.int16), b.reg[s_].view(torch.int16)), f"state {s_}: delayed != sync"
    a.destroy()
    b.destroy()


def test_delayed_small_with_page_list_and_outputs():
    E = 16384
    numels = [3 * E + 5, 100, 2 * E, 9000]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=9, sigma_g=5e-3)
    n = model.plan.n_pages
    listed = [p for p in range(n) if p != 2]
    dp, st, worst = run_resident(model, 5, oracle.Hyper(max_grad_norm=0.5, skip_mode=1),
                                 page_list=listed, stepper="delayed")
    dp.destroy()


def test_delayed_applies_each_gradient_with_the_hyper_and_page_list_it_came_with():
    # a learning-rate / decay / clip schedule and a page list that changes from call to call:
    # N delayed calls + flush == N synchronous steps bit for bit, and == the oracle's stepper
    E = 16384
    numels = [3 * E + 5, 100, 2 * E, 9000, E]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=12, sigma_g=5e-3)
    n, n_t = model.plan.n_pages, len(specs)
    T = 6
    hs = [oracle.Hyper(lr=1e-4 * (t + 1), weight_decay=0.01 * (t % 3), max_grad_norm=0.2 * (t + 1))
          for t in range(T)]
    lists = [None, [0, 2, 5], [1], None, [6, 0, 3, 1], [4]]
    a = DevicePool(n, E)   # synchronous
    b = DevicePool(n, E)   # one step stale
    for dp in (a, b):
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    gbuf = DevicePool(n, E, states=(apm.APM_G16,))
    pages = list(range(n))
    used = [model.plan.pages[p].used for p in pages]
    st = oracle.PagedAdamWState(model.host_pages(model.p_flat, pages).view(np.float32), used)
    d = oracle.DelayedStepper(st)
    for t in range(T):
        g = model.grad_flat(t + 1)
        apm.apm_pack_tensors(a.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_pack_tensors(gbuf.pool, apm.APM_G16, model.tensors(g), n_t)
        lst = lists[t]
        k = n if lst is None else len(lst)
        apm.apm_page_adamw_step(a.pool, lst, k, t + 1, to_hyper(hs[t]))
        apm.apm_step_delayed(b.pool, lst, k, gbuf.reg[apm.APM_G16], to_hyper(hs[t]))
        torch.cuda.synchronize()
        d.step(model.host_pages(g, pages), hs[t], lst)
    flush_h = to_hyper(oracle.Hyper(lr=7.0, weight_decay=0.5))   # belongs to no gradient
    apm.apm_step_delayed(b.pool, None, n, None, flush_h)
    d.step(None, oracle.Hyper(lr=7.0))
    torch.cuda.synchronize()
    assert apm.apm_delayed_applied(b.pool) == T
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        assert torch.equal(a.reg[s_].view(torch.int16), b.reg[s_].view(torch.int16)), f"state {s_}: delayed != sync"
    for name, s_, want in (("p", apm.APM_P32, st.p), ("m", apm.APM_M32, st.m), ("v", apm.APM_V32, st.v)):
        check_state_close(name, b.rows_f32(s_, pages), want, used)
    for dp in (a, b, gbuf):
        dp.destroy()


def test_delayed_zero_copy_handover_equals_sync():
    # the producer writes its gradient pages straight into the half handed out by
    # apm_delayed_grad_buffer (here: by packing into a pool whose G16 class aliases that half)
    E = 16384
    numels = [3 * E + 5, 100, 2 * E, 9000, E]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=10, sigma_g=5e-3)
    n, n_t = model.plan.n_pages, len(specs)
    hy = to_hyper(oracle.Hyper(max_grad_norm=0.5))
    a = DevicePool(n, E)
    b = DevicePool(n, E, states=(apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16))
    for dp in (a, b):
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    halves = {}
    for t in range(1, 6):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(a.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(a.pool, None, n, t, hy)
        ptr = apm.apm_delayed_grad_buffer(b.pool)
        if ptr not in halves:
            # NO_ZERO: the library hands the halves out zero-filled, and pack leaves gaps alone
            halves[ptr] = apm.apm_pool_create(apm.APM_DEV_GPU, E, n, state_mask=1 << apm.APM_G16,
                                              flags=apm.APM_POOL_NO_ZERO, base={apm.APM_G16: ptr})
        apm.apm_pack_tensors(halves[ptr], apm.APM_G16, model.tensors(g), n_t)
        apm.apm_step_delayed(b.pool, None, n, ptr, hy)
        torch.cuda.synchronize()
    assert len(halves) == 2
    apm.apm_step_delayed(b.pool, None, n, None, hy)
    torch.cuda.synchronize()
    assert apm.apm_delayed_applied(b.pool) == 5
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        assert torch.equal(a.reg[s_].view(torch.int16), b.reg[s_].view(torch.int16)), f"state {s_}"
    for h in halves.values():
        h.destroy()
    a.destroy()
    b.destroy()


def test_delayed_accumulation_matches_oracle_and_presummed_sync():
    # three micro-gradients per update: the first starts the collection, two are accumulated
    E = 16384
    numels = [3 * E + 5, 100, 2 * E, 9000, E]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=11, sigma_g=5e-3)
    plan, n, n_t = model.plan, model.plan.n_pages, len(specs)
    h = oracle.Hyper(max_grad_norm=0.5)
    hy = to_hyper(h)
    a = DevicePool(n, E)                       # synchronous, on the pre-summed gradient
    b = DevicePool(n, E)                       # delayed + accumulate
    for dp in (a, b):
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    pages = list(range(n))
    st = oracle.PagedAdamWState(model.host_pages(model.p_flat, pages).view(np.float32), plan.used())
    d = oracle.DelayedStepper(st)
    stage = DevicePool(n, E, states=(apm.APM_G16,))
    for t in range(1, 4):
        gs = [model.grad_flat(10 * t + k) for k in range(3)]
        rows = [model.host_pages(g, pages) for g in gs]
        d.step(rows[0], h)
        d.accumulate(rows[1])
        d.accumulate(rows[2])
        total = (gs[0] + gs[1]) + gs[2]                    # bf16 additions: fp32 sum, nearest even
        apm.apm_pack_tensors(a.pool, apm.APM_G16, model.tensors(total), n_t)
        torch.cuda.synchronize()
        assert np.array_equal(a.rows_b16(apm.APM_G16, pages), d.buffered), "oracle sum != library bf16 sum"
        apm.apm_page_adamw_step(a.pool, None, n, t, hy)
        apm.apm_pack_tensors(stage.pool, apm.APM_G16, model.tensors(gs[0]), n_t)
        apm.apm_step_delayed(b.pool, None, n, stage.reg[apm.APM_G16], hy)
        for k in (1, 2):
            apm.apm_pack_tensors(stage.pool, apm.APM_G16, model.tensors(gs[k]), n_t)
            apm.apm_delayed_accumulate(b.pool, None if k == 1 else pages[::-1], n, stage.reg[apm.APM_G16])
        torch.cuda.synchronize()
    apm.apm_step_delayed(b.pool, None, n, None, hy)
    d.step(None, h)
    torch.cuda.synchronize()
    with pytest.raises(apm.ApmError) as e:
        apm.apm_delayed_accumulate(b.pool, None, n, stage.reg[apm.APM_G16])
    assert e.value.code == apm.APM_ESTATE
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        assert torch.equal(a.reg[s_].view(torch.int16), b.reg[s_].view(torch.int16)), f"state {s_}"
    used = plan.used()
    check_state_close("p32", b.rows_f32(apm.APM_P32, pages), st.p, used)
    check_state_close("m32", b.rows_f32(apm.APM_M32, pages), st.m, used)
    check_state_close("v32", b.rows_f32(apm.APM_V32, pages), st.v, used)
    for dp in (a, b, stage):
        dp.destroy()


def test_edge_ragged_lists_page_lists_clip_and_skip():
    # small pages so that tensors span several tiles with ragged tails; odd numels so that tensor
    # pointers are not 16-byte aligned; zero-size tensors; exact-page tensors
    E = 40960
    numels = [E * 2 + 4097, 1, 7, E - 1, E, E + 1, 0, 3 * E + 12345, 255, 8193, 2 * E]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    zero_grad = {3, 8}                      # tensors without gradient -> their sole pages are skipped
    act = lambda t: np.array([i not in zero_grad for i in range(len(numels))])
    model = Model(specs, E, seed=3, sigma_g=2e-3, active_fn=act, pad_elems=1)
    h = oracle.Hyper(max_grad_norm=0.3, skip_mode=1)
    dp, st, worst = run_resident(model, 4, h)
    log(f"edge worst {worst}")
    dp.destroy()
    # a permuted, partial page list: unlisted pages must stay untouched
    model2 = Model(specs, E, seed=4, pad_elems=3)
    n = model2.plan.n_pages
    listed = [p for p in reversed(range(n)) if p % 3 != 1]
    dp, st, worst = run_resident(model2, 3, oracle.Hyper(max_grad_norm=0.05), page_list=listed)
    unl = [p for p in range(n) if p % 3 == 1]
    assert not dp.rows_f32(apm.APM_M32, unl).any() and not dp.rows_b16(apm.APM_P16, unl).any()
    dp.destroy()


@pytest.mark.parametrize("gather,scatter", [(True, True), (True, False), (False, True)])
def test_fused_gather_scatter_is_bit_identical_to_pack_step_unpack(gather, scatter):
    # gradients read straight from the tensors / bf16 parameters written straight to the tensors
    E = 40960
    numels = [E * 2 + 4097, 1, 7, E - 1, E, E + 1, 0, 3 * E + 12345, 255, 8193, 2 * E, 5 * E + 3]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    zero_grad = {3, 8}
    act = lambda t: np.array([i not in zero_grad for i in range(len(numels))])
    model = Model(specs, E, seed=6, sigma_g=2e-3, active_fn=act, align_elems=8)
    n_t, n_pages = len(specs), model.plan.n_pages
    hy = to_hyper(oracle.Hyper(max_grad_norm=0.3, skip_mode=1))
    a = DevicePool(n_pages, E)
    b = DevicePool(n_pages, E)
    for dp in (a, b):
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    q_a = torch.zeros(model.total, dtype=torch.bfloat16, device=DEV)
    q_b = torch.full((model.total,), 7.0, dtype=torch.bfloat16, device=DEV)
    q_a.fill_(7.0)
    norm_a = torch.zeros(n_pages, device=DEV)
    norm_b = torch.zeros(n_pages, device=DEV)
    skip_a = torch.zeros(n_pages, dtype=torch.uint8, device=DEV)
    skip_b = torch.zeros(n_pages, dtype=torch.uint8, device=DEV)
    for t in range(1, 4):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(a.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(a.pool, None, n_pages, t, hy, norm_a, skip_a)
        apm.apm_unpack(a.pool, apm.APM_P16, model.tensors(q_a), n_t)
        if not gather:
            apm.apm_pack_tensors(b.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step_fused(b.pool, None, n_pages, t, hy,
                                      model.tensors(g) if gather else None,
                                      model.tensors(q_b) if scatter else None, n_t, norm_b, skip_b)
        if not scatter:
            apm.apm_unpack(b.pool, apm.APM_P16, model.tensors(q_b), n_t)
        torch.cuda.synchronize()
        assert torch.equal(norm_a, norm_b) and torch.equal(skip_a, skip_b)
        assert skip_a.sum().item() == 2
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32):
        assert torch.equal(a.reg[s_].view(torch.int32), b.reg[s_].view(torch.int32)), f"state {s_}"
    # never-updated tensors: the fused path leaves the caller's tensor alone (still 7.0), the
    # unfused path copies the never-written P16 pages (zeros); everything else is identical
    keep = torch.ones(model.total, dtype=torch.bool, device=DEV)
    for i in zero_grad:
        sl = slice(int(model.off[i]), int(model.off[i]) + numels[i])
        keep[sl] = False
        if scatter:
            assert (q_b[sl] == 7.0).all()
        assert (q_a[sl] == 0.0).all()
    assert torch.equal(q_a.view(torch.int16)[keep], q_b.view(torch.int16)[keep])
    if scatter:     # the P16 page class was never written
        assert not b.reg[apm.APM_P16].view(torch.int16).any()
    # misaligned tensors are refused, not mis-read
    bad = model.grad_flat(1)
    ptrs = [bad.data_ptr() + 2 * int(model.off[i]) + 2 for i in range(n_t)]
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step_fused(b.pool, None, n_pages, 4, hy,
                                      apm.make_tensors(numels, apm.APM_BF16, ptrs), None, n_t)
    assert e.value.code == apm.APM_EINVAL
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step_fused(b.pool, None, n_pages, 4, hy,
                                      apm.make_tensors(numels[:-1], apm.APM_BF16, ptrs[:-1]), None, n_t - 1)
    assert e.value.code == apm.APM_ESTATE
    a.destroy()
    b.destroy()


def test_many_tiny_pages_exercise_grid_chunking_and_minimal_page_size():
    # 70 000 pages of 64 elements: more listed pages than one grid dimension holds (65 535), so the
    # launchers split the list; also the smallest slices (a page is a fraction of one tile)
    E = 64
    rng = np.random.default_rng(0)
    numels = [int(x) for x in rng.choice([1, 7, 8, 63, 64, 65, 130, 640, 6400], size=9000)]
    numels.append(E * 56000 + 5)
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=12, sigma_g=1e-2)
    n = model.plan.n_pages
    assert n > 66000
    sample = sorted(set(range(0, n, 97)) | {0, n - 1, 65534, 65535, 65536})
    dp, st, worst = run_resident(model, 2, oracle.Hyper(max_grad_norm=0.05, skip_mode=1), sample=sample)
    dp.destroy()
    # a permuted list longer than one grid dimension goes through the staged page list
    listed = list(reversed(range(n)))
    dp, st, worst = run_resident(model, 1, oracle.Hyper(max_grad_norm=0.05), sample=sample,
                                 page_list=listed)
    dp.destroy()


@pytest.mark.parametrize("stepper", ["sync", "fused"])
def test_pages_of_very_different_extents_in_a_permuted_list(stepper):
    # Full pages, pages a tenth full and pages holding a hundred elements, enough of each that the
    # library launches them as separate groups with their own grid sizes; the list is permuted so
    # that the per-page outputs must come back in the caller's order.
    E = 1 << 20
    numels = [3 * E + 5000]
    numels += [100000 + 8 * i for i in range(22)]
    numels += [100 + i for i in range(320)]
    numels += [2 * E]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    zero_grad = {5, 40, 41, 300}
    act = lambda t: np.array([i not in zero_grad for i in range(len(numels))])
    model = Model(specs, E, seed=21, sigma_g=2e-3, active_fn=act, align_elems=8)
    n = model.plan.n_pages
    rng = np.random.default_rng(5)
    listed = [int(p) for p in rng.permutation(n) if p % 11 != 3]
    sample = sorted(set(range(0, n, 7)) | {0, 1, 2, 3, 4, 5, 6, n - 3, n - 2, n - 1})
    h = oracle.Hyper(max_grad_norm=0.5, skip_mode=1)
    dp, st, worst = run_resident(model, 2, h, sample=sample, page_list=listed, stepper=stepper)
    log(f"mixed extents [{stepper}] worst {worst}")
    unl = [p for p in range(n) if p % 11 == 3]
    assert not dp.rows_f32(apm.APM_M32, unl).any()
    dp.destroy()
    # all pages in the natural order (no caller list): the reordering is internal only
    dp, st, worst = run_resident(model, 1, oracle.Hyper(), sample=sample, stepper=stepper)
    dp.destroy()


@pytest.mark.parametrize("clip", [0.0, 0.5])
def test_non_finite_gradients_propagate_as_in_the_oracle(clip):
    # inf and NaN gradients get no special treatment: the same elements become NaN on both sides
    # (a NaN page norm poisons its whole page when clipping is on, an infinite one zeroes the
    # page's finite gradients), and everything that stays finite passes the usual gate
    E, n_pages = 4096, 4
    dp = DevicePool(n_pages, E)
    p = synth.normal_f32(0, 1, 0, n_pages * E, 0.02, device=DEV)
    tens_p = apm.make_tensors([n_pages * E], apm.APM_F32, [p])
    apm.apm_pack_tensors(dp.pool, apm.APM_P32, tens_p, 1)
    st = oracle.PagedAdamWState(p.view(n_pages, E).cpu().numpy(), [E] * n_pages)
    hy_o = oracle.Hyper(max_grad_norm=clip)
    hy = to_hyper(hy_o)
    norm_d = torch.zeros(n_pages, dtype=torch.float32, device=DEV)
    for t in (1, 2):
        g = synth.normal_bf16(0, 1000 + t, 0, n_pages * E, 0.05, device=DEV).view(n_pages, E).clone()
        if t == 1:
            g[0, 5] = float("inf")
            g[1, 7] = float("nan")
            g[2, 9] = float("-inf")
            g[2, 4000] = float("nan")
        dp.reg[apm.APM_G16].copy_(g)
        apm.apm_page_adamw_step(dp.pool, None, n_pages, t, hy, norm_d, None)
        torch.cuda.synchronize()
        with np.errstate(all="ignore"):
            norms, _ = st.step(bf16_bits(g), t, hy_o)
        got = norm_d.cpu().numpy()
        assert np.array_equal(np.isnan(got), np.isnan(norms)) and np.array_equal(np.isinf(got), np.isinf(norms))
        fin = np.isfinite(norms)
        assert np.all(np.abs(got[fin] - norms[fin]) <= 1e-6 * np.abs(norms[fin]))
    pages = list(range(n_pages))
    n_nan = 0
    for name, state, want in (("p", apm.APM_P32, st.p), ("m", apm.APM_M32, st.m), ("v", apm.APM_V32, st.v)):
        got = dp.rows_f32(state, pages).astype(np.float64)
        assert np.array_equal(np.isnan(got), np.isnan(want)), f"{name}: NaN in different places"
        assert np.array_equal(np.isinf(got), np.isinf(want)) and np.array_equal(got[np.isinf(got)], want[np.isinf(want)])
        ok = np.isfinite(want)
        assert np.all(np.abs(got[ok] - want[ok]) <= np.maximum(1e-6 * np.abs(want[ok]), 1e-9)), name
        n_nan += int(np.isnan(want).sum())
    assert n_nan > 0 and np.isfinite(st.p[3]).all()
    p16 = dp.rows_b16(apm.APM_P16, pages)
    is_nan16 = ((p16 & 0x7F80) == 0x7F80) & ((p16 & 0x7F) != 0)
    assert np.array_equal(is_nan16, np.isnan(st.p))
    dp.destroy()


@pytest.mark.parametrize("stepper", ["sync", "fused", "delayed"])
def test_minimum_page_size_of_eight_elements(stepper):
    # the smallest page the library accepts: every page is a fraction of one vector tile
    E = 8
    numels = [8, 3, 16, 5, 1, 0, 24, 7, 9, 8]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=17, sigma_g=1e-2, align_elems=8)
    dp, st, worst = run_resident(model, 3, oracle.Hyper(max_grad_norm=0.01, skip_mode=1), stepper=stepper)
    dp.destroy()


def test_maximum_page_size_of_two_to_the_thirty_elements():
    # the largest page the library accepts (4 GiB fp32 pages): one tensor that fills page 0 and
    # spills into page 1, a small tensor alone in page 2.  The update is elementwise, so windows
    # of elements (start, middle, page end, the spill, the small page) go through the oracle; the
    # norms come from a float64 sum of squares over the whole pages.
    E = 1 << 30
    numels = [E + 12345, 777]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    model = Model(specs, E, seed=33, sigma_g=1e-3)
    assert model.plan.n_pages == 3
    n_t = len(specs)
    dp = DevicePool(3, E)
    apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    h = oracle.Hyper()                      # no clip: elements are independent of each other
    hy = to_hyper(h)
    norm_d = torch.zeros(3, dtype=torch.float32, device=DEV)
    windows = [(0, 0, 70000), (0, E // 2 - 3, 5000), (0, E - 4100, 4100), (1, 0, 12345), (2, 0, 777)]
    state = []
    for page, a, n in windows:
        p0 = dp.reg[apm.APM_P32][page, a:a + n].cpu().numpy()
        state.append([p0.astype(np.float64), np.zeros(n), np.zeros(n), np.zeros(n, dtype=np.uint16)])
    for t in (1, 2):
        g = model.grad_flat(t)
        apm.apm_pack_tensors(dp.pool, apm.APM_G16, model.tensors(g), n_t)
        apm.apm_page_adamw_step(dp.pool, None, 3, t, hy, norm_d, None)
        torch.cuda.synchronize()
        gp = dp.reg[apm.APM_G16]
        want_norm = [float(torch.sqrt((gp[k].double() ** 2).sum())) for k in range(3)]
        got = norm_d.cpu().numpy()
        assert np.all(np.abs(got - want_norm) <= 1e-6 * np.abs(want_norm)), (got, want_norm)
        for (page, a, n), (p, m, v, p16) in zip(windows, state):
            oracle.page_adamw(p, m, v, p16, bf16_bits(gp[page, a:a + n]), t, h)
        del g
    for (page, a, n), (p, m, v, p16) in zip(windows, state):
        for name, st_, want in (("p", apm.APM_P32, p), ("m", apm.APM_M32, m), ("v", apm.APM_V32, v)):
            got = dp.reg[st_][page, a:a + n].cpu().numpy()[None, :]
            check_state_close(f"{name} page {page} @ {a}", got, want[None, :], [n])
        got16 = bf16_bits(dp.reg[apm.APM_P16][page, a:a + n])[None, :]
        check_p16(got16, dp.reg[apm.APM_P32][page, a:a + n].cpu().numpy()[None, :], p16[None, :], [n])
    # nothing beyond the used extents was written
    assert not dp.reg[apm.APM_M32][1, 12345:12345 + (1 << 20)].any() and not dp.reg[apm.APM_M32][2, 777:].any()
    dp.destroy()


def test_no_outputs_no_clip_path_matches_path_with_reduce():
    # without clip/skip/outputs the reduce pass is not launched; results must be identical
    E = 16384
    specs = [synth.TensorSpec(0, "a", 5 * E + 100), synth.TensorSpec(1, "b", 77)]
    model = Model(specs, E, seed=5)
    a, _, _ = run_resident(model, 2, oracle.Hyper(), want_outputs=False)
    b, _, _ = run_resident(model, 2, oracle.Hyper(), want_outputs=True)
    for s in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        assert torch.equal(a.reg[s].view(torch.int16), b.reg[s].view(torch.int16))
    a.destroy()
    b.destroy()


def test_outputs_in_pinned_host_memory_equal_outputs_in_device_memory():
    # grad_norm / skip_mask are written by the kernel: any memory the GPU can address will do
    E = 4096
    specs = [synth.TensorSpec(0, "a", 3 * E + 40), synth.TensorSpec(1, "b", 9), synth.TensorSpec(2, "c", 2 * E)]
    model = Model(specs, E, seed=11)
    n = model.plan.n_pages
    dp = DevicePool(n, E)
    apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), len(specs))
    g = model.grad_flat(1)
    g[int(model.off[1]):int(model.off[2])] = 0                    # tensor b: an all-zero page
    apm.apm_pack_tensors(dp.pool, apm.APM_G16, model.tensors(g), len(specs))
    hy = apm.make_hyper(max_grad_norm=0.01, skip_mode=apm.APM_SKIP_UNTOUCHED)
    listed = list(reversed(range(n)))
    norm_d = torch.full((n,), -1.0, dtype=torch.float32, device=DEV)
    skip_d = torch.full((n,), 7, dtype=torch.uint8, device=DEV)
    norm_h = torch.full((n,), -1.0, dtype=torch.float32).pin_memory()
    skip_h = torch.full((n,), 7, dtype=torch.uint8).pin_memory()
    apm.apm_page_adamw_step(dp.pool, listed, n, 1, hy, norm_d, skip_d)
    apm.apm_page_adamw_step(dp.pool, listed, n, 2, hy, norm_h, skip_h)
    torch.cuda.synchronize()
    assert torch.equal(norm_d.cpu().view(torch.int32), norm_h.view(torch.int32))
    assert torch.equal(skip_d.cpu(), skip_h)
    assert int(skip_h.sum()) == 1 and float(norm_h.max()) > 0.01
    dp.destroy()


def test_error_paths_and_page_table():
    E = 1024
    dp = DevicePool(6, E)
    hy = apm.make_hyper()
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step(dp.pool, None, 2, 0, hy)
    assert e.value.code == apm.APM_EINVAL and "step" in str(e.value)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step(dp.pool, [0, 6], 2, 1, hy)
    assert e.value.code == apm.APM_ERANGE
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step(dp.pool, None, 2, 1, apm.make_hyper(beta1=1.0))
    assert e.value.code == apm.APM_EINVAL
    with pytest.raises(apm.ApmError) as e:                    # one page, two updates at once
        apm.apm_page_adamw_step(dp.pool, [3, 1, 3], 3, 1, hy)
    assert e.value.code == apm.APM_EINVAL and "twice" in str(e.value)
    apm.apm_page_adamw_step(dp.pool, None, 0, 1, hy)          # empty list: a no-op
    # layout too large for the pool
    big = apm.make_tensors([7 * E], apm.APM_F32)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_pool_set_layout(dp.pool, big, 1)
    assert e.value.code == apm.APM_ENOMEM
    numels = [2 * E + 10, 5, E + 1]
    res = apm.apm_pool_set_layout(dp.pool, apm.make_tensors(numels, apm.APM_F32, ids=[70, 71, 72]), 3)
    plan = oracle.plan_pack(numels, E)
    assert res.n_pages == plan.n_pages == apm.apm_pool_pages_in_use(dp.pool)
    for k, pe in enumerate(plan.pages):
        info = apm.apm_pool_page_info(dp.pool, k)
        assert info.total_elems == E and info.used_elems == pe.used
        assert info.available_elems == E - pe.used and info.device == apm.APM_DEV_GPU
        ids = [70 + t if t >= 0 else -1 for t in pe.tensor_id]
        assert list(info.tensor_id) == ids and list(info.tensor_elems) == pe.tensor_elems
        assert info.n_tensors == pe.n_tenants() <= 2
    # wrong dtype for the class, mismatching list
    x = torch.zeros(sum(numels), dtype=torch.float32, device=DEV)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_pack_tensors(dp.pool, apm.APM_G16, apm.make_tensors(numels, apm.APM_F32, [x] * 3), 3)
    assert e.value.code == apm.APM_EINVAL
    with pytest.raises(apm.ApmError) as e:
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, apm.make_tensors([5, 5], apm.APM_F32, [x] * 2), 2)
    assert e.value.code == apm.APM_ESTATE
    assert apm.apm_pool_state_ptr(dp.pool, apm.APM_M32, 2) == dp.reg[apm.APM_M32].data_ptr() + 2 * E * 4
    assert apm.apm_pool_state_ptr(dp.pool, apm.APM_M32, 6) is None
    dp.destroy()
