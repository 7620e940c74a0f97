"""apm_page_adamw_step_noalloc (fixed library-owned scratch, nothing allocated on its path) against
apm_page_adamw_step on the same inputs: same kernels, so every state class, the norms and the masks
must agree bit for bit -- on two calls in a row, the second with a smaller input, so that what the
first call left in the shared scratch is seen not to leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2303_02868_amd as apm
    from gpu_helpers import DEV, DevicePool, Model, check_state_close, to_hyper


def _pools(model):
    n, n_t = model.plan.n_pages, len(model.specs)
    a = DevicePool(n, model.E)
    b = DevicePool(n, model.E)
    for dp in (a, b):
        apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), n_t)
    return a, b


def _same(a, b, what):
    for s_ in (apm.APM_P32, apm.APM_M32, apm.APM_V32, apm.APM_P16):
        assert torch.equal(a.reg[s_].view(torch.int16), b.reg[s_].view(torch.int16)), f"{what}: state {s_}"


@pytest.mark.parametrize("h", [oracle.Hyper(max_grad_norm=0.5, skip_mode=1), oracle.Hyper()],
                         ids=["clip_skip", "plain"])
def test_noalloc_step_equals_the_allocating_step_on_two_calls_the_second_smaller(h):
    E = 32768
    # several full pages, a ragged tail, small tensors alone in their pages, one tensor without gradient
    numels = [5 * E + 1000, 17, 2 * E, 5000, E, 3 * E + 8, 4097]
    specs = [synth.TensorSpec(i, f"t{i}", n) for i, n in enumerate(numels)]
    active = lambda step: np.array([True, True, True, False, True, True, step != 2])
    big = Model(specs, E, seed=21, sigma_g=5e-3, active_fn=active)
    small = Model(specs[:3], E, seed=22, sigma_g=5e-3)
    assert small.plan.n_pages < big.plan.n_pages
    hy = to_hyper(h)
    want_out = h.max_grad_norm > 0
    assert big.plan.n_pages <= apm.apm_noalloc_max_pages(E)

    a1, b1 = _pools(big)
    a2, b2 = _pools(small)
    # two calls in a row through the new entry point: big, then small (no synchronisation between)
    outs = []
    for t in (1, 2):
        for model, a, b in ((big, a1, b1), (small, a2, b2)):
            n, n_t = model.plan.n_pages, len(model.specs)
            g = model.grad_flat(t)
            for dp in (a, b):
                apm.apm_pack_tensors(dp.pool, apm.APM_G16, model.tensors(g), n_t)
            na = torch.full((n,), -1.0, dtype=torch.float32, device=DEV) if want_out else None
            ka = torch.full((n,), 7, dtype=torch.uint8, device=DEV) if want_out else None
            nb = torch.full((n,), -2.0, dtype=torch.float32, device=DEV) if want_out else None
            kb = torch.full((n,), 9, dtype=torch.uint8, device=DEV) if want_out else None
            apm.apm_page_adamw_step_noalloc(b.pool, n, t, hy, nb, kb)
            apm.apm_page_adamw_step(a.pool, None, n, t, hy, na, ka)
            outs.append((na, ka, nb, kb))
    torch.cuda.synchronize()
    _same(a1, b1, "big")
    _same(a2, b2, "small")
    for na, ka, nb, kb in outs:
        if want_out:
            assert torch.equal(na, nb) and torch.equal(ka, kb)
    if want_out:
        assert any(bool(k.any()) for _, k, _, _ in outs) and not all(bool(k.all()) for _, k, _, _ in outs)

    # and against the oracle (first model, two steps), to the floating-point gate
    pages = list(range(big.plan.n_pages))
    used = [big.plan.pages[p].used for p in pages]
    st = oracle.PagedAdamWState(big.host_pages(big.p_flat, pages).view(np.float32), used)
    for t in (1, 2):
        st.step(big.host_pages(big.grad_flat(t), pages), t, h)
    for name, s_, want in (("p", apm.APM_P32, st.p), ("m", apm.APM_M32, st.m), ("v", apm.APM_V32, st.v)):
        check_state_close(name, b1.rows_f32(s_, pages), want, used)
    for dp in (a1, b1, a2, b2):
        dp.destroy()


def test_noalloc_step_rejects_what_its_scratch_cannot_hold_and_bad_arguments():
    E = 1 << 14
    cap = apm.apm_noalloc_max_pages(E)
    assert apm.apm_noalloc_scratch_bytes() == 4 << 20 and cap == (apm.apm_noalloc_scratch_bytes() - 768) // (32 + 12)
    n = 4
    dp = apm.apm_pool_create(apm.APM_DEV_GPU, 8, n)
    cap8 = apm.apm_noalloc_max_pages(8)                    # tiny pages: many of them are cheap
    assert cap8 == cap
    hy = apm.make_hyper()
    big = apm.apm_pool_create(apm.APM_DEV_GPU, 8, cap8 + 1)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step_noalloc(big, cap8 + 1, 1, hy)
    assert e.value.code == apm.APM_ERANGE and "fixed scratch" in str(e.value)
    apm.apm_page_adamw_step_noalloc(big, cap8, 1, hy)      # the limit itself is accepted
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step_noalloc(dp, 1, 0, hy)      # step < 1
    assert e.value.code == apm.APM_EINVAL
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step_noalloc(dp, n + 1, 1, hy)  # more pages than the pool has
    assert e.value.code == apm.APM_ERANGE
    part = apm.apm_pool_create(apm.APM_DEV_GPU, 8, 4, state_mask=apm.FP32_STATES)
    with pytest.raises(apm.ApmError) as e:
        apm.apm_page_adamw_step_noalloc(part, 1, 1, hy)
    assert e.value.code == apm.APM_ESTATE
    torch.cuda.synchronize()
    for p in (dp, big, part):
        p.destroy()
