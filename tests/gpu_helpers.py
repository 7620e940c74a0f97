"""Shared machinery of the GPU parity tests: seeded device inputs, the HIP path driven through the
C-ABI binding, and the oracle driven on the same bits (copied from the input tensors, never from
anything the HIP path produced)."""
from __future__ import annotations

import os
from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

import oracle
import paper_2303_02868_amd as apm
import synth

DEV = "cuda:0"
STREAM_P = 1
HOST_THREADS = min(16, os.cpu_count() or 1)


def stream_g(step: int) -> int:
    return 1000 + step


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a bf16 tensor, on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f32_bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def gen_flat(seed: int, stream: int, total: int, sigma: float, bf16: bool, chunk: int = 1 << 26):
    """Flat device tensor of `total` seeded values (tensor-space element index = position)."""
    out = torch.empty(total, dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
    fn = synth.normal_bf16 if bf16 else synth.normal_f32
    for a in range(0, total, chunk):
        n = min(chunk, total - a)
        out[a:a + n] = fn(seed, stream, a, n, sigma, device=DEV)
    return out


class Model:
    """A synthetic model: a tensor list whose tensors are slices of flat device buffers."""

    def __init__(self, specs: Sequence[synth.TensorSpec], E: int, seed: int = 0,
                 sigma_p: float = 0.02, sigma_g: float = 1e-3,
                 active_fn: Optional[Callable[[int], np.ndarray]] = None, pad_elems: int = 0,
                 align_elems: int = 1):
        self.specs = list(specs)
        self.numels = [t.numel for t in self.specs]
        self.E = E
        self.seed, self.sigma_p, self.sigma_g = seed, sigma_p, sigma_g
        self.active_fn = active_fn
        # pad_elems shifts every tensor by that many elements per preceding tensor, to produce
        # unaligned tensor pointers when wanted
        # align_elems rounds every tensor start up to that many elements (8 = 16-byte aligned bf16)
        self.off = np.zeros(len(self.specs) + 1, dtype=np.int64)
        for i, n in enumerate(self.numels):
            self.off[i + 1] = -(-(self.off[i] + n + pad_elems) // align_elems) * align_elems
        self.total = int(self.off[-1])
        self.plan = oracle.plan_pack(self.numels, E)
        self.p_flat = gen_flat(seed, STREAM_P, self.total, sigma_p, bf16=False)

    def grad_flat(self, step: int) -> torch.Tensor:
        if self.active_fn is None:
            return gen_flat(self.seed, stream_g(step), self.total, self.sigma_g, bf16=True)
        g = torch.zeros(self.total, dtype=torch.bfloat16, device=DEV)
        for i in np.nonzero(self.active_fn(step))[0]:       # tensors without gradient stay zero
            a, n = int(self.off[i]), self.numels[i]
            g[a:a + n] = synth.normal_bf16(self.seed, stream_g(step), a, n, self.sigma_g, device=DEV)
        return g

    def tensors(self, flat: torch.Tensor):
        """apm_tensor array whose data pointers are the tensors' slices of `flat`."""
        dtype = apm.APM_BF16 if flat.dtype == torch.bfloat16 else apm.APM_F32
        base, item = flat.data_ptr(), flat.element_size()
        ptrs = [base + int(self.off[i]) * item for i in range(len(self.specs))]
        return apm.make_tensors(self.numels, dtype, ptrs, ids=[t.id for t in self.specs])

    def host_pages(self, flat: torch.Tensor, pages: Sequence[int]) -> np.ndarray:
        """Rows = the listed pages as the oracle packer lays them out, built on the host from the
        tensor-space input `flat` (uint32 bits for fp32 inputs, uint16 bits for bf16 inputs)."""
        is16 = flat.dtype == torch.bfloat16
        out = np.zeros((len(pages), self.E), dtype=np.uint16 if is16 else np.uint32)
        row = {p: r for r, p in enumerate(pages)}
        for s in self.plan.segments:
            r = row.get(s.page)
            if r is None:
                continue
            a = int(self.off[s.tensor]) + s.tensor_off
            piece = flat[a:a + s.n]
            bits = bf16_bits(piece) if is16 else piece.cpu().numpy().view(np.uint32)
            out[r, s.page_off:s.page_off + s.n] = bits
        return out


class DevicePool:
    """A GPU pool over caller-owned torch regions, so tests can read raw pages."""

    def __init__(self, n_pages: int, E: int, states=(0, 1, 2, 3, 4)):
        self.n_pages, self.E = n_pages, E
        self.reg = {}
        for s in states:
            dt = torch.float32 if s <= apm.APM_V32 else torch.bfloat16
            self.reg[s] = torch.zeros((n_pages, E), dtype=dt, device=DEV)
        mask = sum(1 << s for s in states)
        self.pool = apm.apm_pool_create(apm.APM_DEV_GPU, E, n_pages, state_mask=mask,
                                        base={s: t for s, t in self.reg.items()})

    def rows_f32(self, state: int, pages: Sequence[int]) -> np.ndarray:
        idx = torch.as_tensor(list(pages), device=DEV)
        return self.reg[state][idx].cpu().numpy()

    def rows_b16(self, state: int, pages: Sequence[int]) -> np.ndarray:
        idx = torch.as_tensor(list(pages), device=DEV)
        return bf16_bits(self.reg[state][idx])

    def destroy(self):
        self.pool.destroy()


def to_hyper(h: oracle.Hyper):
    return apm.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.max_grad_norm, h.skip_mode)


def check_state_close(name: str, got: np.ndarray, want: np.ndarray, used: Sequence[int],
                      rel: float = 1e-6, floor: float = 1e-9):
    """The parity gate for fp32 state: |gpu - oracle| <= max(rel*|oracle|, floor) on the used
    extent of every row.  Returns the largest relative error with a 1e-15 floor (reported)."""
    worst = 0.0
    for r, n in enumerate(used):
        g = got[r, :n].astype(np.float64)
        w = want[r, :n]
        err = np.abs(g - w)
        tol = np.maximum(rel * np.abs(w), floor)
        bad = err > tol
        assert not bad.any(), (f"{name}: row {r} elem {int(np.argmax(bad))}: gpu {g[np.argmax(bad)]!r} "
                               f"oracle {w[np.argmax(bad)]!r}")
        if n:
            worst = max(worst, float(np.max(err / np.maximum(np.abs(w), 1e-15))))
    return worst


def check_p16(got_p16: np.ndarray, got_p32: np.ndarray, want_p16: np.ndarray, used: Sequence[int],
              touched: Optional[Sequence[bool]] = None):
    """p16 is bit-exactly the cast of the GPU's own fp32 master, and within one bf16 ulp (plus the
    1e-9 absolute floor of the fp32 gate, which matters where p passes close to zero) of the
    oracle's p16, whose fp32 master may differ in the last place."""
    for r, n in enumerate(used):
        if touched is not None and not touched[r]:      # never updated: p16 keeps its initial bits
            assert np.array_equal(got_p16[r, :n], want_p16[r, :n]), f"p16 row {r} (never updated)"
            continue
        assert np.array_equal(got_p16[r, :n], oracle.bf16_rne(f32_bits(got_p32[r, :n]))), f"p16 row {r}"
        a = oracle.bf16_bits_to_f64(got_p16[r, :n])
        b = oracle.bf16_bits_to_f64(want_p16[r, :n])
        big = np.maximum(np.maximum(np.abs(a), np.abs(b)), 2.0 ** -126)
        ulp = np.exp2(np.floor(np.log2(big)) - 7)
        bad = np.abs(a - b) > ulp + 1e-9
        assert not bad.any(), f"p16 row {r} elem {int(np.argmax(bad))}: {a[np.argmax(bad)]} vs oracle {b[np.argmax(bad)]}"


def check_padding_zero(dp: DevicePool, plan: oracle.PackPlan, pages: Sequence[int]):
    """Unused elements of the listed pages are zero in every class."""
    mask = np.ones((len(pages), plan.page_elems), dtype=bool)
    row = {p: r for r, p in enumerate(pages)}
    for s in plan.segments:
        r = row.get(s.page)
        if r is not None:
            mask[r, s.page_off:s.page_off + s.n] = False
    for st in dp.reg:
        rows = dp.rows_f32(st, pages).view(np.uint32) if st <= apm.APM_V32 else dp.rows_b16(st, pages)
        assert not rows[mask].any(), f"state {st}: padding not zero"


def run_resident(model: Model, steps: int, h: oracle.Hyper, sample: Optional[Sequence[int]] = None,
                 page_list: Optional[Sequence[int]] = None, want_outputs: bool = True,
                 stepper: str = "sync"):
    """Runs `steps` AdamW steps through the HIP path on all pages (or `page_list`) and through the
    oracle on the sampled pages (default: all), then applies the parity gates.
    stepper: "sync" = pack g16 + apm_page_adamw_step, "fused" = apm_page_adamw_step_fused reading g16
    from and writing p16 to tensors (the form bench.py times), "delayed" = apm_step_delayed + flush."""
    plan = model.plan
    n_pages, E = plan.n_pages, model.E
    sample = list(range(n_pages)) if sample is None else list(sample)
    listed = list(range(n_pages)) if page_list is None else list(page_list)
    listed_set = set(listed)
    used = [plan.pages[p].used for p in sample]
    hy = to_hyper(h)

    dp = DevicePool(n_pages, E)
    res = apm.apm_pack_tensors(dp.pool, apm.APM_P32, model.tensors(model.p_flat), len(model.specs))
    assert res.n_pages == n_pages
    assert res.segments == [(s.tensor, s.tensor_off, s.page, s.page_off, s.n) for s in plan.segments]
    assert abs(res.fragmentation - plan.fragmentation) < 1e-12
    torch.cuda.synchronize()

    p_rows = model.host_pages(model.p_flat, sample)                       # uint32 bits
    assert np.array_equal(dp.rows_f32(apm.APM_P32, sample).view(np.uint32), p_rows), "pack p32 not bit-exact"
    st = oracle.PagedAdamWState(p_rows.view(np.float32), used)

    norm_d = torch.full((len(listed),), -1.0, dtype=torch.float32, device=DEV) if want_outputs else None
    skip_d = torch.full((len(listed),), 7, dtype=torch.uint8, device=DEV) if want_outputs else None
    pages_arg = None if page_list is None else listed
    if stepper == "delayed":
        apm.apm_delayed_set_outputs(dp.pool, norm_d, skip_d)
    last_outputs = None
    q_flat = torch.zeros(model.total, dtype=torch.bfloat16, device=DEV) if stepper == "fused" else None
    touched = [False] * len(sample)
    for t in range(1, steps + 1):
        g_flat = model.grad_flat(t)
        g_rows = model.host_pages(g_flat, sample)
        if stepper == "sync":
            apm.apm_pack_tensors(dp.pool, apm.APM_G16, model.tensors(g_flat), len(model.specs))
            apm.apm_page_adamw_step(dp.pool, pages_arg, len(listed), t, hy, norm_d, skip_d)
        elif stepper == "fused":
            apm.apm_page_adamw_step_fused(dp.pool, pages_arg, len(listed), t, hy, model.tensors(g_flat),
                                          model.tensors(q_flat), len(model.specs), norm_d, skip_d)
        else:
            # the producer writes its gradient in page layout into its own buffer (a second pool
            # over g_pack would do the same; the G16 class of dp serves as that buffer here)
            apm.apm_pack_tensors(dp.pool, apm.APM_G16, model.tensors(g_flat), len(model.specs))
            apm.apm_step_delayed(dp.pool, pages_arg, len(listed), dp.reg[apm.APM_G16], hy)
            assert apm.apm_delayed_applied(dp.pool) == t - 1
        torch.cuda.synchronize()
        if stepper == "sync":
            assert np.array_equal(dp.rows_b16(apm.APM_G16, sample), g_rows), "pack g16 not bit-exact"
        upd = [r for r, p in enumerate(sample) if p in listed_set]
        norms, skips = st.step(g_rows, t, h, pages=upd, threads=HOST_THREADS)
        last_outputs = (upd, norms, skips)
        for r, sk in zip(upd, skips):
            touched[r] = touched[r] or not sk
        if want_outputs and stepper in ("sync", "fused"):
            check_outputs(norm_d, skip_d, listed, sample, upd, norms, skips)
        del g_flat
    if stepper == "delayed":
        apm.apm_step_delayed(dp.pool, pages_arg, len(listed), None, hy)
        torch.cuda.synchronize()
        assert apm.apm_delayed_applied(dp.pool) == steps
        if want_outputs:
            check_outputs(norm_d, skip_d, listed, sample, *last_outputs)

    got_p = dp.rows_f32(apm.APM_P32, sample)
    got_m = dp.rows_f32(apm.APM_M32, sample)
    got_v = dp.rows_f32(apm.APM_V32, sample)
    if stepper == "fused":      # p16 went to the tensors: lay them out like pages for the check
        got_p16 = model.host_pages(q_flat, sample)
        assert not dp.reg[apm.APM_P16].view(torch.int16).any() and not dp.reg[apm.APM_G16].view(torch.int16).any()
    else:
        got_p16 = dp.rows_b16(apm.APM_P16, sample)
    worst = {
        "p": check_state_close("p32", got_p, st.p, used),
        "m": check_state_close("m32", got_m, st.m, used),
        "v": check_state_close("v32", got_v, st.v, used),
    }
    check_p16(got_p16, got_p, st.p16, used, touched)
    check_padding_zero(dp, plan, sample)
    dp.q_flat = q_flat
    return dp, st, worst


def check_outputs(norm_d, skip_d, listed, sample, upd, norms, skips):
    norm_g = norm_d.cpu().numpy()
    skip_g = skip_d.cpu().numpy()
    pos = {p: i for i, p in enumerate(listed)}
    for r, nrm, sk in zip(upd, norms, skips):
        i = pos[sample[r]]
        assert int(skip_g[i]) == int(sk), f"skip mask differs on page {sample[r]}"
        assert abs(float(norm_g[i]) - float(nrm)) <= 1e-6 * abs(float(nrm)), f"norm page {sample[r]}: {norm_g[i]} vs {nrm}"


def unpack_all(model: Model, dp: DevicePool, state: int) -> torch.Tensor:
    """apm_unpack of one class into a fresh flat buffer."""
    dt = torch.float32 if state <= apm.APM_V32 else torch.bfloat16
    flat = torch.zeros(model.total, dtype=dt, device=DEV)
    apm.apm_unpack(dp.pool, state, model.tensors(flat), len(model.specs))
    torch.cuda.synchronize()
    return flat
