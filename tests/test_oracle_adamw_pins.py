"""Pins of the AdamW oracle to things other than itself: exact rational closed forms, torch's
float64 AdamW, high-precision brute force on 3 elements, and invariants."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import Hyper

H = Hyper()  # lr 1e-4, betas 0.9/0.999, eps 1e-8, wd 0.01


def bf16_bits(x):
    """bf16 bit patterns of values that are exactly representable in bf16 (checked)."""
    a = np.asarray(x, dtype=np.float32)
    u = a.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "test value is not a bf16 number"
    return (u >> 16).astype(np.uint16)


def some_bf16_values(n, seed, scale=1e-3):
    rng = np.random.default_rng(seed)
    a = (rng.standard_normal(n) * scale).astype(np.float32)
    u = a.view(np.uint32) & np.uint32(0xFFFF0000)
    return u.view(np.float32).copy()


def run_steps(p0, grads, h, t0=1):
    """grads: list of fp32 arrays holding bf16-representable values."""
    n = p0.size
    p = p0.astype(np.float64).copy()
    m = np.zeros(n)
    v = np.zeros(n)
    p16 = np.zeros(n, dtype=np.uint16)
    outs = []
    for k, g in enumerate(grads):
        outs.append(oracle.page_adamw(p, m, v, p16, bf16_bits(g), t0 + k, h))
    return p, m, v, p16, outs


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.max(np.abs(a - b) / np.maximum(np.abs(b), 1e-300))


def test_first_step_closed_form_exact_rational():
    # m = v = 0, t = 1:  p' - p = -lr*g/(|g|+eps) - lr*wd*p  exactly over the rationals.
    g = some_bf16_values(257, 1)
    g[:3] = [0.0, 2.0 ** -126, -1.0]          # zero, tiny, large
    p0 = (np.random.default_rng(2).standard_normal(257) * 0.02).astype(np.float32)
    p, m, v, _, _ = run_steps(p0, [g], H)
    lr, eps, wd = Fraction(H.lr), Fraction(H.eps), Fraction(H.weight_decay)
    for i in range(g.size):
        gi, pi = Fraction(float(g[i])), Fraction(float(p0[i]))
        want = pi - lr * gi / (abs(gi) + eps) - lr * wd * pi
        assert abs(Fraction(p[i]) - want) <= abs(want) * Fraction(1, 10 ** 14) + Fraction(1, 10 ** 30)
        assert abs(Fraction(m[i]) - (1 - Fraction(H.beta1)) * gi) <= abs(gi) * Fraction(1, 10 ** 15)
        assert abs(Fraction(v[i]) - (1 - Fraction(H.beta2)) * gi * gi) <= gi * gi * Fraction(1, 10 ** 15)


@pytest.mark.parametrize("T", [1, 2, 10])
def test_constant_gradient_closed_form(T):
    # g fixed over steps => mhat_t = g, vhat_t = g^2 exactly, so with a = 1-lr*wd, u = lr*g/(|g|+eps):
    #   p_T = p_0 a^T - u (1-a^T)/(1-a),  m_T = (1-b1^T) g,  v_T = (1-b2^T) g^2.
    # Pins bias correction, the 1-based step count and the decay acting on the old p.
    g = some_bf16_values(64, 3)
    p0 = (np.random.default_rng(4).standard_normal(64) * 0.02).astype(np.float32)
    p, m, v, _, _ = run_steps(p0, [g] * T, H)
    lr, eps, wd = Fraction(H.lr), Fraction(H.eps), Fraction(H.weight_decay)
    b1, b2 = Fraction(H.beta1), Fraction(H.beta2)
    a = 1 - lr * wd
    for i in range(g.size):
        gi, pi = Fraction(float(g[i])), Fraction(float(p0[i]))
        u = lr * gi / (abs(gi) + eps)
        want_p = pi * a ** T - u * (1 - a ** T) / (1 - a)
        assert abs(Fraction(p[i]) - want_p) <= abs(want_p) * Fraction(1, 10 ** 13)
        assert abs(Fraction(m[i]) - (1 - b1 ** T) * gi) <= abs(gi) * Fraction(1, 10 ** 14)
        assert abs(Fraction(v[i]) - (1 - b2 ** T) * gi * gi) <= gi * gi * Fraction(1, 10 ** 14)


@pytest.mark.parametrize("clip", [0.0, 0.5])
def test_matches_torch_adamw_float64(clip):
    # Without skip the page update is the textbook decoupled-decay Adam; with clipping it is that
    # preceded by the library's norm clipping of the page's gradient.
    n, T = 1000, 10
    p0 = (np.random.default_rng(5).standard_normal(n) * 0.02).astype(np.float32)
    scale = 1e-3 if clip == 0.0 else 0.05      # norm ~ 1.6 > 0.5: clipping is live
    grads = [some_bf16_values(n, 10 + t, scale) for t in range(T)]
    h = Hyper(max_grad_norm=clip)
    p, m, v, _, outs = run_steps(p0, grads, h)

    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([tp], lr=h.lr, betas=(h.beta1, h.beta2), eps=h.eps,
                            weight_decay=h.weight_decay, amsgrad=False)
    for t in range(T):
        tp.grad = torch.tensor(grads[t], dtype=torch.float64)
        if clip > 0:
            tot = torch.nn.utils.clip_grad_norm_([tp], clip)
            assert abs(float(tot) - float(outs[t][0])) <= 1e-6 * float(tot)
            assert float(tot) > clip
        opt.step()
    st = opt.state[tp]
    assert relerr(p, tp.detach().numpy()) < 1e-12
    assert relerr(m, st["exp_avg"].numpy()) < 1e-12
    assert relerr(v, st["exp_avg_sq"].numpy()) < 1e-12


def test_brute_force_three_elements_high_precision():
    # 3-element tensors, 4 steps, 50-digit decimal arithmetic written from Adam's recurrences.
    getcontext().prec = 50
    p0 = np.array([0.01, -0.03, 0.0], dtype=np.float32)
    grads = [np.array([1.0, -0.5, 0.25], dtype=np.float32) * np.float32(2.0 ** -10),
             np.array([-2.0, 0.0, 0.125], dtype=np.float32) * np.float32(2.0 ** -9),
             np.array([0.0, 0.0, 0.0], dtype=np.float32),
             np.array([3.0, 1.5, -0.75], dtype=np.float32) * np.float32(2.0 ** -11)]
    h = Hyper(max_grad_norm=2.0 ** -9)
    p, m, v, _, outs = run_steps(p0, grads, h)
    D = Decimal
    lr, b1, b2, eps, wd, c = (D(h.lr), D(h.beta1), D(h.beta2), D(h.eps), D(h.weight_decay),
                              D(h.max_grad_norm))
    P = [D(float(x)) for x in p0]
    M = [D(0)] * 3
    V = [D(0)] * 3
    for t, g in enumerate(grads, start=1):
        G = [D(float(x)) for x in g]
        norm = sum(x * x for x in G).sqrt()
        s = min(D(1), c / (norm + D("1e-6")))
        assert abs(D(float(outs[t - 1][0])) - norm) <= norm * D("1e-7")
        for i in range(3):
            gi = s * G[i]
            M[i] = b1 * M[i] + (1 - b1) * gi
            V[i] = b2 * V[i] + (1 - b2) * gi * gi
            mh = M[i] / (1 - b1 ** t)
            vh = V[i] / (1 - b2 ** t)
            P[i] = P[i] - lr * wd * P[i] - lr * mh / (vh.sqrt() + eps)
    for i in range(3):
        assert abs(D(float(p[i])) - P[i]) <= abs(P[i]) * D("1e-13")
        assert abs(D(float(m[i])) - M[i]) <= abs(M[i]) * D("1e-13") + D("1e-40")
        assert abs(D(float(v[i])) - V[i]) <= abs(V[i]) * D("1e-13") + D("1e-40")


def test_zero_gradient_dense_changes_only_by_decay():
    n = 100
    rng = np.random.default_rng(7)
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p = p0.astype(np.float64)
    m = np.zeros(n)
    v = np.abs(rng.standard_normal(n)) * 1e-8
    v0 = v.copy()
    p16 = np.zeros(n, dtype=np.uint16)
    norm, skip = oracle.page_adamw(p, m, v, p16, np.zeros(n, dtype=np.uint16), 3, H)
    assert not skip and norm == 0.0
    assert np.array_equal(p, p0.astype(np.float64) * (1.0 - H.lr * H.weight_decay))
    assert np.all(m == 0.0)
    assert np.array_equal(v, H.beta2 * v0)


def test_skip_mode_leaves_page_bits_untouched_and_mask_rules():
    n = 50
    rng = np.random.default_rng(8)
    h = Hyper(skip_mode=1)
    p = rng.standard_normal(n)
    m = rng.standard_normal(n)
    v = np.abs(rng.standard_normal(n))
    p16 = rng.integers(0, 65535, n).astype(np.uint16)
    before = [a.copy() for a in (p, m, v, p16)]
    g = np.zeros(n, dtype=np.uint16)
    g[7] = 0x8000                                   # -0 counts as zero
    norm, skip = oracle.page_adamw(p, m, v, p16, g, 5, h)
    assert skip and norm == 0.0
    for a, b in zip((p, m, v, p16), before):
        assert a.tobytes() == b.tobytes()
    g[9] = 0x0001                                   # smallest bf16 subnormal: not skipped
    norm, skip = oracle.page_adamw(p, m, v, p16, g, 5, h)
    assert not skip
    assert norm == np.float32(np.float64(2.0) ** -133)
    assert not np.array_equal(p, before[0])
    # brute-force any-nonzero on random sparse pages
    for s in range(20):
        g = np.zeros(n, dtype=np.uint16)
        k = rng.integers(0, 3)
        g[rng.integers(0, n, k)] = rng.choice([0x8000, 0x0000, 0x3C00, 0x8001], k)
        nz, _ = oracle.page_reduce(g)
        assert nz == any((int(x) & 0x7FFF) != 0 for x in g)


def test_padding_zero_stays_plus_zero():
    n = 16
    p = np.zeros(n)
    m = np.zeros(n)
    v = np.zeros(n)
    p16 = np.zeros(n, dtype=np.uint16)
    for t in range(1, 4):
        oracle.page_adamw(p, m, v, p16, np.zeros(n, dtype=np.uint16), t, Hyper(max_grad_norm=1.0))
    for a in (p, m, v):
        assert a.tobytes() == np.zeros(n).tobytes()          # +0, sign bit clear
    assert not p16.any()


def test_norm_of_constant_page_closed_form():
    for n, g0 in [(1, 0.5), (4096, 2.0 ** -10), (1000, -3.0 * 2.0 ** -12)]:
        g = np.full(n, g0, dtype=np.float32)
        nz, s = oracle.page_reduce(bf16_bits(g))
        assert nz
        assert abs(np.sqrt(s) - abs(g0) * np.sqrt(n)) <= 1e-14 * abs(g0) * np.sqrt(n)


def test_clip_inactive_is_bit_identical_and_active_rescales():
    n = 300
    p0 = (np.random.default_rng(9).standard_normal(n) * 0.02).astype(np.float32)
    g = some_bf16_values(n, 10)                      # norm ~ 0.017
    a = run_steps(p0, [g, g], Hyper())
    b = run_steps(p0, [g, g], Hyper(max_grad_norm=1.0))   # norm + 1e-6 <= 1: scale exactly 1
    for x, y in zip(a[:4], b[:4]):
        assert x.tobytes() == y.tobytes()
    # active clipping, first step: u = lr*s|g|/(s|g|+eps) with s = c/(norm+1e-6)
    c = 1e-3
    pc, mc, vc, _, outs = run_steps(p0, [g], Hyper(max_grad_norm=c))
    norm = float(np.sqrt(np.sum(g.astype(np.float64) ** 2)))
    s = c / (norm + 1e-6)
    assert s < 1
    gd = g.astype(np.float64)
    want = p0.astype(np.float64) * (1 - H.lr * H.weight_decay) - H.lr * s * gd / (s * np.abs(gd) + H.eps)
    assert relerr(pc, want) < 1e-13
    assert relerr(mc, (1 - H.beta1) * s * gd) < 1e-13
    assert relerr(vc[gd != 0], ((1 - H.beta2) * (s * gd) ** 2)[gd != 0]) < 1e-13


def test_step_zero_rejected():
    z = np.zeros(4)
    with pytest.raises(ValueError):
        oracle.page_adamw(z.copy(), z.copy(), z.copy(), np.zeros(4, np.uint16),
                          np.zeros(4, np.uint16), 0, H)


def test_p16_is_cast_of_master_and_f32_state_mode():
    n = 200
    p0 = (np.random.default_rng(11).standard_normal(n) * 0.02).astype(np.float32)
    grads = [some_bf16_values(n, 20 + t) for t in range(3)]
    p, m, v, p16, _ = run_steps(p0, grads, Hyper())
    want = torch.tensor(p.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(p16, want)
    p2, m2, v2, _, _ = run_steps(p0, grads, Hyper(round_state_f32=True))
    for a in (p2, m2, v2):
        assert np.array_equal(a, a.astype(np.float32).astype(np.float64))
    assert relerr(p2, p) < 1e-6


def test_update_is_elementwise_independent_of_paging():
    # Without clipping the result for an element does not depend on which page it sits in.
    n = 96
    p0 = (np.random.default_rng(12).standard_normal(n) * 0.02).astype(np.float32)
    grads = [some_bf16_values(n, 30 + t) for t in range(2)]
    whole = run_steps(p0, grads, Hyper())
    parts = [run_steps(p0[a:b], [g[a:b] for g in grads], Hyper()) for a, b in [(0, 40), (40, 96)]]
    for k in range(4):
        assert np.concatenate([parts[0][k], parts[1][k]]).tobytes() == whole[k].tobytes()


@pytest.mark.parametrize("clip", [0.0, 0.5])
@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
def test_non_finite_gradients_propagate_like_the_library_optimizer(clip, bad):
    # No special handling of inf / NaN gradients: plain IEEE propagation, as in torch's AdamW and
    # clip_grad_norm_ (an infinite norm gives scale 0, so inf * 0 = NaN and finite gradients vanish;
    # a NaN norm gives a NaN scale, which poisons the whole page).
    n = 64
    p0 = (np.random.default_rng(2).standard_normal(n) * 0.02).astype(np.float32)
    g1 = some_bf16_values(n, 3, 0.05)
    g1[5] = bad
    g2 = some_bf16_values(n, 4, 0.05)
    h = Hyper(max_grad_norm=clip)
    with np.errstate(all="ignore"):
        p, m, v, p16, outs = run_steps(p0, [g1, g2], h)
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([tp], lr=h.lr, betas=(h.beta1, h.beta2), eps=h.eps,
                            weight_decay=h.weight_decay, amsgrad=False)
    for g in (g1, g2):
        tp.grad = torch.tensor(g, dtype=torch.float64)
        if clip > 0:
            torch.nn.utils.clip_grad_norm_([tp], clip)
        opt.step()
    want = tp.detach().numpy()
    assert np.array_equal(np.isnan(p), np.isnan(want))
    ok = ~np.isnan(want)
    assert not ok.any() or relerr(p[ok], want[ok]) < 1e-12
    n_nan = int(np.isnan(want).sum())
    assert n_nan == (n if (clip > 0 and np.isnan(bad)) else 1)
    # the 16-bit copy of a NaN master is a NaN
    nan16 = (p16 & 0x7F80) == 0x7F80
    assert np.array_equal(nan16 & ((p16 & 0x7F) != 0), np.isnan(want))
