"""One-step-stale stepping: N delayed calls plus a flush equal N synchronous steps bit for bit,
and before the flush the state equals N-1 synchronous steps."""
import numpy as np

import oracle


def make(seed, n_pages=3, Ep=32):
    rng = np.random.default_rng(seed)
    p32 = (rng.standard_normal((n_pages, Ep)) * 0.02).astype(np.float32)
    used = [Ep, 20, 5]
    return p32, used


def grads(seed, T, shape):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(T):
        a = (rng.standard_normal(shape) * 1e-3).astype(np.float32)
        out.append((a.view(np.uint32) >> 16).astype(np.uint16))
    out[2][1, :] = 0     # a page without gradient at one step
    return out


def state_bytes(st):
    return b"".join(a.tobytes() for a in (st.p, st.m, st.v, st.p16))


def test_delayed_plus_flush_equals_sync():
    T = 6
    h = oracle.Hyper(max_grad_norm=0.004, skip_mode=1)
    p32, used = make(0)
    gs = grads(1, T, p32.shape)

    sync = oracle.PagedAdamWState(p32, used)
    snaps = [state_bytes(sync)]
    for t in range(T):
        sync.step(gs[t], t + 1, h)
        snaps.append(state_bytes(sync))

    st = oracle.PagedAdamWState(p32, used)
    d = oracle.DelayedStepper(st)
    for t in range(T):
        out = d.step(gs[t], h)
        assert (out is None) == (t == 0)
        assert state_bytes(st) == snaps[t]          # one step behind the synchronous run
        assert d.applied == t
    d.step(None, h)                                  # flush
    assert state_bytes(st) == snaps[T] and d.applied == T
    assert d.step(None, h) is None                   # nothing left to flush
    assert state_bytes(st) == snaps[T]


def test_gradient_is_applied_with_the_hyper_and_page_list_it_came_with():
    """A learning-rate / decay / clip schedule and a page list that changes from call to call: the
    gradient of call t is applied (during call t+1) with call t's values, so N calls plus a flush
    still equal N synchronous steps; the values passed with a flush are not used."""
    T = 6
    p32, used = make(6)
    gs = grads(7, T, p32.shape)
    hs = [oracle.Hyper(lr=1e-4 * (t + 1), weight_decay=0.01 * (t % 3), max_grad_norm=0.002 * (t + 1))
          for t in range(T)]
    lists = [None, [0, 2], [1], None, [2, 0, 1], [0]]

    sync = oracle.PagedAdamWState(p32, used)
    snaps = [state_bytes(sync)]
    for t in range(T):
        sync.step(gs[t], t + 1, hs[t], lists[t])
        snaps.append(state_bytes(sync))
    assert len(set(snaps)) == T + 1

    st = oracle.PagedAdamWState(p32, used)
    d = oracle.DelayedStepper(st)
    for t in range(T):
        h = oracle.Hyper(**vars(hs[t]))
        d.step(gs[t], h, lists[t])
        h.lr = 123.0                                  # the caller's object is its own again
        assert state_bytes(st) == snaps[t]
    d.step(None, oracle.Hyper(lr=7.0, weight_decay=0.5))   # flush: its values belong to no gradient
    assert state_bytes(st) == snaps[T]


def test_buffered_gradient_is_a_copy():
    p32, used = make(2)
    st = oracle.PagedAdamWState(p32, used)
    d = oracle.DelayedStepper(st)
    g = grads(3, 3, p32.shape)[0]
    d.step(g, oracle.Hyper())
    keep = g.copy()
    g[:] = 0                                         # the producer reuses its buffer
    d.step(None, oracle.Hyper())
    ref = oracle.PagedAdamWState(p32, used)
    ref.step(keep, 1, oracle.Hyper())
    assert state_bytes(st) == state_bytes(ref)


def test_accumulate_matches_library_bf16_addition_and_sums_before_the_update():
    import torch
    rng = np.random.default_rng(5)
    p32, used = make(4)
    st = oracle.PagedAdamWState(p32, used)
    d = oracle.DelayedStepper(st)
    shape = p32.shape
    def rand_bits(scale):
        a = (rng.standard_normal(shape) * scale).astype(np.float32)
        return (a.view(np.uint32) >> 16).astype(np.uint16)
    g1, g2, g3 = rand_bits(1e-3), rand_bits(1e-3), rand_bits(3e-1)
    g2[0, :4] = [0x0001, 0x8001, 0x7F7F, 0x0080]        # subnormals, largest finite, smallest normal
    g1[0, :4] = [0x0001, 0x0001, 0x7F7F, 0x8080]
    d.step(g1, oracle.Hyper())
    d.accumulate(g2)
    d.accumulate(g3)
    tb = lambda bits: torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    want = ((tb(g1) + tb(g2)) + tb(g3)).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(d.buffered, want)
    # the accumulated gradient is what the next call applies
    d.step(None, oracle.Hyper())
    ref = oracle.PagedAdamWState(p32, used)
    ref.step(want, 1, oracle.Hyper())
    assert state_bytes(st) == state_bytes(ref)
    import pytest
    with pytest.raises(RuntimeError):
        d.accumulate(g1)
