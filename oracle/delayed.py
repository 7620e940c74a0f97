"""ORACLE (test infrastructure): one-step-stale form of the lock-free update.

Follows Alg. 2 reduced to one GPU with no SSD and no forward/backward: the updating actor applies
the *buffered* gradient g' ("Update p32, m32, v32 via g'16"), then the buffer is cleared and the
16-bit parameters are refreshed by the cast; a newly produced gradient is accumulated into the
cleared buffer (0 + g = g exactly, one gradient per update).  Each call applies the gradient handed
over by the previous call; a call without a gradient flushes the buffer.

A buffered gradient carries the hyper-parameters and the page list of the call that handed it over:
it is the gradient of that iteration, so it is applied with that iteration's learning rate, decay
and clipping even though the update runs one call later (otherwise N calls plus a flush would not
equal N synchronous steps under a learning-rate schedule).  The hyper-parameters of the applying
call, and of a flush, belong to the gradient that call brings (none for a flush).
"""
from __future__ import annotations

from dataclasses import replace
from typing import Optional, Sequence

import numpy as np

from .adamw import Hyper, PagedAdamWState


class DelayedStepper:
    def __init__(self, state: PagedAdamWState):
        self.state = state
        self.buffered: Optional[np.ndarray] = None   # g' (bf16 bits), None = empty
        self.buffered_h: Optional[Hyper] = None       # hyper-parameters handed over with g'
        self.buffered_pages: Optional[Sequence[int]] = None
        self.applied = 0                              # number of updates applied so far

    def step(self, new_g16_pages: Optional[np.ndarray], h: Hyper,
             pages: Optional[Sequence[int]] = None):
        """Returns (norms, skips) of the update applied by this call, or None if none was."""
        out = None
        if self.buffered is not None:
            self.applied += 1
            out = self.state.step(self.buffered, self.applied, self.buffered_h, self.buffered_pages)
        if new_g16_pages is None:
            self.buffered = self.buffered_h = self.buffered_pages = None
        else:
            self.buffered = new_g16_pages.copy()
            self.buffered_h = replace(h)      # a copy: the caller may change its own object
            self.buffered_pages = None if pages is None else list(pages)
        return out

    def accumulate(self, g16_pages: np.ndarray) -> None:
        """Buffering actor of Alg. 2: g' <- g' + g in 16-bit.  The sum of the two bf16 values is
        formed in fp32 (round to nearest) and rounded to bf16 (nearest even)."""
        if self.buffered is None:
            raise RuntimeError("no gradient is being collected")
        from .adamw import bf16_rne
        a = (self.buffered.astype(np.uint32) << np.uint32(16)).view(np.float32)
        b = (g16_pages.astype(np.uint32) << np.uint32(16)).view(np.float32)
        with np.errstate(over="ignore", invalid="ignore"):
            s = (a + b).astype(np.float32)
        self.buffered = bf16_rne(s.view(np.uint32)).reshape(self.buffered.shape)
