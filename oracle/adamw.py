"""ORACLE (test infrastructure): ctypes front end of page_adamw.c plus a multi-page state holder.

The arithmetic lives in page_adamw.c; this file only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

_lib = None


class _CHyper(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("max_grad_norm", C.c_double),
                ("skip_mode", C.c_int32), ("round_state_f32", C.c_int32)]


@dataclass
class Hyper:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    max_grad_norm: float = 0.0   # <= 0: off
    skip_mode: int = 0           # 0 dense, 1 untouched-if-all-zero
    round_state_f32: bool = False

    def _c(self) -> _CHyper:
        return _CHyper(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay,
                       self.max_grad_norm, self.skip_mode, int(self.round_state_f32))


def lib():
    global _lib
    if _lib is None:
        # ORACLE_LIBRARY: another build of page_adamw.c (the mutation test loads damaged copies
        # this way to show that the pins catch them; it never edits the tracked source)
        L = C.CDLL(os.environ.get("ORACLE_LIBRARY") or _build.build())
        L.oracle_bf16_rne.restype = C.c_uint16
        L.oracle_bf16_rne.argtypes = [C.c_uint32]
        L.oracle_bf16_rne_array.restype = None
        L.oracle_bf16_rne_array.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.oracle_page_reduce.restype = None
        L.oracle_page_reduce.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_int32),
                                         C.POINTER(C.c_double)]
        L.oracle_page_adamw.restype = C.c_int
        L.oracle_page_adamw.argtypes = [C.c_void_p] * 5 + [C.c_int64, C.c_int64,
                                                           C.POINTER(_CHyper),
                                                           C.POINTER(C.c_float),
                                                           C.POINTER(C.c_uint8)]
        _lib = L
    return _lib


def _ptr(a: np.ndarray, dtype) -> int:
    assert a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    return a.ctypes.data


def bf16_rne(f32_bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of fp32 bit patterns (uint32), round to nearest even."""
    f32_bits = np.ascontiguousarray(f32_bits, dtype=np.uint32)
    out = np.empty(f32_bits.shape, dtype=np.uint16)
    lib().oracle_bf16_rne_array(f32_bits.ctypes.data, out.ctypes.data, f32_bits.size)
    return out


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64 (no arithmetic: a bit placement)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def page_reduce(g16: np.ndarray):
    """(any_nonzero, sum of squares in double) of one page's used gradient elements."""
    nz, s = C.c_int32(0), C.c_double(0.0)
    lib().oracle_page_reduce(_ptr(g16, np.uint16), g16.size, C.byref(nz), C.byref(s))
    return bool(nz.value), s.value


def page_adamw(p: np.ndarray, m: np.ndarray, v: np.ndarray, p16: np.ndarray, g16: np.ndarray,
               t: int, h: Hyper):
    """One step on one page's used extent, in place.  Returns (fp32 grad norm, skipped)."""
    n = p.size
    assert m.size == n and v.size == n and p16.size == n and g16.size == n
    norm, skip = C.c_float(0.0), C.c_uint8(0)
    ch = h._c()
    rc = lib().oracle_page_adamw(_ptr(p, np.float64), _ptr(m, np.float64), _ptr(v, np.float64),
                                 _ptr(p16, np.uint16), _ptr(g16, np.uint16), n, t, C.byref(ch),
                                 C.byref(norm), C.byref(skip))
    if rc != 0:
        raise ValueError("step must be >= 1")
    return np.float32(norm.value), bool(skip.value)


class PagedAdamWState:
    """Double-precision p/m/v and bf16 p16 for a set of pages, each with its used extent.

    pages are rows of [n_pages, E] arrays; only [0, used[k]) of row k is ever touched.
    """

    def __init__(self, p32_pages: np.ndarray, used: Sequence[int], p16_pages: Optional[np.ndarray] = None):
        assert p32_pages.dtype == np.float32 and p32_pages.ndim == 2
        self.n_pages, self.E = p32_pages.shape
        self.used = np.asarray(used, dtype=np.int64)
        self.p = p32_pages.astype(np.float64)
        self.m = np.zeros_like(self.p)
        self.v = np.zeros_like(self.p)
        self.p16 = (np.zeros(p32_pages.shape, dtype=np.uint16) if p16_pages is None
                    else p16_pages.copy())

    def step(self, g16_pages: np.ndarray, t: int, h: Hyper, pages: Optional[Sequence[int]] = None,
             threads: int = 1):
        """Apply one step to the listed pages (default all).  Returns (norms fp32, skip uint8),
        indexed like `pages`.  Pages are independent, so `threads` > 1 only spreads whole pages
        over host threads; the per-page arithmetic is unchanged."""
        assert g16_pages.dtype == np.uint16 and g16_pages.shape == self.p.shape
        idx = list(range(self.n_pages) if pages is None else pages)

        def one(k):
            n = int(self.used[k])
            return page_adamw(self.p[k, :n], self.m[k, :n], self.v[k, :n], self.p16[k, :n],
                              g16_pages[k, :n], t, h)

        if threads > 1 and len(idx) > 1:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=threads) as ex:
                res = list(ex.map(one, idx))
        else:
            res = [one(k) for k in idx]
        norms = np.array([r[0] for r in res], dtype=np.float32)
        skips = np.array([int(r[1]) for r in res], dtype=np.uint8)
        return norms, skips
