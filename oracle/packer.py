"""ORACLE (test infrastructure): the page packer, written out as its definition.

Page abstraction (Sec. 4.1, "Page Abstraction" and the Page listing): a page has a total size, the
space still available, and at most two tenant tensors with their occupied sizes.  Tensors smaller
than a page take a page of their own ("Optimal Page Size", last paragraph); larger tensors are
arranged so that no page holds more than two of them.  A tensor is a list of pages, and merging
its pages back into one contiguous buffer (the Tensor listing's merge) is the inverse of packing.

The paper leaves the arrangement open; the deterministic rule used here is this build's reading:
  * tensors are placed in list order, E elements per page, second tenants start on a multiple of
    ALIGN elements;
  * numel == 0: no page;
  * 0 < numel < E: a fresh page, offset 0, and that page takes no second tenant;
  * numel >= E: if an open page exists (one tenant, free space left after alignment) the tensor
    starts there and the page is closed, else it starts a fresh page; it continues through fresh
    pages; if its last page is only partly filled that page becomes the open page;
  * unused elements are zero in every state class.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

ALIGN = 8


@dataclass
class Segment:
    tensor: int       # index in the tensor list
    tensor_off: int   # first element of the tensor covered by this segment
    page: int
    page_off: int     # first element of the page covered
    n: int            # elements


@dataclass
class PageEntry:
    used: int = 0                                  # end offset of the last occupied element
    tensor_id: List[int] = field(default_factory=lambda: [-1, -1])
    tensor_elems: List[int] = field(default_factory=lambda: [0, 0])

    def n_tenants(self) -> int:
        return sum(1 for t in self.tensor_id if t >= 0)


@dataclass
class PackPlan:
    page_elems: int
    segments: List[Segment]
    pages: List[PageEntry]
    total_elems: int

    @property
    def n_pages(self) -> int:
        return len(self.pages)

    @property
    def fragmentation(self) -> float:
        if not self.pages:
            return 0.0
        return 1.0 - self.total_elems / (self.n_pages * self.page_elems)

    def used(self) -> np.ndarray:
        return np.array([p.used for p in self.pages], dtype=np.int64)


def plan_pack(numels: Sequence[int], page_elems: int) -> PackPlan:
    E = int(page_elems)
    assert E > 0 and E % ALIGN == 0
    segments: List[Segment] = []
    pages: List[PageEntry] = []
    open_page = -1   # page index with one tenant and room for a second, or -1

    def place(t, t_off, page, p_off, n):
        e = pages[page]
        slot = e.n_tenants()
        assert slot < 2
        e.tensor_id[slot] = t
        e.tensor_elems[slot] = n
        e.used = p_off + n
        segments.append(Segment(t, t_off, page, p_off, n))

    for t, numel in enumerate(numels):
        numel = int(numel)
        assert numel >= 0
        if numel == 0:
            continue
        if numel < E:
            pages.append(PageEntry())
            place(t, 0, len(pages) - 1, 0, numel)
            continue
        done = 0
        if open_page >= 0:
            start = -(-pages[open_page].used // ALIGN) * ALIGN
            if start < E:
                n = E - start            # numel >= E > n: the tensor fills the page to its end
                place(t, 0, open_page, start, n)
                done = n
            open_page = -1
        while done < numel:
            n = min(E, numel - done)
            pages.append(PageEntry())
            place(t, done, len(pages) - 1, 0, n)
            done += n
            if n < E:
                open_page = len(pages) - 1
    return PackPlan(E, segments, pages, int(sum(int(x) for x in numels)))


def pack(plan: PackPlan, tensors: Sequence[np.ndarray], dtype) -> np.ndarray:
    """Copy the tensors' elements into a zero-filled [n_pages, E] array (bit copy)."""
    out = np.zeros((plan.n_pages, plan.page_elems), dtype=dtype)
    for s in plan.segments:
        src = tensors[s.tensor]
        assert src.dtype == out.dtype
        out[s.page, s.page_off:s.page_off + s.n] = src.reshape(-1)[s.tensor_off:s.tensor_off + s.n]
    return out


def unpack(plan: PackPlan, pages: np.ndarray, numels: Sequence[int]) -> List[np.ndarray]:
    """Inverse of pack: one contiguous array per tensor."""
    out = [np.zeros(int(n), dtype=pages.dtype) for n in numels]
    for s in plan.segments:
        out[s.tensor][s.tensor_off:s.tensor_off + s.n] = pages[s.page, s.page_off:s.page_off + s.n]
    return out
