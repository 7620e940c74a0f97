"""The oracle packer against a hand-worked layout, the page invariants the paper states, brute
force over boundary sizes, and the pack -> unpack identity."""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth

E = 64


def seg_tuples(plan):
    return [(s.tensor, s.tensor_off, s.page, s.page_off, s.n) for s in plan.segments]


def test_hand_worked_layout():
    # E = 64.  numels: 150 (large), 10 (small), 100 (large), 64 (exactly one page), 3 (small), 70.
    #  t0: pages 0,1 full; page 2 holds 22            -> open page 2 (used 22)
    #  t1: small -> page 3 alone; page 2 stays open
    #  t2: starts in page 2 at align8(22) = 24, takes 40; remaining 60 -> page 4 (used 60), open
    #  t3: numel == E is "large": starts in page 4 at align8(60) = 64 = E -> no room, page 4 closed;
    #      fresh page 5, full; nothing open
    #  t4: small -> page 6
    #  t5: 70 -> page 7 full, page 8 holds 6 (open)
    plan = oracle.plan_pack([150, 10, 100, 64, 3, 70], E)
    assert seg_tuples(plan) == [
        (0, 0, 0, 0, 64), (0, 64, 1, 0, 64), (0, 128, 2, 0, 22),
        (1, 0, 3, 0, 10),
        (2, 0, 2, 24, 40), (2, 40, 4, 0, 60),
        (3, 0, 5, 0, 64),
        (4, 0, 6, 0, 3),
        (5, 0, 7, 0, 64), (5, 64, 8, 0, 6),
    ]
    assert plan.n_pages == 9
    assert [p.used for p in plan.pages] == [64, 64, 64, 10, 60, 64, 3, 64, 6]
    assert plan.pages[2].tensor_id == [0, 2] and plan.pages[2].tensor_elems == [22, 40]
    assert plan.pages[3].tensor_id == [1, -1]
    assert plan.fragmentation == pytest.approx(1 - 397 / (9 * 64))


def read_worked_layout(path):
    E, numels, segs, pages, total = None, None, [], [], None
    for line in open(path):
        w = line.split()
        if not w or w[0].startswith("#"):
            continue
        if w[0] == "E":
            E = int(w[1])
        elif w[0] == "numels":
            numels = [int(x) for x in w[1:]]
        elif w[0] == "seg":
            segs.append(tuple(int(x) for x in w[1:]))
        elif w[0] == "page":
            pages.append(tuple(int(x) for x in w[1:]))
        elif w[0] == "total":
            total = int(w[1])
    return E, numels, segs, pages, total


def test_second_hand_worked_layout_two_handovers_in_a_row_and_a_page_aligned_tail(golden_dir):
    # worked on paper (the file says how): an open page handed from tensor to tensor twice in a
    # row, an empty tensor, a small tensor that must not close the open page, numel == E starting
    # inside an open page, and a tensor whose end falls exactly on a page end (no open page after)
    Ew, numels, segs, pages, total = read_worked_layout(os.path.join(golden_dir, "packer_worked_layout_two_handovers.txt"))
    plan = oracle.plan_pack(numels, Ew)
    assert seg_tuples(plan) == segs
    assert plan.n_pages == len(pages) == 12
    got = [(p.used, p.tensor_id[0], p.tensor_id[1], p.tensor_elems[0], p.tensor_elems[1]) for p in plan.pages]
    assert got == pages
    assert plan.total_elems == total == sum(numels)
    assert plan.fragmentation == pytest.approx(1 - total / (12 * Ew))
    check_invariants(numels, plan)


def check_invariants(numels, plan):
    Ep = plan.page_elems
    covered = [0] * len(numels)
    per_page = {}
    for s in plan.segments:
        assert s.n > 0 and 0 <= s.page < plan.n_pages
        assert s.page_off % oracle.packer.ALIGN == 0 and s.page_off + s.n <= Ep
        assert s.tensor_off == covered[s.tensor]             # segments of a tensor are in order
        covered[s.tensor] += s.n
        per_page.setdefault(s.page, []).append(s)
    assert covered == list(numels)
    assert sorted(per_page) == list(range(plan.n_pages))      # every page is used
    for page, segs in per_page.items():
        assert len(segs) <= 2                                  # at most two tensors per page
        segs.sort(key=lambda s: s.page_off)
        if len(segs) == 2:
            assert segs[0].page_off + segs[0].n <= segs[1].page_off   # no overlap
            assert segs[0].tensor != segs[1].tensor
        for s in segs:
            if numels[s.tensor] < Ep:                          # a small tensor owns its page
                assert len(segs) == 1 and s.page_off == 0
        e = plan.pages[page]
        assert e.used == max(s.page_off + s.n for s in segs) <= Ep
        assert sorted(t for t in e.tensor_id if t >= 0) == sorted(s.tensor for s in segs)
    # pages of one tensor are consecutive except that the first may be an earlier open page
    assert plan.total_elems == sum(numels)
    assert plan.fragmentation == pytest.approx(1 - sum(numels) / (plan.n_pages * Ep)) if plan.n_pages else True


def test_boundary_sizes_brute_force():
    sizes = [0, 1, 7, 8, E - 1, E, E + 1, 2 * E, 2 * E + 3, 3 * E - 8]
    for numels in itertools.product(sizes, repeat=3):
        plan = oracle.plan_pack(list(numels), E)
        check_invariants(list(numels), plan)
        # a dense lower bound and the one-page-per-small-tensor upper bound
        total = sum(numels)
        assert plan.n_pages >= -(-total // E)
        assert plan.n_pages <= sum(-(-n // E) for n in numels)


@pytest.mark.parametrize("name,pages,frag_pct", [
    ("cfg1_8pages", 8, 0.0), ("gpt2_small_124m", 223, 46.78), ("gpt_1p3b", 1449, 13.40),
    ("gpt_13b", 12578, 2.54), ("moe_8x64", 4184, 1.32)])
def test_workload_plans(name, pages, frag_pct):
    factory, Ep = synth.WORKLOADS[name]
    numels = [t.numel for t in factory()]
    plan = oracle.plan_pack(numels, Ep)
    check_invariants(numels, plan)
    assert plan.n_pages == pages
    assert round(100 * plan.fragmentation, 2) == pytest.approx(frag_pct, abs=0.006)


def test_pack_unpack_identity_and_zero_padding():
    rng = np.random.default_rng(0)
    numels = [150, 10, 100, 64, 3, 70, 0, 129]
    plan = oracle.plan_pack(numels, E)
    for dtype in (np.uint32, np.uint16):
        tensors = [rng.integers(1, np.iinfo(dtype).max, n).astype(dtype) for n in numels]
        pages = oracle.pack(plan, tensors, dtype)
        back = oracle.unpack(plan, pages, numels)
        for a, b in zip(tensors, back):
            assert a.tobytes() == b.tobytes()
        mask = np.zeros(pages.shape, dtype=bool)
        for s in plan.segments:
            mask[s.page, s.page_off:s.page_off + s.n] = True
        assert not pages[~mask].any()                          # padding is zero
        assert int(mask.sum()) == sum(numels)
