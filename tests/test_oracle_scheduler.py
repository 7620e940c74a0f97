"""Pins for the oracle's phase-1 scheduler (Alg. 1): hand-worked schedules, an independent replay
of the schedule against the memory budget, a check of the finished task list against the
algorithm's two placement rules (no movement later or earlier than they allow), special cases, and
brute force on feasibility."""
import itertools
import os
import random

import pytest

from oracle import scheduler as sch
import schedule_properties as props

HERE = os.path.dirname(os.path.abspath(__file__))


def parse_layers(text):
    layers = []
    for part in text.split(";"):
        pages, size = part.split("/")
        layers.append(sch.Layer([int(p) for p in pages.split(",") if p != ""], int(size)))
    return layers


def tokens(S):
    return " ".join(f"m{t.target}@{t.trigger_id}" if t.operation == sch.MOVE_TO_GPU else f"c{t.target}" for t in S)


def as_tuples(S):
    return [(props.MOVE if t.operation == sch.MOVE_TO_GPU else props.COMPUTE, t.target, t.trigger_id) for t in S]


def own_layer_traces(model):
    return {p: i for i, l in enumerate(model) for p in l.page_list}


def test_hand_worked_examples_from_alg1():
    cases, expect = {}, {}
    for line in open(os.path.join(HERE, "golden", "scheduler_worked_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, rest = line.split(None, 1)
        if rest.startswith("expect"):
            expect[name] = rest.split(None, 1)[1].strip()
        else:
            kv = dict(x.split("=") for x in rest.split())
            cases[name] = (int(kv["gpu_memory"]), parse_layers(kv["layers"]))
    assert sorted(cases) == ["A", "B", "C", "D"]
    for name, (mem, model) in cases.items():
        S = sch.schedule(model, own_layer_traces(model), mem, 1)
        assert tokens(S) == expect[name], name


def replay(S, model, traces, gpu_memory, page_size):
    """Independent check of a schedule: walk it in order with a set of resident pages.  Every page
    is moved exactly once and before the compute that first needs it; at each compute the resident
    pages plus the layer's own need fit into the memory; trigger ids never run backwards, and a
    move's trigger is the layer being scheduled when it was appended: the latest compute before it
    (refill) or the next one (on demand), never later than the layer that needs the page."""
    owner = {p: i for i, l in enumerate(model) for p in l.page_list}
    resident, moved, peak, last_compute, n_compute, last_trigger = set(), set(), 0, 0, 0, 0
    for t in S:
        assert t.trigger_id >= last_trigger, "trigger ids run backwards"
        last_trigger = t.trigger_id
        if t.operation == sch.MOVE_TO_GPU:
            assert t.target not in moved, "page moved twice"
            assert t.trigger_id in (last_compute, n_compute) and t.trigger_id <= owner[t.target]
            moved.add(t.target)
            resident.add(t.target)
            assert len(resident) * page_size <= gpu_memory, "a move overfills the memory"
        else:
            i = t.target
            assert i == n_compute and t.trigger_id == i, "layers compute in order"
            assert set(model[i].page_list) <= resident, "a page of the layer is not on the GPU"
            need = len(resident) * page_size + model[i].size
            assert need <= gpu_memory, "compute overfills the memory"
            peak = max(peak, need)
            resident -= {p for p in resident if traces[p] == i}
            last_compute, n_compute = i, n_compute + 1
    assert n_compute == len(model) and moved == set(traces)
    assert not resident, "every page is released by its last access"
    return peak


def feasible(model, traces, gpu_memory, page_size):
    """A schedule exists iff every layer fits together with what must be resident with it: its own
    pages and the pages of earlier layers that are accessed again at or after it."""
    for i, l in enumerate(model):
        alive = sum(1 for j in range(i) for p in model[j].page_list if traces[p] >= i)
        if (alive + len(l.page_list)) * page_size + l.size > gpu_memory:
            return False
    return True


def random_model(rng, n_layers, max_pages, max_size, reuse):
    model, page = [], 0
    for _ in range(n_layers):
        k = rng.randint(0, max_pages)
        model.append(sch.Layer(list(range(page, page + k)), rng.randint(0, max_size)))
        page += k
    traces = {}
    for i, l in enumerate(model):
        for p in l.page_list:
            traces[p] = rng.randint(i, len(model) - 1) if reuse and rng.random() < 0.3 else i
    return model, traces


@pytest.mark.parametrize("reuse", [False, True])
def test_schedules_replay_within_memory_and_fail_exactly_when_nothing_fits(reuse):
    rng = random.Random(7 + reuse)
    n_ok = n_oom = 0
    for _ in range(600):
        page_size = rng.choice([1, 4])
        model, traces = random_model(rng, rng.randint(1, 7), 4, 6, reuse)
        gpu_memory = rng.randint(0, 30)
        try:
            S = sch.schedule(model, traces, gpu_memory, page_size)
        except sch.OutOfMemory:
            assert not feasible(model, traces, gpu_memory, page_size)
            n_oom += 1
            continue
        assert feasible(model, traces, gpu_memory, page_size)
        peak = replay(S, model, traces, gpu_memory, page_size)
        assert props.check(as_tuples(S), [(l.page_list, l.size) for l in model], traces, gpu_memory, page_size) == peak
        n_ok += 1
    assert n_ok > 100 and n_oom > 100


def test_enough_memory_moves_everything_first_and_tight_memory_moves_late():
    model = [sch.Layer([0, 1], 2), sch.Layer([2], 1), sch.Layer([3, 4, 5], 0)]
    traces = own_layer_traces(model)
    S = sch.schedule(model, traces, 1000, 10)
    assert tokens(S) == "m0@0 m1@0 m2@0 m3@0 m4@0 m5@0 c0 c1 c2"
    # the least memory any schedule can do with: the largest layer (3 pages) -- nothing is
    # prefetched beyond what the one-page margin of the refill rule allows
    S = sch.schedule(model, traces, 30, 10)
    assert tokens(S) == "m0@0 m1@0 c0 m2@0 m3@0 c1 m4@1 m5@2 c2"
    assert replay(S, model, traces, 30, 10) == 30
    with pytest.raises(sch.OutOfMemory):
        sch.schedule(model, traces, 29, 10)


def test_available_memory_counts_pages_until_their_last_access():
    traces = {0: 0, 1: 2, 2: 1}
    S = [sch.Task(sch.MOVE_TO_GPU, 0, 0), sch.Task(sch.MOVE_TO_GPU, 1, 0), sch.Task(sch.COMPUTE, 0, 0)]
    assert sch.get_available_memory(S, traces, 10, 3) == 7          # page 0 released, page 1 kept
    S += [sch.Task(sch.MOVE_TO_GPU, 2, 0), sch.Task(sch.COMPUTE, 1, 1)]
    assert sch.get_available_memory(S, traces, 10, 3) == 7          # page 2 released, page 1 still kept
    S += [sch.Task(sch.COMPUTE, 2, 2)]
    assert sch.get_available_memory(S, traces, 10, 3) == 10


def test_planted_mistakes_are_caught():
    """The replay and the worked examples must notice a wrong schedule: drop the on-demand move,
    release too early, refill without the margin."""
    model = parse_layers("0,1/0;2,3/0")
    traces = own_layer_traces(model)
    good = sch.schedule(model, traces, 2, 1)
    bad = [t for t in good if not (t.operation == sch.MOVE_TO_GPU and t.target == 3)]
    with pytest.raises(AssertionError):
        replay(bad, model, traces, 2, 1)
    swapped = [good[0], good[1], good[3], good[2]] + good[4:]      # a move ahead of the compute that frees its memory
    with pytest.raises(AssertionError):
        replay(swapped, model, traces, 2, 1)


def test_a_valid_schedule_that_is_not_the_greedy_one_is_caught():
    """The placement check must notice a movement that sits later or earlier than the two rules
    allow although the schedule stays within memory, and a wrong trigger id."""
    layers = [([0, 1], 0), ([2, 3], 0), ([4], 0)]
    model = [sch.Layer(pl, sz) for pl, sz in layers]
    traces = own_layer_traces(model)
    good = as_tuples(sch.schedule(model, traces, 4, 1))
    assert " ".join(f"m{t}@{g}" if o == props.MOVE else f"c{t}" for o, t, g in good) == \
        "m0@0 m1@0 m2@0 m3@0 c0 m4@0 c1 c2"
    props.check(good, layers, traces, 4, 1)
    def variant(text):
        out = []
        for tok in text.split():
            if tok[0] == "m":
                page, trig = tok[1:].split("@")
                out.append((props.MOVE, int(page), int(trig)))
            else:
                out.append((props.COMPUTE, int(tok[1:]), int(tok[1:])))
        return out
    for wrong in ("m0@0 m1@0 m2@0 c0 m3@0 m4@0 c1 c2",       # page 3 fits before layer 0 and is held back
                  "m0@0 m1@0 m2@0 m3@0 c0 c1 m4@1 c2",       # page 4 held back past a point with two pages free
                  "m0@0 m1@0 m2@0 m3@0 c0 m4@1 c1 c2",       # right place, trigger of the wrong rule
                  "m0@0 m1@0 m3@0 m2@0 c0 m4@0 c1 c2"):      # out of page order
        props.check_valid(variant(wrong), layers, traces, 4, 1)          # all of them stay within memory
        with pytest.raises(AssertionError):
            props.check_greedy(variant(wrong), layers, traces, 4, 1)
    # the refill rule's margin: with exactly one page free nothing is planned again (page 3 waits
    # for its own layer); planning it right after layer 0 is valid, but not the algorithm's plan
    layers = [([0, 1], 0), ([2, 3], 0)]
    traces = {0: 0, 1: 0, 2: 1, 3: 1}
    props.check(variant("m0@0 m1@0 c0 m2@0 m3@1 c1"), layers, traces, 2, 1)
    props.check_valid(variant("m0@0 m1@0 c0 m2@0 m3@0 c1"), layers, traces, 2, 1)
    with pytest.raises(AssertionError):
        props.check_greedy(variant("m0@0 m1@0 c0 m2@0 m3@0 c1"), layers, traces, 2, 1)
