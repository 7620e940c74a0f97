"""What a phase-1 schedule of Alg. 1 (life-time based scheduling) guarantees, checked on a finished
task list without running any planner: the list is *valid* (every page moved once, before the layer
that first needs it, memory never exceeded, layers in order, everything released) and it is *the
greedy one* -- no movement sits later than the algorithm's two rules allow, and none sits earlier.

Tasks are (operation, target, trigger_id) with operation "move" or "compute"; `layers` is a list of
(page_list, size); `last_access[page]` is the layer whose compute releases the page.

The two rules, in terms of avail(n, c) = memory - page_bytes * (pages among the first n of the page
sequence that are still alive once c layers have computed):
  * before layer j computes, movements are deferred from the end of the sequence while
    avail < size_j (so the next page, had it been planned too, would have left less than size_j --
    at this layer or at a later one that took the plan back this far);
  * after layer j-1 has computed, deferred movements are planned again while avail > one page, with
    trigger j-1; a page of layer j that is still deferred then is planned on demand, trigger j.
"""
MOVE, COMPUTE = "move", "compute"


def check_valid(S, layers, last_access, memory, page_bytes):
    owner = {p: i for i, (pl, _) in enumerate(layers) for p in pl}
    resident, moved, peak, n_compute, last_trigger = set(), set(), 0, 0, 0
    for op, target, trigger in S:
        assert trigger >= last_trigger, "trigger ids run backwards"
        last_trigger = trigger
        if op == MOVE:
            assert target not in moved, "page moved twice"
            assert trigger <= owner[target], "a move is triggered after the layer that needs it"
            moved.add(target)
            resident.add(target)
            assert len(resident) * page_bytes <= memory, "a move overfills the memory"
        else:
            assert target == n_compute and trigger == target, "layers compute in order"
            assert set(layers[target][0]) <= resident, "a page of the layer is not on the GPU"
            need = len(resident) * page_bytes + layers[target][1]
            assert need <= memory, "compute overfills the memory"
            peak = max(peak, need)
            resident -= {p for p in resident if last_access[p] == target}
            n_compute += 1
    assert n_compute == len(layers) and moved == set(owner), "not every layer computed or page moved"
    assert not resident, "a page outlives its last access"
    return peak


def check_greedy(S, layers, last_access, memory, page_bytes):
    order = [p for pl, _ in layers for p in pl]
    owner = {p: i for i, (pl, _) in enumerate(layers) for p in pl}
    P = len(order)

    def avail(n, c):
        return memory - page_bytes * sum(1 for p in order[:n] if last_access[p] >= c)

    moves = [t for t in S if t[0] == MOVE]
    assert [t[1] for t in moves] == order, "movements are not in the order of the layers' page lists"
    # K[j] = movements ahead of compute j; gap[x] = number of computes ahead of the x-th movement
    K, gap, n_moves, n_compute = [], [], 0, 0
    for op, _, _ in S:
        if op == MOVE:
            gap.append(n_compute)
            n_moves += 1
        else:
            K.append(n_moves)
            n_compute += 1
    # not later than allowed: where the plan stops short of everything, some layer from here on
    # (with the same prefix planned) is the reason
    for j, k in enumerate(K):
        if k == P:
            continue
        reasons = [jj for jj in range(j, len(K)) if K[jj] == k and
                   (avail(k + 1, jj) < layers[jj][1] or (jj >= 1 and avail(k, jj) <= page_bytes))]
        assert reasons, f"page {order[k]} could have been moved before layer {j} computes"
    # not earlier than allowed, and with the trigger of the rule that planned it
    for x, (_, page, trigger) in enumerate(moves):
        j = gap[x]
        if j == 0:
            assert trigger == 0, "a movement of the optimistic start carries trigger 0"
        elif avail(x, j) > page_bytes:
            assert trigger == j - 1, f"page {page}: planned again after layer {j - 1}, trigger {trigger}"
        else:
            assert owner[page] == j and trigger == j, f"page {page} is moved although at most one page is free"


def check(S, layers, last_access, memory, page_bytes):
    peak = check_valid(S, layers, last_access, memory, page_bytes)
    check_greedy(S, layers, last_access, memory, page_bytes)
    return peak
