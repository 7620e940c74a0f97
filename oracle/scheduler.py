"""ORACLE (test infrastructure): phase 1 of the life-time based scheduling algorithm (Alg. 1).

What the algorithm is for (Sec. 4.2, "Tensor Life-Time" and "Life-time based Scheduling"): the
model is a list of layers, every page has a trace -- here the index of the layer that accesses it
last, after which its GPU memory is free again -- and the GPU has a fixed amount of memory.  The
output is one list of tasks {operation, page or layer, trigger_id} that the executor walks in
order; a task may start once the compute task named by its trigger id has been reached.

How phase 1 gets there, as this build understands it: the plan starts out as optimistic as it can
be -- every page is brought to the GPU before anything computes -- and is then corrected layer by
layer.  A layer that does not fit next to everything the plan has on the GPU by then pushes the
*latest* planned movements back (they are the ones needed furthest in the future), onto a stack;
once the layer has computed and the pages that die with it are gone, the stack is unwound for as
long as more than one page of memory stays free, most recently deferred page first.  Phase 2 only
re-times all_gather tasks; on one GPU there are none, so it is left out.

Three things the paper does not say, and how they are read here:
  * size(l_i) is the memory the layer's computation needs besides its parameter pages;
  * the memory still available after a plan S (`get_available_memory`) is the GPU memory minus one
    page for every page that S moves in and whose last-access layer has no compute task in S yet;
  * a page of layer i that is still deferred when layer i's turn comes is brought in then, with
    trigger i, before the fit test (otherwise the layer would compute without it), and deferring a
    page that belongs to the current or an earlier layer is refused as out of memory (it is needed
    now, or is still alive, so no plan exists).
Each page belongs to exactly one layer's page_list (the layer of its first access).

The planner below keeps its memory account incrementally (`_Account`) and checks it, at every
layer, against `get_available_memory`, which is the definition evaluated on the task list itself.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence

MOVE_TO_GPU = "move_to_gpu"
COMPUTE = "compute"


@dataclass(frozen=True)
class Layer:
    page_list: Sequence[int]   # pages first accessed by this layer
    size: int                  # bytes the computation needs besides its pages


@dataclass(frozen=True)
class Task:
    operation: str
    target: int                # page (move_to_gpu) or layer index (compute)
    trigger_id: int


class OutOfMemory(Exception):
    pass


def get_available_memory(S: Sequence[Task], traces: Dict[int, int], gpu_memory: int, page_size: int) -> int:
    """Memory left once every task of S has run: moved-in pages stay until the compute of their
    last-access layer is part of S."""
    computed = {t.target for t in S if t.operation == COMPUTE}
    resident = [t.target for t in S if t.operation == MOVE_TO_GPU and traces[t.target] not in computed]
    return gpu_memory - page_size * len(resident)


class _Account:
    """Pages the plan has on the GPU, grouped by the layer whose compute releases them."""

    def __init__(self, traces: Dict[int, int], gpu_memory: int, page_size: int):
        self.traces, self.gpu_memory, self.page_size = traces, gpu_memory, page_size
        self.dies_with: Dict[int, set] = {}
        self.n_resident = 0

    def planned(self, page: int) -> None:
        self.dies_with.setdefault(self.traces[page], set()).add(page)
        self.n_resident += 1

    def deferred(self, page: int) -> None:
        self.dies_with[self.traces[page]].remove(page)
        self.n_resident -= 1

    def computed(self, layer: int) -> None:
        self.n_resident -= len(self.dies_with.pop(layer, ()))

    @property
    def available(self) -> int:
        return self.gpu_memory - self.page_size * self.n_resident


def schedule(model: Sequence[Layer], traces: Dict[int, int], gpu_memory: int, page_size: int) -> List[Task]:
    """Alg. 1, phase 1.  traces[page] = index of the layer that accesses the page last."""
    first_access = {page: i for i, layer in enumerate(model) for page in layer.page_list}
    account = _Account(traces, gpu_memory, page_size)
    S: List[Task] = []
    movements: List[int] = []       # positions in S of the movement tasks, in the order of S
    wait_stack: List[int] = []      # deferred pages; the most recently deferred one is on top

    def plan_move(page: int, trigger: int) -> None:
        movements.append(len(S))
        S.append(Task(MOVE_TO_GPU, page, trigger))
        account.planned(page)

    # the optimistic start: everything is on the GPU before the first layer computes
    for layer in model:
        for page in layer.page_list:
            plan_move(page, 0)

    for i, layer in enumerate(model):
        # pages of this very layer that are still deferred cannot wait any longer
        while wait_stack and first_access[wait_stack[-1]] == i:
            plan_move(wait_stack.pop(), i)
        # make room: the movement planned last is the one that can wait longest
        while account.available < layer.size:
            if not movements or first_access[S[movements[-1]].target] <= i:
                raise OutOfMemory(f"layer {i} does not fit")
            page = S.pop(movements.pop()).target
            # a movement is always the last task of S at this point or is followed by computes
            # only; removing it shifts those computes, whose positions nothing refers to
            account.deferred(page)
            wait_stack.append(page)
        assert account.available == get_available_memory(S, traces, gpu_memory, page_size)
        S.append(Task(COMPUTE, i, i))
        account.computed(i)
        # the layer's memory is free again: unwind the stack while more than a page stays free
        while wait_stack and account.available > page_size:
            plan_move(wait_stack.pop(), i)
        assert account.available == get_available_memory(S, traces, gpu_memory, page_size)
    return S
