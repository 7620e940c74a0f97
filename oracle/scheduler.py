"""ORACLE (test infrastructure): phase 1 of the life-time based scheduling algorithm (Alg. 1).

Alg. 1 takes the model as a list of layers, the trace of each tensor (here: of each page -- the
logical id of the layer that accesses it last, after which its GPU memory is free again,
Sec. 4.2 "Tensor Life-Time"), and the GPU memory, and produces a list of tasks
{operation, page or layer, trigger_id}.  Phase 1: every page's move_to_gpu is put at the start of
the schedule; then, layer by layer, movement tasks are taken off the end of the schedule while the
memory left is less than the layer needs, the layer's compute is appended, and deferred pages are
put back (most recently deferred first) while more than one page of memory is left.  Phase 2 only
re-times all_gather tasks; on one GPU there are none, so it does nothing and is left out.

The steps below follow the listing's order and its notation (S, wait_stack,
get_available_memory).  Where the listing is silent, this build reads it as follows:
  * size(l_i) is the memory the layer's computation needs besides its parameter pages;
  * get_available_memory(S, traces) is the GPU memory minus one page for every page that S moves
    in and whose last-access layer has no compute task in S yet;
  * a page of l_i that is still on the wait_stack when l_i's turn comes is moved on demand: its
    move_to_gpu is appended with trigger i before the memory check (the listing would otherwise
    compute a layer whose page never arrived);
  * taking a movement task off S is refused (OutOfMemory) when the page belongs to the current
    or an earlier layer: those pages are needed now or are still alive, so no schedule exists.
Each page belongs to exactly one layer's page_list (the layer of its first access).
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


def schedule(model: Sequence[Layer], traces: Dict[int, int], gpu_memory: int, page_size: int) -> List[Task]:
    """Alg. 1, phase 1.  traces[page] = index of the layer that accesses the page last."""
    owner = {page: i for i, l in enumerate(model) for page in l.page_list}
    S: List[Task] = []
    wait_stack: List[int] = []
    for l_i in model:
        for page in l_i.page_list:
            S.append(Task(MOVE_TO_GPU, page, 0))
    for i, l_i in enumerate(model):
        while wait_stack and owner[wait_stack[-1]] == i:          # on demand (reading, see above)
            S.append(Task(MOVE_TO_GPU, wait_stack.pop(), i))
        while get_available_memory(S, traces, gpu_memory, page_size) < l_i.size:
            last = max((k for k, t in enumerate(S) if t.operation == MOVE_TO_GPU), default=None)
            if last is None or owner[S[last].target] <= i:
                raise OutOfMemory(f"layer {i} does not fit")
            wait_stack.append(S.pop(last).target)
        S.append(Task(COMPUTE, i, i))
        while wait_stack and get_available_memory(S, traces, gpu_memory, page_size) > page_size:
            S.append(Task(MOVE_TO_GPU, wait_stack.pop(), i))
    return S
