"""Tensor shape lists of the synthetic workloads (shapes only; values come from synth.rng).

The lists stand in for the GPT / T5-MoE models the paper trains on a private corpus: the hot path
consumes only tensor sizes and gradient values, so a GPT-2-style layer layout at the configured
widths reproduces the ragged size mix (a few huge matrices, many tiny vectors) the paper's
tensor-size table shows for one GPT-3 layer.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from .rng import hash64_np


@dataclass(frozen=True)
class TensorSpec:
    id: int
    name: str
    numel: int
    expert: int = -1   # MoE: expert index within its layer, -1 for dense tensors
    layer: int = -1


def gpt_tensor_list(n_layer: int, d: int, ffn: int, vocab: int, n_ctx: int) -> List[TensorSpec]:
    """GPT-2-style decoder: token + position embeddings, per layer LN/qkv/proj/LN/fc/proj with
    biases, final LN; output head tied to the token embedding."""
    out: List[TensorSpec] = []

    def add(name, numel, layer=-1):
        out.append(TensorSpec(len(out), name, int(numel), -1, layer))

    add("wte", vocab * d)
    add("wpe", n_ctx * d)
    for l in range(n_layer):
        add(f"h{l}.ln1.w", d, l)
        add(f"h{l}.ln1.b", d, l)
        add(f"h{l}.attn.qkv.w", d * 3 * d, l)
        add(f"h{l}.attn.qkv.b", 3 * d, l)
        add(f"h{l}.attn.proj.w", d * d, l)
        add(f"h{l}.attn.proj.b", d, l)
        add(f"h{l}.ln2.w", d, l)
        add(f"h{l}.ln2.b", d, l)
        add(f"h{l}.mlp.fc.w", d * ffn, l)
        add(f"h{l}.mlp.fc.b", ffn, l)
        add(f"h{l}.mlp.proj.w", ffn * d, l)
        add(f"h{l}.mlp.proj.b", d, l)
    add("ln_f.w", d)
    add("ln_f.b", d)
    return out


def moe_tensor_list(n_layer: int, d: int, ffn: int, n_expert: int) -> List[TensorSpec]:
    """MoE stack: per layer LN x2, qkv w/b, proj w/b, router d x n_expert, and n_expert expert FFNs
    (W1 d x ffn, W2 ffn x d, no biases); no dense FFN."""
    out: List[TensorSpec] = []

    def add(name, numel, layer, expert=-1):
        out.append(TensorSpec(len(out), name, int(numel), expert, layer))

    for l in range(n_layer):
        add(f"h{l}.ln1.w", d, l)
        add(f"h{l}.ln1.b", d, l)
        add(f"h{l}.attn.qkv.w", d * 3 * d, l)
        add(f"h{l}.attn.qkv.b", 3 * d, l)
        add(f"h{l}.attn.proj.w", d * d, l)
        add(f"h{l}.attn.proj.b", d, l)
        add(f"h{l}.ln2.w", d, l)
        add(f"h{l}.ln2.b", d, l)
        add(f"h{l}.router.w", d * n_expert, l)
        for e in range(n_expert):
            add(f"h{l}.expert{e}.w1", d * ffn, l, e)
            add(f"h{l}.expert{e}.w2", ffn * d, l, e)
    return out


def moe_active_tensors(tensors: List[TensorSpec], step: int, seed: int, n_expert: int,
                       n_active: int) -> np.ndarray:
    """Boolean per tensor: does it receive a gradient at this step?  Dense tensors always do; per
    layer, n_active of n_expert experts (a seeded draw that changes every step) do."""
    n_layer = 1 + max(t.layer for t in tensors)
    active_expert = np.zeros((n_layer, n_expert), dtype=bool)
    for l in range(n_layer):
        keys = hash64_np(seed, 0x4D6F45000000 + step, l * n_expert, n_expert)
        active_expert[l, np.argsort(keys, kind="stable")[:n_active]] = True
    return np.array([t.expert < 0 or active_expert[t.layer, t.expert] for t in tensors], dtype=bool)


def tensor_offsets(tensors: List[TensorSpec]) -> np.ndarray:
    """Exclusive prefix sum of numel: the global element index of each tensor's first element."""
    off = np.zeros(len(tensors) + 1, dtype=np.int64)
    np.cumsum([t.numel for t in tensors], out=off[1:])
    return off


# name -> (tensor list factory, elements per page)
WORKLOADS = {
    # 8 full pages of 262144 elements, one tensor
    "cfg1_8pages": (lambda: [TensorSpec(0, "flat", 8 * 262144)], 262144),
    # 1024 completely full pages, one tensor: no fragmentation (a kernel-tuning reference point)
    "flat_1024pages": (lambda: [TensorSpec(0, "flat", 1024 << 20)], 1 << 20),
    "gpt2_small_124m": (lambda: gpt_tensor_list(12, 768, 3072, 50257, 1024), 1 << 20),
    "gpt_1p3b": (lambda: gpt_tensor_list(24, 2048, 8192, 50257, 2048), 1 << 20),
    "gpt_13b": (lambda: gpt_tensor_list(40, 5120, 20480, 50257, 2048), 1 << 20),
    "moe_8x64": (lambda: moe_tensor_list(8, 1024, 4096, 64), 1 << 20),
}
