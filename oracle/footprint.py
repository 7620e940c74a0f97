"""ORACLE (test infrastructure): the per-layer memory-footprint closed forms of Table 1
(mixed-precision training with Adam), used to check the pool's byte accounting.

Per Transformer layer, ignoring the small tensors as the table's Total row does:
  Params = 16 d^2 + 8 d d_ffn bytes      (16-bit parameter + 16-bit gradient = 4 B per weight)
  Acts   = 40 b s d + 8 b s d_ffn bytes
  Optims = 48 d^2 + 24 d d_ffn bytes     (fp32 master, momentum, variance = 12 B per weight)
"""
from __future__ import annotations


def layer_footprint_bytes(d: int, d_ffn: int, b: int, s: int):
    weights = 4 * d * d + 2 * d * d_ffn           # QKV (3 d^2) + out proj (d^2) + two FFN matrices
    params = 4 * weights
    acts = 40 * b * s * d + 8 * b * s * d_ffn
    optims = 12 * weights
    return params, acts, optims


def model_state_bytes_per_param():
    """(16-bit classes, fp32 classes): p16 + g16, and p32 + m32 + v32."""
    return 2 + 2, 4 + 4 + 4
