"""Table 1 closed forms against the worked numbers the paper prints for GPT-3 175B."""
import os

import oracle


def test_gpt3_175b_worked_numbers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "gpt3_175b_footprint.txt"))
            if l.strip() and not l.startswith("#")]
    assert rows
    for layers, b, s, d, ffn, want_p, want_a, want_o in (map(int, r) for r in rows):
        p, a, o = oracle.layer_footprint_bytes(d, ffn, b, s)
        assert p * layers == want_p * 2 ** 30
        assert a * layers == want_a * 2 ** 30
        assert o * layers == want_o * 2 ** 30


def test_table1_rows_sum_to_totals():
    # Per-row entries of Table 1: QKV 12 d^2 / 36 d^2, out proj 4 d^2 / 12 d^2,
    # FFN 4 d dffn / 12 d dffn twice; totals 16 d^2 + 8 d dffn and 48 d^2 + 24 d dffn.
    d, ffn = 768, 3072
    p, _, o = oracle.layer_footprint_bytes(d, ffn, 1, 1)
    assert p == 12 * d * d + 4 * d * d + 2 * 4 * d * ffn == 16 * d * d + 8 * d * ffn
    assert o == 36 * d * d + 12 * d * d + 2 * 12 * d * ffn == 48 * d * d + 24 * d * ffn
    assert o == 3 * p
    half, full = oracle.model_state_bytes_per_param()
    assert (half, full) == (4, 12) and o // full == p // half
