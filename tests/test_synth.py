"""The seeded input generator: host and torch back ends agree bit for bit, slices regenerate alone,
and the distribution has the stated moments."""
import numpy as np
import torch

import synth


def test_numpy_and_torch_backends_bit_identical():
    a = synth.normal_f32(3, 11, 10 ** 12 + 5, 100000, 0.02)
    b = synth.normal_f32(3, 11, 10 ** 12 + 5, 100000, 0.02, device="cpu").numpy()
    assert a.tobytes() == b.tobytes()
    g = synth.normal_bf16(3, 12, 77, 100000, 1e-3)
    gt = synth.normal_bf16(3, 12, 77, 100000, 1e-3, device="cpu")
    assert gt.dtype == torch.bfloat16
    assert g.tobytes() == gt.view(torch.int16).numpy().tobytes()


def test_slices_regenerate_alone_and_streams_differ():
    full = synth.normal_f32(0, 1, 1000, 5000, 1.0)
    part = synth.normal_f32(0, 1, 1000 + 1234, 100, 1.0)
    assert full[1234:1334].tobytes() == part.tobytes()
    other = synth.normal_f32(0, 2, 1000, 5000, 1.0)
    assert abs(np.corrcoef(full, other)[0, 1]) < 0.05
    assert synth.normal_f32(1, 1, 1000, 5000, 1.0).tobytes() != full.tobytes()


def test_moments():
    x = synth.normal_f32(0, 5, 0, 1 << 20, 0.02).astype(np.float64)
    assert abs(x.mean()) < 1e-4 and abs(x.std() - 0.02) < 2e-4
    k = ((x / x.std()) ** 4).mean()
    assert abs(k - 3.0) < 0.05
    g = synth.normal_bf16(0, 6, 0, 1 << 18, 1e-3)
    gf = (g.astype(np.uint32) << 16).view(np.float32)
    assert abs(gf.std() - 1e-3) < 2e-5


def test_workload_shapes_and_moe_activity():
    counts = {k: (len(f()), sum(t.numel for t in f())) for k, (f, _) in synth.WORKLOADS.items()}
    assert counts["gpt2_small_124m"] == (148, 124439808)
    assert counts["gpt_1p3b"] == (292, 1315723264)
    assert counts["gpt_13b"] == (484, 12853386240)
    assert counts["moe_8x64"] == (1096, 4329111552)
    tl = synth.WORKLOADS["moe_8x64"][0]()
    a3 = synth.moe_active_tensors(tl, 3, 0, 64, 8)
    a4 = synth.moe_active_tensors(tl, 4, 0, 64, 8)
    dense = sum(1 for t in tl if t.expert < 0)
    assert a3.sum() == dense + 8 * 8 * 2 and not np.array_equal(a3, a4)
    assert np.array_equal(a3, synth.moe_active_tensors(tl, 3, 0, 64, 8))
    off = synth.tensor_offsets(tl)
    assert off[-1] == 4329111552 and off[1] == tl[0].numel
