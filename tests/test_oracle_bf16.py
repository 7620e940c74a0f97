"""The fp32 -> bf16 cast of the oracle against the library cast and against the definition of
round-to-nearest-even (nearest representable neighbour, ties to the even mantissa)."""
import numpy as np
import torch

import oracle


def torch_cast(bits_u32):
    t = torch.from_numpy(bits_u32.view(np.float32).copy())
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def patterns():
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = np.array([0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000, 0x1234], dtype=np.uint32)
    grid = (hi[:, None] | lows[None, :]).reshape(-1)
    rng = np.random.default_rng(0)
    rnd = rng.integers(0, 2 ** 32, 1 << 22, dtype=np.uint64).astype(np.uint32)
    return np.concatenate([grid, rnd])


def test_matches_library_cast_on_non_nan():
    u = patterns()
    f = u.view(np.float32)
    ok = ~np.isnan(f)
    got = oracle.bf16_rne(u)
    assert np.array_equal(got[ok], torch_cast(u)[ok])


def test_nan_stays_nan_with_sign():
    u = patterns()
    nan = np.isnan(u.view(np.float32))
    got = oracle.bf16_rne(u[nan])
    assert np.all((got & 0x7F80) == 0x7F80) and np.all((got & 0x007F) != 0)
    assert np.array_equal(got >> 15, (u[nan] >> 31).astype(np.uint16))


def test_is_nearest_even_by_brute_force():
    rng = np.random.default_rng(1)
    u = rng.integers(0, 2 ** 32, 200000, dtype=np.uint64).astype(np.uint32)
    u = np.concatenate([u, np.array([0x3F808000, 0x3F818000, 0x3F80FFFF, 0x7F7FFFFF, 0x00008000,
                                     0x80008000, 0x7F7F8000], dtype=np.uint32)])
    f = u.view(np.float32)
    keep = np.isfinite(f)
    u, x = u[keep], f[keep].astype(np.float64)
    lo_bits = (u >> 16).astype(np.uint16)                     # truncation: neighbour toward zero
    hi_bits = (lo_bits + np.uint16(1)).astype(np.uint16)      # next magnitude up (may be inf)
    lo = oracle.bf16_bits_to_f64(lo_bits)
    hi = oracle.bf16_bits_to_f64(hi_bits)
    hi_mag = np.where(np.isinf(hi), np.ldexp(1.0, 128) * np.sign(hi), hi)  # inf acts as 2^128
    d_lo, d_hi = np.abs(x - lo), np.abs(hi_mag - x)
    want = np.where(d_lo < d_hi, lo_bits, np.where(d_hi < d_lo, hi_bits,
                    np.where((lo_bits & 1) == 0, lo_bits, hi_bits)))
    assert np.array_equal(oracle.bf16_rne(u), want.astype(np.uint16))


def test_matches_library_cast_on_every_fp32_pattern():
    """All 2^32 fp32 bit patterns, in 64 chunks: the oracle's cast equals the library's on every
    non-NaN pattern, and every NaN stays a NaN of the same sign."""
    chunk = 1 << 26
    for c in range(64):
        u = np.arange(c * chunk, (c + 1) * chunk, dtype=np.uint64).astype(np.uint32)
        got = oracle.bf16_rne(u)
        nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        want = torch_cast(u)
        if nan.any():
            assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x007F) != 0)
            assert np.array_equal(got[nan] >> 15, (u[nan] >> 31).astype(np.uint16))
            got[nan] = 0
            want[nan] = 0
        assert np.array_equal(got, want), f"chunk {c}"
