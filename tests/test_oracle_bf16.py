"""Pins for the oracle's bf16 conversion: exhaustive agreement with torch's CPU cast (a library routine that
implements round-to-nearest-even independently) and the defining properties of RNE."""
import numpy as np
import torch


def _all_interesting_f32():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16            # every bf16 value, exactly representable
    lows = np.array([0x0000, 0x0001, 0x7fff, 0x8000, 0x8001, 0xffff], dtype=np.uint32)
    bits = (hi[:, None] | lows[None, :]).reshape(-1)
    return bits.view(np.float32)


def test_bf16_rne_matches_torch_exhaustively(oracle):
    x = _all_interesting_f32()
    got = oracle.bf16_rne(x)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.all(np.isnan(oracle.bf16_widen(got[nan])))       # NaN stays NaN, payload free


def test_bf16_exact_values_roundtrip(oracle):
    h = np.arange(1 << 16, dtype=np.uint16)
    f = oracle.bf16_widen(h)
    ok = ~np.isnan(f)
    assert np.array_equal(oracle.bf16_rne(f)[ok], h[ok])
    assert np.array_equal(f.view(np.uint32), h.astype(np.uint32) << 16)


def test_bf16_ties_go_to_even(oracle):
    # 1.0 = 0x3f80; next bf16 is 0x3f81.  Midpoint 0x3f808000 ties to the even 0x3f80;
    # midpoint above 0x3f81 (0x3f818000) ties to the even 0x3f82.
    x = np.array([0x3f808000, 0x3f818000, 0x3f808001, 0x3f807fff], dtype=np.uint32).view(np.float32)
    assert oracle.bf16_rne(x).tolist() == [0x3f80, 0x3f82, 0x3f81, 0x3f80]
    # rounding up across an exponent boundary and to infinity
    x = np.array([0x3fffffff, 0x7f7fffff], dtype=np.uint32).view(np.float32)
    assert oracle.bf16_rne(x).tolist() == [0x4000, 0x7f80]


def test_bf16_random_nearest(oracle):
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * 0.02).astype(np.float32)
    h = oracle.bf16_rne(x)
    back = oracle.bf16_widen(h).astype(np.float64)
    lo = oracle.bf16_widen((h - 1).astype(np.uint16)).astype(np.float64)
    hi = oracle.bf16_widen((h + 1).astype(np.uint16)).astype(np.float64)
    err = np.abs(back - x)
    assert np.all(err <= np.abs(lo - x)) and np.all(err <= np.abs(hi - x))
