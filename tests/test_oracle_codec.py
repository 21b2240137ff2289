"""Pins for the oracle's low-bit transfer formats (run without a GPU)."""
import os

import numpy as np
import pytest
import torch

from oracle import codec

HERE = os.path.dirname(os.path.abspath(__file__))
TORCH = {"bf16": torch.bfloat16, "f16": torch.float16,
         "fp8_e4m3": torch.float8_e4m3fn, "fp8_e5m2": torch.float8_e5m2}
VIEW = {"bf16": torch.int16, "f16": torch.int16, "fp8_e4m3": torch.uint8, "fp8_e5m2": torch.uint8}


def test_fp8_spot_values_from_the_format_definition():
    with open(os.path.join(HERE, "golden", "fp8_spot_values.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for fmt, code, val in rows:
        got = float(codec.decode(np.array([int(code, 16)]), fmt)[0])
        assert got == float(val), (fmt, code, got)
    assert np.isnan(codec.decode(np.array([0x7F, 0xFF]), "fp8_e4m3")).all()
    assert np.isfinite(codec.decode(np.arange(0x7F), "fp8_e4m3")).all()        # no infinities


@pytest.mark.parametrize("fmt", ["bf16", "f16", "fp8_e4m3", "fp8_e5m2"])
def test_decode_table_matches_torch_cpu(fmt):
    n = 1 << (16 if fmt in ("bf16", "f16") else 8)
    codes = np.arange(n)
    if n == 65536:
        t = torch.from_numpy(codes.astype(np.int32)).to(torch.int16).view(TORCH[fmt]).to(torch.float64).numpy()
    else:
        t = torch.from_numpy(codes.astype(np.uint8)).view(TORCH[fmt]).to(torch.float64).numpy()
    ours = codec.decode(codes, fmt)
    assert np.array_equal(np.isnan(ours), np.isnan(t))
    ok = ~np.isnan(t)
    assert np.array_equal(ours[ok], t[ok])


@pytest.mark.parametrize("fmt", ["bf16", "f16", "fp8_e4m3", "fp8_e5m2"])
def test_encode_is_round_to_nearest_even_like_torch_cpu(fmt):
    rng = np.random.default_rng(0)
    vmax = {"bf16": 3e38, "f16": 65504.0, "fp8_e4m3": 448.0, "fp8_e5m2": 57344.0}[fmt]
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * 0.02,
        rng.standard_normal(100000).astype(np.float32),
        (rng.standard_normal(50000) * vmax / 6).astype(np.float32),
        np.float32(2.0) ** rng.integers(-30, 8, 20000).astype(np.float32) * rng.choice([1.0, 1.5, 1.25, 1.75], 20000).astype(np.float32),
        np.array([0.0, -0.0, vmax, -vmax], dtype=np.float32)])
    x = x[np.abs(x) <= vmax]                       # beyond that the 8-bit formats saturate by choice
    want = torch.from_numpy(x).to(TORCH[fmt]).to(torch.float64).numpy()
    got = codec.decode(codec.encode(x, fmt), fmt)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))


@pytest.mark.parametrize("fmt", ["bf16", "f16", "fp8_e4m3", "fp8_e5m2"])
def test_exact_midpoints_go_to_even(fmt):
    eb, mb = {"bf16": (8, 7), "f16": (5, 10), "fp8_e4m3": (4, 3), "fp8_e5m2": (5, 2)}[fmt]
    codes = np.arange(1, (1 << (eb + mb)) - (1 << mb) - 2)     # finite, below the top
    v = codec.decode(codes, fmt)
    nxt = codec.decode(codes + 1, fmt)
    ok = np.isfinite(v) & np.isfinite(nxt)
    mid = (v[ok] + nxt[ok]) / 2
    enc = codec.encode(mid, fmt).astype(np.int64)
    assert np.all(enc % 2 == 0)
    assert np.all((enc == codes[ok]) | (enc == codes[ok] + 1))
    # a value just above / below the midpoint goes to the nearer neighbour
    up = codec.encode(mid + (nxt[ok] - v[ok]) * 1e-3, fmt).astype(np.int64)
    dn = codec.encode(mid - (nxt[ok] - v[ok]) * 1e-3, fmt).astype(np.int64)
    assert np.array_equal(up, codes[ok] + 1) and np.array_equal(dn, codes[ok])


def test_overflow_rules_and_idempotence():
    assert float(codec.round_to(np.float32(1e6), "fp8_e4m3")) == 448.0        # saturates
    assert float(codec.round_to(np.float32(-1e9), "fp8_e5m2")) == -57344.0
    assert np.isinf(codec.round_to(np.float32(70000.0), "f16"))               # IEEE
    assert float(codec.round_to(np.float32(65519.0), "f16")) == 65504.0
    x = (np.random.default_rng(1).standard_normal(5000) * 0.05).astype(np.float32)
    for fmt in ("bf16", "f16", "fp8_e4m3", "fp8_e5m2"):
        once = codec.round_to(x, fmt)
        assert np.array_equal(codec.round_to(once, fmt), once)


TD = {"bf16": torch.bfloat16, "f16": torch.float16, "fp8_e4m3": torch.float8_e4m3fn, "fp8_e5m2": torch.float8_e5m2}


@pytest.mark.parametrize("fmt", ["bf16", "f16", "fp8_e4m3", "fp8_e5m2"])
def test_stochastic_rounding_brackets_and_is_unbiased(fmt):
    """Every outcome is one of the two representable neighbours of x (found with torch's CPU cast and its bit
    pattern, not with the oracle's table), the largest r16 truncates toward zero, a representable x never moves, and the
    mean over all 65536 values of r16 is x to within gap / 65536."""
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(40) * 0.3).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0, -0.375]                                          # representable in every format
    # neighbours from torch: nearest value, then step one code towards / away from zero
    t = torch.from_numpy(x).to(TD[fmt])
    bits = t.view(torch.uint8 if fmt.startswith("fp8") else torch.int16).to(torch.int32)
    mag = bits & (0x7F if fmt.startswith("fp8") else 0x7FFF)
    near = t.to(torch.float32).abs().numpy().astype(np.float64)
    def val(m):
        m = m.to(torch.uint8 if fmt.startswith("fp8") else torch.int16)
        return m.view(TD[fmt]).to(torch.float32).numpy().astype(np.float64)
    a = np.abs(x).astype(np.float64)
    lo = np.where(near > a, val(torch.clamp(mag - 1, min=0)), near)
    hi = np.where(near > a, near, np.where(near == a, near, val(mag + 1)))
    r_all = np.arange(65536)
    for i in range(x.size):
        out = codec.round_stochastic(np.full(65536, x[i], dtype=np.float32), fmt, r_all).astype(np.float64)
        assert set(np.unique(np.abs(out))) <= {lo[i], hi[i]}, (fmt, x[i])
        assert np.all(np.signbit(out) == np.signbit(x[i])) or a[i] == 0
        if hi[i] > lo[i] and (a[i] - lo[i]) / (hi[i] - lo[i]) <= 65535 / 65536:
            assert abs(out[65535]) == lo[i]                                    # largest r16: toward zero
        assert abs(out.mean() - x[i]) <= (hi[i] - lo[i]) / 65536 + 1e-300
        if lo[i] == hi[i]:
            assert np.all(out == x[i])
    # saturation and NaN
    big = np.finfo(np.float32).max                                            # above every format's largest finite value
    _, vals = codec._finite_table(fmt)
    assert float(codec.round_stochastic(big, fmt, 65535)) == float(np.float32(vals[-1]))
    assert np.isnan(codec.round_stochastic(np.float32("nan"), fmt, 7))


def test_stochastic_rounding_bf16_is_the_add_and_truncate_rule():
    """For bfloat16 the dropped 16 bits of the float32 pattern are the fraction itself: rounding up iff
    r16 < fraction is adding (65535 - r16) to the pattern and cutting the low half off."""
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(5000) * 0.05).astype(np.float32)
    r16 = rng.integers(0, 65536, size=x.size)
    bits = x.view(np.uint32).astype(np.uint64)
    want = (((bits + (65535 - r16).astype(np.uint64)) & np.uint64(0xFFFF0000)).astype(np.uint32)).view(np.float32)
    got = codec.round_stochastic(x, "bf16", r16)
    assert np.array_equal(got, want)
