"""GPU parity: random stream (bit exact) and the fused update + perturb kernel, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import codec, philox

pytestmark = pytest.mark.gpu

# |z_gpu - z_oracle|: the hardware log2 / sqrt are 1-ulp operations (relative 2^-23 on rho <= 4.71) and the hardware
# sin / cos, whose argument u2 is exact, are good to ~2^-22 absolute, times rho: below 2e-6 (measured maximum 4.8e-7)
Z_TOL = 2e-6


def _b():
    from paper_2503_12668_amd import binding
    return binding


@pytest.mark.parametrize("seed,tid,e0,n", [
    (42, 0, 0, 4099),
    (42, 5, 6, 1000),
    ((0xABCDEF01 << 32) | 0x13572468, 77, (1 << 34) + 3, 2051),      # both halves of seed and element index
    (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, (1 << 40) - 17, 300),
    (7, 3, 0, 0),
])
def test_philox_words_bit_exact(seed, tid, e0, n):
    b = _b()
    got = b.op_philox_words(seed, tid, e0, n).cpu().numpy().view(np.uint32)
    want = philox.random_words(seed, tid, e0, n).astype(np.uint32) if n else np.zeros(0, np.uint32)
    assert np.array_equal(got, want)


def test_gaussian_matches_oracle():
    b = _b()
    n = 1 << 20
    got = b.op_gaussian(42, 9, 0, n).cpu().numpy()
    want = philox.gaussian(42, 9, 0, n)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    print("max |dz| =", err.max(), "mean =", err.mean())
    assert err.max() < Z_TOL
    off = b.op_gaussian(42, 9, 1001, 77).cpu().numpy()
    assert np.array_equal(off, got[1001:1078])


WIRE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16,
        "fp8_e4m3": torch.float8_e4m3fn, "fp8_e5m2": torch.float8_e5m2}


def _oracle_k1(theta32, tid, e0, pending, seed_prev, c, seed, eps, wire, compute, scale):
    """The oracle's per-element arithmetic (zo_step canonical form) on a window."""
    from oracle.zo_step import _fma32, _store
    n = theta32.size
    th = theta32
    if pending:
        th = _store(_fma32(np.float32(-c), philox.gaussian(seed_prev, tid, e0, n), th), wire, scale)
    z = philox.gaussian(seed, tid, e0, n)
    wp = _store(_fma32(np.float32(eps), z, th), compute)
    wm = _store(_fma32(np.float32(-eps), z, th), compute)
    return th, wp, wm


@pytest.mark.parametrize("wire,compute,scale", [
    ("f32", "f32", 1.0), ("bf16", "bf16", 1.0), ("f16", "f16", 1.0), ("f32", "bf16", 1.0), ("bf16", "f32", 1.0),
    ("fp8_e4m3", "bf16", 64.0), ("fp8_e5m2", "bf16", 1.0), ("f16", "bf16", 1.0),
])
@pytest.mark.parametrize("pending", [False, True])
def test_update_perturb_window(wire, compute, scale, pending):
    b = _b()
    rng = np.random.default_rng(3)
    n, e0, tid = 3 * 8192 + 2048 + 5, 16 * 1000, 37           # several chunks, ragged tail
    raw = (rng.standard_normal(n) * 0.02).astype(np.float32)
    theta0 = codec.round_to(raw.astype(np.float64) * scale, wire) / np.float32(scale) if wire != "f32" else raw
    theta0 = theta0.astype(np.float32)
    c, eps = np.float32(3e-3 * 1.7), np.float32(1e-3)
    th_o, wp_o, wm_o = _oracle_k1(theta0, tid, e0, pending, 41, c, 42, eps, wire, compute, scale)

    t_dev = (torch.from_numpy(theta0) * scale).to(WIRE[wire]).cuda()
    assert np.array_equal((t_dev.float().cpu().numpy() / np.float32(scale)), theta0)
    wp = torch.zeros(n, dtype=WIRE[compute], device="cuda")
    wm = torch.zeros(n, dtype=WIRE[compute], device="cuda")
    b.op_update_perturb(t_dev, wp, wm, tid, e0, pending, 41, float(c), 42, float(eps), scale=scale)
    torch.cuda.synchronize()
    th_g = t_dev.float().cpu().numpy() / np.float32(scale)
    wp_g, wm_g = wp.float().cpu().numpy(), wm.float().cpu().numpy()

    # z differs by <= Z_TOL between the two sides, so values agree up to that times the multiplier
    # (all that is left of a result where theta and eps z cancel), plus - where that nudges a value
    # across a rounding boundary - one unit of the storage format
    def close(got, want, mult, fmt):
        d = np.abs(got.astype(np.float64) - want.astype(np.float64))
        if fmt == "f32":
            return bool(np.all(d <= mult * Z_TOL + np.spacing(np.abs(want).astype(np.float32))))
        step = np.abs(codec.round_to(np.abs(want) * 1.01 + 1e-30, fmt) - codec.round_to(np.abs(want) * 0.99, fmt)).astype(np.float64)
        step = np.maximum(step, {"f16": 2.0 ** -24, "fp8_e4m3": 2.0 ** -9, "fp8_e5m2": 2.0 ** -16}.get(fmt, 1e-12))   # subnormal spacing
        frac_exact = np.mean(d == 0)
        return bool(np.all(d <= mult * Z_TOL + step / (scale if fmt.startswith("fp8") else 1.0))) and frac_exact > 0.98

    if pending:
        assert close(th_g, th_o, float(c), wire)
    else:
        assert np.array_equal(th_g, theta0)
    assert close(wp_g, wp_o, float(eps) + float(c), compute)
    assert close(wm_g, wm_o, float(eps) + float(c), compute)


def test_update_only_and_small_windows():
    b = _b()
    for n in (1, 7, 8, 9, 2040, 2048, 2049, 4095, 8192, 8193):
        raw = (np.random.default_rng(n).standard_normal(n) * 0.02).astype(np.float32)
        t = torch.from_numpy(raw.copy()).cuda()
        b.op_update_perturb(t, None, None, 3, 0, True, 5, 1e-3, 0, 0.0)
        from oracle.zo_step import _fma32
        want = _fma32(np.float32(-1e-3), philox.gaussian(5, 3, 0, n), raw)
        # z error times c, plus one float32 rounding of the result
        assert np.all(np.abs(t.cpu().numpy() - want) <= 1e-3 * Z_TOL + np.spacing(np.abs(want)))
    # n = 0 is a no-op
    t = torch.zeros(8, device="cuda")
    b.op_update_perturb(t, None, None, 3, 0, True, 5, 1e-3, 0, 0.0, n=0)
    assert float(t.abs().sum()) == 0.0
    with pytest.raises(b.Zo2Error):
        b.op_update_perturb(t, None, None, 3, 4, True, 5, 1e-3, 0, 0.0)       # e0 not a multiple of 8


def test_convert_matches_oracle_codec():
    b = _b()
    x = (np.random.default_rng(0).standard_normal(100003) * 0.05).astype(np.float32)
    x[:4] = [0.0, -0.0, 500.0, -1e9]
    src = torch.from_numpy(x).cuda()
    for fmt in ("bf16", "f16", "fp8_e4m3", "fp8_e5m2"):
        dst = torch.empty(x.size, dtype=WIRE[fmt], device="cuda")
        b.op_convert(src, dst)
        back = torch.empty(x.size, dtype=torch.float32, device="cuda")
        b.op_convert(dst, back)
        got_codes = dst.view(torch.uint8 if fmt.startswith("fp8") else torch.int16).cpu().numpy()
        want_codes = codec.encode(x, fmt)
        assert np.array_equal(got_codes.view(want_codes.dtype), want_codes), fmt
        assert np.array_equal(back.cpu().numpy(), codec.decode(want_codes, fmt).astype(np.float32)), fmt
    # scaled 8-bit: stored = round(x * 64); decoded = stored / 64
    dst = torch.empty(x.size, dtype=WIRE["fp8_e4m3"], device="cuda")
    b.op_convert(src, dst, 1.0, 64.0)
    want = codec.encode(x.astype(np.float64) * 64.0, "fp8_e4m3")
    assert np.array_equal(dst.view(torch.uint8).cpu().numpy(), want)


@pytest.mark.parametrize("fmt", ["fp8_e4m3", "fp8_e5m2"])
def test_8bit_conversions_exhaustively_against_the_oracle_codec(fmt):
    """The kernels convert the 8-bit formats with the hardware's instructions: every one of the 256 codes decodes as the
    oracle's table says, and the encoder agrees with the oracle on every representable value, every midpoint between
    neighbours (ties to even), the float32 neighbours of every midpoint, the subnormal range, values beyond the largest
    finite one (saturation), infinities and NaN."""
    b = _b()
    codes = np.arange(256, dtype=np.uint8)
    dec = codec.decode(codes, fmt).astype(np.float32)
    back = torch.empty(256, dtype=torch.float32, device="cuda")
    b.op_convert(torch.from_numpy(codes).cuda().view(WIRE[fmt]), back)
    got = back.cpu().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(dec)) and np.array_equal(got[~np.isnan(dec)], dec[~np.isnan(dec)])
    assert np.array_equal(np.signbit(got[~np.isnan(dec)]), np.signbit(dec[~np.isnan(dec)]))
    fin = np.sort(dec[np.isfinite(dec)].astype(np.float64))
    mids = (fin[1:] + fin[:-1]) / 2
    pts = np.concatenate([fin, mids]).astype(np.float32)
    pts = np.concatenate([pts, np.nextafter(pts, np.float32(np.inf)), np.nextafter(pts, np.float32(-np.inf))])
    top = float(fin[-1])
    extra = np.array([top * 1.01, top * 1.07, top * 2, 1e30, -top * 1.01, -1e30, np.inf, -np.inf, 1e-30, -1e-30, 1e-45, 0.0, -0.0], dtype=np.float32)
    rng = np.random.default_rng(3)
    rnd = (rng.standard_normal(200000) * np.exp(rng.uniform(-12, 8, 200000))).astype(np.float32)
    x = np.concatenate([pts, extra, rnd])
    dst = torch.empty(x.size, dtype=WIRE[fmt], device="cuda")
    b.op_convert(torch.from_numpy(x).cuda(), dst)
    want = codec.encode(x, fmt)
    gotc = dst.view(torch.uint8).cpu().numpy()
    bad = np.nonzero(gotc != want)[0]
    assert bad.size == 0, (x[bad[:8]], gotc[bad[:8]], want[bad[:8]])
    xn = np.array([np.nan, -np.nan], dtype=np.float32)
    dn = torch.empty(2, dtype=WIRE[fmt], device="cuda")
    b.op_convert(torch.from_numpy(xn).cuda(), dn)
    assert np.all(np.isnan(codec.decode(dn.view(torch.uint8).cpu().numpy(), fmt)))


def test_w_plus_only_and_zero_eps():
    """The single-forward pass writes W+ alone; with eps = 0 it is theta' in the compute format."""
    b = _b()
    n = 2 * 8192 + 77
    raw = (np.random.default_rng(5).standard_normal(n) * 0.02).astype(np.float32)
    t1, t2, t3 = (torch.from_numpy(raw.copy()).cuda() for _ in range(3))
    wp1 = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    wm1 = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    wp2 = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    b.op_update_perturb(t1, wp1, wm1, 9, 64, True, 41, 2e-3, 42, 1e-3)
    b.op_update_perturb(t2, wp2, None, 9, 64, True, 41, 2e-3, 42, 1e-3)
    torch.cuda.synchronize()
    assert torch.equal(wp1, wp2) and torch.equal(t1, t2)
    wp3 = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    b.op_update_perturb(t3, wp3, None, 9, 64, True, 41, 2e-3, 42, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(t3, t1) and torch.equal(wp3, t3.to(torch.bfloat16))
    with pytest.raises(b.Zo2Error):
        b.op_update_perturb(t3, None, wm1, 9, 64, True, 41, 2e-3, 42, 1e-3)       # W- without W+


@pytest.mark.parametrize("wire,scale", [("bf16", 1.0), ("f16", 1.0), ("fp8_e4m3", 64.0), ("fp8_e5m2", 1.0)])
def test_update_with_stochastic_rounding_matches_oracle(wire, scale):
    """theta' stored with stochastic rounding: same neighbour as the oracle wherever z's 4e-6 tolerance cannot move
    the decision, one code apart otherwise; and the codes differ from round-to-nearest in a good share of elements."""
    b = _b()
    rng = np.random.default_rng(8)
    n, e0, tid = 2 * 8192 + 1000 + 3, 8 * 555, 21
    raw = (rng.standard_normal(n) * 0.02).astype(np.float32)
    theta0 = (codec.round_to(raw.astype(np.float64) * scale, wire) / np.float32(scale)).astype(np.float32)
    c = np.float32(2.5e-4)
    from oracle.zo_step import _fma32, _store
    r16 = philox.rounding_bits(41, tid, e0, n)
    want = _store(_fma32(np.float32(-c), philox.gaussian(41, tid, e0, n), theta0), wire, scale, r16)
    nearest = _store(_fma32(np.float32(-c), philox.gaussian(41, tid, e0, n), theta0), wire, scale)
    t_dev = (torch.from_numpy(theta0) * scale).to(WIRE[wire]).cuda()
    b.op_update_perturb(t_dev, None, None, tid, e0, True, 41, float(c), 0, 0.0, scale=scale, stochastic=True)
    torch.cuda.synchronize()
    got = t_dev.float().cpu().numpy() / np.float32(scale)
    same = got == want
    print(wire, "identical", same.mean(), "differs from nearest", (want != nearest).mean())
    assert same.mean() > 0.995
    step = np.abs(codec.round_to(np.abs(want) * 1.01 + 1e-30, wire) - codec.round_to(np.abs(want) * 0.99, wire)).astype(np.float64)
    step = np.maximum(step, {"f16": 2.0 ** -24, "fp8_e4m3": 2.0 ** -9, "fp8_e5m2": 2.0 ** -16}.get(wire, 1e-12)) / scale
    assert np.all(np.abs(got.astype(np.float64) - want) <= step * 1.01 + 1e-12)
    assert (want != nearest).mean() > 0.05
    # the stored values are representable: rounding them again changes nothing
    assert np.array_equal(codec.round_to(got.astype(np.float64) * scale, wire) / np.float32(scale), got)
