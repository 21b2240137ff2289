"""Oracle (test infrastructure): the low-bit transfer formats of AMP mode.

Sec. 5.5: parameters travel between host and device compressed to bfloat16 or
float16 (half the bytes of float32) or to an 8-bit float (a quarter), and are
decompressed to float32 on the device for the update.  The formats are written
out from their definitions:

  bf16     1-8-7,  bias 127, IEEE infinities / NaN
  f16      1-5-10, bias 15,  IEEE infinities / NaN
  fp8_e5m2 1-5-2,  bias 15,  IEEE infinities / NaN
  fp8_e4m3 1-4-3,  bias 7,   no infinity, S.1111.111 is NaN, largest finite 448
                             (the OCP 8-bit floating point "E4M3" definition)

decode() evaluates sign * 2^(E-bias) * (1 + M/2^m) (or the subnormal form) for a
code.  encode() returns the code of the representable value nearest to x, ties
going to the code with an even mantissa; magnitudes beyond the largest finite
value saturate to it in the 8-bit formats and follow IEEE (round to infinity)
in the 16-bit ones.  It is a search over the table of all codes, not a bit
trick.

round_stochastic() is the rounding that lets a low-bit master copy move by steps
far below its spacing (the paper rounds to nearest, which returns theta unchanged
when eta * g * z is under half a unit in the last place; Sec. 5.5 leaves the
rounding open): x goes to one of the two representable values around it, to the
upper one with probability (|x| - lo) / (hi - lo).
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_FORMATS = {           # name: (exponent bits, mantissa bits, bias, ieee_specials, code dtype)
    "bf16": (8, 7, 127, True, np.uint16),
    "f16": (5, 10, 15, True, np.uint16),
    "fp8_e5m2": (5, 2, 15, True, np.uint8),
    "fp8_e4m3": (4, 3, 7, False, np.uint8),
}


def _split(fmt):
    eb, mb, bias, ieee, dt = _FORMATS[fmt]
    return eb, mb, bias, ieee, dt


def decode(codes, fmt):
    """Value (float64) of each code."""
    eb, mb, bias, ieee, _ = _split(fmt)
    c = np.asarray(codes).astype(np.int64)
    sign = np.where((c >> (eb + mb)) & 1, -1.0, 1.0)
    E = (c >> mb) & ((1 << eb) - 1)
    M = c & ((1 << mb) - 1)
    normal = np.ldexp(1.0 + M / float(1 << mb), (E - bias).astype(np.int64))
    subnormal = np.ldexp(M / float(1 << mb), 1 - bias)
    v = np.where(E == 0, subnormal, normal)
    emax = (1 << eb) - 1
    if ieee:
        v = np.where((E == emax) & (M == 0), np.inf, v)
        v = np.where((E == emax) & (M != 0), np.nan, v)
    else:
        v = np.where((E == emax) & (M == (1 << mb) - 1), np.nan, v)
    return sign * v


def _finite_table(fmt):
    eb, mb, bias, ieee, _ = _split(fmt)
    codes = np.arange(1 << (eb + mb), dtype=np.int64)        # sign bit clear
    vals = decode(codes, fmt)
    keep = np.isfinite(vals)
    return codes[keep], vals[keep]                            # ascending in both


def encode(x, fmt):
    """Code of the nearest representable value, ties to even mantissa."""
    eb, mb, bias, ieee, dt = _split(fmt)
    x = np.asarray(x, dtype=np.float64)
    codes, vals = _finite_table(fmt)
    a = np.abs(x)
    hi = np.searchsorted(vals, a, side="left")               # vals[hi-1] < a <= vals[hi]
    hi_c = np.clip(hi, 0, len(vals) - 1)
    lo_c = np.clip(hi - 1, 0, len(vals) - 1)
    d_lo = a - vals[lo_c]
    d_hi = vals[hi_c] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (codes[hi_c] % 2 == 0))
    out = np.where(pick_hi, codes[hi_c], codes[lo_c])
    # beyond the largest finite value
    vmax = vals[-1]
    over = a > vmax
    if dt == np.uint16:
        step = vals[-1] - vals[-2]                            # spacing at the top binade
        to_inf = a >= vmax + step / 2                         # tie goes to the even (2^(emax+1)) side
        inf_code = ((1 << eb) - 1) << mb
        out = np.where(over, np.where(to_inf, inf_code, codes[-1]), out)
    else:
        out = np.where(over, codes[-1], out)                  # the 8-bit formats saturate
    nan_code = (((1 << eb) - 1) << mb) | ((1 << mb) - 1) if not ieee else (((1 << eb) - 1) << mb) | (1 << (mb - 1))
    out = np.where(np.isnan(x), nan_code, out)
    out = out | (np.signbit(x).astype(np.int64) << (eb + mb))
    return out.astype(dt)


_PIECE = 1 << 20


def _piecewise(fn, first, *rest):
    """fn applied to equal cuts of its (same-shaped) array arguments on a thread pool, results joined: the
    roundings here act on every element by itself, so the cut changes nothing."""
    first = np.asarray(first)
    if first.size <= _PIECE:
        return fn(first, *rest)
    flat = [np.asarray(a).reshape(-1) for a in (first,) + rest]
    cuts = list(range(0, first.size, _PIECE)) + [first.size]
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        parts = list(ex.map(lambda ab: fn(*[a[ab[0]:ab[1]] for a in flat]), zip(cuts[:-1], cuts[1:])))
    return np.concatenate(parts).reshape(first.shape)


def round_to(x, fmt):
    """x rounded to the format and returned as float32 (exactly representable there).
    fmt "f32" rounds float64 to float32."""
    if fmt == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    return _piecewise(lambda a: decode(encode(a, fmt), fmt).astype(np.float32), x)


def round_stochastic(x, fmt, r16):
    """Element by element (see _round_stochastic_piece); long arrays are cut into pieces."""
    if fmt == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    return _piecewise(lambda a, r: _round_stochastic_piece(a, fmt, r), x, np.broadcast_to(np.asarray(r16), np.shape(x)))


def _round_stochastic_piece(x, fmt, r16):
    """x rounded to one of its two neighbours lo <= |x| <= hi in the format (sign kept), returned as
    float32: the one further from zero is taken iff r16 < 65536 * (|x| - lo) / (hi - lo), r16 being a
    uniform integer in [0, 65536).  The expectation over r16 is x to within (hi - lo) / 65536.
    Magnitudes beyond the largest finite value go to it (all formats saturate here); NaN stays NaN;
    a representable x is returned unchanged for every r16."""
    if fmt == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    x = np.asarray(x, dtype=np.float64)
    r16 = np.asarray(r16).astype(np.float64)
    _, vals = _finite_table(fmt)
    a = np.abs(x)
    lo = np.clip(np.searchsorted(vals, a, side="right") - 1, 0, len(vals) - 1)     # vals[lo] <= a
    hi = np.minimum(lo + 1, len(vals) - 1)
    gap = vals[hi] - vals[lo]
    frac = np.where(gap > 0, (np.minimum(a, vals[hi]) - vals[lo]) / np.where(gap > 0, gap, 1.0), 0.0)
    v = np.where(r16 < frac * 65536.0, vals[hi], vals[lo])
    v = np.where(np.isnan(x), np.nan, np.copysign(v, x))
    return v.astype(np.float32)
