"""Oracle (test infrastructure): counter-based random direction z.

The paper keeps the perturbation and the update on the same Gaussian vector by
saving and restoring a stateful generator's state per module (Alg. 2, the
Get/SetRngState pair; Sec. 5.1).  Here the "state" of element e of tensor p at
step seed s is the triple (s, p, e) itself: a counter-based generator maps it to
z[p, e], so any block can regenerate its z at any time, in any order.

Generator: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel
random numbers: as easy as 1, 2, 3", SC'11).  Gaussian map: Box-Muller on
16-bit uniforms (one 32-bit word per pair of elements), evaluated in float64
and rounded once to float32.  The paper fixes only that z is standard normal
and reproducible from the seed (Alg. 1, Sec. 5.1); this map is a choice.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox4x32 rounds.  c0..c3: uint32 counters (arrays or scalars,
    broadcast together); k0, k1: python ints (the 64-bit key, low word first).
    Returns four uint32 arrays.

    One round: (c0, c1, c2, c3) <- (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2),
                                    hi(M0*c0) ^ c3 ^ k1, lo(M0*c0));
    then the key is bumped by the Weyl constants."""
    c0, c1, c2, c3 = np.broadcast_arrays(*[np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3)])
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0            # < 2^64, exact in uint64
        p1 = _M1 * c2
        n0 = (p1 >> _S32) ^ c1 ^ np.uint64(k0)
        n1 = p1 & _MASK
        n2 = (p0 >> _S32) ^ c3 ^ np.uint64(k1)
        n3 = p0 & _MASK
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def random_words(seed, tensor_id, e0, n):
    """Words e0 .. e0+n-1 of the random stream of tensor `tensor_id` at step seed
    `seed`.  Word j is output j & 3 of Philox call q = j >> 2 with
    counter (lo32(q), hi32(q), tensor_id, 0), key (lo32(seed), hi32(seed)).
    Elements 2j and 2j+1 of the tensor are drawn from word j (see gaussian)."""
    seed = int(seed)
    e = np.arange(int(e0), int(e0) + int(n), dtype=np.uint64)
    q = e >> np.uint64(2)
    qs, inv = np.unique(q, return_inverse=True)
    w = philox4x32_10(qs & _MASK, qs >> _S32, np.uint64(tensor_id), np.uint64(0),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    w = np.stack(w, axis=1)                       # [calls, 4]
    return w[inv, (e & np.uint64(3)).astype(np.int64)]


_CHUNK = 1 << 20      # elements per piece; a multiple of 8 so pieces start on a Philox call


def gaussian(seed, tensor_id, e0, n):
    """z for elements e0 .. e0+n-1 of a tensor, float32 (see _gaussian_piece).
    Long ranges are cut into pieces evaluated on a thread pool; every element's
    value depends only on (seed, tensor_id, e), so the cut changes nothing."""
    e0 = int(e0)
    n = int(n)
    if n <= _CHUNK:
        return _gaussian_piece(seed, tensor_id, e0, n)
    cuts = [e0] + list(range((e0 // _CHUNK + 1) * _CHUNK, e0 + n, _CHUNK)) + [e0 + n]
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        parts = list(ex.map(lambda ab: _gaussian_piece(seed, tensor_id, ab[0], ab[1] - ab[0]),
                            zip(cuts[:-1], cuts[1:])))
    return np.concatenate(parts)


def _gaussian_piece(seed, tensor_id, e0, n):
    """z for elements e0 .. e0+n-1 of a tensor, float32.

    Philox call q covers elements 8q .. 8q+7; its output word i (0..3) feeds one
    Box-Muller pair: u1 = ((x >> 16) + 1) / 2^16 in (0, 1], u2 = (x & 0xffff) / 2^16
    in [0, 1), rho = sqrt(-2 ln u1); elements 8q+2i, 8q+2i+1 = rho cos(2 pi u2),
    rho sin(2 pi u2).  |z| <= sqrt(32 ln 2) = 4.71."""
    seed = int(seed)
    e0 = int(e0)
    n = int(n)
    q_lo = e0 >> 3
    q_hi = (e0 + n + 7) >> 3
    q = np.arange(q_lo, q_hi, dtype=np.uint64)
    x = philox4x32_10(q & _MASK, q >> _S32, np.uint64(tensor_id), np.uint64(0),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    out = np.empty((q.size, 8), dtype=np.float64)
    for i in range(4):
        xi = x[i].astype(np.uint64)
        u1 = ((xi >> np.uint64(16)).astype(np.float64) + 1.0) / 65536.0
        u2 = (xi & np.uint64(0xFFFF)).astype(np.float64) / 65536.0
        rho = np.sqrt(-2.0 * np.log(u1))
        out[:, 2 * i] = rho * np.cos(2.0 * np.pi * u2)
        out[:, 2 * i + 1] = rho * np.sin(2.0 * np.pi * u2)
    flat = out.reshape(-1)
    lo = e0 - 8 * q_lo
    return flat[lo:lo + n].astype(np.float32)


def rounding_bits(seed, tensor_id, e0, n):
    """16 uniform bits per element e0 .. e0+n-1 for the stochastic rounding of an update that uses the
    direction of step seed `seed`: a second stream of the same generator, told apart from the one z is
    drawn from by the last counter word (1 instead of 0).  Call q = e >> 3 covers 8 elements; element e
    takes the low (e even) or high (e odd) half of output word (e >> 1) & 3."""
    seed = int(seed)
    e = np.arange(int(e0), int(e0) + int(n), dtype=np.uint64)
    q = e >> np.uint64(3)
    qs, inv = np.unique(q, return_inverse=True)
    w = philox4x32_10(qs & _MASK, qs >> _S32, np.uint64(tensor_id), np.uint64(1),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    w = np.stack(w, axis=1).astype(np.uint64)[inv, ((e >> np.uint64(1)) & np.uint64(3)).astype(np.int64)]
    return ((w >> (np.uint64(16) * (e & np.uint64(1)))) & np.uint64(0xFFFF)).astype(np.uint16)
