"""Counter-based random sampling for the FV helpers.  TEST INFRASTRUCTURE ONLY.

The library offers deterministic samplers (hcnn_sample_ternary / _gaussian / _uniform): every output element is a
fixed function of (seed, stream, element index), so that they can be checked bit for bit.  This module writes
that function out independently:

  * the word source is Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
    1, 2, 3", SC'11): key = (seed low word, seed high word), counter = (element index low word, element index
    high word, stream low word, kind * 2^24 + attempt); one call gives four 32-bit words w0..w3, consumed in
    order; when a sampler needs more it moves on to attempt + 1;
  * ternary (kind 1, secret key and encryption mask u, Sec. 2.1): a word w is accepted unless w = 2^32 - 1
    (so that the accepted words split evenly), value = w mod 3 - 1;
  * rounded Gaussian (kind 2, the "small" errors of Sec. 2.1; sigma = 3.2, values beyond 19 redrawn): words are
    taken in pairs (a, b): the magnitude is the number of table thresholds T[0..19] that are <= a, a pair with
    a >= T[19] is rejected; the sign is minus when the lowest bit of b is set; T[v] = floor(2^32 * P(|X| <= v)) for
    X = round(N(0, 3.2^2)) (the 20 numbers are a shared format constant, listed in the design document);
  * uniform residues (kind 3, the public polynomials a of Sec. 2.1): element index = (poly * k + limb) * n + coeff;
    a word w is accepted when w < p * floor(2^32 / p), value = w mod p.
"""
import math

import numpy as np

KIND_TERNARY, KIND_GAUSSIAN, KIND_UNIFORM = 1, 2, 3
SIGMA, CUT = 3.2, 19

_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """counter: four uint32 arrays (or scalars), key: two -> four uint32 arrays."""
    c = [np.asarray(x, dtype=np.uint64) & 0xFFFFFFFF for x in counter]
    c = list(np.broadcast_arrays(*c))
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = c[0] * np.uint64(_M0)
        p1 = c[2] * np.uint64(_M1)
        hi0, lo0 = p0 >> np.uint64(32), p0 & np.uint64(0xFFFFFFFF)
        hi1, lo1 = p1 >> np.uint64(32), p1 & np.uint64(0xFFFFFFFF)
        c = [hi1 ^ c[1] ^ np.uint64(k0), lo1, hi0 ^ c[3] ^ np.uint64(k1), lo0]
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return [x.astype(np.uint32) for x in c]


def gaussian_thresholds():
    """T[v] = floor(2^32 * P(|X| <= v)), v = 0..19, X = round(N(0, sigma^2))."""
    def cdf(x):
        return 0.5 * (1.0 + math.erf(x / (SIGMA * math.sqrt(2.0))))
    out, acc = [], 0.0
    for v in range(CUT + 1):
        if v == 0:
            acc = cdf(0.5) - cdf(-0.5)
        else:
            acc += 2.0 * (cdf(v + 0.5) - cdf(v - 0.5))
        out.append(int(math.floor(acc * 4294967296.0)))
    return out


# the shared format constant (see the module text); gaussian_thresholds() regenerates it
GAUSS_T = (533280463, 1549416568, 2428136261, 3117868636, 3609276189, 3927060812, 4113592370, 4212972233,
           4261030606, 4282124752, 4290528529, 4293567340, 4294564687, 4294861785, 4294942112, 4294961823,
           4294966213, 4294967101, 4294967264, 4294967291)


def _words(seed, stream, kind, index, attempt):
    idx = np.asarray(index, dtype=np.uint64)
    return philox4x32_10([idx & np.uint64(0xFFFFFFFF), idx >> np.uint64(32), int(stream) & 0xFFFFFFFF,
                          (kind << 24) + attempt], [int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF])


def _sample(seed, stream, kind, count, accept_value, words_per_try):
    """Generic rejection loop over the word stream of every element; accept_value(list of word arrays) returns
    (accepted mask, values)."""
    index = np.arange(count, dtype=np.uint64)
    out = np.zeros(count, dtype=np.int64)
    todo = np.ones(count, dtype=bool)
    attempt = 0
    while todo.any():
        w = _words(seed, stream, kind, index, attempt)
        for s in range(0, 4, words_per_try):
            ok, val = accept_value([x for x in w[s:s + words_per_try]])
            take = todo & ok
            out[take] = val[take]
            todo &= ~ok
        attempt += 1
        assert attempt < 256
    return out


def sample_ternary(seed, stream, count_polys, n):
    def f(ws):
        w = ws[0].astype(np.int64)
        return w != 0xFFFFFFFF, w % 3 - 1
    return _sample(seed, stream, KIND_TERNARY, count_polys * n, f, 1).astype(np.int32).reshape(count_polys, n)


def sample_gaussian(seed, stream, count_polys, n):
    t = np.array(GAUSS_T, dtype=np.int64)

    def f(ws):
        a, b = ws[0].astype(np.int64), ws[1].astype(np.int64)
        mag = (a[:, None] >= t[None, :]).sum(axis=1)
        return a < t[CUT], np.where(b & 1, -mag, mag)
    return _sample(seed, stream, KIND_GAUSSIAN, count_polys * n, f, 2).astype(np.int32).reshape(count_polys, n)


def sample_uniform(seed, stream, count_polys, moduli, n):
    k = len(moduli)
    p = np.tile(np.repeat(np.array(moduli, dtype=np.int64), n), count_polys)        # modulus of every element

    def f(ws):
        w = ws[0].astype(np.int64)
        return w < p * (4294967296 // p), w % p
    return _sample(seed, stream, KIND_UNIFORM, count_polys * k * n, f, 1).astype(np.uint32).reshape(count_polys, k, n)
