"""CPU oracle for the RNS-form FV hot path of HCNN.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
this module.  It shares no code, table or constant generator with the HIP path.

Every operation is the plain definition written out:
  * polynomial products are schoolbook products in Z_p[X]/(X^n+1) or in
    Z[X]/(X^n+1) (Sec. 2.1: R = Z[X]/<X^N+1>, R_q = R/qR);
  * the NTT is direct evaluation at the 2n-th roots of unity (the CRT
    decomposition of Sec. 2.1.1, applied to a ciphertext prime);
  * residue vectors are turned into integers with the CRT reconstruction map of
    the worked example in Sec. 3.1.2 (Plaintext Space CRT Decomposition);
  * t/q scaling (Decrypt, HMult step 2 in Sec. 2.1) is exact rounding of a
    rational number in Python integers.
The O(n^2) loops run in C (oracle/ckernels.c); all big-integer work is Python.

Conventions the paper leaves open (each also listed in the design document):
  primes      largest primes below 2^30 congruent to 1 mod 2n, descending
  psi         x^((p-1)/2n) for the smallest x >= 2 that gives psi^n = -1 mod p
  NTT order   output index j holds the value at psi^(2*brev(j)+1)
  [.]_q       centred representative in [-(q-1)/2, (q-1)/2] before the tensor
  evk         one component per RNS prime, digit i of c2 is (c2 mod q_i) in [0,q_i),
              key i carries g_i = (q/q_i) * ((q/q_i)^-1 mod q_i)
  Delta*m     m lifted to [0,t)
"""
import ctypes
from functools import lru_cache

import numpy as np

from . import build as _build

_u32p = ctypes.POINTER(ctypes.c_uint32)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_i32p = ctypes.POINTER(ctypes.c_int32)


def _lib():
    return _build.load()


def num_threads() -> int:
    return int(_lib().orc_num_threads())


# --------------------------------------------------------------------------
# number theory
# --------------------------------------------------------------------------
def is_prime(x: int) -> bool:
    """Deterministic Miller-Rabin (bases 2..37 decide every x < 3.3e24)."""
    if x < 2:
        return False
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)
    for sp in small:
        if x % sp == 0:
            return x == sp
    d, r = x - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in small:
        y = pow(a, d, x)
        if y in (1, x - 1):
            continue
        for _ in range(r - 1):
            y = y * y % x
            if y == x - 1:
                break
        else:
            return False
    return True


def ntt_primes(n: int, count: int, below: int = 1 << 30) -> list:
    """The `count` largest primes < below with p = 1 (mod 2n), in descending order."""
    out = []
    c = (below - 2) // (2 * n) * (2 * n) + 1
    while len(out) < count:
        if c < 2 * n:
            raise ValueError("not enough primes")
        if is_prime(c):
            out.append(c)
        c -= 2 * n
    return out


def root_of_unity(n: int, p: int) -> int:
    """psi = x^((p-1)/2n) mod p for the smallest x >= 2 that makes psi^n = -1 (mod p);
    such psi is a primitive 2n-th root of unity."""
    assert (p - 1) % (2 * n) == 0
    x = 2
    while True:
        psi = pow(x, (p - 1) // (2 * n), p)
        if pow(psi, n, p) == p - 1:
            return psi
        x += 1


def brev(j: int, bits: int) -> int:
    r = 0
    for _ in range(bits):
        r = (r << 1) | (j & 1)
        j >>= 1
    return r


def crt_reconstruct(residues, moduli) -> int:
    """CRT map of Sec. 3.1.2: y = sum_i (y_i * ((M/m_i)^-1 mod m_i)) * (M/m_i), reduced mod M."""
    M = 1
    for m in moduli:
        M *= m
    y = 0
    for yi, mi in zip(residues, moduli):
        Mi = M // mi
        y += (int(yi) * pow(Mi, -1, mi)) * Mi
    return y % M


def icrt(x: int, moduli) -> list:
    """Inverse CRT map of Sec. 3.1.2."""
    return [x % m for m in moduli]


def centre(x: int, M: int) -> int:
    """Representative of x mod M in [-(M-1)/2, (M-1)/2] (M odd)."""
    x %= M
    return x - M if x > (M - 1) // 2 else x


def round_div(num: int, den: int) -> int:
    """Nearest integer to num/den (den > 0).  A tie would make the result depend on a
    rounding convention the paper does not give; the callers' arguments exclude
    ties (den odd and coprime to the factor t), so a tie is an error here."""
    assert den > 0
    two = 2 * num + den
    if two % (2 * den) == 0:
        raise ArithmeticError("tie in rounding division")
    return two // (2 * den)


# --------------------------------------------------------------------------
# negacyclic NTT by direct evaluation
# --------------------------------------------------------------------------
@lru_cache(maxsize=256)
def _psi_tables(n: int, p: int, natural: bool):
    psi = root_of_unity(n, p)
    pw = np.empty(2 * n, dtype=np.uint32)
    v = 1
    for e in range(2 * n):
        pw[e] = v
        v = v * psi % p
    bits = n.bit_length() - 1
    if natural:
        expo = np.array([2 * j + 1 for j in range(n)], dtype=np.uint32)
    else:
        expo = np.array([2 * brev(j, bits) + 1 for j in range(n)], dtype=np.uint32)
    return psi, pw, expo


def _as_u32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint32))


def ntt_forward(a, p: int, natural: bool = False):
    """ahat[j] = sum_i a_i psi^((2*brev(j)+1) i) mod p  (natural=True: exponent 2j+1)."""
    a = _as_u32(a)
    n = a.shape[-1]
    _, pw, expo = _psi_tables(n, p, natural)
    out = np.empty_like(a)
    flat_in, flat_out = a.reshape(-1, n), out.reshape(-1, n)
    for r in range(flat_in.shape[0]):
        _lib().orc_ntt_eval(n, p, pw.ctypes.data_as(_u32p), expo.ctypes.data_as(_u32p),
                            flat_in[r].ctypes.data_as(_u32p), flat_out[r].ctypes.data_as(_u32p))
    return out


def ntt_inverse(ahat, p: int, natural: bool = False):
    """The polynomial of degree < n whose forward transform is ahat."""
    ahat = _as_u32(ahat)
    n = ahat.shape[-1]
    _, pw, expo = _psi_tables(n, p, natural)
    n_inv = pow(n, -1, p)
    out = np.empty_like(ahat)
    flat_in, flat_out = ahat.reshape(-1, n), out.reshape(-1, n)
    for r in range(flat_in.shape[0]):
        _lib().orc_ntt_interp(n, p, pw.ctypes.data_as(_u32p), expo.ctypes.data_as(_u32p), n_inv,
                              flat_in[r].ctypes.data_as(_u32p), flat_out[r].ctypes.data_as(_u32p))
    return out


# --------------------------------------------------------------------------
# schoolbook products
# --------------------------------------------------------------------------
def poly_mul_mod(a, b, p: int):
    """a*b in Z_p[X]/(X^n+1), schoolbook."""
    a, b = _as_u32(a), _as_u32(b)
    n = a.shape[0]
    assert a.shape == b.shape == (n,)
    c = np.empty(n, dtype=np.uint32)
    _lib().orc_negacyclic_mod(n, p, a.ctypes.data_as(_u32p), b.ctypes.data_as(_u32p),
                              c.ctypes.data_as(_u32p))
    return c


def _to_sign_magnitude(xs, w):
    n = len(xs)
    neg = np.fromiter((1 if x < 0 else 0 for x in xs), dtype=np.uint8, count=n)
    buf = b"".join(abs(x).to_bytes(8 * w, "little") for x in xs)
    mag = np.frombuffer(buf, dtype=np.uint64).reshape(n, w).copy()
    return mag, neg


def poly_mul_int(a, b):
    """a*b in Z[X]/(X^n+1) for lists of Python integers, schoolbook."""
    n = len(a)
    assert len(b) == n
    amax = max(1, max(abs(x) for x in a))
    bmax = max(1, max(abs(x) for x in b))
    w = (max(amax, bmax).bit_length() + 63) // 64
    wo = ((n * amax * bmax).bit_length() + 63) // 64 + 1
    am, an = _to_sign_magnitude(a, w)
    bm, bn = _to_sign_magnitude(b, w)
    pos = np.empty((n, wo), dtype=np.uint64)
    neg = np.empty((n, wo), dtype=np.uint64)
    _lib().orc_negacyclic_int(n, w, wo, am.ctypes.data_as(_u64p), an.ctypes.data_as(_u8p),
                              bm.ctypes.data_as(_u64p), bn.ctypes.data_as(_u8p),
                              pos.ctypes.data_as(_u64p), neg.ctypes.data_as(_u64p))
    pb, nb = pos.tobytes(), neg.tobytes()
    step = 8 * wo
    return [int.from_bytes(pb[m * step:(m + 1) * step], "little")
            - int.from_bytes(nb[m * step:(m + 1) * step], "little") for m in range(n)]


# --------------------------------------------------------------------------
# FV scheme (Sec. 2.1)
# --------------------------------------------------------------------------
class Context:
    """Ring degree n, ciphertext primes q_0..q_{k-1} (q = their product), plaintext modulus t."""

    def __init__(self, n: int, q_primes, t: int):
        assert n >= 2 and n & (n - 1) == 0
        self.n = n
        self.q = [int(p) for p in q_primes]
        self.k = len(self.q)
        self.t = int(t)
        self.Q = 1
        for p in self.q:
            assert is_prime(p) and (p - 1) % (2 * n) == 0
            self.Q *= p
        assert len(set(self.q)) == self.k
        assert is_prime(self.t) and self.t not in self.q
        self.delta = self.Q // self.t          # floor(q/t), Encrypt in Sec. 2.1

    # -- representation changes ------------------------------------------
    def to_rns(self, ints):
        """Integer polynomial -> residues [k][n] in [0, q_l)."""
        out = np.empty((self.k, self.n), dtype=np.uint32)
        for l, p in enumerate(self.q):
            out[l] = [x % p for x in ints]
        return out

    def small_to_rns(self, small):
        return self.to_rns([int(x) for x in small])

    def lift(self, rns):
        """Residues [k][n] -> integers in [0, q)."""
        rns = np.asarray(rns)
        cols = rns.T.tolist()
        return [crt_reconstruct(col, self.q) for col in cols]

    def lift_centred(self, rns):
        return [centre(x, self.Q) for x in self.lift(rns)]

    # -- R_q arithmetic ---------------------------------------------------
    def mul_rq(self, a_rns, b_rns):
        return np.stack([poly_mul_mod(a_rns[l], b_rns[l], p) for l, p in enumerate(self.q)])

    def add_rq(self, a_rns, b_rns):
        out = np.empty((self.k, self.n), dtype=np.uint32)
        for l, p in enumerate(self.q):
            out[l] = (a_rns[l].astype(np.uint64) + b_rns[l].astype(np.uint64)) % p
        return out

    def neg_rq(self, a_rns):
        out = np.empty((self.k, self.n), dtype=np.uint32)
        for l, p in enumerate(self.q):
            out[l] = (p - a_rns[l].astype(np.uint64) % p) % p
        return out


def keygen(ctx: Context, s, a, e, a_evk, e_evk):
    """KeyGen of Sec. 2.1 with the randomness passed in.

    s [n] ternary; a [k][n] uniform residues; e [n] small;
    a_evk [k][k][n] uniform residues (one a_i per component), e_evk [k][n] small.
    Returns pk [2][k][n] = (e - a s, a) and evk [k][2][k][n] with
    evk[i] = (g_i s^2 - (a_i s + e_i), a_i), g_i = (q/q_i) ((q/q_i)^-1 mod q_i).
    """
    s_r = ctx.small_to_rns(s)
    pk0 = ctx.add_rq(ctx.neg_rq(ctx.mul_rq(a, s_r)), ctx.small_to_rns(e))
    pk = np.stack([pk0, _as_u32(a)])
    s2 = ctx.mul_rq(s_r, s_r)
    evk = np.empty((ctx.k, 2, ctx.k, ctx.n), dtype=np.uint32)
    for i in range(ctx.k):
        Qi = ctx.Q // ctx.q[i]
        g = Qi * pow(Qi, -1, ctx.q[i]) % ctx.Q
        g_s2 = np.empty((ctx.k, ctx.n), dtype=np.uint32)
        for l, p in enumerate(ctx.q):
            g_s2[l] = (s2[l].astype(np.uint64) * (g % p)) % p
        body = ctx.add_rq(ctx.mul_rq(a_evk[i], s_r), ctx.small_to_rns(e_evk[i]))
        evk[i, 0] = ctx.add_rq(g_s2, ctx.neg_rq(body))
        evk[i, 1] = a_evk[i]
    return pk, evk


def encrypt(ctx: Context, pk, m, u, e1, e2):
    """Encrypt of Sec. 2.1: c = (pk0 u + e1 + floor(q/t) m, pk1 u + e2), m in [0,t)."""
    u_r = ctx.small_to_rns(u)
    dm = ctx.to_rns([ctx.delta * int(x) for x in m])
    c0 = ctx.add_rq(ctx.add_rq(ctx.mul_rq(pk[0], u_r), ctx.small_to_rns(e1)), dm)
    c1 = ctx.add_rq(ctx.mul_rq(pk[1], u_r), ctx.small_to_rns(e2))
    return np.stack([c0, c1])


def decrypt(ctx: Context, s, ct):
    """Decrypt of Sec. 2.1: m = round((t/q) (c0 + c1 s mod q)) mod t.  Accepts 2 or 3 components
    (a 3-component ciphertext decrypts under (1, s, s^2))."""
    s_r = ctx.small_to_rns(s)
    acc = _as_u32(ct[0])
    spow = s_r
    for comp in range(1, len(ct)):
        acc = ctx.add_rq(acc, ctx.mul_rq(ct[comp], spow))
        if comp + 1 < len(ct):
            spow = ctx.mul_rq(spow, s_r)
    x = ctx.lift(acc)
    dtype = np.uint32 if ctx.t < (1 << 32) else np.uint64        # plaintext words: 32 bits unless t needs more
    return np.array([round_div(ctx.t * xi, ctx.Q) % ctx.t for xi in x], dtype=dtype)


def noise_bits(ctx: Context, s, ct) -> int:
    """Size of the noise in a ciphertext: with x = [c0 + c1 s]_q, t*x = q*(m + t*a) + r for the centred
    remainder r = [t*x]_q, and v = r/q is the invariant noise of the ciphertext (Decrypt of Sec. 2.1
    returns m exactly while |v| < 1/2; the noise budget of Sec. 5.5 is -log2(2 max|v|), i.e.
    log2(q) - 1 - log2(max|r|)).  Returns the bit length of max_j |r_j| (0 when every r_j = 0)."""
    s_r = ctx.small_to_rns(s)
    x = ctx.lift(ctx.add_rq(_as_u32(ct[0]), ctx.mul_rq(ct[1], s_r)))
    worst = 0
    for xi in x:
        r = centre(ctx.t * xi % ctx.Q, ctx.Q)
        worst = max(worst, abs(r))
    return int(worst).bit_length()


def noise_budget_bits(ctx: Context, bits: int) -> float:
    """Noise budget in bits for a noise of `bits` bits: log2(q) - 1 - bits, a lower bound that is less
    than one bit below -log2(2 max|v|)."""
    import math
    return math.log2(ctx.Q) - 1 - bits


def hmult_scaled(ctx: Context, ct1, ct2):
    """HMult steps 1 and the scaling of step 2 (Sec. 2.1): the tensor over the integers on
    centred lifts, then round(t/q * .) per coefficient, reduced mod q.  Returns [3][k][n]."""
    c01, c11 = ctx.lift_centred(ct1[0]), ctx.lift_centred(ct1[1])
    c02, c12 = ctx.lift_centred(ct2[0]), ctx.lift_centred(ct2[1])
    d0 = poly_mul_int(c01, c02)
    d1 = [x + y for x, y in zip(poly_mul_int(c01, c12), poly_mul_int(c11, c02))]
    d2 = poly_mul_int(c11, c12)
    out = np.empty((3, ctx.k, ctx.n), dtype=np.uint32)
    for b, d in enumerate((d0, d1, d2)):
        out[b] = ctx.to_rns([round_div(ctx.t * x, ctx.Q) for x in d])
    return out


def relinearize(ctx: Context, y, evk):
    """Relinearize of Sec. 2.1 with RNS digits: c'_b = y_b + sum_i evk[i][b] * D_i in R_q,
    D_i = the polynomial with coefficients (y_2 mod q_i) in [0, q_i)."""
    out = np.stack([_as_u32(y[0]).copy(), _as_u32(y[1]).copy()])
    for i in range(ctx.k):
        digit = [int(v) for v in y[2][i]]
        d_r = ctx.to_rns(digit)
        for b in range(2):
            out[b] = ctx.add_rq(out[b], ctx.mul_rq(evk[i][b], d_r))
    return out


def hmult(ctx: Context, ct1, ct2, evk):
    return relinearize(ctx, hmult_scaled(ctx, ct1, ct2), evk)


def square_relin(ctx: Context, ct, evk):
    """HSquare = HMult(c, c) (Sec. 4.1 / micro-benchmarks)."""
    return hmult(ctx, ct, ct, evk)


def scalar_mac(ctx: Context, cts, idx_row, w_row):
    """Convolution-type node (Sec. 3.2 / 4.3): sum_tau w_tau * ct_{idx_tau} in R_q^2, no bias.
    HMultPlain by the constant polynomial w (signed integer), HAdd of the results."""
    T = len(idx_row)
    w = np.ascontiguousarray(np.asarray(w_row, dtype=np.int32))
    out = np.empty((2, ctx.k, ctx.n), dtype=np.uint32)
    rows_t = ctypes.POINTER(ctypes.c_uint32) * T
    for b in range(2):
        for l, p in enumerate(ctx.q):
            keep = [np.ascontiguousarray(cts[int(i)][b][l], dtype=np.uint32) for i in idx_row]
            rows = rows_t(*[r.ctypes.data_as(_u32p) for r in keep])
            _lib().orc_scalar_mac(ctx.n, p, T, rows, w.ctypes.data_as(_i32p),
                                  out[b, l].ctypes.data_as(_u32p))
    return out


# --------------------------------------------------------------------------
# slot packing (Sec. 2.1.1): R_t = prod_j Z_t[X]/(X - alpha_j), alpha_j = psi_t^(2j+1)
# --------------------------------------------------------------------------
def slot_encode(values, n: int, t: int):
    """Polynomial in R_t whose value at psi_t^(2j+1) is values[j]."""
    return ntt_inverse(np.asarray(values, dtype=np.uint32) % t, t, natural=True)


def slot_decode(poly, n: int, t: int):
    return ntt_forward(np.asarray(poly, dtype=np.uint32) % t, t, natural=True)


def slot_eval(polys, n: int, t: int, slots):
    """Values of the chosen slots only: polys [m][n] in R_t -> [m][len(slots)], slot j being the value
    of the polynomial at psi_t^(2j+1) (the evaluation view of the plaintext CRT map, Sec. 2.1.1).
    Written as the evaluation itself, for use where only a few slots of many polynomials are needed."""
    psi = root_of_unity(n, t)
    if t >= (1 << 24):
        # wide plaintext modulus (the 43-bit t of the MNIST parameter sets): Python integers throughout
        rows = [[int(v) % t for v in row] for row in np.asarray(polys)]
        assert all(len(r) == n for r in rows)
        out = np.zeros((len(rows), len(slots)), dtype=object)
        for col, j in enumerate(slots):
            x = pow(psi, 2 * int(j) + 1, t)
            powers = [1] * n
            for i in range(1, n):
                powers[i] = powers[i - 1] * x % t
            for r, row in enumerate(rows):
                out[r, col] = sum(map(int.__mul__, row, powers)) % t
        return out
    polys = np.asarray(polys, dtype=np.int64) % t
    assert polys.ndim == 2 and polys.shape[1] == n
    out = np.zeros((polys.shape[0], len(slots)), dtype=np.int64)
    for col, j in enumerate(slots):
        x = pow(psi, 2 * int(j) + 1, t)
        powers = np.ones(n, dtype=np.int64)
        for i in range(1, n):
            powers[i] = powers[i - 1] * x % t
        out[:, col] = (polys @ powers) % t          # n terms below 2^48 each: exact in int64
    return out
