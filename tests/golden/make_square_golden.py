#!/usr/bin/env python3
"""Writes tests/golden/config5_square_sha256.txt: SHA-256 of every output row of two whole squarings with
relinearisation (HMult(c, c) of Sec. 2.1: tensor over the integers on centred lifts, exact rounding of t/q times
it, relinearisation with one key component per RNS prime) at the deep-modulus configuration (n = 32768, 24
ciphertext primes), computed by the CPU oracle alone on that configuration's seeded inputs.

    python tests/golden/make_square_golden.py        (about ten minutes on 8 cores)

Only oracle/ and the seeded generators are used; nothing here touches the HIP library.  The GPU test draws the
same inputs in the same order from the same generator and compares the hashes of its own output rows.
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import fv                          # noqa: E402
from workloads import generators as gen        # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config5_square_sha256.txt")
GENUINE, RANDOM = 1, 17                        # the second genuine encryption; the 18th random ciphertext


def row_hashes(ct):
    return [[hashlib.sha256(np.ascontiguousarray(ct[b, l], dtype="<u4").tobytes()).hexdigest()
             for l in range(ct.shape[1])] for b in range(2)]


def inputs():
    """Keys and ciphertexts of configuration 5 in the draw order of the GPU test: key randomness, two plaintext
    polynomials with their encryption randomness, thirty ciphertexts of uniformly random residues."""
    cfg = gen.CONFIGS[5]
    n, k, t = cfg["n"], cfg["k"], cfg["t"]
    q = fv.ntt_primes(n, k)
    octx = fv.Context(n, q, t)
    rng = gen.rng_for(5, 0)
    kr = gen.key_randomness(rng, q, n)
    pk, evk = fv.keygen(octx, kr["s"], kr["a"], kr["e"], kr["a_evk"], kr["e_evk"])
    polys = rng.integers(0, t, size=(2, n), dtype=np.int64).astype(np.uint32)
    er = gen.encryption_randomness(rng, n, 2)
    rnd = gen.uniform_residues(rng, q, n, lead=(30, 2))
    genuine = fv.encrypt(octx, pk, polys[GENUINE], er["u"][GENUINE], er["e1"][GENUINE], er["e2"][GENUINE])
    return octx, evk, genuine, rnd[RANDOM]


def main():
    t0 = time.time()
    octx, evk, genuine, random_ct = inputs()
    print("keys and inputs: %.0f s" % (time.time() - t0), flush=True)
    lines = ["# SHA-256 of the little-endian uint32 words of every output row (polynomial b, prime l) of",
             "# oracle.fv.square_relin -- HMult(c, c) of Sec. 2.1 (tensor, scaling by t/q, relinearisation with",
             "# RNS digits) -- at n = 32768 with the 24 largest 30-bit primes = 1 mod 2n, t = 65537, on two",
             "# ciphertexts of the seeded configuration 5: 'genuine' = the second genuine encryption, 'random' =",
             "# the 18th ciphertext of uniformly random residues.  Written by tests/golden/make_square_golden.py.",
             "# name b l sha256"]
    for name, ct in (("genuine", genuine), ("random", random_ct)):
        t1 = time.time()
        out = fv.square_relin(octx, ct, evk)
        print("%s: oracle squaring %.0f s" % (name, time.time() - t1), flush=True)
        for b, row in enumerate(row_hashes(out)):
            for l, h in enumerate(row):
                lines.append("%s %d %d %s" % (name, b, l, h))
    with open(OUT, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
