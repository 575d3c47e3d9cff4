"""The C ABI without a GPU: the HIP library loads, exports every symbol the header declares,
rejects invalid arguments before touching a device, and its host-side parameter helpers follow
the stated rules."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import fv
from paper_1811_00778_amd import _capi, build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    path = hip_build.build(force=False)
    return _capi.declare(ctypes.CDLL(path))


def _gpu():
    import torch
    return torch.cuda.is_available()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "hcnn.h")).read()
    names = set(re.findall(r"\b(hcnn_[a-z0-9_]+)\s*\(", header))
    assert names == set(_capi.SIGNATURES), names ^ set(_capi.SIGNATURES)
    for name in names:
        assert getattr(lib, name) is not None


def test_prime_rule_matches_oracle_rule(lib):
    for n, cnt in ((1024, 6), (8192, 17), (16384, 34), (32768, 50)):
        assert _capi.gen_primes(lib, n, cnt) == fv.ntt_primes(n, cnt)
    assert lib.hcnn_gen_primes(1000, 3, (ctypes.c_uint32 * 3)()) == _capi.ERR["N"]
    assert lib.hcnn_gen_primes(1024, 0, (ctypes.c_uint32 * 3)()) == _capi.ERR["ARG"]
    assert lib.hcnn_gen_primes(1024, 3, None) == _capi.ERR["NULL"]


@pytest.mark.parametrize("n,k,want", [(1024, 2, 3), (8192, 8, 9), (16384, 16, 18), (32768, 24, 26)])
def test_min_aux_count_is_minimal_by_big_integers(lib, n, k, want):
    t = 65537
    cand = _capi.gen_primes(lib, n, k + k + 8)
    q, rest = cand[:k], cand[k:]
    got = _capi.min_aux_count(lib, n, q, t, rest)
    Q = int(np.prod([int(v) for v in q], dtype=object))
    bound = t * n * Q + 1
    prod, need = 1, 0
    while prod <= bound:
        prod *= rest[need]
        need += 1
    assert got == need == want


def test_ctx_create_rejects_bad_arguments(lib):
    n, k, t = 1024, 2, 65537
    cand = _capi.gen_primes(lib, n, 6)
    q, p = cand[:2], cand[2:5]

    def create(n_, q_, p_, t_):
        h = ctypes.c_void_p()
        rc = lib.hcnn_ctx_create(ctypes.byref(h), n_, len(q_), _capi.u32_array(q_), len(p_),
                                 _capi.u32_array(p_) if p_ else None, t_, None)
        if rc == 0:
            lib.hcnn_ctx_destroy(h)
        return rc

    E = _capi.ERR
    assert create(1000, q, p, t) == E["N"]
    assert create(512, q, p, t) == E["N"]
    assert create(65536, q, p, t) == E["N"]
    assert create(n, [q[0], q[0]], p, t) == E["PRIME"]                 # repeated
    assert create(n, [q[0], q[1] - 2048], p, t) in (E["PRIME"],)       # not prime (or not 1 mod 2n)
    assert create(n, [q[0], 12289], p, t) == E["PRIME"]                # prime, but below 2^29
    assert create(n, q, [q[0]] + p[1:], t) == E["PRIME"]               # auxiliary prime repeats a q prime
    assert create(2048, q, p, t) in (E["PRIME"], E["OK"], E["NODEVICE"])  # 1 mod 2048 need not hold
    assert create(n, q, p, 65536) == E["T"]
    assert create(n, q, p, 1) == E["T"]
    assert create(n, q, p, q[0]) == E["T"]                             # t among the ciphertext primes
    assert create(n, q, p, p[0]) == E["T"]                             # ... or the auxiliary primes
    assert create(n, q, p, (1 << 47) + 5) == E["T"]                    # too wide (2^47 + 5 is prime)
    assert create(n, q, p, 5522259017729 + 2) == E["T"]                # wide and composite
    assert create(n, q, p, 5522259017729) in (E["AUX"], E["OK"], E["NODEVICE"])   # the 43-bit modulus needs a larger k'
    assert create(n, q, p[:2], t) == E["AUX"]                          # k' = 2 is too small here
    assert lib.hcnn_ctx_create(None, n, 2, _capi.u32_array(q), 0, None, t, None) == E["NULL"]
    h = ctypes.c_void_p()
    assert lib.hcnn_ctx_create(ctypes.byref(h), n, 0, _capi.u32_array(q), 0, None, t, None) == E["ARG"]
    assert lib.hcnn_ctx_create(ctypes.byref(h), n, 33, _capi.u32_array(q * 17), 0, None, t, None) == E["ARG"]
    if not _gpu():
        # valid arguments but no device: a clean error, not a crash, and no fallback
        assert create(n, q, p, t) == E["NODEVICE"]


def test_null_context_is_rejected(lib):
    E = _capi.ERR
    assert lib.hcnn_ntt_fwd(None, None, 1) == E["NULL"]
    assert lib.hcnn_ct_square_relin(None, None, 1, None) == E["NULL"]
    assert lib.hcnn_ct_scalar_mac(None, None, 1, None, None, 1, 1, 1, 1, None) == E["NULL"]
    assert lib.hcnn_ctx_destroy(None) == E["NULL"]
    assert lib.hcnn_strerror(E["AUX"]).decode().startswith("auxiliary basis")
    assert lib.hcnn_strerror(0).decode() == "ok"


def test_binding_has_no_cpu_fallback():
    if _gpu():
        pytest.skip("GPU present")
    from paper_1811_00778_amd import binding
    with pytest.raises(RuntimeError):
        binding.Context(1024, [1, 2], [3], 65537)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_set_option_validation_needs_no_device(lib):
    # options are checked before anything touches a device; a null context is rejected first
    assert lib.hcnn_set_option(None, _capi.OPT_PROFILE, 1) == _capi.ERR["NULL"]
    assert lib.hcnn_get_stat(None, 0, None) == _capi.ERR["NULL"]
    assert lib.hcnn_profile_read(None, 0, None, None, None) == _capi.ERR["NULL"]
    assert lib.hcnn_measure_ceiling(None, 0, None) == _capi.ERR["NULL"]
    assert lib.hcnn_ct_square_relin_noalloc(None, None, 1, None) == _capi.ERR["NULL"]
