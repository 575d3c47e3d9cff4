"""Kernel sources checked on the CPU: the library compiled with -DHCNN_HOSTEMU runs the same
kernel phase bodies and host orchestration as loops, and must match the oracle bit for bit.
(The product path itself is tested in test_gpu_parity.py; nothing here touches a GPU.)"""
import numpy as np
import pytest

import emu
import parity_cases as pc


class EmuBackend:
    def __init__(self):
        self.lib = emu.lib()

    def make_ctx(self, n, q, p, t):
        return emu.EmuContext(n, q, p, t)

    @staticmethod
    def dev(a):
        return emu.aligned(np.ascontiguousarray(a))

    @staticmethod
    def host(buf):
        return buf


@pytest.fixture(scope="module")
def backend():
    return EmuBackend()


@pytest.mark.parametrize("n,k,n_polys,rows", [(1024, 2, 3, None), (2048, 3, 2, 3), (4096, 2, 1, 2),
                                             (8192, 2, 1, 1), (16384, 1, 1, 1), (32768, 1, 10, 1)])
def test_ntt_all_sizes(backend, n, k, n_polys, rows):
    pc.check_ntt(backend, n, k, n_polys, rows)


@pytest.mark.parametrize("n,k", [(1024, 2), (2048, 3)])
def test_keygen_encrypt_decrypt(backend, n, k):
    pc.check_keygen_encrypt_decrypt(backend, n, k)


@pytest.mark.parametrize("n,k", [(1024, 2), (2048, 5)])
def test_scalar_mac(backend, n, k):
    pc.check_scalar_mac(backend, n, k)
    pc.check_mac_linear_in_ntt_domain(backend, n, k)


def test_square_relin_tiny_config(backend):
    pc.check_square_relin(backend, 1024, 2)


def test_square_relin_chunked_ragged(backend):
    pc.check_square_relin(backend, 1024, 3, n_random=4, n_genuine=1, chunk=2)
    pc.check_square_relin(backend, 1024, 3, n_random=5, n_genuine=1)      # one group of four sharing key loads + two singles
    pc.check_square_relin(backend, 1024, 3, n_random=2, n_genuine=0, chunk=2, relin_order=1)   # ciphertext-major order forced


def test_square_relin_batch_split_into_rounds_and_remainder(backend):
    """The default policy sizes its rounds from the occupancy that the platform layer reports for the compiled
    kernels (this build: a fixed count for its single compute unit).  A batch of three rounds of the one-kernel
    relinearisation plus two ciphertexts, large enough for the one-kernel tensor, must take the mixed route: the
    tensor in one kernel, the whole rounds through the one-kernel relinearisation, the two left over through the
    separate kernels."""
    s = pc.Setup(backend, 1024, 2)
    s.ctx.set_relin_key(backend.dev(s.evk))
    rnd, L = s.ctx.relin_fused_round(), 2 + len(s.p)
    assert rnd >= 1
    n_ct = 3 * rnd + 2
    assert n_ct * L >= s.ctx.tensor_fused_threshold()
    cts = pc.gen.uniform_residues(s.rng, s.q, 1024, lead=(n_ct, 2))
    s.ctx.set_profile(True)
    out = backend.host(s.ctx.ct_square_relin(backend.dev(cts)))
    prof = s.ctx.profile()
    assert prof["tensor"][0] == 1 and prof["tensor"][1] == n_ct * L * 5
    assert prof["relin_fused"][0] == 1 and prof["relin_fused"][1] == 3 * rnd * 2 * (2 + 2)
    assert prof["relin_mac"][0] == 1 and prof["ntt_fwd"][1] == 2 * 2 * 2            # the two left over: digit rows only
    for i in (0, 3 * rnd - 1, 3 * rnd, 3 * rnd + 1):
        assert np.array_equal(out[i], pc.fv.square_relin(s.octx, cts[i], s.evk)), i
    # a batch below the tensor threshold and below 3/4 of a round: separate kernels throughout
    s.ctx.reset_stats()
    small = max(1, (3 * rnd - 1) // 4)
    s.ctx.ct_square_relin(backend.dev(cts[:small]))
    prof = s.ctx.profile()
    if small * L < s.ctx.tensor_fused_threshold() and small * 4 < rnd * 3:
        assert prof["tensor"][0] == 0 and prof["relin_fused"][0] == 0 and prof["relin_mac"][0] >= 1
    s.ctx.close()


def test_square_relin_noalloc_equals_allocating_entry_point(backend):
    """The entry point that works in the library's static array: same residues as hcnn_ct_square_relin on two calls in
    a row (the second smaller), no work buffer allocated; a parameter set beyond the array is refused."""
    from paper_1811_00778_amd import _capi
    s = pc.Setup(backend, 1024, 3)
    s.ctx.set_relin_key(backend.dev(s.evk))
    for count in (11, 2):
        cts = backend.dev(pc.gen.uniform_residues(s.rng, s.q, 1024, lead=(count, 2)))
        out = s.ctx.ct_square_relin_noalloc(cts, np.zeros_like(cts))
        assert s.ctx.scratch_bytes() == 0
        assert np.array_equal(out[count - 1], pc.fv.square_relin(s.octx, cts[count - 1], s.evk))
        ref = emu.EmuContext(1024, s.q, s.p, s.t)
        ref.set_relin_key(backend.dev(s.evk))
        assert np.array_equal(out, ref.ct_square_relin(cts))
        ref.close()
    s.ctx.close()
    big = pc.Setup(backend, 32768, 30, with_keys=False)
    x = backend.dev(np.zeros((1, 2, 30, 32768), dtype=np.uint32))
    with pytest.raises(_capi.HcnnError) as err:
        big.ctx.ct_square_relin_noalloc(x, np.zeros_like(x))
    assert err.value.code == _capi.ERR["SCRATCH"]
    big.ctx.close()


def test_square_relin_exact_comparison_path(backend):
    pc.check_square_relin(backend, 1024, 2, force_exact=True)
    pc.check_square_relin(backend, 2048, 4, n_random=1, n_genuine=1, force_exact=True)


def test_square_relin_more_than_16_limbs(backend):
    # k = 17 > 16 exercises the intermediate reductions of the 64-bit inner products
    pc.check_square_relin(backend, 1024, 17, n_random=1, n_genuine=1)


@pytest.mark.parametrize("k,k_aux,big_t", [(3, 4, False), (5, 6, False), (6, 7, False), (7, 8, False), (8, 9, False),
                                           (9, 10, False), (10, 11, False), (11, 12, False), (12, 13, False),
                                           (4, 6, True), (6, 8, True), (8, 10, True), (10, 12, True), (11, 13, True),
                                           (12, 14, True), (14, 16, True), (16, 18, True), (24, 26, True)])
def test_square_relin_register_variants_of_standard_bases(backend, k, k_aux, big_t):
    # the basis sizes of the benchmark configurations, at a ring degree the oracle finishes quickly;
    # a larger plaintext modulus makes k' = k + 2 necessary already at n = 1024
    t = pc.slot_prime_above(1024, 1 << 22) if big_t else 65537
    pc.check_square_relin(backend, 1024, k, n_random=1, n_genuine=1, t=t, expect_k_aux=k_aux)
    pc.check_square_relin(backend, 1024, k, n_random=1, n_genuine=0, t=t, force_exact=True)


def test_square_relin_at_a_degree_with_die_aware_block_orders(backend):
    # n = 8192: 8 coefficient tiles per row, the size from which the inner-product kernel orders its
    # workgroups by accelerator die; three ciphertexts so that the ciphertext index is exercised too
    pc.check_square_relin(backend, 8192, 2, n_random=3, n_genuine=0)
    pc.check_square_relin(backend, 8192, 2, n_random=6, n_genuine=0, relin_order=2)    # key-major order forced
    # one ciphertext: the forced one-kernel relinearisation takes its single-round form (16 residues per thread)
    pc.check_square_relin(backend, 8192, 2, n_random=1, n_genuine=0)


def test_square_relin_largest_ring_two_workgroups_per_forward_row(backend):
    # n = 32768: the forward transforms run as two workgroups per row, out of place, the extended rows staged in the
    # array of the tensor
    pc.check_square_relin(backend, 32768, 2, n_random=2, n_genuine=0)


def test_measure_ceiling_arguments(backend):
    # the diagnostic rejects an unknown probe; the host emulation does not time its launches and reports 0
    from paper_1811_00778_amd import _capi
    import ctypes
    s = pc.Setup(backend, 1024, 2, with_keys=False)
    v = ctypes.c_double(-1.0)
    lib = s.ctx.raw.lib
    assert lib.hcnn_measure_ceiling(s.ctx.raw.handle, len(_capi.CEILINGS), ctypes.byref(v)) == _capi.ERR["ARG"]
    assert lib.hcnn_measure_ceiling(s.ctx.raw.handle, -1, ctypes.byref(v)) == _capi.ERR["ARG"]
    assert lib.hcnn_measure_ceiling(s.ctx.raw.handle, 0, None) == _capi.ERR["NULL"]
    assert lib.hcnn_measure_ceiling(s.ctx.raw.handle, len(_capi.CEILINGS) - 1, ctypes.byref(v)) == 0 and v.value == 0.0
    s.ctx.close()


def test_general_hmult(backend):
    pc.check_mul_relin(backend, 1024, 2)
    pc.check_mul_relin(backend, 2048, 3, force_exact=True)
    pc.check_mul_relin(backend, 1024, 8)


def test_conv_square_layer(backend):
    pc.check_conv_layer_small(backend)


def test_random_parameter_sweep(backend):
    pc.check_random_sweep(backend, 6, seed=7, sizes=(1024,))


def test_counter_based_samplers(backend):
    pc.check_samplers(backend, 1024, 2)
    pc.check_samplers(backend, 2048, 3, seed_id=2)


def test_noise_read_out(backend):
    pc.check_noise_bits(backend, 1024, 2)
    pc.check_noise_bits(backend, 1024, 5)


def test_wide_plaintext_modulus(backend):
    pc.check_wide_plaintext(backend)
    pc.check_wide_plaintext(backend, 1024, 5, seed_id=2, force_exact=True)


def test_plaintext_crt_channels(backend):
    pc.check_crt_channels(backend)


def test_small_network_layer_by_layer(backend):
    pc.check_small_network(backend)


def test_wrappers_check_every_shape_before_the_call(backend):
    """The C ABI takes bare pointers, so the Python wrappers are the only place where a wrongly sized buffer can be
    caught before a kernel reads or writes past it: each argument's full shape is checked, and a scalar MAC whose
    output overlaps its input is refused."""
    n, k = 1024, 2
    s = pc.Setup(backend, n, k)
    ctx, dev = s.ctx, backend.dev
    kr = s.kr
    good = dict(s=dev(kr["s"]), a=dev(kr["a"]), e=dev(kr["e"]), a_evk=dev(kr["a_evk"]), e_evk=dev(kr["e_evk"]))
    ctx.keygen(**good)
    for name, bad in (("s", np.zeros(n // 2, np.int32)), ("a", np.zeros((k + 1, n), np.uint32)),
                      ("e", np.zeros((2, n), np.int32)), ("a_evk", np.zeros((k, k, n // 2), np.uint32)),
                      ("e_evk", np.zeros((k + 1, n), np.int32))):
        with pytest.raises(ValueError):
            ctx.keygen(**dict(good, **{name: dev(bad)}))
    with pytest.raises(ValueError):
        ctx.keygen(good["s"], good["a"], good["e"], good["a_evk"], None)
    slots, polys, er, cts = s.encrypt_oracle(2)
    pk, m, u, e1, e2 = dev(s.pk), dev(polys), dev(er["u"]), dev(er["e1"]), dev(er["e2"])
    ctx.encrypt(pk, m, u, e1, e2)
    with pytest.raises(ValueError):
        ctx.encrypt(dev(np.zeros((2, k, n // 2), np.uint32)), m, u, e1, e2)
    with pytest.raises(ValueError):
        ctx.encrypt(pk, m, dev(er["u"][:1]), e1, e2)
    with pytest.raises(ValueError):
        ctx.encrypt(pk, m, u, e1, dev(np.zeros((2, n + 4), np.int32)))
    dcts = dev(cts)
    with pytest.raises(ValueError):
        ctx.decrypt(dev(np.zeros(n + 1, np.int32)), dcts)
    with pytest.raises(ValueError):
        ctx.noise_bits(dev(np.zeros((1, n), np.int32)), dcts)
    ctx.set_relin_key(dev(s.evk))
    with pytest.raises(ValueError):
        ctx.ct_mul_relin(dcts, dcts, out=dev(np.zeros((1, 2, k, n), np.uint32)))
    with pytest.raises(ValueError):
        ctx.ct_square_relin(dcts, out=dev(np.zeros((3, 2, k, n), np.uint32)))
    idx, w = dev(np.array([[0, 1]], np.uint32)), dev(np.ones((1, 1, 2), np.int32))
    with pytest.raises(ValueError):
        ctx.ct_scalar_mac(dcts, idx, w, 1, out=dcts[:1].reshape((1, 1, 2, k, n)))        # overlaps its input
    with pytest.raises(ValueError):
        ctx.ct_scalar_mac(dcts, idx, dev(np.ones((1, 1, 3), np.int32)), 1)
    ctx.close()
