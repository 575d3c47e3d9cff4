"""Parity of the HIP path with the CPU oracle on a real MI355X, through the C ABI
(torch only allocates the device buffers).  Bit-exact: all of it is integer work."""
import sys
import time

import numpy as np
import pytest

import parity_cases as pc
from oracle import fv
from workloads import generators as gen

pytestmark = pytest.mark.gpu


def say(msg):
    print("[gpu-parity] " + msg, flush=True)
    sys.stdout.flush()


class GpuBackend:
    def __init__(self):
        from paper_1811_00778_amd import binding
        self.binding = binding
        self.lib = binding.lib()
        self._ctx = None

    def make_ctx(self, n, q, p, t):
        self._ctx = self.binding.Context(n, q, p, t)
        return self._ctx

    def dev(self, a):
        return self._ctx.to_device(np.ascontiguousarray(a))

    def host(self, buf):
        return self._ctx.to_host_u32(buf)


@pytest.fixture(scope="module")
def backend():
    return GpuBackend()


@pytest.mark.parametrize("n,k,n_polys,rows", [(1024, 2, 16, None), (2048, 3, 5, 4), (4096, 2, 3, 2),
                                             (8192, 8, 7, 3), (16384, 3, 2, 2), (32768, 2, 160, 2)])
def test_ntt_all_sizes(backend, n, k, n_polys, rows):
    say("ntt n=%d k=%d polys=%d" % (n, k, n_polys))
    pc.check_ntt(backend, n, k, n_polys, rows)


@pytest.mark.parametrize("n,k", [(1024, 2), (2048, 3)])
def test_keygen_encrypt_decrypt(backend, n, k):
    say("keygen/encrypt/decrypt n=%d k=%d" % (n, k))
    pc.check_keygen_encrypt_decrypt(backend, n, k)


@pytest.mark.parametrize("n,k", [(1024, 2), (2048, 5)])
def test_scalar_mac(backend, n, k):
    say("scalar_mac n=%d k=%d" % (n, k))
    pc.check_scalar_mac(backend, n, k)
    pc.check_mac_linear_in_ntt_domain(backend, n, k)


def test_square_relin_tiny_config(backend):
    say("square_relin n=1024 k=2")
    pc.check_square_relin(backend, 1024, 2)


def test_square_relin_chunked_ragged(backend):
    say("square_relin chunked n=1024 k=3")
    pc.check_square_relin(backend, 1024, 3, n_random=4, n_genuine=1, chunk=2)
    pc.check_square_relin(backend, 1024, 3, n_random=5, n_genuine=1)      # one group of four sharing key loads + two singles
    pc.check_square_relin(backend, 1024, 3, n_random=2, n_genuine=0, chunk=2, relin_order=1)   # ciphertext-major order forced
    pc.check_square_relin(backend, 8192, 2, n_random=6, n_genuine=0, relin_order=2)            # key-major order


def test_square_relin_largest_rings_residue_exact(backend):
    """Whole squarings at n = 16384 and n = 32768 against the oracle residue by residue; two primes keep the
    oracle's O(n^2) products to seconds (the full-size configurations have tests of their own below)."""
    say("square_relin n=16384 k=2, n=32768 k=2 and k=6, every residue")
    pc.check_square_relin(backend, 16384, 2, n_random=1, n_genuine=1, check_decrypt=False)   # a 60-bit q has no room for the result's noise
    pc.check_square_relin(backend, 32768, 2, n_random=1, n_genuine=0)
    pc.check_square_relin(backend, 32768, 6, n_random=1, n_genuine=0)


def test_square_relin_whole_rounds_plus_remainder(backend):
    """A batch that the default policy splits: whole rounds of the one-kernel relinearisation (sized from the
    occupancy that the runtime reports for the compiled kernel), the rest through the separate kernels.  Sampled
    ciphertexts against the oracle, every ciphertext against the two forced forms."""
    n, k = 4096, 4
    s = pc.Setup(backend, n, k)
    s.ctx.set_relin_key(backend.dev(s.evk))
    rnd = s.ctx.relin_fused_round()
    say("square_relin n=4096 k=4: one round of %d ciphertexts in one kernel + three through the separate kernels" % rnd)
    assert 8 <= rnd <= 2048
    n_ct = rnd + 3
    cts = gen.uniform_residues(s.rng, s.q, n, lead=(n_ct, 2))
    dev = backend.dev(cts)
    s.ctx.set_profile(True)
    out = backend.host(s.ctx.ct_square_relin(dev))
    prof = s.ctx.profile()
    assert prof["relin_fused"][0] == 1 and prof["relin_fused"][1] == rnd * k * (k + 2)
    assert prof["relin_mac"][0] == 1                       # three singles
    s.ctx.set_profile(False)
    for i in (0, rnd // 2 + 3, rnd - 1, rnd, rnd + 2):
        assert np.array_equal(out[i], fv.square_relin(s.octx, cts[i], s.evk)), i
    for mode in (1, 2):
        s.ctx.set_fusion(mode)
        assert np.array_equal(backend.host(s.ctx.ct_square_relin(dev)), out), mode
    s.ctx.close()


@pytest.mark.parametrize("n,k", [(8192, 3), (8192, 5), (8192, 7), (8192, 9), (8192, 12), (4096, 6), (16384, 3), (16384, 5)])
def test_square_relin_every_form_at_the_large_rings(backend, n, k):
    """Whole ciphertexts against the oracle at the ring sizes of the paper's parameter sets with prime counts off
    the specialised base-conversion sizes; default policy, one-kernel forms and separate kernels each."""
    say("square_relin, all forms, n=%d k=%d" % (n, k))
    pc.check_square_relin(backend, n, k, n_random=1, n_genuine=1, seed_id=k, check_decrypt=not (n == 16384 and k < 5))


def test_square_relin_exact_comparison_path(backend):
    say("square_relin forced exact comparison")
    pc.check_square_relin(backend, 1024, 2, force_exact=True)
    pc.check_square_relin(backend, 2048, 4, n_random=1, n_genuine=1, force_exact=True)


def test_square_relin_more_than_16_limbs(backend):
    say("square_relin k=17")
    pc.check_square_relin(backend, 1024, 17, n_random=1, n_genuine=1)


@pytest.mark.parametrize("k,k_aux,big_t", [(3, 4, False), (5, 6, False), (6, 7, False), (7, 8, False), (8, 9, False),
                                           (9, 10, False), (10, 11, False), (11, 12, False), (12, 13, False),
                                           (4, 6, True), (6, 8, True), (8, 10, True), (10, 12, True), (11, 13, True),
                                           (12, 14, True), (14, 16, True), (16, 18, True), (24, 26, True)])
def test_square_relin_register_variants_of_standard_bases(backend, k, k_aux, big_t):
    say("square_relin n=1024 k=%d k_aux=%d" % (k, k_aux))
    t = pc.slot_prime_above(1024, 1 << 22) if big_t else 65537
    pc.check_square_relin(backend, 1024, k, n_random=1, n_genuine=1, t=t, expect_k_aux=k_aux)
    pc.check_square_relin(backend, 1024, k, n_random=1, n_genuine=0, t=t, force_exact=True)


def test_general_hmult(backend):
    say("mul_relin")
    pc.check_mul_relin(backend, 1024, 2)
    pc.check_mul_relin(backend, 2048, 3, force_exact=True)
    pc.check_mul_relin(backend, 1024, 8)
    pc.check_mul_relin(backend, 32768, 2, check_decrypt=False)     # a 60-bit q has no room for the product's noise


def test_conv_square_layer(backend):
    say("conv + square small layer")
    pc.check_conv_layer_small(backend)


def test_hot_path_under_graph_capture(backend):
    """Scalar MAC + squaring recorded into a HIP graph on a side stream and replayed: every replay, with eager
    work and synchronisations between the replays, must reproduce the eager result bit for bit."""
    import torch
    say("graph capture of scalar MAC + squaring, three replays")
    for n, k in ((4096, 4), (16384, 2)):            # the second size uses kernels with more than 48 KiB of LDS
        _graph_capture_case(backend, n, k)


def _graph_capture_case(backend, n, k):
    import torch
    s = pc.Setup(backend, n, k, seed_id=2, stream=41)
    ctx, dev = s.ctx, backend.dev
    ctx.set_relin_key(dev(s.evk))
    cts = dev(gen.uniform_residues(s.rng, s.q, n, lead=(6, 2)))
    idx = dev(np.array([[0, 1, 2], [3, 4, 5]], dtype=np.uint32))
    w = dev(np.array([[[1, -2, 3], [4, 5, -6]], [[-7, 8, 9], [1, 1, 1]]], dtype=np.int32))
    eager_mac = ctx.ct_scalar_mac(cts, idx, w, 9)
    eager_sq = ctx.ct_square_relin(eager_mac.reshape((4, 2, k, n)))
    if n <= 4096:
        want = np.stack([fv.square_relin(s.octx, backend.host(eager_mac.reshape((4, 2, k, n)))[i], s.evk) for i in (0, 3)])
        assert np.array_equal(backend.host(eager_sq)[[0, 3]], want)
    g_mac, g_sq = torch.zeros_like(eager_mac), torch.zeros_like(eager_sq)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        ctx.use_stream(side)
        ctx.ct_square_relin(ctx.ct_scalar_mac(cts, idx, w, 9, out=g_mac).reshape((4, 2, k, n)), out=g_sq)   # warm-up
    side.synchronize()
    with torch.cuda.graph(graph, stream=side):
        ctx.ct_square_relin(ctx.ct_scalar_mac(cts, idx, w, 9, out=g_mac).reshape((4, 2, k, n)), out=g_sq)
    ctx.use_stream()
    for rep in range(3):
        g_mac.zero_(); g_sq.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g_mac, eager_mac) and torch.equal(g_sq, eager_sq), ("replay", rep)
        ctx.ct_square_relin(cts[rep:rep + 2])                     # eager work between the replays
        torch.cuda.synchronize()
    ctx.close()


def test_two_contexts_on_two_streams(backend):
    """Two contexts (two plaintext channels) bound to two HIP streams of default priority work at the same time,
    each with its own scratch memory; both must produce what they produce alone."""
    import torch
    say("two contexts on two streams")
    n, k = 4096, 4
    setups = [pc.Setup(backend, n, k, t=t, seed_id=2, stream=61 + i) for i, t in enumerate((65537, 2424833))]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    cts, alone = [], []
    for s in setups:
        backend._ctx = s.ctx
        s.ctx.set_relin_key(backend.dev(s.evk))
        x = backend.dev(gen.uniform_residues(s.rng, s.q, n, lead=(48, 2)))
        cts.append(x)
        alone.append(s.ctx.ct_square_relin(x).clone())
    torch.cuda.synchronize()
    outs = [torch.zeros_like(a) for a in alone]
    for rep in range(3):
        for s, st, x, o in zip(setups, streams, cts, outs):
            with torch.cuda.stream(st):
                s.ctx.use_stream(st)
                s.ctx.ct_square_relin(x, out=o)
        torch.cuda.synchronize()
        for o, a in zip(outs, alone):
            assert torch.equal(o, a), ("concurrent run", rep)
            o.zero_()
    want = fv.square_relin(setups[1].octx, backend.host(cts[1])[5], setups[1].evk)
    assert np.array_equal(backend.host(alone[1])[5], want)
    for s in setups:
        s.ctx.use_stream()
        s.ctx.close()


def test_random_parameter_sweep(backend):
    say("seeded sweep over 60 random parameter sets and shapes")
    pc.check_random_sweep(backend, 60, seed=20261127)


def test_counter_based_samplers(backend):
    say("samplers n=1024 k=2, n=8192 k=3")
    pc.check_samplers(backend, 1024, 2)
    pc.check_samplers(backend, 8192, 3, seed_id=2)


def test_noise_read_out(backend):
    say("noise read-out n=1024 k=2, n=2048 k=5, n=8192 k=8")
    pc.check_noise_bits(backend, 1024, 2)
    pc.check_noise_bits(backend, 2048, 5)
    pc.check_noise_bits(backend, 8192, 8, seed_id=2)


def test_wide_plaintext_modulus(backend):
    say("43-bit plaintext modulus: n=1024 k=5, n=4096 k=6 with the exact rounding path forced")
    pc.check_wide_plaintext(backend)
    pc.check_wide_plaintext(backend, 4096, 6, seed_id=2, force_exact=True)


def test_plaintext_crt_channels(backend):
    say("two plaintext moduli of the CIFAR-10 parameter set as CRT channels")
    pc.check_crt_channels(backend)


def test_small_network_layer_by_layer(backend):
    say("miniature network (padded conv, square, pooling, fully connected), every layer against the oracle")
    pc.check_small_network(backend)


def test_options_and_profile(backend):
    """Option validation, the per-kernel profile and the counters on a live context."""
    from paper_1811_00778_amd import _capi
    s = pc.Setup(backend, 1024, 2)
    ctx = s.ctx
    with pytest.raises(_capi.HcnnError):
        ctx.set_ambiguity_band(3)                      # below the error bound of the estimate
    with pytest.raises(_capi.HcnnError):
        ctx.set_ambiguity_band(2 ** 27)
    with pytest.raises(_capi.HcnnError):
        ctx.set_relin_order(7)
    with pytest.raises(_capi.HcnnError):
        ctx.ct_square_relin(backend.dev(np.zeros((1, 2, 2, 1024), dtype=np.uint32)))     # no key yet
    ctx.set_relin_key(backend.dev(s.evk))
    ctx.set_profile(True)
    x = backend.dev(gen.uniform_residues(s.rng, s.q, 1024, lead=(3, 2)))
    ctx.ntt_fwd(x); ctx.ntt_inv(x)
    ctx.ct_square_relin(x)
    prof = ctx.profile()
    # three ciphertexts are far from a round of the one-kernel relinearisation: separate kernels
    assert prof["ntt_fwd"][0] == 3 and prof["ntt_fwd"][1] == 3 * 2 * 2 + 3 * 2 * 5 + 3 * 4   # rows: plain, extended, digits
    assert prof["ntt_inv"][0] == 3 and prof["scale"][0] == 1 and prof["base_ext"][0] == 1
    assert prof["relin_mac"][0] == 1 and prof["relin_fused"][0] == 0 and prof["tensor"][0] == 0   # one launch of singles
    assert all(v[2] > 0 for k, v in prof.items() if v[0])
    ctx.reset_stats()
    assert all(v[0] == 0 for v in ctx.profile().values())
    with pytest.raises(_capi.HcnnError):
        ctx.set_fusion(3)
    ctx.set_fusion(2)
    ctx.ct_square_relin(x)
    prof = ctx.profile()
    assert prof["ntt_fwd"][0] == 0 and prof["ntt_inv"][0] == 0 and prof["relin_mac"][0] == 0
    assert prof["tensor"][0] == 1 and prof["tensor"][1] == 3 * 5 * 5                         # 2 forward + 3 inverse rows per (ct, limb)
    assert prof["relin_fused"][0] == 1 and prof["relin_fused"][1] == 3 * 2 * (2 + 2)         # k forward + 2 inverse rows each
    assert ctx.scratch_bytes() > 0
    ctx.close()


def test_measured_ceilings_are_plausible(backend):
    """The diagnostic entry point behind the bench line's `measured_ceilings`: streaming rates below the 8 TB/s of the
    memory and above a tenth of it, instruction-issue rates between a quarter of and twice 256 CU x 64 lanes x 2.4 GHz."""
    from paper_1811_00778_amd import _capi
    s = pc.Setup(backend, 1024, 2, with_keys=False)
    c = s.ctx.measured_ceilings()
    assert set(c) == set(_capi.CEILINGS)
    for name in ("copy_GBps", "read_GBps", "write_GBps"):
        assert 800.0 < c[name] < 8000.0, (name, c[name])
    for name in ("mul_lo_u32_Tops", "mul_hi_u32_Tops", "mad_u64_u32_Tops", "mad_i64_i32_Tops", "add_u32_Tops"):
        assert 9.8 < c[name] < 2 * 39.4, (name, c[name])
    s.ctx.close()


def test_empty_batches_are_noops(backend):
    s = pc.Setup(backend, 1024, 2)
    ctx = s.ctx
    ctx.set_relin_key(backend.dev(s.evk))
    import torch
    empty = torch.empty((0, 2, 2, 1024), dtype=torch.int32, device=ctx.device)
    assert ctx.ct_square_relin(empty).shape[0] == 0
    ctx.ntt_fwd(torch.empty((0, 2, 1024), dtype=torch.int32, device=ctx.device))
    ctx.close()


# ------------------------------------------------------------------ full-size configurations
def _oracle_rows_check(name, got_row, want_row):
    assert np.array_equal(got_row, want_row), name


def test_config2_full_batch_ntt_and_squarings(backend, progress):
    """n=8192, 8 primes, 64 random ciphertexts: transforms on the whole batch (sampled rows against the
    oracle, round trip on everything), 64 squarings in one call (six whole ciphertexts against the oracle,
    residue by residue; every residue of all 64 canonical)."""
    cfg = gen.CONFIGS[2]
    n, k = cfg["n"], cfg["k"]
    say("config 2: setup")
    s = pc.Setup(backend, n, k, seed_id=2)
    cts = gen.uniform_residues(s.rng, s.q, n, lead=(cfg["n_ct"], 2))
    buf = backend.dev(cts)
    s.ctx.ntt_fwd(buf)
    hat = backend.host(buf).copy()
    for (i, b, l) in [(0, 0, 0), (17, 1, 3), (63, 1, 7)]:
        say("config 2: oracle NTT row %s" % ((i, b, l),))
        assert np.array_equal(hat[i, b, l], fv.ntt_forward(cts[i, b, l], s.q[l]))
    s.ctx.ntt_inv(buf)
    assert np.array_equal(backend.host(buf), cts)
    say("config 2: 64 squarings on the GPU")
    s.ctx.set_relin_key(backend.dev(s.evk))
    out = backend.host(s.ctx.ct_square_relin(backend.dev(cts)))
    for l, p in enumerate(s.q):
        assert int(out[:, :, l].max()) < p
    for i in (0, 5, 21, 38, 50, 63):
        t0 = time.time()
        want = fv.square_relin(s.octx, cts[i], s.evk)
        progress("config 2: oracle squaring of ciphertext %d took %.1f s" % (i, time.time() - t0))
        assert np.array_equal(out[i], want), i
    s.ctx.close()


def test_config3_mnist_conv_layer(backend):
    """n=8192, 8 primes: 784 genuinely encrypted pixel ciphertexts (values 0..255 in 8192 slots), 5 filters
    5x5 stride 2 -> 720 outputs by scalar MAC, then 720 squarings.  Sampled outputs against the oracle,
    and the decrypted result against the plain convolution squared."""
    from paper_1811_00778_amd import layers
    cfg = gen.CONFIGS[3]
    n, k, t = cfg["n"], cfg["k"], cfg["t"]
    cv = cfg["conv"]
    say("config 3: setup")
    s = pc.Setup(backend, n, k, seed_id=3)
    n_in = cv["c_in"] * cv["h"] * cv["w"]
    slots = gen.slot_values(s.rng, n_in, n, 256)
    er = gen.encryption_randomness(s.rng, n, n_in)
    say("config 3: slot encoding of 784 images planes (oracle side)")
    polys = np.stack([fv.slot_encode(slots[i], n, t) for i in range(n_in)])
    say("config 3: GPU encryption of 784 ciphertexts")
    dcts = s.ctx.encrypt(backend.dev(s.pk), backend.dev(polys), backend.dev(er["u"]), backend.dev(er["e1"]),
                         backend.dev(er["e2"]))
    cts = backend.host(dcts)
    for i in (0, 500):
        say("config 3: oracle encryption %d" % i)
        assert np.array_equal(cts[i], fv.encrypt(s.octx, s.pk, polys[i], er["u"][i], er["e1"][i], er["e2"][i]))
    weights = gen.int_weights(s.rng, (cv["filters"], cv["c_in"], cv["fh"], cv["fw"]), cv["w_bound"])
    idx, valid, (ho, wo) = layers.conv_index_table(cv["c_in"], cv["h"], cv["w"], cv["fh"], cv["fw"], cv["stride"])
    wt = layers.conv_weight_table(weights, idx.shape[0])
    say("config 3: scalar MAC 784 -> 720")
    mac = s.ctx.ct_scalar_mac(dcts, backend.dev(idx), backend.dev(wt), cv["w_bound"])
    F, G = cv["filters"], ho * wo
    assert F * G == cfg["n_square"]
    hmac = backend.host(mac)
    for (f, g) in [(0, 0), (1, 77), (2, 143), (4, 100), (3, 12), (4, 143)]:
        assert np.array_equal(hmac[f, g], fv.scalar_mac(s.octx, cts, idx[g], wt[g, f])), ("mac", f, g)
    say("config 3: 720 squarings")
    s.ctx.set_relin_key(backend.dev(s.evk))
    sq = backend.host(s.ctx.ct_square_relin(mac.reshape((F * G, 2, k, n))))
    o = 2 * G + 143
    t0 = time.time()
    want = fv.square_relin(s.octx, hmac[2, 143], s.evk)
    say("config 3: oracle squaring took %.1f s" % (time.time() - t0))
    assert np.array_equal(sq[o], want)
    img = slots.astype(np.int64).reshape(cv["c_in"], cv["h"], cv["w"], n)
    for (f, j, kk) in [(0, 0, 0), (4, 11, 11)]:
        acc = np.zeros(n, dtype=np.int64)
        for c in range(cv["c_in"]):
            for dy in range(cv["fh"]):
                for dx in range(cv["fw"]):
                    acc += int(weights[f, c, dy, dx]) * img[c, j * cv["stride"] + dy, kk * cv["stride"] + dx]
        got = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], sq[f * G + j * wo + kk]), n, t)
        assert np.array_equal(got.astype(np.int64), (acc % t) ** 2 % t), ("conv^2", f, j, kk)
    s.ctx.close()


def _gpu_encrypt_random_plaintexts(backend, s, count, batch=256):
    """`count` genuine encryptions of uniformly drawn plaintext polynomials (coefficients in [0,t)),
    made on the GPU in batches; returns (device ciphertexts, host plaintext polynomials, randomness)."""
    import torch
    n = s.n
    polys = s.rng.integers(0, s.t, size=(count, n), dtype=np.int64).astype(np.uint32)
    er = gen.encryption_randomness(s.rng, n, count)
    out = torch.empty((count, 2, s.k, n), dtype=torch.int32, device=s.ctx.device)
    dpk = backend.dev(s.pk)
    for c0 in range(0, count, batch):
        sl = slice(c0, min(count, c0 + batch))
        out[sl] = s.ctx.encrypt(dpk, backend.dev(polys[sl]), backend.dev(er["u"][sl]), backend.dev(er["e1"][sl]),
                                backend.dev(er["e2"][sl]))
    return out, polys, er


def test_config4_cifar_conv_layer(backend, progress):
    """n=16384, 16 primes: 3072 encrypted inputs, 8 filters 3x3x3 stride 2 -> 1800 outputs, 1800 squarings.
    Sampled MAC outputs and four whole squarings against the oracle, residue by residue; the decrypted result
    of another output against the plain convolution squared."""
    from paper_1811_00778_amd import layers
    cfg = gen.CONFIGS[4]
    n, k, t = cfg["n"], cfg["k"], cfg["t"]
    cv = cfg["conv"]
    say("config 4: setup (k_aux follows from t*n*q)")
    s = pc.Setup(backend, n, k, seed_id=4)
    assert len(s.p) == k + 2
    n_in = cv["c_in"] * cv["h"] * cv["w"]
    say("config 4: GPU encryption of %d ciphertexts" % n_in)
    dcts, polys, er = _gpu_encrypt_random_plaintexts(backend, s, n_in)
    i = 1234
    t0 = time.time()
    want = fv.encrypt(s.octx, s.pk, polys[i], er["u"][i], er["e1"][i], er["e2"][i])
    say("config 4: oracle encryption took %.1f s" % (time.time() - t0))
    assert np.array_equal(backend.host(dcts[i]), want)
    weights = gen.int_weights(s.rng, (cv["filters"], cv["c_in"], cv["fh"], cv["fw"]), cv["w_bound"])
    idx, valid, (ho, wo) = layers.conv_index_table(cv["c_in"], cv["h"], cv["w"], cv["fh"], cv["fw"], cv["stride"])
    wt = layers.conv_weight_table(weights, idx.shape[0])
    F, G = cv["filters"], ho * wo
    assert F * G == cfg["n_square"] and idx.shape[1] == 27
    say("config 4: scalar MAC %d -> %d" % (n_in, F * G))
    mac = s.ctx.ct_scalar_mac(dcts, backend.dev(idx), backend.dev(wt), cv["w_bound"])
    for (f, g) in [(0, 0), (7, G - 1), (3, 100)]:
        need = sorted(set(int(v) for v in idx[g]))
        sub = {v: backend.host(dcts[v]) for v in need}
        local = np.stack([sub[int(v)] for v in idx[g]])
        want = fv.scalar_mac(s.octx, local, list(range(len(idx[g]))), wt[g, f])
        assert np.array_equal(backend.host(mac[f, g]), want), ("mac", f, g)
    say("config 4: %d squarings" % (F * G))
    s.ctx.set_relin_key(backend.dev(s.evk))
    flat = mac.reshape((F * G, 2, k, n))
    sq = s.ctx.ct_square_relin(flat)
    # decrypted output (f, j, kk) against the plain layer on the slot values of its 27 inputs
    f, j, kk = 5, 7, 9
    g = j * wo + kk
    slots = {int(v): fv.slot_decode(polys[int(v)], n, t).astype(np.int64) for v in idx[g]}
    acc = np.zeros(n, dtype=np.int64)
    for tau, v in enumerate(idx[g]):
        acc += int(wt[g, f, tau]) * slots[int(v)]
    t0 = time.time()
    got = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], backend.host(sq[f * G + g])), n, t)
    say("config 4: oracle decryption took %.1f s" % (time.time() - t0))
    assert np.array_equal(got.astype(np.int64), (acc % t) ** 2 % t)
    # four whole squarings (first and last output of the layer and two in between), residue for residue
    for o in (0, 2 * G + 17, 5 * G + 101, F * G - 1):
        t0 = time.time()
        want = fv.square_relin(s.octx, backend.host(flat[o]), s.evk)
        progress("config 4: oracle squaring of output %d took %.1f s" % (o, time.time() - t0))
        assert np.array_equal(backend.host(sq[o]), want), o
    s.ctx.close()


def _golden_square_hashes():
    """{(name, b, l): sha256} of tests/golden/config5_square_sha256.txt (written by the oracle alone)."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config5_square_sha256.txt")
    table = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, b, l, h = line.split()
        table[(name, int(b), int(l))] = h
    return table


def test_config5_deep_modulus(backend, progress):
    """n=32768, 24 primes (26 auxiliary): 32 squarings with relinearisation and a 1024 -> 10 scalar MAC.
    Squarings: one ciphertext of random residues against the oracle run here, residue by residue; that and a
    genuine one against the stored hashes of the oracle's output rows; the genuine one also through oracle
    decryption (slot-wise square); every residue of all 32 canonical.  The MAC is compared residue for residue."""
    import hashlib
    import torch
    from paper_1811_00778_amd import layers
    cfg = gen.CONFIGS[5]
    n, k, t = cfg["n"], cfg["k"], cfg["t"]
    say("config 5: setup")
    s = pc.Setup(backend, n, k, seed_id=5)
    assert len(s.p) == k + 2
    s.ctx.set_relin_key(backend.dev(s.evk))
    say("config 5: inputs (2 genuine + 30 random ciphertexts)")
    dgen, polys, er = _gpu_encrypt_random_plaintexts(backend, s, 2)
    t0 = time.time()
    want = fv.encrypt(s.octx, s.pk, polys[1], er["u"][1], er["e1"][1], er["e2"][1])
    say("config 5: oracle encryption took %.1f s" % (time.time() - t0))
    assert np.array_equal(backend.host(dgen[1]), want)
    rnd = gen.uniform_residues(s.rng, s.q, n, lead=(30, 2))
    batch = torch.cat([dgen, backend.dev(rnd)])
    say("config 5: 32 squarings")
    sq = s.ctx.ct_square_relin(batch)
    hsq = backend.host(sq)
    for l, p in enumerate(s.q):
        assert int(hsq[:, :, l].max()) < p, ("canonical residues", l)
    # stored hashes of the oracle's output rows (tests/golden/make_square_golden.py draws the same inputs)
    golden = _golden_square_hashes()
    for name, i in (("genuine", 1), ("random", 2 + 17)):
        for b in range(2):
            for l in range(k):
                got = hashlib.sha256(np.ascontiguousarray(hsq[i, b, l], dtype="<u4").tobytes()).hexdigest()
                assert got == golden[(name, b, l)], ("config 5 squaring row", name, b, l)
    # the oracle itself, now, on another ciphertext of random residues
    t0 = time.time()
    progress("config 5: oracle squaring of one ciphertext (n = 32768, 24 primes) started")
    want = fv.square_relin(s.octx, rnd[5], s.evk)
    progress("config 5: oracle squaring took %.1f s" % (time.time() - t0))
    assert np.array_equal(hsq[2 + 5], want)
    t0 = time.time()
    got = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], hsq[1]), n, t)
    say("config 5: oracle decryption took %.1f s" % (time.time() - t0))
    m = fv.slot_decode(polys[1], n, t).astype(np.uint64)
    assert np.array_equal(got, (m * m % t).astype(np.uint32))
    del hsq
    # determinism across chunkings of the batch: same residues when squared four at a time
    s.ctx.set_square_chunk(4)
    sq4 = s.ctx.ct_square_relin(batch)
    assert torch.equal(sq, sq4)
    del sq4, batch, sq
    say("config 5: fully connected MAC 1024 -> 10")
    fc = cfg["fc"]
    cts = gen.uniform_residues(s.rng, s.q, n, lead=(fc["n_in"], 2))
    w = gen.int_weights(s.rng, (fc["n_out"], fc["n_in"]), fc["w_bound"])
    out = s.ctx.ct_scalar_mac(backend.dev(cts), backend.dev(layers.fc_index_table(fc["n_in"])),
                              backend.dev(layers.fc_weight_table(w)), fc["w_bound"])
    for o in (0, 9):
        t0 = time.time()
        want = fv.scalar_mac(s.octx, cts, list(range(fc["n_in"])), w[o])
        say("config 5: oracle MAC output %d took %.1f s" % (o, time.time() - t0))
        assert np.array_equal(backend.host(out[o, 0]), want)
    s.ctx.close()
