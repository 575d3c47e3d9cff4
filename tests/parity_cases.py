"""Parity cases shared by the CPU checker of the kernel sources (tests/emu.py) and the
GPU tests: each function drives the C ABI through a backend and compares with the
oracle element by element (bit-exact: everything here is integer work).

A backend provides
    lib                 the loaded C library (for the host-only helpers)
    make_ctx(n,q,p,t)   context object with the OpsMixin methods
    dev(np_array)       buffer usable by the context (device tensor / aligned ndarray)
    host(buffer)        numpy uint32 view of the buffer's contents
"""
import numpy as np

from oracle import fv
from paper_1811_00778_amd import _capi, layers
from workloads import generators as gen


class Setup:
    """Moduli from the library's own rule, checked against the oracle's rule, plus keys from the oracle."""

    def __init__(self, backend, n, k, t=65537, seed_id=1, stream=0, with_keys=True):
        self.b, self.n, self.k, self.t = backend, n, k, t
        cand = _capi.gen_primes(backend.lib, n, k + min(32, k + 8))
        assert cand == fv.ntt_primes(n, len(cand))
        self.q = cand[:k]
        k_aux = _capi.min_aux_count(backend.lib, n, self.q, t, cand[k:])
        self.p = cand[k:k + k_aux]
        Q, P = 1, 1
        for v in self.q:
            Q *= v
        for v in self.p:
            P *= v
        assert P > t * n * Q + 1                       # enough range for the scaled tensor
        assert k_aux == 1 or P // self.p[-1] <= t * n * Q + 1   # and minimal
        self.octx = fv.Context(n, self.q, t)
        self.ctx = backend.make_ctx(n, self.q, self.p, t)
        self.rng = gen.rng_for(seed_id, stream)
        if with_keys:
            self.kr = gen.key_randomness(self.rng, self.q, n)
            self.pk, self.evk = fv.keygen(self.octx, self.kr["s"], self.kr["a"], self.kr["e"],
                                          self.kr["a_evk"], self.kr["e_evk"])

    def encrypt_oracle(self, count, high=None):
        high = self.t if high is None else high
        slots = gen.slot_values(self.rng, count, self.n, high)
        er = gen.encryption_randomness(self.rng, self.n, count)
        polys = np.stack([fv.slot_encode(slots[i], self.n, self.t) for i in range(count)])
        cts = np.stack([fv.encrypt(self.octx, self.pk, polys[i], er["u"][i], er["e1"][i], er["e2"][i])
                        for i in range(count)])
        return slots, polys, er, cts


def check_ntt(backend, n, k, n_polys, sample_rows, seed_id=1):
    s = Setup(backend, n, k, seed_id=seed_id, with_keys=False)
    x = gen.uniform_residues(s.rng, s.q, n, lead=(n_polys,))
    # corner values: 0, 1, p-1 in a few positions of the first polynomial
    for l, p in enumerate(s.q):
        x[0, l, 0], x[0, l, 1], x[0, l, n - 1] = 0, 1, p - 1
    buf = backend.dev(x)
    s.ctx.ntt_fwd(buf)
    got = backend.host(buf).copy()
    rows = [(i, l) for i in range(n_polys) for l in range(k)]
    pick = rows if sample_rows is None or sample_rows >= len(rows) else \
        [rows[j] for j in sorted(set(np.linspace(0, len(rows) - 1, sample_rows).astype(int).tolist()))]
    for i, l in pick:
        assert np.array_equal(got[i, l], fv.ntt_forward(x[i, l], s.q[l])), ("ntt_fwd", n, i, l)
    for l, p in enumerate(s.q):
        assert int(got[:, l].max()) < p                       # canonical residues
    s.ctx.ntt_inv(buf)
    assert np.array_equal(backend.host(buf), x), ("ntt roundtrip", n)
    # inverse alone against the oracle's interpolation on one row
    y = gen.uniform_residues(s.rng, s.q, n, lead=(1,))
    buf = backend.dev(y)
    s.ctx.ntt_inv(buf)
    assert np.array_equal(backend.host(buf)[0, k - 1], fv.ntt_inverse(y[0, k - 1], s.q[k - 1])), ("ntt_inv", n)
    s.ctx.close()


def check_keygen_encrypt_decrypt(backend, n, k, count=3, seed_id=1):
    s = Setup(backend, n, k, seed_id=seed_id)
    kr = s.kr
    gpk, gevk = s.ctx.keygen(backend.dev(kr["s"]), backend.dev(kr["a"]), backend.dev(kr["e"]),
                             backend.dev(kr["a_evk"]), backend.dev(kr["e_evk"]))
    assert np.array_equal(backend.host(gpk), s.pk), "keygen pk"
    assert np.array_equal(backend.host(gevk), s.evk), "keygen evk"
    slots, polys, er, cts = s.encrypt_oracle(count)
    gcts = s.ctx.encrypt(backend.dev(s.pk), backend.dev(polys), backend.dev(er["u"]), backend.dev(er["e1"]),
                         backend.dev(er["e2"]))
    assert np.array_equal(backend.host(gcts), cts), "encrypt"
    got = backend.host(s.ctx.decrypt(backend.dev(kr["s"]), gcts))
    assert np.array_equal(got, polys), "decrypt(encrypt)"
    want = np.stack([fv.decrypt(s.octx, kr["s"], cts[i]) for i in range(count)])
    assert np.array_equal(got, want), "decrypt vs oracle"
    # decrypt of noise-saturated (uniform) ciphertexts still has a defined value
    rnd = gen.uniform_residues(s.rng, s.q, n, lead=(2, 2))
    got = backend.host(s.ctx.decrypt(backend.dev(kr["s"]), backend.dev(rnd)))
    want = np.stack([fv.decrypt(s.octx, kr["s"], rnd[i]) for i in range(2)])
    assert np.array_equal(got, want), "decrypt random"
    s.ctx.close()


def check_scalar_mac(backend, n, k, seed_id=1):
    s = Setup(backend, n, k, seed_id=seed_id, with_keys=False)
    n_in = 9
    cts = gen.uniform_residues(s.rng, s.q, n, lead=(n_in, 2))
    for l, p in enumerate(s.q):                      # extreme residues
        cts[0, 0, l, :8] = p - 1
        cts[1, 1, l, :8] = 0
    dcts = backend.dev(cts)

    def run(idx, w, bound):
        out = backend.host(s.ctx.ct_scalar_mac(dcts, backend.dev(idx), backend.dev(w), bound))
        G, F, T = w.shape
        assert out.shape == (F, G, 2, k, n)
        for g in range(G):
            for f in range(F):
                assert np.array_equal(out[f, g], fv.scalar_mac(s.octx, cts, idx[g], w[g, f])), ("mac", g, f)

    # small weights, several filters, repeated indices, ragged group count
    idx = s.rng.integers(0, n_in, size=(3, 7)).astype(np.uint32)
    run(idx, gen.int_weights(s.rng, (3, 5, 7), 15), 15)
    # T = 1, F = 1 and F = 16
    run(idx[:, :1].copy(), gen.int_weights(s.rng, (3, 1, 1), 8), 8)
    run(idx[:1].copy(), gen.int_weights(s.rng, (1, 16, 7), 31), 31)
    # extreme weights force intermediate reductions of the partial sums (2 terms per reduction)
    big = 2 ** 31 - 1
    w = gen.int_weights(s.rng, (2, 2, 7), big)
    w[0, 0, :] = big
    w[0, 1, :] = -big
    run(idx[:2].copy(), w, big)
    # large (not extreme) weights: the staged kernel reduces its partial sums every 4 terms
    mid = 2 ** 29
    idx40 = s.rng.integers(0, n_in, size=(2, 41)).astype(np.uint32)
    w40 = gen.int_weights(s.rng, (2, 3, 41), mid)
    w40[1, 2, :] = -mid
    run(idx40, w40, mid)
    # rows of 27 and 9 terms (padded by one and by three terms; at up to 8 filters the form that skips the padding
    # terms' multiply-adds), with partial sums reduced every 4 terms and with small weights
    idx27 = s.rng.integers(0, n_in, size=(2, 27)).astype(np.uint32)
    w27 = gen.int_weights(s.rng, (2, 8, 27), mid)
    w27[0, 7, :] = mid
    run(idx27, w27, mid)
    run(idx27[:, :9].copy(), gen.int_weights(s.rng, (2, 3, 9), 7), 7)
    # a gather row too long for the LDS-staged kernel takes the direct variant ((1+F)*T*4 > 64 KiB)
    long_idx = s.rng.integers(0, n_in, size=(1, 5000)).astype(np.uint32)
    run(long_idx, gen.int_weights(s.rng, (1, 3, 5000), 100), 100)
    # all-zero weights and bound 0
    run(idx[:1].copy(), np.zeros((1, 2, 7), dtype=np.int32), 0)
    assert s.ctx.bad_inputs() == 0
    # out-of-range index / weight beyond the bound are skipped and counted, without faulting
    bad_idx = idx[:1].copy()
    bad_idx[0, 2] = n_in + 5
    w1 = gen.int_weights(s.rng, (1, 1, 7), 3)
    out = backend.host(s.ctx.ct_scalar_mac(dcts, backend.dev(bad_idx), backend.dev(w1), 3))
    keep = [j for j in range(7) if j != 2]
    assert np.array_equal(out[0, 0], fv.scalar_mac(s.octx, cts, bad_idx[0, keep], w1[0, 0, keep]))
    assert s.ctx.bad_inputs() == 1
    w1[0, 0, 4] = 99
    out = backend.host(s.ctx.ct_scalar_mac(dcts, backend.dev(idx[:1].copy()), backend.dev(w1), 3))
    keep = [j for j in range(7) if j != 4]
    assert np.array_equal(out[0, 0], fv.scalar_mac(s.octx, cts, idx[0, keep], w1[0, 0, keep]))
    assert s.ctx.bad_inputs() == 2
    s.ctx.close()


def check_mac_linear_in_ntt_domain(backend, n, k, seed_id=1):
    """MAC of transformed inputs equals the transform of the MAC."""
    s = Setup(backend, n, k, seed_id=seed_id, with_keys=False)
    cts = gen.uniform_residues(s.rng, s.q, n, lead=(4, 2))
    idx = np.array([[0, 1, 2, 3]], dtype=np.uint32)
    w = gen.int_weights(s.rng, (1, 2, 4), 15)
    a = s.ctx.ct_scalar_mac(backend.dev(cts), backend.dev(idx), backend.dev(w), 15)
    s.ctx.ntt_fwd(a)
    hat = backend.dev(cts)
    s.ctx.ntt_fwd(hat)
    b = s.ctx.ct_scalar_mac(hat, backend.dev(idx), backend.dev(w), 15)
    assert np.array_equal(backend.host(a), backend.host(b))
    s.ctx.close()


def slot_prime_above(n, lower):
    """Smallest prime t > lower with t = 1 (mod 2n) (a plaintext modulus that still supports slots)."""
    t = lower - lower % (2 * n) + 2 * n + 1
    while not fv.is_prime(t):
        t += 2 * n
    return t


def check_square_relin(backend, n, k, n_random=2, n_genuine=1, seed_id=1, chunk=None, force_exact=False,
                       check_decrypt=True, t=65537, expect_k_aux=None, relin_order=None):
    s = Setup(backend, n, k, t=t, seed_id=seed_id)
    if relin_order is not None:
        s.ctx.set_fusion(1)             # the order concerns the separate inner-product kernel
        s.ctx.set_relin_order(relin_order)
    if expect_k_aux is not None:
        assert len(s.p) == expect_k_aux
    s.ctx.set_relin_key(backend.dev(s.evk))
    if n_genuine:
        slots, polys, er, gcts = s.encrypt_oracle(n_genuine)
    rnd = gen.uniform_residues(s.rng, s.q, n, lead=(n_random, 2))
    # centred-lift corner cases: residues of 0, +-1 and +-(q-1)/2 in the first coefficients
    Q = s.octx.Q
    for pos, val in enumerate((0, 1, -1, (Q - 1) // 2, -((Q - 1) // 2))):
        for l, p in enumerate(s.q):
            rnd[0, 0, l, pos] = val % p
            rnd[0, 1, l, pos] = (-val) % p
    cts = np.concatenate([gcts, rnd]) if n_genuine else rnd
    if chunk:
        s.ctx.set_square_chunk(chunk)
    if force_exact:
        s.ctx.set_ambiguity_band(2 ** 26)
    out = backend.host(s.ctx.ct_square_relin(backend.dev(cts)))
    want = np.stack([fv.square_relin(s.octx, cts[i], s.evk) for i in range(len(cts))])
    assert np.array_equal(out, want), ("square_relin", n, k)
    if force_exact:
        assert s.ctx.exact_fallbacks() > n          # the exact comparison really ran
    if check_decrypt and n_genuine:
        m2 = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], out[0]), n, s.t)
        assert np.array_equal(m2, (slots[0].astype(np.uint64) ** 2 % s.t).astype(np.uint32))
    # in place
    buf = backend.dev(cts)
    s.ctx.ct_square_relin(buf, out=buf)
    assert np.array_equal(backend.host(buf), want), "square_relin in place"
    if relin_order is None and n <= 16384:
        # the same with relinearisation forced into its one-kernel form (small batches take the separate kernels
        # by default) and into the three separate kernels (the only form for larger rings)
        for mode in (2, 1):
            s.ctx.set_fusion(mode)
            out = backend.host(s.ctx.ct_square_relin(backend.dev(cts)))
            assert np.array_equal(out, want), ("square_relin, relinearisation form", mode, n, k)
        s.ctx.set_fusion(0)
    s.ctx.close()


def check_mul_relin(backend, n, k, seed_id=1, force_exact=False, check_decrypt=True):
    """General HMult on genuine and on uniformly random ciphertext pairs."""
    s = Setup(backend, n, k, seed_id=seed_id, stream=3)
    s.ctx.set_relin_key(backend.dev(s.evk))
    slots, polys, er, gcts = s.encrypt_oracle(2)
    rnd = gen.uniform_residues(s.rng, s.q, n, lead=(3, 2))
    a = np.concatenate([gcts[:1], rnd[:2], rnd[2:3]])
    b = np.concatenate([gcts[1:2], rnd[1:3], rnd[2:3]])          # last pair: a ciphertext with itself
    if force_exact:
        s.ctx.set_ambiguity_band(2 ** 26)
    out = backend.host(s.ctx.ct_mul_relin(backend.dev(a), backend.dev(b)))
    want = np.stack([fv.hmult(s.octx, a[i], b[i], s.evk) for i in range(len(a))])
    assert np.array_equal(out, want), ("mul_relin", n, k)
    assert np.array_equal(out[3], fv.square_relin(s.octx, a[3], s.evk))
    if check_decrypt:
        m = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], out[0]), n, s.t)
        assert np.array_equal(m, (slots[0].astype(np.uint64) * slots[1] % s.t).astype(np.uint32))
    # in place on the first operand, relinearisation forced into its one-kernel form
    s.ctx.set_fusion(2)
    buf = backend.dev(a)
    s.ctx.ct_mul_relin(buf, backend.dev(b), out=buf)
    assert np.array_equal(backend.host(buf), want)
    s.ctx.close()


def check_conv_layer_small(backend, seed_id=1):
    """A small convolution + square layer end to end: 1x6x6 image, 2 filters 3x3 stride 2 (+ one padded)."""
    n, k = 1024, 3
    s = Setup(backend, n, k, seed_id=seed_id, stream=7)
    s.ctx.set_relin_key(backend.dev(s.evk))
    c_in, h, w_, F, fh, fw, stride = 1, 6, 6, 2, 3, 3, 2
    slots, polys, er, cts = s.encrypt_oracle(c_in * h * w_, high=4)
    weights = gen.int_weights(s.rng, (F, c_in, fh, fw), 3)
    idx, valid, (ho, wo) = layers.conv_index_table(c_in, h, w_, fh, fw, stride)
    wt = layers.conv_weight_table(weights, idx.shape[0])
    mac = s.ctx.ct_scalar_mac(backend.dev(cts), backend.dev(idx), backend.dev(wt), 3)
    sq = backend.host(s.ctx.ct_square_relin(mac.reshape((F * ho * wo, 2, k, n))))
    # plain convolution on the slot values, written directly from the layer definition
    img = slots.astype(np.int64).reshape(c_in, h, w_, n)
    for f in range(F):
        for j in range(ho):
            for kk in range(wo):
                acc = np.zeros(n, dtype=np.int64)
                for c in range(c_in):
                    for dy in range(fh):
                        for dx in range(fw):
                            acc += int(weights[f, c, dy, dx]) * img[c, j * stride + dy, kk * stride + dx]
                want = (acc % s.t) ** 2 % s.t
                o = f * ho * wo + j * wo + kk
                got = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], sq[o]), n, s.t)
                assert np.array_equal(got.astype(np.int64), want), ("conv+square", f, j, kk)
    s.ctx.close()


def check_small_network(backend, seed_id=1):
    """A CIFAR-shaped miniature (padded 3x3 convolution, square, 2x2 sum pooling, fully connected) run through
    the network runner; every layer's ciphertexts must equal the oracle's, residue by residue, and the result
    must decrypt to the plain network on the slot values."""
    from oracle import plain_net
    from paper_1811_00778_amd import network
    n, k = 1024, 4
    spec = (("conv", 3, 3, 3, 1, 1), ("square",), ("pool", 2), ("fc", 2))
    in_shape = (2, 4, 4)
    s = Setup(backend, n, k, seed_id=seed_id, stream=9)
    s.ctx.set_relin_key(backend.dev(s.evk))
    n_in = in_shape[0] * in_shape[1] * in_shape[2]
    slots, polys, er, cts = s.encrypt_oracle(n_in, high=16)
    weights = [None if shp is None else gen.int_weights(s.rng, shp, 3)
               for shp in network.weight_shapes(spec, in_shape)]
    plan = network.Plan(spec, in_shape, weights, backend.dev)
    out, kept = plan.run(s.ctx, backend.dev(cts), keep=True)
    # the oracle, layer by layer, on its own previous output
    cur = cts
    prev = in_shape
    for li, (layer, shp) in enumerate(zip(spec, network.shapes(spec, in_shape))):
        if layer[0] == "square":
            cur = np.stack([fv.square_relin(s.octx, cur[i], s.evk) for i in range(cur.shape[0])])
        else:
            if layer[0] == "conv":
                idx, valid, _ = layers.conv_index_table(prev[0], prev[1], prev[2], layer[2], layer[3], layer[4], layer[5])
                wt = layers.conv_weight_table(weights[li], idx.shape[0], valid)
            elif layer[0] == "pool":
                idx, wt, _ = layers.pool_index_table(prev[0], prev[1], prev[2], layer[1])
            else:
                idx = layers.fc_index_table(prev[0] * prev[1] * prev[2])
                wt = layers.fc_weight_table(weights[li])
            G, F, T = wt.shape
            cur = np.stack([fv.scalar_mac(s.octx, cur, idx[g], wt[g, f]) for f in range(F) for g in range(G)])
        assert cur.shape[0] == shp[0] * shp[1] * shp[2]
        assert np.array_equal(backend.host(kept[li]), cur), ("network layer", li, layer)
        prev = shp
    want = plain_net.evaluate(spec, weights, slots.astype(np.int64).reshape(in_shape + (n,)), s.t).reshape(2, n)
    final = backend.host(out)
    for o in range(2):
        got = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], final[o]), n, s.t).astype(np.int64)
        assert np.array_equal(got, want[o]), ("network output", o)
    s.ctx.close()


def check_crt_channels(backend, seed_id=1):
    """Plaintext-space CRT decomposition (Sec. 3.1.2): the same integer computation run as independent
    channels with coprime plaintext moduli t_1, t_2 (the first two of the CIFAR-10 parameter set), then
    recombined.  A fully connected node and a square whose true integer results exceed either modulus but
    not half their product: every channel's ciphertexts equal the oracle's residue by residue, each
    channel decrypts to the result mod t_i, and the CRT map returns the integers themselves."""
    n, k = 1024, 4
    ts = (2424833, 2654209)
    n_in, n_out = 9, 2
    rng = gen.rng_for(seed_id, 21)
    slots = rng.integers(0, 256, size=(n_in, n)).astype(np.int64)          # the same integers in every channel
    weights = gen.int_weights(rng, (n_out, n_in), 15)
    idx = layers.fc_index_table(n_in)
    wt = layers.fc_weight_table(weights)
    true = (weights.astype(np.int64) @ slots) ** 2                           # over Z: up to (9*15*255)^2 ~ 1.2e9
    assert int(true.max()) > max(ts) and 2 * int(true.max()) < ts[0] * ts[1]
    residues = []
    for ch, t in enumerate(ts):
        s = Setup(backend, n, k, t=t, seed_id=seed_id, stream=22 + ch)
        s.ctx.set_relin_key(backend.dev(s.evk))
        er = gen.encryption_randomness(s.rng, n, n_in)
        polys = np.stack([fv.slot_encode(slots[i] % t, n, t) for i in range(n_in)])
        cts = np.stack([fv.encrypt(s.octx, s.pk, polys[i], er["u"][i], er["e1"][i], er["e2"][i]) for i in range(n_in)])
        mac = s.ctx.ct_scalar_mac(backend.dev(cts), backend.dev(idx), backend.dev(wt), 15)
        got = backend.host(s.ctx.ct_square_relin(mac.reshape((n_out, 2, k, n))))
        want = np.stack([fv.square_relin(s.octx, fv.scalar_mac(s.octx, cts, idx[0], wt[0, o]), s.evk) for o in range(n_out)])
        assert np.array_equal(got, want), ("channel ciphertexts", t)
        dec = np.stack([fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], got[o]), n, t) for o in range(n_out)]).astype(np.int64)
        assert np.array_equal(dec, true % t), ("channel plaintext", t)
        residues.append(dec)
        s.ctx.close()
    for o in range(n_out):
        for j in range(0, n, 37):
            assert fv.crt_reconstruct([int(residues[0][o, j]), int(residues[1][o, j])], list(ts)) == int(true[o, j])


def check_noise_bits(backend, n, k, seed_id=1):
    """hcnn_noise_bits against the oracle's exact read-out: fresh ciphertexts, a weighted sum, its square, a
    noise-free ciphertext, the zero ciphertext and noise-saturated (uniformly random) ones."""
    s = Setup(backend, n, k, seed_id=seed_id, stream=31)
    s.ctx.set_relin_key(backend.dev(s.evk))
    slots, polys, er, cts = s.encrypt_oracle(4, high=256)
    w = np.array([[[3, -2, 1, 5]]], dtype=np.int32)
    idx = np.arange(4, dtype=np.uint32)[None, :]
    mac = s.ctx.ct_scalar_mac(backend.dev(cts), backend.dev(idx), backend.dev(w), 5)
    sq = s.ctx.ct_square_relin(mac.reshape((1, 2, k, n)))
    flat = np.stack([s.octx.to_rns([(s.octx.Q // s.t) * int(v) for v in polys[0]]), np.zeros((k, n), dtype=np.uint32)])
    rnd = gen.uniform_residues(s.rng, s.q, n, lead=(2, 2))
    batch = np.concatenate([cts, backend.host(mac).reshape((1, 2, k, n)), backend.host(sq),
                            flat[None], np.zeros((1, 2, k, n), dtype=np.uint32), rnd])
    got = backend.host(s.ctx.noise_bits(backend.dev(s.kr["s"]), backend.dev(batch)))
    want = np.array([fv.noise_bits(s.octx, s.kr["s"], batch[i]) for i in range(batch.shape[0])], dtype=np.uint32)
    assert np.array_equal(got, want), (got, want)
    assert want[7] == 0 and want[4] > want[0] and want[5] > want[4], want   # zero; sum noisier than fresh; square noisier
    s.ctx.close()


WIDE_T = 5522259017729          # the 43-bit plaintext modulus of the MNIST parameter sets (parameter table, Sec. 4.2)


def check_wide_plaintext(backend, n=1024, k=5, seed_id=1, force_exact=False):
    """A plaintext modulus above 2^32 (64-bit plaintext words): encrypt, decrypt, squaring with
    relinearisation and the noise read-out against the oracle, residue by residue and word by word."""
    t = WIDE_T
    s = Setup(backend, n, k, t=t, seed_id=seed_id, stream=51)
    assert len(s.p) == k + 2                                     # t*n has more than 30 bits
    ctx = s.ctx
    if force_exact:
        ctx.set_ambiguity_band(1 << 26)
    ctx.set_relin_key(backend.dev(s.evk))
    count = 3
    polys = s.rng.integers(0, t, size=(count, n), dtype=np.int64).astype(np.uint64)
    er = gen.encryption_randomness(s.rng, n, count)
    cts = np.stack([fv.encrypt(s.octx, s.pk, [int(v) for v in polys[i]], er["u"][i], er["e1"][i], er["e2"][i])
                    for i in range(count)])
    gcts = ctx.encrypt(backend.dev(s.pk), backend.dev(polys), backend.dev(er["u"]), backend.dev(er["e1"]),
                       backend.dev(er["e2"]))
    assert np.array_equal(backend.host(gcts), cts), "wide encrypt"
    dec = backend.host(ctx.decrypt(backend.dev(s.kr["s"]), gcts))
    assert dec.dtype == np.uint64 and np.array_equal(dec, polys), "wide decrypt(encrypt)"
    sq = backend.host(ctx.ct_square_relin(gcts))
    want = np.stack([fv.square_relin(s.octx, cts[i], s.evk) for i in range(count)])
    assert np.array_equal(sq, want), "wide squaring"
    dsq = backend.host(ctx.decrypt(backend.dev(s.kr["s"]), backend.dev(sq)))
    assert np.array_equal(dsq, np.stack([fv.decrypt(s.octx, s.kr["s"], want[i]) for i in range(count)])), "wide decrypt"
    picks = [0, 3, n - 1]
    before = fv.slot_eval(polys, n, t, picks)
    after = fv.slot_eval(dsq, n, t, picks)
    for i in range(count):
        for c in range(len(picks)):
            assert int(after[i, c]) == int(before[i, c]) ** 2 % t, ("slot squares", i, c)
    rnd = gen.uniform_residues(s.rng, s.q, n, lead=(2, 2))
    got = backend.host(ctx.decrypt(backend.dev(s.kr["s"]), backend.dev(rnd)))
    assert np.array_equal(got, np.stack([fv.decrypt(s.octx, s.kr["s"], rnd[i]) for i in range(2)])), "wide decrypt random"
    batch = np.concatenate([cts[:1], sq[:1], rnd[:1]])
    bits = backend.host(ctx.noise_bits(backend.dev(s.kr["s"]), backend.dev(batch)))
    assert [int(b) for b in bits] == [fv.noise_bits(s.octx, s.kr["s"], batch[i]) for i in range(3)], "wide noise"
    # the 32-bit entry points refuse a wide context
    try:
        ctx.raw.call("hcnn_decrypt", ctx._ptr(backend.dev(s.kr["s"])), ctx._ptr(gcts), 1,
                     ctx._ptr(backend.dev(np.zeros((1, n), dtype=np.uint32))))
        raise AssertionError("hcnn_decrypt accepted a wide plaintext modulus")
    except _capi.HcnnError as exc:
        assert exc.code == _capi.ERR["T"]
    ctx.close()


def check_samplers(backend, n, k, seed_id=1):
    """hcnn_sample_* against the oracle's independent implementation of the same counter-based generator, element by
    element; then keys and an encryption made from device samples only decrypt correctly."""
    from oracle import rng
    s = Setup(backend, n, k, seed_id=seed_id, with_keys=False)
    ctx = s.ctx
    seed, polys = 0x1234567887654321 + seed_id, 5
    assert np.array_equal(backend.host(ctx.sample_ternary(seed, 1, polys)).view(np.int32), rng.sample_ternary(seed, 1, polys, n))
    assert np.array_equal(backend.host(ctx.sample_gaussian(seed, 2, polys)).view(np.int32), rng.sample_gaussian(seed, 2, polys, n))
    assert np.array_equal(backend.host(ctx.sample_uniform(seed, 3, polys)), rng.sample_uniform(seed, 3, polys, s.q, n))
    # zero polynomials: nothing is written, nothing fails
    assert backend.host(ctx.sample_ternary(seed, 1, 0)).size == 0
    # the whole key and encryption flow from device samples
    sk = ctx.sample_ternary(seed, 10, 1)
    a = ctx.sample_uniform(seed, 11, 1)
    e = ctx.sample_gaussian(seed, 12, 1)
    a_evk = ctx.sample_uniform(seed, 13, k)
    e_evk = ctx.sample_gaussian(seed, 14, k)
    pk, evk = ctx.keygen(sk[0], a[0], e[0], a_evk, e_evk)
    ctx.set_relin_key(evk)
    m = s.rng.integers(0, s.t, size=(2, n), dtype=np.int64).astype(np.uint32)
    cts = ctx.encrypt(pk, backend.dev(m), ctx.sample_ternary(seed, 20, 2), ctx.sample_gaussian(seed, 21, 2),
                      ctx.sample_gaussian(seed, 22, 2))
    assert np.array_equal(backend.host(ctx.decrypt(sk[0], cts)), m)
    sk_h = backend.host(sk).view(np.int32)[0]
    assert np.array_equal(fv.decrypt(s.octx, sk_h, backend.host(cts)[1]), m[1])
    ctx.close()


def check_random_sweep(backend, iterations, seed, sizes=(1024, 2048, 4096)):
    """Seeded sweep over random parameter sets and shapes: ring degree, number of primes (1..7), plaintext modulus,
    ambiguity band, form of the relinearisation, batch size, gather geometry (groups, filters, terms) and weight bounds up to 2^31 - 1, with
    extreme residues planted in the inputs; squaring, general product, scalar MAC and noise read-out must equal
    the oracle on every draw."""
    rng = np.random.default_rng(seed)
    for it in range(iterations):
        n = int(rng.choice(sizes))
        k = int(rng.integers(1, 8))
        t = int(rng.choice([65537, 2424833, 12289]))
        if (t - 1) % (2 * n):
            t = 65537
        s = Setup(backend, n, k, t=t, seed_id=int(rng.integers(1, 1000)), stream=int(rng.integers(0, 100)))
        s.ctx.set_relin_key(backend.dev(s.evk))
        if rng.random() < 0.3:
            s.ctx.set_ambiguity_band(int(2 ** rng.integers(7, 27)))
        s.ctx.set_fusion(int(rng.integers(0, 3)))
        n_ct = int(rng.integers(1, 7))
        cts = gen.uniform_residues(s.rng, s.q, n, lead=(n_ct, 2))
        for l, p in enumerate(s.q):
            pos = rng.integers(0, n, size=8)
            cts[0, 0, l, pos] = rng.choice([0, 1, p - 1, (p - 1) // 2, (p + 1) // 2], size=8)
        tag = (it, n, k, t, n_ct)
        out = backend.host(s.ctx.ct_square_relin(backend.dev(cts)))
        for i in range(n_ct):
            assert np.array_equal(out[i], fv.square_relin(s.octx, cts[i], s.evk)), ("square",) + tag
        if n_ct >= 2:
            prod = backend.host(s.ctx.ct_mul_relin(backend.dev(cts[:1]), backend.dev(cts[1:2])))
            assert np.array_equal(prod[0], fv.hmult(s.octx, cts[0], cts[1], s.evk)), ("product",) + tag
        G, F, T = int(rng.integers(1, 4)), int(rng.integers(1, 17)), int(rng.integers(1, 40))
        bound = int(rng.choice([1, 7, 255, 2 ** 20, 2 ** 31 - 1]))
        idx = rng.integers(0, n_ct, size=(G, T)).astype(np.uint32)
        w = rng.integers(-bound, bound + 1, size=(G, F, T)).astype(np.int32)
        mac = backend.host(s.ctx.ct_scalar_mac(backend.dev(cts), backend.dev(idx), backend.dev(w), bound))
        g, f = int(rng.integers(0, G)), int(rng.integers(0, F))
        assert np.array_equal(mac[f, g], fv.scalar_mac(s.octx, cts, idx[g], w[g, f])), ("mac", G, F, T, bound) + tag
        bits = backend.host(s.ctx.noise_bits(backend.dev(s.kr["s"]), backend.dev(cts[:1])))
        assert int(bits[0]) == fv.noise_bits(s.octx, s.kr["s"], cts[0]), ("noise",) + tag
        s.ctx.close()
