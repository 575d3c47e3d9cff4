"""Whole HCNN-shaped networks on one GPU with synthetic integer weights, one image per plaintext slot.

MNIST shape (Table 1): conv 5x5x5 stride 2 -> square -> conv 50x5x5x5 stride 2 -> square -> fully connected 800 -> 10.
CIFAR-10 shape (Table 2) at the paper's full widths: three blocks of padded 3x3 convolution (32 / 64 / 128 filters),
square and 2x2 average pooling, then fully connected 2048 -> 256 -> 10; parameter set 5 of Sec. 4.2 (N = 2^13, 300-bit q)
with the first of its ten plaintext moduli, i.e. one CRT channel.

The decrypted outputs must equal the network evaluated in plain integers mod t on the slot values
(every slot for MNIST, sampled slots for CIFAR-10).  Residue-level parity of each operation with the oracle is the
business of test_gpu_parity.py; here the oracle decrypts and supplies the plain network."""
import sys
import time

import numpy as np
import pytest

import parity_cases as pc
from oracle import fv, plain_net
from workloads import generators as gen

pytestmark = pytest.mark.gpu


def say(msg):
    print("[gpu-network] " + msg, flush=True)
    sys.stdout.flush()


def _weights(rng, spec, in_shape, bound):
    from paper_1811_00778_amd import network
    return [None if shp is None else gen.int_weights(rng, shp, bound)
            for shp in network.weight_shapes(spec, in_shape)]


def test_mnist_network_end_to_end():
    import torch
    from test_gpu_parity import GpuBackend
    from paper_1811_00778_amd import network
    backend = GpuBackend()
    n, k, t = 8192, 8, 65537
    s = pc.Setup(backend, n, k, seed_id=3, stream=11)
    ctx, dev = s.ctx, backend.dev
    ctx.set_relin_key(dev(s.evk))
    rng = s.rng
    say("plaintexts and GPU encryption of 784 ciphertexts")
    polys = rng.integers(0, t, size=(784, n), dtype=np.int64).astype(np.uint32)
    er = gen.encryption_randomness(rng, n, 784)
    cts = ctx.encrypt(dev(s.pk), dev(polys), dev(er["u"]), dev(er["e1"]), dev(er["e2"]))
    weights = _weights(rng, network.MNIST_HCNN, network.MNIST_INPUT, 15)
    plan = network.Plan(network.MNIST_HCNN, network.MNIST_INPUT, weights, dev)
    plan.run(ctx, cts)                                   # warm-up (allocator, first launches)
    torch.cuda.synchronize()
    t0 = time.time()
    a5 = plan.run(ctx, cts)
    torch.cuda.synchronize()
    say("encrypted network (1520 squarings): %.1f ms on the GPU" % ((time.time() - t0) * 1e3))
    assert a5.shape[0] == 10
    out = backend.host(a5)

    say("plain evaluation mod t on the slot values")
    slots = np.stack([fv.slot_decode(polys[i], n, t) for i in range(784)]).astype(np.int64)   # [784][n]
    want = plain_net.evaluate(network.MNIST_HCNN, weights, slots.reshape(1, 28, 28, n), t).reshape(10, n)
    say("oracle decryption of the ten outputs")
    for o in range(10):
        got = fv.slot_decode(fv.decrypt(s.octx, s.kr["s"], out[o]), n, t).astype(np.int64)
        assert np.array_equal(got, want[o]), ("network output", o)

    # noise budget after every layer (the quantity plotted in the noise-growth figure of Sec. 5.5): read out on the
    # GPU for every ciphertext of every layer, checked against the oracle on the first ciphertext of each layer
    d_sk = dev(s.kr["s"])
    _, kept = plan.run(ctx, cts, keep=True)
    stages = [("fresh", cts)] + [(layer[0], a) for layer, a in zip(network.MNIST_HCNN, kept)]
    budgets = []
    for name, a in stages:
        bits = backend.host(ctx.noise_bits(d_sk, a))
        assert int(bits[0]) == fv.noise_bits(s.octx, s.kr["s"], backend.host(a[:1])[0]), ("noise read-out", name)
        budgets.append(fv.noise_budget_bits(s.octx, int(bits.max())))
        say("noise budget after %-6s (%4d ciphertexts): %6.1f bits" % (name, a.shape[0], budgets[-1]))
    assert all(b1 > b2 for b1, b2 in zip(budgets, budgets[1:])) and budgets[-1] > 0
    ctx.close()


def test_mnist_network_paper_parameter_set():
    """The MNIST-shaped network at parameter set 1 of Sec. 4.2 as printed: N = 2^13, a 330-bit q (eleven 30-bit
    primes) and the 43-bit plaintext modulus 5522259017729, i.e. a single plaintext channel with 64-bit plaintext
    words.  Outputs decrypted by the oracle, compared with the plain network on sampled slots."""
    import torch
    from test_gpu_parity import GpuBackend
    from paper_1811_00778_amd import network
    backend = GpuBackend()
    n, k, t = 8192, 11, pc.WIDE_T
    s = pc.Setup(backend, n, k, t=t, seed_id=3, stream=13, with_keys=False)
    ctx, dev = s.ctx, backend.dev
    rng = s.rng
    kr = gen.key_randomness(rng, s.q, n)
    pk, evk = ctx.keygen(dev(kr["s"]), dev(kr["a"]), dev(kr["e"]), dev(kr["a_evk"]), dev(kr["e_evk"]))
    ctx.set_relin_key(evk)
    say("parameter set 1: k=%d, k'=%d, t=%d; GPU encryption of 784 ciphertexts from 64-bit plaintext words" % (k, len(s.p), t))
    polys = rng.integers(0, t, size=(784, n), dtype=np.int64).astype(np.uint64)
    er = gen.encryption_randomness(rng, n, 784)
    cts = ctx.encrypt(pk, dev(polys), dev(er["u"]), dev(er["e1"]), dev(er["e2"]))
    weights = _weights(rng, network.MNIST_HCNN, network.MNIST_INPUT, 15)
    plan = network.Plan(network.MNIST_HCNN, network.MNIST_INPUT, weights, dev)
    plan.run(ctx, cts)
    torch.cuda.synchronize()
    t0 = time.time()
    out = plan.run(ctx, cts)
    torch.cuda.synchronize()
    say("encrypted network: %.1f ms on the GPU" % ((time.time() - t0) * 1e3))
    bits = backend.host(ctx.noise_bits(dev(kr["s"]), out))
    say("noise budget left in the outputs: %.1f bits" % fv.noise_budget_bits(s.octx, int(bits.max())))
    host_out = backend.host(out)
    picks = [0, 4097, n - 1]
    say("plain evaluation mod t on %d sampled slots (Python integers)" % len(picks))
    x = fv.slot_eval(polys, n, t, picks).reshape(1, 28, 28, len(picks))
    want = plain_net.evaluate(network.MNIST_HCNN, weights, x, t).reshape(10, len(picks))
    gpu_dec = backend.host(ctx.decrypt(dev(kr["s"]), out))
    for o in range(10):
        m = fv.decrypt(s.octx, kr["s"], host_out[o])
        assert np.array_equal(m, gpu_dec[o]), ("GPU decryption", o)
        got = fv.slot_eval(m[None, :], n, t, picks)[0]
        assert [int(v) for v in got] == [int(v) for v in want[o]], ("network output", o)
    ctx.close()


def test_cifar10_network_full_width_end_to_end():
    import torch
    from test_gpu_parity import GpuBackend
    from paper_1811_00778_amd import network
    backend = GpuBackend()
    n, k, t = 8192, 10, 2424833
    free, _total = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs about 50 GiB of device memory")
    s = pc.Setup(backend, n, k, t=t, seed_id=4, stream=12, with_keys=False)
    ctx, dev = s.ctx, backend.dev
    rng = s.rng
    say("keys on the GPU (key generation is checked against the oracle elsewhere)")
    kr = gen.key_randomness(rng, s.q, n)
    pk, evk = ctx.keygen(dev(kr["s"]), dev(kr["a"]), dev(kr["e"]), dev(kr["a_evk"]), dev(kr["e_evk"]))
    ctx.set_relin_key(evk)
    n_in = 3 * 32 * 32
    say("plaintexts and GPU encryption of %d ciphertexts" % n_in)
    polys = rng.integers(0, t, size=(n_in, n), dtype=np.int64).astype(np.uint32)
    cts = torch.empty((n_in, 2, k, n), dtype=torch.int32, device="cuda")
    for i0 in range(0, n_in, 512):
        er = gen.encryption_randomness(rng, n, 512)
        cts[i0:i0 + 512] = ctx.encrypt(pk, dev(polys[i0:i0 + 512]), dev(er["u"]), dev(er["e1"]), dev(er["e2"]))
    del er
    weights = _weights(rng, network.CIFAR10_HCNN, network.CIFAR10_INPUT, 7)
    say("gather tables")
    plan = network.Plan(network.CIFAR10_HCNN, network.CIFAR10_INPUT, weights, dev)
    torch.cuda.synchronize()
    say("encrypted network: 57344 squarings, about 10.8 million ciphertext-by-scalar products")
    t0 = time.time()
    out = plan.run(ctx, cts)
    torch.cuda.synchronize()
    say("encrypted network: %.2f s on the GPU (cold), exact-rounding fall-backs %d" % (time.time() - t0, ctx.exact_fallbacks()))
    assert out.shape[0] == 10
    host_out = backend.host(out)
    del out
    torch.cuda.empty_cache()

    picks = [0, 1, 4097, 7000, n - 1]
    say("plain evaluation mod t on %d sampled slots" % len(picks))
    x = fv.slot_eval(polys, n, t, picks).reshape(3, 32, 32, len(picks))
    want = plain_net.evaluate(network.CIFAR10_HCNN, weights, x, t).reshape(10, len(picks))
    say("oracle decryption of the ten outputs")
    for o in range(10):
        m = fv.decrypt(s.octx, kr["s"], host_out[o])
        got = fv.slot_eval(m[None, :], n, t, picks)[0]
        assert np.array_equal(got, want[o]), ("network output", o, got, want[o])
    ctx.close()


def test_cifar10_network_ten_crt_channels():
    """The CIFAR-10-shaped network as the paper deploys it (Sec. 3.1.2, parameter set 5): ten independent plaintext
    channels, one per modulus of the parameter table, whose decrypted outputs are recombined by the CRT map into the
    integers the network produces over Z (up to ~180 bits here, far beyond any single modulus).  Every input
    ciphertext encrypts a constant polynomial (the pixel value in every slot), so the same integers enter every
    channel without slot encoding; the expected integers come from the plain network evaluated in Python integers."""
    import os
    import torch
    from test_gpu_parity import GpuBackend
    from paper_1811_00778_amd import network
    path = os.path.join(os.path.dirname(__file__), "golden", "cifar_plaintext_moduli.txt")
    moduli = [int(l) for l in open(path) if l.strip() and l[0] != "#"]
    free, _total = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs about 50 GiB of device memory")
    backend = GpuBackend()
    n, k = 8192, 10
    spec, in_shape = network.CIFAR10_HCNN, network.CIFAR10_INPUT
    n_in = in_shape[0] * in_shape[1] * in_shape[2]
    rng = gen.rng_for(4, 14)
    pixels = rng.integers(0, 16, size=n_in).astype(np.int64)
    weights = _weights(rng, spec, in_shape, 3)
    big = 1
    for t in moduli:
        big *= t
    say("plain network over the integers")
    true = plain_net.evaluate(spec, weights, pixels.reshape(in_shape + (1,)), big).reshape(10)
    true = [int(v) if int(v) <= big // 2 else int(v) - big for v in true]           # centred representatives
    assert max(abs(v) for v in true) > max(moduli) ** 4 and 2 * max(abs(v) for v in true) < big
    kr = None
    er = gen.encryption_randomness(rng, n, 256)            # reused for every block of 256 inputs and every channel
    residues = []
    total = 0.0
    for ch, t in enumerate(moduli):
        s = pc.Setup(backend, n, k, t=t, seed_id=4, stream=15, with_keys=False)
        ctx, dev = s.ctx, backend.dev
        if kr is None:
            kr = gen.key_randomness(rng, s.q, n)
        pk, evk = ctx.keygen(dev(kr["s"]), dev(kr["a"]), dev(kr["e"]), dev(kr["a_evk"]), dev(kr["e_evk"]))
        ctx.set_relin_key(evk)
        polys = np.zeros((n_in, n), dtype=np.uint32)
        polys[:, 0] = pixels % t
        cts = torch.empty((n_in, 2, k, n), dtype=torch.int32, device="cuda")
        d_er = {name: dev(v) for name, v in er.items()}
        for i0 in range(0, n_in, 256):
            cts[i0:i0 + 256] = ctx.encrypt(pk, dev(polys[i0:i0 + 256]), d_er["u"], d_er["e1"], d_er["e2"])
        plan = network.Plan(spec, in_shape, weights, dev)
        torch.cuda.synchronize()
        t0 = time.time()
        out = plan.run(ctx, cts)
        torch.cuda.synchronize()
        total += time.time() - t0
        host_out = backend.host(out)
        dec = backend.host(ctx.decrypt(dev(kr["s"]), out))
        del out, cts, plan
        torch.cuda.empty_cache()
        want0 = fv.decrypt(s.octx, kr["s"], host_out[0])                            # one oracle decryption per channel
        assert np.array_equal(dec[0], want0), ("GPU decryption", t)
        assert not dec[:, 1:].any(), ("outputs are constant polynomials", t)
        assert [int(v) for v in dec[:, 0]] == [v % t for v in true], ("channel", t)
        residues.append([int(v) for v in dec[:, 0]])
        say("channel %2d, t = %7d: network evaluated and decrypted" % (ch, t))
        ctx.close()
    say("ten channels: %.2f s on the GPU in total (each a cold run: first launches, scratch and feature-map allocation)" % total)
    for o in range(10):
        v = fv.crt_reconstruct([residues[ch][o] for ch in range(10)], moduli)
        v = v if v <= big // 2 else v - big
        assert v == true[o], ("recombined output", o)
