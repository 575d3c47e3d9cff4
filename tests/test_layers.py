"""Index tables for convolution-type layers: counts printed in the paper and the layer definition."""
import os

import numpy as np

from paper_1811_00778_amd import layers

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            out[key] = vals
    return out


def test_mnist_layer_counts_match_paper_table():
    g = _golden("mnist_layer_counts.txt")
    idx, valid, (ho, wo) = layers.conv_index_table(1, 28, 28, 5, 5, 2)
    F = 5
    assert 28 * 28 == int(g["layer1_inputs"][0])
    assert F * ho * wo == int(g["layer1_outputs"][0]) == int(g["layer2_hsquare"][0])
    assert F * idx.size == int(g["layer1_hmultplain"][0])
    assert valid.all() and idx.max() == 26 * 28 + 26     # 12 placements of stride 2 reach row and column 26
    idx3, _, (h3, w3) = layers.conv_index_table(5, 12, 12, 5, 5, 2)
    assert 50 * h3 * w3 == int(g["layer3_outputs"][0])
    # per output neuron the paper counts one filter plane (25 products), not 5 channels x 25
    assert 50 * h3 * w3 * 25 == int(g["layer3_hmultplain"][0])
    assert 10 * 800 == int(g["layer5_hmultplain"][0])
    total = int(g["layer1_hmultplain"][0]) + int(g["layer3_hmultplain"][0]) + int(g["layer5_hmultplain"][0])
    assert total == int(g["total_hmultplain"][0])
    assert 720 + 800 == int(g["total_hsquare"][0])


def test_ciphertext_size_formula():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "ciphertext_size.txt")) if l[0] not in "#\n"]
    for case, N, logq, nbytes in rows[1:]:
        assert 2 * int(N) * int(logq) // 8 == int(nbytes)
    # this build: 30-bit primes in 32-bit words, [2][k][n] uint32
    assert 2 * 8 * 8192 * 4 == 512 * 1024


def test_conv_table_matches_direct_convolution():
    rng = np.random.default_rng(3)
    c_in, h, w, F, fh, fw, s, pad = 3, 9, 8, 4, 3, 3, 2, 1
    x = rng.integers(0, 256, size=(c_in, h, w))
    wt = rng.integers(-7, 8, size=(F, c_in, fh, fw))
    idx, valid, (ho, wo) = layers.conv_index_table(c_in, h, w, fh, fw, s, pad)
    wtab = layers.conv_weight_table(wt, idx.shape[0], valid)
    flat = x.reshape(-1)
    got = np.einsum("gft,gt->fg", wtab, flat[idx]).reshape(F, ho, wo)
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad)))
    for f in range(F):
        for j in range(ho):
            for k in range(wo):
                assert got[f, j, k] == (wt[f] * xp[:, j * s:j * s + fh, k * s:k * s + fw]).sum()
    # placement rule of the blocking section: top-left input index j*s*w + k*s (no padding)
    idx0, _, (ho0, wo0) = layers.conv_index_table(1, h, w, fh, fw, s)
    for j in range(ho0):
        for k in range(wo0):
            assert idx0[j * wo0 + k, 0] == j * s * w + k * s


def test_fc_tables():
    w = np.arange(30, dtype=np.int32).reshape(3, 10)
    assert layers.fc_index_table(10).tolist() == [list(range(10))]
    assert layers.fc_weight_table(w).shape == (1, 3, 10)


def test_pool_table_is_all_ones_convolution_per_channel():
    rng = np.random.default_rng(4)
    C, h, w, e = 3, 8, 6, 2
    x = rng.integers(0, 100, size=(C, h, w))
    idx, ones, (ho, wo) = layers.pool_index_table(C, h, w, e)
    assert (ho, wo) == (4, 3) and idx.shape == (C * ho * wo, e * e) and ones.min() == ones.max() == 1
    got = np.einsum("gft,gt->g", ones, x.reshape(-1)[idx]).reshape(C, ho, wo)
    want = x.reshape(C, ho, e, wo, e).sum(axis=(2, 4))
    assert np.array_equal(got, want)
    # CIFAR-10 network of the paper: 32x32x32 -> 16x16x32 -> conv -> 8x8x64 -> conv -> 4x4x128 by 2x2 pooling
    for ch, side in ((32, 32), (64, 16), (128, 8)):
        idx, _, (ho, wo) = layers.pool_index_table(ch, side, side, 2)
        assert ch * ho * wo == ch * (side // 2) ** 2


def test_padded_stride1_conv_keeps_the_feature_map_size():
    # first layer of the paper's CIFAR-10 network: 3x3x3 filters, stride 1, padding -> 32 x 32 x 32
    idx, valid, (ho, wo) = layers.conv_index_table(3, 32, 32, 3, 3, 1, pad=1)
    assert (ho, wo) == (32, 32) and idx.shape == (1024, 27)
    assert valid.sum() == 27 * 1024 - 3 * (4 * 5 + 4 * 30 * 3)        # corner and edge placements lose terms


def test_network_shapes_match_paper_tables():
    """Layer sizes and squaring counts of both architectures against the paper's tables."""
    from paper_1811_00778_amd import network
    rows = [l.split() for l in open(os.path.join(GOLDEN, "cifar_layer_sizes.txt")) if l[0] not in "#\n"]
    table = [r for r in rows if r[0].isdigit()]
    extra = {r[0]: int(r[1]) for r in rows if not r[0].isdigit()}
    shp = network.shapes(network.CIFAR10_HCNN, network.CIFAR10_INPUT)
    assert len(shp) == len(table) == len(network.CIFAR10_HCNN)
    hmult = 0
    for layer, got, row in zip(network.CIFAR10_HCNN, shp, table):
        assert layer[0] == row[1]
        assert got == (int(row[2]), int(row[3]), int(row[4]))
        assert got[0] * got[1] * got[2] == int(row[5])
        hmult += int(row[6])
    assert hmult == extra["total_hmult"]
    assert network.op_counts(network.CIFAR10_HCNN, network.CIFAR10_INPUT)[1] == extra["total_hmult"]
    c, h, w = network.CIFAR10_INPUT
    assert c * h * w == extra["input_neurons"]
    g = _golden("mnist_layer_counts.txt")
    mshp = network.shapes(network.MNIST_HCNN, network.MNIST_INPUT)
    assert mshp[0] == (5, 12, 12) and mshp[2] == (50, 4, 4) and mshp[4] == (10, 1, 1)
    assert network.op_counts(network.MNIST_HCNN, network.MNIST_INPUT)[1] == int(g["total_hsquare"][0])
    ws = network.weight_shapes(network.CIFAR10_HCNN, network.CIFAR10_INPUT)
    assert ws[0] == (32, 3, 3, 3) and ws[3] == (64, 32, 3, 3) and ws[6] == (128, 64, 3, 3)
    assert ws[9] == (256, 2048) and ws[10] == (10, 256) and ws[1] is None and ws[2] is None
