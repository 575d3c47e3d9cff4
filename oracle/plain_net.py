"""Plain-integer evaluation of an HCNN-shaped network modulo t.  TEST INFRASTRUCTURE ONLY.

The encrypted network computes, in every plaintext slot independently, the same network on
the slot's integers modulo t (Sec. 3.1: SIMD packing puts one image per slot; Sec. 3.2 and
Tables 1-2: convolution without bias, square activation, average pooling evaluated as a
window sum, fully connected layers).  This module writes that computation out with numpy
integer arrays; it knows nothing of ciphertexts.  Feature maps are [C][H][W][S] for S slots.

For t below 2^31 the arrays are int64 (every intermediate stays far below 2^63); for a wider t (the 43-bit
modulus of the MNIST parameter sets) they hold Python integers (dtype=object), which cannot overflow.

Layer specs are the tuples used by the network runner:
    ("conv", filters, fh, fw, stride, pad), ("pool", extent), ("fc", n_out), ("square",)
"""
import numpy as np


def _dtype(t):
    return np.int64 if t < (1 << 31) else object


def conv_mod(x, w, stride, pad, t):
    """y[f, j, k] = sum_{c,dy,dx} w[f,c,dy,dx] * x[c, j*stride+dy-pad, k*stride+dx-pad]  (zero outside), mod t."""
    C, H, W, S = x.shape
    F, Cw, fh, fw = w.shape
    assert C == Cw
    dt = _dtype(t)
    if pad:
        xp = np.zeros((C, H + 2 * pad, W + 2 * pad, S), dtype=dt)
        xp[:, pad:pad + H, pad:pad + W] = x
    else:
        xp = x.astype(dt)
    ho, wo = (H + 2 * pad - fh) // stride + 1, (W + 2 * pad - fw) // stride + 1
    y = np.zeros((F, ho, wo, S), dtype=dt)
    for f in range(F):
        acc = np.zeros((ho, wo, S), dtype=dt)
        for c in range(C):
            for dy in range(fh):
                for dx in range(fw):
                    acc += int(w[f, c, dy, dx]) * xp[c, dy:dy + stride * ho:stride, dx:dx + stride * wo:stride]
            acc %= t                       # keeps |acc| far below 2^63 for any channel count
        y[f] = acc
    return y % t


def sum_pool_mod(x, extent, t):
    """Window sums with stride = extent (the division of average pooling is folded into the scale, Sec. 4.3)."""
    C, H, W, S = x.shape
    ho, wo = (H - extent) // extent + 1, (W - extent) // extent + 1
    y = np.zeros((C, ho, wo, S), dtype=_dtype(t))
    for dy in range(extent):
        for dx in range(extent):
            y += x[:, dy:dy + extent * ho:extent, dx:dx + extent * wo:extent]
    return y % t


def fc_mod(x, w, t):
    """y[o] = sum_i w[o, i] * x.flat[i], mod t, inputs flattened in (c, row, column) order."""
    C, H, W, S = x.shape
    dt = _dtype(t)
    flat = x.reshape(C * H * W, S).astype(dt)
    y = np.zeros((w.shape[0], S), dtype=dt)
    step = 1024                           # partial sums of at most 1024 terms stay below 2^63
    for i0 in range(0, flat.shape[0], step):
        y = (y + w[:, i0:i0 + step].astype(dt) @ flat[i0:i0 + step]) % t
    return y.reshape(w.shape[0], 1, 1, S)


def evaluate(spec, weights, x, t, keep=False):
    """Applies the layers of `spec` to x [C][H][W][S] modulo t; weights[i] belongs to layer i (None if unused)."""
    x = np.asarray(x, dtype=_dtype(t)) % t
    kept = []
    for layer, w in zip(spec, weights):
        kind = layer[0]
        if kind == "conv":
            x = conv_mod(x, np.asarray(w), layer[4], layer[5], t)
        elif kind == "pool":
            x = sum_pool_mod(x, layer[1], t)
        elif kind == "fc":
            x = fc_mod(x, np.asarray(w), t)
        elif kind == "square":
            x = x * x % t
        else:
            raise ValueError(kind)
        if keep:
            kept.append(x)
    return (x, kept) if keep else x
