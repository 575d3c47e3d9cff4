"""Layer-by-layer evaluation of HCNN-shaped networks through the C ABI.

A network is a tuple of layer specs applied to a feature map of ciphertexts (one ciphertext per
neuron, Sec. 3.1; feature map [C][H][W] = ciphertext index c*H*W + r*W + x):

    ("conv", filters, fh, fw, stride, pad)   convolution without bias          -> hcnn_ct_scalar_mac
    ("pool", extent)                         average pooling as a sum (Sec. 4.3) -> hcnn_ct_scalar_mac
    ("fc", n_out)                            fully connected                   -> hcnn_ct_scalar_mac
    ("square",)                              square activation                 -> hcnn_ct_square_relin

Everything here is indexing and call sequencing; all arithmetic runs in the library's kernels.
MNIST_HCNN and CIFAR10_HCNN are the architectures of Tables 1 and 2.
"""
import numpy as np

from . import layers

MNIST_HCNN = (("conv", 5, 5, 5, 2, 0), ("square",), ("conv", 50, 5, 5, 2, 0), ("square",), ("fc", 10))
MNIST_INPUT = (1, 28, 28)
CIFAR10_HCNN = (("conv", 32, 3, 3, 1, 1), ("square",), ("pool", 2),
                ("conv", 64, 3, 3, 1, 1), ("square",), ("pool", 2),
                ("conv", 128, 3, 3, 1, 1), ("square",), ("pool", 2),
                ("fc", 256), ("fc", 10))
CIFAR10_INPUT = (3, 32, 32)

_MAX_FILTERS = 16            # filters per hcnn_ct_scalar_mac call
_STAGED_LDS_BYTES = 64 * 1024   # the library stages a gather row and its weights in LDS up to this size


def shapes(spec, in_shape):
    """Feature-map shape after every layer: list of (C, H, W), one entry per layer."""
    c, h, w = in_shape
    out = []
    for layer in spec:
        kind = layer[0]
        if kind == "conv":
            _, f, fh, fw, stride, pad = layer
            h, w, c = (h + 2 * pad - fh) // stride + 1, (w + 2 * pad - fw) // stride + 1, f
        elif kind == "pool":
            e = layer[1]
            h, w = (h - e) // e + 1, (w - e) // e + 1
        elif kind == "fc":
            c, h, w = layer[1], 1, 1
        elif kind != "square":
            raise ValueError("unknown layer kind %r" % (kind,))
        out.append((c, h, w))
    return out


def weight_shapes(spec, in_shape):
    """Weight array shape per layer (None for layers without weights): conv [F][C][fh][fw], fc [n_out][n_in]."""
    prev = in_shape
    out = []
    for layer, shp in zip(spec, shapes(spec, in_shape)):
        if layer[0] == "conv":
            out.append((layer[1], prev[0], layer[2], layer[3]))
        elif layer[0] == "fc":
            out.append((layer[1], prev[0] * prev[1] * prev[2]))
        else:
            out.append(None)
        prev = shp
    return out


def op_counts(spec, in_shape):
    """(ciphertext-by-scalar products, squarings) of one evaluation.  Products are counted densely: every
    filter tap on every input channel at every placement, padding included (the complexity tables of
    Sec. 4.1 count fewer: one filter plane per output neuron for MNIST, non-zero trained weights for
    CIFAR-10).  The squarings are the HMult column of those tables.  Pooling only adds ciphertexts."""
    prev = in_shape
    n_mul, n_sq = 0, 0
    for layer, shp in zip(spec, shapes(spec, in_shape)):
        c, h, w = shp
        if layer[0] == "conv":
            n_mul += c * h * w * prev[0] * layer[2] * layer[3]
        elif layer[0] == "fc":
            n_mul += c * prev[0] * prev[1] * prev[2]
        elif layer[0] == "square":
            n_sq += c * h * w
        prev = shp
    return n_mul, n_sq


class Plan:
    """Gather tables of a network, built once on the host and uploaded once."""

    def __init__(self, spec, in_shape, weights, to_device):
        self.spec, self.in_shape = spec, in_shape
        self.steps = []
        prev = in_shape
        for layer, shp, wt in zip(spec, shapes(spec, in_shape), weights):
            kind = layer[0]
            if kind == "square":
                self.steps.append(("square",))
            else:
                if kind == "conv":
                    _, f, fh, fw, stride, pad = layer
                    idx, valid, _ = layers.conv_index_table(prev[0], prev[1], prev[2], fh, fw, stride, pad)
                    w = layers.conv_weight_table(wt, idx.shape[0], valid if pad else None)
                elif kind == "pool":
                    idx, w, _ = layers.pool_index_table(prev[0], prev[1], prev[2], layer[1])
                else:
                    idx = layers.fc_index_table(prev[0] * prev[1] * prev[2])
                    w = layers.fc_weight_table(wt)
                bound = int(np.abs(w).max()) if w.size else 0
                G, F, T = w.shape
                t_pad = (T + 3) // 4 * 4
                per_call = max(1, min(_MAX_FILTERS, (_STAGED_LDS_BYTES // 4 - 8) // t_pad - 1))
                calls = [(f0, min(F, f0 + per_call), to_device(np.ascontiguousarray(w[:, f0:min(F, f0 + per_call), :])))
                         for f0 in range(0, F, per_call)]
                # pooling groups are already in (channel, row, column) order with one "filter"
                self.steps.append(("mac", to_device(idx), calls, bound, G, F))
            prev = shp
        self.out_shape = prev

    def run(self, ctx, cts, keep=False):
        """Evaluates the network on cts [C*H*W][2][k][n]; returns the output ciphertexts (and, with keep,
        the list of every layer's output)."""
        kept = []
        for step in self.steps:
            if step[0] == "square":
                cts = ctx.ct_square_relin(cts)
            else:
                _, d_idx, calls, bound, G, F = step
                out = ctx._empty((F, G) + tuple(cts.shape[1:]), "u32")
                for f0, f1, d_w in calls:
                    ctx.ct_scalar_mac(cts, d_idx, d_w, bound, out=out[f0:f1])
                cts = out.reshape((F * G,) + tuple(cts.shape[1:]))
            if keep:
                kept.append(cts)
        return (cts, kept) if keep else cts


def _main(argv=None):
    """python -m paper_1811_00778_amd.network {mnist,cifar10} [--n N] [--k K] [--t T] [--reps R]
    Times one evaluation of the network on random ciphertexts, random integer weights and a random (not
    genuine) evaluation key, all resident on the GPU; meant for profiling runs."""
    import argparse
    import time

    import torch

    from . import binding
    ap = argparse.ArgumentParser(prog="python -m paper_1811_00778_amd.network")
    ap.add_argument("name", choices=("mnist", "cifar10"))
    ap.add_argument("--n", type=int, default=8192)
    ap.add_argument("--k", type=int, default=0, help="30-bit primes in q (default: 11 for mnist, 10 for cifar10)")
    ap.add_argument("--t", type=int, default=0, help="plaintext modulus (default: 65537 / 2424833)")
    ap.add_argument("--reps", type=int, default=2)
    args = ap.parse_args(argv)
    spec, in_shape = (MNIST_HCNN, MNIST_INPUT) if args.name == "mnist" else (CIFAR10_HCNN, CIFAR10_INPUT)
    k = args.k or (11 if args.name == "mnist" else 10)
    t = args.t or (65537 if args.name == "mnist" else 2424833)
    q, p = binding.choose_moduli(args.n, k, t)
    ctx = binding.Context(args.n, q, p, t)
    # uniformly random canonical residues (below each q_l), drawn on the device by the library's sampler
    ctx.set_relin_key(ctx.sample_uniform(1811, 2, k * 2).reshape((k, 2, k, args.n)))
    rng = np.random.default_rng(1811)
    bound = 15 if args.name == "mnist" else 7
    weights = [None if s is None else rng.integers(-bound, bound + 1, size=s).astype(np.int32)
               for s in weight_shapes(spec, in_shape)]
    plan = Plan(spec, in_shape, weights, ctx.to_device)
    n_in = in_shape[0] * in_shape[1] * in_shape[2]
    cts = ctx.sample_uniform(1811, 1, n_in * 2).reshape((n_in, 2, k, args.n))
    n_mul, n_sq = op_counts(spec, in_shape)
    for r in range(args.reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = plan.run(ctx, cts)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        print("%s n=%d k=%d k_aux=%d t=%d: evaluation %d%s %.4f s (%d squarings, %d scalar products)"
              % (args.name, args.n, k, len(p), t, r, " (cold)" if r == 0 else "", dt, n_sq, n_mul), flush=True)
        del out
    ctx.close()


if __name__ == "__main__":
    _main()
