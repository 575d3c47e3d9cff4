"""Micro-benchmarks of single entry points on random data (for profiling runs and size sweeps).

    python -m paper_1811_00778_amd.probe ntt    [--n N] [--k K] [--polys P] [--reps R]
    python -m paper_1811_00778_amd.probe square [--n N] [--k K] [--t T] [--cts C] [--reps R]

Times the calls with HIP events on the context's stream and prints one line per operation.
"""
import argparse

import torch

from . import binding


def _time(fn, reps):
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps          # ms per call


def main(argv=None):
    ap = argparse.ArgumentParser(prog="python -m paper_1811_00778_amd.probe")
    ap.add_argument("what", choices=("ntt", "square"))
    ap.add_argument("--n", type=int, default=8192)
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--t", type=int, default=65537)
    ap.add_argument("--polys", type=int, default=1024, help="ntt: polynomials of k limbs each")
    ap.add_argument("--cts", type=int, default=1024, help="square: ciphertexts")
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args(argv)
    n, k = args.n, args.k
    q, p = binding.choose_moduli(n, k, args.t)
    ctx = binding.Context(n, q, p, args.t)
    gen = torch.Generator(device=ctx.device)
    gen.manual_seed(1811)
    rnd = lambda *shape: torch.randint(0, 1 << 29, shape, dtype=torch.int32, device=ctx.device, generator=gen)
    if args.what == "ntt":
        buf = rnd(args.polys, k, n)
        rows = args.polys * k
        for name, fn in (("forward", ctx.ntt_fwd), ("inverse", ctx.ntt_inv)):
            ms = _time(lambda: fn(buf), args.reps)
            print("ntt %s n=%d rows=%d: %.1f us per call, %.2f ns per row, %.0f GB/s (read + write of every row)"
                  % (name, n, rows, ms * 1e3, ms * 1e6 / rows, rows * n * 8 / ms / 1e6), flush=True)
    else:
        ctx.set_relin_key(rnd(k, 2, k, n))
        cts = rnd(args.cts, 2, k, n)
        out = torch.empty_like(cts)
        ms = _time(lambda: ctx.ct_square_relin(cts, out=out), args.reps)
        print("square+relin n=%d k=%d k_aux=%d cts=%d: %.3f ms per call, %.0f squarings per second"
              % (n, k, len(p), args.cts, ms, args.cts / ms * 1e3), flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
