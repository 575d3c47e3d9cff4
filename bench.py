#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
    python bench.py --only ntt|square|mac-layer [...]      one operation alone, for profiler runs and size sweeps

Workload ("primitive-8192"): n = 8192, q = 8 x 30-bit primes, t = 65537, a batch of 64
ciphertexts of uniformly random residues resident in HBM.  One step is one pass of the
whole hot path over the batch:
    forward + inverse NTT of the 128 polynomials (8 limbs each),
    a scalar multiply-accumulate layer (5 filters of 5x5 terms on an 8x8 grid of the
    64 ciphertexts -> 80 outputs, weights uniform in [-15, 15]),
    64 ciphertext squarings with scaling and relinearisation.
The printed JSON line reports squarings (with relinearisation) per second over whole steps,
the roofline position of the kernel that takes most of the step, and the CPU oracle timed on
a bounded sample (whose residues are also compared with the GPU's).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
ALU_PEAK_TOPS = 39.3           # 256 CU x 64 lanes x 2.4 GHz 32-bit integer VALU instructions / s
HBM_COUNTER_PROFILE = os.path.join(ROOT, "profiles", "bench_primitive8192_hbm_counters.md")


def counted_traffic(kernel_prefix):
    """HBM bytes per launch that the FETCH_SIZE / WRITE_SIZE counters attribute to a kernel of this workload, as the
    committed rocprofv3 summary records them (fetch KiB + write KiB of the table row whose kernel name starts with
    `kernel_prefix`); None when the summary has no such row."""
    try:
        for line in open(HBM_COUNTER_PROFILE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 4 and cells[0].startswith(kernel_prefix):
                return int((float(cells[2]) + float(cells[3])) * 1024)
    except (OSError, ValueError):
        pass
    return None


def time_layer(cid, torch, binding, layers, gen, reps=3, relin_order=0, square=True):
    """One conv layer + square activation at the shape of configuration `cid`: ms for the scalar MAC,
    ms for the squarings, compulsory-traffic bandwidth of the MAC.  Inputs are uniformly random canonical residues
    drawn on the device by the library's counter-based sampler (timing does not depend on the values)."""
    cfg = gen.CONFIGS[cid]
    n, k, t = cfg["n"], cfg["k"], cfg["t"]
    fc = cfg.get("fc")
    cv = cfg.get("conv") or dict(c_in=fc["n_in"], h=1, w=1, filters=fc["n_out"], fh=1, fw=1, stride=1,
                                 w_bound=fc["w_bound"])          # a fully connected layer is a 1x1 "image"
    q, p = binding.choose_moduli(n, k, t)
    ctx = binding.Context(n, q, p, t, device="cuda:0")
    rng = gen.rng_for(cid, 1)
    kr = gen.key_randomness(rng, q, n)
    dev = ctx.to_device
    _, evk = ctx.keygen(dev(kr["s"]), dev(kr["a"]), dev(kr["e"]), dev(kr["a_evk"]), dev(kr["e_evk"]))
    ctx.set_relin_key(evk)
    ctx.set_relin_order(relin_order)
    n_in = cv["c_in"] * cv["h"] * cv["w"]
    cts = ctx.sample_uniform(gen.SEED_BASE + cid, 1, n_in * 2).reshape((n_in, 2, k, n))     # uniform below each q_l
    idx_h, _, (ho, wo) = layers.conv_index_table(cv["c_in"], cv["h"], cv["w"], cv["fh"], cv["fw"], cv["stride"])
    F, G = cv["filters"], idx_h.shape[0]
    w_h = layers.conv_weight_table(gen.int_weights(rng, (F, cv["c_in"], cv["fh"], cv["fw"]), cv["w_bound"]), G)
    idx, w = dev(idx_h), dev(w_h)
    mac_out = torch.empty((F, G, 2, k, n), dtype=torch.int32, device=ctx.device)
    flat = mac_out.reshape((F * G, 2, k, n))
    if fc:                                        # deep-modulus configuration: square the stated batch instead
        flat = cts[:cfg["n_square"]]
    sq_out = torch.empty_like(flat)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    mac_ms, sq_ms = [], []
    for r in range(reps + 1):
        ev[0].record()
        ctx.ct_scalar_mac(cts, idx, w, cv["w_bound"], out=mac_out)
        ev[1].record()
        if square:
            ctx.ct_square_relin(flat, out=sq_out)
        ev[2].record()
        torch.cuda.synchronize()
        if r:                                     # first repetition warms up (scratch allocation)
            mac_ms.append(ev[0].elapsed_time(ev[1]))
            sq_ms.append(ev[1].elapsed_time(ev[2]))
    ctx.close()
    ct_bytes = 2 * k * n * 4
    mac = sorted(mac_ms)[len(mac_ms) // 2]
    sq = sorted(sq_ms)[len(sq_ms) // 2]
    out = dict(n=n, k=k, inputs=n_in, outputs=F * G, terms=int(idx_h.shape[1]), mac_ms=round(mac, 4),
               mac_compulsory_GBps=round((n_in + F * G) * ct_bytes / (mac * 1e-3) / 1e9, 1),
               mac_hbm_frac=round((n_in + F * G) * ct_bytes / (mac * 1e-3) / 1e9 / HBM_PEAK_GBS, 4))
    if square:
        out.update(square_relin_ms=round(sq, 4), layer_ms=round(mac + sq, 4),
                   squarings=int(flat.shape[0]), squarings_per_s=round(flat.shape[0] / (sq * 1e-3), 1))
    return out


def run_only(args, torch, binding, layers, gen):
    """`--only`: one operation alone on random canonical residues, one line per operation (for profiler runs and
    size sweeps; the JSON line of the benchmark is not printed)."""
    def timed(fn, reps):
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

    if args.only == "mac-layer":
        cfg = dict(gen.CONFIGS[args.config])
        if args.filters:
            cfg["conv"] = dict(cfg["conv"], filters=args.filters)
        saved = gen.CONFIGS[args.config]
        gen.CONFIGS[args.config] = cfg
        try:
            print(json.dumps(time_layer(args.config, torch, binding, layers, gen, reps=args.reps, square=False)), flush=True)
        finally:
            gen.CONFIGS[args.config] = saved
        return
    n, k, t = args.n, args.k, args.t
    q, p = binding.choose_moduli(n, k, t)
    ctx = binding.Context(n, q, p, t)
    if args.only == "ntt":
        buf = ctx.sample_uniform(1811, 1, args.polys)
        rows = args.polys * k
        for name, fn in (("forward", ctx.ntt_fwd), ("inverse", ctx.ntt_inv)):
            ms = timed(lambda: fn(buf), args.reps)
            print("ntt %s n=%d rows=%d: %.1f us per call, %.2f ns per row, %.0f GB/s (read + write of every row)"
                  % (name, n, rows, ms * 1e3, ms * 1e6 / rows, rows * n * 8 / ms / 1e6), flush=True)
    else:
        ctx.set_relin_key(ctx.sample_uniform(1811, 2, k * 2).reshape((k, 2, k, n)))     # random, not a genuine key
        ctx.set_fusion(args.fusion)
        cts = ctx.sample_uniform(1811, 3, args.cts * 2).reshape((args.cts, 2, k, n))
        out = torch.empty_like(cts)
        ms = timed(lambda: ctx.ct_square_relin(cts, out=out), args.reps)
        print("square+relin n=%d k=%d k_aux=%d cts=%d: %.3f ms per call, %.0f squarings per second"
              % (n, k, len(p), args.cts, ms, args.cts / ms * 1e3), flush=True)
        ctx.reset_stats()
        ctx.set_profile(True)
        ctx.ct_square_relin(cts, out=out)
        for name, (launches, blocks, tms) in ctx.profile().items():
            if launches:
                print("    %-12s %3d launches %9d blocks %8.3f ms  (%.2f ns per block)"
                      % (name, launches, blocks, tms, tms * 1e6 / blocks), flush=True)
        ctx.set_profile(False)
    ctx.close()


def time_primitives(n, k, torch, binding, gen, batch=64, reps=30):
    """The FHE primitives of the paper's micro-benchmark table (Sec. 5.3: KeyGen, Enc, Dec, HAdd, HSquare,
    HMultPlain, HMult) at one of its parameter sizes, t = 65537: microseconds per operation when issued one at a
    time (back to back on one stream) and when issued as one call over a batch.  Randomness is supplied by the
    caller (already on the device)."""
    import numpy as np
    t = 65537
    q, p = binding.choose_moduli(n, k, t)
    ctx = binding.Context(n, q, p, t, device="cuda:0")
    rng = gen.rng_for(2, 9)
    kr = gen.key_randomness(rng, q, n)
    dev = ctx.to_device
    d_kr = {name: dev(v) for name, v in kr.items()}
    pk, evk = ctx.keygen(d_kr["s"], d_kr["a"], d_kr["e"], d_kr["a_evk"], d_kr["e_evk"])
    ctx.set_relin_key(evk)
    er = gen.encryption_randomness(rng, n, batch)
    d_er = {name: dev(v) for name, v in er.items()}
    m = dev(rng.integers(0, t, size=(batch, n), dtype=np.int64).astype(np.uint32))
    cts = ctx.encrypt(pk, m, d_er["u"], d_er["e1"], d_er["e2"])
    one = lambda x: x[:1]
    idx1, w1 = dev(np.zeros((1, 1), dtype=np.uint32)), dev(np.full((1, 1, 1), 7, dtype=np.int32))
    idx2, w2 = dev(np.array([[0, 1]], dtype=np.uint32)), dev(np.ones((1, 1, 2), dtype=np.int32))
    idxb = dev(np.arange(batch, dtype=np.uint32)[:, None].copy())
    wb = dev(np.full((batch, 1, 1), 7, dtype=np.int32))
    idxa = dev(np.stack([np.arange(batch), (np.arange(batch) + 1) % batch], axis=1).astype(np.uint32))
    wa = dev(np.ones((batch, 1, 2), dtype=np.int32))
    out1 = torch.empty_like(cts[:1]); outb = torch.empty_like(cts)
    mac1 = torch.empty((1, 1) + tuple(cts.shape[1:]), dtype=torch.int32, device=ctx.device)
    macb = torch.empty((1, batch) + tuple(cts.shape[1:]), dtype=torch.int32, device=ctx.device)
    ops = {
        "keygen": (lambda: ctx.keygen(d_kr["s"], d_kr["a"], d_kr["e"], d_kr["a_evk"], d_kr["e_evk"]), None),
        "encrypt": (lambda: ctx.encrypt(pk, one(m), one(d_er["u"]), one(d_er["e1"]), one(d_er["e2"])),
                    lambda: ctx.encrypt(pk, m, d_er["u"], d_er["e1"], d_er["e2"])),
        # randomness drawn on the device by the counter-based samplers, then Encrypt
        "sample+encrypt": (lambda: ctx.encrypt(pk, one(m), ctx.sample_ternary(7, 1, 1), ctx.sample_gaussian(7, 2, 1),
                                               ctx.sample_gaussian(7, 3, 1)),
                           lambda: ctx.encrypt(pk, m, ctx.sample_ternary(7, 1, batch), ctx.sample_gaussian(7, 2, batch),
                                               ctx.sample_gaussian(7, 3, batch))),
        "decrypt": (lambda: ctx.decrypt(d_kr["s"], cts[:1]), lambda: ctx.decrypt(d_kr["s"], cts)),
        "hadd": (lambda: ctx.ct_scalar_mac(cts, idx2, w2, 1, out=mac1), lambda: ctx.ct_scalar_mac(cts, idxa, wa, 1, out=macb)),
        "hmultplain": (lambda: ctx.ct_scalar_mac(cts, idx1, w1, 7, out=mac1), lambda: ctx.ct_scalar_mac(cts, idxb, wb, 7, out=macb)),
        "hsquare": (lambda: ctx.ct_square_relin(cts[:1], out=out1), lambda: ctx.ct_square_relin(cts, out=outb)),
        "hmult": (lambda: ctx.ct_mul_relin(cts[:1], cts[1:2], out=out1), lambda: ctx.ct_mul_relin(cts, cts.roll(1, 0).contiguous(), out=outb)),
    }
    res = {}
    for name, (single, batched) in ops.items():
        row = {}
        for label, fn, div in (("single_us", single, 1), ("batched_us_per_op", batched, batch)):
            if fn is None:
                continue
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            row[label] = round((time.perf_counter() - t0) / reps / div * 1e6, 2)
        res[name] = row
    ctx.close()
    return dict(n=n, k=k, k_aux=len(p), batch=batch, ops=res)


def time_network(name, spec, in_shape, n, k, t, w_bound, torch, binding, network, gen, reps=2):
    """A whole HCNN-shaped network (architecture tables of Sec. 3.2) at a ring degree and modulus size of the
    paper's parameter table, one plaintext channel, random ciphertexts and random integer weights resident in
    HBM: seconds per evaluation, excluding encryption and table upload."""
    free, _ = torch.cuda.mem_get_info()
    shp = [in_shape] + network.shapes(spec, in_shape)
    ct_bytes = 2 * k * n * 4
    need = 2.5 * max(a[0] * a[1] * a[2] for a in shp) * ct_bytes + 8 * 2 ** 30
    if free < need:
        return dict(skipped="needs about %.0f GiB of device memory" % (need / 2 ** 30))
    q, p = binding.choose_moduli(n, k, t)
    ctx = binding.Context(n, q, p, t, device="cuda:0")
    rng = gen.rng_for(2, 7)
    kr = gen.key_randomness(rng, q, n)
    dev = ctx.to_device
    _, evk = ctx.keygen(dev(kr["s"]), dev(kr["a"]), dev(kr["e"]), dev(kr["a_evk"]), dev(kr["e_evk"]))
    ctx.set_relin_key(evk)
    weights = [None if ws is None else gen.int_weights(rng, ws, w_bound) for ws in network.weight_shapes(spec, in_shape)]
    plan = network.Plan(spec, in_shape, weights, dev)
    n_in = in_shape[0] * in_shape[1] * in_shape[2]
    cts = ctx.sample_uniform(gen.SEED_BASE + 77, 1, n_in * 2).reshape((n_in, 2, k, n))      # uniform below each q_l
    times = []
    for r in range(reps + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = plan.run(ctx, cts)
        torch.cuda.synchronize()
        if r:                                      # the first evaluation allocates scratch and feature maps
            times.append(time.perf_counter() - t0)
        del out
    # one more evaluation with per-launch events: where the time goes, by kernel class
    ctx.reset_stats()
    ctx.set_profile(True)
    out = plan.run(ctx, cts)
    torch.cuda.synchronize()
    kernel_ms = {name: round(ms, 2) for name, (_l, _b, ms) in ctx.profile().items() if ms > 0}
    ctx.set_profile(False)
    del out
    ctx.close()
    torch.cuda.empty_cache()
    n_mul, n_sq = network.op_counts(spec, in_shape)
    sec = sorted(times)[len(times) // 2]
    return dict(n=n, k=k, k_aux=len(p), t=t, inputs=n_in, squarings=n_sq, scalar_products_dense=n_mul,
                seconds=round(sec, 4), squarings_per_s=round(n_sq / sec, 1), kernel_ms=kernel_ms)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=12, help="squarings the oracle computes for cpu_baseline")
    ap.add_argument("--no-profile", action="store_true", help="no per-kernel events inside the timed region")
    ap.add_argument("--no-layers", action="store_true", help="skip the conv-layer timings (configs 3 and 4)")
    ap.add_argument("--no-networks", action="store_true", help="skip the whole-network timings")
    ap.add_argument("--no-primitives", action="store_true", help="skip the per-primitive latencies")
    ap.add_argument("--relin-order", type=int, default=0, help="HCNN_OPT_RELIN_ORDER (tuning experiments)")
    ap.add_argument("--only", choices=("ntt", "square", "mac-layer"),
                    help="time one operation alone and exit: ntt (--n --k --polys), square (--n --k --t --cts), "
                         "mac-layer (--config 3|4|5 [--filters F])")
    ap.add_argument("--n", type=int, default=8192)
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--t", type=int, default=65537)
    ap.add_argument("--polys", type=int, default=1024, help="--only ntt: polynomials of k limbs each")
    ap.add_argument("--cts", type=int, default=1024, help="--only square: ciphertexts")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="--only mac-layer: configuration whose layer shape is used")
    ap.add_argument("--filters", type=int, default=0, help="--only mac-layer: override the filter count")
    ap.add_argument("--fusion", type=int, default=0, help="HCNN_OPT_FUSION (tuning experiments)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured streaming / instruction-issue ceilings")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one plain device copy of 256 MiB (a reference dispatch for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the path shards by ciphertext with no exchange step, "
              "and this build has no multi-GPU launcher (use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1811_00778_amd import binding, layers
    from workloads import generators as gen

    if args.only:
        run_only(args, torch, binding, layers, gen)
        return

    cfg = gen.CONFIGS[2]
    n, k, t, n_ct = cfg["n"], cfg["k"], cfg["t"], cfg["n_ct"]
    q, p = binding.choose_moduli(n, k, t)
    ctx = binding.Context(n, q, p, t, device="cuda:0")
    dev = ctx.to_device
    rng = gen.rng_for(2, 1)
    kr = gen.key_randomness(rng, q, n)
    _, evk = ctx.keygen(dev(kr["s"]), dev(kr["a"]), dev(kr["e"]), dev(kr["a_evk"]), dev(kr["e_evk"]))
    ctx.set_relin_key(evk)
    ctx.set_relin_order(args.relin_order)
    cts_host = gen.uniform_residues(rng, q, n, lead=(n_ct, 2))
    cts = dev(cts_host)
    F, wb = 5, 15
    idx_h, _, (ho, wo) = layers.conv_index_table(1, 8, 8, 5, 5, 1)
    G, T = idx_h.shape
    w_h = layers.conv_weight_table(gen.int_weights(rng, (F, 1, 5, 5), wb), G)
    idx, w = dev(idx_h), dev(w_h)
    ntt_buf = cts.clone()
    mac_out = torch.empty((F, G, 2, k, n), dtype=torch.int32, device=ctx.device)
    sq_out = torch.empty_like(cts)

    def step():
        ctx.ntt_fwd(ntt_buf)
        ctx.ntt_inv(ntt_buf)
        ctx.ct_scalar_mac(cts, idx, w, wb, out=mac_out)
        ctx.ct_square_relin(cts, out=sq_out)

    if args.copy_calibration:
        ref = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device=ctx.device)       # 256 MiB read + 256 MiB written
        ref2 = torch.empty_like(ref)
        ref2.copy_(ref)
        torch.cuda.synchronize()
        del ref, ref2

    # ---- warm-up: the W steps asked for, then on until the step time has settled (clocks and caches reach their
    #      steady state after some tenths of a second, more than a handful of 0.3 ms steps): windows of 10 steps
    #      until two in a row agree within 2 %, at least 0.3 s and at most 3 s in all
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    warm_t0, prev, settle_steps = time.perf_counter(), None, 0
    while True:
        w0 = time.perf_counter()
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        window = time.perf_counter() - w0
        settle_steps += 10
        spent = time.perf_counter() - warm_t0
        if spent > 3.0 or (spent >= 0.3 and prev is not None and abs(window - prev) <= 0.02 * prev):
            break
        prev = window

    # ---- timed region: exactly K steps, nothing else on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- the same K steps once more with a HIP event pair around every kernel launch (on the launch
    #      stream); kept out of the region above because the event records themselves cost ~10 % there
    prof, elapsed_prof = {}, None
    if not args.no_profile:
        ctx.reset_stats()
        ctx.set_profile(True)
        torch.cuda.synchronize()
        tp0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        elapsed_prof = time.perf_counter() - tp0
        prof = ctx.profile()
        ctx.set_profile(False)
    fallbacks = ctx.exact_fallbacks()

    ms_per_step = elapsed * 1e3 / args.steps
    value = n_ct * args.steps / elapsed

    # ---- the device's own ceilings, measured now by the library's streaming and instruction-issue kernels
    ceilings = None if args.no_ceilings else {name: round(v, 1) for name, v in ctx.measured_ceilings().items()}

    # ---- per-kernel view; a roofline entry per kernel class, the one with the largest total time on top
    ct_bytes = 2 * k * n * 4
    row4 = 4 * n                                           # bytes of one row
    L_ = k + len(p)
    butterflies = (n // 2) * (n.bit_length() - 1)
    kernels = {}
    for name, (launches, blocks, ms) in prof.items():
        if launches:
            kernels[name] = dict(launches=launches, blocks=blocks, total_ms=round(ms, 4),
                                 avg_ms=round(ms / launches, 5), share=round(ms / (elapsed_prof * 1e3), 4))
    # algorithmic HBM bytes of the launches of one step, per class (a plain row is read and written once; the three
    # tensor components of a (ciphertext, limb) pair share two reads; the one-kernel relinearisation reads y and
    # writes the result, the key comes from L2; the scalar MAC reads every input and writes every output once)
    plain_rows = ntt_buf.numel() // n
    step_bytes = {
        "ntt_fwd": plain_rows * 2 * row4 + n_ct * 2 * L_ * 2 * row4,
        "ntt_inv": plain_rows * 2 * row4 + n_ct * 5 * L_ * row4,
        "relin_fused": n_ct * 5 * k * row4,
        "scalar_mac": (n_ct + F * G) * ct_bytes,
        "base_ext": n_ct * 2 * L_ * row4,
        "scale": n_ct * 3 * (L_ + k) * row4,
    }
    profile_rows = {"ntt_fwd": "NttFwd<13, 5, 5, 0>", "ntt_inv": "NttInv<13, 5, 2>", "relin_fused": "RelinFused",
                    "scalar_mac": "Mac", "base_ext": "ExtKernelT", "scale": "ScaleKernelR"}

    def class_roofline(name):
        kd = kernels[name]
        avg_s = kd["total_ms"] / kd["launches"] * 1e-3
        per_step = kd["launches"] / args.steps
        out = dict(kernel=name, avg_launch_ms=round(avg_s * 1e3, 5))
        bytes_per_launch = step_bytes[name] / per_step if name in step_bytes else None
        if name in ("ntt_fwd", "ntt_inv", "relin_fused", "tensor"):
            # The transform is bound by integer VALU issue as much as by HBM: a lazy butterfly is 7 VALU instructions
            # on this chip (high multiplication, multiplication, multiply-add, a 2-instruction conditional subtraction,
            # 2 additions / subtractions), i.e. 7 * (n/2) * log2(n) per row = 5.7 instructions per byte moved, above
            # the chip's balance of 39.3e12 / 8e12 = 4.9.  achieved = algorithmic instructions per launch / average
            # launch time; `blocks` counts the transformed rows.
            instr = kd["blocks"] / kd["launches"] * butterflies * 7
            ach = instr / avg_s / 1e12
            out.update(bound="alu", achieved=round(ach, 2), peak=ALU_PEAK_TOPS, unit="T int32 lane-instr/s",
                       frac=round(ach / ALU_PEAK_TOPS, 4), algorithmic_instr_per_launch=int(instr))
            if ceilings:
                # the slowest of the three multiplication forms a butterfly uses, as measured on this device
                issue = min(ceilings[c] for c in ("mul_lo_u32_Tops", "mul_hi_u32_Tops", "mad_u64_u32_Tops"))
                out["frac_of_measured_issue_rate"] = round(ach / issue, 4)
        else:
            out.update(bound="hbm", peak=HBM_PEAK_GBS, unit="GB/s")
            if bytes_per_launch:
                ach = bytes_per_launch / avg_s / 1e9
                out.update(achieved=round(ach, 1), frac=round(ach / HBM_PEAK_GBS, 4))
                if ceilings:
                    out["frac_of_measured_copy_rate"] = round(ach / ceilings["copy_GBps"], 4)
        if bytes_per_launch:
            out.update(algorithmic_bytes_per_launch=int(bytes_per_launch),
                       hbm_GBps=round(bytes_per_launch / avg_s / 1e9, 1),
                       hbm_frac=round(bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS, 4))
        # HBM bytes that the FETCH_SIZE / WRITE_SIZE counters attribute to a launch of this kernel on this workload,
        # as recorded in the committed rocprofv3 summary (None if it has no row for it)
        out["traffic"] = counted_traffic(profile_rows.get(name, name))
        out["traffic_source"] = "profiles/bench_primitive8192_hbm_counters.md" if out["traffic"] else None
        return out

    roofline = None
    if kernels:
        dom = max(kernels, key=lambda kname: kernels[kname]["total_ms"])
        roofline = class_roofline(dom)
        roofline["classes"] = {name: class_roofline(name) for name in ("ntt_fwd", "ntt_inv", "scalar_mac", "relin_fused",
                                                                       "scale", "base_ext") if name in kernels and name != dom}
        # NTT launches of the step, time per row (the small launches of this batch fill one round of workgroups)
        roofline["ntt_ns_per_row"] = {name: round(kernels[name]["total_ms"] * 1e6 / kernels[name]["blocks"], 2)
                                      for name in ("ntt_fwd", "ntt_inv") if name in kernels}

    # ---- the layer-shaped workloads of the metric ("encrypted conv layer ms"): scalar MAC + square
    #      activation on MNIST- and CIFAR-10-shaped layers, random ciphertexts resident in HBM
    layers_out = {}
    if not args.no_layers:
        for cid in (3, 4, 5):
            layers_out[gen.CONFIGS[cid]["name"]] = time_layer(cid, torch, binding, layers, gen, relin_order=args.relin_order)

    # ---- whole networks at the sizes of the paper's parameter table (Sec. 4.2), one plaintext channel each:
    #      MNIST set 1 (N = 2^13, 330-bit q, the 43-bit t = 5522259017729), CIFAR-10 set 5 (N = 2^13, 300-bit q, t = its first plaintext modulus), and
    #      the CIFAR-10 shape again at N = 2^14 with a 360-bit q
    networks_out = {}
    if not args.no_networks:
        from paper_1811_00778_amd import network
        networks_out["mnist-hcnn"] = time_network("mnist", network.MNIST_HCNN, network.MNIST_INPUT, 8192, 11, 5522259017729, 15,
                                                  torch, binding, network, gen)
        networks_out["cifar10-hcnn"] = time_network("cifar10", network.CIFAR10_HCNN, network.CIFAR10_INPUT, 8192, 10,
                                                    2424833, 7, torch, binding, network, gen)
        networks_out["cifar10-hcnn-n16384"] = time_network("cifar10", network.CIFAR10_HCNN, network.CIFAR10_INPUT,
                                                           16384, 12, 65537, 7, torch, binding, network, gen)

    # ---- the primitives of the paper's micro-benchmark table at its parameter sizes 2 and 4 (360-bit q)
    primitives_out = {}
    if not args.no_primitives:
        primitives_out["n8192-q360"] = time_primitives(8192, 12, torch, binding, gen)
        primitives_out["n16384-q360"] = time_primitives(16384, 12, torch, binding, gen)

    # ---- CPU oracle on a bounded sample of the same squarings (also a parity check)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fv
        octx = fv.Context(n, q, t)
        evk_h = ctx.to_host_u32(evk)
        got = ctx.to_host_u32(sq_out)
        sample = list(range(0, n_ct, max(1, n_ct // args.cpu_sample)))[:args.cpu_sample]
        tc0 = time.perf_counter()
        ok = True
        for i in sample:
            want = fv.square_relin(octx, cts_host[i], evk_h)
            ok = ok and bool(np.array_equal(got[i], want))
        tc = time.perf_counter() - tc0
        cpu = dict(value=round(len(sample) / tc, 4), unit="squarings+relin/s", cores=fv.num_threads(), kind="oracle",
                   sample="%d of the %d squarings of the step (ciphertexts %s), %.1f s" % (len(sample), n_ct, sample, tc),
                   matches_gpu=ok)

    line = {
        "metric": "homomorphic squarings+relin/sec at n=8192",
        "value": round(value, 2),
        "unit": "squarings+relin/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settling_steps_after_warmup": settle_steps,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": "primitive-8192: n=8192, 8x30-bit primes, t=65537, 64 random ciphertexts; "
                               "step = NTT fwd+inv of 128 polys + scalar MAC 64->80 (5 filters x 25 terms) "
                               "+ 64 squarings with relinearisation",
                   "n": n, "k": k, "k_aux": len(p), "batch": n_ct},
        "roofline": roofline,
        "measured_ceilings": ceilings,
        "cpu_baseline": cpu,
        "conv_layers": layers_out,
        "networks": networks_out,
        "primitives": primitives_out,
        "kernels": kernels,
        "profiled_pass_ms_per_step": None if elapsed_prof is None else round(elapsed_prof * 1e3 / args.steps, 4),
        "exact_rounding_fallbacks": fallbacks,
        "context": {"paper_primitives_ms_v100_sets_2_and_4": {"keygen": [12.377, 21.392], "encrypt": [0.935, 1.496],
                                                              "decrypt": [0.075, 0.098], "hadd": [0.052, 0.054],
                                                              "hsquare": [1.679, 2.371], "hmultplain": [0.033, 0.035],
                                                              "hmult": [2.014, 2.769]},
                    "paper_hsquare_ms_v100": 1.679, "paper_mnist_s_v100": 5.16,
                    "paper_cifar10_s_1gpu_per_channel": 553.89, "paper_cifar10_s_4gpu_per_channel": 304.43},
    }
    print(json.dumps(line))
    ctx.close()


if __name__ == "__main__":
    main()
