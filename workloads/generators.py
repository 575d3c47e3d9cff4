"""Seeded synthetic inputs (shapes and value ranges of the paper's MNIST / CIFAR-10
workloads; the datasets and trained weights themselves are not used).

Nothing in this module performs arithmetic of the method: it draws raw random
numbers with numpy's default_rng and describes workload shapes.  Moduli are
passed in by the caller (each side generates its own primes).
"""
import numpy as np

SEED_BASE = 181100778 * 10

# Workload shapes.  id 1..5 follow the benchmark configurations; "conv"/"fc"
# describe the scalar-MAC layer, "n_square" the number of squarings.
CONFIGS = {
    1: dict(name="tiny", n=1024, k=2, t=65537, n_ct=8, n_square=1,
            fc=dict(n_in=8, n_out=1, w_bound=8)),
    2: dict(name="primitive-8192", n=8192, k=8, t=65537, n_ct=64, n_square=64),
    3: dict(name="mnist-conv1", n=8192, k=8, t=65537, n_ct=784, n_square=720,
            conv=dict(c_in=1, h=28, w=28, filters=5, fh=5, fw=5, stride=2, w_bound=15)),
    4: dict(name="cifar-conv", n=16384, k=16, t=65537, n_ct=3072, n_square=1800,
            conv=dict(c_in=3, h=32, w=32, filters=8, fh=3, fw=3, stride=2, w_bound=7)),
    5: dict(name="deep-relin", n=32768, k=24, t=65537, n_ct=1024, n_square=32,
            fc=dict(n_in=1024, n_out=10, w_bound=31)),
}


def rng_for(config_id: int, stream: int = 0) -> np.random.Generator:
    """Independent generator per (configuration, stream)."""
    return np.random.default_rng([SEED_BASE + int(config_id), int(stream)])


def ternary(rng, n: int) -> np.ndarray:
    """iid uniform on {-1, 0, 1}."""
    return rng.integers(-1, 2, size=n, dtype=np.int64).astype(np.int32)


def rounded_gaussian(rng, n: int, sigma: float = 3.2, cut: int = 19) -> np.ndarray:
    """Round-to-nearest of N(0, sigma^2); draws with |x| > cut are redrawn."""
    out = np.rint(rng.normal(0.0, sigma, size=n)).astype(np.int64)
    bad = np.abs(out) > cut
    while bad.any():
        out[bad] = np.rint(rng.normal(0.0, sigma, size=int(bad.sum()))).astype(np.int64)
        bad = np.abs(out) > cut
    return out.astype(np.int32)


def uniform_residues(rng, moduli, n: int, lead=()) -> np.ndarray:
    """uint32 array [*lead][len(moduli)][n], row l iid uniform in [0, moduli[l])."""
    lead = tuple(lead)
    out = np.empty(lead + (len(moduli), n), dtype=np.uint32)
    for l, p in enumerate(moduli):
        out[..., l, :] = rng.integers(0, int(p), size=lead + (n,), dtype=np.int64)
    return out


def slot_values(rng, count: int, n: int, high: int) -> np.ndarray:
    """count slot vectors of n iid uniform integers in [0, high)."""
    return rng.integers(0, int(high), size=(count, n), dtype=np.int64).astype(np.uint32)


def int_weights(rng, shape, bound: int) -> np.ndarray:
    """iid uniform integers in [-bound, bound]."""
    return rng.integers(-int(bound), int(bound) + 1, size=shape, dtype=np.int64).astype(np.int32)


def key_randomness(rng, moduli, n: int) -> dict:
    """Raw draws for KeyGen: secret, public-key a and e, one (a_i, e_i) per evaluation-key component."""
    k = len(moduli)
    return dict(
        s=ternary(rng, n),
        a=uniform_residues(rng, moduli, n),
        e=rounded_gaussian(rng, n),
        a_evk=uniform_residues(rng, moduli, n, lead=(k,)),
        e_evk=np.stack([rounded_gaussian(rng, n) for _ in range(k)]),
    )


def encryption_randomness(rng, n: int, count: int) -> dict:
    """Raw draws for `count` encryptions: u ternary, e1 and e2 rounded Gaussian."""
    return dict(
        u=np.stack([ternary(rng, n) for _ in range(count)]),
        e1=np.stack([rounded_gaussian(rng, n) for _ in range(count)]),
        e2=np.stack([rounded_gaussian(rng, n) for _ in range(count)]),
    )
