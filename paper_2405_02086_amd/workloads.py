"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's
callers.  This module draws numbers and nothing else: no norm, no threshold, no
projection arithmetic lives here, and it imports neither the GPU binding nor
the oracle.

Every workload is a host fp32 array from numpy's PCG64 stream seeded with
BASE_SEED + index, so the bytes are reproducible on any machine.  The radius is
given as a fraction of the input's own l_{1,q} norm; whoever calls the
projection turns that fraction into eta with its own norm routine.
"""
from dataclasses import dataclass
import numpy as np

BASE_SEED = 240502000


@dataclass(frozen=True)
class Workload:
    name: str
    shape: tuple          # (n, m) for matrices, (d0, d1, d2) for tensors
    dist: str             # "normal" | "normal_colscale" | "laplace" | "uniform"
    eta_frac: float       # eta = eta_frac * ||Y||_{1,q}
    seed: int
    variants: tuple       # which projections are run on it: "l1inf", "l11", "l12", "tri"


WORKLOADS = {
    # small case the oracle finishes instantly
    "small_256x128": Workload("small_256x128", (256, 128), "normal", 0.1, BASE_SEED + 1, ("l1inf",)),
    # headline mid-size case: per-column scales log-uniform in [0.01, 1]
    "square_4096": Workload("square_4096", (4096, 4096), "normal_colscale", 0.3, BASE_SEED + 2, ("l1inf",)),
    # skewed shapes, Laplace entries
    "tall_262144x256": Workload("tall_262144x256", (262144, 256), "laplace", 0.05, BASE_SEED + 3, ("l1inf",)),
    "wide_256x262144": Workload("wide_256x262144", (256, 262144), "laplace", 0.05, BASE_SEED + 4, ("l1inf",)),
    # tri-level tensor
    "tensor_256x256x256": Workload("tensor_256x256x256", (256, 256, 256), "normal", 0.2, BASE_SEED + 5, ("tri",)),
    # 1 GiB case, three variants
    "square_16384": Workload("square_16384", (16384, 16384), "normal", 0.1, BASE_SEED + 6, ("l1inf", "l11", "l12")),
    # the shape and distribution of the paper's own timing figures (Sec. 6.1)
    "paper_1000x10000": Workload("paper_1000x10000", (1000, 10000), "uniform", None, BASE_SEED + 7, ("l1inf",)),
}


def _fill(rng, out, dist):
    """Fill the flat fp32 array `out` chunk by chunk (bounded temporaries)."""
    step = 1 << 24
    for lo in range(0, out.size, step):
        hi = min(out.size, lo + step)
        if dist == "normal":
            out[lo:hi] = rng.standard_normal(hi - lo, dtype=np.float32)
        elif dist == "laplace":
            out[lo:hi] = rng.laplace(0.0, 1.0, hi - lo).astype(np.float32)
        elif dist == "uniform":
            out[lo:hi] = rng.random(hi - lo, dtype=np.float32)
        else:
            raise ValueError(dist)


def generate(shape, dist="normal", seed=BASE_SEED):
    """Return a C-order fp32 array of `shape` drawn from `dist` with `seed`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    shape = tuple(int(s) for s in shape)
    out = np.empty(int(np.prod(shape, dtype=np.int64)), dtype=np.float32)
    if dist == "normal_colscale":
        assert len(shape) == 2
        scale = np.power(10.0, rng.uniform(-2.0, 0.0, shape[1])).astype(np.float32)
        _fill(rng, out, "normal")
        out = out.reshape(shape)
        out *= scale[None, :]
        return out
    _fill(rng, out, dist)
    return out.reshape(shape)


def make(name):
    """Return (workload, Y) for a named workload."""
    w = WORKLOADS[name]
    return w, generate(w.shape, w.dist, w.seed)
