"""Seeded parity cases shared by the GPU tests: inputs from workloads.synth, constants and
expected values from the oracle only (nothing here is produced by the HIP path)."""
from __future__ import annotations

import functools
from dataclasses import dataclass

import numpy as np

from oracle import ivftq_oracle as orc
from workloads import synth


@dataclass
class Case:
    name: str
    X: np.ndarray
    Q: np.ndarray
    cent: np.ndarray      # float32 unit centroids [L, d]
    Pi: np.ndarray        # float32 rotation [d, d]
    c: np.ndarray         # float32 codebook centroids
    tau: np.ndarray       # float32 boundaries
    b: int                # bits stored per coordinate (Stage 1 + sign bit)
    nprobe: int
    k: int
    sign_bit: bool = False

    @property
    def b_stage1(self):
        return self.b - (1 if self.sign_bit else 0)

    @property
    def d(self):
        return self.X.shape[1]

    @property
    def nlist(self):
        return self.cent.shape[0]


def _generic(d, n, nq, seed):
    """A clustered set in an arbitrary dimension (for shapes no workload config has)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 77]))
    means = rng.standard_normal((24, d)).astype(np.float32)
    X = means[rng.integers(0, 24, n)] + 0.35 * rng.standard_normal((n, d), dtype=np.float32)
    Q = means[rng.integers(0, 24, nq)] + 0.35 * rng.standard_normal((nq, d), dtype=np.float32)
    return X.astype(np.float32), Q.astype(np.float32)


_SPECS = {
    # name: (source, n, nq, nlist, b, nprobe, k, kmeans_iters, train_rows)
    "tiny":     ("tiny", 20_000, 200, 64, 4, 8, 10, 10, 20_000),       # the small configuration, whole
    "d128":     ("1m", 30_011, 160, 256, 4, 16, 10, 3, 10_000),        # several tiles + a ragged tail
    "d96_b2":   ("d96", 20_037, 120, 128, 2, 16, 10, 3, 8_000),
    "d96_b3":   ("d96", 20_037, 120, 128, 3, 16, 10, 3, 8_000),
    "d96_b4":   ("d96", 20_037, 120, 128, 4, 32, 10, 3, 8_000),
    "d200":     ("d200", 15_013, 100, 128, 4, 32, 100, 3, 8_000),
    "d100_b5":  ("gen100", 5_003, 64, 32, 5, 5, 7, 3, 5_003),          # d not a multiple of 32
    "d70_b6":   ("gen70", 3_001, 40, 20, 6, 3, 5, 3, 3_001),           # d not a multiple of 4
    "d8_b1":    ("gen8", 1_000, 33, 7, 1, 7, 3, 3, 1_000),             # smallest d, 1 bit, nprobe = nlist
    "d256_b8":  ("gen256", 2_005, 32, 16, 8, 4, 10, 3, 2_005),         # largest d and b: biggest tiles, tables and words
    "d16_b7":   ("gen16", 1_500, 32, 8, 7, 3, 5, 3, 1_500),            # 7-bit codes straddle word boundaries
    # Stage 1 + sign-bit refinement (b here is the Stage-1 width; one more bit is stored)
    "d96_b3s":  ("d96", 20_037, 120, 128, 3, 16, 10, 3, 8_000),         # 4 stored bits: the batched scan covers it
    "d128_b4s": ("1m", 12_007, 90, 128, 4, 16, 10, 3, 8_000),           # 5 stored bits
}


@functools.lru_cache(maxsize=None)
def get_case(name: str) -> Case:
    src, n, nq, nlist, b, nprobe, k, iters, train = _SPECS[name]
    if src == "tiny":
        w = synth.config_tiny()
        X, Q = synth.database(w, 0, n), synth.queries(w, nq)
        seed = w.seed
    elif src == "1m":
        w = synth.config_1m()
        X, Q = synth.database(w, 0, n), synth.queries(w, nq)
        seed = w.seed
    elif src == "d96":
        w = synth.config_10m_d96(b)
        X, Q = synth.database(w, 0, n), synth.queries(w, nq)
        seed = w.seed
    elif src == "d200":
        w = synth.config_10m_d200()
        X, Q = synth.database(w, 0, n), synth.queries(w, nq)
        seed = w.seed
    else:
        d = int(src[3:])
        seed = 5
        X, Q = _generic(d, n, nq, seed)
    d = X.shape[1]
    cent, _ = orc.train_coarse(X[:train], nlist, iters, synth.kmeans_init_indices(seed, train, nlist))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(seed, d))
    if name.endswith("s"):        # sign-bit refinement: the merged 2K-level tables
        c, tau = orc.refined_codebook_fp32(b, d)
        return Case(name, X, Q, cent.astype(np.float32), Pi.astype(np.float32), c, tau, b + 1, nprobe, k, sign_bit=True)
    c, tau = orc.codebook_fp32(b, d)
    return Case(name, X, Q, cent.astype(np.float32), Pi.astype(np.float32), c, tau, b, nprobe, k)


@functools.lru_cache(maxsize=None)
def oracle_encode(name: str):
    cs = get_case(name)
    return orc.encode(cs.X, cs.cent, cs.Pi, cs.tau)


def oracle_index(name: str) -> orc.ListIndex:
    cs = get_case(name)
    enc = oracle_encode(name)
    idx = orc.ListIndex(cs.cent, cs.Pi, cs.c, cs.tau)
    idx.add_encoded(enc["assign"], np.arange(len(cs.X), dtype=np.int64), enc["codes"], enc["gamma16"])
    return idx


ALL_CASES = list(_SPECS)
