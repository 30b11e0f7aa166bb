"""Seeded synthetic workloads for the SLIDE training step.

This module only draws random inputs (batches, initial weights, hash-function
parameters).  It holds none of the method's arithmetic, so that the CPU oracle
and the HIP library can both be fed from it without sharing any computation.

Every array comes from ``numpy.random.default_rng([seed, stream, step])`` so a
batch can be regenerated from its (seed, step) alone.

The shapes stand in for the extreme-classification workloads of the paper's
Table 1 (135,909 features at 0.055 % density, 670,091 labels) and for the
hyper-parameters of its Section 4.1 (DWTA with K = 6, sparse random projections
with K = 9, Adam constants).  No record of any public dataset is reproduced.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

HASH_SIMHASH = 0
HASH_DWTA = 1

# stream identifiers for default_rng([seed, stream, step])
_S_WEIGHTS, _S_HASH, _S_BATCH_X, _S_BATCH_Y, _S_HIDDEN, _S_PERM = 1, 2, 3, 4, 5, 6


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one synthetic SLIDE workload (symbols as in the paper's Section 4.1:
    K hash functions per table, L tables)."""

    name: str
    input_dim: int          # D; 0 = dense-hidden mode (hidden activations are the input)
    hidden_dim: int         # H
    num_classes: int        # N, output neurons held by this GPU
    batch: int              # B
    hash_kind: int
    K: int
    L: int
    bucket_cap: int         # C
    rebuild_every: int      # R; 0 = never inside the step
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    dwta_bin: int = 8       # m
    overflow_policy: int = 1
    sample_budget: int = 0           # retrieved neurons per sample kept in training (0 = all)
    sample_fill: bool = False        # fill an unmet budget with uniformly drawn neurons
    sample_seed: int = 1
    incremental_rebuild: bool = False   # scheduled rebuilds rehash only the rows updated since the last build
    row_major_mode: int = 0             # 0 = the library decides, 1 = sample-major kernels, 2 = row-major kernels
    # input recipe
    nnz_mode: str = "poisson"        # "exact" | "poisson"
    nnz_mean: float = 75.0
    feat_zipf_s: Optional[float] = 1.0   # None = uniform feature indices
    value_mode: str = "lognormal"    # "uniform" | "lognormal"
    lab_mode: str = "poisson"        # "exact" | "poisson"
    lab_mean: float = 5.0
    lab_zipf_s: Optional[float] = 1.1    # None = uniform labels
    steps: int = 25

    @property
    def dense_hidden(self) -> bool:
        return self.input_dim == 0

    @property
    def num_hashes(self) -> int:      # NH = K * L elementary hash functions
        return self.K * self.L

    @property
    def srp_nnz(self) -> int:         # S: coordinates per sparse random projection
        return -(-self.hidden_dim // 3)

    @property
    def code_bits(self) -> int:
        if self.hash_kind == HASH_DWTA:
            return self.K * int(math.log2(self.dwta_bin))
        return self.K

    @property
    def num_buckets(self) -> int:
        return 1 << self.code_bits


def config(i: int) -> Workload:
    """The five benchmark configurations (0 = tiny plumbing run ... 4 = near-billion parameters),
    then shapes of the paper's other settings (5: second workload at batch 1024, 6-7: batch 2048,
    8: hidden 1024 at batch 1024)."""
    if i == 0:
        return Workload("cfg0-tiny", 1000, 32, 2000, 32, HASH_SIMHASH, 4, 8, 16, 5, lr=1e-3,
                        nnz_mode="exact", nnz_mean=20, feat_zipf_s=None, value_mode="uniform",
                        lab_mode="exact", lab_mean=1, lab_zipf_s=None, steps=10)
    if i == 1:
        return Workload("cfg1-shard167k", 0, 128, 167523, 256, HASH_DWTA, 6, 400, 128, 0,
                        lab_mode="exact", lab_mean=5, lab_zipf_s=1.1)
    if i == 2:
        return Workload("cfg2-670k", 135909, 128, 670091, 256, HASH_DWTA, 6, 400, 128, 50)
    if i == 3:
        return Workload("cfg3-wide325k", 1617899, 128, 325056, 256, HASH_SIMHASH, 9, 50, 128, 50,
                        nnz_mean=42.0, lab_mean=3.0)
    if i == 4:
        return Workload("cfg4-825m", 135909, 1024, 670091, 512, HASH_DWTA, 8, 200, 256, 0)
    if i == 5:   # the paper's second workload (Section 4.1, Table 1): a word-embedding model, one
        # input index per sample, 253,855 -> 200 -> 253,855; its K, L and C are not stated (taken
        # from the sparse-random-projection setting above), word frequencies Zipfian
        return Workload("cfg5-text8-shape", 253855, 200, 253855, 1024, HASH_SIMHASH, 9, 50, 128, 50,
                        nnz_mode="exact", nnz_mean=1, feat_zipf_s=1.0, value_mode="uniform",
                        lab_mode="exact", lab_mean=1, lab_zipf_s=1.0)
    if i == 6:   # 670K-class shape at the paper's low-bandwidth cluster setting: hidden 256, batch 2048
        return Workload("cfg6-670k-b2048-h256", 135909, 256, 670091, 2048, HASH_DWTA, 6, 400, 128, 50)
    if i == 7:   # and at its large-batch setting: hidden 1024, batch 2048
        return Workload("cfg7-670k-b2048-h1024", 135909, 1024, 670091, 2048, HASH_DWTA, 8, 200, 128, 0)
    if i == 8:   # the large-batch experiment's other row: hidden 1024, batch 1024
        return Workload("cfg8-670k-b1024-h1024", 135909, 1024, 670091, 1024, HASH_DWTA, 8, 200, 128, 0)
    raise ValueError("config index must be 0..8")


def small(kind: int = HASH_DWTA, **over) -> Workload:
    """A reduced workload with the same structure (Zipf features and labels, Poisson
    counts) for element-by-element parity tests; spans several tiles and ragged tails."""
    base = dict(name="small", input_dim=3001, hidden_dim=128, num_classes=20011, batch=37,
                hash_kind=kind, K=(3 if kind == HASH_DWTA else 7), L=23, bucket_cap=16,
                rebuild_every=3, lr=1e-3, nnz_mean=30.0, lab_mean=3.0, steps=6)
    base.update(over)
    return Workload(**base)


# --------------------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------------------
def _rng(seed: int, stream: int, step: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream), int(step)])


class _FiniteZipf:
    """Inverse-CDF sampler of P(rank r) proportional to r^-s on ranks 1..n, with the
    rank -> id map a fixed seeded permutation."""

    def __init__(self, n: int, s: float, seed: int, tag: int):
        w = np.arange(1, n + 1, dtype=np.float64) ** (-float(s))
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]
        self.perm = _rng(seed, _S_PERM, tag).permutation(n).astype(np.int64)
        self.n = n

    def draw(self, rng: np.random.Generator, k: int) -> np.ndarray:
        r = np.searchsorted(self.cdf, rng.random(k), side="left")
        return self.perm[np.minimum(r, self.n - 1)]


def _distinct(rng, k: int, n: int, sampler: Optional[_FiniteZipf]) -> np.ndarray:
    """k distinct ids in [0, n), ascending (rejection until enough distinct ones)."""
    k = min(k, n)
    if sampler is None:
        return np.sort(rng.choice(n, size=k, replace=False)).astype(np.int32)
    got = np.empty(0, dtype=np.int64)
    while got.size < k:
        cand = sampler.draw(rng, 2 * (k - got.size) + 4)
        merged = np.concatenate([got, cand])
        _, first = np.unique(merged, return_index=True)
        got = merged[np.sort(first)][:k]
    return np.sort(got).astype(np.int32)


class Generator:
    """Draws weights, hash parameters and a fresh batch per step for one workload."""

    def __init__(self, wl: Workload, seed: int = 0):
        self.wl, self.seed = wl, seed
        self._fz = (None if wl.dense_hidden or wl.feat_zipf_s is None
                    else _FiniteZipf(wl.input_dim, wl.feat_zipf_s, seed, 0))
        self._lz = (None if wl.lab_zipf_s is None
                    else _FiniteZipf(wl.num_classes, wl.lab_zipf_s, seed, 1))

    # ---- parameters --------------------------------------------------------------
    def weights(self) -> dict:
        """Xavier-uniform W1 [D][H] and W2 [N][H]; biases zero."""
        wl, rng = self.wl, _rng(self.seed, _S_WEIGHTS)
        out = {}
        if not wl.dense_hidden:
            a1 = math.sqrt(6.0 / (wl.input_dim + wl.hidden_dim))
            out["W1"] = rng.uniform(-a1, a1, size=(wl.input_dim, wl.hidden_dim)).astype(np.float32)
            out["b1"] = np.zeros(wl.hidden_dim, dtype=np.float32)
        a2 = math.sqrt(6.0 / (wl.hidden_dim + wl.num_classes))
        W2 = np.empty((wl.num_classes, wl.hidden_dim), dtype=np.float32)
        step = 1 << 16
        for lo in range(0, wl.num_classes, step):       # chunked: keeps the fp64 temporary small
            hi = min(lo + step, wl.num_classes)
            W2[lo:hi] = rng.uniform(-a2, a2, size=(hi - lo, wl.hidden_dim))
        out["W2"] = W2
        out["b2"] = np.zeros(wl.num_classes, dtype=np.float32)
        return out

    def hash_params(self, draw: int = 0) -> dict:
        """DWTA: ceil(NH / (H // m)) permutations of the H coordinates.
        SimHash: per bit, S distinct ascending coordinates and their signs.
        Plus the odd 32-bit multipliers of the densification probe and of the
        bucket-overflow priority.  `draw` numbers the redraws (0 = the initial functions)."""
        wl, rng = self.wl, _rng(self.seed, _S_HASH, draw)
        H, NH = wl.hidden_dim, wl.num_hashes
        out = {}
        if wl.hash_kind == HASH_DWTA:
            P = H // wl.dwta_bin
            NP = -(-NH // P)
            out["dwta_perm"] = np.stack([rng.permutation(H) for _ in range(NP)]).astype(np.int32)
        else:
            S = wl.srp_nnz
            idx = np.stack([np.sort(rng.choice(H, size=S, replace=False)) for _ in range(NH)])
            out["srp_idx"] = idx.astype(np.int32)
            out["srp_sign"] = (rng.integers(0, 2, size=(NH, S)) * 2 - 1).astype(np.int8)
        odd = (rng.integers(0, 1 << 31, size=4, dtype=np.int64) * 2 + 1).astype(np.uint32)
        out["dens_a"], out["dens_b"], out["prio_a"], out["prio_b"] = (int(x) for x in odd)
        return out

    # ---- batches -----------------------------------------------------------------
    def _counts(self, rng, mode: str, mean: float, hi: int) -> np.ndarray:
        B = self.wl.batch
        if mode == "exact":
            c = np.full(B, int(mean), dtype=np.int64)
        else:
            c = rng.poisson(mean, size=B)
        return np.clip(c, 1, hi).astype(np.int64)

    def batch(self, step: int) -> dict:
        """One batch: CSR features (or dense hidden activations) and CSR labels."""
        wl = self.wl
        B = wl.batch
        out = {"batch": B}
        if wl.dense_hidden:
            r = _rng(self.seed, _S_HIDDEN, step)
            out["hidden"] = np.maximum(r.standard_normal((B, wl.hidden_dim)), 0).astype(np.float32)
        else:
            r = _rng(self.seed, _S_BATCH_X, step)
            nnz = self._counts(r, wl.nnz_mode, wl.nnz_mean, wl.input_dim)
            indptr = np.zeros(B + 1, dtype=np.int32)
            indptr[1:] = np.cumsum(nnz)
            idx = np.empty(indptr[-1], dtype=np.int32)
            val = np.empty(indptr[-1], dtype=np.float32)
            for i in range(B):
                k = int(nnz[i])
                idx[indptr[i]:indptr[i + 1]] = _distinct(r, k, wl.input_dim, self._fz)
                if wl.value_mode == "uniform":
                    v = 1.0 - r.random(k)                 # (0, 1]
                else:
                    v = r.lognormal(0.0, 1.0, size=k)
                v = v / np.sqrt(np.sum(v * v))
                val[indptr[i]:indptr[i + 1]] = v.astype(np.float32)
            out.update(x_indptr=indptr, x_indices=idx, x_values=val)
        r = _rng(self.seed, _S_BATCH_Y, step)
        nl = self._counts(r, wl.lab_mode, wl.lab_mean, wl.num_classes)
        yptr = np.zeros(B + 1, dtype=np.int32)
        yptr[1:] = np.cumsum(nl)
        yidx = np.empty(yptr[-1], dtype=np.int32)
        for i in range(B):
            yidx[yptr[i]:yptr[i + 1]] = _distinct(r, int(nl[i]), wl.num_classes, self._lz)
        out.update(y_indptr=yptr, y_indices=yidx)
        return out
