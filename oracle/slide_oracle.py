"""ctypes front end of the CPU oracle (slide_oracle.c) and the step composed from it.

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's cpu_baseline leg
may import this.  It shares no code with the HIP library and never calls it.

The step is composed here in the order of the paper's Algorithm 1: retrieve active
neurons, feed forward, compute errors, backpropagate, Adam, scheduled table rebuild.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slide_oracle.c")
_LIB = os.path.join(_HERE, "libslide_oracle.so")

SIMHASH, DWTA = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no intrinsics, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-fno-fast-math", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Hash(C.Structure):
    _fields_ = [("kind", C.c_int32), ("H", C.c_int32), ("K", C.c_int32), ("L", C.c_int32),
                ("m", C.c_int32), ("S", C.c_int32),
                ("dwta_perm", C.c_void_p), ("srp_idx", C.c_void_p), ("srp_sign", C.c_void_p),
                ("dens_a", C.c_uint32), ("dens_b", C.c_uint32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32, i64, u32, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_double
        L.orc_hidden_forward.argtypes = [i32, i64, i32, vp, vp, vp, vp, vp, vp]
        L.orc_hash_codes.argtypes = [C.POINTER(_Hash), vp, i64, vp]
        L.orc_tables_build.argtypes = [vp, i64, i32, i32, i32, u32, u32, u32]
        L.orc_tables_build.restype = vp
        L.orc_tables_free.argtypes = [vp]
        L.orc_tables_free.restype = None
        L.orc_tables_overflowed.argtypes = [vp]
        L.orc_tables_overflowed.restype = i64
        L.orc_tables_entries.argtypes = [vp, i32]
        L.orc_tables_entries.restype = i64
        L.orc_tables_bucket.argtypes = [vp, i32, u32, vp, i32]
        L.orc_tables_fingerprint.argtypes = [vp]
        L.orc_tables_fingerprint.restype = C.c_uint64
        L.orc_active_sets.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp, vp, vp]
        L.orc_output_forward_backward.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.orc_output_grads.argtypes = [i32, i32, vp, vp, vp, vp, i64, vp, vp, vp]
        L.orc_hidden_grads.argtypes = [i32, i32, vp, vp, vp, vp, i64, vp, vp, vp]
        L.orc_adam_rows.argtypes = [vp, vp, vp, i32, i64, vp, vp, dbl, dbl, dbl, dbl, i64]
        L.orc_num_threads.restype = i32
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    """Number of OpenMP threads the oracle's loops use from now on (the OpenMP runtime's own call)."""
    lib()
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


# --------------------------------------------------------------------------------------
# thin wrappers
# --------------------------------------------------------------------------------------
class HashFn:
    """K*L elementary hash functions grouped into L table codes (Section 4.1)."""

    def __init__(self, kind, H, K, L, m=8, dwta_perm=None, srp_idx=None, srp_sign=None,
                 dens_a=1, dens_b=1):
        self.kind, self.H, self.K, self.L, self.m = int(kind), int(H), int(K), int(L), int(m)
        self._perm = None if dwta_perm is None else _c(dwta_perm, np.int32)
        self._idx = None if srp_idx is None else _c(srp_idx, np.int32)
        self._sgn = None if srp_sign is None else _c(srp_sign, np.int8)
        S = 0 if self._idx is None else self._idx.shape[1]
        self.c = _Hash(self.kind, self.H, self.K, self.L, self.m, S,
                       _p(self._perm), _p(self._idx), _p(self._sgn),
                       int(dens_a) & 0xffffffff, int(dens_b) & 0xffffffff)

    def codes(self, V) -> np.ndarray:
        V = _c(V, np.float32).reshape(-1, self.H)
        out = np.empty((V.shape[0], self.L), dtype=np.uint32)
        rc = lib().orc_hash_codes(C.byref(self.c), _p(V), V.shape[0], _p(out))
        if rc:
            raise ValueError("orc_hash_codes: bad hash configuration")
        return out


class Tables:
    def __init__(self, codes, C_cap, policy, r, prio_a, prio_b):
        codes = _c(codes, np.uint32)
        self.N, self.L = codes.shape
        self.C = int(C_cap)
        self._h = lib().orc_tables_build(_p(codes), self.N, self.L, self.C, int(policy),
                                         int(r) & 0xffffffff, int(prio_a) & 0xffffffff,
                                         int(prio_b) & 0xffffffff)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_tables_free(self._h)
            self._h = None

    def bucket(self, t, code) -> np.ndarray:
        buf = np.empty(self.C, dtype=np.int32)
        n = lib().orc_tables_bucket(self._h, int(t), int(code), _p(buf), self.C)
        return buf[:n].copy()

    @property
    def overflowed(self) -> int:
        return int(lib().orc_tables_overflowed(self._h))

    def entries(self, t) -> int:
        return int(lib().orc_tables_entries(self._h, int(t)))

    def fingerprint(self) -> int:
        return int(lib().orc_tables_fingerprint(self._h))

    def active_sets(self, codes, y_indptr, y_indices, include_labels=True):
        """Returns (as_ptr, ids, is_label, candidates).  Label entries outside [0, N) are left out of
        the sets; their number is kept in self.bad_labels."""
        codes = _c(codes, np.uint32)
        B = codes.shape[0]
        yp, yi = _c(y_indptr, np.int32), _c(y_indices, np.int32)
        as_ptr = np.zeros(B + 1, dtype=np.int64)
        ncand, nbad = C.c_int64(0), C.c_int64(0)
        rc = lib().orc_active_sets(self._h, _p(codes), B, _p(yp), _p(yi), int(include_labels),
                                   _p(as_ptr), None, None, C.byref(ncand), C.byref(nbad))
        assert rc == 0
        self.bad_labels = int(nbad.value)
        ids = np.empty(max(int(as_ptr[-1]), 1), dtype=np.int32)
        lab = np.zeros(max(int(as_ptr[-1]), 1), dtype=np.uint8)
        rc = lib().orc_active_sets(self._h, _p(codes), B, _p(yp), _p(yi), int(include_labels),
                                   _p(as_ptr), _p(ids), _p(lab), None, None)
        assert rc == 0
        A = int(as_ptr[-1])
        return as_ptr, ids[:A], lab[:A], int(ncand.value)


def hidden_forward(D, H, indptr, idx, val, W1, b1) -> np.ndarray:
    indptr, idx, val = _c(indptr, np.int32), _c(idx, np.int32), _c(val, np.float32)
    B = indptr.shape[0] - 1
    h = np.empty((B, H), dtype=np.float32)
    rc = lib().orc_hidden_forward(B, int(D), int(H), _p(indptr), _p(idx), _p(val), _p(W1), _p(b1), _p(h))
    if rc:
        raise ValueError("orc_hidden_forward: feature index out of range")
    return h


def output_forward_backward(h, as_ptr, as_ids, is_label, W2, b2):
    B, H = h.shape
    A = int(as_ptr[-1])
    z, p, d = (np.zeros(max(A, 1)) for _ in range(3))
    loss_i, dh = np.zeros(B), np.zeros((B, H))
    lib().orc_output_forward_backward(B, H, _p(h), _p(as_ptr), _p(as_ids), _p(is_label), _p(W2),
                                      _p(b2), _p(z), _p(p), _p(d), _p(loss_i), _p(dh))
    return z[:A], p[:A], d[:A], loss_i, dh


def output_grads(h, as_ptr, as_ids, delta, uniq):
    B, H = h.shape
    U = uniq.shape[0]
    gW, gb = np.zeros((max(U, 1), H)), np.zeros(max(U, 1))
    d = np.zeros(1) if delta.shape[0] == 0 else delta
    rc = lib().orc_output_grads(B, H, _p(h), _p(as_ptr), _p(as_ids), _p(d), U, _p(uniq), _p(gW), _p(gb))
    assert rc == 0
    return gW[:U], gb[:U]


def hidden_grads(H, indptr, idx, val, dh, uniq1):
    B = indptr.shape[0] - 1
    U1 = uniq1.shape[0]
    gW, gb = np.zeros((max(U1, 1), H)), np.zeros(H)
    rc = lib().orc_hidden_grads(B, H, _p(indptr), _p(idx), _p(val), _p(dh), U1, _p(uniq1), _p(gW), _p(gb))
    assert rc == 0
    return gW[:U1], gb


def adam_rows(W, M, V, ids, g, lr, beta1, beta2, eps, t):
    """In place on fp32 W, M, V (matrix [*, H] or vector)."""
    assert W.dtype == M.dtype == V.dtype == np.float32 and W.flags.c_contiguous
    rowlen = 1 if W.ndim == 1 else W.shape[1]
    ids = _c(ids, np.int32)
    g = _c(g, np.float64)
    lib().orc_adam_rows(_p(W), _p(M), _p(V), rowlen, ids.shape[0], _p(ids), _p(g),
                        float(lr), float(beta1), float(beta2), float(eps), int(t))


# --------------------------------------------------------------------------------------
# the step
# --------------------------------------------------------------------------------------
# --------------------------------------------------------------------------------------
# Sampling budget (Section 3.7: when the tables return more neurons than the budget, a uniform
# random subset of the budget's size is kept -- the paper uses reservoir sampling; when they return
# fewer, the rest of the budget may be filled with uniformly drawn neurons).  The labels are always
# kept and do not count against the budget.  Random numbers come from a counter-based generator,
# so the same (seed, step, sample, neuron / draw number) gives the same number anywhere:
#   mix   = the 32-bit finaliser of MurmurHash3 (a bijection on 32-bit integers)
#   base  = mix(seed + 0x9E3779B9 * step + 0x7F4A7C15 * sample)
#   prio  = mix(base + 0x9E3779B1 * (neuron + 1))         distinct neurons -> distinct priorities
#   draw  = floor(mix((base ^ 0xA5A5A5A5) + 0x632BE5AB * (d + 1)) * N / 2^32)
# Kept subset = the `budget` retrieved non-label neurons of smallest priority.  Fill = draws
# d = 0, 1, 2, ... in order, each accepted if not yet in the set, until the budget is reached or
# 4 * budget + 64 draws are used.
# --------------------------------------------------------------------------------------
_M32 = np.uint64(0xFFFFFFFF)


def sample_mix(x):
    x = np.asarray(x, dtype=np.uint64) & _M32
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x85EBCA6B)) & _M32
    x ^= x >> np.uint64(13)
    x = (x * np.uint64(0xC2B2AE35)) & _M32
    x ^= x >> np.uint64(16)
    return x


def sample_base(seed, step, sample):
    return sample_mix(np.uint64(seed) + np.uint64(0x9E3779B9) * np.uint64(step) + np.uint64(0x7F4A7C15) * np.uint64(sample))


def sample_prio(base, neurons):
    return sample_mix(np.uint64(base) + np.uint64(0x9E3779B1) * (np.asarray(neurons, dtype=np.uint64) + np.uint64(1)))


def sample_draw(base, d, N):
    x = sample_mix((np.uint64(base) ^ np.uint64(0xA5A5A5A5)) + np.uint64(0x632BE5AB) * (np.asarray(d, dtype=np.uint64) + np.uint64(1)))
    return ((x * np.uint64(N)) >> np.uint64(32)).astype(np.int64)


def apply_budget(cand, labels, N, budget, fill, seed, step, sample):
    """cand: retrieved neurons (ascending, unique); labels: the sample's valid distinct labels.
    Returns the non-label members of the active set after the budget rule, ascending."""
    C_ = np.setdiff1d(np.asarray(cand, dtype=np.int64), np.asarray(labels, dtype=np.int64))
    base = sample_base(seed, step, sample)
    if C_.size > budget:
        order = np.argsort(sample_prio(base, C_), kind="stable")
        return np.sort(C_[order[:budget]])
    if fill and C_.size < budget:
        present = set(C_.tolist()) | set(int(y) for y in labels)
        added, need, d, dmax = [], budget - C_.size, 0, 4 * budget + 64
        while need > 0 and d < dmax:
            j = int(sample_draw(base, d, N))
            d += 1
            if j not in present:
                present.add(j)
                added.append(j)
                need -= 1
        return np.sort(np.concatenate([C_, np.array(added, dtype=np.int64)]))
    return C_



class SlideOracle:
    """Model state + one training step.  `weights` arrays are copied; fp32 storage."""

    def __init__(self, *, input_dim, hidden_dim, num_classes, hash_kind, K, L, bucket_cap,
                 rebuild_every, lr, beta1=0.9, beta2=0.999, eps=1e-8, dwta_bin=8,
                 overflow_policy=1, weights, hash_params, sample_budget=0,
                 sample_fill=False, sample_seed=1):
        self.D, self.H, self.N = int(input_dim), int(hidden_dim), int(num_classes)
        self.C, self.R, self.policy = int(bucket_cap), int(rebuild_every), int(overflow_policy)
        self.lr, self.beta1, self.beta2, self.eps = float(lr), float(beta1), float(beta2), float(eps)
        self.budget, self.fill, self.sample_seed = int(sample_budget), bool(sample_fill), int(sample_seed)
        self._hash_shape = (hash_kind, K, L, dwta_bin)
        self.set_hash_params(hash_params)
        self.p = {k: np.array(v, dtype=np.float32, copy=True) for k, v in weights.items()}
        self.m = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.v = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.t = 0            # global step (1-based after the first step)
        self.r = 0            # rebuilds so far
        self.tables = None

    @property
    def dense_hidden(self):
        return self.D == 0

    def set_hash_params(self, hash_params):
        """New hash functions (Algorithm 1 redraws them when it rebuilds the tables); the tables
        must be rebuilt before the next step."""
        kind, K, L, m = self._hash_shape
        self.hp = dict(hash_params)
        self.hash = HashFn(kind, self.H, K, L, m, self.hp.get("dwta_perm"), self.hp.get("srp_idx"),
                           self.hp.get("srp_sign"), self.hp["dens_a"], self.hp["dens_b"])
        self.tables = None

    def build_tables(self, first=True):
        """Tables over the rows of the current W2 (biases are not hashed)."""
        if not first:
            self.r += 1
        self.tables = Tables(self.hash.codes(self.p["W2"]), self.C, self.policy, self.r,
                             self.hp["prio_a"], self.hp["prio_b"])
        return self.tables

    def forward_hidden(self, batch):
        if self.dense_hidden:
            return _c(batch["hidden"], np.float32)
        return hidden_forward(self.D, self.H, batch["x_indptr"], batch["x_indices"],
                              batch["x_values"], self.p["W1"], self.p["b1"])

    def train_step(self, batch, update=True):
        """One step; returns every intermediate.  update=False leaves the state alone."""
        assert self.tables is not None, "build_tables() first"
        out = {}
        h = self.forward_hidden(batch)
        codes = self.hash.codes(h)
        if self.budget > 0:
            as_ptr, as_ids, lab, ncand = self._budgeted_active_sets(codes, batch)
        else:
            as_ptr, as_ids, lab, ncand = self.tables.active_sets(codes, batch["y_indptr"], batch["y_indices"])
        z, p, delta, loss_i, dh = output_forward_backward(h, as_ptr, as_ids, lab, self.p["W2"], self.p["b2"])
        uniq = np.unique(as_ids).astype(np.int32)
        gW2, gb2 = output_grads(h, as_ptr, as_ids, delta, uniq)
        yi_all = _c(batch["y_indices"], np.int32)
        out.update(h=h, codes=codes, as_ptr=as_ptr, as_ids=as_ids, is_label=lab, candidates=ncand,
                   bad_labels=int(np.count_nonzero((yi_all < 0) | (yi_all >= self.N))),
                   z=z, p=p, delta=delta, loss_i=loss_i, loss=float(np.mean(loss_i)), dh=dh,
                   uniq=uniq, gW2=gW2, gb2=gb2)
        if not self.dense_hidden:
            uniq1 = np.unique(batch["x_indices"]).astype(np.int32)
            gW1, gb1 = hidden_grads(self.H, _c(batch["x_indptr"], np.int32), _c(batch["x_indices"], np.int32),
                                    _c(batch["x_values"], np.float32), dh, uniq1)
            out.update(uniq1=uniq1, gW1=gW1, gb1=gb1)
        if update:
            self.t += 1
            a = (self.lr, self.beta1, self.beta2, self.eps, self.t)
            adam_rows(self.p["W2"], self.m["W2"], self.v["W2"], uniq, gW2, *a)
            adam_rows(self.p["b2"], self.m["b2"], self.v["b2"], uniq, gb2, *a)
            if not self.dense_hidden:
                adam_rows(self.p["W1"], self.m["W1"], self.v["W1"], out["uniq1"], out["gW1"], *a)
                adam_rows(self.p["b1"], self.m["b1"], self.v["b1"], np.arange(self.H, dtype=np.int32),
                          out["gb1"], *a)
            out["rebuilt"] = bool(self.R > 0 and self.t % self.R == 0)
            if out["rebuilt"]:
                self.build_tables(first=False)
        return out

    def _budgeted_active_sets(self, codes, batch):
        """Active sets of the step about to run (number self.t + 1) under the sampling budget."""
        yp, yi = _c(batch["y_indptr"], np.int32), _c(batch["y_indices"], np.int32)
        c_ptr, c_ids, _, ncand = self.tables.active_sets(codes, yp, yi, include_labels=False)
        B = codes.shape[0]
        ptr, ids, lab = [0], [], []
        for i in range(B):
            y = yi[yp[i]:yp[i + 1]]
            y = np.unique(y[(y >= 0) & (y < self.N)]).astype(np.int64)
            kept = apply_budget(c_ids[c_ptr[i]:c_ptr[i + 1]], y, self.N, self.budget, self.fill, self.sample_seed,
                                self.t + 1, i)
            allv = np.union1d(kept, y)
            ids.append(allv)
            lab.append(np.isin(allv, y))
            ptr.append(ptr[-1] + allv.size)
        return (np.array(ptr, dtype=np.int64), np.concatenate(ids).astype(np.int32) if ids else np.empty(0, np.int32),
                np.concatenate(lab).astype(np.uint8) if lab else np.empty(0, np.uint8), ncand)

    def predict(self, batch, topk, mode=0):
        """mode 0: scores over the LSH active set without labels; mode 1: over all N.
        Returns ids [B][topk] (-1 padded) and scores; ties go to the lower id."""
        h = self.forward_hidden(batch)
        B = h.shape[0]
        ids = np.full((B, topk), -1, dtype=np.int32)
        sc = np.full((B, topk), -np.inf)
        if mode == 0:
            codes = self.hash.codes(h)
            as_ptr, as_ids, _, _ = self.tables.active_sets(codes, batch["y_indptr"], batch["y_indices"],
                                                           include_labels=False)
        for i in range(B):
            cand = as_ids[as_ptr[i]:as_ptr[i + 1]] if mode == 0 else np.arange(self.N, dtype=np.int32)
            if cand.size == 0:
                continue
            z = self.p["W2"][cand].astype(np.float64) @ h[i].astype(np.float64) + self.p["b2"][cand]
            order = np.lexsort((cand, -z))[:topk]
            ids[i, :order.size] = cand[order]
            sc[i, :order.size] = z[order]
        return ids, sc
