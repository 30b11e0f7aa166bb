"""Thin ctypes binding of libslide_hip.so (same names as include/slide.h) plus a small helper that
owns the device buffers as torch tensors.  Argument marshalling only: every step of the path runs in
the HIP kernels.  PyTorch is used for device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libslide_hip.so")

SLIDE_OK, SLIDE_EINVAL, SLIDE_ENOMEM, SLIDE_EHIP, SLIDE_ESTATE, SLIDE_EDATA = 0, -1, -2, -3, -4, -5
HASH_SIMHASH, HASH_DWTA = 0, 1
KEEP_LOWEST_ID, KEEP_PRIORITY = 0, 1
FLAG_BAD_FEATURE, FLAG_UNSORTED, FLAG_BAD_LABEL = 1, 2, 4
ABI_VERSION = 4
ROWS_AUTO, ROWS_NEVER, ROWS_ALWAYS = 0, 1, 2
STATIC_MAX_BATCH = 64
STAGES = ["hidden", "lookup", "forward", "combine", "update", "rebuild"]
NUM_STAGES = len(STAGES)

EXPORTS = ["slide_query_memory", "slide_init", "slide_build_tables", "slide_set_hash_params", "slide_train_step",
           "slide_predict", "slide_predict_static",
           "slide_status", "slide_get_stats", "slide_profile", "slide_profile_read", "slide_reset_stats", "slide_destroy", "slide_last_error", "slide_debug_copy", "slide_debug_hash",
           "slide_debug_get_bucket", "slide_debug_get_active", "slide_debug_get_hidden"]


class slide_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("abi_version", C.c_uint32),
                ("input_dim", C.c_int64), ("num_classes", C.c_int64),
                ("hidden_dim", C.c_int32), ("max_batch", C.c_int32),
                ("max_nnz_per_batch", C.c_int32), ("max_labels_per_batch", C.c_int32),
                ("hash_kind", C.c_int32), ("K", C.c_int32), ("L", C.c_int32), ("dwta_bin", C.c_int32),
                ("srp_nnz", C.c_int32), ("bucket_cap", C.c_int32), ("overflow_policy", C.c_int32),
                ("rebuild_every", C.c_int32),
                ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("sample_budget", C.c_int32), ("sample_fill", C.c_int32), ("sample_seed", C.c_uint32),
                ("incremental_rebuild", C.c_int32), ("row_major_mode", C.c_int32)]


class slide_mem_req(C.Structure):
    _fields_ = [("tables_bytes", C.c_size_t), ("workspace_bytes", C.c_size_t)]


class slide_buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("W1", "b1", "W2", "b2", "mW1", "vW1", "mb1", "vb1", "mW2", "vW2",
                                          "mb2", "vb2")] + \
               [("tables", C.c_void_p), ("tables_bytes", C.c_size_t),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class slide_hash_params(C.Structure):
    _fields_ = [("dwta_perm", C.c_void_p), ("srp_idx", C.c_void_p), ("srp_sign", C.c_void_p),
                ("dens_a", C.c_uint32), ("dens_b", C.c_uint32), ("prio_a", C.c_uint32), ("prio_b", C.c_uint32)]


class slide_batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("nnz", C.c_int32), ("num_labels", C.c_int32),
                ("x_indptr", C.c_void_p), ("x_indices", C.c_void_p), ("x_values", C.c_void_p),
                ("hidden", C.c_void_p), ("y_indptr", C.c_void_p), ("y_indices", C.c_void_p),
                ("dhidden_out", C.c_void_p)]


class slide_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("active_pairs", "unique_out_rows", "unique_in_rows", "candidates",
                                         "overflowed_buckets", "steps", "rebuilds", "rehashed_rows", "sum_active_pairs",
                                         "sum_unique_out_rows", "sum_unique_in_rows", "sum_candidates",
                                         "sum_steps")]


_lib = None


def load_library(path: str = LIB_PATH):
    """Loads the built library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise RuntimeError("libslide_hip.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # torch ships its own HIP runtime (same soname as the system one).  It must be the one already
    # mapped when this library is loaded, or the process ends up with two runtimes that do not see
    # each other's device memory.
    import torch  # noqa: F401
    L = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    L.slide_query_memory.argtypes = [C.POINTER(slide_config), C.POINTER(slide_mem_req)]
    L.slide_init.argtypes = [C.POINTER(slide_config), C.POINTER(slide_buffers), C.POINTER(slide_hash_params),
                             C.POINTER(vp)]
    L.slide_build_tables.argtypes = [vp, vp]
    L.slide_set_hash_params.argtypes = [vp, vp, vp]
    L.slide_train_step.argtypes = [vp, C.POINTER(slide_batch), vp, vp]
    L.slide_predict.argtypes = [vp, C.POINTER(slide_batch), i32, i32, vp, vp, vp]
    L.slide_predict_static.argtypes = [vp, C.POINTER(slide_batch), i32, vp, vp, vp]
    L.slide_status.argtypes = [vp, vp, C.POINTER(C.c_uint32)]
    L.slide_get_stats.argtypes = [vp, vp, C.POINTER(slide_stats)]
    L.slide_profile.argtypes = [vp, C.c_uint32]
    L.slide_profile_read.argtypes = [vp, vp, vp, vp]
    L.slide_reset_stats.argtypes = [vp, vp]
    L.slide_destroy.argtypes = [vp]
    L.slide_last_error.argtypes = [vp]
    L.slide_last_error.restype = C.c_char_p
    L.slide_debug_copy.argtypes = [vp, vp, C.c_size_t, vp]
    L.slide_debug_hash.argtypes = [vp, vp, i64, vp, vp]
    L.slide_debug_get_bucket.argtypes = [vp, i32, C.c_uint32, vp, i32, C.POINTER(C.c_int)]
    L.slide_debug_get_active.argtypes = [vp, vp, vp, vp, vp, vp, i64]
    L.slide_debug_get_hidden.argtypes = [vp, vp, vp]
    for n in EXPORTS:
        if n != "slide_last_error":
            getattr(L, n).restype = C.c_int
    _lib = L
    return L


class SlideError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("slide error %d: %s" % (code, msg))
        self.code = code


def make_config(*, input_dim, hidden_dim, num_classes, max_batch, max_nnz_per_batch, max_labels_per_batch,
                hash_kind, K, L, bucket_cap, rebuild_every, lr, beta1=0.9, beta2=0.999, eps=1e-8, dwta_bin=8,
                srp_nnz=0, overflow_policy=KEEP_PRIORITY, sample_budget=0, sample_fill=False,
                sample_seed=1, incremental_rebuild=False, row_major_mode=ROWS_AUTO) -> slide_config:
    c = slide_config()
    c.struct_size, c.abi_version = C.sizeof(slide_config), ABI_VERSION
    c.input_dim, c.num_classes, c.hidden_dim, c.max_batch = input_dim, num_classes, hidden_dim, max_batch
    c.max_nnz_per_batch, c.max_labels_per_batch = max_nnz_per_batch, max_labels_per_batch
    c.hash_kind, c.K, c.L, c.dwta_bin, c.srp_nnz, c.bucket_cap = hash_kind, K, L, dwta_bin, srp_nnz, bucket_cap
    c.overflow_policy, c.rebuild_every = overflow_policy, rebuild_every
    c.lr, c.beta1, c.beta2, c.eps = lr, beta1, beta2, eps
    c.sample_budget, c.sample_fill, c.sample_seed = sample_budget, int(bool(sample_fill)), sample_seed
    c.incremental_rebuild = int(bool(incremental_rebuild))
    c.row_major_mode = int(row_major_mode)
    return c


def debug_copy(dst, src, stream_ptr: int):
    """Plain copy kernel of the library on two equally sized device tensors (measurement aid)."""
    L = load_library()
    nbytes = src.numel() * src.element_size()
    rc = L.slide_debug_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, C.c_void_p(stream_ptr))
    if rc:
        raise SlideError(rc, "slide_debug_copy")


def query_memory(cfg: slide_config) -> slide_mem_req:
    L = load_library()
    req = slide_mem_req()
    rc = L.slide_query_memory(C.byref(cfg), C.byref(req))
    if rc:
        raise SlideError(rc, L.slide_last_error(None).decode())
    return req


class Slide:
    """Owns the device buffers (torch tensors) of one model and forwards calls to the C ABI."""

    def __init__(self, cfg: slide_config, weights: dict, hash_params: dict, device="cuda:0"):
        import torch
        self.torch = torch
        self.L = load_library()
        self.cfg = cfg
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.dense_hidden = cfg.input_dim == 0
        f32 = torch.float32
        self.p, self.m, self.v = {}, {}, {}
        names = ["W2", "b2"] + ([] if self.dense_hidden else ["W1", "b1"])
        for n in names:
            self.p[n] = torch.from_numpy(np.ascontiguousarray(weights[n], dtype=np.float32)).to(self.dev)
            self.m[n] = torch.zeros_like(self.p[n])
            self.v[n] = torch.zeros_like(self.p[n])
        req = query_memory(cfg)
        self.mem = (req.tables_bytes, req.workspace_bytes)
        self.tables = torch.empty(req.tables_bytes, dtype=torch.uint8, device=self.dev)
        self.workspace = torch.empty(req.workspace_bytes, dtype=torch.uint8, device=self.dev)
        self.d_loss = torch.zeros(1, dtype=f32, device=self.dev)
        b = slide_buffers()
        for n in names:
            setattr(b, n, self.p[n].data_ptr())
            setattr(b, "m" + n, self.m[n].data_ptr())
            setattr(b, "v" + n, self.v[n].data_ptr())
        b.tables, b.tables_bytes = self.tables.data_ptr(), req.tables_bytes
        b.workspace, b.workspace_bytes = self.workspace.data_ptr(), req.workspace_bytes
        hp = self._hash_struct(hash_params)
        self.ctx = C.c_void_p()
        rc = self.L.slide_init(C.byref(cfg), C.byref(b), C.byref(hp), C.byref(self.ctx))
        if rc:
            raise SlideError(rc, self.L.slide_last_error(None).decode())
        self._batch_keep = None

    # ---- helpers ---------------------------------------------------------------------------
    def _hash_struct(self, hash_params: dict):
        hp = slide_hash_params()
        self._keep = []
        for key, dt in (("dwta_perm", np.int32), ("srp_idx", np.int32), ("srp_sign", np.int8)):
            if hash_params.get(key) is not None:
                a = np.ascontiguousarray(hash_params[key], dtype=dt)
                self._keep.append(a)
                setattr(hp, key, a.ctypes.data)
        hp.dens_a, hp.dens_b = hash_params["dens_a"], hash_params["dens_b"]
        hp.prio_a, hp.prio_b = hash_params["prio_a"], hash_params["prio_b"]
        return hp

    def _check(self, rc):
        if rc:
            raise SlideError(rc, self.L.slide_last_error(self.ctx).decode())

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.dev).cuda_stream)

    def to_device(self, batch: dict) -> dict:
        """Copies a host batch (numpy arrays) to the device once; the result can be reused."""
        t = self.torch
        out = {"batch": int(batch["batch"])}
        for k in ("x_indptr", "x_indices", "x_values", "hidden", "y_indptr", "y_indices"):
            if batch.get(k) is not None:
                a = batch[k]
                out[k] = a.to(self.dev) if isinstance(a, t.Tensor) else t.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        out["nnz"] = int(batch["x_indptr"][-1]) if batch.get("x_indptr") is not None else 0
        out["num_labels"] = int(batch["y_indptr"][-1]) if batch.get("y_indptr") is not None else 0
        return out

    def _marshal(self, db: dict, dhidden_out=None) -> slide_batch:
        b = slide_batch()
        b.batch, b.nnz, b.num_labels = db["batch"], db["nnz"], db["num_labels"]
        for k in ("x_indptr", "x_indices", "x_values", "hidden", "y_indptr", "y_indices"):
            if k in db:
                setattr(b, k, db[k].data_ptr())
        if dhidden_out is not None:
            b.dhidden_out = dhidden_out.data_ptr()
        self._batch_keep = db
        return b

    # ---- the C ABI ---------------------------------------------------------------------------
    def build_tables(self):
        self._check(self.L.slide_build_tables(self.ctx, self._stream()))

    def set_hash_params(self, hash_params: dict):
        hp = self._hash_struct(hash_params)
        self._check(self.L.slide_set_hash_params(self.ctx, C.byref(hp), self._stream()))

    def train_step(self, db: dict, dhidden_out=None):
        """Enqueues one step; returns the device tensor holding the loss (no synchronisation)."""
        b = self._marshal(db, dhidden_out)
        self._check(self.L.slide_train_step(self.ctx, C.byref(b), C.c_void_p(self.d_loss.data_ptr()), self._stream()))
        return self.d_loss

    def predict(self, db: dict, topk: int, mode: int = 0):
        t = self.torch
        ids = t.empty((db["batch"], topk), dtype=t.int32, device=self.dev)
        sc = t.empty((db["batch"], topk), dtype=t.float32, device=self.dev)
        b = self._marshal(db)
        self._check(self.L.slide_predict(self.ctx, C.byref(b), mode, topk, C.c_void_p(ids.data_ptr()),
                                         C.c_void_p(sc.data_ptr()), self._stream()))
        return ids, sc

    def predict_static(self, db: dict, topk: int, out=None):
        """slide_predict_static: scores over all neurons with the library's static scratch; the output
        tensors may be passed in (then nothing is allocated on the way)."""
        t = self.torch
        if out is None:
            out = (t.empty((db["batch"], topk), dtype=t.int32, device=self.dev),
                   t.empty((db["batch"], topk), dtype=t.float32, device=self.dev))
        ids, sc = out
        b = self._marshal(db)
        self._check(self.L.slide_predict_static(self.ctx, C.byref(b), topk, C.c_void_p(ids.data_ptr()),
                                                C.c_void_p(sc.data_ptr()), self._stream()))
        return ids, sc

    def status(self) -> int:
        flags = C.c_uint32(0)
        rc = self.L.slide_status(self.ctx, self._stream(), C.byref(flags))
        if rc not in (SLIDE_OK, SLIDE_EDATA):
            self._check(rc)
        return int(flags.value)

    def stats(self) -> dict:
        s = slide_stats()
        self._check(self.L.slide_get_stats(self.ctx, self._stream(), C.byref(s)))
        return {n: int(getattr(s, n)) for n, _ in slide_stats._fields_}

    def reset_stats(self):
        self._check(self.L.slide_reset_stats(self.ctx, self._stream()))

    def profile(self, stage_mask: int):
        self._check(self.L.slide_profile(self.ctx, stage_mask))

    def profile_read(self):
        ms = np.zeros(NUM_STAGES, dtype=np.float64)
        n = np.zeros(NUM_STAGES, dtype=np.int64)
        self._check(self.L.slide_profile_read(self.ctx, self._stream(), ms.ctypes.data, n.ctypes.data))
        return ms, n

    def destroy(self):
        if self.ctx:
            self.L.slide_destroy(self.ctx)
            self.ctx = C.c_void_p()

    # ---- read-backs ----------------------------------------------------------------------------
    def debug_hash(self, vectors) -> np.ndarray:
        t = self.torch
        v = t.from_numpy(np.ascontiguousarray(vectors, dtype=np.float32)).to(self.dev)
        out = t.empty((v.shape[0], self.cfg.L), dtype=t.int32, device=self.dev)
        self._check(self.L.slide_debug_hash(self.ctx, C.c_void_p(v.data_ptr()), v.shape[0],
                                            C.c_void_p(out.data_ptr()), self._stream()))
        t.cuda.synchronize()
        return out.cpu().numpy().view(np.uint32)

    def debug_bucket(self, table: int, code: int) -> np.ndarray:
        buf = np.empty(self.cfg.bucket_cap, dtype=np.int32)
        n = C.c_int(0)
        self._check(self.L.slide_debug_get_bucket(self.ctx, table, code, buf.ctypes.data, buf.shape[0], C.byref(n)))
        return buf[:n.value].copy()

    def debug_active(self):
        B = self._batch_keep["batch"]
        as_ptr = np.zeros(B + 1, dtype=np.int64)
        rc = self.L.slide_debug_get_active(self.ctx, as_ptr.ctypes.data, None, None, None, None, 0)
        if rc not in (SLIDE_OK, SLIDE_ENOMEM):
            self._check(rc)
        A = int(as_ptr[-1])
        ids, lab = np.empty(max(A, 1), np.int32), np.empty(max(A, 1), np.uint8)
        z, d = np.empty(max(A, 1), np.float32), np.empty(max(A, 1), np.float32)
        self._check(self.L.slide_debug_get_active(self.ctx, as_ptr.ctypes.data, ids.ctypes.data, lab.ctypes.data,
                                                  z.ctypes.data, d.ctypes.data, max(A, 1)))
        return as_ptr, ids[:A], lab[:A], z[:A], d[:A]

    def debug_hidden(self, want_grad=True):
        B, H = self._batch_keep["batch"], self.cfg.hidden_dim
        h = np.empty((B, H), np.float32)
        dh = np.empty((B, H), np.float32) if want_grad else None
        self._check(self.L.slide_debug_get_hidden(self.ctx, h.ctypes.data, None if dh is None else dh.ctypes.data))
        return h, dh


def config_from_workload(wl, max_nnz_per_batch=None, max_labels_per_batch=None) -> slide_config:
    """slide_config for a synth.Workload (capacities default to generous multiples of the means)."""
    if max_nnz_per_batch is None:
        max_nnz_per_batch = 0 if wl.dense_hidden else int(wl.batch * (wl.nnz_mean * 2 + 64))
    if max_labels_per_batch is None:
        max_labels_per_batch = int(wl.batch * (wl.lab_mean * 3 + 16))
    return make_config(input_dim=wl.input_dim, hidden_dim=wl.hidden_dim, num_classes=wl.num_classes,
                       max_batch=wl.batch, max_nnz_per_batch=max_nnz_per_batch,
                       max_labels_per_batch=max_labels_per_batch, hash_kind=wl.hash_kind, K=wl.K, L=wl.L,
                       bucket_cap=wl.bucket_cap, rebuild_every=wl.rebuild_every, lr=wl.lr, beta1=wl.beta1,
                       beta2=wl.beta2, eps=wl.eps, dwta_bin=wl.dwta_bin,
                       srp_nnz=wl.srp_nnz if wl.hash_kind == HASH_SIMHASH else 0,
                       overflow_policy=wl.overflow_policy, sample_budget=wl.sample_budget,
                       sample_fill=wl.sample_fill, sample_seed=wl.sample_seed,
                       incremental_rebuild=wl.incremental_rebuild, row_major_mode=wl.row_major_mode)
