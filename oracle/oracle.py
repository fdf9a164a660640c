"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE - not part of the product).

Loads ``dpaps_oracle.c`` compiled for fp32 (``Oracle("f32")``) or fp64
(``Oracle("f64")``) and exposes the parameter-server primitives (Table
"Primitives", Sec. 3.1), the blocked matrix-factorization epoch (Sec. 2.2.2,
Sec. 4.1) and the knowledge-graph-embedding step (``kge_oracle.c``) on numpy arrays.  Nothing here is imported by the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "dpaps_oracle.c"), os.path.join(_HERE, "kge_oracle.c")]
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c99", "-Wall", "-fopenmp"]

STAT_NAMES = ["pull_local", "pull_remote", "push_local", "push_remote", "relocated", "localize_keys",
              "msg_acc_req", "msg_acc_fwd", "msg_acc_reply", "msg_loc_req", "msg_loc_instruct", "msg_loc_transfer",
              "cache_hit", "cache_stale"]

OK, EINVAL, EKEY, EWORKER, ECONFLICT, ENOMEM, EREMOTE = 0, -1, -2, -3, -4, -5, -7


def lib_path(prec: str) -> str:
    return os.path.join(_HERE, f"liboracle_{prec}.so")


def build(force: bool = False) -> None:
    """Compile the oracle with gcc for both precisions (a second or two)."""
    srcs = [s for s in _SRC if os.path.exists(s)]
    for prec, real in (("f32", "float"), ("f64", "double")):
        out = lib_path(prec)
        if not force and os.path.exists(out) and all(os.path.getmtime(out) >= os.path.getmtime(s) for s in srcs):
            continue
        subprocess.check_call(["gcc", *CFLAGS, f"-DREAL={real}", "-o", out, *srcs, "-lm"])


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


class Oracle:
    """One parameter server (K keys x L values, W workers) on the CPU."""

    def __init__(self, prec: str, num_keys: int, value_len: int, num_workers: int):
        build()
        self.prec = prec
        self.dtype = np.float32 if prec == "f32" else np.float64
        self._ct = C.c_float if prec == "f32" else C.c_double
        lib = C.CDLL(lib_path(prec))
        self.lib = lib
        lib.orc_ps_create.restype = C.c_void_p
        lib.orc_ps_create.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        lib.orc_ps_destroy.argtypes = [C.c_void_p]
        lib.orc_mf_train_sse.restype = C.c_double
        assert lib.orc_real_bytes() == np.dtype(self.dtype).itemsize
        self.K, self.L, self.W = int(num_keys), int(value_len), int(num_workers)
        self.h = lib.orc_ps_create(self.K, self.L, self.W)
        if not self.h:
            raise OracleError(EINVAL, "ps_create")

    def close(self):
        if getattr(self, "h", None):
            self.lib.orc_ps_destroy(C.c_void_p(self.h))
            self.h = None

    __del__ = close

    # -- primitives -----------------------------------------------------
    def _keys(self, keys):
        return np.ascontiguousarray(keys, dtype=np.int64)

    def pull(self, keys, worker: int = -1) -> np.ndarray:
        k = self._keys(keys)
        out = np.empty((k.size, self.L), dtype=self.dtype)
        rc = self.lib.orc_ps_pull(C.c_void_p(self.h), C.c_int32(worker), _p(k, C.c_int64), C.c_int64(k.size), _p(out, self._ct))
        if rc:
            raise OracleError(rc, "pull")
        return out

    def push(self, keys, deltas, worker: int = -1) -> None:
        k = self._keys(keys)
        d = np.ascontiguousarray(deltas, dtype=self.dtype).reshape(k.size, self.L)
        rc = self.lib.orc_ps_push(C.c_void_p(self.h), C.c_int32(worker), _p(k, C.c_int64), C.c_int64(k.size), _p(d, self._ct))
        if rc:
            raise OracleError(rc, "push")

    def location_caches(self, on: bool) -> None:
        """Sec. 3.3 "Location caching": switch the per-node location caches on (empty) or off."""
        rc = self.lib.orc_ps_location_caches(C.c_void_p(self.h), C.c_int32(1 if on else 0))
        if rc:
            raise OracleError(rc, "location_caches")

    def localize(self, keys, worker: int) -> None:
        k = self._keys(keys)
        rc = self.lib.orc_ps_localize(C.c_void_p(self.h), _p(k, C.c_int64), C.c_int64(k.size), C.c_int32(worker))
        if rc:
            raise OracleError(rc, "localize")

    def owner(self, keys=None) -> np.ndarray:
        k = np.arange(self.K, dtype=np.int64) if keys is None else self._keys(keys)
        out = np.empty(k.size, dtype=np.int32)
        rc = self.lib.orc_ps_owner(C.c_void_p(self.h), _p(k, C.c_int64), C.c_int64(k.size), _p(out, C.c_int32))
        if rc:
            raise OracleError(rc, "owner")
        return out

    def home(self, keys=None) -> np.ndarray:
        k = np.arange(self.K, dtype=np.int64) if keys is None else self._keys(keys)
        out = np.empty(k.size, dtype=np.int32)
        rc = self.lib.orc_ps_home(C.c_void_p(self.h), _p(k, C.c_int64), C.c_int64(k.size), _p(out, C.c_int32))
        if rc:
            raise OracleError(rc, "home")
        return out

    def stats(self) -> dict:
        out = np.zeros(self.lib.orc_stats_count(), dtype=np.int64)
        self.lib.orc_ps_stats(C.c_void_p(self.h), _p(out, C.c_int64))
        return dict(zip(STAT_NAMES, (int(x) for x in out)))

    # -- matrix factorization -----------------------------------------------
    def mf_sgd_epoch(self, m, n, rows, cols, vals, row_bounds, col_bounds, block_ptr, schedule, lr, lam, classic=False) -> None:
        """schedule: int32 [S, T, 3] array or list of [T_s, 3] arrays of (worker, row block, col block).
        classic: nothing is relocated, every access goes to wherever the key lives (a classic parameter server)."""
        strata = [np.ascontiguousarray(s, dtype=np.int32).reshape(-1, 3) for s in schedule]
        tasks = np.concatenate(strata) if strata else np.zeros((0, 3), np.int32)
        sptr = np.concatenate([[0], np.cumsum([s.shape[0] for s in strata])]).astype(np.int32)
        rb = np.ascontiguousarray(row_bounds, dtype=np.int64)
        cb = np.ascontiguousarray(col_bounds, dtype=np.int64)
        bp = np.ascontiguousarray(block_ptr, dtype=np.int64)
        assert bp.size == (rb.size - 1) * (cb.size - 1) + 1
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        cols = np.ascontiguousarray(cols, dtype=np.int32)
        vals = np.ascontiguousarray(vals, dtype=np.float32)
        rc = (self.lib.orc_mf_sgd_epoch_classic if classic else self.lib.orc_mf_sgd_epoch)(
            C.c_void_p(self.h), C.c_int64(m), C.c_int64(n), _p(rows, C.c_int32), _p(cols, C.c_int32), _p(vals, C.c_float),
            C.c_int32(rb.size - 1), C.c_int32(cb.size - 1), _p(rb, C.c_int64), _p(cb, C.c_int64), _p(bp, C.c_int64),
            _p(tasks, C.c_int32), _p(sptr, C.c_int32), C.c_int32(len(strata)),
            C.c_double(float(np.float32(lr))), C.c_double(float(np.float32(lam))))
        if rc:
            raise OracleError(rc, "mf_sgd_epoch")

    def mf_sgd_epoch_workers(self, m, n, rows, cols, vals, row_bounds, col_bounds, block_ptr, schedule, lr, lam, threads: int = 0) -> int:
        """The epoch with the workers of a subepoch on all host cores (same result as mf_sgd_epoch bit for bit);
        returns the number of threads that ran."""
        strata = [np.ascontiguousarray(s, dtype=np.int32).reshape(-1, 3) for s in schedule]
        tasks = np.concatenate(strata) if strata else np.zeros((0, 3), np.int32)
        sptr = np.concatenate([[0], np.cumsum([s.shape[0] for s in strata])]).astype(np.int32)
        rb = np.ascontiguousarray(row_bounds, dtype=np.int64)
        cb = np.ascontiguousarray(col_bounds, dtype=np.int64)
        bp = np.ascontiguousarray(block_ptr, dtype=np.int64)
        assert bp.size == (rb.size - 1) * (cb.size - 1) + 1
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        cols = np.ascontiguousarray(cols, dtype=np.int32)
        vals = np.ascontiguousarray(vals, dtype=np.float32)
        used = C.c_int32(0)
        rc = self.lib.orc_mf_sgd_epoch_workers(
            C.c_void_p(self.h), C.c_int64(m), C.c_int64(n), _p(rows, C.c_int32), _p(cols, C.c_int32), _p(vals, C.c_float),
            C.c_int32(rb.size - 1), C.c_int32(cb.size - 1), _p(rb, C.c_int64), _p(cb, C.c_int64), _p(bp, C.c_int64),
            _p(tasks, C.c_int32), _p(sptr, C.c_int32), C.c_int32(len(strata)),
            C.c_double(float(np.float32(lr))), C.c_double(float(np.float32(lam))), C.c_int32(threads), C.byref(used))
        if rc:
            raise OracleError(rc, "mf_sgd_epoch_workers")
        return int(used.value)

    def mf_train_sse(self, m, rows, cols, vals) -> float:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        cols = np.ascontiguousarray(cols, dtype=np.int32)
        vals = np.ascontiguousarray(vals, dtype=np.float32)
        return float(self.lib.orc_mf_train_sse(C.c_void_p(self.h), C.c_int64(m), C.c_int64(rows.size),
                                               _p(rows, C.c_int32), _p(cols, C.c_int32), _p(vals, C.c_float)))


    # -- knowledge graph embeddings (ComplEx) ----------------------------------
    def kge_score(self, D, es, wr, eo) -> float:
        """Score of one triple; each argument holds 2 D numbers (real parts, then imaginary parts)."""
        a = [np.ascontiguousarray(x, dtype=self.dtype).reshape(2 * D) for x in (es, wr, eo)]
        self.lib.orc_kge_score.restype = self._ct
        return float(self.lib.orc_kge_score(C.c_int32(D), _p(a[0], self._ct), _p(a[1], self._ct), _p(a[2], self._ct)))

    def kge_step(self, num_entities, D, subj, rel, obj, neg_subj, neg_obj, lr, eps, worker: int = -1) -> float:
        """One mini-batch step (see kge_oracle.c); returns the summed loss of all scored triples."""
        subj, rel, obj = (np.ascontiguousarray(x, dtype=np.int32) for x in (subj, rel, obj))
        B = subj.size
        ns_ = np.ascontiguousarray(neg_subj, dtype=np.int32).reshape(B, -1) if B else np.zeros((0, 0), np.int32)
        no_ = np.ascontiguousarray(neg_obj, dtype=np.int32).reshape(B, -1) if B else np.zeros((0, 0), np.int32)
        loss = C.c_double(0.0)
        real = self._ct
        rc = self.lib.orc_kge_step(
            C.c_void_p(self.h), C.c_int32(worker), C.c_int64(num_entities), C.c_int32(D), C.c_int64(B), _p(subj, C.c_int32),
            _p(rel, C.c_int32), _p(obj, C.c_int32), C.c_int32(ns_.shape[1]), _p(ns_, C.c_int32), C.c_int32(no_.shape[1]),
            _p(no_, C.c_int32), real(float(np.float32(lr))), real(float(np.float32(eps))), C.byref(loss))
        if rc:
            raise OracleError(rc, "kge_step")
        return loss.value

    def kge_epoch(self, num_entities, D, subj, rel, obj, neg_subj, neg_obj, part_ptr, batch, lookahead, lr, eps) -> float:
        """One epoch over triples partitioned over workers (see kge_oracle.c); returns the summed loss."""
        subj, rel, obj = (np.ascontiguousarray(x, dtype=np.int32) for x in (subj, rel, obj))
        n = subj.size
        ns_ = np.ascontiguousarray(neg_subj, dtype=np.int32).reshape(n, -1)
        no_ = np.ascontiguousarray(neg_obj, dtype=np.int32).reshape(n, -1)
        pp = np.ascontiguousarray(part_ptr, dtype=np.int64)
        loss = C.c_double(0.0)
        real = self._ct
        rc = self.lib.orc_kge_epoch(
            C.c_void_p(self.h), C.c_int64(num_entities), C.c_int32(D), _p(subj, C.c_int32), _p(rel, C.c_int32), _p(obj, C.c_int32),
            C.c_int32(ns_.shape[1]), _p(ns_, C.c_int32), C.c_int32(no_.shape[1]), _p(no_, C.c_int32), _p(pp, C.c_int64),
            C.c_int32(pp.size - 1), C.c_int64(batch), C.c_int32(lookahead), real(float(np.float32(lr))), real(float(np.float32(eps))),
            C.byref(loss))
        if rc:
            raise OracleError(rc, "kge_epoch")
        return loss.value


def mf_block_ratings(m, n, rows, cols, vals, row_bounds, col_bounds):
    """Entries stored block by block for the subepochs (Sec. 2.2.2); returns
    (rows, cols, vals, block_ptr)."""
    build()
    lib = C.CDLL(lib_path("f32"))
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    rb = np.ascontiguousarray(row_bounds, dtype=np.int64)
    cb = np.ascontiguousarray(col_bounds, dtype=np.int64)
    ro, co, vo = np.empty_like(rows), np.empty_like(cols), np.empty_like(vals)
    bp = np.zeros((rb.size - 1) * (cb.size - 1) + 1, dtype=np.int64)
    rc = lib.orc_mf_block_ratings(C.c_int64(m), C.c_int64(n), C.c_int64(rows.size), _p(rows, C.c_int32), _p(cols, C.c_int32),
                                  _p(vals, C.c_float), C.c_int32(rb.size - 1), C.c_int32(cb.size - 1), _p(rb, C.c_int64),
                                  _p(cb, C.c_int64), _p(ro, C.c_int32), _p(co, C.c_int32), _p(vo, C.c_float), _p(bp, C.c_int64))
    if rc:
        raise OracleError(rc, "mf_block_ratings")
    return ro, co, vo, bp
