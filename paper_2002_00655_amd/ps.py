"""Thin binding of the C-ABI library ``libdpaps.so`` (see ``include/dpaps.h``).

Argument marshalling only: every function here hands device pointers of torch
tensors (torch is used for device memory and streams, nothing else) and host
pointers of numpy arrays to the entry point of the same name.  There is no
fallback: if the library has not been built, importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdpaps.so")

PS_OK, PS_EINVAL, PS_EKEY, PS_EWORKER, PS_ECONFLICT, PS_ENOMEM, PS_EHIP, PS_EREMOTE, PS_ELAYOUT, PS_ELIMIT, PS_ESTALL = \
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10
STAT_NAMES = ["pull_local", "pull_remote", "push_local", "push_remote", "relocated", "localize_keys",
              "msg_acc_req", "msg_acc_fwd", "msg_acc_reply", "msg_loc_req", "msg_loc_instruct", "msg_loc_transfer",
              "cache_hit", "cache_stale"]
OPT_MF_EXACT, OPT_MF_CACHE_ROWS, OPT_MF_WAVES, OPT_MF_PROFILE, OPT_MF_GROUPED, OPT_MF_HEAVY_LEN, OPT_PUSH_SEQUENTIAL, OPT_MF_TEAM_MAX, OPT_MF_CLASSIC, OPT_LOCATION_CACHES, OPT_KGE_EXACT = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11

EXPORTS = ["ps_create", "ps_destroy", "ps_pull", "ps_push", "ps_push_noalloc", "ps_localize", "ps_owner", "ps_stats", "ps_status",
           "ps_set_option", "ps_last_error", "mf_block_ratings", "mf_load_ratings", "mf_sgd_epoch", "mf_sgd_epoch_handoff", "mf_train_sse",
           "mf_profile_read", "kge_sgd_step", "kge_sgd_epoch"]


class PSError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str = ""):
        super().__init__(f"{what}: status {code}" + (f" ({detail})" if detail else ""))
        self.code = code


def load_library() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2002_00655_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.ps_create.argtypes = [i64, i32, i32, C.POINTER(vp)]
    lib.ps_destroy.argtypes = [vp]
    lib.ps_pull.argtypes = [vp, i32, vp, i64, vp, vp]
    lib.ps_push.argtypes = [vp, i32, vp, i64, vp, vp]
    lib.ps_push_noalloc.argtypes = [vp, i32, vp, i64, vp, vp]
    lib.ps_localize.argtypes = [vp, vp, i64, i32, vp]
    lib.ps_owner.argtypes = [vp, vp, i64, vp, vp]
    lib.ps_stats.argtypes = [vp, vp, vp]
    lib.ps_status.argtypes = [vp, vp]
    lib.ps_set_option.argtypes = [vp, i32, i64]
    lib.ps_last_error.argtypes = [vp]
    lib.ps_last_error.restype = C.c_char_p
    lib.mf_block_ratings.argtypes = [i64, i64, i64, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.mf_load_ratings.argtypes = [vp, i64, i64, i64, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.mf_sgd_epoch.argtypes = [vp, vp, vp, i32, f32, f32, vp]
    lib.mf_sgd_epoch_handoff.argtypes = [vp, f32, f32, vp, vp]
    lib.mf_train_sse.argtypes = [vp, vp, vp]
    lib.mf_profile_read.argtypes = [vp, vp, vp, vp]
    lib.kge_sgd_step.argtypes = [vp, i32, i64, i32, i64, vp, vp, vp, i32, vp, i32, vp, f32, f32, vp, vp]
    lib.kge_sgd_epoch.argtypes = [vp, i64, i32, i64, vp, vp, vp, i32, vp, i32, vp, vp, i32, i64, i32, f32, f32, vp, vp]
    for name in EXPORTS:
        if name != "ps_last_error":
            getattr(lib, name).restype = C.c_int
    return lib


_lib = load_library()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    return t


def _host(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _flatten_schedule(schedule):
    strata = [np.ascontiguousarray(s, dtype=np.int32).reshape(-1, 3) for s in schedule]
    tasks = np.concatenate(strata) if strata else np.zeros((0, 3), np.int32)
    sptr = np.concatenate([[0], np.cumsum([s.shape[0] for s in strata])]).astype(np.int32)
    return np.ascontiguousarray(tasks), sptr, len(strata)


class ParameterServer:
    """Handle of one server: ``num_keys`` keys x ``value_len`` fp32 values, ``num_workers`` workers."""

    def __init__(self, num_keys: int, value_len: int, num_workers: int):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the parameter server runs on the device only")
        torch.cuda.init()
        torch.cuda.current_stream()
        self.K, self.L, self.W = int(num_keys), int(value_len), int(num_workers)
        h = C.c_void_p()
        rc = _lib.ps_create(self.K, self.L, self.W, C.byref(h))
        if rc:
            raise PSError(rc, "ps_create")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None) and _lib is not None:       # (at interpreter exit the module's globals may be gone)
            _lib.ps_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, rc: int, what: str) -> None:
        if rc:
            raise PSError(rc, what, (_lib.ps_last_error(self._h) or b"").decode())

    # -- primitives -----------------------------------------------------------
    def pull(self, keys: torch.Tensor, worker: int = -1, out: torch.Tensor | None = None) -> torch.Tensor:
        keys = _dev(keys, torch.int64)
        n = keys.numel()
        if out is None:
            out = torch.empty((n, self.L), dtype=torch.float32, device=keys.device)
        _dev(out, torch.float32)
        self._check(_lib.ps_pull(self._h, worker, keys.data_ptr(), n, out.data_ptr(), _stream()), "ps_pull")
        return out

    def push(self, keys: torch.Tensor, deltas: torch.Tensor, worker: int = -1) -> None:
        keys, deltas = _dev(keys, torch.int64), _dev(deltas, torch.float32)
        if deltas.numel() != keys.numel() * self.L:
            raise ValueError("deltas must hold value_len floats per key")
        self._check(_lib.ps_push(self._h, worker, keys.data_ptr(), keys.numel(), deltas.data_ptr(), _stream()), "ps_push")

    def push_noalloc(self, keys: torch.Tensor, deltas: torch.Tensor, worker: int = -1) -> None:
        """ps_push with the library's fixed scratch array: no device allocation (see include/dpaps.h)."""
        keys, deltas = _dev(keys, torch.int64), _dev(deltas, torch.float32)
        if deltas.numel() != keys.numel() * self.L:
            raise ValueError("deltas must hold value_len floats per key")
        self._check(_lib.ps_push_noalloc(self._h, worker, keys.data_ptr(), keys.numel(), deltas.data_ptr(), _stream()), "ps_push_noalloc")

    def localize(self, keys: torch.Tensor, worker: int) -> None:
        keys = _dev(keys, torch.int64)
        self._check(_lib.ps_localize(self._h, keys.data_ptr(), keys.numel(), worker, _stream()), "ps_localize")

    def owner(self, keys: torch.Tensor | None = None) -> torch.Tensor:
        if keys is None:
            keys = torch.arange(self.K, dtype=torch.int64, device="cuda")
        keys = _dev(keys, torch.int64)
        out = torch.empty(keys.numel(), dtype=torch.int32, device=keys.device)
        self._check(_lib.ps_owner(self._h, keys.data_ptr(), keys.numel(), out.data_ptr(), _stream()), "ps_owner")
        return out

    def stats(self) -> dict:
        out = np.zeros(len(STAT_NAMES), dtype=np.int64)
        self._check(_lib.ps_stats(self._h, out.ctypes.data, _stream()), "ps_stats")
        return dict(zip(STAT_NAMES, (int(x) for x in out)))

    def status(self) -> None:
        self._check(_lib.ps_status(self._h, _stream()), "ps_status")

    def set_option(self, option: int, value: int) -> None:
        self._check(_lib.ps_set_option(self._h, option, value), "ps_set_option")

    # -- matrix factorization ---------------------------------------------------
    def mf_load_ratings(self, m, n, rows, cols, vals, row_bounds, col_bounds, block_ptr) -> None:
        rows, cols, vals = _dev(rows, torch.int32), _dev(cols, torch.int32), _dev(vals, torch.float32)
        rb, cb, bp = _host(row_bounds, np.int64), _host(col_bounds, np.int64), _host(block_ptr, np.int64)
        if bp.size != (rb.size - 1) * (cb.size - 1) + 1:
            raise ValueError("block_ptr must have d_row*d_col+1 entries")
        self._check(_lib.mf_load_ratings(self._h, m, n, rows.numel(), rows.data_ptr(), cols.data_ptr(), vals.data_ptr(),
                                         rb.size - 1, cb.size - 1, rb.ctypes.data, cb.ctypes.data, bp.ctypes.data,
                                         _stream()), "mf_load_ratings")
        self._mf_grid = (rb.size - 1, cb.size - 1)

    def mf_sgd_epoch(self, schedule, lr: float, lam: float) -> None:
        """schedule: int32 [S, T, 3] array or list of [T_s, 3] arrays of (worker, row block, column block)."""
        tasks, sptr, ns = _flatten_schedule(schedule)
        self._check(_lib.mf_sgd_epoch(self._h, tasks.ctypes.data, sptr.ctypes.data, ns, float(lr), float(lam), _stream()),
                    "mf_sgd_epoch")

    def mf_sgd_epoch_raw(self, tasks: np.ndarray, sptr: np.ndarray, lr: float, lam: float) -> None:
        self._check(_lib.mf_sgd_epoch(self._h, tasks.ctypes.data, sptr.ctypes.data, sptr.size - 1, float(lr), float(lam),
                                      _stream()), "mf_sgd_epoch")

    def mf_sgd_epoch_handoff(self, lr: float, lam: float, want_order: bool = True):
        """An epoch with column blocks handed from worker to worker (see include/dpaps.h).  Returns the recorded
        order as an int32 array [d_row, d_col, 2] of (column block, workers that had it before), or None."""
        d_row, d_col = self._mf_grid
        order = np.empty((d_row, d_col, 2), dtype=np.int32) if want_order else None
        self._check(_lib.mf_sgd_epoch_handoff(self._h, float(lr), float(lam), order.ctypes.data if want_order else None,
                                              _stream()), "mf_sgd_epoch_handoff")
        return order

    def mf_profile_read(self):
        """(summed SGD kernel time in ms, number of launches) since the last call; needs OPT_MF_PROFILE."""
        ms, cnt = C.c_double(0.0), C.c_int64(0)
        self._check(_lib.mf_profile_read(self._h, C.addressof(ms), C.addressof(cnt), _stream()), "mf_profile_read")
        return float(ms.value), int(cnt.value)

    def mf_train_sse(self) -> float:
        out = C.c_double(0.0)
        self._check(_lib.mf_train_sse(self._h, C.addressof(out), _stream()), "mf_train_sse")
        return float(out.value)

    def kge_sgd_step(self, num_entities, dim, subj, rel, obj, neg_subj, neg_obj, lr, eps, worker: int = -1,
                     want_loss: bool = True):
        """One mini-batch step of ComplEx training (see include/dpaps.h); returns the summed loss or None."""
        subj, rel, obj = _dev(subj, torch.int32), _dev(rel, torch.int32), _dev(obj, torch.int32)
        batch = subj.numel()
        ns_ = _dev(neg_subj, torch.int32).reshape(batch, -1) if batch else torch.zeros((0, 0), dtype=torch.int32)
        no_ = _dev(neg_obj, torch.int32).reshape(batch, -1) if batch else torch.zeros((0, 0), dtype=torch.int32)
        loss = C.c_double(0.0)
        self._check(_lib.kge_sgd_step(self._h, worker, num_entities, dim, batch, subj.data_ptr(), rel.data_ptr(), obj.data_ptr(),
                                      ns_.shape[1], ns_.data_ptr(), no_.shape[1], no_.data_ptr(), float(lr), float(eps),
                                      C.addressof(loss) if want_loss else None, _stream()), "kge_sgd_step")
        return float(loss.value) if want_loss else None

    def kge_sgd_epoch(self, num_entities, dim, subj, rel, obj, neg_subj, neg_obj, part_ptr, batch, lookahead, lr, eps,
                      want_loss: bool = True):
        """One epoch over workers with relation partitioning and pre-localization (see include/dpaps.h)."""
        subj, rel, obj = _dev(subj, torch.int32), _dev(rel, torch.int32), _dev(obj, torch.int32)
        n = subj.numel()
        ns_ = _dev(neg_subj, torch.int32).reshape(n, -1) if n else torch.zeros((0, 0), dtype=torch.int32)
        no_ = _dev(neg_obj, torch.int32).reshape(n, -1) if n else torch.zeros((0, 0), dtype=torch.int32)
        pp = _host(part_ptr, np.int64)
        loss = C.c_double(0.0)
        self._check(_lib.kge_sgd_epoch(self._h, num_entities, dim, n, subj.data_ptr(), rel.data_ptr(), obj.data_ptr(), ns_.shape[1],
                                       ns_.data_ptr(), no_.shape[1], no_.data_ptr(), pp.ctypes.data, pp.size - 1, int(batch),
                                       int(lookahead), float(lr), float(eps), C.addressof(loss) if want_loss else None, _stream()),
                    "kge_sgd_epoch")
        return float(loss.value) if want_loss else None


def mf_block_ratings(m, n, rows, cols, vals, row_bounds, col_bounds):
    """Device version of the block-by-block data layout; returns (rows, cols, vals, block_ptr[host])."""
    rows, cols, vals = _dev(rows, torch.int32), _dev(cols, torch.int32), _dev(vals, torch.float32)
    rb, cb = _host(row_bounds, np.int64), _host(col_bounds, np.int64)
    ro, co, vo = torch.empty_like(rows), torch.empty_like(cols), torch.empty_like(vals)
    bp = np.zeros((rb.size - 1) * (cb.size - 1) + 1, dtype=np.int64)
    rc = _lib.mf_block_ratings(m, n, rows.numel(), rows.data_ptr(), cols.data_ptr(), vals.data_ptr(), rb.size - 1,
                               cb.size - 1, rb.ctypes.data, cb.ctypes.data, ro.data_ptr(), co.data_ptr(), vo.data_ptr(),
                               bp.ctypes.data, _stream())
    if rc:
        raise PSError(rc, "mf_block_ratings")
    return ro, co, vo, bp
