"""Python binding of the kgc C ABI (include/kgc.h): argument marshalling only.

Every step of the join runs in the HIP library ``libkgc.so`` built from
``csrc/``; PyTorch is used for device memory and the stream.  There is no CPU
fallback: importing works without a GPU (so the exported symbols can be
checked), but any compute call fails loudly if the library or a device is
missing.

Names follow the C ABI: ``kgc_create``, ``kgc_join``, ``kgc_norms``,
``kgc_get_stats``, ``kgc_last_error``, ``kgc_destroy``, ``kgc_version``.  The
class ``Join`` is a thin convenience wrapper around them.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from . import build as _build

KGC_F32, KGC_BF16 = 0, 1
KGC_PRUNE_AUTO, KGC_PRUNE_OFF, KGC_PRUNE_ON = 0, 1, 2
KGC_OK, KGC_OVERFLOW = 0, 1
KGC_E_INVALID, KGC_E_NOMEM, KGC_E_HIP = -1, -2, -3

EXPORTS = ["kgc_create", "kgc_join", "kgc_join_range", "kgc_join_ab", "kgc_join_se", "kgc_join_blocks", "kgc_top1", "kgc_topk", "kgc_topk_range", "kgc_norms", "kgc_get_stats", "kgc_last_error", "kgc_destroy",
           "kgc_version", "kgc_calibrate_mfma", "kgc_join_static"]


class kgc_triple(ctypes.Structure):
    _fields_ = [("h", ctypes.c_int32), ("r", ctypes.c_int32), ("t", ctypes.c_int32), ("dist", ctypes.c_float)]


class kgc_config(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("max_d", ctypes.c_int32), ("prune", ctypes.c_int32),
                ("tile_cfg", ctypes.c_int32), ("workspace_bytes", ctypes.c_int64), ("stream", ctypes.c_void_p),
                ("group_radius", ctypes.c_float), ("range_kib", ctypes.c_int32), ("factorised", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 3)]


class kgc_stats(ctypes.Structure):
    _fields_ = [("triples_total", ctypes.c_uint64), ("tiles_total", ctypes.c_uint64),
                ("tiles_evaluated", ctypes.c_uint64), ("tiles_pruned", ctypes.c_uint64),
                ("pairs_evaluated", ctypes.c_uint64), ("candidates", ctypes.c_uint64),
                ("emitted", ctypes.c_uint64), ("join_launches", ctypes.c_uint64), ("groups", ctypes.c_uint64),
                ("ms_total", ctypes.c_float), ("ms_precompute", ctypes.c_float), ("ms_prune", ctypes.c_float),
                ("ms_join", ctypes.c_float), ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
                ("k_padded", ctypes.c_int32), ("relation_batches", ctypes.c_int32), ("join_variant", ctypes.c_int32),
                ("exact_blocks", ctypes.c_int32)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


_lib = None


class kgc_cursor(ctypes.Structure):
    """Where a join over blocks stands (include/kgc.h); all zero to start."""
    _fields_ = [("unit", ctypes.c_uint64), ("units", ctypes.c_uint64), ("need", ctypes.c_uint64), ("reserved", ctypes.c_uint64)]


def library_path() -> str:
    return _build.LIB


def load_library():
    """Load libkgc.so.  It is built first when no built library exists.  A library older than its sources is loaded
    as it is, with a warning (a rebuild takes minutes and the GPU tests must not spend them): run
    ``python -m paper_2307_12059_amd.build`` after a change, or set KGC_REBUILD_STALE=1 to have it done here."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    elif _build.stale():
        if os.environ.get("KGC_REBUILD_STALE") == "1":
            _build.build()
        else:
            import warnings
            warnings.warn("libkgc.so is older than its sources: loading it as it is (rebuild with "
                          "`python -m paper_2307_12059_amd.build`)", RuntimeWarning, stacklevel=2)
    lib = ctypes.CDLL(_build.LIB)
    vp = ctypes.c_void_p
    lib.kgc_create.restype = ctypes.c_int
    lib.kgc_create.argtypes = [ctypes.POINTER(kgc_config), ctypes.POINTER(vp)]
    lib.kgc_join.restype = ctypes.c_int
    lib.kgc_join.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32,
                             ctypes.c_float, vp, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_join_static.restype = ctypes.c_int
    lib.kgc_join_static.argtypes = lib.kgc_join.argtypes
    lib.kgc_join_range.restype = ctypes.c_int
    lib.kgc_join_range.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32,
                                   ctypes.c_float, ctypes.c_int32, ctypes.c_int32, vp, ctypes.c_uint64,
                                   ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_join_blocks.restype = ctypes.c_int
    lib.kgc_join_blocks.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                    ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(kgc_cursor), vp, ctypes.c_uint64,
                                    ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_join_se.restype = ctypes.c_int
    lib.kgc_join_se.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                vp, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_join_ab.restype = ctypes.c_int
    lib.kgc_join_ab.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                ctypes.c_float, vp, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_top1.restype = ctypes.c_int
    lib.kgc_top1.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                             ctypes.POINTER(kgc_triple)]
    lib.kgc_topk.restype = ctypes.c_int
    lib.kgc_topk.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                             ctypes.c_uint64, vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_topk_range.restype = ctypes.c_int
    lib.kgc_topk_range.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                   ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64, vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.kgc_norms.restype = ctypes.c_int
    lib.kgc_norms.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, vp, vp]
    lib.kgc_get_stats.restype = ctypes.c_int
    lib.kgc_get_stats.argtypes = [vp, ctypes.POINTER(kgc_stats)]
    lib.kgc_last_error.restype = ctypes.c_char_p
    lib.kgc_last_error.argtypes = [vp]
    lib.kgc_destroy.restype = None
    lib.kgc_destroy.argtypes = [vp]
    lib.kgc_version.restype = ctypes.c_char_p
    lib.kgc_version.argtypes = []
    lib.kgc_calibrate_mfma.restype = ctypes.c_int
    lib.kgc_calibrate_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_float)]
    _lib = lib
    return lib


# ---- the C ABI, one Python function per entry point ----
def kgc_version() -> str:
    return load_library().kgc_version().decode()


def kgc_create(cfg: Optional[kgc_config] = None):
    """Returns (code, handle); handle is an opaque integer (None on failure)."""
    out = ctypes.c_void_p()
    rc = load_library().kgc_create(ctypes.byref(cfg) if cfg is not None else None, ctypes.byref(out))
    return rc, (out.value if rc == KGC_OK else None)


def kgc_destroy(handle) -> None:
    if handle:
        load_library().kgc_destroy(ctypes.c_void_p(handle))


def kgc_last_error(handle) -> str:
    return load_library().kgc_last_error(ctypes.c_void_p(handle)).decode()


def kgc_get_stats(handle) -> dict:
    st = kgc_stats()
    rc = load_library().kgc_get_stats(ctypes.c_void_p(handle), ctypes.byref(st))
    if rc != KGC_OK:
        raise RuntimeError("kgc_get_stats failed")
    return st.as_dict()


def kgc_join(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, delta: float, out_ptr: int, cap: int):
    """Raw call on device addresses.  Returns (code, count)."""
    count = ctypes.c_uint64(0)
    rc = load_library().kgc_join(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R, p,
                                 ctypes.c_float(delta), ctypes.c_void_p(out_ptr), cap, ctypes.byref(count))
    return rc, int(count.value)


def kgc_join_static(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, delta: float, out_ptr: int, cap: int):
    """Raw call on device addresses: the dense join with its scratch in the library's static device array.  Returns (code, count)."""
    count = ctypes.c_uint64(0)
    rc = load_library().kgc_join_static(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R, p,
                                        ctypes.c_float(delta), ctypes.c_void_p(out_ptr), cap, ctypes.byref(count))
    return rc, int(count.value)


def kgc_join_range(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, delta: float, r_begin: int,
                   r_end: int, out_ptr: int, cap: int):
    """Raw call on device addresses, relations r_begin <= r < r_end only.  Returns (code, count)."""
    count = ctypes.c_uint64(0)
    rc = load_library().kgc_join_range(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R,
                                       p, ctypes.c_float(delta), r_begin, r_end, ctypes.c_void_p(out_ptr), cap,
                                       ctypes.byref(count))
    return rc, int(count.value)


def kgc_join_ab(handle, A_ptr: int, B_ptr: int, N: int, d: int, R: int, b_per_relation: bool, p: int, delta: float,
                out_ptr: int, cap: int):
    """Raw call on device addresses: the join on caller-supplied connector outputs.  Returns (code, count)."""
    count = ctypes.c_uint64(0)
    rc = load_library().kgc_join_ab(ctypes.c_void_p(handle), ctypes.c_void_p(A_ptr), ctypes.c_void_p(B_ptr), N, d, R,
                                    1 if b_per_relation else 0, p, ctypes.c_float(delta), ctypes.c_void_p(out_ptr), cap,
                                    ctypes.byref(count))
    return rc, int(count.value)


def kgc_join_blocks(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, delta: float, block_rows: int,
                    rel_block: int, cursor: "kgc_cursor", out_ptr: int, cap: int):
    """Raw call on device addresses: the join block by block; ``cursor`` is updated in place.  Returns (code, count)."""
    count = ctypes.c_uint64(0)
    rc = load_library().kgc_join_blocks(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R, p,
                                        ctypes.c_float(delta), block_rows, rel_block, ctypes.byref(cursor),
                                        ctypes.c_void_p(out_ptr), cap, ctypes.byref(count))
    return rc, int(count.value)


def kgc_join_se(handle, E_ptr: int, N: int, d: int, Wl_ptr: int, Wr_ptr: int, R: int, p: int, delta: float, out_ptr: int,
                cap: int):
    """Raw call on device addresses: the structured-embedding join (connectors formed on the device).  Returns (code, count)."""
    count = ctypes.c_uint64(0)
    rc = load_library().kgc_join_se(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(Wl_ptr),
                                    ctypes.c_void_p(Wr_ptr), R, p, ctypes.c_float(delta), ctypes.c_void_p(out_ptr), cap,
                                    ctypes.byref(count))
    return rc, int(count.value)


def kgc_top1(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, exclude_self: bool):
    """Raw call on device addresses.  Returns (code, kgc_triple)."""
    out = kgc_triple()
    rc = load_library().kgc_top1(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R, p,
                                 1 if exclude_self else 0, ctypes.byref(out))
    return rc, out


def kgc_topk(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, exclude_self: bool, k: int, out_ptr: int):
    """Raw call on device addresses.  Returns (code, found)."""
    found = ctypes.c_uint64(0)
    rc = load_library().kgc_topk(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R, p,
                                 1 if exclude_self else 0, k, ctypes.c_void_p(out_ptr), ctypes.byref(found))
    return rc, int(found.value)


def kgc_topk_range(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, p: int, exclude_self: bool, r_begin: int,
                   r_end: int, k: int, out_ptr: int):
    """Raw call on device addresses.  Returns (code, found)."""
    found = ctypes.c_uint64(0)
    rc = load_library().kgc_topk_range(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R, p,
                                       1 if exclude_self else 0, r_begin, r_end, k, ctypes.c_void_p(out_ptr),
                                       ctypes.byref(found))
    return rc, int(found.value)


def kgc_calibrate_mfma(wave_tile: int, feed: int, ms_target: int, stream: int = 0):
    """Returns (code, TFLOP/s, ms of the timed launch)."""
    tf, ms = ctypes.c_double(0.0), ctypes.c_float(0.0)
    rc = load_library().kgc_calibrate_mfma(wave_tile, feed, ms_target, ctypes.c_void_p(stream), ctypes.byref(tf), ctypes.byref(ms))
    return rc, float(tf.value), float(ms.value)


def kgc_norms(handle, E_ptr: int, N: int, d: int, R_ptr: int, R: int, nB_ptr: int, nA_ptr: int) -> int:
    return load_library().kgc_norms(ctypes.c_void_p(handle), ctypes.c_void_p(E_ptr), N, d, ctypes.c_void_p(R_ptr), R,
                                    ctypes.c_void_p(nB_ptr), ctypes.c_void_p(nA_ptr))


# ---- convenience wrapper over torch tensors ----
class Join:
    """Owns one kgc handle bound to the current torch stream.

    ``E`` and ``Rv`` are CUDA tensors, float32 or bfloat16 (matching ``dtype``),
    contiguous.  ``join`` returns a dict of numpy arrays ``h, r, t, dist``
    (the first min(count, cap) records), ``count``, ``code`` and ``stats``.
    """

    def __init__(self, dtype: str = "f32", prune: int = KGC_PRUNE_AUTO, tile_cfg: int = 0, max_d: int = 0,
                 workspace_bytes: int = 0, group_radius: float = 0.0, range_kib: int = 0,
                 factorised: bool = False):
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("kgc needs a GPU: torch.cuda.is_available() is False and there is no CPU fallback")
        cfg = kgc_config()
        cfg.dtype = {"f32": KGC_F32, "bf16": KGC_BF16}[dtype]
        cfg.prune = prune
        cfg.tile_cfg = tile_cfg
        cfg.max_d = max_d
        cfg.workspace_bytes = workspace_bytes
        cfg.group_radius = group_radius
        cfg.range_kib = range_kib
        cfg.factorised = 1 if factorised else 0
        cfg.stream = torch.cuda.current_stream().cuda_stream
        rc, h = kgc_create(cfg)
        if rc != KGC_OK:
            raise RuntimeError(f"kgc_create failed with code {rc}")
        self.handle = h
        self.dtype = dtype
        self._torch = torch

    def close(self):
        if getattr(self, "handle", None):
            kgc_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, E, Rv):
        torch = self._torch
        want = torch.float32 if self.dtype == "f32" else torch.bfloat16
        for x in (E, Rv):
            if not (x.is_cuda and x.is_contiguous() and x.dtype == want and x.dim() == 2):
                raise ValueError("E and Rv must be contiguous 2-D CUDA tensors of the handle's dtype")
        if E.shape[0] and Rv.shape[0] and E.shape[1] != Rv.shape[1]:
            raise ValueError("E and Rv must share d")

    def join(self, E, Rv, p: int, delta: float, cap: int, out=None, fetch: bool = True, r_range=None) -> dict:
        """``r_range = (r_begin, r_end)`` restricts the join to those relations (kgc_join_range)."""
        torch = self._torch
        self._check(E, Rv)
        N, d = E.shape[0], (E.shape[1] if E.shape[0] else Rv.shape[1])
        R = Rv.shape[0]
        if out is None:
            out = torch.empty((max(cap, 1), 4), dtype=torch.int32, device=E.device)
        if r_range is None:
            rc, count = kgc_join(self.handle, E.data_ptr(), N, d, Rv.data_ptr(), R, p, float(delta), out.data_ptr(), cap)
        else:
            rc, count = kgc_join_range(self.handle, E.data_ptr(), N, d, Rv.data_ptr(), R, p, float(delta),
                                       int(r_range[0]), int(r_range[1]), out.data_ptr(), cap)
        if rc < 0:
            raise RuntimeError(f"kgc_join failed with code {rc}: {kgc_last_error(self.handle)}")
        res = {"code": rc, "count": count, "stats": kgc_get_stats(self.handle), "out": out}
        if fetch:
            n = min(count, cap)
            host = out[:n].cpu().numpy()
            res.update({"h": host[:, 0].copy(), "r": host[:, 1].copy(), "t": host[:, 2].copy(),
                        "dist": host[:, 3].copy().view("float32")})
        return res

    def join_ab(self, A, B, p: int, delta: float, cap: int) -> dict:
        """The general form: ``A`` is R x N x d, ``B`` is N x d (shared) or R x N x d (per relation)."""
        torch = self._torch
        if A.dim() != 3 or B.dim() not in (2, 3) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be R x N x d and B N x d or R x N x d, contiguous")
        if A.dtype != B.dtype or A.dtype != (torch.float32 if self.dtype == "f32" else torch.bfloat16) or not A.is_cuda or not B.is_cuda:
            raise ValueError("A and B must be CUDA tensors of the handle's dtype")
        R, N, d = A.shape
        per_rel = B.dim() == 3
        if tuple(B.shape[-2:]) != (N, d) or (per_rel and B.shape[0] != R):
            raise ValueError("B does not match A")
        out = torch.empty((max(cap, 1), 4), dtype=torch.int32, device=A.device)
        rc, count = kgc_join_ab(self.handle, A.data_ptr(), B.data_ptr(), N, d, R, per_rel, p, float(delta), out.data_ptr(), cap)
        if rc < 0:
            raise RuntimeError(f"kgc_join_ab failed with code {rc}: {kgc_last_error(self.handle)}")
        n = min(count, cap)
        host = out[:n].cpu().numpy()
        return {"code": rc, "count": count, "stats": kgc_get_stats(self.handle), "h": host[:, 0].copy(),
                "r": host[:, 1].copy(), "t": host[:, 2].copy(), "dist": host[:, 3].copy().view("float32")}

    def join_blocks(self, E, Rv, p: int, delta: float, cap: int, block_rows: int, rel_block: int, cursor=None) -> dict:
        """One call of the join block by block: runs units from ``cursor`` on until the buffer of ``cap`` records is
        full or all are done.  Returns the records of the completed units, ``code``, ``count`` and the updated ``cursor``
        (pass it to the next call while ``code`` is KGC_OVERFLOW)."""
        torch = self._torch
        self._check(E, Rv)
        if cursor is None:
            cursor = kgc_cursor()
        N, d = E.shape
        out = torch.empty((max(cap, 1), 4), dtype=torch.int32, device=E.device)
        rc, count = kgc_join_blocks(self.handle, E.data_ptr(), N, d, Rv.data_ptr(), Rv.shape[0], p, float(delta), block_rows,
                                    rel_block, cursor, out.data_ptr(), cap)
        if rc < 0:
            raise RuntimeError(f"kgc_join_blocks failed with code {rc}: {kgc_last_error(self.handle)}")
        host = out[:count].cpu().numpy()
        return {"code": rc, "count": count, "cursor": cursor, "stats": kgc_get_stats(self.handle), "h": host[:, 0].copy(),
                "r": host[:, 1].copy(), "t": host[:, 2].copy(), "dist": host[:, 3].copy().view("float32")}

    def join_se(self, E, W_lhs, W_rhs, p: int, delta: float, cap: int, fetch: bool = True) -> dict:
        """The structured-embedding join: ``E`` is N x d, ``W_lhs`` and ``W_rhs`` are R x d x d.  ``fetch=False`` leaves
        the records on the device (``out``) and returns counts and stats only."""
        torch = self._torch
        want = torch.float32 if self.dtype == "f32" else torch.bfloat16
        for x in (E, W_lhs, W_rhs):
            if not (x.is_cuda and x.is_contiguous() and x.dtype == want):
                raise ValueError("E, W_lhs and W_rhs must be contiguous CUDA tensors of the handle's dtype")
        N, d = E.shape
        R = W_lhs.shape[0]
        if tuple(W_lhs.shape) != (R, d, d) or tuple(W_rhs.shape) != (R, d, d):
            raise ValueError("W_lhs and W_rhs must be R x d x d")
        out = torch.empty((max(cap, 1), 4), dtype=torch.int32, device=E.device)
        rc, count = kgc_join_se(self.handle, E.data_ptr(), N, d, W_lhs.data_ptr(), W_rhs.data_ptr(), R, p, float(delta),
                                out.data_ptr(), cap)
        if rc < 0:
            raise RuntimeError(f"kgc_join_se failed with code {rc}: {kgc_last_error(self.handle)}")
        if not fetch:
            return {"code": rc, "count": count, "stats": kgc_get_stats(self.handle), "out": out}
        n = min(count, cap)
        host = out[:n].cpu().numpy()
        return {"code": rc, "count": count, "stats": kgc_get_stats(self.handle), "h": host[:, 0].copy(),
                "r": host[:, 1].copy(), "t": host[:, 2].copy(), "dist": host[:, 3].copy().view("float32")}

    def top1(self, E, Rv, p: int, exclude_self: bool = False):
        """The triple with the smallest distance (None when no triple is eligible): dict h, r, t, dist."""
        self._check(E, Rv)
        rc, rec = kgc_top1(self.handle, E.data_ptr(), E.shape[0], E.shape[1], Rv.data_ptr(), Rv.shape[0], p, exclude_self)
        if rc < 0:
            raise RuntimeError(f"kgc_top1 failed with code {rc}: {kgc_last_error(self.handle)}")
        if rec.h < 0:
            return None
        return {"h": int(rec.h), "r": int(rec.r), "t": int(rec.t), "dist": float(rec.dist)}

    def topk(self, E, Rv, p: int, k: int, exclude_self: bool = False, r_range=None) -> dict:
        """The k smallest-distance triples, sorted by (dist, r, h, t) on the host: dict h, r, t, dist, count.
        ``r_range = (r_begin, r_end)`` restricts the search to those relations (one relation: its k best pairs)."""
        import numpy as np
        torch = self._torch
        self._check(E, Rv)
        out = torch.empty((max(k, 1), 4), dtype=torch.int32, device=E.device)
        lo, hi = (0, Rv.shape[0]) if r_range is None else (int(r_range[0]), int(r_range[1]))
        rc, found = kgc_topk_range(self.handle, E.data_ptr(), E.shape[0], E.shape[1], Rv.data_ptr(), Rv.shape[0], p,
                                   exclude_self, lo, hi, k, out.data_ptr())
        if rc < 0:
            raise RuntimeError(f"kgc_topk failed with code {rc}: {kgc_last_error(self.handle)}")
        host = out[:found].cpu().numpy()
        h, r, t, dist = host[:, 0].copy(), host[:, 1].copy(), host[:, 2].copy(), host[:, 3].copy().view("float32")
        order = np.lexsort((t, h, r, dist))
        return {"h": h[order], "r": r[order], "t": t[order], "dist": dist[order], "count": found}

    def norms(self, E, Rv, want_nA: bool = True):
        torch = self._torch
        self._check(E, Rv)
        N, d, R = E.shape[0], E.shape[1], Rv.shape[0]
        nB = torch.empty(N, dtype=torch.float32, device=E.device)
        nA = torch.empty((R, N), dtype=torch.float32, device=E.device) if want_nA else None
        rc = kgc_norms(self.handle, E.data_ptr(), N, d, Rv.data_ptr(), R, nB.data_ptr(),
                       nA.data_ptr() if nA is not None else 0)
        if rc < 0:
            raise RuntimeError(f"kgc_norms failed with code {rc}: {kgc_last_error(self.handle)}")
        return nB, nA
