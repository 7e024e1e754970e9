"""Python face of libtrim.so: argument marshalling only.

Every function has the name and meaning of the C entry point in include/trim.h.  Tensors
are torch CUDA (HIP) tensors used purely as device memory; work is enqueued on torch's
current stream.  There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtrim.so")

TRIM_MAX_K = 1024
TRIM_MAX_BATCH = 4096
TRIM_MAX_NPROBE = 4096

EXPORTS = ("trim_shape_supported", "trim_fs_shape_supported", "trim_fs_encode", "trim_fs_build_lut",
           "trim_fs_train_pq", "trim_train_pq", "trim_train_ivf", "trim_estimate_gamma", "trim_estimate_gamma_normal", "trim_encode", "trim_pack_scan_head", "trim_codes_tiled_bytes", "trim_pack_codes_tiled",
           "trim_build_lut", "trim_search_knn",
           "trim_search_range", "trim_search_range_static", "trim_static_scratch_bytes", "trim_range_workspace_bytes", "trim_ivf_probe", "trim_query_order",
           "trim_list_bounds_bytes", "trim_pack_list_bounds",
           "trim_ceiling_stream_read", "trim_ceiling_lds_gather",
           "trim_strerror", "trim_last_hip_error", "trim_version")


class TrimError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().trim_strerror(status).decode()
        if status == -4:
            msg += f" (hipError {lib().trim_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


class TrimCapacityError(RuntimeError):
    def __init__(self, required: int, capacity: int):
        self.required, self.capacity = required, capacity
        super().__init__(f"range search needs room for {required} results, buffer holds {capacity}")


class _IndexView(C.Structure):
    _fields_ = [("n", C.c_int64), ("d", C.c_int32), ("M", C.c_int32), ("base", C.c_void_p),
                ("codes", C.c_void_p), ("dlx", C.c_void_p), ("ids", C.c_void_p),
                ("codebooks", C.c_void_p), ("scan_head", C.c_void_p), ("codes_tiled", C.c_void_p),
                ("code_bits", C.c_int32)]


class _Candidates(C.Structure):
    _fields_ = [("nlist", C.c_int32), ("nprobe", C.c_int32), ("list_offsets", C.c_void_p),
                ("probes", C.c_void_p), ("max_candidates", C.c_int64), ("list_bounds", C.c_void_p)]


class _Stats(C.Structure):
    _fields_ = [("n_scanned", C.c_void_p), ("n_exact", C.c_void_p), ("work", C.c_void_p)]


TRIM_WORK_COUNTERS = 8
WORK_NAMES = ("first_pass", "skipped", "code_bytes", "lookups", "rows", "full_code")


_lib = None


def lib() -> C.CDLL:
    """Load libtrim.so (built in-tree by paper_2508_17828_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2508_17828_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.trim_strerror.restype = C.c_char_p
        L.trim_version.restype = C.c_char_p
        L.trim_range_workspace_bytes.restype = C.c_size_t
        L.trim_range_workspace_bytes.argtypes = [C.c_int64, C.c_int64]
        L.trim_shape_supported.argtypes = [C.c_int32, C.c_int32]
        L.trim_fs_shape_supported.argtypes = [C.c_int32, C.c_int32]
        L.trim_fs_encode.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        L.trim_fs_build_lut.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_void_p]
        L.trim_fs_train_pq.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
        L.trim_encode.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
        L.trim_pack_scan_head.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                          C.c_void_p]
        L.trim_train_pq.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.trim_train_ivf.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        L.trim_estimate_gamma.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_float,
                                          C.c_void_p, C.c_void_p, C.c_void_p]
        L.trim_estimate_gamma_normal.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                                 C.c_float, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.c_void_p]
        L.trim_codes_tiled_bytes.restype = C.c_size_t
        L.trim_codes_tiled_bytes.argtypes = [C.c_int64, C.c_int32]
        L.trim_pack_codes_tiled.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
        L.trim_build_lut.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                     C.c_void_p, C.c_int32, C.c_void_p]
        L.trim_search_knn.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                      C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.trim_list_bounds_bytes.restype = C.c_size_t
        L.trim_list_bounds_bytes.argtypes = [C.c_int32, C.c_int32]
        L.trim_pack_list_bounds.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.trim_ceiling_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p]
        L.trim_ceiling_lds_gather.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.trim_query_order.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.trim_search_range.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_float, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
        L.trim_search_range_static.argtypes = L.trim_search_range.argtypes[:16] + [C.c_void_p]
        L.trim_static_scratch_bytes.restype = C.c_size_t
        L.trim_ivf_probe.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                     C.c_int32, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor], dtype, what: str):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what}: need a contiguous {dtype} tensor on the GPU, got "
                        f"{t.dtype} on {t.device}, contiguous={t.is_contiguous()}")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise TrimError(status, where)


def _codebook_M(codebooks: torch.Tensor, d: int) -> int:
    M = codebooks.shape[0]
    if codebooks.dim() != 3 or codebooks.shape[1] != 256 or M * codebooks.shape[2] != d:
        raise TypeError(f"codebooks: need shape [M][256][d/M] with d={d}, got {tuple(codebooks.shape)}")
    return M


@dataclass
class Index:
    """Device-resident index of Section 3.3: raw vectors, codes, landmark distances, centroids."""
    base: torch.Tensor                    # [n][d] float32
    codes: torch.Tensor                   # [n][M] uint8
    dlx: torch.Tensor                     # [n] float32
    codebooks: torch.Tensor               # [M][256][d/M] float32
    ids: Optional[torch.Tensor] = None    # [n] int32
    list_offsets: Optional[torch.Tensor] = None   # [nlist+1] int64 (device)
    max_list_len: int = 0                 # host copy of the longest list's length
    scan_head: Optional[torch.Tensor] = None      # [n][12] uint8, from trim_pack_scan_head
    codes_tiled: Optional[torch.Tensor] = None    # uint8, from trim_pack_codes_tiled
    list_bounds: Optional[torch.Tensor] = None    # uint8, from trim_pack_list_bounds
    code_bits: int = 8                            # 4: codes [n][M/2], codebooks [M][16][d/M] (trim_fs_encode)

    @property
    def n(self): return self.base.shape[0]
    @property
    def d(self): return self.base.shape[1]
    @property
    def M(self): return self.codebooks.shape[0]

    def _view(self) -> _IndexView:
        return _IndexView(self.n, self.d, self.M, _ptr(self.base, torch.float32, "base"),
                          _ptr(self.codes, torch.uint8, "codes"), _ptr(self.dlx, torch.float32, "dlx"),
                          _ptr(self.ids, torch.int32, "ids"),
                          _ptr(self.codebooks, torch.float32, "codebooks"),
                          _ptr(self.scan_head, torch.uint8, "scan_head"),
                          _ptr(self.codes_tiled, torch.uint8, "codes_tiled"), self.code_bits)

    def _cand(self, probes: Optional[torch.Tensor], max_candidates: int = 0):
        if probes is None:
            return None, self.n
        assert self.list_offsets is not None and probes.dim() == 2
        nprobe = probes.shape[1]
        mc = max_candidates or min(self.n, nprobe * self.max_list_len) or self.n
        c = _Candidates(self.list_offsets.shape[0] - 1, nprobe,
                        _ptr(self.list_offsets, torch.int64, "list_offsets"),
                        _ptr(probes, torch.int32, "probes"), mc,
                        _ptr(self.list_bounds, torch.uint8, "list_bounds"))
        return c, mc


def trim_shape_supported(d: int, M: int) -> bool:
    return bool(lib().trim_shape_supported(d, M))


def trim_fs_shape_supported(d: int, M: int) -> bool:
    return bool(lib().trim_fs_shape_supported(d, M))


def _codebook_fs_M(codebooks: torch.Tensor, d: int) -> int:
    M = codebooks.shape[0]
    if codebooks.dim() != 3 or codebooks.shape[1] != 16 or M * codebooks.shape[2] != d or M % 2:
        raise TypeError(f"codebooks: need shape [M][16][d/M] with d={d} and M even, got {tuple(codebooks.shape)}")
    return M


def trim_fs_encode(base: torch.Tensor, codebooks: torch.Tensor):
    n, d = base.shape
    M = _codebook_fs_M(codebooks, d)
    codes = torch.empty((n, M // 2), dtype=torch.uint8, device=base.device)
    dlx = torch.empty((n,), dtype=torch.float32, device=base.device)
    _check(lib().trim_fs_encode(_ptr(base, torch.float32, "base"), n, d,
                                _ptr(codebooks, torch.float32, "codebooks"), M,
                                _ptr(codes, torch.uint8, "codes"), _ptr(dlx, torch.float32, "dlx"),
                                _stream()), "trim_fs_encode")
    return codes, dlx


def trim_fs_build_lut(queries: torch.Tensor, codebooks: torch.Tensor, out: Optional[torch.Tensor] = None):
    nq, d = queries.shape
    M = _codebook_fs_M(codebooks, d)
    if out is None:
        out = torch.empty((nq, M, 16), dtype=torch.float32, device=queries.device)
    _check(lib().trim_fs_build_lut(_ptr(queries, torch.float32, "queries"), nq, d,
                                   _ptr(codebooks, torch.float32, "codebooks"), M,
                                   _ptr(out, torch.float32, "lut"), _stream()), "trim_fs_build_lut")
    return out


def trim_fs_train_pq(train: torch.Tensor, M: int, iters: int, init_rows: torch.Tensor) -> torch.Tensor:
    ns, d = train.shape
    if d % M or M % 2 or init_rows.numel() != 16:
        raise TypeError(f"trim_fs_train_pq: need d % M == 0, M even and 16 initial rows, got d={d}, M={M}, "
                        f"{init_rows.numel()} rows")
    codebooks = torch.empty((M, 16, d // M), dtype=torch.float32, device=train.device)
    assign = torch.empty((ns, M), dtype=torch.uint8, device=train.device)
    _check(lib().trim_fs_train_pq(_ptr(train, torch.float32, "train"), ns, d, M, iters,
                                  _ptr(init_rows, torch.int32, "init_rows"),
                                  _ptr(codebooks, torch.float32, "codebooks"),
                                  _ptr(assign, torch.uint8, "assign_ws"), _stream()), "trim_fs_train_pq")
    return codebooks


def trim_train_pq(train: torch.Tensor, M: int, iters: int, init_rows: torch.Tensor) -> torch.Tensor:
    ns, d = train.shape
    if d % M or init_rows.numel() != 256:
        raise TypeError(f"trim_train_pq: need d % M == 0 and 256 initial rows, got d={d}, M={M}, "
                        f"{init_rows.numel()} rows")
    codebooks = torch.empty((M, 256, d // M), dtype=torch.float32, device=train.device)
    codes = torch.empty((ns, M), dtype=torch.uint8, device=train.device)
    dlx = torch.empty((ns,), dtype=torch.float32, device=train.device)
    _check(lib().trim_train_pq(_ptr(train, torch.float32, "train"), ns, d, M, iters,
                               _ptr(init_rows, torch.int32, "init_rows"),
                               _ptr(codebooks, torch.float32, "codebooks"), _ptr(codes, torch.uint8, "codes_ws"),
                               _ptr(dlx, torch.float32, "dlx_ws"), _stream()), "trim_train_pq")
    return codebooks


def trim_train_ivf(train: torch.Tensor, nlist: int, iters: int, init_rows: torch.Tensor) -> torch.Tensor:
    ns, d = train.shape
    if init_rows.numel() != nlist:
        raise TypeError(f"trim_train_ivf: need {nlist} initial rows, got {init_rows.numel()}")
    centroids = torch.empty((nlist, d), dtype=torch.float32, device=train.device)
    assign = torch.empty((ns,), dtype=torch.int32, device=train.device)
    _check(lib().trim_train_ivf(_ptr(train, torch.float32, "train"), ns, d, nlist, iters,
                                _ptr(init_rows, torch.int32, "init_rows"),
                                _ptr(centroids, torch.float32, "centroids"),
                                _ptr(assign, torch.int32, "assign_ws"), _stream()), "trim_train_ivf")
    return centroids


def trim_estimate_gamma(index: "Index", sample_rows: torch.Tensor, sample_queries: torch.Tensor, p: float):
    """Returns (gamma [1] float32 on the device, gamma_x [S] float32)."""
    S, Q = sample_rows.numel(), sample_queries.shape[0]
    gx = torch.empty((S,), dtype=torch.float32, device=sample_queries.device)
    g = torch.empty((1,), dtype=torch.float32, device=sample_queries.device)
    view = index._view()
    _check(lib().trim_estimate_gamma(C.byref(view), _ptr(sample_rows, torch.int32, "sample_rows"), S,
                                     _ptr(sample_queries, torch.float32, "sample_queries"), Q, p,
                                     _ptr(gx, torch.float32, "gamma_x"), _ptr(g, torch.float32, "gamma"),
                                     _stream()), "trim_estimate_gamma")
    return g, gx


def trim_estimate_gamma_normal(index: "Index", sample_rows: torch.Tensor, normals: torch.Tensor, p: float,
                               grid: int = 20001):
    """Returns (gamma [1] float32 on the device, gamma_x [S] float32)."""
    S, Q = sample_rows.numel(), normals.shape[0]
    gx = torch.empty((S,), dtype=torch.float32, device=normals.device)
    g = torch.empty((1,), dtype=torch.float32, device=normals.device)
    work = torch.empty((Q, 3), dtype=torch.float64, device=normals.device)
    view = index._view()
    _check(lib().trim_estimate_gamma_normal(C.byref(view), _ptr(sample_rows, torch.int32, "sample_rows"), S,
                                            _ptr(normals, torch.float32, "normals"), Q, p, grid,
                                            _ptr(work, torch.float64, "work"),
                                            _ptr(gx, torch.float32, "gamma_x"), _ptr(g, torch.float32, "gamma"),
                                            _stream()), "trim_estimate_gamma_normal")
    return g, gx


def trim_encode(base: torch.Tensor, codebooks: torch.Tensor):
    n, d = base.shape
    M = _codebook_M(codebooks, d)
    codes = torch.empty((n, M), dtype=torch.uint8, device=base.device)
    dlx = torch.empty((n,), dtype=torch.float32, device=base.device)
    _check(lib().trim_encode(_ptr(base, torch.float32, "base"), n, d,
                             _ptr(codebooks, torch.float32, "codebooks"), M,
                             _ptr(codes, torch.uint8, "codes"), _ptr(dlx, torch.float32, "dlx"),
                             _stream()), "trim_encode")
    return codes, dlx


def trim_pack_scan_head(codes: torch.Tensor, dlx: torch.Tensor) -> torch.Tensor:
    n, M = codes.shape
    head = torch.empty((n, 12), dtype=torch.uint8, device=codes.device)
    _check(lib().trim_pack_scan_head(_ptr(codes, torch.uint8, "codes"), _ptr(dlx, torch.float32, "dlx"),
                                     n, M, _ptr(head, torch.uint8, "head"), _stream()),
           "trim_pack_scan_head")
    return head


def trim_pack_codes_tiled(codes: torch.Tensor) -> torch.Tensor:
    n, M = codes.shape
    tiled = torch.empty((int(lib().trim_codes_tiled_bytes(n, M)),), dtype=torch.uint8, device=codes.device)
    _check(lib().trim_pack_codes_tiled(_ptr(codes, torch.uint8, "codes"), n, M,
                                       _ptr(tiled, torch.uint8, "codes_tiled"), _stream()),
           "trim_pack_codes_tiled")
    return tiled


def trim_build_lut(queries: torch.Tensor, codebooks: torch.Tensor, mfma: bool = False,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
    nq, d = queries.shape
    M = _codebook_M(codebooks, d)
    if out is None:
        out = torch.empty((nq, M, 256), dtype=torch.float32, device=queries.device)
    _check(lib().trim_build_lut(_ptr(queries, torch.float32, "queries"), nq, d,
                                _ptr(codebooks, torch.float32, "codebooks"), M,
                                _ptr(out, torch.float32, "lut"), int(mfma), _stream()),
           "trim_build_lut")
    return out


def trim_search_knn(index: Index, queries: torch.Tensor, k: int, gamma: float, batch: int,
                    probes: Optional[torch.Tensor] = None, lut: Optional[torch.Tensor] = None,
                    want_stats: bool = True, want_mask: bool = False, out=None,
                    query_order: Optional[torch.Tensor] = None, want_work: bool = False):
    """Returns dict(ids [nq][k] int32, d2 [nq][k] float32, n_scanned, n_exact, mask, work)."""
    nq = queries.shape[0]
    dev = queries.device
    if out is None:
        out_ids = torch.empty((nq, k), dtype=torch.int32, device=dev)
        out_d2 = torch.empty((nq, k), dtype=torch.float32, device=dev)
    else:
        out_ids, out_d2 = out
    cand, mc = index._cand(probes)
    ns = ne = None
    stats = None
    if want_stats:
        ns = torch.empty((nq,), dtype=torch.int32, device=dev)
        ne = torch.empty((nq,), dtype=torch.int32, device=dev)
        stats = _Stats(_ptr(ns, torch.int32, "n_scanned"), _ptr(ne, torch.int32, "n_exact"), None)
    work = None
    if want_work:
        work = torch.empty((nq, TRIM_WORK_COUNTERS), dtype=torch.int32, device=dev)
        stats = stats or _Stats(None, None, None)
        stats.work = work.data_ptr()
    mask = None
    mw = 0
    if want_mask:
        mw = (mc + 31) // 32
        mask = torch.empty((nq, mw), dtype=torch.int32, device=dev)
    view = index._view()
    _check(lib().trim_search_knn(C.byref(view), _ptr(queries, torch.float32, "queries"), nq,
                                 _ptr(lut, torch.float32, "lut"),
                                 C.byref(cand) if cand is not None else None, k, gamma, batch,
                                 _ptr(query_order, torch.int32, "query_order"),
                                 _ptr(out_ids, torch.int32, "out_ids"),
                                 _ptr(out_d2, torch.float32, "out_d2"),
                                 C.byref(stats) if stats is not None else None,
                                 _ptr(mask, torch.int32, "mask"), mw, _stream()),
           "trim_search_knn")
    return dict(ids=out_ids, d2=out_d2, n_scanned=ns, n_exact=ne, mask=mask, work=work)


def trim_range_workspace_bytes(nq: int, max_candidates: int) -> int:
    return int(lib().trim_range_workspace_bytes(nq, max_candidates))


def trim_search_range(index: Index, queries: torch.Tensor, radius: float, gamma: float,
                      probes: Optional[torch.Tensor] = None, lut: Optional[torch.Tensor] = None,
                      capacity: int = 0, want_stats: bool = True, want_mask: bool = False,
                      workspace: Optional[torch.Tensor] = None, static_scratch: bool = False,
                      want_work: bool = False, query_order: Optional[torch.Tensor] = None):
    """CSR results in scan order: dict(offsets [nq+1] int64, ids, d2, n_scanned, n_exact, mask).

    Synchronises once to read the result count; raises TrimCapacityError if a caller-given
    capacity is too small (capacity 0 = size the buffers from a first counting call).
    static_scratch: call trim_search_range_static (the library's own scratch area, no workspace)."""
    nq = queries.shape[0]
    dev = queries.device
    cand, mc = index._cand(probes)
    need = trim_range_workspace_bytes(nq, mc)
    if workspace is None and not static_scratch:
        workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
    offsets = torch.empty((nq + 1,), dtype=torch.int64, device=dev)
    required = torch.zeros((1,), dtype=torch.int64, device=dev)
    ns = ne = None
    stats = None
    if want_stats:
        ns = torch.empty((nq,), dtype=torch.int32, device=dev)
        ne = torch.empty((nq,), dtype=torch.int32, device=dev)
        stats = _Stats(_ptr(ns, torch.int32, "n_scanned"), _ptr(ne, torch.int32, "n_exact"), None)
    work = None
    if want_work:
        work = torch.empty((nq, TRIM_WORK_COUNTERS), dtype=torch.int32, device=dev)
        stats = stats or _Stats(None, None, None)
        stats.work = work.data_ptr()
    mask = None
    mw = 0
    if want_mask:
        mw = (mc + 31) // 32
        mask = torch.empty((nq, mw), dtype=torch.int32, device=dev)
    view = index._view()

    def call(cap, oi, od):
        if static_scratch:
            _check(lib().trim_search_range_static(
                C.byref(view), _ptr(queries, torch.float32, "queries"), nq,
                _ptr(lut, torch.float32, "lut"), C.byref(cand) if cand is not None else None,
                radius, gamma, _ptr(query_order, torch.int32, "query_order"),
                _ptr(offsets, torch.int64, "offsets"), _ptr(oi, torch.int32, "out_ids"),
                _ptr(od, torch.float32, "out_d2"), cap, _ptr(required, torch.int64, "required"),
                C.byref(stats) if stats is not None else None, _ptr(mask, torch.int32, "mask"), mw,
                _stream()), "trim_search_range_static")
            return
        _check(lib().trim_search_range(
            C.byref(view), _ptr(queries, torch.float32, "queries"), nq,
            _ptr(lut, torch.float32, "lut"), C.byref(cand) if cand is not None else None,
            radius, gamma, _ptr(query_order, torch.int32, "query_order"),
            _ptr(offsets, torch.int64, "offsets"), _ptr(oi, torch.int32, "out_ids"),
            _ptr(od, torch.float32, "out_d2"), cap, _ptr(required, torch.int64, "required"),
            C.byref(stats) if stats is not None else None, _ptr(mask, torch.int32, "mask"), mw,
            C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream()), "trim_search_range")

    if capacity <= 0:
        call(0, None, None)
        capacity = max(1, int(required.item()))
    out_ids = torch.empty((capacity,), dtype=torch.int32, device=dev)
    out_d2 = torch.empty((capacity,), dtype=torch.float32, device=dev)
    call(capacity, out_ids, out_d2)
    req = int(required.item())
    if req > capacity:
        raise TrimCapacityError(req, capacity)
    return dict(offsets=offsets, ids=out_ids[:req], d2=out_d2[:req], n_scanned=ns, n_exact=ne,
                mask=mask, required=req, work=work)


def trim_ivf_probe(queries: torch.Tensor, centroids: torch.Tensor, nprobe: int) -> torch.Tensor:
    nq, d = queries.shape
    probes = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device)
    _check(lib().trim_ivf_probe(_ptr(queries, torch.float32, "queries"), nq, d,
                                _ptr(centroids, torch.float32, "centroids"), centroids.shape[0],
                                nprobe, _ptr(probes, torch.int32, "probes"), _stream()),
           "trim_ivf_probe")
    return probes


def trim_query_order(probes: torch.Tensor, nlist: int) -> torch.Tensor:
    nq, nprobe = probes.shape
    order = torch.empty((nq,), dtype=torch.int32, device=probes.device)
    _check(lib().trim_query_order(_ptr(probes, torch.int32, "probes"), nq, nprobe, nlist,
                                  _ptr(order, torch.int32, "order"), _stream()), "trim_query_order")
    return order


def trim_pack_list_bounds(index: "Index") -> torch.Tensor:
    """Per-list summaries (occurring codes per subspace, largest landmark distance) for the
    list-level pruning of trim_search_knn."""
    assert index.list_offsets is not None
    nlist = index.list_offsets.shape[0] - 1
    out = torch.empty((lib().trim_list_bounds_bytes(nlist, index.codes.shape[1]),), dtype=torch.uint8,
                      device=index.base.device)
    view = index._view()
    _check(lib().trim_pack_list_bounds(C.byref(view), _ptr(index.list_offsets, torch.int64, "list_offsets"),
                                       nlist, _ptr(out, torch.uint8, "out"), _stream()),
           "trim_pack_list_bounds")
    return out


def trim_ceiling_stream_read(buf: torch.Tensor, blocks: int, sink: torch.Tensor) -> None:
    assert sink.numel() >= blocks
    _check(lib().trim_ceiling_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), blocks,
                                          _ptr(sink, torch.int32, "sink"), _stream()),
           "trim_ceiling_stream_read")


def trim_ceiling_lds_gather(blocks: int, iters: int, seed: int, sink: torch.Tensor,
                            entry_floats: int = 1) -> None:
    assert sink.numel() >= blocks * 512
    _check(lib().trim_ceiling_lds_gather(blocks, iters, entry_floats, seed,
                                         _ptr(sink, torch.float32, "sink"), _stream()),
           "trim_ceiling_lds_gather")
