"""ctypes face of oracle/trim_oracle.c (test infrastructure; see that file's header).

Every function takes and returns numpy arrays; argument checking only, no arithmetic.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


def _cpu_has_v3() -> bool:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    fl = set(line.split(":")[1].split())
                    return {"avx2", "fma", "bmi2", "movbe", "f16c"} <= fl
    except OSError:
        pass
    return False


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        names = ["libtrim_oracle_v3.so", "libtrim_oracle.so"] if _cpu_has_v3() else ["libtrim_oracle.so"]
        path = next((os.path.join(_HERE, n) for n in names
                     if os.path.exists(os.path.join(_HERE, n))), None)
        if path is None:
            from . import build as _b
            _b.build()
            path = os.path.join(_HERE, names[0])
        _lib = C.CDLL(path)
        _lib.trim_oracle_exact_d2.restype = C.c_float
        _lib.trim_oracle_plb_from_s.restype = C.c_float
        _lib.trim_oracle_plb_from_s.argtypes = [C.c_float, C.c_float, C.c_float]
    return _lib


def _p(a, dtype):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], \
        (getattr(a, "dtype", None), dtype)
    return a.ctypes.data_as(C.c_void_p)


f32, u8, i32, i64, u32, f64 = (np.dtype(t) for t in
                               ("float32", "uint8", "int32", "int64", "uint32", "float64"))


def exact_d2(q: np.ndarray, x: np.ndarray) -> np.float32:
    d = q.shape[0]
    assert d % 4 == 0 and x.shape[0] == d
    return np.float32(lib().trim_oracle_exact_d2(_p(q, f32), _p(x, f32), C.c_int(d)))


def plb_from_s(s: float, b: float, gamma: float) -> np.float32:
    return np.float32(lib().trim_oracle_plb_from_s(float(s), float(b), float(gamma)))


def encode(base: np.ndarray, codebooks: np.ndarray):
    n, d = base.shape
    M = codebooks.shape[0]
    assert codebooks.shape == (M, 256, d // M) and d % M == 0
    codes = np.empty((n, M), dtype=np.uint8)
    dlx = np.empty(n, dtype=np.float32)
    lib().trim_oracle_encode(_p(base, f32), C.c_int64(n), C.c_int(d), _p(codebooks, f32),
                             C.c_int(M), _p(codes, u8), _p(dlx, f32))
    return codes, dlx


def build_lut(queries: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    nq, d = queries.shape
    M = codebooks.shape[0]
    assert codebooks.shape == (M, 256, d // M) and d % M == 0
    lut = np.empty((nq, M, 256), dtype=np.float32)
    lib().trim_oracle_build_lut(_p(queries, f32), C.c_int64(nq), C.c_int(d),
                                _p(codebooks, f32), C.c_int(M), _p(lut, f32))
    return lut


class Index:
    """The stored data of Section 3.3's preprocessing phase, as plain arrays."""

    def __init__(self, base, codes, dlx, codebooks, ids=None, list_offsets=None,
                 centroids=None):
        self.base, self.codes, self.dlx, self.codebooks = base, codes, dlx, codebooks
        self.ids, self.list_offsets, self.centroids = ids, list_offsets, centroids
        self.n, self.d = base.shape
        self.M = codebooks.shape[0]
        assert d_ok(self.d, self.M)
        assert codes.shape == (self.n, self.M) and dlx.shape == (self.n,)


def d_ok(d, M):
    return d % 4 == 0 and d % M == 0


def _cand_args(ix: Index, probes):
    if probes is None:
        return C.c_int(0), None, None
    assert ix.list_offsets is not None and probes.ndim == 2
    return C.c_int(probes.shape[1]), _p(ix.list_offsets, i64), _p(probes, i32)


def max_candidates(ix: Index, probes) -> int:
    if probes is None:
        return ix.n
    lens = np.diff(ix.list_offsets)
    return int(lens[probes].sum(axis=1).max()) if probes.size else 0


def search_knn(ix: Index, queries, k, gamma, batch, probes=None, lut=None, want_mask=False):
    assert batch >= 1
    nq = queries.shape[0]
    out_ids = np.empty((nq, k), dtype=np.int32)
    out_d2 = np.empty((nq, k), dtype=np.float32)
    n_scanned = np.empty(nq, dtype=np.int32)
    n_exact = np.empty(nq, dtype=np.int32)
    mw = (max_candidates(ix, probes) + 31) // 32
    mask = np.zeros((nq, mw), dtype=np.uint32) if want_mask else None
    npb, lo, pr = _cand_args(ix, probes)
    lib().trim_oracle_search_knn(
        _p(ix.base, f32), _p(ix.codes, u8), _p(ix.dlx, f32), _p(ix.ids, i32),
        _p(ix.codebooks, f32), C.c_int64(ix.n), C.c_int(ix.d), C.c_int(ix.M),
        _p(queries, f32), C.c_int64(nq), _p(lut, f32), npb, lo, pr, C.c_int(k),
        C.c_float(gamma), C.c_int(batch), _p(out_ids, i32), _p(out_d2, f32),
        _p(n_scanned, i32), _p(n_exact, i32), _p(mask, u32), C.c_int64(mw))
    return dict(ids=out_ids, d2=out_d2, n_scanned=n_scanned, n_exact=n_exact, mask=mask)


def search_range(ix: Index, queries, radius, gamma, probes=None, lut=None, want_mask=False):
    """radius is an unsquared distance (Section 2.1); it is squared once in binary32."""
    nq = queries.shape[0]
    radius2 = np.float32(radius) * np.float32(radius)
    counts = np.zeros(nq, dtype=np.int64)
    n_scanned = np.empty(nq, dtype=np.int32)
    n_exact = np.empty(nq, dtype=np.int32)
    mw = (max_candidates(ix, probes) + 31) // 32
    mask = np.zeros((nq, mw), dtype=np.uint32) if want_mask else None
    npb, lo, pr = _cand_args(ix, probes)

    def call(offsets, oi, od, m):
        lib().trim_oracle_search_range(
            _p(ix.base, f32), _p(ix.codes, u8), _p(ix.dlx, f32), _p(ix.ids, i32),
            _p(ix.codebooks, f32), C.c_int64(ix.n), C.c_int(ix.d), C.c_int(ix.M),
            _p(queries, f32), C.c_int64(nq), _p(lut, f32), npb, lo, pr,
            C.c_float(radius2), C.c_float(gamma), _p(counts, i64), _p(offsets, i64),
            _p(oi, i32), _p(od, f32), _p(n_scanned, i32), _p(n_exact, i32), _p(m, u32),
            C.c_int64(mw))

    call(None, None, None, None)
    offsets = np.zeros(nq + 1, dtype=np.int64)
    np.cumsum(counts, out=offsets[1:])
    out_ids = np.empty(int(offsets[-1]), dtype=np.int32)
    out_d2 = np.empty(int(offsets[-1]), dtype=np.float32)
    call(offsets, out_ids, out_d2, mask)
    return dict(offsets=offsets, ids=out_ids, d2=out_d2, n_scanned=n_scanned,
                n_exact=n_exact, mask=mask)


def brute_knn(ix: Index, queries, k, probes=None):
    nq = queries.shape[0]
    out_ids = np.empty((nq, k), dtype=np.int32)
    out_d2 = np.empty((nq, k), dtype=np.float32)
    npb, lo, pr = _cand_args(ix, probes)
    lib().trim_oracle_brute_knn(_p(ix.base, f32), _p(ix.ids, i32), C.c_int64(ix.n),
                                C.c_int(ix.d), _p(queries, f32), C.c_int64(nq), npb, lo, pr,
                                C.c_int(k), _p(out_ids, i32), _p(out_d2, f32))
    return out_ids, out_d2


def brute_knn_f64(base, queries, k, ids=None):
    nq = queries.shape[0]
    n, d = base.shape
    out_ids = np.empty((nq, k), dtype=np.int32)
    out_d2 = np.empty((nq, k), dtype=np.float64)
    lib().trim_oracle_brute_knn_f64(_p(base, f32), _p(ids, i32), C.c_int64(n), C.c_int(d),
                                    _p(queries, f32), C.c_int64(nq), C.c_int(k),
                                    _p(out_ids, i32), _p(out_d2, f64))
    return out_ids, out_d2


def exact_pairs(base, queries, qrow, pos):
    out = np.empty(qrow.shape[0], dtype=np.float32)
    lib().trim_oracle_exact_pairs(_p(base, f32), C.c_int(base.shape[1]), _p(queries, f32),
                                  _p(qrow, i64), _p(pos, i64), C.c_int64(qrow.shape[0]),
                                  _p(out, f32))
    return out


def plb_pairs(lut, codes, dlx, qrow, pos, gamma):
    M = codes.shape[1]
    s = np.empty(qrow.shape[0], dtype=np.float32)
    g = np.empty(qrow.shape[0], dtype=np.float32)
    lib().trim_oracle_plb_pairs(_p(lut, f32), C.c_int(M), _p(codes, u8), _p(dlx, f32),
                                _p(qrow, i64), _p(pos, i64), C.c_int64(qrow.shape[0]),
                                C.c_float(gamma), _p(s, f32), _p(g, f32))
    return s, g


def ivf_probe(queries, centroids, nprobe):
    nq, d = queries.shape
    nlist = centroids.shape[0]
    probes = np.empty((nq, nprobe), dtype=np.int32)
    lib().trim_oracle_ivf_probe(_p(queries, f32), C.c_int64(nq), C.c_int(d),
                                _p(centroids, f32), C.c_int(nlist), C.c_int(nprobe),
                                _p(probes, i32))
    return probes


def num_threads() -> int:
    return int(lib().trim_oracle_num_threads())
