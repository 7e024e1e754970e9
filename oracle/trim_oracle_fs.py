"""ctypes face of oracle/trim_oracle_fs.c: the scan over 4-bit landmark codes (test
infrastructure; see that file's header).  numpy arrays in and out; no arithmetic here."""
from __future__ import annotations

import ctypes as C

import numpy as np

from .trim_oracle import _cand_args, _p, f32, i32, i64, lib, max_candidates, u8, u32


class Index:
    """Stored data of Section 3.3's preprocessing with 4-bit codes: m subspaces of 16
    centroids; codes [n][m/2], subspace 2i in the low half of byte i."""

    def __init__(self, base, codes, dlx, codebooks, ids=None, list_offsets=None, centroids=None):
        self.base, self.codes, self.dlx, self.codebooks = base, codes, dlx, codebooks
        self.ids, self.list_offsets, self.centroids = ids, list_offsets, centroids
        self.n, self.d = base.shape
        self.m = codebooks.shape[0]
        assert codebooks.shape == (self.m, 16, self.d // self.m) and self.m % 2 == 0 and self.d % self.m == 0
        assert codes.shape == (self.n, self.m // 2) and dlx.shape == (self.n,)


def unpack(codes: np.ndarray, m: int) -> np.ndarray:
    """[n][m/2] packed bytes -> [n][m] codes (pure re-indexing: low half first)."""
    out = np.empty((codes.shape[0], m), dtype=np.uint8)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


def encode(base: np.ndarray, codebooks: np.ndarray):
    n, d = base.shape
    m = codebooks.shape[0]
    assert codebooks.shape == (m, 16, d // m) and m % 2 == 0
    codes = np.zeros((n, m // 2), dtype=np.uint8)
    dlx = np.empty(n, dtype=np.float32)
    lib().trim_oracle_fs_encode(_p(base, f32), C.c_int64(n), C.c_int(d), _p(codebooks, f32), C.c_int(m),
                                _p(codes, u8), _p(dlx, f32))
    return codes, dlx


def build_lut(queries: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    nq, d = queries.shape
    m = codebooks.shape[0]
    lut = np.empty((nq, m, 16), dtype=np.float32)
    lib().trim_oracle_fs_build_lut(_p(queries, f32), C.c_int64(nq), C.c_int(d), _p(codebooks, f32),
                                   C.c_int(m), _p(lut, f32))
    return lut


def table_sum(T: np.ndarray, code: np.ndarray) -> np.float32:
    f = lib().trim_oracle_fs_table_sum
    f.restype = C.c_float
    return np.float32(f(_p(T, f32), _p(code, u8), C.c_int(T.shape[0])))


def search_knn(ix: Index, queries, k, gamma, batch, probes=None, lut=None, want_mask=False):
    nq = queries.shape[0]
    out_ids = np.empty((nq, k), dtype=np.int32)
    out_d2 = np.empty((nq, k), dtype=np.float32)
    n_scanned = np.empty(nq, dtype=np.int32)
    n_exact = np.empty(nq, dtype=np.int32)
    mw = (max_candidates(ix, probes) + 31) // 32
    mask = np.zeros((nq, mw), dtype=np.uint32) if want_mask else None
    npb, lo, pr = _cand_args(ix, probes)
    lib().trim_oracle_fs_search_knn(
        _p(ix.base, f32), _p(ix.codes, u8), _p(ix.dlx, f32), _p(ix.ids, i32), _p(ix.codebooks, f32),
        C.c_int64(ix.n), C.c_int(ix.d), C.c_int(ix.m), _p(queries, f32), C.c_int64(nq), _p(lut, f32),
        npb, lo, pr, C.c_int(k), C.c_float(gamma), C.c_int(batch), _p(out_ids, i32), _p(out_d2, f32),
        _p(n_scanned, i32), _p(n_exact, i32), _p(mask, u32), C.c_int64(mw))
    return dict(ids=out_ids, d2=out_d2, n_scanned=n_scanned, n_exact=n_exact, mask=mask)


def search_range(ix: Index, queries, radius, gamma, probes=None, lut=None, want_mask=False):
    nq = queries.shape[0]
    radius2 = np.float32(radius) * np.float32(radius)
    counts = np.zeros(nq, dtype=np.int64)
    n_scanned = np.empty(nq, dtype=np.int32)
    n_exact = np.empty(nq, dtype=np.int32)
    mw = (max_candidates(ix, probes) + 31) // 32
    mask = np.zeros((nq, mw), dtype=np.uint32) if want_mask else None
    npb, lo, pr = _cand_args(ix, probes)

    def call(offsets, oi, od, m):
        lib().trim_oracle_fs_search_range(
            _p(ix.base, f32), _p(ix.codes, u8), _p(ix.dlx, f32), _p(ix.ids, i32), _p(ix.codebooks, f32),
            C.c_int64(ix.n), C.c_int(ix.d), C.c_int(ix.m), _p(queries, f32), C.c_int64(nq), _p(lut, f32),
            npb, lo, pr, C.c_float(radius2), C.c_float(gamma), _p(counts, i64), _p(offsets, i64),
            _p(oi, i32), _p(od, f32), _p(n_scanned, i32), _p(n_exact, i32), _p(m, u32), C.c_int64(mw))

    call(None, None, None, None)
    offsets = np.zeros(nq + 1, dtype=np.int64)
    np.cumsum(counts, out=offsets[1:])
    out_ids = np.empty(int(offsets[-1]), dtype=np.int32)
    out_d2 = np.empty(int(offsets[-1]), dtype=np.float32)
    call(offsets, out_ids, out_d2, mask)
    return dict(offsets=offsets, ids=out_ids, d2=out_d2, n_scanned=n_scanned, n_exact=n_exact, mask=mask)


def plb_pairs(lut, codes, dlx, qrow, pos, gamma):
    m = lut.shape[1]
    s = np.empty(qrow.shape[0], dtype=np.float32)
    g = np.empty(qrow.shape[0], dtype=np.float32)
    lib().trim_oracle_fs_plb_pairs(_p(lut, f32), C.c_int(m), _p(codes, u8), _p(dlx, f32), _p(qrow, i64),
                                   _p(pos, i64), C.c_int64(qrow.shape[0]), C.c_float(gamma), _p(s, f32),
                                   _p(g, f32))
    return s, g
