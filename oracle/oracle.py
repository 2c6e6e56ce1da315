"""ctypes front end of the fp64 CPU oracle (oracle/sa_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product package.  It neither
imports nor is imported by the HIP path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from .build import LIB, build_oracle

_lib = None

TRIANGULAR, INTERVAL_SLASH, BLOCK_CLUSTER = 0, 1, 2


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build_oracle()
        _lib = C.CDLL(LIB)
        _lib.oracle_triangular_count.restype = C.c_int64
        _lib.oracle_mask_count.restype = C.c_int64
    return _lib


def _p(a, t):
    return None if a is None else a.ctypes.data_as(C.POINTER(t))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16
    return a


@dataclass
class Budgets:
    sink_blocks: int
    local_blocks: int
    k_vertical: int
    k_slash: int
    k_blocks: int
    probe_v: int = 4
    probe_s: int = 4
    lift_num: int = 4
    lift_den: int = 1
    block_select: int = 0   # 0: one global top-k over the block map, 1: the same fraction of every row,
                            # 2: global top-k on the row-normalised key blk[R][C] * (R + 1)
    diagonal_select: int = 0  # 0: element-exact diagonals, 1: every selected diagonal widened to blocks


@dataclass
class Index:
    pattern: np.ndarray
    n_cols: np.ndarray
    cols: np.ndarray
    n_offs: np.ndarray
    offs: np.ndarray
    rowptr: np.ndarray
    blkcols: np.ndarray

    def arrays(self):
        return [self.pattern, self.n_cols, self.cols, self.n_offs, self.offs, self.rowptr,
                self.blkcols]


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def default_scale(d):
    return 1.0 / float(np.sqrt(float(d)))


def dense_rows(Q, K, V, scale=None, rows=None):
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    Hq, N, d = Q.shape
    Hkv = K.shape[0]
    scale = default_scale(d) if scale is None else scale
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        nrows = rows.size
    else:
        nrows = N
    O = np.empty((Hq, nrows, d), np.float64)
    ws = np.empty((Hq, nrows), np.float64)
    rc = lib().oracle_dense_rows(_p(Q, C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16),
                                 Hq, Hkv, N, d, C.c_double(scale), _p(rows, C.c_int32), nrows,
                                 _p(O, C.c_double), _p(ws, C.c_double))
    assert rc == 0
    return O, ws


def dense_weights(Q, K, h, scale=None):
    Q, K = _u16(Q), _u16(K)
    Hq, N, d = Q.shape
    scale = default_scale(d) if scale is None else scale
    A = np.empty((N, N), np.float64)
    rc = lib().oracle_dense_weights(_p(Q, C.c_uint16), _p(K, C.c_uint16), Hq, K.shape[0], N, d,
                                    C.c_double(scale), h, _p(A, C.c_double))
    assert rc == 0
    return A


def window_weights(Q, K, w, scale=None):
    Q, K = _u16(Q), _u16(K)
    Hq, N, d = Q.shape
    scale = default_scale(d) if scale is None else scale
    A = np.empty((Hq, w, N), np.float64)
    rc = lib().oracle_window_weights(_p(Q, C.c_uint16), _p(K, C.c_uint16), Hq, K.shape[0], N, d,
                                     w, C.c_double(scale), _p(A, C.c_double))
    assert rc == 0
    return A


def estimate(Q, K, b, w, scale=None):
    Q, K = _u16(Q), _u16(K)
    Hq, N, d = Q.shape
    scale = default_scale(d) if scale is None else scale
    nb = N // b
    v = np.empty((Hq, N), np.float64)
    s = np.empty((Hq, N), np.float64)
    blk = np.empty((Hq, nb, nb), np.float64)
    rc = lib().oracle_estimate(_p(Q, C.c_uint16), _p(K, C.c_uint16), Hq, K.shape[0], N, d, b, w,
                               C.c_double(scale), _p(v, C.c_double), _p(s, C.c_double),
                               _p(blk, C.c_double))
    assert rc == 0
    return v, s, blk


def triangular_count(nb, sink_blocks, local_blocks):
    return int(lib().oracle_triangular_count(nb, sink_blocks, local_blocks))


def default_budgets(N, b, rho) -> Budgets:
    out = (C.c_int32 * 5)()
    rc = lib().oracle_default_budgets(N, b, C.c_double(rho), out)
    assert rc == 0
    return Budgets(*[int(x) for x in out])


def block_capacity(N, b, bud: Budgets):
    # the per-row rule rounds every row's share up: at most one block per row above k_blocks
    nb = N // b
    kb = bud.k_blocks + (nb if bud.block_select == 1 else 0)
    cap = max(kb, triangular_count(nb, bud.sink_blocks, bud.local_blocks))
    if bud.diagonal_select == 1:
        # a diagonal touches at most two key blocks per row block
        cap = max(cap, sum(min(R + 1, 2 * min(bud.k_slash, N) + 1) for R in range(nb)))
    return cap


def build_index(v, s, blk, N, b, w, bud: Budgets, override=None) -> Index:
    v = np.ascontiguousarray(v, np.float32)
    s = np.ascontiguousarray(s, np.float32)
    blk = np.ascontiguousarray(blk, np.float32)
    Hq = v.shape[0]
    nb = N // b
    cap = block_capacity(N, b, bud)
    if override is not None:
        override = np.ascontiguousarray(override, np.int32)
    idx = Index(np.empty(Hq, np.int32), np.empty(Hq, np.int32),
                np.empty((Hq, bud.k_vertical), np.int32), np.empty(Hq, np.int32),
                np.empty((Hq, bud.k_slash), np.int32), np.empty((Hq, nb + 1), np.int32),
                np.empty((Hq, cap), np.int32))
    i32 = C.c_int32
    rc = lib().oracle_build_index(_p(v, C.c_float), _p(s, C.c_float), _p(blk, C.c_float), Hq, N,
                                  b, w, bud.sink_blocks, bud.local_blocks, bud.k_vertical,
                                  bud.k_slash, bud.k_blocks, bud.probe_v, bud.probe_s,
                                  bud.lift_num, bud.lift_den, _p(override, i32), cap,
                                  _p(idx.pattern, i32), _p(idx.n_cols, i32), _p(idx.cols, i32),
                                  _p(idx.n_offs, i32), _p(idx.offs, i32), _p(idx.rowptr, i32),
                                  _p(idx.blkcols, i32), bud.block_select, bud.diagonal_select)
    assert rc == 0
    return idx


def choose_pattern(v, s, N, b, w, bud: Budgets) -> int:
    v = np.ascontiguousarray(v, np.float32)
    s = np.ascontiguousarray(s, np.float32)
    return int(lib().oracle_choose_pattern(_p(v, C.c_float), _p(s, C.c_float), N, b, w,
                                           bud.sink_blocks, bud.local_blocks, bud.probe_v,
                                           bud.probe_s, bud.lift_num, bud.lift_den))


def _idx_args(idx: Index):
    i32 = C.c_int32
    a = [np.ascontiguousarray(x, np.int32) for x in idx.arrays()]
    return a, [_p(a[1], i32), _p(a[2], i32), _p(a[3], i32), _p(a[4], i32), _p(a[5], i32),
               _p(a[6], i32)]


def masked_rows(Q, K, V, b, idx: Index, rows=None, scale=None):
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    Hq, N, d = Q.shape
    scale = default_scale(d) if scale is None else scale
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        nrows = rows.size
    else:
        nrows = N
    O = np.empty((Hq, nrows, d), np.float64)
    ws = np.empty((Hq, nrows), np.float64)
    kept = np.empty((Hq, nrows), np.int64)
    keep_alive, ptrs = _idx_args(idx)
    rc = lib().oracle_masked_rows(_p(Q, C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16), Hq,
                                  K.shape[0], N, d, b, C.c_double(scale), idx.cols.shape[1],
                                  idx.offs.shape[1], idx.blkcols.shape[1], *ptrs,
                                  _p(rows, C.c_int32), nrows, _p(O, C.c_double),
                                  _p(ws, C.c_double), _p(kept, C.c_int64))
    assert rc == 0
    return O, ws, kept


def mask_count(N, b, h, idx: Index) -> int:
    keep_alive, ptrs = _idx_args(idx)
    return int(lib().oracle_mask_count(N, b, h, idx.cols.shape[1], idx.offs.shape[1],
                                       idx.blkcols.shape[1], *ptrs))
