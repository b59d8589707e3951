"""Python face of the CPU oracle (oracle/swarm_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's CPU-baseline
leg.  Nothing in the product path imports this package, and this package imports nothing from
the HIP path.  All arrays are host numpy arrays; bf16 travels as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        L = C.CDLL(_build.LIB)
        L.oracle_score.restype = C.c_int
        L.oracle_select.restype = C.c_int
        L.oracle_trace.restype = C.c_int
        L.oracle_coact_dense.restype = C.c_int
        L.oracle_coact_update.restype = C.c_int
        L.oracle_coact_rows.restype = C.c_int
        L.oracle_map.restype = C.c_int
        L.oracle_density.restype = C.c_int
        L.oracle_score_rows.restype = C.c_int
        L.oracle_expand_clusters.restype = C.c_int
        L.oracle_submission_order.restype = C.c_int
        L.oracle_window_assign.restype = C.c_int
        L.oracle_hardware_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def hardware_threads() -> int:
    return int(lib().oracle_hardware_threads())


class OracleError(RuntimeError):
    def __init__(self, fn, code):
        super().__init__(f"{fn} returned {code}")
        self.code = code


def score(kind: str, keys: np.ndarray, q: np.ndarray, G: int = 1, nthreads: int = 1):
    """keys: uint16 [H][N][d] (kind 'token') or [H][N][2][d] (kind 'page'); q: uint16 [B][H*G][d].
    Returns (scores float32 [B][H][N], scores float64, abs-term sums float64)."""
    keys = _c(keys, np.uint16)
    q = _c(q, np.uint16)
    H, N, d = keys.shape[0], keys.shape[1], keys.shape[-1]
    B = q.shape[0]
    assert q.shape == (B, H * G, d), (q.shape, (B, H * G, d))
    assert keys.shape == ((H, N, d) if kind == "token" else (H, N, 2, d))
    f32 = np.empty((B, H, N), np.float32)
    f64 = np.empty((B, H, N), np.float64)
    ab = np.empty((B, H, N), np.float64)
    rc = lib().oracle_score(C.c_int(0 if kind == "token" else 1), _p(keys), _p(q), B, H, G, N, d,
                            _p(f32), _p(f64), _p(ab), nthreads)
    if rc:
        raise OracleError("oracle_score", rc)
    return f32, f64, ab


def select(scores: np.ndarray, k: int, nthreads: int = 1) -> np.ndarray:
    """scores float32 [..., N] -> int32 [..., k], ascending index."""
    scores = _c(scores, np.float32)
    N = scores.shape[-1]
    rows = scores.size // N
    idx = np.empty(scores.shape[:-1] + (k,), np.int32)
    rc = lib().oracle_select(_p(scores), C.c_int64(rows), N, k, _p(idx), nthreads)
    if rc:
        raise OracleError("oracle_select", rc)
    return idx


def trace(idx: np.ndarray, N: int) -> np.ndarray:
    """idx int32 [rows][H][k] -> A uint8 [H][rows][N]."""
    idx = _c(idx, np.int32)
    rows, H, k = idx.shape
    A = np.empty((H, rows, N), np.uint8)
    rc = lib().oracle_trace(_p(idx), C.c_int64(rows), H, k, N, _p(A))
    if rc:
        raise OracleError("oracle_trace", rc)
    return A


def coact_dense(A: np.ndarray) -> np.ndarray:
    """A uint8 [rows][N] -> C int32 [N][N] by the triple-loop definition."""
    A = _c(A, np.uint8)
    rows, N = A.shape
    Cm = np.empty((N, N), np.int32)
    rc = lib().oracle_coact_dense(_p(A), C.c_int64(rows), N, _p(Cm))
    if rc:
        raise OracleError("oracle_coact_dense", rc)
    return Cm


def coact_update(idx: np.ndarray, N: int, Cm: np.ndarray | None = None, decay_q16: int = 65536,
                 nthreads: int = 1) -> np.ndarray:
    """One window: C <- decay(C) + counts(idx).  idx int32 [rows][H][k]; C int32 [H][N][N]
    (updated in place when given, else starts from zero)."""
    idx = _c(idx, np.int32)
    rows, H, k = idx.shape
    if Cm is None:
        Cm = np.zeros((H, N, N), np.int32)
    assert Cm.dtype == np.int32 and Cm.shape == (H, N, N) and Cm.flags.c_contiguous
    rc = lib().oracle_coact_update(_p(idx), C.c_int64(rows), H, k, N, _p(Cm), C.c_uint32(decay_q16), nthreads)
    if rc:
        raise OracleError("oracle_coact_update", rc)
    return Cm


def coact_rows(idx: np.ndarray, N: int, h: int, r0: int, r1: int, nthreads: int = 1) -> np.ndarray:
    """Rows [r0, r1) of head h's co-activation counts, from zero: idx int32 [rows][H][k] -> int32 [r1-r0][N]."""
    idx = _c(idx, np.int32)
    rows, H, k = idx.shape
    out = np.empty((r1 - r0, N), np.int32)
    rc = lib().oracle_coact_rows(_p(idx), C.c_int64(rows), H, k, N, h, r0, r1, _p(out), nthreads)
    if rc:
        raise OracleError("oracle_coact_rows", rc)
    return out


def density(Cm: np.ndarray, tau: float, flags: int = 0, totals: np.ndarray | None = None, nthreads: int = 1):
    """C int32 [H][N][N] -> (rho int32 [H][N], queue int32 [H][N], totals int64 [H]).
    flags bit 0: leave out j = i; bit 1: strict "<"."""
    Cm = _c(Cm, np.int32)
    H, N, N2 = Cm.shape
    assert N == N2
    rho = np.empty((H, N), np.int32)
    queue = np.empty((H, N), np.int32)
    tot = np.empty(H, np.int64)
    tin = None
    if totals is not None:
        tin = _c(totals, np.int64)
        assert tin.shape == (H,)
    rc = lib().oracle_density(_p(Cm), H, N, _p(tin) if tin is not None else None, C.c_double(tau), C.c_uint32(flags),
                              _p(rho), _p(queue), _p(tot), nthreads)
    if rc:
        raise OracleError("oracle_density", rc)
    return rho, queue, tot


def window_assign(sel: np.ndarray, N: int, new_ids: np.ndarray, medoids: np.ndarray, tau: float,
                  primary: np.ndarray | None = None, size: np.ndarray | None = None, D: int = 0):
    """sel int32 [W][H][k]; new_ids int32 [H][n_new]; medoids int32 [H][Nc]; primary/size int32 [H][Nc] or None.
    Returns (f int32 [H][n_new][Nc], member uint8 [H][n_new][Nc], disk int32 [H][n_new][Nc] or None)."""
    sel = _c(sel, np.int32)
    W, H, k = sel.shape
    new_ids = _c(new_ids, np.int32)
    medoids = _c(medoids, np.int32)
    n_new, Nc = new_ids.shape[1], medoids.shape[1]
    assert new_ids.shape == (H, n_new) and medoids.shape == (H, Nc)
    f = np.empty((H, n_new, Nc), np.int32)
    member = np.empty((H, n_new, Nc), np.uint8)
    disk = None
    if primary is not None:
        primary, size = _c(primary, np.int32), _c(size, np.int32)
        assert primary.shape == (H, Nc) and size.shape == (H, Nc) and D >= 1
        disk = np.empty((H, n_new, Nc), np.int32)
    rc = lib().oracle_window_assign(_p(sel), W, H, k, N, _p(new_ids), n_new, _p(medoids), Nc, C.c_double(tau),
                                    _p(primary), _p(size), D, _p(f), _p(member), _p(disk))
    if rc:
        raise OracleError("oracle_window_assign", rc)
    return f, member, disk


def score_rows(kind: str, keys: np.ndarray, row_ids: np.ndarray, q: np.ndarray, G: int = 1):
    """Scores of the listed entries only: row_ids int32 [H][M] -> (f32, f64, abs) each [B][H][M]."""
    keys = _c(keys, np.uint16)
    q = _c(q, np.uint16)
    row_ids = _c(row_ids, np.int32)
    H, N, d = keys.shape[0], keys.shape[1], keys.shape[-1]
    M = row_ids.shape[1]
    B = q.shape[0]
    assert row_ids.shape == (H, M) and q.shape == (B, H * G, d)
    f32 = np.empty((B, H, M), np.float32)
    f64 = np.empty((B, H, M), np.float64)
    ab = np.empty((B, H, M), np.float64)
    rc = lib().oracle_score_rows(0 if kind == "token" else 1, _p(keys), _p(row_ids), M, _p(q), B, H, G, N, d, _p(f32), _p(f64), _p(ab))
    if rc:
        raise OracleError("oracle_score_rows", rc)
    return f32, f64, ab


def expand_clusters(clusters: np.ndarray, H: int, Nc: int, cl_off: np.ndarray, cl_entries: np.ndarray, cap_e: int):
    """clusters int32 [groups][Sc] (-1 padding); cl_off int32 [H][Nc+1]; cl_entries int32 [H][E] ->
    (entries int32 [groups][cap_e] (-1 padded), count int32 [groups])."""
    clusters = _c(clusters, np.int32)
    cl_off, cl_entries = _c(cl_off, np.int32), _c(cl_entries, np.int32)
    groups, Sc = clusters.shape
    E = cl_entries.shape[1]
    assert cl_off.shape == (H, Nc + 1) and cl_entries.shape == (H, E)
    entries = np.empty((groups, cap_e), np.int32)
    count = np.empty(groups, np.int32)
    rc = lib().oracle_expand_clusters(_p(clusters), C.c_int64(groups), Sc, H, Nc, _p(cl_off), _p(cl_entries), E, _p(entries),
                                      _p(count), cap_e)
    if rc:
        raise OracleError("oracle_expand_clusters", rc)
    return entries, count


def submission_order(q_off: np.ndarray, q_cluster: np.ndarray):
    """q_off int32 [groups][D+1], q_cluster int32 [groups][cap] -> (order [groups][cap], batch_off [groups][cap+1], nb [groups])."""
    q_off, q_cluster = _c(q_off, np.int32), _c(q_cluster, np.int32)
    groups, D1 = q_off.shape
    cap = q_cluster.shape[1]
    order = np.empty((groups, cap), np.int32)
    batch_off = np.empty((groups, cap + 1), np.int32)
    nb = np.empty(groups, np.int32)
    rc = lib().oracle_submission_order(_p(q_off), _p(q_cluster), C.c_int64(groups), D1 - 1, cap, _p(order), _p(batch_off), _p(nb))
    if rc:
        raise OracleError("oracle_submission_order", rc)
    return order, batch_off, nb


def map_requests(sel: np.ndarray, H: int, N: int, e2c: np.ndarray, Nc: int, replicas: np.ndarray, D: int,
                 weight: np.ndarray | None = None, resident: np.ndarray | None = None, cap: int | None = None,
                 nthreads: int = 1):
    """sel int32 [groups][S]; e2c int32 [H][N]; replicas int32 [H*Nc][R]; weight int32 [H*Nc] or None;
    resident uint32 bitmap [ceil(H*Nc/32)] or None.
    Returns (q_off [groups][D+1], q_cluster [groups][cap], q_load [groups][D])."""
    sel = _c(sel, np.int32)
    groups, S = sel.shape
    e2c = _c(e2c, np.int32)
    replicas = _c(replicas, np.int32)
    R = replicas.shape[1]
    assert e2c.shape == (H, N) and replicas.shape == (H * Nc, R)
    if weight is not None:
        weight = _c(weight, np.int32)
        assert weight.shape == (H * Nc,)
    if resident is not None:
        resident = _c(resident, np.uint32)
        assert resident.size >= (H * Nc + 31) // 32
    if cap is None:
        cap = min(S, Nc)
    q_off = np.empty((groups, D + 1), np.int32)
    q_cluster = np.empty((groups, cap), np.int32)
    q_load = np.empty((groups, D), np.int32)
    rc = lib().oracle_map(_p(sel), C.c_int64(groups), S, H, N, _p(e2c), Nc, _p(replicas), R, D, _p(weight),
                          _p(resident), _p(q_off), _p(q_cluster), _p(q_load), cap, nthreads)
    if rc:
        raise OracleError("oracle_map", rc)
    return q_off, q_cluster, q_load
