"""ctypes binding of libswarm (include/swarm.h).  Argument marshalling only.

Module-level functions carry the C names and take raw device pointers; the `Swarm` class wraps
them for torch tensors (torch supplies device memory and the stream, nothing else).  Every step
of the path runs inside the HIP library.  If the library cannot be loaded this module raises:
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

from . import build as _build

SWARM_OK, SWARM_EINVAL, SWARM_ENOMEM, SWARM_EHIP, SWARM_EOVERFLOW, SWARM_EDATA = 0, -1, -2, -3, -4, -5
SWARM_KEYS_TOKEN, SWARM_KEYS_PAGE_MINMAX = 0, 1
SWARM_CHECK_IDX = 1
SWARM_DEV_BAD_ENTRY, SWARM_DEV_BAD_CLUSTER, SWARM_DEV_BAD_SSD, SWARM_DEV_CAP, SWARM_DEV_DUP_ENTRY = 1, 2, 4, 8, 16
SWARM_DEV_BAD_OFFSETS, SWARM_DEV_OVERFLOW = 32, 64

EXPORTS = ["swarm_create", "swarm_destroy", "swarm_last_error", "swarm_source_hash", "swarm_device_status", "swarm_score", "swarm_score_select", "swarm_score_select_static",
           "swarm_coact_accumulate", "swarm_coact_build_density", "swarm_map_requests", "swarm_map_requests_streams", "swarm_coact_density", "swarm_window_assign", "swarm_score_select_indexed", "swarm_expand_clusters",
           "swarm_submission_order", "swarm_step", "swarm_calibrate", "swarm_capture_begin", "swarm_capture_end",
           "swarm_graph_launch", "swarm_graph_destroy"]


class swarm_keys(C.Structure):
    _fields_ = [("kind", C.c_int32), ("data", C.c_void_p), ("H", C.c_int32), ("N", C.c_int32), ("d", C.c_int32),
                ("G", C.c_int32)]


class SwarmError(RuntimeError):
    def __init__(self, fn: str, code: int, text: str = ""):
        super().__init__(f"{fn} -> {code}: {text}")
        self.code = code


_lib = None


def load() -> C.CDLL:
    """Loads the built library (building it first only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    L = C.CDLL(_build.LIB)
    vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
    L.swarm_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    L.swarm_destroy.argtypes = [vp]
    L.swarm_last_error.argtypes = [vp]
    L.swarm_last_error.restype = C.c_char_p
    L.swarm_source_hash.argtypes = []
    L.swarm_source_hash.restype = C.c_char_p
    L.swarm_device_status.argtypes = [vp, C.POINTER(u32)]
    L.swarm_score_select.argtypes = [vp, C.POINTER(swarm_keys), vp, i32, i32, vp, vp]
    L.swarm_score_select_static.argtypes = [vp, C.POINTER(swarm_keys), vp, i32, i32, vp]
    L.swarm_score.argtypes = [vp, C.POINTER(swarm_keys), vp, i32, vp]
    L.swarm_coact_accumulate.argtypes = [vp, vp, i64, i32, i32, i32, vp, u32, u32]
    L.swarm_map_requests.argtypes = [vp, vp, i64, i32, i32, i32, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, i32]
    L.swarm_map_requests_streams.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, i32]
    L.swarm_step.argtypes = [vp, vp, vp, i32, vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, i32]
    L.swarm_coact_build_density.argtypes = [vp, vp, i64, i32, i32, i32, vp, u32, C.c_double, u32, vp, vp, vp]
    L.swarm_coact_density.argtypes = [vp, vp, i32, i32, vp, C.c_double, C.c_uint32, vp, vp, vp]
    L.swarm_window_assign.argtypes = [vp, vp, i32, i32, i32, i32, vp, i32, vp, i32, C.c_double, vp, vp, i32, vp, vp, vp]
    L.swarm_score_select_indexed.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp]
    L.swarm_expand_clusters.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, i32, vp, vp, i32]
    L.swarm_submission_order.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp, vp]
    L.swarm_calibrate.argtypes = [vp, i32, vp, C.c_size_t, i32, C.POINTER(C.c_double)]
    L.swarm_capture_begin.argtypes = [vp]
    L.swarm_capture_end.argtypes = [vp, C.POINTER(vp)]
    L.swarm_graph_launch.argtypes = [vp, vp]
    L.swarm_graph_destroy.argtypes = [vp]
    for name in EXPORTS:
        if name not in ("swarm_last_error", "swarm_source_hash"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


# ---- raw layer: the C names, raw pointers ---------------------------------------------------

def swarm_create(device: int, hip_stream: int) -> int:
    ctx = C.c_void_p()
    rc = load().swarm_create(C.byref(ctx), device, C.c_void_p(hip_stream))
    if rc != SWARM_OK:
        raise SwarmError("swarm_create", rc, load().swarm_last_error(None).decode())
    return ctx.value


def swarm_destroy(ctx: int) -> None:
    load().swarm_destroy(C.c_void_p(ctx))


def swarm_last_error(ctx: int) -> str:
    return load().swarm_last_error(C.c_void_p(ctx)).decode()


def swarm_source_hash() -> str:
    return load().swarm_source_hash().decode()


def library_is_current() -> bool:
    """True when the loaded library was built from the sources now on disk (its compiled-in hash matches)."""
    return swarm_source_hash() == _build.source_hash()


def swarm_device_status(ctx: int) -> Tuple[int, int]:
    flags = C.c_uint32(0)
    rc = load().swarm_device_status(C.c_void_p(ctx), C.byref(flags))
    return rc, flags.value


def swarm_score_select(ctx: int, kind: int, data: int, H: int, N: int, d: int, G: int, q: int, B: int, k: int,
                       out_idx: int, out_scores: Optional[int]) -> int:
    ks = swarm_keys(kind, data, H, N, d, G)
    return load().swarm_score_select(C.c_void_p(ctx), C.byref(ks), C.c_void_p(q), B, k, C.c_void_p(out_idx),
                                     C.c_void_p(out_scores))


def swarm_score_select_static(ctx: int, kind: int, data: int, H: int, N: int, d: int, G: int, q: int, B: int, k: int,
                              out_idx: int) -> int:
    ks = swarm_keys(kind, data, H, N, d, G)
    return load().swarm_score_select_static(C.c_void_p(ctx), C.byref(ks), C.c_void_p(q), B, k, C.c_void_p(out_idx))


def swarm_score(ctx: int, kind: int, data: int, H: int, N: int, d: int, G: int, q: int, B: int, out_scores: int) -> int:
    ks = swarm_keys(kind, data, H, N, d, G)
    return load().swarm_score(C.c_void_p(ctx), C.byref(ks), C.c_void_p(q), B, C.c_void_p(out_scores))


def swarm_step(ctx: int, kind: int, data: int, H: int, N: int, d: int, G: int, q: int, k: int, out_idx: int,
               out_scores: Optional[int], e2c: int, Nc: int, replicas: int, R: int, D: int, weight: Optional[int],
               resident: Optional[int], q_off: int, q_cluster: int, q_load: int, cap: int) -> int:
    ks = swarm_keys(kind, data, H, N, d, G)
    return load().swarm_step(C.c_void_p(ctx), C.byref(ks), C.c_void_p(q), k, C.c_void_p(out_idx), C.c_void_p(out_scores),
                             C.c_void_p(e2c), Nc, C.c_void_p(replicas), R, D, C.c_void_p(weight), C.c_void_p(resident),
                             C.c_void_p(q_off), C.c_void_p(q_cluster), C.c_void_p(q_load), cap)


SWARM_CAL_HBM_READ, SWARM_CAL_HBM_WRITE, SWARM_CAL_MFMA_I8, SWARM_CAL_MFMA_FP4 = 0, 1, 2, 3
SWARM_RHO_EXCLUDE_SELF, SWARM_RHO_STRICT = 1, 2
SWARM_COACT_POPCOUNT = 2


def swarm_window_assign(ctx: int, sel: int, W: int, H: int, k: int, N: int, new_ids: int, n_new: int, medoids: int, Nc: int,
                        tau: float, primary: Optional[int], size: Optional[int], D: int, f_out: Optional[int], member: int,
                        disk: Optional[int]) -> int:
    return load().swarm_window_assign(C.c_void_p(ctx), C.c_void_p(sel), W, H, k, N, C.c_void_p(new_ids), n_new,
                                      C.c_void_p(medoids), Nc, tau, C.c_void_p(primary), C.c_void_p(size), D,
                                      C.c_void_p(f_out), C.c_void_p(member), C.c_void_p(disk))


def swarm_score_select_indexed(ctx: int, kind: int, data: int, H: int, N: int, d: int, G: int, row_ids: int, M: int, q: int, B: int,
                               k: int, out_idx: int, out_scores: Optional[int]) -> int:
    ks = swarm_keys(kind, data, H, N, d, G)
    return load().swarm_score_select_indexed(C.c_void_p(ctx), C.byref(ks), C.c_void_p(row_ids), M, C.c_void_p(q), B, k,
                                             C.c_void_p(out_idx), C.c_void_p(out_scores))


def swarm_expand_clusters(ctx: int, clusters: int, groups: int, Sc: int, H: int, Nc: int, cl_off: int, cl_entries: int, E: int,
                          entries: int, count: int, cap_e: int) -> int:
    return load().swarm_expand_clusters(C.c_void_p(ctx), C.c_void_p(clusters), groups, Sc, H, Nc, C.c_void_p(cl_off),
                                        C.c_void_p(cl_entries), E, C.c_void_p(entries), C.c_void_p(count), cap_e)


def swarm_submission_order(ctx: int, q_off: int, q_cluster: int, groups: int, D: int, cap: int, order: int, batch_off: int,
                           nb: int) -> int:
    return load().swarm_submission_order(C.c_void_p(ctx), C.c_void_p(q_off), C.c_void_p(q_cluster), groups, D, cap,
                                         C.c_void_p(order), C.c_void_p(batch_off), C.c_void_p(nb))


def swarm_coact_density(ctx: int, Cptr: int, H: int, N: int, totals_in: Optional[int], tau: float, flags: int, rho: int,
                        queue: Optional[int], totals_out: Optional[int]) -> int:
    return load().swarm_coact_density(C.c_void_p(ctx), C.c_void_p(Cptr), H, N, C.c_void_p(totals_in), tau, flags,
                                      C.c_void_p(rho), C.c_void_p(queue), C.c_void_p(totals_out))


def swarm_calibrate(ctx: int, what: int, buf: int, nbytes: int, reps: int):
    out = C.c_double(0.0)
    rc = load().swarm_calibrate(C.c_void_p(ctx), what, C.c_void_p(buf), nbytes, reps, C.byref(out))
    return rc, out.value


def swarm_coact_accumulate(ctx: int, idx: int, rows: int, H: int, k: int, N: int, Cptr: int, decay_q16: int,
                           flags: int) -> int:
    return load().swarm_coact_accumulate(C.c_void_p(ctx), C.c_void_p(idx), rows, H, k, N, C.c_void_p(Cptr),
                                         decay_q16, flags)


def swarm_coact_build_density(ctx: int, idx: int, rows: int, H: int, k: int, N: int, Cptr: int, flags: int, tau: float,
                              rho_flags: int, rho: int, queue: Optional[int], totals_out: Optional[int]) -> int:
    return load().swarm_coact_build_density(C.c_void_p(ctx), C.c_void_p(idx), rows, H, k, N, C.c_void_p(Cptr), flags, tau,
                                            rho_flags, C.c_void_p(rho), C.c_void_p(queue), C.c_void_p(totals_out))


def swarm_map_requests(ctx: int, sel: int, groups: int, S: int, H: int, N: int, e2c: int, Nc: int, replicas: int,
                       R: int, D: int, weight: Optional[int], resident: Optional[int], q_off: int, q_cluster: int,
                       q_load: int, cap: int) -> int:
    return load().swarm_map_requests(C.c_void_p(ctx), C.c_void_p(sel), groups, S, H, N, C.c_void_p(e2c), Nc,
                                     C.c_void_p(replicas), R, D, C.c_void_p(weight), C.c_void_p(resident),
                                     C.c_void_p(q_off), C.c_void_p(q_cluster), C.c_void_p(q_load), cap)


def swarm_map_requests_streams(ctx: int, idx: int, steps: int, B: int, H: int, k: int, N: int, e2c: int, Nc: int, replicas: int,
                               R: int, D: int, weight: Optional[int], resident: Optional[int], q_off: int, q_cluster: int,
                               q_load: int, cap: int) -> int:
    return load().swarm_map_requests_streams(C.c_void_p(ctx), C.c_void_p(idx), steps, B, H, k, N, C.c_void_p(e2c), Nc,
                                             C.c_void_p(replicas), R, D, C.c_void_p(weight), C.c_void_p(resident),
                                             C.c_void_p(q_off), C.c_void_p(q_cluster), C.c_void_p(q_load), cap)


def swarm_capture_begin(ctx: int) -> int:
    return load().swarm_capture_begin(C.c_void_p(ctx))


def swarm_capture_end(ctx: int) -> Tuple[int, Optional[int]]:
    g = C.c_void_p()
    rc = load().swarm_capture_end(C.c_void_p(ctx), C.byref(g))
    return rc, g.value


def swarm_graph_launch(ctx: int, graph: int) -> int:
    return load().swarm_graph_launch(C.c_void_p(ctx), C.c_void_p(graph))


def swarm_graph_destroy(graph: int) -> int:
    return load().swarm_graph_destroy(C.c_void_p(graph))


# ---- tensor layer ---------------------------------------------------------------------------

class Swarm:
    """One library context on the current torch stream of `device`."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        self.torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2603_17803_amd needs an MI355X; no GPU is visible")
        self.device = torch.device("cuda", device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.ctx = swarm_create(device, self.stream.cuda_stream)

    def close(self):
        if getattr(self, "ctx", None):
            swarm_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, fn: str, rc: int):
        if rc != SWARM_OK:
            raise SwarmError(fn, rc, swarm_last_error(self.ctx))

    def _dev(self, t, dtype=None, name="tensor"):
        if t.device != self.device or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous tensor on {self.device}")
        if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
            raise ValueError(f"{name} has dtype {t.dtype}, expected {dtype}")
        return t.data_ptr()

    def score_select(self, kind: str, keys, q, k: int, G: int = 1, out_idx=None, out_scores=None,
                     want_scores: bool = False):
        """keys: bf16 (or int16 bit patterns) [H][N][d] ('token') or [H][N][2][d] ('page');
        q: [B][H*G][d].  Returns (idx int32 [B][H][k], scores fp32 [B][H][N] or None)."""
        torch = self.torch
        b16 = (torch.bfloat16, torch.int16, torch.uint16)
        H, N, d = keys.shape[0], keys.shape[1], keys.shape[-1]
        B = q.shape[0]
        if tuple(q.shape) != (B, H * G, d):
            raise ValueError(f"q has shape {tuple(q.shape)}, expected {(B, H * G, d)}")
        want = (H, N, d) if kind == "token" else (H, N, 2, d)
        if tuple(keys.shape) != want:
            raise ValueError(f"keys has shape {tuple(keys.shape)}, expected {want}")
        if out_idx is None:
            out_idx = torch.empty((B, H, k), dtype=torch.int32, device=self.device)
        if out_scores is None and want_scores:
            out_scores = torch.empty((B, H, N), dtype=torch.float32, device=self.device)
        rc = swarm_score_select(self.ctx, SWARM_KEYS_TOKEN if kind == "token" else SWARM_KEYS_PAGE_MINMAX,
                                self._dev(keys, b16, "keys"), H, N, d, G, self._dev(q, b16, "q"), B, k,
                                self._dev(out_idx, torch.int32, "out_idx"),
                                None if out_scores is None else self._dev(out_scores, torch.float32, "out_scores"))
        self._check("swarm_score_select", rc)
        return out_idx, out_scores

    def score(self, kind: str, keys, q, G: int = 1, out_scores=None):
        """Scores only: returns fp32 [B][H][N]."""
        torch = self.torch
        b16 = (torch.bfloat16, torch.int16, torch.uint16)
        H, N, d = keys.shape[0], keys.shape[1], keys.shape[-1]
        B = q.shape[0]
        if tuple(q.shape) != (B, H * G, d):
            raise ValueError(f"q has shape {tuple(q.shape)}, expected {(B, H * G, d)}")
        if out_scores is None:
            out_scores = torch.empty((B, H, N), dtype=torch.float32, device=self.device)
        rc = swarm_score(self.ctx, SWARM_KEYS_TOKEN if kind == "token" else SWARM_KEYS_PAGE_MINMAX,
                         self._dev(keys, b16, "keys"), H, N, d, G, self._dev(q, b16, "q"), B,
                         self._dev(out_scores, torch.float32, "out_scores"))
        self._check("swarm_score", rc)
        return out_scores

    def coact_accumulate(self, idx, N: int, Cm, decay_q16: int = 65536, flags: int = 0):
        """idx int32 [rows][H][k]; Cm int32 [H][N][N] updated in place."""
        torch = self.torch
        rows, H, k = idx.shape
        if tuple(Cm.shape) != (H, N, N):
            raise ValueError(f"C has shape {tuple(Cm.shape)}, expected {(H, N, N)}")
        rc = swarm_coact_accumulate(self.ctx, self._dev(idx, torch.int32, "idx"), rows, H, k, N,
                                    self._dev(Cm, torch.int32, "C"), decay_q16, flags)
        self._check("swarm_coact_accumulate", rc)
        return Cm

    def coact_build_density(self, idx, N: int, Cm, tau: float, flags: int = 0, rho_flags: int = 0, want_queue: bool = True,
                            out=None):
        """idx int32 [rows][H][k]; Cm int32 [H][N][N] overwritten with the counts -> (rho, queue or None, totals) as
        coact_density gives them for that Cm; `out` = (rho, queue or None, totals) reuses the caller's tensors."""
        torch = self.torch
        rows, H, k = idx.shape
        if tuple(Cm.shape) != (H, N, N):
            raise ValueError(f"C has shape {tuple(Cm.shape)}, expected {(H, N, N)}")
        if out is not None:
            rho, queue, totals = out
            if tuple(rho.shape) != (H, N) or (queue is not None and tuple(queue.shape) != (H, N)) or tuple(totals.shape) != (H,):
                raise ValueError("out must be (rho [H][N], queue [H][N] or None, totals [H])")
        else:
            rho = torch.empty((H, N), dtype=torch.int32, device=self.device)
            queue = torch.empty((H, N), dtype=torch.int32, device=self.device) if want_queue else None
            totals = torch.empty((H,), dtype=torch.int64, device=self.device)
        rc = swarm_coact_build_density(self.ctx, self._dev(idx, torch.int32, "idx"), rows, H, k, N, self._dev(Cm, torch.int32, "C"),
                                       flags, float(tau), rho_flags, self._dev(rho, torch.int32, "rho"),
                                       None if queue is None else self._dev(queue, torch.int32, "queue"),
                                       self._dev(totals, torch.int64, "totals"))
        self._check("swarm_coact_build_density", rc)
        return rho, queue, totals

    def coact_density(self, Cm, tau: float, flags: int = 0, totals_in=None, want_queue: bool = True, out=None):
        """Cm int32 [H][N][N] -> (rho int32 [H][N], queue int32 [H][N] or None, totals int64 [H]);
        `out` = (rho, queue or None, totals) reuses the caller's tensors (needed while recording)."""
        torch = self.torch
        H, N, N2 = Cm.shape
        if N != N2:
            raise ValueError("C must be [H][N][N]")
        if out is not None:
            rho, queue, totals = out
            if tuple(rho.shape) != (H, N) or (queue is not None and tuple(queue.shape) != (H, N)) or tuple(totals.shape) != (H,):
                raise ValueError("out must be (rho [H][N], queue [H][N] or None, totals [H])")
        else:
            rho = torch.empty((H, N), dtype=torch.int32, device=self.device)
            queue = torch.empty((H, N), dtype=torch.int32, device=self.device) if want_queue else None
            totals = torch.empty((H,), dtype=torch.int64, device=self.device)
        rc = swarm_coact_density(self.ctx, self._dev(Cm, torch.int32, "C"), H, N,
                                 None if totals_in is None else self._dev(totals_in, torch.int64, "totals_in"), float(tau),
                                 flags, self._dev(rho, torch.int32, "rho"),
                                 None if queue is None else self._dev(queue, torch.int32, "queue"),
                                 self._dev(totals, torch.int64, "totals"))
        self._check("swarm_coact_density", rc)
        return rho, queue, totals

    def window_assign(self, sel, N: int, new_ids, medoids, tau: float, primary=None, size=None, D: int = 0,
                      want_counts: bool = True):
        """sel int32 [W][H][k]; new_ids int32 [H][n_new]; medoids int32 [H][Nc] ->
        (f int32 [H][n_new][Nc] or None, member uint8 [H][n_new][Nc], disk int32 [H][n_new][Nc] or None)."""
        torch = self.torch
        W, H, k = sel.shape
        n_new, Nc = new_ids.shape[1], medoids.shape[1]
        if tuple(new_ids.shape) != (H, n_new) or tuple(medoids.shape) != (H, Nc):
            raise ValueError("new_ids must be [H][n_new] and medoids [H][Nc]")
        f = torch.empty((H, n_new, Nc), dtype=torch.int32, device=self.device) if want_counts else None
        member = torch.empty((H, n_new, Nc), dtype=torch.uint8, device=self.device)
        disk = None
        if primary is not None:
            if tuple(primary.shape) != (H, Nc) or tuple(size.shape) != (H, Nc):
                raise ValueError("primary and size must be [H][Nc]")
            disk = torch.empty((H, n_new, Nc), dtype=torch.int32, device=self.device)
        rc = swarm_window_assign(self.ctx, self._dev(sel, torch.int32, "sel"), W, H, k, N,
                                 self._dev(new_ids, torch.int32, "new_ids"), n_new, self._dev(medoids, torch.int32, "medoids"),
                                 Nc, float(tau), None if primary is None else self._dev(primary, torch.int32, "primary"),
                                 None if size is None else self._dev(size, torch.int32, "size"), D,
                                 None if f is None else self._dev(f, torch.int32, "f"),
                                 self._dev(member, torch.uint8, "member"),
                                 None if disk is None else self._dev(disk, torch.int32, "disk"))
        self._check("swarm_window_assign", rc)
        return f, member, disk

    def score_select_indexed(self, kind: str, keys, row_ids, q, k: int, G: int = 1, want_scores: bool = False):
        """Scores and selects over the listed entries only: row_ids int32 [H][M]; returns (positions int32 [B][H][k],
        scores fp32 [B][H][M] or None)."""
        torch = self.torch
        b16 = (torch.bfloat16, torch.int16, torch.uint16)
        H, N, d = keys.shape[0], keys.shape[1], keys.shape[-1]
        B, M = q.shape[0], row_ids.shape[1]
        if tuple(q.shape) != (B, H * G, d) or tuple(row_ids.shape) != (H, M):
            raise ValueError("q must be [B][H*G][d] and row_ids [H][M]")
        out_idx = torch.empty((B, H, k), dtype=torch.int32, device=self.device)
        out_scores = torch.empty((B, H, M), dtype=torch.float32, device=self.device) if want_scores else None
        rc = swarm_score_select_indexed(self.ctx, SWARM_KEYS_TOKEN if kind == "token" else SWARM_KEYS_PAGE_MINMAX,
                                        self._dev(keys, b16, "keys"), H, N, d, G, self._dev(row_ids, torch.int32, "row_ids"), M,
                                        self._dev(q, b16, "q"), B, k, self._dev(out_idx, torch.int32, "out_idx"),
                                        None if out_scores is None else self._dev(out_scores, torch.float32, "out_scores"))
        self._check("swarm_score_select_indexed", rc)
        return out_idx, out_scores

    def expand_clusters(self, clusters, H: int, Nc: int, cl_off, cl_entries, cap_e: int):
        """clusters int32 [groups][Sc] -> (entries int32 [groups][cap_e] (-1 padded), count int32 [groups])."""
        torch = self.torch
        groups, Sc = clusters.shape
        E = cl_entries.shape[1]
        if tuple(cl_off.shape) != (H, Nc + 1) or cl_entries.shape[0] != H:
            raise ValueError("cl_off must be [H][Nc+1] and cl_entries [H][E]")
        entries = torch.empty((groups, cap_e), dtype=torch.int32, device=self.device)
        count = torch.empty((groups,), dtype=torch.int32, device=self.device)
        rc = swarm_expand_clusters(self.ctx, self._dev(clusters, torch.int32, "clusters"), groups, Sc, H, Nc,
                                   self._dev(cl_off, torch.int32, "cl_off"), self._dev(cl_entries, torch.int32, "cl_entries"), E,
                                   self._dev(entries, torch.int32, "entries"), self._dev(count, torch.int32, "count"), cap_e)
        self._check("swarm_expand_clusters", rc)
        return entries, count

    def submission_order(self, q_off, q_cluster):
        """(q_off [groups][D+1], q_cluster [groups][cap]) -> (order [groups][cap], batch_off [groups][cap+1], nb [groups])."""
        torch = self.torch
        groups, D1 = q_off.shape
        cap = q_cluster.shape[1]
        order = torch.empty((groups, cap), dtype=torch.int32, device=self.device)
        batch_off = torch.empty((groups, cap + 1), dtype=torch.int32, device=self.device)
        nb = torch.empty((groups,), dtype=torch.int32, device=self.device)
        rc = swarm_submission_order(self.ctx, self._dev(q_off, torch.int32, "q_off"), self._dev(q_cluster, torch.int32, "q_cluster"),
                                    groups, D1 - 1, cap, self._dev(order, torch.int32, "order"),
                                    self._dev(batch_off, torch.int32, "batch_off"), self._dev(nb, torch.int32, "nb"))
        self._check("swarm_submission_order", rc)
        return order, batch_off, nb

    def map_requests(self, sel, H: int, N: int, e2c, Nc: int, replicas, D: int, weight=None, resident=None,
                     cap: Optional[int] = None, out=None):
        """sel int32 [groups][S].  Returns (q_off [groups][D+1], q_cluster [groups][cap], q_load [groups][D])."""
        torch = self.torch
        groups, S = sel.shape
        R = replicas.shape[1]
        if tuple(e2c.shape) != (H, N) or tuple(replicas.shape) != (H * Nc, R):
            raise ValueError("e2c must be [H][N] and replicas [H*Nc][R]")
        if weight is not None and tuple(weight.shape) != (H * Nc,):
            raise ValueError("weight must be [H*Nc]")
        if resident is not None and resident.numel() < (H * Nc + 31) // 32:
            raise ValueError("resident bitmap too short")
        if cap is None:
            cap = min(S, Nc)
        if out is None:
            q_off = torch.empty((groups, D + 1), dtype=torch.int32, device=self.device)
            q_cluster = torch.empty((groups, cap), dtype=torch.int32, device=self.device)
            q_load = torch.empty((groups, D), dtype=torch.int32, device=self.device)
        else:
            q_off, q_cluster, q_load = out
        rc = swarm_map_requests(self.ctx, self._dev(sel, torch.int32, "sel"), groups, S, H, N,
                                self._dev(e2c, torch.int32, "e2c"), Nc, self._dev(replicas, torch.int32, "replicas"),
                                R, D, None if weight is None else self._dev(weight, torch.int32, "weight"),
                                None if resident is None else self._dev(resident, (torch.int32, torch.uint32), "resident"),
                                self._dev(q_off, torch.int32, "q_off"), self._dev(q_cluster, torch.int32, "q_cluster"),
                                self._dev(q_load, torch.int32, "q_load"), cap)
        self._check("swarm_map_requests", rc)
        return q_off, q_cluster, q_load

    def map_requests_streams(self, idx, N: int, e2c, Nc: int, replicas, D: int, weight=None, resident=None,
                             cap: Optional[int] = None, out=None):
        """idx int32 [steps][B][H][k] (or [B][H][k] for one step), as score_select writes it: the B streams of a step
        are merged per head.  Returns (q_off [steps*H][D+1], q_cluster [steps*H][cap], q_load [steps*H][D])."""
        torch = self.torch
        if idx.dim() == 3:
            idx = idx.unsqueeze(0)
        steps, B, H, k = idx.shape
        R = replicas.shape[1]
        if tuple(e2c.shape) != (H, N) or tuple(replicas.shape) != (H * Nc, R):
            raise ValueError("e2c must be [H][N] and replicas [H*Nc][R]")
        if weight is not None and tuple(weight.shape) != (H * Nc,):
            raise ValueError("weight must be [H*Nc]")
        if resident is not None and resident.numel() < (H * Nc + 31) // 32:
            raise ValueError("resident bitmap too short")
        if cap is None:
            cap = min(B * k, Nc)
        if out is None:
            out = (torch.empty((steps * H, D + 1), dtype=torch.int32, device=self.device),
                   torch.empty((steps * H, cap), dtype=torch.int32, device=self.device),
                   torch.empty((steps * H, D), dtype=torch.int32, device=self.device))
        q_off, q_cluster, q_load = out
        rc = swarm_map_requests_streams(self.ctx, self._dev(idx, torch.int32, "idx"), steps, B, H, k, N,
                                        self._dev(e2c, torch.int32, "e2c"), Nc, self._dev(replicas, torch.int32, "replicas"), R, D,
                                        None if weight is None else self._dev(weight, torch.int32, "weight"),
                                        None if resident is None else self._dev(resident, (torch.int32, torch.uint32), "resident"),
                                        self._dev(q_off, torch.int32, "q_off"), self._dev(q_cluster, torch.int32, "q_cluster"),
                                        self._dev(q_load, torch.int32, "q_load"), cap)
        self._check("swarm_map_requests_streams", rc)
        return out

    def step(self, kind: str, keys, q, k: int, e2c, Nc: int, replicas, D: int, G: int = 1, weight=None, resident=None,
             cap: Optional[int] = None, out_idx=None, out_scores=None, want_scores: bool = False, out=None):
        """One decode step of one stream: q [H*G][d] -> (idx int32 [H][k], scores or None, (q_off, q_cluster, q_load))."""
        torch = self.torch
        b16 = (torch.bfloat16, torch.int16, torch.uint16)
        H, N, d = keys.shape[0], keys.shape[1], keys.shape[-1]
        R = replicas.shape[1]
        if tuple(q.shape) != (H * G, d):
            raise ValueError(f"q has shape {tuple(q.shape)}, expected {(H * G, d)}")
        want = (H, N, d) if kind == "token" else (H, N, 2, d)
        if tuple(keys.shape) != want:
            raise ValueError(f"keys has shape {tuple(keys.shape)}, expected {want}")
        if tuple(e2c.shape) != (H, N) or tuple(replicas.shape) != (H * Nc, R):
            raise ValueError("e2c must be [H][N] and replicas [H*Nc][R]")
        if weight is not None and tuple(weight.shape) != (H * Nc,):
            raise ValueError("weight must be [H*Nc]")
        if resident is not None and resident.numel() < (H * Nc + 31) // 32:
            raise ValueError("resident bitmap too short")
        if cap is None:
            cap = min(k, Nc)
        if out_idx is None:
            out_idx = torch.empty((H, k), dtype=torch.int32, device=self.device)
        if out_scores is None and want_scores:
            out_scores = torch.empty((H, N), dtype=torch.float32, device=self.device)
        if out is None:
            out = (torch.empty((H, D + 1), dtype=torch.int32, device=self.device),
                   torch.empty((H, cap), dtype=torch.int32, device=self.device),
                   torch.empty((H, D), dtype=torch.int32, device=self.device))
        q_off, q_cluster, q_load = out
        rc = swarm_step(self.ctx, SWARM_KEYS_TOKEN if kind == "token" else SWARM_KEYS_PAGE_MINMAX,
                        self._dev(keys, b16, "keys"), H, N, d, G, self._dev(q, b16, "q"), k,
                        self._dev(out_idx, torch.int32, "out_idx"),
                        None if out_scores is None else self._dev(out_scores, torch.float32, "out_scores"),
                        self._dev(e2c, torch.int32, "e2c"), Nc, self._dev(replicas, torch.int32, "replicas"), R, D,
                        None if weight is None else self._dev(weight, torch.int32, "weight"),
                        None if resident is None else self._dev(resident, (torch.int32, torch.uint32), "resident"),
                        self._dev(q_off, torch.int32, "q_off"), self._dev(q_cluster, torch.int32, "q_cluster"),
                        self._dev(q_load, torch.int32, "q_load"), cap)
        self._check("swarm_step", rc)
        return out_idx, out_scores, out

    def calibrate(self, what: int, buf, reps: int = 5) -> float:
        """Measured rate of a minimal kernel (GB/s for the memory measurements over `buf`, TOP/s for the MFMA loop)."""
        rc, value = swarm_calibrate(self.ctx, what, self._dev(buf, None, "buf"), buf.numel() * buf.element_size(), reps)
        self._check("swarm_calibrate", rc)
        return value

    def capture_begin(self):
        self._check("swarm_capture_begin", swarm_capture_begin(self.ctx))

    def capture_end(self) -> int:
        rc, g = swarm_capture_end(self.ctx)
        self._check("swarm_capture_end", rc)
        return g

    def graph_launch(self, graph: int):
        self._check("swarm_graph_launch", swarm_graph_launch(self.ctx, graph))

    def device_status(self) -> int:
        """Synchronises, returns and clears the sticky SWARM_DEV_* flags."""
        rc, flags = swarm_device_status(self.ctx)
        if rc not in (SWARM_OK, SWARM_EDATA):
            raise SwarmError("swarm_device_status", rc, swarm_last_error(self.ctx))
        return flags
