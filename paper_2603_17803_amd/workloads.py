"""Seeded synthetic workloads for the score -> select -> co-activation -> request-mapping path.

This module only *draws inputs*: topic centres, keys, page summaries, queries, the
entry->cluster map and the replica table.  It contains none of the method's arithmetic
(no scoring, selection, counting or scheduling) and is imported by the tests, the
benchmark and the smoke check alike; neither the CPU oracle nor the HIP path is
imported from here.

The inputs stand in for the activation behaviour the paper observes on real models:
KV entries are activated in stable, recurring, strongly correlated groups (Section 3,
"co-activation" observation; Section 5.1).  A topic mixture gives exactly that
structure: keys are a topic centre plus noise, a query is a (possibly different)
topic centre plus noise, so same-topic entries score high together.

All randomness comes from numpy's Philox counter-based generator keyed by
(seed, sub-stream), so every array is reproducible independently of the others.
bf16 values are carried as uint16 bit patterns (numpy has no bf16 dtype).
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 2603178030
NOISE = 0.3

# sub-stream ids
_S_CENTRE, _S_TOPIC, _S_KEYNOISE, _S_QTOPIC, _S_QNOISE, _S_REPL, _S_PERM = range(7)


@dataclass(frozen=True)
class Config:
    """Shape of one workload.  N counts scored entries per KV head (tokens or pages)."""
    name: str
    index: int            # position in the benchmark's configuration list (seeds derive from it)
    H: int                # KV heads
    N: int                # entries (tokens or pages) per head
    unit: str             # "token" or "page"
    page_size: int        # tokens per page (1 for token-level)
    T: int                # decode steps
    k: int                # top-k per (stream, head, step)
    B: int                # decode streams per step
    G: int                # query heads per KV head
    M: int                # topic centres per head
    Nc: int               # clusters per head
    D: int                # SSDs
    R: int                # replicas per cluster
    d: int = 128
    zipf_entries: bool = False     # entry->topic popularity Zipf(1.1) instead of uniform
    zipf_queries: bool = False     # query->topic popularity Zipf(1.1), re-permuted per phase
    phase_len: int = 0             # steps per drift phase (0 = no drift)
    decay_window: int = 0          # steps per decayed-update window (0 = single undecayed build)
    decay_q16: int = 65536

    def scaled(self, **kw) -> "Config":
        """A smaller (or otherwise altered) instance that keeps the same recipe and seed."""
        return dataclasses.replace(self, **kw)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


CONFIGS: Dict[str, Config] = {
    "tiny": Config("tiny", 0, H=1, N=4096, unit="token", page_size=1, T=256, k=64, B=1, G=1,
                   M=32, Nc=64, D=4, R=2),
    "llama8b_32k": Config("llama8b_32k", 1, H=8, N=2048, unit="page", page_size=16, T=2048, k=128,
                          B=1, G=1, M=256, Nc=256, D=8, R=2),
    "long_128k": Config("long_128k", 2, H=8, N=8192, unit="page", page_size=16, T=4096, k=256,
                        B=1, G=1, M=1024, Nc=1024, D=8, R=3, zipf_entries=True),
    "token_stress": Config("token_stress", 3, H=1, N=65536, unit="token", page_size=1, T=8192,
                           k=1024, B=1, G=1, M=2048, Nc=2048, D=8, R=4),
    "drift_batch": Config("drift_batch", 4, H=8, N=2048, unit="page", page_size=16, T=8192, k=128,
                          B=64, G=4, M=512, Nc=512, D=8, R=2, zipf_queries=True, phase_len=1024,
                          decay_window=256, decay_q16=64881),
}


def _rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64((stream << 32) | sub)]))


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of uint16 bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def zipf_weights(M: int, s: float = 1.1) -> np.ndarray:
    w = 1.0 / np.arange(1, M + 1, dtype=np.float64) ** s
    return w / w.sum()


def centres(cfg: Config) -> np.ndarray:
    """Topic centres, float32 [H][M][d], i.i.d. N(0,1)."""
    out = np.empty((cfg.H, cfg.M, cfg.d), dtype=np.float32)
    for h in range(cfg.H):
        out[h] = _rng(cfg.seed, _S_CENTRE, h).standard_normal((cfg.M, cfg.d), dtype=np.float32)
    return out


def entry_topics(cfg: Config) -> np.ndarray:
    """Topic of every scored entry (token or page), int32 [H][N]."""
    out = np.empty((cfg.H, cfg.N), dtype=np.int32)
    p = zipf_weights(cfg.M) if cfg.zipf_entries else None
    for h in range(cfg.H):
        g = _rng(cfg.seed, _S_TOPIC, h)
        if p is None:
            out[h] = g.integers(0, cfg.M, size=cfg.N, dtype=np.int32)
        else:
            out[h] = g.choice(cfg.M, size=cfg.N, p=p).astype(np.int32)
    return out


def keys(cfg: Config, cen: Optional[np.ndarray] = None, topics: Optional[np.ndarray] = None,
         return_raw: bool = False):
    """Key-side input of the scoring step.

    token unit: bf16 [H][N][d]         (centre[topic] + 0.3*noise)
    page unit : bf16 [H][N][2][d]      (channel-wise min, then max, of the page's bf16 token keys;
                                        the topic is drawn per page)
    With return_raw=True the bf16 token keys [H][N][page_size][d] are returned as well.
    """
    cen = centres(cfg) if cen is None else cen
    topics = entry_topics(cfg) if topics is None else topics
    ps = cfg.page_size if cfg.unit == "page" else 1
    if cfg.unit == "token":
        out = np.empty((cfg.H, cfg.N, cfg.d), dtype=np.uint16)
    else:
        out = np.empty((cfg.H, cfg.N, 2, cfg.d), dtype=np.uint16)
    raw_all = np.empty((cfg.H, cfg.N, ps, cfg.d), dtype=np.uint16) if return_raw else None
    chunk = max(1, (1 << 22) // (ps * cfg.d))
    for h in range(cfg.H):
        g = _rng(cfg.seed, _S_KEYNOISE, h)
        for n0 in range(0, cfg.N, chunk):
            n1 = min(cfg.N, n0 + chunk)
            noise = g.standard_normal((n1 - n0, ps, cfg.d), dtype=np.float32)
            raw = f32_to_bf16(cen[h][topics[h, n0:n1]][:, None, :] + np.float32(NOISE) * noise)
            if return_raw:
                raw_all[h, n0:n1] = raw
            if cfg.unit == "token":
                out[h, n0:n1] = raw[:, 0, :]
            else:
                f = bf16_to_f32(raw)
                out[h, n0:n1, 0] = f32_to_bf16(f.min(axis=1))   # exact: min/max of bf16 values are bf16
                out[h, n0:n1, 1] = f32_to_bf16(f.max(axis=1))
    return (out, raw_all) if return_raw else out


def query_topics(cfg: Config, t0: int, t1: int) -> np.ndarray:
    """Topic behind every query, int32 [t1-t0][B][H*G].  Each step has its own sub-stream, so any
    step range can be drawn on its own.  With drift, the rank->centre permutation of the Zipf
    popularity changes every phase_len steps."""
    out = np.empty((t1 - t0, cfg.B, cfg.H * cfg.G), dtype=np.int32)
    p = zipf_weights(cfg.M) if cfg.zipf_queries else None
    perm_cache: Dict[int, np.ndarray] = {}
    for t in range(t0, t1):
        g = _rng(cfg.seed, _S_QTOPIC, t)
        if p is None:
            out[t - t0] = g.integers(0, cfg.M, size=(cfg.B, cfg.H * cfg.G), dtype=np.int32)
        else:
            ph = t // cfg.phase_len if cfg.phase_len else 0
            if ph not in perm_cache:
                perm_cache[ph] = _rng(cfg.seed, _S_PERM, ph).permutation(cfg.M)
            ranks = g.choice(cfg.M, size=(cfg.B, cfg.H * cfg.G), p=p)
            out[t - t0] = perm_cache[ph][ranks].astype(np.int32)
    return out


def queries(cfg: Config, t0: int, t1: int, cen: Optional[np.ndarray] = None,
            return_topics: bool = False):
    """Queries for steps [t0, t1): bf16 [t1-t0][B][H*G][d] = centre[z] + 0.3*noise."""
    cen = centres(cfg) if cen is None else cen
    z = query_topics(cfg, t0, t1)
    out = np.empty((t1 - t0, cfg.B, cfg.H * cfg.G, cfg.d), dtype=np.uint16)
    head_of = np.arange(cfg.H * cfg.G) // cfg.G
    for t in range(t0, t1):
        noise = _rng(cfg.seed, _S_QNOISE, t).standard_normal((cfg.B, cfg.H * cfg.G, cfg.d), dtype=np.float32)
        c = cen[head_of[None, :], z[t - t0]]            # [B][H*G][d]
        out[t - t0] = f32_to_bf16(c + np.float32(NOISE) * noise)
    return (out, z) if return_topics else out


def cluster_tables(cfg: Config, topics: Optional[np.ndarray] = None, random_replicas: bool = False
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Mapper inputs: e2c int32 [H][N] (cluster of an entry = its topic), weight int32 [H*Nc]
    (cluster size in entries) and replicas int32 [H*Nc][R].

    The primary SSD of cluster i follows the paper's round-robin placement (Section 5.2,
    the SSD-tier placement equation): id_i = p_global mod D, then p_global += |C_i|; the r-th
    replica sits floor(D/R) devices further on.  random_replicas=True draws R distinct SSDs
    per cluster instead.
    """
    topics = entry_topics(cfg) if topics is None else topics
    e2c = topics.astype(np.int32)
    weight = np.zeros((cfg.H, cfg.Nc), dtype=np.int32)
    for h in range(cfg.H):
        weight[h] = np.bincount(e2c[h], minlength=cfg.Nc)[: cfg.Nc]
    replicas = np.empty((cfg.H, cfg.Nc, cfg.R), dtype=np.int32)
    if random_replicas:
        g = _rng(cfg.seed, _S_REPL, 0)
        for h in range(cfg.H):
            for c in range(cfg.Nc):
                replicas[h, c] = g.permutation(cfg.D)[: cfg.R]
    else:
        stride = max(1, cfg.D // cfg.R)
        p_global = 0
        for h in range(cfg.H):
            for c in range(cfg.Nc):
                first = p_global % cfg.D
                replicas[h, c] = (first + stride * np.arange(cfg.R)) % cfg.D
                p_global += int(weight[h, c])
    return e2c, weight.reshape(-1), replicas.reshape(cfg.H * cfg.Nc, cfg.R)


def random_selections(rows: int, H: int, k: int, N: int, seed: int, topic_like: bool = True) -> np.ndarray:
    """Synthetic selections int32 [rows][H][k]: k distinct ascending entry ids per (row, head),
    for exercising the co-activation and mapping steps without running the scorer.  With
    topic_like=True half of each selection is a contiguous run (recurring groups)."""
    g = _rng(seed, 99, 0)
    out = np.empty((rows, H, k), dtype=np.int32)
    for r in range(rows):
        for h in range(H):
            if topic_like and k >= 2 and N >= 2 * k:
                run = k // 2
                start = int(g.integers(0, N - run + 1))
                a = np.arange(start, start + run)
                rest = np.setdiff1d(g.choice(N, size=min(N, 2 * k), replace=False), a)[: k - run]
                sel = np.concatenate([a, rest])
            else:
                sel = g.choice(N, size=k, replace=False)
            out[r, h] = np.sort(sel)
    return out
