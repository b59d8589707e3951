"""Pins of the oracle's medoid-indexed retrieval helpers: listed-row scoring (must equal the full
scorer at those rows, an independently pinned function), cluster expansion and submission order (hand
fixture, closed forms, invariants), and the padding value in the mapping step."""
import json
import os

import numpy as np

import oracle
from paper_2603_17803_amd import workloads as W

G_ = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "retrieval_hand_case.json")))


def test_score_rows_is_the_full_scorer_at_those_rows():
    for name in ("tiny", "llama8b_32k"):
        cfg = W.CONFIGS[name].scaled(N=96, T=1, H=2 if name == "tiny" else 3, G=2, B=2)
        K, q = W.keys(cfg), W.queries(cfg, 0, 1)[0]
        rng = np.random.default_rng(1)
        ids = np.stack([rng.choice(cfg.N, 17, replace=False) for _ in range(cfg.H)]).astype(np.int32)
        f32, f64, ab = oracle.score_rows(cfg.unit, K, ids, q, G=cfg.G)
        full32, full64, fullab = oracle.score(cfg.unit, K, q, G=cfg.G)
        for h in range(cfg.H):
            assert np.array_equal(f32[:, h], full32[:, h][:, ids[h]])
            assert np.array_equal(f64[:, h], full64[:, h][:, ids[h]]) and np.array_equal(ab[:, h], fullab[:, h][:, ids[h]])


def test_expand_clusters_hand_case_and_union():
    e = G_["expand"]
    entries, count = oracle.expand_clusters(np.array(e["clusters"], np.int32), e["H"], e["Nc"], np.array(e["cl_off"], np.int32),
                                            np.array(e["cl_entries"], np.int32), e["cap_e"])
    assert entries.tolist() == e["entries"] and count.tolist() == e["count"]
    # random clusters: the expansion, taken as a set, is the union of the activated clusters' members
    rng = np.random.default_rng(9)
    H, Nc, N = 2, 30, 200
    sizes = rng.integers(0, 9, (H, Nc))
    off = np.zeros((H, Nc + 1), np.int32)
    off[:, 1:] = np.cumsum(sizes, axis=1)
    E = int(off[:, -1].max())
    ent = np.full((H, E), -7, np.int32)
    for h in range(H):
        ent[h, :off[h, -1]] = rng.integers(0, N, off[h, -1])
    clusters = rng.integers(-1, Nc, (6, 12)).astype(np.int32)
    entries, count = oracle.expand_clusters(clusters, H, Nc, off, ent, cap_e=12 * 8)
    for g in range(6):
        h = g % H
        act = sorted(set(c for c in clusters[g].tolist() if c >= 0))
        want = [x for c in act for x in ent[h, off[h, c]:off[h, c + 1]].tolist()]
        assert entries[g, :count[g]].tolist() == want and (entries[g, count[g]:] == -1).all()


def test_submission_order_hand_case_and_invariants():
    s = G_["submission"]
    order, batch_off, nb = oracle.submission_order(np.array(s["q_off"], np.int32), np.array(s["q_cluster"], np.int32))
    assert order.tolist() == s["order"] and batch_off.tolist() == s["batch_off"] and nb.tolist() == s["nb"]
    # from real buckets: a permutation of the routed items; batch b = b-th item of every bucket, ascending SSD
    cfg = W.CONFIGS["tiny"]
    e2c, weight, rep = W.cluster_tables(cfg)
    sel = W.random_selections(5, cfg.H, 40, cfg.N, seed=3)[:, 0, :]
    q_off, q_clu, _ = oracle.map_requests(sel, cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight)
    order, batch_off, nb = oracle.submission_order(q_off, q_clu)
    for g in range(5):
        n = q_off[g, -1]
        assert sorted(order[g, :n].tolist()) == sorted(q_clu[g, :n].tolist())
        lens = np.diff(q_off[g])
        assert nb[g] == lens.max()
        for b in range(nb[g]):
            want = [q_clu[g, q_off[g, d] + b] for d in range(cfg.D) if lens[d] > b]
            assert order[g, batch_off[g, b]:batch_off[g, b + 1]].tolist() == want


def test_map_skips_padding_entries():
    cfg = W.CONFIGS["tiny"]
    e2c, weight, rep = W.cluster_tables(cfg)
    sel = W.random_selections(3, cfg.H, 20, cfg.N, seed=8)[:, 0, :]
    padded = np.concatenate([sel, np.full((3, 5), -1, np.int32)], axis=1)[:, np.random.default_rng(0).permutation(25)]
    a = oracle.map_requests(sel, cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight, cap=20)
    b = oracle.map_requests(padded, cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight, cap=20)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
