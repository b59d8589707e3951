"""Pins for the oracle's trace, co-activation and request-mapping steps (CPU only).

Co-activation counts follow Section 5.1 Step 1; the mapper follows Section 6.1.  Pins: hand-worked
fixtures, numpy's integer matmul for the dense definition, closed forms, invariants, and the
special cases (one replica, full replication, identity clustering) whose answer is known
without running any scheduler.
"""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2603_17803_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_coact_hand_case_dense_and_update():
    g = json.load(open(os.path.join(GOLD, "coact_hand_case.json")))
    sel = np.array(g["selections"], np.int32)[:, None, :]          # [rows][H=1][k]
    A = oracle.trace(sel, g["N"])
    assert A.shape == (1, 3, 4) and A.sum() == 9
    assert oracle.coact_dense(A[0]).tolist() == g["C"]
    assert oracle.coact_update(sel, g["N"])[0].tolist() == g["C"]


def test_trace_rows_and_heads():
    sel = np.array([[[0, 2], [1, 3]], [[1, 2], [0, 3]]], np.int32)   # rows=2, H=2, k=2
    A = oracle.trace(sel, 4)
    assert A[0].tolist() == [[1, 0, 1, 0], [0, 1, 1, 0]]
    assert A[1].tolist() == [[0, 1, 0, 1], [1, 0, 0, 1]]
    with pytest.raises(oracle.OracleError):
        oracle.trace(np.array([[[0, 4]]], np.int32), 4)


def test_dense_definition_equals_integer_matmul_and_pair_form():
    sel = W.random_selections(rows=37, H=3, k=9, N=50, seed=5)
    A = oracle.trace(sel, 50)
    Cu = oracle.coact_update(sel, 50, nthreads=4)
    for h in range(3):
        ref = A[h].astype(np.int64).T @ A[h].astype(np.int64)
        assert np.array_equal(oracle.coact_dense(A[h]), ref)
        assert np.array_equal(Cu[h], ref)
    assert np.array_equal(Cu, oracle.coact_update(sel, 50, nthreads=1))


def test_row_blocks_of_the_counts():
    """Row blocks of C (for matrices too large to hold whole): the hand fixture's rows, numpy's integer matmul on
    the block's columns of the trace, ragged block edges, every thread count, and the activation counts on the
    block's diagonal."""
    g = json.load(open(os.path.join(GOLD, "coact_hand_case.json")))
    sel = np.array(g["selections"], np.int32)[:, None, :]
    assert oracle.coact_rows(sel, g["N"], 0, 1, 3).tolist() == g["C"][1:3]
    rows, H, k, N = 41, 3, 7, 53
    sel = W.random_selections(rows, H, k, N, seed=11)
    A = oracle.trace(sel, N).astype(np.int64)
    for h in range(H):
        full = A[h].T @ A[h]
        for r0, r1, nt in ((0, N, 1), (0, 1, 2), (5, 29, 3), (29, N, 8), (N - 1, N, 4)):
            blk = oracle.coact_rows(sel, N, h, r0, r1, nthreads=nt)
            assert np.array_equal(blk, full[r0:r1])
            counts = np.bincount(sel[:, h].ravel(), minlength=N)
            assert np.array_equal(blk[np.arange(r1 - r0), np.arange(r0, r1)], counts[r0:r1])
    with pytest.raises(oracle.OracleError):
        oracle.coact_rows(sel, N, H, 0, 4)                           # no such head
    with pytest.raises(oracle.OracleError):
        oracle.coact_rows(np.array([[[0, 0]]], np.int32), 4, 0, 0, 4)   # repeated entry


def test_coact_invariants():
    rows, H, k, N = 64, 2, 16, 200
    sel = W.random_selections(rows, H, k, N, seed=7)
    Cm = oracle.coact_update(sel, N, nthreads=2)
    for h in range(H):
        c = Cm[h]
        assert np.array_equal(c, c.T)
        counts = np.bincount(sel[:, h].ravel(), minlength=N)         # independent histogram
        assert np.array_equal(np.diag(c), counts)
        assert np.array_equal(c.sum(1), k * counts)
        assert c.sum() == rows * k * k                               # grand total = normaliser of the probability equation
        assert (c <= np.minimum.outer(counts, counts)).all()


def test_coact_closed_forms():
    N, k = 40, 5
    S = np.array([3, 7, 8, 20, 39], np.int32)
    sel = np.tile(S, (11, 1))[:, None, :]
    c = oracle.coact_update(sel, N)[0]
    want = np.zeros((N, N), np.int64); want[np.ix_(S, S)] = 11       # constant selection: 11 * 1_S 1_S^T
    assert np.array_equal(c, want)
    # disjoint topic-pure selections: block diagonal with the per-topic step counts
    blocks = [np.arange(0, 5), np.arange(5, 10), np.arange(10, 15)]
    order = [0, 1, 1, 2, 0, 0, 1]
    sel = np.stack([blocks[t] for t in order]).astype(np.int32)[:, None, :]
    c = oracle.coact_update(sel, 15)[0]
    want = np.zeros((15, 15), np.int64)
    for t, cnt in enumerate([3, 3, 1]):
        want[np.ix_(blocks[t], blocks[t])] = cnt
    assert np.array_equal(c, want)


def test_decay_hand_values_and_limits():
    g = json.load(open(os.path.join(GOLD, "coact_hand_case.json")))
    pairs = g["decay_pairs"]
    N = len(pairs)
    C0 = np.zeros((1, N, N), np.int32)
    C0[0, np.arange(N), np.arange(N)] = [p[0] for p in pairs]
    C0[0, 0, 1] = C0[0, 1, 0] = 1000
    sel = np.array([[[0, 1]]], np.int32)                             # one row activating entries 0 and 1
    c = oracle.coact_update(sel, N, C0.copy(), decay_q16=g["decay_q16"])[0]
    add = np.zeros((N, N), np.int64); add[:2, :2] = 1
    assert np.diag(c).tolist() == [p[1] + int(add[i, i]) for i, p in enumerate(pairs)]
    assert c[0, 1] == 990 + 1 and c[1, 0] == 990 + 1                 # decay first, then the undecayed new evidence
    # 65536 keeps, 0 discards
    keep = oracle.coact_update(sel, N, C0.copy(), decay_q16=65536)[0]
    assert np.array_equal(keep, C0[0] + add)
    drop = oracle.coact_update(sel, N, C0.copy(), decay_q16=0)[0]
    assert np.array_equal(drop, add)
    # two undecayed windows == one window holding both
    s1 = W.random_selections(5, 1, 4, N, seed=1, topic_like=False)
    s2 = W.random_selections(6, 1, 4, N, seed=2, topic_like=False)
    two = oracle.coact_update(s2, N, oracle.coact_update(s1, N))
    one = oracle.coact_update(np.concatenate([s1, s2]), N)
    assert np.array_equal(one, two)


def test_decay_keeps_symmetry_and_diag_recurrence():
    N, k = 60, 6
    Cm = np.zeros((1, N, N), np.int32)
    diag = np.zeros(N, np.int64)
    for w in range(4):
        sel = W.random_selections(30, 1, k, N, seed=10 + w)
        oracle.coact_update(sel, N, Cm, decay_q16=60000)
        diag = (diag * 60000 + 32768) // 65536 + np.bincount(sel.ravel(), minlength=N)
        assert np.array_equal(Cm[0], Cm[0].T)
        assert np.array_equal(np.diag(Cm[0]), diag)


def test_coact_rejects_bad_selections():
    with pytest.raises(oracle.OracleError):
        oracle.coact_update(np.array([[[0, 5]]], np.int32), 5)
    with pytest.raises(oracle.OracleError):
        oracle.coact_update(np.array([[[2, 2]]], np.int32), 5)


def test_coact_count_overflow_is_an_error_not_a_wrap():
    # counts are exact in int32 or the update fails: the last representable count may be reached, not passed
    sel = np.array([[[0, 1]], [[0, 2]]], np.int32)                       # entry 0 twice, pairs (0,1), (0,2) once
    big = np.iinfo(np.int32).max
    C0 = np.zeros((1, 3, 3), np.int32)
    C0[0, 0, 0] = big - 2
    C0[0, 0, 1] = C0[0, 1, 0] = big - 1
    out = oracle.coact_update(sel, 3, C0.copy(), 65536)
    assert out[0, 0, 0] == big and out[0, 0, 1] == big and out[0, 1, 0] == big and out[0, 0, 2] == 1
    C0[0, 0, 0] = big - 1                                                # two increments would pass the limit
    with pytest.raises(oracle.OracleError) as e:
        oracle.coact_update(sel, 3, C0.copy(), 65536)
    assert e.value.code == -5
    # decay first, then add: the same matrix is fine once it has been halved
    out = oracle.coact_update(sel, 3, C0.copy(), 32768)
    assert out[0, 0, 0] == (big - 1 + 1) // 2 + 2


# ------------------------------------------------------------------ request mapping

def bitmap(ids, nbits):
    out = np.zeros((nbits + 31) // 32, np.uint32)
    for i in ids:
        out[i >> 5] |= np.uint32(1 << (i & 31))
    return out


def test_map_hand_case():
    g = json.load(open(os.path.join(GOLD, "map_hand_case.json")))
    args = dict(H=g["H"], N=g["N"], e2c=np.array([g["e2c"]], np.int32), Nc=g["Nc"],
                replicas=np.array(g["replicas"], np.int32), D=g["D"], weight=np.array(g["weight"], np.int32))
    sel = np.array(g["sel"], np.int32)
    off, clu, load = oracle.map_requests(sel, **args)
    assert off.tolist() == g["q_off"] and clu.tolist() == g["q_cluster"] and load.tolist() == g["q_load"]
    off, clu, load = oracle.map_requests(sel, resident=bitmap(g["resident_clusters"], g["Nc"]), **args)
    assert off.tolist() == g["resident_q_off"]
    assert clu.tolist() == g["resident_q_cluster"]
    assert load.tolist() == g["resident_q_load"]


def test_map_single_replica_is_a_table_lookup():
    cfg = W.CONFIGS["llama8b_32k"].scaled(N=256, H=2, T=1, M=32, Nc=32, R=1, D=4)
    e2c, weight, rep = W.cluster_tables(cfg, random_replicas=True)
    sel = W.random_selections(6, 1, 20, cfg.N, seed=3)[:, 0]         # 6 groups
    off, clu, load = oracle.map_requests(sel, cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight)
    for g in range(6):
        h = g % cfg.H
        cl = np.unique(e2c[h][sel[g]])
        for dsk in range(cfg.D):
            want = [c for c in cl if rep[h * cfg.Nc + c, 0] == dsk]
            assert clu[g, off[g, dsk]:off[g, dsk + 1]].tolist() == want
            assert load[g, dsk] == sum(weight[h * cfg.Nc + c] for c in want)


def test_map_full_replication_unit_weights_is_round_robin():
    H, N, Nc, D = 1, 64, 64, 4
    e2c = np.arange(N, dtype=np.int32)[None]
    rep = np.tile(np.arange(D, dtype=np.int32), (Nc, 1))
    sel = np.array([[5, 9, 9, 11, 20, 33, 34, 35, 60, 61, 62]], np.int32)
    off, clu, load = oracle.map_requests(sel, H, N, e2c, Nc, rep, D)
    distinct = np.unique(sel[0])
    for j, c in enumerate(distinct):                                 # j-th distinct item -> SSD j mod D
        dsk = j % D
        assert c in clu[0, off[0, dsk]:off[0, dsk + 1]]
    assert load[0].max() - load[0].min() <= 1 and load[0].sum() == distinct.size


def test_map_identity_clustering_is_the_per_entry_rule_and_replication_order():
    # Entry-level scheduling exactly as the paper words it: entries without replicas go straight to
    # their SSD *first* (ascending replication factor), so replicated entries see those loads.
    H, N, D, R = 1, 6, 2, 2
    e2c = np.arange(N, dtype=np.int32)[None]
    rep = np.array([[0, 1], [0, 1], [0, -1], [0, -1], [0, -1], [1, -1]], np.int32)
    sel = np.arange(N, dtype=np.int32)[None]
    off, clu, load = oracle.map_requests(sel, H, N, e2c, N, rep, D)
    # singles: 2,3,4 -> ssd0 (load 3), 5 -> ssd1 (load 1); then 0 -> ssd1 (2), 1 -> ssd1 (3)
    assert clu[0, off[0, 0]:off[0, 1]].tolist() == [2, 3, 4]
    assert clu[0, off[0, 1]:off[0, 2]].tolist() == [5, 0, 1]
    assert load[0].tolist() == [3, 3]
    # had ids been visited in plain ascending order, entry 0 would have gone to ssd0: the order matters


def test_map_invariants_on_a_skewed_workload():
    cfg = W.CONFIGS["long_128k"].scaled(N=1024, T=1, M=64, Nc=64, H=2)
    e2c, weight, rep = W.cluster_tables(cfg)
    sel = W.random_selections(10, 1, 48, cfg.N, seed=4)[:, 0]
    off, clu, load = oracle.map_requests(sel, cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight, nthreads=3)
    for g in range(10):
        h = g % cfg.H
        distinct = np.unique(e2c[h][sel[g]])
        assert off[g, 0] == 0 and off[g, -1] == distinct.size
        assert sorted(clu[g, :distinct.size].tolist()) == distinct.tolist()      # each exactly once
        assert (clu[g, distinct.size:] == -1).all()
        assert load[g].sum() == weight[h * cfg.Nc + distinct].sum()
        for dsk in range(cfg.D):
            q = clu[g, off[g, dsk]:off[g, dsk + 1]]
            assert (np.diff(q) > 0).all()                                        # uniform R: ascending ids
            assert all(dsk in rep[h * cfg.Nc + c] for c in q)
            assert load[g, dsk] == weight[h * cfg.Nc + q].sum()


def test_map_greedy_choice_is_least_loaded_at_every_step():
    # replay the emitted assignment in visiting order and check each choice was a least-loaded replica
    cfg = W.CONFIGS["llama8b_32k"].scaled(N=512, T=1, M=64, Nc=64, H=1, R=3)
    e2c, weight, rep = W.cluster_tables(cfg, random_replicas=True)
    sel = W.random_selections(4, 1, 64, cfg.N, seed=6)[:, 0]
    off, clu, _ = oracle.map_requests(sel, cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight)
    for g in range(4):
        where = {}
        for dsk in range(cfg.D):
            for c in clu[g, off[g, dsk]:off[g, dsk + 1]]:
                where[int(c)] = dsk
        load = [0] * cfg.D
        for c in sorted(where):
            cand = rep[c]
            best = min(cand, key=lambda s: (load[s], s))
            assert where[c] == best
            load[best] += int(weight[c])


def test_map_errors():
    e2c = np.zeros((1, 4), np.int32)
    rep = np.zeros((1, 1), np.int32)
    with pytest.raises(oracle.OracleError):
        oracle.map_requests(np.array([[7]], np.int32), 1, 4, e2c, 1, rep, 2)      # entry out of range
    with pytest.raises(oracle.OracleError):
        oracle.map_requests(np.array([[1]], np.int32), 1, 4, e2c, 1, np.array([[5]], np.int32), 2)
