"""Pins of the oracle's local-window cluster maintenance (Section 6.2): a hand-worked fixture, the
identity with the co-activation oracle (f is a sub-block of the window's A^T A, an independently pinned
function), limiting radii and the placement recurrence."""
import json
import os

import numpy as np

import oracle
from paper_2603_17803_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden", "window_hand_case.json")


def test_window_hand_case():
    g = json.load(open(GOLD))
    sel = np.array(g["sel"], np.int32)
    new_ids, med = np.array(g["new_ids"], np.int32), np.array(g["medoids"], np.int32)
    for case in g["cases"]:
        f, member, disk = oracle.window_assign(sel, g["N"], new_ids, med, case["tau"])
        assert f.tolist() == g["f"] and disk is None
        assert member.tolist() == case["member"], case
    p = g["placement"]
    f, member, disk = oracle.window_assign(sel, g["N"], new_ids, med, p["tau"], np.array(p["primary"], np.int32),
                                           np.array(p["size"], np.int32), g["D"])
    assert disk.tolist() == p["disk"]


def test_window_counts_are_a_block_of_the_window_coactivation():
    H, N, k, Wn = 3, 96, 9, 40
    sel = W.random_selections(Wn, H, k, N, seed=21, topic_like=True)
    Cm = oracle.coact_update(sel, N)
    rng = np.random.default_rng(2)
    new_ids = np.stack([rng.choice(N, 17, replace=False) for _ in range(H)]).astype(np.int32)
    med = np.stack([rng.choice(N, 11, replace=False) for _ in range(H)]).astype(np.int32)
    f, member, _ = oracle.window_assign(sel, N, new_ids, med, 0.9)
    for h in range(H):
        assert np.array_equal(f[h], Cm[h][np.ix_(new_ids[h], med[h])])
    assert np.array_equal(member.astype(bool), f > 0.1 * Wn)            # 1 - f/W < 0.9  <=>  f > 0.1 W (40 * 0.1 = 4 exactly)
    # an entry compared with itself as medoid: f = its activation count
    f2, _, _ = oracle.window_assign(sel, N, med, med, 0.5)
    for h in range(H):
        assert np.array_equal(np.diagonal(f2[h]), np.diagonal(Cm[h])[med[h]])


def test_window_limits_and_placement_recurrence():
    H, N, k, Wn, D = 2, 50, 5, 16, 5
    sel = W.random_selections(Wn, H, k, N, seed=4, topic_like=False)
    new_ids = np.tile(np.arange(10, 22, dtype=np.int32), (H, 1))
    med = np.tile(np.arange(0, 8, dtype=np.int32), (H, 1))
    assert oracle.window_assign(sel, N, new_ids, med, 1.0 + 1e-12)[1].all()          # d <= 1 < tau
    assert not oracle.window_assign(sel, N, new_ids, med, 0.0)[1].any()              # d >= 0, strict
    f, member, _ = oracle.window_assign(sel, N, new_ids, med, 1.0)
    assert np.array_equal(member.astype(bool), f > 0)                                # d < 1 <=> co-activated at least once
    primary = np.tile(np.arange(8, dtype=np.int32) % D, (H, 1))
    size = np.tile((np.arange(8, dtype=np.int32) * 3 + 1), (H, 1))
    _, member, disk = oracle.window_assign(sel, N, new_ids, med, 1.0, primary, size, D)
    for h in range(H):
        for c in range(8):
            joined = np.flatnonzero(member[h, :, c])
            want = [(primary[h, c] + size[h, c] + j + 1) % D for j in range(len(joined))]   # j-th joiner sees size + j
            assert disk[h, joined, c].tolist() == want
            assert (disk[h, member[h, :, c] == 0, c] == -1).all()
