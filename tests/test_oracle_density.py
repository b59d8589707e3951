"""Pins of the oracle's density pass (Section 5.1: probability, distance, density, medoid queue).

None of these re-types the oracle's loop and compares it with itself: a hand-worked fixture, closed
forms (block-diagonal counts, constant counts), limiting radii, invariants of the queue, and the
integer-threshold identity the device code relies on (checked here against the literal fp64 form).
"""
import json
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "density_hand_case.json")


def test_density_hand_case():
    g = json.load(open(GOLD))
    Cm = np.array(g["C"], np.int32)[None]
    for case in g["cases"]:
        rho, queue, tot = oracle.density(Cm, case["tau"], case["flags"])
        assert tot[0] == g["total"]
        assert rho[0].tolist() == case["rho"], case
        assert queue[0].tolist() == case["queue"], case
    r = g["rescaled"]
    rho, queue, tot = oracle.density(Cm, r["tau"], r["flags"], totals=np.array([r["totals_in"]], np.int64))
    assert tot[0] == r["totals_in"] and rho[0].tolist() == r["rho"] and queue[0].tolist() == r["queue"]


def test_density_block_diagonal_closed_form():
    """Disjoint groups that are always activated together: C is block diagonal with constant blocks,
    so with a radius between the in-block and the cross-block distance rho[i] = size of i's block."""
    sizes = [5, 1, 9, 3]
    counts = [40, 7, 12, 100]
    N = sum(sizes)
    Cm = np.zeros((1, N, N), np.int32)
    o = 0
    block_of = []
    for s, c in zip(sizes, counts):
        Cm[0, o:o + s, o:o + s] = c
        block_of += [s] * s
        o += s
    total = sum(s * s * c for s, c in zip(sizes, counts))
    tau = 1.0 - 0.5 * min(counts) / total            # below 1 (cross-block) and above every in-block distance
    rho, queue, tot = oracle.density(Cm, tau)
    assert tot[0] == total
    assert rho[0].tolist() == block_of
    assert oracle.density(Cm, tau, flags=1)[0][0].tolist() == [b - 1 for b in block_of]
    # queue: blocks in descending size, inside a block ascending id
    assert queue[0].tolist() == sorted(range(N), key=lambda i: (-block_of[i], i))
    # a radius that admits only the heaviest block
    tau2 = 1.0 - 0.5 * (100 + 40) / total
    assert oracle.density(Cm, tau2)[0][0].tolist() == [0] * 5 + [0] + [0] * 9 + [3] * 3


def test_density_limits_and_monotonicity():
    rng = np.random.default_rng(3)
    A = rng.integers(0, 2, (50, 40)).astype(np.int32)
    Cm = (A.T @ A).astype(np.int32)[None]
    N = 40
    assert (oracle.density(Cm, 1.0)[0] == N).all()                    # d <= 1 always
    assert (oracle.density(Cm, 1.0, flags=1)[0] == N - 1).all()
    assert (oracle.density(Cm, -1e-9)[0] == 0).all()                  # d >= 0 always
    nz = (Cm[0] > 0).sum(axis=1)
    assert np.array_equal(oracle.density(Cm, 1.0, flags=2)[0][0], nz)    # strict at 1: exactly the nonzero counts
    prev = np.zeros(N, np.int64)
    for tau in np.linspace(0.9, 1.0, 23):
        rho = oracle.density(Cm, float(tau))[0][0]
        assert (rho >= prev).all()                                    # a larger radius never loses a neighbour
        prev = rho
    # symmetric counts -> the neighbour relation is symmetric -> sum of rho = number of related ordered pairs
    tau = 0.995
    rho = oracle.density(Cm, tau)[0][0]
    rel = (1.0 - Cm[0] / float(Cm[0].sum())) <= tau
    assert np.array_equal(rel, rel.T) and rho.sum() == rel.sum()
    # an all-zero matrix has no defined probabilities: nothing is counted
    z = oracle.density(np.zeros((2, 7, 7), np.int32), 1.0)
    assert (z[0] == 0).all() and (z[2] == 0).all() and z[1].tolist() == [list(range(7))] * 2


def test_density_queue_is_a_stable_descending_permutation():
    rng = np.random.default_rng(5)
    Cm = rng.integers(0, 6, (3, 64, 64)).astype(np.int32)
    Cm = Cm + Cm.transpose(0, 2, 1)
    rho, queue, _ = oracle.density(Cm, 0.9993, nthreads=4)
    for h in range(3):
        q = queue[h]
        assert sorted(q.tolist()) == list(range(64))
        r = rho[h][q]
        assert (np.diff(r) <= 0).all()
        same = np.diff(r) == 0
        assert (np.diff(q)[same] > 0).all()                           # equal density: ascending entry id
    assert np.array_equal(rho, oracle.density(Cm, 0.9993, nthreads=1)[0])


def test_density_integer_threshold_identity():
    """d(c) = 1 - c/total is non-increasing in the integer count c (one correctly rounded division and
    one subtraction), so 'd <= tau' is 'c >= c*' for one integer c*.  The device code counts with c*;
    here the literal fp64 form is compared with the threshold form on many (total, tau) pairs."""
    rng = np.random.default_rng(7)
    for _ in range(200):
        total = int(rng.integers(1, 2 ** 40))
        tau = float(rng.choice([rng.random(), 1.0 - rng.random() * 1e-9, 1.0 - 10.0 ** -rng.integers(1, 12)]))
        cs = np.unique(np.concatenate([rng.integers(0, 2 ** 31, 64), np.arange(0, 50)])).astype(np.int64)
        cs = cs[cs <= total]
        d = 1.0 - cs.astype(np.float64) / float(total)
        for strict in (False, True):
            ok = d < tau if strict else d <= tau
            if ok.any():
                first = np.argmax(ok)
                assert ok[first:].all(), (total, tau)                 # an up-set in c
