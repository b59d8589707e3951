"""Pins for the oracle's score and select steps (CPU only).

Score follows Section 2.3 (query-key inner product) and, for pages, the channel-wise upper
bound over the page's [min,max] box.  Select keeps the k highest scores (Section 2.3) with the
lowest-index tie-break.  Each pin is independent of the oracle's own code: hand-worked values,
numpy's matmul / lexsort on the special cases that reduce to them, and invariants.
"""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2603_17803_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf(x):
    b = W.f32_to_bf16(np.asarray(x, np.float32))
    assert np.array_equal(W.bf16_to_f32(b), np.asarray(x, np.float32)), "fixture value not bf16-exact"
    return b


def test_bf16_decoding_known_bit_patterns():
    # IEEE: bf16 = top half of binary32.  0x3F80=1, 0xC000=-2, 0x3E80=0.25, 0x4049=3.140625, 0x0080=2^-126
    bits = np.array([0x3F80, 0xC000, 0x3E80, 0x4049, 0x0080, 0x8000], np.uint16)
    want = [1.0, -2.0, 0.25, 3.140625, 2.0 ** -126, -0.0]
    keys = bits.reshape(1, 6, 1)
    q = np.array([0x3F80], np.uint16).reshape(1, 1, 1)          # q = 1.0
    _, s64, _ = oracle.score("token", keys, q)
    assert s64[0, 0].tolist() == want


def test_score_hand_cases():
    g = json.load(open(os.path.join(GOLD, "score_hand_cases.json")))
    for case in g["token"]:
        keys = bf(case["keys"])[None]
        q = bf(case["q"])[None, None]
        f32, f64, _ = oracle.score("token", keys, q)
        assert f64[0, 0].tolist() == case["expect"]
        assert f32[0, 0].tolist() == case["expect"]
    for case in g["page"]:
        keys = np.stack([bf(case["min"]), bf(case["max"])], axis=1)[None]      # [1][P][2][d]
        q = bf(case["q"])[None, None]
        _, f64, _ = oracle.score("page", keys, q)
        assert f64[0, 0].tolist() == case["expect"]
    case = g["gqa"]
    _, f64, _ = oracle.score("token", bf(case["keys"])[None], bf(case["q"])[None], G=2)
    assert f64[0, 0].tolist() == case["expect"]


def test_token_score_equals_numpy_matmul_and_indexing():
    # several heads / streams / query heads with distinct data: catches a wrong head or stream index
    cfg = W.CONFIGS["llama8b_32k"].scaled(unit="token", page_size=1, N=300, H=3, G=2, B=2, T=2)
    K = W.keys(cfg)
    q = W.queries(cfg, 0, 1)[0]                     # [B][H*G][d]
    f32, f64, ab = oracle.score("token", K, q, G=cfg.G, nthreads=3)
    Kd = W.bf16_to_f32(K).astype(np.float64)
    qd = W.bf16_to_f32(q).astype(np.float64)
    for b in range(cfg.B):
        for h in range(cfg.H):
            ref = sum(Kd[h] @ qd[b, h * cfg.G + g] for g in range(cfg.G))
            np.testing.assert_allclose(f64[b, h], ref, rtol=0, atol=1e-10)
            refabs = sum(np.abs(Kd[h] * qd[b, h * cfg.G + g]).sum(1) for g in range(cfg.G))
            np.testing.assert_allclose(ab[b, h], refabs, rtol=1e-12)
    assert np.array_equal(f32, f64.astype(np.float32))


def test_thread_count_does_not_change_results():
    cfg = W.CONFIGS["llama8b_32k"].scaled(N=64, H=4, T=1)
    K = W.keys(cfg)
    q = W.queries(cfg, 0, 1)[0]
    a = oracle.score("page", K, q)[1]
    b = oracle.score("page", K, q, nthreads=5)[1]
    assert np.array_equal(a, b)


def test_page_of_one_token_is_the_token_score():
    cfg = W.CONFIGS["tiny"].scaled(N=257, T=1)
    K = W.keys(cfg)                                  # [1][N][d]
    q = W.queries(cfg, 0, 1)[0]
    page = np.stack([K, K], axis=2)                  # min == max
    a = oracle.score("token", K, q)[1]
    b = oracle.score("page", page, q)[1]
    assert np.array_equal(a, b)


def test_page_score_bounds_every_token_in_the_page_and_sign_cases():
    cfg = W.CONFIGS["llama8b_32k"].scaled(N=96, H=2, T=1)
    S, raw = W.keys(cfg, return_raw=True)            # S [H][P][2][d], raw [H][P][16][d]
    q = W.queries(cfg, 0, 1)[0]
    _, page, _ = oracle.score("page", S, q)
    rawd = W.bf16_to_f32(raw).astype(np.float64)
    qd = W.bf16_to_f32(q).astype(np.float64)
    for h in range(cfg.H):
        tok = np.einsum("ptc,c->pt", rawd[h], qd[0, h])
        assert (page[0, h] >= tok.max(1) - 1e-9).all()
    # all-positive query picks max, all-negative picks min
    qpos = W.f32_to_bf16(np.abs(W.bf16_to_f32(q)))
    qneg = W.f32_to_bf16(-np.abs(W.bf16_to_f32(q)))
    Sd = W.bf16_to_f32(S).astype(np.float64)
    _, ppos, _ = oracle.score("page", S, qpos)
    _, pneg, _ = oracle.score("page", S, qneg)
    for h in range(cfg.H):
        np.testing.assert_allclose(ppos[0, h], Sd[h, :, 1] @ W.bf16_to_f32(qpos[0, h]).astype(np.float64), atol=1e-10)
        np.testing.assert_allclose(pneg[0, h], Sd[h, :, 0] @ W.bf16_to_f32(qneg[0, h]).astype(np.float64), atol=1e-10)


def test_gqa_is_the_sum_of_the_group_heads():
    cfg = W.CONFIGS["drift_batch"].scaled(N=40, H=2, G=3, B=2, T=1, M=16, Nc=16)
    S = W.keys(cfg)
    q = W.queries(cfg, 0, 1)[0]                      # [B][H*G][d]
    _, grouped, _ = oracle.score("page", S, q, G=cfg.G)
    total = np.zeros_like(grouped)
    for g in range(cfg.G):
        qg = np.stack([q[:, h * cfg.G + g] for h in range(cfg.H)], axis=1)
        total += oracle.score("page", S, qg, G=1)[1]
    np.testing.assert_allclose(grouped, total, atol=1e-10)


# ------------------------------------------------------------------ select

def np_topk(scores, k):
    """Library statement of the rule: stable order by (score desc, index asc), first k, ascending."""
    s = np.where(np.isnan(scores), -np.inf, scores.astype(np.float64))
    nan_last = np.isnan(scores)
    order = np.lexsort((np.arange(scores.size), -s, nan_last))
    return np.sort(order[:k]).astype(np.int32)


def test_select_matches_lexsort_on_random_and_quantised_scores():
    rng = np.random.default_rng(1)
    for N, k in [(50, 7), (1000, 64), (1000, 1000), (333, 1)]:
        s = rng.standard_normal((4, N)).astype(np.float32)
        sq = np.round(s * 2) / 2                     # heavy ties
        for arr in (s, sq.astype(np.float32)):
            got = oracle.select(arr, k, nthreads=2)
            for r in range(arr.shape[0]):
                assert np.array_equal(got[r], np_topk(arr[r], k))


def test_select_crafted_ties_and_special_values():
    N = 16
    assert oracle.select(np.zeros((1, N), np.float32), 5)[0].tolist() == [0, 1, 2, 3, 4]
    s = np.array([[1, 3, 2, 3, 2, 2, 0, 3]], np.float32)
    assert oracle.select(s, 4)[0].tolist() == [1, 2, 3, 7]          # three 3s, then the first 2
    assert oracle.select(s, 5)[0].tolist() == [1, 2, 3, 4, 7]
    z = np.array([[-0.0, 0.0, -0.0, -1.0, 0.0]], np.float32)        # -0 ties with +0
    assert oracle.select(z, 2)[0].tolist() == [0, 1]
    n = np.array([[np.nan, -np.inf, 1.0, np.nan, -5.0]], np.float32)
    assert oracle.select(n, 3)[0].tolist() == [1, 2, 4]             # NaN below -inf
    assert oracle.select(n, 4)[0].tolist() == [0, 1, 2, 4]          # first NaN by index
    inf = np.array([[np.inf, 1e38, -1e38, np.inf]], np.float32)
    assert oracle.select(inf, 2)[0].tolist() == [0, 3]


def test_select_output_is_k_distinct_ascending():
    rng = np.random.default_rng(2)
    s = rng.standard_normal((8, 512)).astype(np.float32)
    idx = oracle.select(s, 100)
    assert (np.diff(idx, axis=1) > 0).all() and idx.min() >= 0 and idx.max() < 512
    # every selected score >= every unselected score
    for r in range(8):
        mask = np.zeros(512, bool); mask[idx[r]] = True
        assert s[r][mask].min() >= s[r][~mask].max()


def test_select_rejects_bad_k():
    with pytest.raises(oracle.OracleError):
        oracle.select(np.zeros((1, 4), np.float32), 5)
    with pytest.raises(oracle.OracleError):
        oracle.select(np.zeros((1, 4), np.float32), 0)
