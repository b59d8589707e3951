"""GPU parity at the full sizes of the benchmark configurations, in the launch shapes bench.py uses.

Per stage:
  scores     : sampled decode steps against the oracle, within the score tolerance;
  selections : the oracle's select on the GPU's own scores for the sampled steps, bit-exact; every
               step: k distinct ascending indices;
  C          : every element against the oracle's counts from the GPU's selections, bit-exact (the whole
               matrix at once up to 8 x 8192^2; 65536^2 in blocks of 4096 rows, which the oracle builds
               one at a time); also symmetric, diagonal = activation counts (independent histogram of
               the selections), row sums = k * diagonal, grand total = rows * k^2;
  queues     : sampled groups against the oracle, bit-exact.
"""
import numpy as np
import pytest

import oracle
from paper_2603_17803_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


@pytest.fixture(scope="module")
def sw():
    from paper_2603_17803_amd import binding
    s = binding.Swarm(0)
    yield s
    s.close()


def run_full(sw, cfg, sample_steps, rng):
    K = W.keys(cfg)
    qs = W.queries(cfg, 0, cfg.T)
    e2c, weight, rep = W.cluster_tables(cfg)
    Kd, q_d = dev(K), dev(qs)
    e2c_d, w_d, rep_d = dev(e2c), dev(weight), dev(rep)
    T, H, N, k = cfg.T, cfg.H, cfg.N, cfg.k
    idx_all = torch.empty((T, H, k), dtype=torch.int32, device="cuda")
    cap = min(k, cfg.Nc)
    q_off = torch.empty((T, H, cfg.D + 1), dtype=torch.int32, device="cuda")
    q_clu = torch.empty((T, H, cap), dtype=torch.int32, device="cuda")
    q_load = torch.empty((T, H, cfg.D), dtype=torch.int32, device="cuda")
    sampled = set(int(t) for t in sample_steps)
    kept_scores = {}
    for t in range(T):
        want = t in sampled
        _, sc = sw.score_select(cfg.unit, Kd, q_d[t], k, G=cfg.G, out_idx=idx_all[t:t + 1], want_scores=want)
        if want:
            kept_scores[t] = sc
        sw.map_requests(idx_all[t], H, N, e2c_d, cfg.Nc, rep_d, cfg.D, w_d, cap=cap,
                        out=(q_off[t], q_clu[t], q_load[t]))
    Cm = torch.empty((H, N, N), dtype=torch.int32, device="cuda")
    sw.coact_accumulate(idx_all, N, Cm, decay_q16=0)
    torch.cuda.synchronize()
    assert sw.device_status() == 0

    idx = idx_all.cpu().numpy()
    # selections: k distinct ascending, in range, every step
    assert (np.diff(idx, axis=-1) > 0).all() and idx.min() >= 0 and idx.max() < N

    for t in sorted(sampled):
        sc = kept_scores[t].cpu().numpy()
        _, ref64, ab = oracle.score(cfg.unit, K, qs[t], G=cfg.G, nthreads=8)
        terms = cfg.d * (2 if cfg.unit == "page" else 1) * cfg.G
        tol = np.maximum(1e-3 * np.abs(ref64), terms * 2.0 ** -24 * ab)
        assert (np.abs(sc - ref64) <= tol).all()
        assert np.array_equal(idx[t][None], oracle.select(sc, k, nthreads=8))
        ref_q = oracle.map_requests(idx[t], H, N, e2c, cfg.Nc, rep, cfg.D, weight, cap=cap, nthreads=8)
        for got, ref in zip((q_off[t], q_clu[t], q_load[t]), ref_q):
            assert np.array_equal(got.cpu().numpy(), ref)

    # co-activation properties, on the device (torch is only the container here)
    for h in range(H):
        c = Cm[h]
        counts = torch.bincount(idx_all[:, h].reshape(-1).long(), minlength=N).to(torch.int64)
        assert torch.equal(torch.diagonal(c).to(torch.int64), counts)
        rs = torch.zeros(N, dtype=torch.int64, device="cuda")
        step = max(1, (1 << 27) // N)
        for r0 in range(0, N, step):                          # symmetric, block by block
            blk = c[r0:r0 + step]
            assert torch.equal(blk, c[:, r0:r0 + step].t())
            rs[r0:r0 + step] = blk.sum(dim=1, dtype=torch.int64)
        assert torch.equal(rs, k * counts)
        assert int(rs.sum()) == T * k * k
        # sampled entries: half among the frequently selected entries, half anywhere
        hot = torch.argsort(counts, descending=True)[:256].cpu().numpy()
        ii = np.concatenate([rng.choice(hot, 24), rng.integers(0, N, 24)])
        jj = np.concatenate([rng.choice(hot, 24), rng.integers(0, N, 24)])
        sel_h = idx[:, h, :]
        member = {int(e): (sel_h == e).any(axis=1) for e in set(ii.tolist()) | set(jj.tolist())}
        got = c[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy()
        want = np.array([int((member[int(a)] & member[int(b)]).sum()) for a, b in zip(ii, jj)])
        assert np.array_equal(got, want)
    # every element against the oracle (Section 5.1 Step 1's counts from the same selections)
    if H * N * N * 4 <= (4 << 30):
        C_ref = oracle.coact_update(idx, N, nthreads=16)
        assert np.array_equal(Cm.cpu().numpy(), C_ref)
        del C_ref
    else:
        BLK = 4096                                            # 1 GiB of counts per block at N = 65536
        for h in range(H):
            for r0 in range(0, N, BLK):
                r1 = min(N, r0 + BLK)
                ref = oracle.coact_rows(idx, N, h, r0, r1, nthreads=16)
                assert np.array_equal(Cm[h, r0:r1].cpu().numpy(), ref), (h, r0)
                del ref
    # the whole matrix once more by the independent route (AND + popcount on the bit trace), compared on the device
    C2 = torch.empty_like(Cm)
    sw.coact_accumulate(idx_all, N, C2, decay_q16=0, flags=2)
    assert torch.equal(Cm, C2)
    del C2
    if N <= 8192:
        # density pass over the C just built, against the oracle on the same matrix (Section 5.1, Steps 1-3)
        C_host = Cm.cpu().numpy()
        tau = 1.0 - 0.25 * float(C_host.max()) / (float(T) * k * k)
        rho, queue, tot = sw.coact_density(Cm, tau)
        r_rho, r_queue, r_tot = oracle.density(C_host, tau, nthreads=16)
        assert (r_tot == T * k * k).all() and np.array_equal(tot.cpu().numpy(), r_tot)
        assert np.array_equal(rho.cpu().numpy(), r_rho) and np.array_equal(queue.cpu().numpy(), r_queue)
        assert 0 < int(r_rho.max()) < N
        del C_host
    # build + density in one pass (the radius test inside the C kernel) against the two calls, on the device
    tau = 1.0 - 0.25 * float(Cm.max()) / (float(T) * k * k)
    rho2, queue2, tot2 = sw.coact_density(Cm, tau)
    C3 = torch.empty_like(Cm)
    rho3, queue3, tot3 = sw.coact_build_density(idx_all, N, C3, tau)
    assert torch.equal(C3, Cm) and torch.equal(tot3, tot2) and torch.equal(rho3, rho2) and torch.equal(queue3, queue2)
    assert 0 < int(rho3.max()) < N and sw.device_status() == 0
    del C3, Cm
    torch.cuda.empty_cache()


def test_long_context_full_size(sw):
    """The benchmark's workload: 8 heads x 8192 page summaries, 4096 steps, k = 256, C 8 x 8192^2."""
    cfg = W.CONFIGS["long_128k"]
    rng = np.random.default_rng(11)
    run_full(sw, cfg, rng.choice(cfg.T, 6, replace=False), rng)


def test_llama_layer_full_size(sw):
    cfg = W.CONFIGS["llama8b_32k"]
    rng = np.random.default_rng(12)
    run_full(sw, cfg, rng.choice(cfg.T, 6, replace=False), rng)


def test_token_stress_full_size(sw):
    """One head, 65536 token keys, 8192 steps, k = 1024: the 65536 x 65536 int32 co-activation build (16 GiB)."""
    cfg = W.CONFIGS["token_stress"]
    rng = np.random.default_rng(13)
    run_full(sw, cfg, rng.choice(cfg.T, 3, replace=False), rng)


def test_counts_up_to_the_row_limit_stay_exact(sw):
    """The matrix cores accumulate the 0/1 products in fp32, which holds integers exactly up to 2^24: the most
    trace rows one call accepts.  A trace of that length whose first entry is selected in every row must come
    out as exactly 2^24, and the neighbouring counts as their closed forms."""
    rows, N = 1 << 24, 8
    t = torch.arange(rows, device="cuda", dtype=torch.int32)
    idx = torch.empty((rows, 1, 2), dtype=torch.int32, device="cuda")
    idx[:, 0, 0] = 0
    idx[:, 0, 1] = torch.where(t % 5 == 0, 2, 1).to(torch.int32) + torch.where(t % 7 == 0, 2, 0).to(torch.int32)   # 1, 2, 3 or 4
    n2 = int((torch.where(t % 5 == 0, 2, 1) + torch.where(t % 7 == 0, 2, 0) == 2).sum())
    n1 = int((torch.where(t % 5 == 0, 2, 1) + torch.where(t % 7 == 0, 2, 0) == 1).sum())
    n3 = int((torch.where(t % 5 == 0, 2, 1) + torch.where(t % 7 == 0, 2, 0) == 3).sum())
    n4 = rows - n1 - n2 - n3
    for route in (0, 2):
        Cm = torch.full((1, N, N), -1, dtype=torch.int32, device="cuda")
        sw.coact_accumulate(idx, N, Cm, decay_q16=0, flags=route)
        want = np.zeros((N, N), np.int64)
        want[0, 0] = rows
        for e, n in ((1, n1), (2, n2), (3, n3), (4, n4)):
            want[e, e] = want[0, e] = want[e, 0] = n
        assert np.array_equal(Cm[0].cpu().numpy().astype(np.int64), want), route
    assert want[0, 0] == 16777216 and sw.device_status() == 0
    # one more such call on top of it: the update itself is integer arithmetic, so the sum passes 2^24 exactly
    sw.coact_accumulate(idx, N, Cm, decay_q16=65536)
    assert np.array_equal(Cm[0].cpu().numpy().astype(np.int64), 2 * want)
    del idx, Cm
    torch.cuda.empty_cache()


def test_select_long_rows_sliced_and_streaming(sw):
    """Few long rows are selected in two stages (slices, then their winners); many rows of more than 65536
    entries take the streaming kernel.  Both against the oracle on the device's own scores."""
    for B, N, k in ((1, 65536, 1024), (2, 40000, 700), (1, 200000, 300), (40, 66000, 50),
                    (1, 65536, 2000), (1, 65536, 4000), (3, 131072, 3000), (2, 30000, 9000)):   # every width of the winners' merge
        cfg = W.CONFIGS["tiny"].scaled(N=N, k=k, T=1, d=8, B=B)
        K = W.keys(cfg)
        q = W.queries(cfg, 0, 1)[0]
        idx, sc = sw.score_select("token", dev(K), dev(q), k, want_scores=True)
        sc = sc.cpu().numpy()
        assert np.array_equal(idx.cpu().numpy(), oracle.select(sc, k, nthreads=8)), (B, N, k)
    # heavy ties across slices: the lowest indices win
    vals = np.zeros(50000, np.float32)
    vals[::7] = 1.0
    cfg = W.CONFIGS["tiny"].scaled(N=50000, k=9000, T=1, d=8)
    K = np.full((1, 50000, 8), 0x8000, np.uint16)
    K[0, :, 0] = (vals.view(np.uint32) >> 16).astype(np.uint16)
    qd = dev(np.full((1, 1, 8), 0x3F80, np.uint16))
    idx, sc = sw.score_select("token", dev(K), qd, 9000, want_scores=True)
    assert np.array_equal(idx.cpu().numpy(), oracle.select(sc.cpu().numpy(), 9000))


def test_select_rows_longer_than_the_register_path(sw):
    """More than 65536 entries in a single row (sliced selection)."""
    cfg = W.CONFIGS["tiny"].scaled(N=70000, k=300, T=1, d=8)
    K = W.keys(cfg)
    q = W.queries(cfg, 0, 1)[0]
    idx, sc = sw.score_select("token", dev(K), dev(q), cfg.k, want_scores=True)
    sc = sc.cpu().numpy()
    assert np.array_equal(idx.cpu().numpy(), oracle.select(sc, cfg.k))
    _, ref64, ab = oracle.score("token", K, q)
    assert (np.abs(sc - ref64) <= np.maximum(1e-3 * np.abs(ref64), 8 * 2.0 ** -24 * ab)).all()


def test_drifting_batch_decayed_windows_scaled(sw):
    """Batched, grouped-query scoring with a decayed co-activation update per window (the drifting
    workload at reduced size: 8 streams, 4 query heads per KV head, 5 windows of 16 steps)."""
    cfg = W.CONFIGS["drift_batch"].scaled(N=384, B=8, T=80, k=24, phase_len=32, decay_window=16, M=64, Nc=64)
    K = W.keys(cfg)
    Kd = dev(K)
    e2c, weight, rep = W.cluster_tables(cfg)
    e2c_d, w_d, rep_d = dev(e2c), dev(weight), dev(rep)
    Cd = torch.zeros((cfg.H, cfg.N, cfg.N), dtype=torch.int32, device="cuda")
    Cref = np.zeros((cfg.H, cfg.N, cfg.N), np.int32)
    for w0 in range(0, cfg.T, cfg.decay_window):
        qs = W.queries(cfg, w0, w0 + cfg.decay_window)
        rows = cfg.decay_window * cfg.B
        idx_win = torch.empty((rows, cfg.H, cfg.k), dtype=torch.int32, device="cuda")
        for t in range(cfg.decay_window):
            out_idx = idx_win[t * cfg.B:(t + 1) * cfg.B]
            _, sc = sw.score_select("page", Kd, dev(qs[t]), cfg.k, G=cfg.G, out_idx=out_idx, want_scores=True)
            sel = out_idx.permute(1, 0, 2).reshape(cfg.H, cfg.B * cfg.k).contiguous()     # streams of a step merged per head
            got = sw.map_requests(sel, cfg.H, cfg.N, e2c_d, cfg.Nc, rep_d, cfg.D, w_d)
            if t % 5 == 0:
                sc_h = sc.cpu().numpy()
                _, ref64, ab = oracle.score("page", K, qs[t], G=cfg.G, nthreads=8)
                tol = np.maximum(1e-3 * np.abs(ref64), 2 * cfg.d * cfg.G * 2.0 ** -24 * ab)
                assert (np.abs(sc_h - ref64) <= tol).all()
                assert np.array_equal(out_idx.cpu().numpy(), oracle.select(sc_h, cfg.k, nthreads=8))
                ref = oracle.map_requests(sel.cpu().numpy(), cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight, nthreads=8)
                for g_, r_ in zip(got, ref):
                    assert np.array_equal(g_.cpu().numpy(), r_)
        decay = 65536 if w0 == 0 else cfg.decay_q16
        sw.coact_accumulate(idx_win, cfg.N, Cd, decay_q16=decay)
        oracle.coact_update(idx_win.cpu().numpy(), cfg.N, Cref, decay, nthreads=8)
        assert np.array_equal(Cd.cpu().numpy(), Cref)
    assert np.array_equal(Cref, np.transpose(Cref, (0, 2, 1)))
    assert sw.device_status() == 0


def test_drifting_batch_full_size_across_phase_changes(sw):
    """The drifting batch at its full shape (8 heads x 2048 pages, 64 streams x 4 query heads per KV head, k = 128)
    over its first 2176 decode steps: a half window of 128 steps, then eight decayed windows of 256 steps (16384
    trace rows each).  The windows [896, 1152) and [1920, 2176) straddle the changes of the topic mixture at steps
    1024 and 2048, and eight consecutive decays bring the counts towards their steady state.  Scores run on the
    matrix-core scorer; sampled steps (among them the last step of a phase and the first of the next) against
    the oracle; C after every window against the oracle in full."""
    cfg = W.CONFIGS["drift_batch"]
    H, N, B, k = cfg.H, cfg.N, cfg.B, cfg.k
    K = W.keys(cfg)
    Kd = dev(K)
    e2c, weight, rep = W.cluster_tables(cfg)
    e2c_d, w_d, rep_d = dev(e2c), dev(weight), dev(rep)
    Cd = torch.zeros((H, N, N), dtype=torch.int32, device="cuda")
    Cref = np.zeros((H, N, N), np.int32)
    windows = [(0, 128, 65536)] + [(128 + 256 * w, 128 + 256 * (w + 1), cfg.decay_q16) for w in range(8)]
    assert any(a < cfg.phase_len < b for a, b, _ in windows) and any(a < 2 * cfg.phase_len < b for a, b, _ in windows)
    sampled = {0, 127, 128, cfg.phase_len - 1, cfg.phase_len, 1500, 2 * cfg.phase_len - 1, 2 * cfg.phase_len, 2175}
    distinct = []
    for t0, t1, decay in windows:
        steps = t1 - t0
        qs = W.queries(cfg, t0, t1)
        idx_win = torch.empty((steps * B, H, k), dtype=torch.int32, device="cuda")
        for t in range(steps):
            out_idx = idx_win[t * B:(t + 1) * B]
            want = (t0 + t) in sampled
            _, sc = sw.score_select("page", Kd, dev(qs[t]), k, G=cfg.G, out_idx=out_idx, want_scores=want)
            got = sw.map_requests_streams(out_idx, N, e2c_d, cfg.Nc, rep_d, cfg.D, w_d)    # the 64 streams of a step merged per head
            if want:
                sel = out_idx.permute(1, 0, 2).reshape(H, B * k).contiguous()
                sc_h = sc.cpu().numpy()
                _, ref64, ab = oracle.score("page", K, qs[t], G=cfg.G, nthreads=16)
                tol = np.maximum(1e-3 * np.abs(ref64), 2 * cfg.d * cfg.G * 2.0 ** -24 * ab)
                assert (np.abs(sc_h - ref64) <= tol).all()
                assert np.array_equal(out_idx.cpu().numpy(), oracle.select(sc_h, k, nthreads=16))
                ref = oracle.map_requests(sel.cpu().numpy(), H, N, e2c, cfg.Nc, rep, cfg.D, weight, nthreads=16)
                for g_, r_ in zip(got, ref):
                    assert np.array_equal(g_.cpu().numpy(), r_)
                distinct.append(int(ref[0][:, -1].max()))
        sw.coact_accumulate(idx_win, N, Cd, decay_q16=decay)
        oracle.coact_update(idx_win.cpu().numpy(), N, Cref, decay, nthreads=16)
        assert np.array_equal(Cd.cpu().numpy(), Cref), (t0, t1)
    assert np.array_equal(Cref, np.transpose(Cref, (0, 2, 1)))
    assert max(distinct) > 96                      # the merged selections are long lists (the mapper's split into SSD families)
    assert sw.device_status() == 0
