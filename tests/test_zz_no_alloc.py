"""The entry point that allocates nothing (swarm_score_select_static) against swarm_score_select, through the C-ABI.

Both run the same kernels; only the home of the scratch differs (a static device array instead of the context's
buffers), so the selections must be identical.  Calls come in pairs, the second with a smaller input than the
first, because the static array keeps the previous call's contents.  Collected last on purpose: a failure here
must not hide the other GPU tests behind pytest -x."""
import numpy as np
import pytest

from paper_2603_17803_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def both(binding, ctx, cfg, seed_step=0):
    """(status, idx) of the static entry point and of swarm_score_select on the same seeded inputs."""
    K, q = dev(W.keys(cfg)), dev(W.queries(cfg, seed_step, seed_step + 1)[0])
    kind = binding.SWARM_KEYS_TOKEN if cfg.unit == "token" else binding.SWARM_KEYS_PAGE_MINMAX
    out_a = torch.full((cfg.B, cfg.H, cfg.k), -7, dtype=torch.int32, device="cuda")
    out_b = torch.full((cfg.B, cfg.H, cfg.k), -9, dtype=torch.int32, device="cuda")
    rc_a = binding.swarm_score_select_static(ctx, kind, K.data_ptr(), cfg.H, cfg.N, cfg.d, cfg.G, q.data_ptr(), cfg.B, cfg.k,
                                             out_a.data_ptr())
    rc_b = binding.swarm_score_select(ctx, kind, K.data_ptr(), cfg.H, cfg.N, cfg.d, cfg.G, q.data_ptr(), cfg.B, cfg.k,
                                      out_b.data_ptr(), None)
    torch.cuda.synchronize()
    return rc_a, rc_b, out_a.cpu().numpy(), out_b.cpu().numpy()


def test_static_scratch_entry_point_matches_the_allocating_one():
    from paper_2603_17803_amd import binding
    ctx = binding.swarm_create(0, torch.cuda.current_stream().cuda_stream)
    try:
        pairs = [
            # the benchmark's shape, then a smaller ragged one with several streams
            (W.CONFIGS["long_128k"].scaled(T=1), W.CONFIGS["llama8b_32k"].scaled(N=777, k=5, T=1, H=2, B=3)),
            # one long row (sliced selection: scores + the slices' winners), then a short token-level row
            (W.CONFIGS["token_stress"].scaled(T=1), W.CONFIGS["tiny"].scaled(N=100, k=7, T=1)),
            # many streams (matrix-core scorer: scores + folded weights), then fewer streams over fewer pages
            (W.CONFIGS["drift_batch"].scaled(T=1, B=64), W.CONFIGS["drift_batch"].scaled(T=1, B=9, N=300, k=11)),
        ]
        for first, second in pairs:
            for cfg in (first, second):
                rc_a, rc_b, a, b = both(binding, ctx, cfg)
                assert rc_a == binding.SWARM_OK and rc_b == binding.SWARM_OK, binding.swarm_last_error(ctx)
                assert np.array_equal(a, b), cfg
                assert (np.diff(a, axis=-1) > 0).all() and a.min() >= 0 and a.max() < cfg.N
        # shapes beyond the static array are refused before anything is enqueued
        big = W.CONFIGS["tiny"].scaled(N=3 << 20, k=4, T=1, d=8)
        K = torch.zeros((1, big.N, 8), dtype=torch.int16, device="cuda")
        q = torch.zeros((1, 1, 8), dtype=torch.int16, device="cuda")
        out = torch.zeros((1, 1, 4), dtype=torch.int32, device="cuda")
        rc = binding.swarm_score_select_static(ctx, binding.SWARM_KEYS_TOKEN, K.data_ptr(), 1, big.N, 8, 1, q.data_ptr(), 1, 4,
                                               out.data_ptr())
        assert rc == binding.SWARM_EINVAL and "static scratch" in binding.swarm_last_error(ctx)
        rc, flags = binding.swarm_device_status(ctx)
        assert rc == binding.SWARM_OK and flags == 0
    finally:
        binding.swarm_destroy(ctx)
