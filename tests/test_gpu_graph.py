"""GPU: a recorded call sequence (HIP graph) must give, on every replay, what the same calls give when run
eagerly -- with the inputs refreshed, other work of the same context and synchronisations in between."""
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
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def test_replays_of_a_recorded_pass_equal_the_eager_calls():
    from paper_2603_17803_amd import binding
    cfg = W.CONFIGS["llama8b_32k"].scaled(T=5)
    T, H, N, k, D = cfg.T, cfg.H, cfg.N, cfg.k, cfg.D
    tau = 1.0 - 2e-5
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        sw = binding.Swarm(0, stream=stream)
        Kd = dev(W.keys(cfg))
        e2c, weight, rep = W.cluster_tables(cfg)
        e2c_d, rep_d, w_d = dev(e2c), dev(rep), dev(weight)
        cap = min(k, cfg.Nc)
        qsets = [dev(W.queries(cfg, s * T, (s + 1) * T)) for s in range(3)]          # [T][1][H*G][d] each
        q_buf = torch.empty_like(qsets[0])
        idx_all = torch.empty((T, H, k), dtype=torch.int32, device="cuda")
        q_off = torch.empty((T, H, D + 1), dtype=torch.int32, device="cuda")
        q_clu = torch.empty((T, H, cap), dtype=torch.int32, device="cuda")
        q_load = torch.empty((T, H, D), dtype=torch.int32, device="cuda")
        Cm = torch.zeros((H, N, N), dtype=torch.int32, device="cuda")
        rho = torch.empty((H, N), dtype=torch.int32, device="cuda")
        queue = torch.empty((H, N), dtype=torch.int32, device="cuda")
        totals = torch.empty((H,), dtype=torch.int64, device="cuda")
        outputs = (idx_all, q_off, q_clu, q_load, Cm, rho, queue, totals)

        def one_pass():
            for t in range(T):
                sw.step(cfg.unit, Kd, q_buf[t, 0], k, e2c_d, cfg.Nc, rep_d, D, G=cfg.G, weight=w_d, cap=cap,
                        out_idx=idx_all[t], out=(q_off[t], q_clu[t], q_load[t]))
            sw.coact_accumulate(idx_all, N, Cm, decay_q16=65536)                      # accumulates: a skipped replay shows
            sw.coact_density(Cm, tau, out=(rho, queue, totals))

        # eager: three passes with three sets of queries, C growing from zero
        eager = []
        for s in range(3):
            q_buf.copy_(qsets[s])
            one_pass()
            stream.synchronize()
            eager.append([o.clone() for o in outputs])
        assert sw.device_status() == 0
        # the eager passes are themselves right: first pass against the oracle
        idx0 = eager[0][0].cpu().numpy()
        assert np.array_equal(eager[0][4].cpu().numpy(), oracle.coact_update(idx0, N, nthreads=8))
        assert not torch.equal(eager[0][0], eager[1][0]) and not torch.equal(eager[1][5], eager[2][5])

        sw.capture_begin()
        one_pass()
        graph = sw.capture_end()
        try:
            Cm.zero_()
            other = dev(W.random_selections(700, H, k, N, seed=77))
            C_other = torch.zeros_like(Cm)
            for s in range(3):
                q_buf.copy_(qsets[s])
                sw.graph_launch(graph)
                # eager work of the same context between the replays; its longer trace outgrows the scratch
                # the recorded pass uses, which must stay valid for the next replay
                sw.coact_accumulate(other[: 100 + 300 * s], N, C_other, decay_q16=0)
                stream.synchronize()
                for name, got, want in zip(("idx", "q_off", "q_cluster", "q_load", "C", "rho", "queue", "totals"),
                                           outputs, eager[s]):
                    assert torch.equal(got, want), f"replay {s}: {name} differs from the eager pass"
            assert np.array_equal(C_other.cpu().numpy(), oracle.coact_update(other[:700].cpu().numpy(), N, nthreads=8))
            # a fourth replay after the scratch has grown
            Cm.zero_()
            q_buf.copy_(qsets[0])
            sw.graph_launch(graph)
            stream.synchronize()
            for got, want in zip(outputs, eager[0]):
                assert torch.equal(got, want)
            assert sw.device_status() == 0
        finally:
            binding.swarm_graph_destroy(graph)
            sw.close()


def test_recording_refuses_calls_that_would_allocate():
    from paper_2603_17803_amd import binding
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        sw = binding.Swarm(0, stream=stream)
        N, H, k = 512, 1, 16
        sel = dev(W.random_selections(64, H, k, N, seed=3))
        big = dev(W.random_selections(2048, H, k, N, seed=4))
        Cm = torch.zeros((H, N, N), dtype=torch.int32, device="cuda")
        sw.coact_accumulate(sel, N, Cm, decay_q16=0)
        stream.synchronize()
        want = Cm.clone()
        sw.capture_begin()
        sw.coact_accumulate(sel, N, Cm, decay_q16=0)
        with pytest.raises(binding.SwarmError) as e:
            sw.coact_accumulate(big, N, Cm, decay_q16=0)          # longer trace: scratch would have to grow
        assert e.value.code == binding.SWARM_EINVAL
        graph = sw.capture_end()
        try:
            Cm.zero_()
            sw.graph_launch(graph)
            stream.synchronize()
            assert torch.equal(Cm, want)
            assert np.array_equal(want.cpu().numpy(), oracle.coact_update(sel.cpu().numpy(), N, nthreads=4))
        finally:
            binding.swarm_graph_destroy(graph)
            sw.close()
