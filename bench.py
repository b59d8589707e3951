#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One benchmark "step" is one pass of the whole path over a workload.  Default: the long-context workload (8 KV
heads, 128K tokens in 16-token pages = 8192 page summaries per head, 4096 decode steps, top-256): for every
decode step, score + select, then request mapping of that step's selection; after the last step, scatter all
selections into the trace and build the co-activation matrix C = A^T A.  Decode steps are strictly sequential
(one stream, in order).  To keep the page summaries from being served out of the 256 MB last-level cache,
consecutive decode steps read from `--layers` distinct copies of the summaries (as the layers of a model
would), 16 x 33.5 MB by default.

`--workload drift_batch` runs the batched workload instead (64 decode streams x 4 query heads per KV head over a
shared prefix): per batch step score + select of all streams, one merged request mapping per head, and a decayed
co-activation update every 256 steps.

Prints one JSON line: steps/s of the whole pass, the roofline of the dominant kernel and of the co-activation
build, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
INT8_MFMA_PEAK_TOPS = 5000.0      # the figure the co-activation target is quoted on
FP4_MFMA_PEAK_TOPS = 10100.0      # dense peak of the 4-bit matrix-core form the build runs on
BF16_MFMA_PEAK_TFLOPS = 2500.0


def counter_traffic(workload):
    """HBM bytes per scoring launch from the committed counter summary (FETCH_SIZE + WRITE_SIZE runs, scaled on a plain
    copy), or None when there is none for this workload or the scoring source has changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"score_kernel_{workload}_hbm_traffic.txt")
    src = os.path.join(ROOT, "paper_2603_17803_amd", "csrc", "score.hip")
    try:
        text = open(path).read()
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    m_bytes = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", text, re.M)
    m_hash = re.search(r"^score_hip_sha256:\s*([0-9a-f]{64})", text, re.M)
    if not m_bytes or not m_hash or m_hash.group(1) != digest:
        return None
    return int(m_bytes.group(1))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="long_128k")
    ap.add_argument("--layers", type=int, default=0, help="distinct copies of the key-side buffer rotated through (0: enough for 512 MB)")
    ap.add_argument("--decode-steps", type=int, default=0, help="override T (0 = the workload's)")
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying a graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-coact", action="store_true",
                    help="profiling aid: only the trace + C build of the workload, on seeded synthetic selections")
    ap.add_argument("--only-steps", action="store_true",
                    help="profiling aid: only the decode steps (score, select, map), replayed --steps times, no stage timings")
    ap.add_argument("--stage-reps", type=int, default=20, help="replays per stage-isolated timing (median and min reported)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the path runs on ONE GPU; --gpus above 1 is not supported (there are no collectives)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2603_17803_amd import binding, workloads as W

    cfg = W.CONFIGS[args.workload]
    if args.decode_steps:
        cfg = cfg.scaled(T=args.decode_steps)
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    if args.only_coact:
        only_coact(args, cfg, binding, W, torch, stream)
    elif cfg.B > 1:
        batched(args, cfg, binding, W, torch, np, stream)
    else:
        single_stream(args, cfg, binding, W, torch, np, stream)


class Harness:
    """Graph capture, whole-pass timing and stage-isolated timing shared by the workloads."""

    def __init__(self, args, sw, torch, stream):
        self.args, self.sw, self.torch, self.stream = args, sw, torch, stream

    def runner(self, fn):
        fn()                                             # eager once: grows scratch, warms caches
        self.stream.synchronize()
        if self.args.no_graph:
            return fn
        self.sw.capture_begin()
        fn()
        g = self.sw.capture_end()
        return lambda: self.sw.graph_launch(g)

    def timed(self, run, reps, warm):
        torch, stream = self.torch, self.stream
        for _ in range(warm):
            run()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        e0.record(stream)
        for _ in range(reps):
            run()
        e1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - w0
        return wall, e0.elapsed_time(e1) * 1e-3

    def stage(self, fn, reps, per):
        """Replays fn `reps` times as its own graph, one pair of HIP events per replay on the launch stream:
        (median, min) microseconds per unit."""
        torch, stream = self.torch, self.stream
        run = self.runner(fn)
        run()
        stream.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in evs:
            e0.record(stream)
            run()
            e1.record(stream)
        stream.synchronize()
        ts = sorted(e0.elapsed_time(e1) * 1e3 / per for e0, e1 in evs)
        return ts[len(ts) // 2], ts[0]

    def peaks(self, binding):
        """What minimal kernels reach on this device, next to the nominal peaks."""
        torch, sw = self.torch, self.sw
        big = torch.empty(1 << 30, dtype=torch.int32, device="cuda")           # 4 GiB, far above the last-level cache
        out = {"hbm_read_GBs": round(sw.calibrate(binding.SWARM_CAL_HBM_READ, big, 5), 1),
               "hbm_write_GBs": round(sw.calibrate(binding.SWARM_CAL_HBM_WRITE, big, 5), 1),
               "mfma_i8_TOPs": round(sw.calibrate(binding.SWARM_CAL_MFMA_I8, big, 5), 1),
               "mfma_fp4_TOPs": round(sw.calibrate(binding.SWARM_CAL_MFMA_FP4, big, 5), 1),
               "note": "plain 16-byte streaming over 4 GiB; register-resident loops of v_mfma_i32_32x32x32_i8 and of the 4-bit v_mfma_f32_32x32x64_f8f6f4"}
        del big
        return out


def coact_rooflines(H, N, rows, coact_ms, peaks, decayed):
    """Both roofs of the co-activation build and the one that binds it.  C is written once (read and written when an
    old matrix is updated), so below peak_ops / peak_bytes operations per byte it is the memory system."""
    Tpad = (rows + 511) // 512 * 512
    tiles = (N + 255) // 256 * 2                                               # tiles of 128 x 128 along one side (the trace is padded to 256 entries)
    issued_ops = 2.0 * H * (tiles * (tiles + 1) // 2) * 128 * 128 * Tpad        # MFMA ops actually issued (tiles on or above the diagonal)
    nbytes = H * N * N * 4 * (2 if decayed else 1) + H * N * (Tpad // 8)
    tops = issued_ops / (coact_ms * 1e-3) / 1e12
    gbs = nbytes / (coact_ms * 1e-3) / 1e9
    hbm_bound = issued_ops / nbytes < FP4_MFMA_PEAK_TOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    mfma = {"achieved": round(tops, 1), "peak": FP4_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(tops / FP4_MFMA_PEAK_TOPS, 4),
            "frac_of_int8_peak_5000": round(tops / INT8_MFMA_PEAK_TOPS, 4),
            "frac_of_measured_fp4_peak": round(tops / peaks["mfma_fp4_TOPs"], 4)}
    hbm = {"achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "bytes": nbytes,
           "frac_of_measured_write_peak": round(gbs / peaks["hbm_write_GBs"], 4)}
    roof = hbm if hbm_bound else mfma
    return {"kernel": "coact_syrk_kernel (4-bit matrix-core form, exact counts)", "bound": "hbm" if hbm_bound else "mfma",
            "achieved": roof["achieved"], "peak": roof["peak"], "unit": roof["unit"], "frac": roof["frac"],
            "why": "ops per byte of C moved (%.0f) against the 4-bit balance point (%.0f)" % (
                issued_ops / nbytes, FP4_MFMA_PEAK_TOPS * 1e12 / (HBM_PEAK_GBS * 1e9)),
            "mfma": mfma, "hbm": hbm, "issued_ops": issued_ops}


def single_stream(args, cfg, binding, W, torch, np, stream):
    T, H, N, k = cfg.T, cfg.H, cfg.N, cfg.k

    def dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()

    K = W.keys(cfg)
    qs = W.queries(cfg, 0, T)
    e2c, weight, rep = W.cluster_tables(cfg)
    row_bytes = (2 if cfg.unit == "page" else 1) * cfg.d * 2
    nlayers = args.layers or max(2, -(-(512 << 20) // (H * N * row_bytes)))

    with torch.cuda.stream(stream):
        K0 = dev(K)
        layers = [K0] + [K0.clone() for _ in range(nlayers - 1)]
        q_d = dev(qs)                                    # [T][1][H*G][d]
        e2c_d, w_d, rep_d = dev(e2c), dev(weight), dev(rep)
        idx_all = torch.empty((T, H, k), dtype=torch.int32, device="cuda")
        cap = min(k, cfg.Nc)
        q_off = torch.empty((T, H, cfg.D + 1), dtype=torch.int32, device="cuda")
        q_clu = torch.empty((T, H, cap), dtype=torch.int32, device="cuda")
        q_load = torch.empty((T, H, cfg.D), dtype=torch.int32, device="cuda")
        Cm = torch.zeros((H, N, N), dtype=torch.int32, device="cuda")
    stream.synchronize()
    sw = binding.Swarm(0, stream=stream)
    hx = Harness(args, sw, torch, stream)

    def select_steps():
        for t in range(T):
            sw.score_select(cfg.unit, layers[t % len(layers)], q_d[t], k, G=cfg.G, out_idx=idx_all[t:t + 1])

    score_buf = torch.empty((1, H, N), dtype=torch.float32, device="cuda")

    def score_steps():
        for t in range(T):
            sw.score(cfg.unit, layers[t % len(layers)], q_d[t], G=cfg.G, out_scores=score_buf)

    def map_steps():
        for t in range(T):
            sw.map_requests(idx_all[t], H, N, e2c_d, cfg.Nc, rep_d, cfg.D, w_d, cap=cap,
                            out=(q_off[t], q_clu[t], q_load[t]))

    def coact():
        sw.coact_accumulate(idx_all, N, Cm, decay_q16=0)

    def decode_steps():
        for t in range(T):
            sw.step(cfg.unit, layers[t % len(layers)], q_d[t, 0], k, e2c_d, cfg.Nc, rep_d, cfg.D, G=cfg.G, weight=w_d,
                    cap=cap, out_idx=idx_all[t], out=(q_off[t], q_clu[t], q_load[t]))

    def whole_pass():
        decode_steps()
        coact()

    if args.only_steps:
        run = hx.runner(decode_steps)
        wall, ev = hx.timed(run, args.steps, max(args.warmup, 1))
        print(json.dumps({"only": "steps", "workload": cfg.name, "decode_steps": T, "us_per_step": round(ev / args.steps / T * 1e6, 3)}), flush=True)
        sw.close()
        return

    run_all = hx.runner(whole_pass)
    wall, ev = hx.timed(run_all, args.steps, max(args.warmup - 1, 0))
    flags = sw.device_status()
    assert flags == 0, f"device flags {flags}"
    steps_per_s = T * args.steps / wall

    reps = args.stage_reps
    score_us, score_us_min = hx.stage(score_steps, reps, T)
    sel_us, sel_us_min = hx.stage(select_steps, reps, T)
    step_us, step_us_min = hx.stage(decode_steps, reps, T)
    map_us, map_us_min = hx.stage(map_steps, reps, T)
    coact_us, coact_us_min = hx.stage(coact, reps, 1)

    def coact_popcount():
        sw.coact_accumulate(idx_all, N, Cm, decay_q16=0, flags=binding.SWARM_COACT_POPCOUNT)

    pop_us, pop_us_min = hx.stage(coact_popcount, max(3, reps // 4), 1)
    coact()                                                                      # leave the matrix-core result in C
    tau = 1.0 - 0.25 * float(Cm.max()) / (float(T) * k * k)

    def density():
        sw.coact_density(Cm, tau)

    dens_us, dens_us_min = hx.stage(density, reps, 1)
    # the same C, rho and queue in one pass: the radius test applied to C's tiles while they are in registers
    sep_rho, sep_queue, _ = sw.coact_density(Cm, tau)
    fused_out = (torch.empty((H, N), dtype=torch.int32, device="cuda"), torch.empty((H, N), dtype=torch.int32, device="cuda"),
                 torch.empty((H,), dtype=torch.int64, device="cuda"))

    def build_density():
        sw.coact_build_density(idx_all, N, Cm, tau, out=fused_out)

    fused_us, fused_us_min = hx.stage(build_density, reps, 1)
    stream.synchronize()
    assert torch.equal(fused_out[0], sep_rho) and torch.equal(fused_out[1], sep_queue), "fused density differs from the two-call result"
    # cluster maintenance over the last 256 steps: 256 new entries against one medoid per cluster
    g = np.random.default_rng(cfg.seed + 17)
    new_d = dev(np.stack([g.choice(N, 256, replace=False) for _ in range(H)]).astype(np.int32))
    med_d = dev(np.stack([g.choice(N, cfg.Nc, replace=False) for _ in range(H)]).astype(np.int32))
    win_sel = idx_all[T - 256:]

    def window():
        sw.window_assign(win_sel, N, new_d, med_d, 1.0 - 8.0 / 256, want_counts=False)

    win_us, win_us_min = hx.stage(window, reps, 1)
    # medoid index: score and select over one medoid per cluster instead of every page
    kc = max(1, min(cfg.Nc, k // 8))

    def medoid_steps():
        for t in range(0, T, 8):
            sw.score_select_indexed(cfg.unit, layers[t % len(layers)], med_d, q_d[t], kc, G=cfg.G)

    med_us, med_us_min = hx.stage(medoid_steps, reps, T // 8)
    coact_ms = coact_us * 1e-3
    # the same sweep out of one buffer: served by the 256 MB last-level cache, not by HBM
    layers_all, layers[:] = list(layers), [layers[0]]
    hot_us, _ = hx.stage(score_steps, reps, T)
    layers[:] = layers_all

    peaks = hx.peaks(binding)
    sweep_bytes = H * N * row_bytes + H * cfg.G * cfg.d * 2 + H * N * 4      # key side + queries in, fp32 scores out
    score_gbs = sweep_bytes / (score_us * 1e-6) / 1e9
    # the unit the metric names: one decode step's score + select (and the whole step with its mapping) moves one sweep
    # of the key side, the scores staying in cache, and k indices out
    unit_bytes = H * N * row_bytes + H * cfg.G * cfg.d * 2 + H * k * 4
    roof_steps = HBM_PEAK_GBS * 1e9 / unit_bytes
    dense_ops = 2.0 * H * N * N * T
    increments = float(T) * H * k * k                                            # the trace's own work: k^2 pair counts per row
    roof_coact = coact_rooflines(H, N, T, coact_ms, peaks, decayed=False)
    roof_coact.update({"dense_equivalent_tops": round(dense_ops / (coact_ms * 1e-3) / 1e12, 1),
                       "ms_per_build_incl_trace": round(coact_ms, 3), "ms_min": round(coact_us_min * 1e-3, 3),
                       "pair_increments_per_s": round(increments / (coact_ms * 1e-3), 0),
                       "popcount_route_ms": round(pop_us * 1e-3, 3)})

    out = {
        "metric": "decode steps/s, whole path (score+select+map per step, trace+C build per pass), 128K ctx",
        "value": round(steps_per_s, 1), "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 keys/queries, fp32 scores; counts: 4-bit (E2M1) 0/1 operands, fp32 accumulate (exact below 2^24), int32 C",
        "data": "synthetic (seeded topic mixture standing in for real activation traces)",
        "config": {"workload": cfg.name, "H": H, "pages_per_head": N, "decode_steps": T, "k": k, "clusters": cfg.Nc,
                   "ssds": cfg.D, "replicas": cfg.R, "rotating_key_buffers": len(layers),
                   "graph_replay": not args.no_graph},
        "roofline": {"kernel": "score kernel (one decode step's sweep of the key side)", "bound": "hbm",
                     "achieved": round(score_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(score_gbs / HBM_PEAK_GBS, 4), "traffic": counter_traffic(cfg.name),
                     "bytes_per_launch": sweep_bytes, "us_per_launch": round(score_us, 3),
                     "us_per_launch_min": round(score_us_min, 3), "frac_of_measured_read_peak": round(score_gbs / peaks["hbm_read_GBs"], 4),
                     "cache_resident_single_buffer_GBs": round(sweep_bytes / (hot_us * 1e-6) / 1e9, 1)},
        "roofline_units": {"what": "the units the metric names, against the HBM roof of one sweep of the key side per decode step "
                                   "(%d bytes -> %.0f steps/s at 8 TB/s); these are chains of dependent kernels, so the fraction "
                                   "prices their latency, not a kernel's bandwidth" % (unit_bytes, roof_steps),
                           "bytes_per_step": unit_bytes, "roof_steps_per_s": round(roof_steps, 0),
                           "score_select": {"us_per_step": round(sel_us, 3), "steps_per_s": round(1e6 / sel_us, 1),
                                            "frac": round(1e6 / sel_us / roof_steps, 4)},
                           "whole_step": {"us_per_step": round(step_us, 3), "steps_per_s": round(1e6 / step_us, 1),
                                          "frac": round(1e6 / step_us / roof_steps, 4)}},
        "roofline_coact": roof_coact,
        "density_pass": {"what": "grand total, rho and medoid queue from C (two sweeps of C plus an N^2 ranking)",
                         "ms": round(dens_us * 1e-3, 3), "ms_min": round(dens_us_min * 1e-3, 3), "bound": "hbm",
                         "bytes": 2 * H * N * N * 4, "achieved_GBs": round(2 * H * N * N * 4 / (dens_us * 1e-6) / 1e9, 1)},
        "build_density_one_pass": {"what": "trace + C + rho + queue with the radius test in the C kernel's epilogue (C written once, never read)",
                                   "ms": round(fused_us * 1e-3, 3), "ms_min": round(fused_us_min * 1e-3, 3),
                                   "two_calls_ms": round(coact_ms + dens_us * 1e-3, 3)},
        "window_maintenance": {"what": "last 256 steps, 256 new entries x %d medoids per head: trace bits + counts + membership" % cfg.Nc,
                               "us": round(win_us, 1), "us_min": round(win_us_min, 1)},
        "medoid_index": {"what": "score + select over %d medoids per head (top %d) instead of %d pages" % (cfg.Nc, kc, N),
                         "us_per_step": round(med_us, 3), "us_min": round(med_us_min, 3),
                         "speedup_vs_full_score_select": round(sel_us / med_us, 2)},
        "measured_peaks": peaks,
        "stages": {"timing": f"median (min) over {reps} graph replays, HIP events on the launch stream",
                   "step_us": round(step_us, 3), "step_us_min": round(step_us_min, 3),
                   "score_us_per_step": round(score_us, 3), "score_select_us_per_step": round(sel_us, 3),
                   "score_select_us_min": round(sel_us_min, 3), "map_us_per_step": round(map_us, 3),
                   "map_us_min": round(map_us_min, 3), "map_groups_per_s": round(H * 1e6 / map_us, 0),
                   "coact_ms_per_pass": round(coact_ms, 3), "score_select_steps_per_s": round(1e6 / sel_us, 1),
                   "decode_steps_per_s_without_C_build": round(1e6 / step_us, 1), "event_s_per_pass": round(ev / args.steps, 5)},
        "paper_context": "paper reports 2.41x lower I/O time and 2.72x higher bandwidth utilisation (Xeon 6530, 8x H20, "
                         "<=8 NVMe SSDs); no number for this path",
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, K, qs, e2c, weight, rep, np)
    print(json.dumps(out), flush=True)
    sw.close()


def batched(args, cfg, binding, W, torch, np, stream):
    """Many decode streams per step (the drifting batch): score + select of all streams, one merged request mapping per
    head and step, a decayed co-activation update per window.  One pass = T batch steps = T / window windows."""
    T, H, N, k, B, G = cfg.T, cfg.H, cfg.N, cfg.k, cfg.B, cfg.G
    win = cfg.decay_window or T
    nwin_q = max(1, min(T // win, (cfg.phase_len or win) // win))       # windows with queries of their own (one drift phase)
    nwin = T // win

    def dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()

    K = W.keys(cfg)
    qs = W.queries(cfg, 0, nwin_q * win)                               # [steps][B][H*G][d]; later windows replay these
    e2c, weight, rep = W.cluster_tables(cfg)
    row_bytes = (2 if cfg.unit == "page" else 1) * cfg.d * 2
    nlayers = args.layers or max(2, -(-(512 << 20) // (H * N * row_bytes)))
    cap = min(B * k, cfg.Nc)
    with torch.cuda.stream(stream):
        K0 = dev(K)
        layers = [K0] + [K0.clone() for _ in range(nlayers - 1)]
        q_d = dev(qs)
        e2c_d, w_d, rep_d = dev(e2c), dev(weight), dev(rep)
        idx_win = torch.empty((win, B, H, k), dtype=torch.int32, device="cuda")
        q_off = torch.empty((win, H, cfg.D + 1), dtype=torch.int32, device="cuda")
        q_clu = torch.empty((win, H, cap), dtype=torch.int32, device="cuda")
        q_load = torch.empty((win, H, cfg.D), dtype=torch.int32, device="cuda")
        Cm = torch.zeros((H, N, N), dtype=torch.int32, device="cuda")
        score_buf = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    stream.synchronize()
    sw = binding.Swarm(0, stream=stream)
    hx = Harness(args, sw, torch, stream)
    rows_view = idx_win.view(win * B, H, k)

    def score_steps(w=0):
        for t in range(win):
            tt = w * win + t
            sw.score(cfg.unit, layers[tt % nlayers], q_d[tt], G=G, out_scores=score_buf)

    def select_steps(w=0):
        for t in range(win):
            tt = w * win + t
            sw.score_select(cfg.unit, layers[tt % nlayers], q_d[tt], k, G=G, out_idx=idx_win[t])

    def map_steps():
        for t in range(win):
            sw.map_requests_streams(idx_win[t], N, e2c_d, cfg.Nc, rep_d, cfg.D, w_d, cap=cap, out=(q_off[t], q_clu[t], q_load[t]))

    def coact():
        sw.coact_accumulate(rows_view, N, Cm, decay_q16=cfg.decay_q16)

    def window(w):
        for t in range(win):
            tt = w * win + t
            sw.score_select(cfg.unit, layers[tt % nlayers], q_d[tt], k, G=G, out_idx=idx_win[t])
            sw.map_requests_streams(idx_win[t], N, e2c_d, cfg.Nc, rep_d, cfg.D, w_d, cap=cap, out=(q_off[t], q_clu[t], q_load[t]))
        coact()

    runs = [hx.runner(lambda w=w: window(w)) for w in range(nwin_q)]

    def whole_pass():
        for i in range(nwin):
            runs[i % nwin_q]()

    wall, ev = hx.timed(whole_pass, args.steps, max(args.warmup - 1, 0))
    flags = sw.device_status()
    assert flags == 0, f"device flags {flags}"
    steps_per_s = T * args.steps / wall

    reps = args.stage_reps
    score_us, score_us_min = hx.stage(score_steps, reps, win)
    sel_us, sel_us_min = hx.stage(select_steps, reps, win)
    map_us, map_us_min = hx.stage(map_steps, reps, win)
    coact_us, coact_us_min = hx.stage(coact, reps, 1)
    peaks = hx.peaks(binding)

    L = (2 if cfg.unit == "page" else 1) * cfg.d
    sweep_bytes = H * N * row_bytes + B * H * G * cfg.d * 2 + B * H * N * 4          # key side + queries in, fp32 scores out
    score_gbs = sweep_bytes / (score_us * 1e-6) / 1e9
    flop = 2.0 * H * (-(-B // 32) * 32) * G * (-(-N // 128) * 128) * L                # matrix-core flop actually issued (whole 32 x 32 tiles)
    tflops = flop / (score_us * 1e-6) / 1e12
    unit_bytes = H * N * row_bytes + B * H * G * cfg.d * 2 + B * H * k * 4
    roof_steps = HBM_PEAK_GBS * 1e9 / unit_bytes
    coact_ms = coact_us * 1e-3
    roof_coact = coact_rooflines(H, N, win * B, coact_ms, peaks, decayed=True)
    roof_coact.update({"ms_per_window_incl_trace": round(coact_ms, 3), "ms_min": round(coact_us_min * 1e-3, 3),
                       "trace_rows_per_window": win * B})
    step_us = wall / args.steps / T * 1e6
    out = {
        "metric": "batch decode steps/s, whole path (score+select of %d streams, merged map per step, decayed C update per %d steps)" % (B, win),
        "value": round(steps_per_s, 1), "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 keys/queries on the bf16 matrix cores, fp32 scores; counts: 4-bit (E2M1) 0/1 operands, fp32 accumulate (exact below 2^24), int32 C",
        "data": "synthetic (seeded drifting topic mixture standing in for real activation traces)",
        "config": {"workload": cfg.name, "H": H, "pages_per_head": N, "streams": B, "query_heads_per_kv_head": G, "batch_steps": T, "k": k,
                   "clusters": cfg.Nc, "ssds": cfg.D, "replicas": cfg.R, "decay_window_steps": win, "decay_q16": cfg.decay_q16,
                   "rotating_key_buffers": nlayers, "windows_with_own_queries": nwin_q, "graph_replay": not args.no_graph},
        "stream_steps_per_s": round(steps_per_s * B, 1),
        "roofline": {"kernel": "score_batched_kernel (one batch step: the key side once per 32-stream tile, %d streams x %d query heads on the bf16 matrix cores)" % (B, G),
                     "bound": "hbm", "achieved": round(score_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(score_gbs / HBM_PEAK_GBS, 4), "traffic": counter_traffic(cfg.name),
                     "bytes_per_launch": sweep_bytes, "us_per_launch": round(score_us, 3), "us_per_launch_min": round(score_us_min, 3),
                     "mfma": {"achieved": round(tflops, 1), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                              "frac": round(tflops / BF16_MFMA_PEAK_TFLOPS, 4), "flop_per_launch": flop},
                     "why": "%.0f flop per byte against the bf16 balance point (%.0f): the sweep binds" % (
                         flop / sweep_bytes, BF16_MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9))},
        "roofline_units": {"what": "one batch step against the HBM roof of one sweep of the key side plus the queries (%d bytes -> %.0f steps/s "
                                   "at 8 TB/s); chains of dependent kernels, so the fraction prices their latency" % (unit_bytes, roof_steps),
                           "bytes_per_step": unit_bytes, "roof_steps_per_s": round(roof_steps, 0),
                           "score_select": {"us_per_step": round(sel_us, 3), "steps_per_s": round(1e6 / sel_us, 1),
                                            "frac": round(1e6 / sel_us / roof_steps, 4)},
                           "whole_step": {"us_per_step": round(step_us, 3), "steps_per_s": round(1e6 / step_us, 1),
                                          "frac": round(1e6 / step_us / roof_steps, 4)}},
        "roofline_coact": roof_coact,
        "measured_peaks": peaks,
        "stages": {"timing": f"median (min) over {reps} graph replays of one window of {win} steps, HIP events on the launch stream",
                   "score_us_per_step": round(score_us, 3), "score_us_min": round(score_us_min, 3),
                   "score_select_us_per_step": round(sel_us, 3), "score_select_us_min": round(sel_us_min, 3),
                   "map_us_per_step": round(map_us, 3), "map_us_min": round(map_us_min, 3),
                   "map_groups_per_s": round(H * 1e6 / map_us, 0), "coact_ms_per_window": round(coact_ms, 3),
                   "step_us_whole_pass": round(step_us, 3), "event_s_per_pass": round(ev / args.steps, 5)},
        "paper_context": "paper reports 2.41x lower I/O time and 2.72x higher bandwidth utilisation (Xeon 6530, 8x H20, "
                         "<=8 NVMe SSDs); no number for this path",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_batched(cfg, K, qs, e2c, weight, rep, np)
    print(json.dumps(out), flush=True)
    sw.close()


def only_coact(args, cfg, binding, W, torch, stream):
    """The co-activation build alone (for counter runs: a handful of dispatches instead of a whole pass)."""
    T, H, N, k = cfg.T, cfg.H, cfg.N, cfg.k
    with torch.cuda.stream(stream):
        idx = torch.from_numpy(W.random_selections(T, H, k, N, seed=cfg.seed)).cuda()
        Cm = torch.zeros((H, N, N), dtype=torch.int32, device="cuda")
    stream.synchronize()
    sw = binding.Swarm(0, stream=stream)
    for _ in range(max(args.warmup, 1)):
        sw.coact_accumulate(idx, N, Cm, decay_q16=0)
    stream.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        sw.coact_accumulate(idx, N, Cm, decay_q16=0)
    e1.record(stream)
    stream.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    tiles = (N + 255) // 256 * 2
    issued = 2.0 * H * (tiles * (tiles + 1) // 2) * 128 * 128 * ((T + 511) // 512 * 512)
    print(json.dumps({"only": "coact", "workload": cfg.name, "ms_per_build_incl_trace": round(ms, 3), "issued_ops": issued,
                      "TOPs": round(issued / (ms * 1e-3) / 1e12, 1), "frac_of_int8_peak_5000": round(issued / (ms * 1e-3) / 5e15, 4),
                      "frac_of_fp4_peak_10100": round(issued / (ms * 1e-3) / 10.1e15, 4),
                      "C_write_GBs": round(H * N * N * 4 / (ms * 1e-3) / 1e9, 1)}), flush=True)
    sw.close()


def cpu_baseline(cfg, K, qs, e2c, weight, rep, np):
    """The oracle, as it stands, on a bounded sample of decode steps of the same workload."""
    import oracle
    nthr = oracle.hardware_threads()
    nthr_used = min(nthr, 64)

    def per_step(steps, idx):
        for t in range(steps):
            sc, _, _ = oracle.score(cfg.unit, K, qs[t], G=cfg.G, nthreads=nthr_used)
            idx[t] = oracle.select(sc, cfg.k, nthreads=nthr_used)[0]
            oracle.map_requests(idx[t], cfg.H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight, nthreads=nthr_used)

    def run(steps):
        t0 = time.perf_counter()
        idx = np.empty((steps, cfg.H, cfg.k), np.int32)
        per_step(steps, idx)
        Cm = oracle.coact_update(idx, cfg.N, nthreads=nthr_used)
        del Cm
        return time.perf_counter() - t0

    # sizing probe: the per-step work and the counting rate on their own, so that the fixed cost of a fresh C
    # (2 GB of zeroed pages on the long-context workload) does not pass for per-step cost
    probe_steps = 8
    idx = np.empty((probe_steps, cfg.H, cfg.k), np.int32)
    t0 = time.perf_counter()
    per_step(probe_steps, idx)
    step_s = (time.perf_counter() - t0) / probe_steps
    Cp = oracle.coact_update(idx, cfg.N, nthreads=nthr_used)              # touches every page once
    t0 = time.perf_counter()
    oracle.coact_update(idx, cfg.N, Cp, nthreads=nthr_used)
    count_s = (time.perf_counter() - t0) / probe_steps
    del Cp
    steps = int(max(8, min(cfg.T, 15.0 / max(step_s + count_s, 1e-6))))
    dt = run(steps)
    return {"value": round(steps / dt, 2), "unit": "steps/s", "cores": nthr_used, "kind": "oracle",
            "sample": f"first {steps} of {cfg.T} decode steps: score+select+map per step, then trace + C build "
                      f"({cfg.H}x{cfg.N}x{cfg.N} int32) over those steps"}


def cpu_baseline_batched(cfg, K, qs, e2c, weight, rep, np):
    """The oracle on a bounded sample of batch steps: score, select, merged map per step, one decayed update at the end."""
    import oracle
    nthr_used = min(oracle.hardware_threads(), 64)
    B, H, k = cfg.B, cfg.H, cfg.k

    def run(steps):
        t0 = time.perf_counter()
        idx = np.empty((steps, B, H, k), np.int32)
        for t in range(steps):
            sc, _, _ = oracle.score(cfg.unit, K, qs[t], G=cfg.G, nthreads=nthr_used)
            idx[t] = oracle.select(sc, k, nthreads=nthr_used)
            merged = np.ascontiguousarray(idx[t].transpose(1, 0, 2)).reshape(H, B * k)
            oracle.map_requests(merged, H, cfg.N, e2c, cfg.Nc, rep, cfg.D, weight, nthreads=nthr_used)
        Cm = np.zeros((H, cfg.N, cfg.N), np.int32)
        oracle.coact_update(idx.reshape(steps * B, H, k), cfg.N, Cm, cfg.decay_q16, nthreads=nthr_used)
        return time.perf_counter() - t0

    probe = run(2)
    steps = int(max(4, min(len(qs), cfg.T, 15.0 / max(probe / 2, 1e-6))))
    dt = run(steps)
    return {"value": round(steps / dt, 2), "unit": "steps/s", "cores": nthr_used, "kind": "oracle",
            "sample": f"first {steps} of {cfg.T} batch steps ({B} streams each): score+select+merged map per step, then one decayed "
                      f"trace + C update ({H}x{cfg.N}x{cfg.N} int32) over those steps"}


if __name__ == "__main__":
    main()
