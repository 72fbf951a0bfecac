#!/usr/bin/env python3
"""Benchmark of the SAPS-PSGD round on one MI355X.

A step is one whole round (Alg. 2 lines 5-10 for all n workers): mask generation, compaction,
pairwise averaging, fused with the SGD-momentum step where the workload has gradients.
Inputs are seeded synthetic models shaped like the paper's CNN workloads and are resident in
HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "mnist_cnn", "cifar10_cnn"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg (no cpu_baseline, no parity check)")
    ap.add_argument("--cpu-rounds", type=int, default=None)
    ap.add_argument("--tune", default="", help="comma list knob=value, e.g. ppb=8,xcd=1,nt=1,path=1")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build keeps all n worker replicas in the HBM of ONE GPU; there is no multi-GPU path "
              "(run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2002_09692_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    binding.load_library()
    # everything runs on one ordinary (non-null) stream: launches on the null stream measured several
    # microseconds slower each, which matters for the launch-bound small workloads
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)

    wl = synth.workload(args.workload)
    steps = args.steps if args.steps is not None else wl.rounds
    warm = args.warmup
    n, N, ld = wl.n, wl.N, wl.ld()
    cap = synth.recommended_capacity(wl)
    seed = 0

    t0 = time.time()
    X0 = synth.make_models(wl, ld)
    G0 = synth.make_grads(wl, 0, ld) if wl.fused else None
    log(f"[bench] {wl.name}: n={n} N={N} ld={ld} cap={cap} inputs generated in {time.time() - t0:.1f}s")
    # bandwidth workloads draw their matchings from the library's own Alg. 3 peer selection
    selector = (binding.PeerSelector(wl.bandwidth(), wl.B_thres, wl.T_thres, wl.matching_seed)
                if wl.matching == "bandwidth" else None)
    peers = {t: wl.peers(t, selector) for t in range(1, max(warm + steps, wl.rounds) + 8)}

    # X, G, V are carved back to back out of one device arena (a flat parameter arena is the natural
    # home of n replicas); besides fewer allocations this keeps the three streams from starting at
    # the same offset inside a 2 MiB page, which measures 3-5 % faster than three separate tensors
    arena = torch.empty((3 if wl.has_buffer else 2 if wl.fused else 1) * n * ld, dtype=torch.float32, device="cuda")
    X = arena[0:n * ld].view(n, ld); X.copy_(torch.from_numpy(X0))
    G = V = None
    if wl.fused:
        G = arena[n * ld:2 * n * ld].view(n, ld); G.copy_(torch.from_numpy(G0))
        if wl.has_buffer:
            V = arena[2 * n * ld:3 * n * ld].view(n, ld); V.zero_()
    idx = torch.zeros(cap, dtype=torch.int32, device="cuda")
    msg = torch.zeros((n, cap), dtype=torch.float32, device="cuda")
    Ks = torch.zeros(max(warm + steps, wl.rounds) + 8, dtype=torch.int64, device="cuda")
    lr, mu = (wl.lr, wl.mu) if wl.fused else (0.0, 0.0)

    ctx = binding.SapsContext(n, N, ld, cap, wl.seg_c, wl.seg_off)
    knobs = {"ppb": binding.TUNE_PAIRS_PER_BLOCK, "xcd": binding.TUNE_XCD_REMAP, "nt": binding.TUNE_NONTEMPORAL,
             "path": binding.TUNE_EXCHANGE_PATH, "bpc": binding.TUNE_BLOCKS_PER_CU}
    for kv in filter(None, args.tune.split(",")):
        k, v = kv.split("=")
        ctx.saps_set_tuning(knobs[k], int(v))

    # ---- CPU oracle leg: timed baseline and a bit-exact check of the same rounds on the GPU
    cpu = None
    parity = "not checked (--no-cpu)"
    if not args.no_cpu:
        from oracle import saps_oracle as O
        r_cpu = args.cpu_rounds if args.cpu_rounds is not None else wl.rounds   # the workload's whole trajectory
        Xo = X0.copy(); Vo = np.zeros_like(Xo) if wl.has_buffer else None
        t_cpu = 0.0
        Kc = []
        for t in range(1, r_cpu + 1):
            t1 = time.perf_counter()
            rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, lr, mu, seed, t, peers[t], wl.seg_c, wl.seg_off, msg_ld=cap)
            t_cpu += time.perf_counter() - t1
            assert rc == O.OK, rc
            Kc.append(K)
            ctx.saps_round(X, G, V, lr, mu, seed, t, peers[t], idx, msg, Ks[t:t + 1])
        st, Kg = ctx.saps_poll_status()
        assert st == 0 and Kg == Kc[-1], (st, Kg, Kc[-1])
        same = (np.array_equal(X.cpu().numpy().view(np.uint32), Xo.view(np.uint32))
                and (V is None or np.array_equal(V.cpu().numpy().view(np.uint32), Vo.view(np.uint32)))
                and np.array_equal(idx.cpu().numpy().view(np.uint32)[:Kg], idx_o[:Kg])
                and np.array_equal(msg.cpu().numpy()[:, :Kg].view(np.uint32), msg_o[:, :Kg].view(np.uint32)))
        parity = f"bit-exact vs oracle after {r_cpu} round(s): X, V, idx, msg, K" if same else "MISMATCH vs oracle"
        log(f"[bench] oracle: {r_cpu} round(s) in {t_cpu:.2f}s; parity: {parity}")
        assert same, "GPU result differs from the CPU oracle"
        cpu = {"value": n * N * r_cpu / t_cpu, "unit": "model coords/s", "cores": 1, "kind": "oracle",
               "sample": f"{r_cpu} full round(s) of {wl.name} on the same inputs, single thread, "
                         f"{os.cpu_count()} host cores visible", "s_per_round": t_cpu / r_cpu}
        del Xo, Vo
        # restart from the initial state so that the timed rounds are the workload's rounds 1..K
        X.copy_(torch.from_numpy(X0))
        if V is not None:
            V.zero_()

    # ---- copy yardstick (same access shape, one read + one write per element)
    scratch = torch.empty_like(X)
    ctx.saps_profile_enable(True)
    for _ in range(3):
        ctx.saps_stream_copy(scratch, X)
    ctx.saps_profile_read()
    for _ in range(10):
        ctx.saps_stream_copy(scratch, X)
    cl, cms = ctx.saps_profile_read()
    copy_gbps = 2 * 4 * X.numel() * cl / (cms * 1e-3) / 1e9
    del scratch
    ctx.saps_profile_enable(False)

    # ---- warm-up
    t = 0
    for _ in range(warm):
        t += 1
        ctx.saps_round(X, G, V, lr, mu, seed, t, peers[t], idx, msg, Ks[t:t + 1])
    ctx.saps_poll_status(check=True)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` rounds, dominant kernel bracketed by HIP events on the same stream
    ctx.saps_profile_enable(True)
    ev0 = torch.cuda.Event(enable_timing=True); ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        t += 1
        ctx.saps_round(X, G, V, lr, mu, seed, t, peers[t], idx, msg, Ks[t:t + 1])
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3
    ev_ms = ev0.elapsed_time(ev1)
    kl, kms = ctx.saps_profile_read()
    st, _ = ctx.saps_poll_status()
    assert st == 0, "capacity overflow during the timed rounds"
    ms_per_step = wall_ms / steps
    Kt = Ks[warm + 1: warm + 1 + steps].cpu().numpy().astype(np.float64)
    K_mean = float(Kt.mean())

    # ---- the same `steps` rounds captured once into a HIP graph and replayed (secondary figure; possible
    # because a round is nothing but kernel launches when the matching fits the kernel arguments)
    graph_ms_per_step = None
    if n <= 128:
        ctx.saps_profile_enable(False)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        t_g = warm
        with torch.cuda.graph(g, stream=stream):
            for _ in range(steps):
                t_g += 1
                ctx.saps_round(X, G, V, lr, mu, seed, t_g, peers[t_g], idx, msg, Ks[t_g:t_g + 1])
        g.replay()
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        graph_ms_per_step = (time.perf_counter() - w0) * 1e3 / steps
        assert ctx.saps_poll_status()[0] == 0
        ctx.saps_profile_enable(True)

    # ---- consensus diagnostics on the final state (outside the timed region)
    D_dev = torch.zeros(1, dtype=torch.float64, device="cuda")
    mean_dev = torch.empty(N, dtype=torch.float32, device="cuda")
    cons_ms = {}
    for label, m_out in (("disagreement_only", None), ("with_mean_output", mean_dev)):
        for _ in range(2):
            ctx.saps_consensus(X, m_out, D_dev)
        ctx.saps_profile_read()
        for _ in range(10):
            ctx.saps_consensus(X, m_out, D_dev)
        dl, dms = ctx.saps_profile_read()
        cons_ms[label] = dms / dl
    consensus = {"disagreement_sum_sq": float(D_dev.item()),
                 "kernel_ms": cons_ms["disagreement_only"],
                 "algorithmic_GBps": 4.0 * n * N / (cons_ms["disagreement_only"] * 1e-3) / 1e9,
                 "kernel_ms_with_mean_output": cons_ms["with_mean_output"],
                 "algorithmic_GBps_with_mean_output": (4.0 * n * N + 4.0 * N) / (cons_ms["with_mean_output"] * 1e-3) / 1e9,
                 "bytes_per_unit": "4 B per worker-coordinate read (+ 4 B per coordinate when the mean is written)"}

    # ---- algorithmic bytes of the dominant kernel per launch
    if wl.fused:
        kernel = "fused_round_kernel (update + mask + compaction + averaging)"
        per = 20.0 if wl.has_buffer else 12.0
        alg_bytes = per * n * N + 4.0 * n * K_mean + 4.0 * K_mean
        bytes_per_unit = ("20 B per worker-coordinate (x,g,v read; x,v written)" if wl.has_buffer else
                          "12 B per worker-coordinate (x,g read; x written)") + " + 4 B per packed value + 4 B per index"
    else:
        kernel = "exchange kernel (index-list gather/average/scatter or tile walk)"
        alg_bytes = 12.0 * n * K_mean + 4.0 * K_mean
        bytes_per_unit = "12 B per worker per kept coordinate (read x, write x, write msg) + 4 B per index"
    k_ms = kms / max(kl, 1)
    achieved = alg_bytes / (k_ms * 1e-3) / 1e9

    # exchange-only rounds touch isolated values, but HBM moves whole lines: bytes of the 128-byte lines
    # read and 32-byte sectors written that hold the last round's kept coordinates, for comparison
    line_bytes = None
    if not wl.fused:
        K_last = int(Ks[warm + steps].item())
        j = idx[:K_last].to(torch.int64) & 0xFFFFFFFF
        lines = int(torch.unique(j >> 5).numel()); sectors = int(torch.unique(j >> 3).numel())
        line_bytes = {"lines_128B_read_per_row": lines, "sectors_32B_written_per_row": sectors,
                      "bytes_per_launch": float(n) * (128.0 * lines + 32.0 * sectors) + 4.0 * n * K_last + 4.0 * K_last}

    # measured HBM bytes per launch of the dominant kernel (rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
    # same command, scaled by the copy kernel of known size; summaries under profiles/)
    traffic = traffic_detail = None
    tf = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tf):
        with open(tf) as f:
            traffic_detail = json.load(f).get(args.workload)
        if traffic_detail:
            traffic = traffic_detail["total_bytes"]

    out = {
        "metric": "model coords/s per SAPS round",
        "value": n * N / (ms_per_step * 1e-3),
        "unit": "model coords/s",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "n_workers": n, "N": N, "ld": ld,
                   "c": sorted(set(wl.seg_c)), "segments": len(wl.seg_sizes),
                   "round": "fused update+exchange" if wl.fused else "exchange only",
                   "lr": lr, "momentum": mu,
                   "matching": "Alg. 3 peer selection (B_thres 50 Mbps, T_thres 10)" if selector else wl.matching,
                   "gradients": "one synthetic draw reused every round" if wl.fused else None,
                   "msg_capacity": cap, "tune": args.tune or "default",
                   "layout": "X|G|V back to back in one device arena, row stride ld"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_detail": traffic_detail,
                     "kernel": kernel, "kernel_ms": k_ms, "kernel_launches": kl,
                     "algorithmic_bytes_per_launch": alg_bytes, "bytes_per_unit": bytes_per_unit,
                     "copy_yardstick_GBps": copy_gbps, "frac_of_copy": achieved / copy_gbps,
                     "line_granular": line_bytes},
        "cpu_baseline": cpu,
        "parity": parity,
        "whole_round_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "event_ms_per_step": ev_ms / steps,
        "graph_replay_ms_per_step": graph_ms_per_step,
        "K_mean": K_mean,
        "consensus": consensus,
        "traffic_per_worker_bytes": {"measured_8K": 8.0 * K_mean, "paper_2N_over_c_x4B": 8.0 * wl.expected_K},
        "paper_context": "Table IV, 32 workers, c=100: SAPS-PSGD reaches its target accuracies with 10/120/80 MB of "
                         "traffic per worker (hardware unnamed); the paper reports no timing for this path",
    }
    ctx.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
