#!/usr/bin/env python3
"""Benchmark of the ClusterKV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: ck_cluster_keys (init, 10 x {assignment, metadata,
update}) followed by one decode step (ck_select_clusters, ck_gather_indices,
ck_sparse_decode_attn).  The default workload is the Llama-3-8B-shaped layer at a
32k context with B = 1024.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBPS = 8000.0             # MI355X HBM3E peak
USE_GRAPHS = True                  # --no-graphs clears it


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_layer_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batch8", action="store_true",
                    help="skip the extra decode-only measurement at batch 8, B=2048")
    ap.add_argument("--no-incremental", action="store_true",
                    help="skip the 1024-step decode loop with incremental clustering (batch 16)")
    ap.add_argument("--no-long-context", action="store_true",
                    help="skip the 128k-context leg (C=1600: K-means + one decode step)")
    ap.add_argument("--no-recall", action="store_true",
                    help="skip the recall-rate curves (cluster vs page selection vs exact top-B)")
    ap.add_argument("--no-offload", action="store_true",
                    help="skip the host-resident K/V leg (cluster cache over pinned host memory)")
    ap.add_argument("--extras", action="store_true",
                    help="also run the clustering-variants leg (metrics, run-until-convergence) "
                         "and the 32-layer driver leg (side-stream clustering, sinks, full-KV "
                         "first layers); off by default so that the default run's kernel trace "
                         "holds only launches of the timed workloads")
    ap.add_argument("--no-full-depth", action="store_true",
                    help="skip the full-depth configuration (all 32 layers x 8 sequences as one "
                         "batch of 2048 head-problems, ~36 GiB of HBM): the decode workload "
                         "on which the HBM roofline fraction is meaningful")
    ap.add_argument("--counter-legs", action="store_true",
                    help="launch each kernel of the timed workloads a few times and nothing else "
                         "(no timing, no JSON figures): the run to put under rocprofv3 --pmc, "
                         "which serialises dispatches and needs few of them")
    ap.add_argument("--no-graphs", action="store_true",
                    help="time the HIP-graph legs as plain launches instead (for runs under a "
                         "counter-collecting profiler, which does not survive graph replays)")
    return ap.parse_args()


def event_ms(fn, reps):
    """Average milliseconds of fn() over reps calls, HIP events on the current stream."""
    import torch
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / reps


def train_stats(fn, reps, trains=7):
    """Several back-to-back trains of `reps` calls, one HIP event pair around each train:
    mean, median and minimum of the per-call time over the trains, in milliseconds."""
    ts = sorted(event_ms(fn, reps) for _ in range(trains))
    return {"mean": sum(ts) / len(ts), "median": ts[len(ts) // 2], "min": ts[0],
            "calls_per_train": reps, "trains": trains}


def per_launch_ms(fn, reps):
    """Average duration of ONE call, each call bracketed by its own event pair."""
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]


def read_clocks():
    """Shader and memory clock as the SMI tool reports them at this moment (MHz), or
    the reason why not.  Called while a long train of kernels is queued on the GPU."""
    import re
    import subprocess
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ):
        # under the profiler every child process loads its tool library, which touches the
        # GPU before the SMI script starts its interpreter; do not start one there
        return {"unavailable": "running under a profiler"}
    for cmd in (["/opt/rocm/bin/rocm-smi", "--showclocks"], ["rocm-smi", "--showclocks"]):
        try:
            out = subprocess.run(cmd, capture_output=True, text=True, timeout=20).stdout
        except Exception as e:                              # tool missing or not permitted
            err = repr(e)
            continue
        clocks = {}
        for name in ("sclk", "mclk", "fclk", "socclk"):
            m = re.search(name + r" clock level:?\s*\S*\s*\((\d+)\s*Mhz\)", out, re.I)
            if m:
                clocks[name + "_MHz"] = int(m.group(1))
        if clocks:
            return clocks
        err = "no clock lines in the tool's output"
    return {"unavailable": err}


def decode_bytes(cfg, st, C):
    """Algorithmic HBM bytes of one decode step, from the actual recalled counts."""
    n_tok = st.n_tokens.cpu().numpy().astype("int64")
    n_sel = st.n_sel_clusters.cpu().numpy().astype("int64")
    hp = n_tok.size
    d, G = cfg.d, cfg.G
    select = hp * (C * d * 2 + C * 4 + G * d * 2) + hp * C * 4
    gather = int(n_sel.sum()) * 4 * 2 + int(n_tok.sum()) * 4 * 2
    attn = int(n_tok.sum()) * (d * 2 * 2 + 4) + hp * G * d * 2 * 2
    kv = int(n_tok.sum()) * d * 2 * 2
    return dict(select=select, gather=gather, attn=attn, total=select + gather + attn, kv=kv,
                mean_tokens=float(n_tok.mean()))


def _np64(t):
    import numpy as np
    return t.float().cpu().numpy().astype(np.float64)


def _selection_gaps(r):
    """Smallest gap between neighbours of the score order up to and across the recall
    boundary of one oracle decode step (absolute, in score units)."""
    import numpy as np
    sc = r["scores"][r["order"]]
    hi = min(r["n_sel"] + 1, len(sc))
    return float(np.min(sc[:hi - 1] - sc[1:hi])) if hi > 1 else float("inf")


def cpu_baseline(cfg, w, init, q, budget_s=12.0):
    """The oracle, as it stands, on the host cores: whole head-problems of the
    workload (full K-means + metadata + one decode step each) until about
    budget_s seconds of CPU time are spent.  Also counts, on what it computes, the
    near-tie cases in which the integer outputs may legitimately differ."""
    import numpy as np
    from oracle import clusterkv_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    done = 0
    t_km = t_dec = 0.0
    near_keys = all_keys = near_sel_rel = near_sel_abs = 0
    t_start = time.perf_counter()
    for hp in range(cfg.S * cfg.Hkv):
        s, h = divmod(hp, cfg.Hkv)
        keys = _np64(w.K[s, h, :cfg.N])
        vals = _np64(w.V[s, h, :cfg.N])
        qg = _np64(q[s, h * cfg.G:(h + 1) * cfg.G])
        t0 = time.perf_counter()
        mu, labels, sizes, tr = O.kmeans(keys, init[s, h].numpy(), cfg.n_iter, "bf16")
        sizes, offsets, sidx = O.build_metadata(labels, cfg.C)
        t1 = time.perf_counter()
        r = O.decode_step(qg, keys, vals, O.round_to_bf16(mu), sizes, offsets, sidx, cfg.B)
        t2 = time.perf_counter()
        t_km += t1 - t0
        t_dec += t2 - t1
        done += 1
        near_keys += int(sum((g < 1e-4).sum() for g in tr.gap))
        all_keys += cfg.n_iter * cfg.N
        near_sel_rel += int(O.selection_near_tie(r["scores"], r["order"], r["n_sel"]))
        near_sel_abs += int(_selection_gaps(r) < 1e-4)
        if time.perf_counter() - t_start > budget_s:
            break
    return {"value": done * cfg.N / (t_km + t_dec), "unit": "keys/s", "cores": int(threads),
            "host_cpu_count": os.cpu_count(), "kind": "oracle",
            "sample": f"{done} of {cfg.S * cfg.Hkv} head-problems of {cfg.name}: {cfg.n_iter}-iteration "
                      f"K-means over {cfg.N} keys (C={cfg.C}) + metadata + one decode step each",
            "kmeans_s_per_head_problem": t_km / done,
            "decode_step_s_per_head_problem": t_dec / done,
            "near_tie_rates": {
                "assignment_keys_top2_cosine_gap_below_1e-4": near_keys / max(all_keys, 1),
                "selection_steps_relative_band_1e-4(1+|s|)": near_sel_rel / done,
                "selection_steps_absolute_gap_below_1e-4": near_sel_abs / done,
                "head_problem_steps_counted": done}}


def cpu_baseline_other_configs(budget_s=12.0):
    """The oracle on the other configurations, each on a bounded sample: the tiny one
    whole; the 128k context on a few K-means iterations of one head (extrapolated to ten);
    full depth and incremental decode share the 32k layer's K-means shape, so only
    their decode steps are timed (16 sampled head-problems each)."""
    import numpy as np
    import torch
    from ck_synth import Config, MixtureWorkload, get_config, sample_init_indices
    from oracle import clusterkv_oracle as O
    out = {}
    # ---- tiny, whole
    cfg = get_config(0)
    w = MixtureWorkload(cfg, device="cpu")
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    q = w.query()
    t0 = time.perf_counter()
    for hp in range(cfg.S * cfg.Hkv):
        s, h = divmod(hp, cfg.Hkv)
        keys, vals = _np64(w.K[s, h]), _np64(w.V[s, h])
        mu, labels, sizes, _ = O.kmeans(keys, init[s, h].numpy(), cfg.n_iter, "bf16")
        sizes, offsets, sidx = O.build_metadata(labels, cfg.C)
        O.decode_step(_np64(q[s, h * cfg.G:(h + 1) * cfg.G]), keys, vals, O.round_to_bf16(mu),
                      sizes, offsets, sidx, cfg.B)
    dt = time.perf_counter() - t0
    out[cfg.name] = {"keys_per_s": cfg.S * cfg.Hkv * cfg.N / dt, "seconds": dt,
                     "sample": "all head-problems, K-means + one decode step"}
    # ---- 128k context: one head, two iterations, scaled to ten
    cfg = get_config(3)
    one = Config("long_one_head", 1, 1, 1, cfg.G, cfg.d, cfg.N, cfg.M, cfg.C, 2, cfg.B, cfg.seed)
    w = MixtureWorkload(one, device="cpu")
    init = sample_init_indices(w.K, one.C, one.seed)
    keys = _np64(w.K[0, 0])
    t0 = time.perf_counter()
    O.kmeans(keys, init[0, 0].numpy(), 2, "bf16")
    dt = time.perf_counter() - t0
    out[cfg.name] = {"kmeans_s_per_head_problem_extrapolated": dt * cfg.n_iter / 2,
                     "keys_per_s_extrapolated": cfg.N / (dt * cfg.n_iter / 2),
                     "sample": "1 of 8 head-problems, 2 of 10 K-means iterations, time scaled x5"}
    # ---- decode steps at B = 2048 (full depth) and with a recent window (incremental)
    for idx, recent in ((2, 0), (4, 160)):
        cfg = get_config(idx)
        one = Config("sample", 1, 2, cfg.Hkv, cfg.Hq, cfg.d, cfg.N, cfg.M, cfg.C, 1, cfg.B,
                     cfg.seed)
        w = MixtureWorkload(one, device="cpu", extra_tokens=recent)
        for _ in range(recent):
            w.append_token()
        q = w.query()
        rng = np.random.default_rng(idx)
        t_dec = 0.0
        n = 0
        for hp in range(one.S * one.Hkv):                    # 16 head-problems
            s, h = divmod(hp, one.Hkv)
            keys, vals = _np64(w.K[s, h]), _np64(w.V[s, h])
            # a stand-in clustering (random labels): the decode step's cost does not
            # depend on how good the clusters are
            labels = rng.integers(0, cfg.C, cfg.N)
            sizes, offsets, sidx = O.build_metadata(labels, cfg.C)
            mu, _ = O.update(keys[:cfg.N], labels, np.zeros((cfg.C, cfg.d)))
            t0 = time.perf_counter()
            O.decode_step(_np64(q[s, h * cfg.G:(h + 1) * cfg.G]), keys, vals, O.round_to_bf16(mu),
                          sizes, offsets, sidx, cfg.B, recent_begin=cfg.N,
                          recent_end=cfg.N + recent)
            t_dec += time.perf_counter() - t0
            n += 1
        out[cfg.name] = {"decode_step_s_per_head_problem": t_dec / n,
                         "decode_step_s_whole_config_extrapolated":
                             t_dec / n * cfg.head_problems * cfg.decode_steps,
                         "kmeans": "same shape per head-problem as llama3_8b_layer_32k: see "
                                   "kmeans_s_per_head_problem there, times "
                                   f"{cfg.head_problems} head-problems",
                         "sample": f"{n} head-problems with random cluster labels, one decode "
                                   f"step each (B={cfg.B}, {recent} unclustered recent tokens)"}
    return out


def counter_legs(cfg, w, st, sh, q, cluster, decode):
    """A 1 GiB device copy (the calibration of the byte counters), then three launches of
    every kernel of the 32k layer (clustering, the assignment alone, the decode step, the
    attention alone) and of the batch-8 layer (64 head-problems, B = 2048)."""
    import torch
    import paper_2412_03213_amd as ck
    from ck_synth import Config, MixtureWorkload, get_config, sample_init_indices
    dev = "cuda:0"
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst

    def legs(cfg, w, st, sh, q, cluster, decode):
        HP = cfg.S * cfg.Hkv
        for _ in range(3):
            cluster()
        mu_hat = st.cluster_ws[:HP * cfg.C * cfg.d * 2].view(torch.bfloat16).view(
            cfg.S, cfg.Hkv, cfg.C, cfg.d)
        labels2 = torch.empty_like(st.labels)
        for _ in range(3):
            ck.ck_kmeans_assign(sh, w.K, 0, cfg.N, mu_hat, 0, cfg.C, labels2)
        for _ in range(3):
            decode()
        for _ in range(3):
            ck.ck_sparse_decode_attn(sh, q, w.K, w.V, st.token_idx, st.n_tokens, cfg.B, st.out,
                                     workspace=st.attn_ws)
        torch.cuda.synchronize()

    legs(cfg, w, st, sh, q, cluster, decode)
    c2 = get_config(2)
    cfg8 = Config("batch8_layer", 1, c2.S, c2.Hkv, c2.Hq, c2.d, c2.N, c2.M, c2.C, c2.n_iter, c2.B,
                  c2.seed)
    w8 = MixtureWorkload(cfg8, device=dev)
    w8.token_center = None
    init8 = sample_init_indices(w8.K, cfg8.C, cfg8.seed).to(dev)
    sh8 = ck.Shape(cfg8.S, cfg8.Hq, cfg8.Hkv, cfg8.N, cfg8.C)
    st8 = ck.ClusterState(sh8, dev, budget=cfg8.B)
    q8 = w8.query()

    def cluster8():
        st8.n_clusters = 0
        st8.cluster(w8.K, init8, 0, cfg8.N, cfg8.C, cfg8.n_iter)

    legs(cfg8, w8, st8, sh8, q8, cluster8, lambda: ck.decode_step(st8, q8, w8.K, w8.V))
    print(json.dumps({"counter_legs": "done", "workloads": [cfg.name, "batch-8 layer (64 "
                      "head-problems, N=32768, C=400, B=2048)"]}))


def graph_ms(fn, reps, per_graph=1):
    """`per_graph` consecutive calls of fn (the layers of a model run one after another)
    captured into one HIP graph; average time per call over `reps` replays."""
    import torch
    if not USE_GRAPHS:
        return event_ms(fn, reps)
    one = fn

    def fn():
        for _ in range(per_graph):
            one()
    reps = max(reps // per_graph, 5)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    for _ in range(5):
        g.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        g.replay()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / reps / per_graph


def measured_peaks(dev):
    """What the chip sustains in the simplest possible kernels: a register-only bf16
    MFMA loop, once with constant operands and once with random ones (the clock the chip
    holds under matrix load depends on how many operand bits toggle: the random-operand
    figure is the one that bounds a kernel working on real keys), and a device copy."""
    import torch
    import paper_2412_03213_amd as ck
    sink = torch.zeros(4, device=dev)
    clocks = torch.zeros(2, dtype=torch.int64, device=dev)
    g = torch.Generator(device=dev).manual_seed(11)
    rnd = torch.randn(64 * 16 * 8, generator=g, device=dev).to(torch.bfloat16).contiguous()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = {}
    for tag, operands in (("constant_operands", None), ("random_operands", rnd)):
        ck.ck_probe_mfma_bf16(1024, 200, sink, operands, clocks)
        torch.cuda.synchronize()
        a.record()
        fl = ck.ck_probe_mfma_bf16(1024, 4000, sink, operands, clocks)
        b.record()
        b.synchronize()
        cyc, tick = (int(x) for x in clocks.cpu())
        out["mfma_bf16_TFLOPs_register_loop_" + tag] = fl / (a.elapsed_time(b) * 1e-3) / 1e12
        out["shader_MHz_in_loop_" + tag] = cyc / max(tick, 1) * 100.0
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    a.record()
    for _ in range(5):
        dst.copy_(src)
    b.record()
    b.synchronize()
    out["copy_GBps_read_plus_write"] = 5 * 2 * src.numel() / (a.elapsed_time(b) * 1e-3) / 1e9
    out["note"] = ("register-only MFMA loops (4 independent accumulators per wavefront, 8 "
                   "wavefronts per compute unit) and a 1 GiB device copy: what the simplest "
                   "possible kernels sustain on this chip; the shader clock is read inside the "
                   "loop (cycle counter over the 100 MHz counter)")
    return out


def read_traffic(kernel, workload):
    """HBM bytes per launch of a kernel on a workload as measured with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE, calibrated), from the committed summary if present."""
    path = os.path.join(ROOT, "profiles", "k_assign_stream_and_k_attn_pmc.md")
    tag = f"traffic_bytes_per_launch[{kernel}, {workload}]:"
    try:
        for line in open(path):
            if line.startswith(tag):
                return float(line[len(tag):])
    except OSError:
        pass
    return None


def main():
    global USE_GRAPHS
    args = parse()
    USE_GRAPHS = not args.no_graphs
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (head-problems are independent; "
              "no multi-GPU path exists) -- rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2412_03213_amd as ck
    from ck_synth import MixtureWorkload, get_config, sample_init_indices

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    cfg = get_config(args.workload)
    if cfg.layers != 1:
        print("bench.py: pick a single-layer workload", file=sys.stderr)
        sys.exit(2)
    w = MixtureWorkload(cfg, device=dev)
    init = sample_init_indices(w.K, cfg.C, cfg.seed)
    init_d = init.to(dev)
    q = w.query()
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, dev, budget=cfg.B)
    HP = cfg.S * cfg.Hkv

    def cluster():
        st.n_clusters = 0
        st.cluster(w.K, init_d, 0, cfg.N, cfg.C, cfg.n_iter)

    def decode():
        ck.decode_step(st, q, w.K, w.V)

    def step():
        cluster()
        decode()

    if args.counter_legs:
        counter_legs(cfg, w, st, sh, q, cluster, decode)
        return
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    keys_per_step = HP * cfg.N

    # ---- parts of the step, HIP events on the launch stream ----
    reps = max(args.steps, 10)
    cluster_st = train_stats(cluster, reps)
    cluster_ms = cluster_st["mean"]
    decode_st = train_stats(decode, 10 * reps)
    decode_ms = decode_st["mean"]
    decode_graph_ms = graph_ms(decode, 10 * reps, per_graph=32)     # 32 steps per replay
    db = decode_bytes(cfg, st, cfg.C)

    # dominant kernel: the MFMA assignment, one launch at a time
    ws = st.cluster_ws
    n_hat = HP * cfg.C * cfg.d
    mu_hat = ws[:n_hat * 2].view(torch.bfloat16).view(cfg.S, cfg.Hkv, cfg.C, cfg.d)
    labels2 = torch.empty_like(st.labels)

    def assign():
        ck.ck_kmeans_assign(sh, w.K, 0, cfg.N, mu_hat, 0, cfg.C, labels2)

    for _ in range(3):
        assign()
    a_avg, a_med, a_min = per_launch_ms(assign, 10 * reps)
    assign_flops = 2.0 * HP * cfg.N * cfg.C * cfg.d
    a_st = train_stats(assign, 10 * reps)       # back-to-back launches, one event pair per train
    a_train = a_st["mean"]
    achieved_tflops = assign_flops / (a_train * 1e-3) / 1e12
    # clocks while the assignment kernel runs: queue about two seconds of launches, ask the
    # SMI tool, then drain
    for _ in range(int(2000.0 / a_train)):
        assign()
    clocks = read_clocks()
    torch.cuda.synchronize()
    # the same launch on constant data (all keys and all centroids the same vector): same
    # instruction stream, far fewer operand bits toggling, so a higher clock under load
    K_flat = torch.ones_like(w.K)
    hat_flat = torch.full_like(mu_hat, 128.0 ** -0.5)

    def assign_flat():
        ck.ck_kmeans_assign(sh, K_flat, 0, cfg.N, hat_flat, 0, cfg.C, labels2)

    for _ in range(3):
        assign_flat()
    a_flat = train_stats(assign_flat, 10 * reps)["mean"]
    del K_flat, hat_flat

    # sparse attention alone (partial + merge kernels of one call)
    def attn():
        ck.ck_sparse_decode_attn(sh, q, w.K, w.V, st.token_idx, st.n_tokens, cfg.B, st.out,
                                 workspace=st.attn_ws)

    at_avg, at_med, at_min = per_launch_ms(attn, 10 * reps)

    # the computation the path approximates: decode attention over the whole KV cache
    full_out = torch.empty_like(st.out)
    full_ws = torch.empty(ck.ck_workspace_bytes(sh, 1, cfg.N), dtype=torch.uint8, device=dev)

    def full_attn():
        ck.ck_full_decode_attn(sh, q, w.K, w.V, cfg.N, full_out, workspace=full_ws)

    for _ in range(3):
        full_attn()
    full_ms = event_ms(full_attn, 5 * reps)
    full_bytes = 2.0 * HP * cfg.N * cfg.d * 2

    result = {
        "metric": "decode us/layer & recalled-KV GB/s at 32k ctx, B=1024; K-means keys/s",
        "value": keys_per_step / (ms_per_step * 1e-3),
        "unit": "keys/s (K-means over all keys + one decode step, whole step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "S": cfg.S, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "d": cfg.d,
                   "N": cfg.N, "C": cfg.C, "kmeans_iters": cfg.n_iter, "B": cfg.B,
                   "mixture_centers": cfg.M, "selection": "whole clusters"},
        "kmeans_keys_per_s": keys_per_step / (cluster_ms * 1e-3),
        "kmeans_key_assignments_per_s": keys_per_step * cfg.n_iter / (cluster_ms * 1e-3),
        "kmeans_ms": cluster_ms, "kmeans_ms_median": cluster_st["median"],
        "kmeans_ms_min": cluster_st["min"],
        "decode_us_per_layer": decode_ms * 1e3,
        "decode_us_per_layer_median": decode_st["median"] * 1e3,
        "decode_us_per_layer_min": decode_st["min"] * 1e3,
        "decode_us_per_layer_hipgraph": decode_graph_ms * 1e3,
        "decode_us_per_layer_best": min(decode_ms, decode_graph_ms) * 1e3,
        "hipgraph_note": "the SAME layer's decode step 32 times per graph replay: its recalled "
                         "rows stay in the caches between steps (warm).  The per-layer time "
                         "over 32 DISTINCT layers is decode_full_depth_32layers."
                         "distinct_layers_batch1 / _batch8",
        "clocks_during_assignment_train": clocks,
        "recalled_kv_GBps": db["kv"] / (decode_ms * 1e-3) / 1e9,
        "recalled_tokens_mean": db["mean_tokens"],
        "roofline": {"kernel": "k_assign_stream (bf16 MFMA assignment, centroid table in LDS; "
                               "one launch = one K-means iteration over all head-problems)",
                     "bound": "mfma", "achieved": achieved_tflops, "peak": PEAK_BF16_MFMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved_tflops / PEAK_BF16_MFMA_TFLOPS,
                     "traffic": read_traffic("k_assign_stream", cfg.name),
                     "flops_per_launch": assign_flops,
                     "launch_ms_avg": a_train, "launch_ms_median": a_st["median"],
                     "launch_ms_min": a_st["min"],
                     "launch_ms_avg_note": "average over a back-to-back train of launches between "
                                           "one HIP event pair; a pair around every single launch "
                                           "adds ~3 us of dispatch latency",
                     "launch_ms_single_pair_avg": a_avg, "launch_ms_single_pair_min": a_min,
                     "launch_ms_avg_constant_data": a_flat,
                     "constant_data_note": "the same launch with every key and every centroid "
                                           "the same vector: identical instruction stream; the "
                                           "difference is the clock the chip holds under matrix "
                                           "load (see measured_peaks: random against constant "
                                           "operands)"},
        "roofline_decode": {"kernels": "ck_decode_step = one launch of k_attn (scoring, "
                                       "selection, gather, attention; the last workgroup of a "
                                       "head-problem merges its splits)",
                            "bound": "hbm", "achieved": db["total"] / (decode_ms * 1e-3) / 1e9,
                            "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": db["total"] / (decode_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                            "bytes_per_step": db["total"],
                            "traffic": read_traffic("k_attn", cfg.name),
                            "attn_call_us_avg": at_avg * 1e3,
                            "attn_GBps": db["attn"] / (at_avg * 1e-3) / 1e9,
                            "note": "batch 1: 8 head-problems, latency bound (a chain of "
                                    "dependent memory round trips, 5 MB per step)"},
    }

    result["full_kv_decode"] = {
        "us_per_layer": full_ms * 1e3, "GBps": full_bytes / (full_ms * 1e-3) / 1e9,
        "frac_of_hbm_peak": full_bytes / (full_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "speedup_of_compressed_decode": full_ms / decode_ms,
        "note": "ck_full_decode_attn over all N tokens of the same layer (split-KV + merge)"}
    if not args.no_recall:
        result["recall_rate"] = recall_curves(cfg, w, st, sh)
    if args.extras:
        result["kmeans_variants"] = kmeans_variants(cfg, w, init_d, reps)
        result["recall_vs_cluster_count"] = recall_vs_clusters(cfg, w)
    if args.extras:
        result["layer_stack_32"] = layer_stack(cfg, w, init_d)
    if not args.no_offload:
        result["offloaded_kv_cluster_cache"] = [offloaded_kv(cfg, w, st, sh, sticky=p)
                                                for p in (0.8, 0.95)]
    result["measured_peaks"] = measured_peaks(dev)
    if not args.no_batch8:
        result["decode_batch8_B2048"] = big_decode(reps, layers=1)
    if not args.no_long_context:
        result["long_context_128k"] = long_context(reps)
    if not args.no_incremental:
        result["incremental_decode_b16"] = incremental_decode()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, w, init, q)
        result["cpu_baseline"]["other_configs"] = cpu_baseline_other_configs()
    if not args.no_full_depth:
        del w, st
        torch.cuda.empty_cache()
        fd = big_decode(max(reps // 2, 5), layers=32)
        result["decode_full_depth_32layers"] = fd
        # the per-layer decode figures over distinct layers, next to the headline fields
        result["decode_us_per_layer_distinct_layers_batch1"] = \
            fd["distinct_layers_batch1"]["decode_us_per_layer"]
        result["decode_us_per_layer_distinct_layers_batch8"] = \
            fd["distinct_layers_batch8"]["decode_us_per_layer"]
    # a plain copy of known size: lets a rocprofv3 --pmc run of this script calibrate
    # FETCH_SIZE / WRITE_SIZE (256 MiB read + 256 MiB written)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps(result))


def recall_curves(cfg, w, st, sh, n_queries=8, page_size=16, budgets=None, with_pages=True):
    """Recall rate |I_T & I_true| / B against the exact top-B tokens (by summed q.k of the
    group), averaged over head-problems and queries, for budgets 256..2048: the cluster
    selection of the clustered state `st` in both budget modes, and the page-granular
    selector.  All selections, the exact top-B and the hit counts run in the library."""
    import torch
    import paper_2412_03213_amd as ck
    dev = w.K.device
    HP, N = cfg.S * cfg.Hkv, cfg.N
    budgets = budgets or list(range(256, 2049, 256))
    n_pages = (N + page_size - 1) // page_size
    pk = torch.empty(cfg.S, cfg.Hkv, n_pages, cfg.d, dtype=w.K.dtype, device=dev)
    ck.ck_page_keys(sh, w.K, 0, N, page_size, pk)
    shp = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, n_pages, sh.C_cap)
    tscore = torch.empty(cfg.S, cfg.Hkv, N, dtype=torch.float32, device=dev)
    pscore = torch.empty(cfg.S, cfg.Hkv, n_pages, dtype=torch.float32, device=dev)
    cscore = torch.empty(cfg.S, cfg.Hkv, sh.C_cap, dtype=torch.float32, device=dev)
    sel = torch.empty(cfg.S, cfg.Hkv, sh.C_cap, dtype=torch.int32, device=dev)
    nsel = torch.empty(HP, dtype=torch.int32, device=dev)
    nseltok = torch.empty(HP, dtype=torch.int32, device=dev)
    ntok = torch.empty(HP, dtype=torch.int32, device=dev)
    nref = torch.empty(HP, dtype=torch.int32, device=dev)
    npg = torch.empty(HP, dtype=torch.int32, device=dev)
    hits = torch.empty(HP, dtype=torch.int32, device=dev)
    acc = {"clusterkv_trim_last": [0.0] * len(budgets), "clusterkv_whole": [0.0] * len(budgets),
           f"page{page_size}": [0.0] * len(budgets)}
    if not with_pages:
        del acc[f"page{page_size}"]
    for _ in range(n_queries):
        q = w.query()
        ck.ck_token_scores(sh, q, w.K, 0, N, tscore)
        ck.ck_token_scores(shp, q, pk, 0, n_pages, pscore)
        for bi, B in enumerate(budgets):
            ref = torch.empty(HP, B, dtype=torch.int32, device=dev)
            tok = torch.empty(HP, B, dtype=torch.int32, device=dev)
            ck.ck_topk_select(HP, tscore, N, 0, N, B, ref, nref)
            for name, mode in (("clusterkv_trim_last", ck.CK_SEL_TRIM_LAST),
                               ("clusterkv_whole", ck.CK_SEL_WHOLE)):
                ck.ck_select_clusters(sh, q, st.centroids, st.sizes, st.n_clusters, B, mode, sel,
                                      nsel, nseltok, cscore)
                ck.ck_gather_indices(sh, sel, nsel, st.offsets, st.sorted_idx, B, mode, tok, ntok)
                ck.ck_recall_hits(HP, tok, ntok, ref, nref, hits)
                acc[name][bi] += float(hits.sum()) / (HP * B)
            if not with_pages:
                continue
            pidx = torch.empty(HP, B // page_size, dtype=torch.int32, device=dev)
            ck.ck_topk_select(HP, pscore, n_pages, 0, n_pages, B // page_size, pidx, npg)
            ck.ck_expand_pages(HP, pidx, npg, page_size, 0, N, tok, ntok)
            ck.ck_recall_hits(HP, tok, ntok, ref, nref, hits)
            acc[f"page{page_size}"][bi] += float(hits.sum()) / (HP * B)
    out = {"budgets": budgets, "queries": n_queries, "head_problems": HP,
           "note": "synthetic mixture keys; I_true = exact top-B by the group's summed q.k; "
                   "trim_last recalls exactly B tokens, whole clusters at most B"}
    for k, v in acc.items():
        out[k] = [round(x / n_queries, 4) for x in v]
    return out


def recall_vs_clusters(cfg, w, counts=(100, 200, 400, 800), budget=1024):
    """Recall rate at a fixed budget against the number of prefill clusters C0 (the
    ablation of Section V-B): the layer is clustered anew for every C0; selections, exact
    top-B and hit counts run in the library as for the other curves."""
    import paper_2412_03213_amd as ck
    from ck_synth import sample_init_indices
    dev = w.K.device
    out = {"budget": budget, "clusters": list(counts), "clusterkv_trim_last": [],
           "clusterkv_whole": [], "kmeans_ms": []}
    for C0 in counts:
        sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, C0)
        st = ck.ClusterState(sh, dev, budget=budget)
        init = sample_init_indices(w.K, C0, cfg.seed + C0).to(dev)

        def cluster():
            st.n_clusters = 0
            st.cluster(w.K, init, 0, cfg.N, C0, cfg.n_iter)

        cluster()
        out["kmeans_ms"].append(event_ms(cluster, 3))
        rc = recall_curves(cfg, w, st, sh, n_queries=4, budgets=[budget], with_pages=False)
        out["clusterkv_trim_last"].append(rc["clusterkv_trim_last"][0])
        out["clusterkv_whole"].append(rc["clusterkv_whole"][0])
    return out


def kmeans_variants(cfg, w, init_d, reps):
    """The clustering options beside the default: assignment metric (time of the fixed
    10-iteration run and recall at the configured budget) and the run-until-convergence
    loop (iterations each head-problem took, time of the whole call)."""
    import torch
    import paper_2412_03213_amd as ck
    dev = w.K.device
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    out = {}
    for name, flag in (("cosine", ck.CK_METRIC_COSINE), ("l2", ck.CK_METRIC_L2),
                       ("inner_product", ck.CK_METRIC_IP)):
        st = ck.ClusterState(sh, dev, budget=cfg.B)

        def cluster():
            st.n_clusters = 0
            st.cluster(w.K, init_d, 0, cfg.N, cfg.C, cfg.n_iter, flags=flag)

        cluster()
        ms = event_ms(cluster, max(3, reps // 4))
        rc = recall_curves(cfg, w, st, sh, n_queries=4, budgets=[cfg.B], with_pages=False)
        out[name] = {"kmeans_ms": ms, f"recall_at_B{cfg.B}_trim_last": rc["clusterkv_trim_last"][0]}
    st = ck.ClusterState(sh, dev, budget=cfg.B)
    iters = torch.zeros(cfg.S, cfg.Hkv, dtype=torch.int32, device=dev)
    cap = 100

    def converge():
        st.n_clusters = 0
        st.cluster(w.K, init_d, 0, cfg.N, cfg.C, cap, flags=ck.CK_KM_UNTIL_CONVERGED,
                   iters_done=iters)

    converge()
    ms = event_ms(converge, 3)
    it = iters.flatten().cpu().tolist()
    out["until_converged_cosine"] = {"cap": cap, "iterations_min": min(it),
                                     "iterations_mean": sum(it) / len(it),
                                     "iterations_max": max(it), "kmeans_ms": ms}
    return out


def offloaded_kv(cfg, w, st, sh, steps=64, sticky=0.8):
    """K/V home copy in pinned host memory, read by the GPU itself over the host link;
    decode steps with the cluster cache (R = 1) and, for comparison, with the cache emptied
    before every step (every recalled row crosses the link).  Queries keep their target
    center between steps with probability `sticky`."""
    import torch
    import paper_2412_03213_amd as ck
    dev = w.K.device
    HP = cfg.S * cfg.Hkv
    Kh = torch.empty(w.K.shape, dtype=w.K.dtype, pin_memory=True)
    Vh = torch.empty(w.V.shape, dtype=w.V.dtype, pin_memory=True)
    Kh.copy_(w.K)
    Vh.copy_(w.V)
    torch.cuda.synchronize()
    K_home, V_home = ck.ck_host_device_ptr(Kh), ck.ck_host_device_ptr(Vh)
    cache = ck.ClusterCache(sh, dev, cap_tokens=cfg.B)
    qs = [w.query(sticky=sticky) for _ in range(steps)]
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def run(with_cache):
        ck.ck_cache_reset(sh, cache)
        miss = torch.zeros(HP, dtype=torch.int64, device=dev)
        tok = torch.zeros(HP, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        a.record()
        for q in qs:
            if not with_cache:
                ck.ck_cache_reset(sh, cache)
            ck.cached_decode_step(st, cache, q, K_home, V_home)
            miss += cache.miss_tokens.view(HP)
            tok += st.n_sel_tokens.view(HP)
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / len(qs), int(miss.sum()), int(tok.sum())

    run(True)
    ms_c, miss_c, tok_c = run(True)
    ms_n, miss_n, tok_n = run(False)
    row = 2 * cfg.d * w.K.element_size()
    return {"workload": f"{cfg.name}, K/V home in pinned host memory, {steps} steps, "
                        f"query center kept with p={sticky}",
            "cached_us_per_step": ms_c * 1e3, "uncached_us_per_step": ms_n * 1e3,
            "speedup_from_cache": ms_n / ms_c,
            "hit_rate_tokens": 1.0 - miss_c / max(tok_c, 1),
            "host_link_GBps_cached": miss_c * row / len(qs) / (ms_c * 1e-3) / 1e9,
            "host_link_GBps_uncached": miss_n * row / len(qs) / (ms_n * 1e-3) / 1e9,
            "note": "the hit rate is a property of the synthetic query stream, not of real "
                    "attention; times include two small bookkeeping adds per step"}


def layer_stack(cfg, w, init_d, n_layers=32):
    """The paper's serving arrangement on one sequence: 32 layers, 16 attention sinks, the
    first two layers on the full KV cache, prefill clustering of every layer on a side
    stream while a stand-in for the layer's dense work (one [N x 4096] x [4096 x 14336] bf16
    GEMM) runs on the main stream.  All layers share one synthetic K/V (same shapes, same
    work; only the memory is saved)."""
    import torch
    import paper_2412_03213_amd as ck
    dev = w.K.device
    stack = ck.LayerStack(n_layers, cfg.S, cfg.Hq, cfg.Hkv, cfg.N, 0, cfg.C, cfg.B, dev,
                          n_sink=16, full_kv_layers=2, n_iter=cfg.n_iter)
    sink_init = init_d.clamp(min=16)
    x = torch.randn(cfg.N, 4096, device=dev, dtype=torch.bfloat16)
    wt = torch.randn(4096, 14336, device=dev, dtype=torch.bfloat16)
    y = torch.empty(cfg.N, 14336, device=dev, dtype=torch.bfloat16)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        torch.cuda.current_stream().wait_stream(stack.side)
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps

    def dense_only():
        for _ in range(n_layers):
            torch.matmul(x, wt, out=y)

    def overlapped():
        for l in range(n_layers):
            torch.matmul(x, wt, out=y)
            stack.cluster_prefill(l, w.K, sink_init)

    def serial():
        for l in range(n_layers):
            torch.matmul(x, wt, out=y)
            if stack.compressed(l):
                st = stack.states[l]
                st.n_clusters = 0
                st.cluster(w.K, sink_init, 16, cfg.N - 16, cfg.C, cfg.n_iter)

    t_dense, t_over, t_serial = timed(dense_only), timed(overlapped), timed(serial)
    q = w.query()

    def decode_policy():
        for l in range(n_layers):
            stack.decode(l, q, w.K, w.V, cfg.N)

    def decode_full():
        for l in range(n_layers):
            ck.ck_full_decode_attn(stack.sh, q, w.K, w.V, cfg.N, stack.full_out,
                                   workspace=stack.full_ws)

    d_pol, d_full = timed(decode_policy, 20), timed(decode_full, 20)
    return {"workload": f"{n_layers} layers x {cfg.name}, 16 sinks, first 2 layers full KV",
            "prefill_dense_standin_ms": t_dense,
            "prefill_with_clustering_on_side_stream_ms": t_over,
            "prefill_with_clustering_in_line_ms": t_serial,
            "clustering_overhead_hidden_frac":
                1.0 - (t_over - t_dense) / max(t_serial - t_dense, 1e-9),
            "decode_attention_us_per_token_policy": d_pol * 1e3,
            "decode_attention_us_per_token_full_kv": d_full * 1e3,
            "decode_attention_speedup": d_full / d_pol}


def long_context(reps):
    """The 128k-context configuration (C = 1600 clusters, B = 2048): K-means, the
    assignment kernel's MFMA fraction at this cluster count, and one decode step."""
    import torch
    import paper_2412_03213_amd as ck
    from ck_synth import MixtureWorkload, get_config, sample_init_indices
    cfg = get_config(3)
    dev = "cuda:0"
    w = MixtureWorkload(cfg, device=dev)
    w.token_center = None
    init = sample_init_indices(w.K, cfg.C, cfg.seed).to(dev)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, dev, budget=cfg.B)
    HP = cfg.S * cfg.Hkv

    def cluster():
        st.n_clusters = 0
        st.cluster(w.K, init, 0, cfg.N, cfg.C, cfg.n_iter)

    cluster()
    km = event_ms(cluster, 3)
    mu_hat = st.cluster_ws[:HP * cfg.C * cfg.d * 2].view(torch.bfloat16).view(
        cfg.S, cfg.Hkv, cfg.C, cfg.d)
    labels2 = torch.empty_like(st.labels)

    def assign():
        ck.ck_kmeans_assign(sh, w.K, 0, cfg.N, mu_hat, 0, cfg.C, labels2)

    for _ in range(3):
        assign()
    a_ms = event_ms(assign, 2 * reps)
    flops = 2.0 * HP * cfg.N * cfg.C * cfg.d
    q = w.query()

    def decode():
        ck.decode_step(st, q, w.K, w.V)

    for _ in range(5):
        decode()
    d_ms = event_ms(decode, 10 * reps)
    db = decode_bytes(cfg, st, cfg.C)
    tf = flops / (a_ms * 1e-3) / 1e12
    full_out = torch.empty_like(st.out)
    full_ws = torch.empty(ck.ck_workspace_bytes(sh, 1, cfg.N), dtype=torch.uint8, device=dev)

    def full_attn():
        ck.ck_full_decode_attn(sh, q, w.K, w.V, cfg.N, full_out, workspace=full_ws)

    for _ in range(3):
        full_attn()
    f_ms = event_ms(full_attn, 2 * reps)
    return {"workload": f"{cfg.name}: N={cfg.N}, C={cfg.C}, B={cfg.B}, {HP} head-problems",
            "full_kv_decode_us": f_ms * 1e3,
            "full_kv_GBps": 2.0 * HP * cfg.N * cfg.d * 2 / (f_ms * 1e-3) / 1e9,
            "speedup_of_compressed_decode": f_ms / d_ms,
            "kmeans_ms": km, "kmeans_keys_per_s": HP * cfg.N / (km * 1e-3),
            "roofline_assign": {"bound": "mfma", "achieved": tf, "peak": PEAK_BF16_MFMA_TFLOPS,
                                "unit": "TFLOP/s", "frac": tf / PEAK_BF16_MFMA_TFLOPS,
                                "flops_per_launch": flops, "launch_ms_avg": a_ms},
            "decode_us_per_layer": d_ms * 1e3,
            "recalled_kv_GBps": db["kv"] / (d_ms * 1e-3) / 1e9,
            "decode_bytes_per_step": db["total"]}


def incremental_decode():
    """The incremental configuration: 16 sequences at a 32k context decode 1024 steps;
    every 320 steps the newest 320 tokens are clustered into 4 more clusters per head;
    tokens not clustered yet are always attended.  K/V rows and queries of all steps are
    generated beforehand; the timed loop holds library calls only."""
    import torch
    import paper_2412_03213_amd as ck
    from ck_synth import MixtureWorkload, get_config, sample_init_indices
    cfg = get_config(4)
    dev = "cuda:0"
    steps, m, cp = cfg.decode_steps, cfg.m_incr, cfg.c_incr
    w = MixtureWorkload(cfg, device=dev, extra_tokens=steps)
    w.token_center = torch.zeros(cfg.S, cfg.Hkv, cfg.N + steps, dtype=torch.int64, device=dev)
    for _ in range(steps):
        w.append_token()
    qs = [w.query() for _ in range(steps)]
    n_events = steps // m
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N + steps, cfg.C + n_events * cp)
    st = ck.ClusterState(sh, dev, budget=cfg.B, max_recent=m)
    init0 = sample_init_indices(w.K, cfg.C, cfg.seed, 0, cfg.N).to(dev)
    inits = [sample_init_indices(w.K, cp, cfg.seed + 1 + j, cfg.N + j * m, m).to(dev)
             for j in range(n_events)]
    t_prefill = event_ms(lambda: (setattr(st, "n_clusters", 0),
                                  st.cluster(w.K, init0, 0, cfg.N, cfg.C, cfg.n_iter)), 1)
    # size the clustering workspace for both call shapes before the timed loop
    st.cluster_ws = torch.empty(max(st.cluster_ws.numel(), 1 << 20), dtype=torch.uint8, device=dev)

    def run():
        st.n_clusters = cfg.C
        kv_bytes = []
        for t in range(1, steps + 1):
            rb = cfg.N + m * ((t - 1) // m)
            ck.decode_step(st, qs[t - 1], w.K, w.V, recent_begin=rb, recent_end=cfg.N + t)
            if t % m == 0:
                j = t // m - 1
                st.cluster(w.K, inits[j], cfg.N + j * m, m, cp, cfg.n_iter)

    run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    a.record()
    run()
    b.record()
    b.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = a.elapsed_time(b)
    n_tok = float(st.n_tokens.sum().item())
    hp = cfg.S * cfg.Hkv
    # bytes of an average step: recalled K/V + mean recent window (m/2 rows) + centroid table
    mean_recent = (m - 1) / 2 + 1
    kv_bytes = (n_tok + hp * mean_recent) * cfg.d * 2 * 2
    step_bytes = kv_bytes + hp * (cfg.C + n_events * cp / 2) * cfg.d * 2
    us = gpu_ms * 1e3 / steps
    final_clusters = st.n_clusters
    ev = event_ms(lambda: (setattr(st, "n_clusters", cfg.C),
                           st.cluster(w.K, inits[0], cfg.N, m, cp, cfg.n_iter)), 20)
    return {"workload": f"{cfg.name}: S={cfg.S}, N0={cfg.N}, {steps} steps, B={cfg.B}, "
                        f"{cp} clusters per {m} generated tokens",
            "decode_us_per_step_incl_reclustering": us,
            "host_wall_us_per_step": wall * 1e6 / steps,
            "recalled_kv_GBps": kv_bytes / (us * 1e-6) / 1e9,
            "roofline": {"bound": "hbm", "achieved": step_bytes / (us * 1e-6) / 1e9,
                         "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                         "frac": step_bytes / (us * 1e-6) / 1e9 / PEAK_HBM_GBPS},
            "incremental_clustering_us_per_event": ev * 1e3,
            "prefill_kmeans_ms": t_prefill,
            "final_clusters_per_head": final_clusters}


def graph_seq_ms(fns, reps):
    """The calls `fns` (one per layer, each on its own data) captured one after another
    into ONE HIP graph; average time per call over `reps` replays, plus median and
    minimum over the replays."""
    import torch
    if not USE_GRAPHS:
        def all_calls():
            for f in fns:
                f()
        st = train_stats(all_calls, reps)
        return {k: st[k] / len(fns) for k in ("mean", "median", "min")}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for f in fns:
            f()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for f in fns:
            f()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(reps)]
    for a, b in evs:
        a.record()
        g.replay()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) / len(fns) for a, b in evs)
    return {"mean": sum(ts) / len(ts), "median": ts[len(ts) // 2], "min": ts[0]}


def big_decode(reps, layers):
    """Decode-only measurement on the full-depth configuration (8 sequences,
    B = 2048), where a step moves enough bytes for the HBM roofline to mean
    something.  layers = 1: one layer (64 head-problems).  layers = 32: the K/V, tables
    and metadata of all 32 layers x 8 sequences are resident (about 36 GiB), and the
    decode step is timed (a) as 32 launches, layer after layer, each over its own
    layer's slice, in one HIP graph -- the order a model runs them in, and every layer's
    recalled rows come from HBM, not from a cache the previous replay warmed: the
    PRIMARY per-layer figure -- for the batch of 8 sequences and for sequence 0 alone
    (batch 1, B = 1024); and (b) as ONE launch over all 2048 head-problems, which no
    model can do (layers depend on each other): an upper bound, labelled so."""
    import torch
    import paper_2412_03213_amd as ck
    from ck_synth import Config, MixtureWorkload, get_config, sample_init_indices
    c1, c2 = get_config(1), get_config(2)
    cfg = Config(f"full_depth_{layers}_layers", 1, c2.S * layers, c2.Hkv, c2.Hq, c2.d, c2.N, c2.M,
                 c2.C, c2.n_iter, c2.B, c2.seed)
    dev = "cuda:0"
    w = MixtureWorkload(cfg, device=dev)
    w.token_center = None
    init = sample_init_indices(w.K, cfg.C, cfg.seed).to(dev)
    sh = ck.Shape(cfg.S, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
    st = ck.ClusterState(sh, dev, budget=cfg.B)
    t_cluster = event_ms(lambda: (setattr(st, "n_clusters", 0),
                                  st.cluster(w.K, init, 0, cfg.N, cfg.C, cfg.n_iter)), 2)
    q = w.query()

    def decode():
        ck.decode_step(st, q, w.K, w.V)

    for _ in range(5):
        decode()
    ms = event_ms(decode, 10 * reps)
    ms_graph = graph_ms(decode, 10 * reps, per_graph=32 if layers == 1 else 1)
    db = decode_bytes(cfg, st, cfg.C)

    def attn():
        ck.ck_sparse_decode_attn(sh, q, w.K, w.V, st.token_idx, st.n_tokens, cfg.B, st.out,
                                 workspace=st.attn_ws)

    at_avg, at_med, at_min = per_launch_ms(attn, 10 * reps)
    best = min(ms, ms_graph)
    gbps = db["total"] / (best * 1e-3) / 1e9
    what = "one layer" if layers == 1 else \
        "UPPER BOUND: all 32 layers launched as ONE batch (a model cannot: layers depend on each other)"
    out = {"workload": f"{what}; full_depth_32layers_b8: {cfg.S * cfg.Hkv} head-problems, "
                       f"N=32768, C=400, B=2048",
           "decode_us_per_step": ms * 1e3, "decode_us_per_step_hipgraph": ms_graph * 1e3,
           "decode_us_per_layer": best * 1e3 / layers,
           "bytes_per_step": db["total"],
           "recalled_kv_GBps": db["kv"] / (best * 1e-3) / 1e9,
           "recalled_tokens_mean": db["mean_tokens"],
           "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                        "frac": gbps / PEAK_HBM_GBPS,
                        "traffic": read_traffic("k_attn", "batch8_layer") if layers == 1 else None},
           "attn_call_us_avg": at_avg * 1e3, "attn_call_us_min": at_min * 1e3,
           "attn_GBps": db["attn"] / (at_avg * 1e-3) / 1e9,
           "kmeans_ms": t_cluster,
           "kmeans_keys_per_s": cfg.S * cfg.Hkv * cfg.N / (t_cluster * 1e-3)}
    if layers == 1:
        out["note"] = "the same layer replayed: its recalled rows stay in the caches (warm)"
        return out

    # ---- the primary timing: layer after layer, each over its own slice ----
    def layer_calls(S_l, budget):
        shl = ck.Shape(S_l, cfg.Hq, cfg.Hkv, cfg.N, cfg.C)
        ws = torch.empty(ck.ck_workspace_bytes(shl, 1, budget), dtype=torch.uint8, device=dev)
        calls = []
        for l in range(layers):
            a, b = l * c2.S, l * c2.S + S_l
            args = (shl, q[a:b], w.K[a:b], w.V[a:b], st.centroids[a:b], st.sizes[a:b],
                    st.offsets[a:b], st.sorted_idx[a:b], st.n_clusters, budget, ck.CK_SEL_WHOLE,
                    st.scores[a:b], st.sel_clusters[a:b], st.n_sel_clusters[a:b],
                    st.n_sel_tokens[a:b], st.token_idx[a:b], st.n_tokens[a:b], st.out[a:b])
            calls.append(lambda args=args: ck.ck_decode_step(*args, workspace=ws))
        return calls

    for name, S_l, budget in (("distinct_layers_batch8", c2.S, c2.B),
                              ("distinct_layers_batch1", 1, c1.B)):
        calls = layer_calls(S_l, budget)
        tg = graph_seq_ms(calls, max(reps, 10))
        idx = torch.cat([torch.arange(l * c2.S, l * c2.S + S_l) for l in range(layers)]).to(dev)
        n_tok = st.n_tokens[idx].cpu().numpy().astype("int64")
        n_sel = st.n_sel_clusters[idx].cpu().numpy().astype("int64")
        hp_l = S_l * cfg.Hkv
        per_layer = (hp_l * layers * (cfg.C * cfg.d * 2 + cfg.C * 8 + cfg.G * cfg.d * 2)
                     + int(n_sel.sum()) * 8 + int(n_tok.sum()) * 8
                     + int(n_tok.sum()) * (cfg.d * 4 + 4) + hp_l * layers * cfg.G * cfg.d * 4) / layers
        kv = int(n_tok.sum()) * cfg.d * 4 / layers
        g = per_layer / (tg["mean"] * 1e-3) / 1e9
        out[name] = {"what": f"32 ck_decode_step launches over 32 different layers ({S_l} "
                             f"sequence(s), {hp_l} head-problems, B={budget} each) in one HIP "
                             f"graph; time per layer",
                     "decode_us_per_layer": tg["mean"] * 1e3,
                     "decode_us_per_layer_median": tg["median"] * 1e3,
                     "decode_us_per_layer_min": tg["min"] * 1e3,
                     "bytes_per_layer": per_layer,
                     "recalled_kv_GBps": kv / (tg["mean"] * 1e-3) / 1e9,
                     "recalled_tokens_mean": float(n_tok.mean()),
                     "roofline": {"bound": "hbm", "achieved": g, "peak": PEAK_HBM_GBPS,
                                  "unit": "GB/s", "frac": g / PEAK_HBM_GBPS}}
    return out


if __name__ == "__main__":
    main()
