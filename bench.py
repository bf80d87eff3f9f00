#!/usr/bin/env python3
"""Benchmark of the AdaSD verification hot path on one MI355X.

One step = one decode round's verification on the headline workload (B=32 sequences, k=8 drafted
positions, V=128256, bf16 logits resident in HBM): adasd_verify (normalisers, entropies, JS distance,
posterior, both acceptance tests, first reject, correction/bonus token) with the update step of
adasd_update_thresholds applied by the same call (options.apply_update; --separate-update makes it
a second call).  Inputs rotate over several distinct seeded batches (> 512 MB in total) so
that no cache carries logits from one step to the next.

Prints ONE JSON line: throughput in verified positions/s, the HBM roofline fraction of the
statistics kernels (algorithmic bytes / measured kernel time), and the CPU oracle timed on the same
workload as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
TARGET_FRAC = 0.70             # the build's goal for the statistics stage on the headline workload
# Bytes per launch that the statistics stage moves between the L2 caches and the fabric on the HEADLINE
# workload: STORED constants, not measured by this script.  They come from the rocprofv3 counter runs whose
# summaries are kept under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads
# for a plain copy of known size).  These counters sit at the L2: they cannot tell HBM from the 256 MB
# Infinity Cache behind it, so this is L2-miss traffic, an upper bound of the HBM bytes.
STAGE_TRAFFIC = {
    "single_read": (133.05e6, "profiles/l2_miss_traffic_pmc_verify_B32_k8_V128256.md: k_stats_fused 132.78 MB + 0.27 MB"),
    "two_kernel": (263.66e6, "profiles/l2_miss_traffic_pmc_verify_B32_k8_V128256.md: k_rowstats 131.38 MB + 0.13 MB, "
                             "k_jsd 132.06 MB + 0.08 MB"),
}
# shapes: the headline workload is the one the metric is quoted on; "large" is a side measurement
WORKLOADS = {"headline": (32, 8, 128256, 4),      # 4 sets x 139.5 MB of logits
             "large": (128, 16, 152064, 2),       # 2 sets x 1.28 GB
             "closed_loop": (64, 16, 128256, 0)}  # fresh logits every round, generated on the device
LIST_CAP = 8192


def closed_loop(args, am, torch, B, k_max, V):
    """Decode rounds from the initial state (T_G = 0, empty lists): per round, one adasd_draft_step call per
    drafted token on the rows of the sequences still drafting (stop rule H(q) > T_G, drawn token x ~ q), then
    adasd_verify on the ragged windows with the update step applied.  Fresh logits every round, generated on
    the device with the recipe of the closed-loop configuration (std 3, spike 8, per-sequence mixing weight
    on a +-0.02 random walk in [0.4, 0.99]); generation is outside every timed region."""
    from paper_2512_11280_amd import workloads as wl
    dev = "cuda"
    src = wl.ClosedLoopDeviceSource(B, V, k_max)
    cap = 16384
    ws = am.Workspace(B, k_max, V, torch.bfloat16)
    state = am.State(B, cap)
    out = am.binding.alloc_verify_result(B, k_max)
    opts = am.Options(apply_update=1)
    H = torch.empty(B, dtype=torch.float32, device=dev)
    stop = torch.empty(B, dtype=torch.uint8, device=dev)
    dst = torch.empty(B, dtype=torch.int32, device=dev)
    xT = torch.zeros(k_max, B, dtype=torch.int32, device=dev)
    rounds = args.warmup + args.steps
    wall = 0.0
    kern_ms = [0.0] * 6
    draft_calls = 0
    positions = 0
    accepted = 0
    for r in range(rounds):
        # ---- this round's logits (untimed)
        t, d = src.next_round()
        active = torch.ones(B, dtype=torch.uint8, device=dev)
        lens = torch.zeros(B, dtype=torch.int32, device=dev)
        xT.zero_()
        timed = r >= args.warmup
        if timed:
            am.profile_enable(k_max + 8)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        # ---- drafting: one call per drafted token while any sequence is still drafting
        n_calls = 0
        for step in range(k_max):
            am.draft_step(d[:, step], ws, T_G=state.T_G, active=active, step=step, k_max=k_max, seed=7, round0=r,
                          H_out=H, stop_out=stop, token_out=xT[step], status_out=dst)
            n_calls += 1
            lens += active.to(torch.int32)
            active = active & (1 - stop)
            if not bool(active.any()):          # (the host has to know when to stop calling the draft model)
                break
        x = xT.clamp(min=0).t().contiguous()
        # ---- verification of the ragged windows, state updated by the same call
        am.verify(t, d, x, ws, state=state, draft_len=lens, seed=7, round0=r, options=opts, out=out)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if timed:
            wall += t1 - t0
            for c in range(6):
                ms, _ = am.profile_read(c)
                kern_ms[c] += ms
            am.profile_disable()
            draft_calls += n_calls
            positions += int(lens.sum())
            accepted += int(out.n_accept.sum())
        if r % 50 == 0:
            print(f"round {r}: mean window {float(lens.float().mean()):.2f}", file=sys.stderr, flush=True)
    host = state.to_host()
    steps = args.steps
    kern_total = sum(kern_ms)
    line = {
        "metric": "verified positions/sec and achieved HBM GB/s (% peak) at B=32,k=8,V=128256 bf16",
        "value": positions / wall,
        "unit": "verified positions/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"closed loop B={B} V={V} k_max={k_max} bf16, {steps} decode rounds from the initial "
                               f"state, fresh logits each round (device-generated), list capacity {cap}",
                   "step": "adasd_draft_step per drafted token while any sequence drafts, then adasd_verify with "
                           "options.apply_update on the ragged windows; wall time includes the host's per-call "
                           "stop check and the small tensor ops of the loop"},
        "roofline": None,
        "cpu_baseline": None,
        "closed_loop": {
            "mean_window_k_b": positions / (steps * B),
            "mean_accepted_length": accepted / (steps * B),
            "draft_calls_per_round": draft_calls / steps,
            "kernel_us_per_round": {"row_stats": kern_ms[0] / steps * 1e3, "jsd": kern_ms[1] / steps * 1e3,
                                    "decide": kern_ms[2] / steps * 1e3, "sample": kern_ms[3] / steps * 1e3,
                                    "draft_step_all_calls": kern_ms[5] / steps * 1e3},
            "draft_step_kernel_us_per_call": kern_ms[5] / max(draft_calls, 1) * 1e3,
            "positions_per_s_kernel_time_only": positions / (kern_total * 1e-3) if kern_total > 0 else None,
            "list_lengths_at_end": {"accepted_mean": float(host["nA"].mean()), "rejected_mean": float(host["nR"].mean())},
            "T_G_mean_at_end": float(host["T_G"].mean()),
        },
    }
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="headline",
                    help="headline: B=32 k=8 V=128256 (the metric's workload); large: B=128 k=16 V=152064; "
                         "closed_loop: B=64 k_max=16 V=128256, a step is one decode round (drafting calls until "
                         "every sequence has stopped, then verify + update) from the initial state "
                         "(side measurements, no CPU baseline, no counter-derived traffic figure)")
    ap.add_argument("--sets", type=int, default=0, help="rotating input sets (0: the workload's default)")
    ap.add_argument("--stats-path", type=int, default=0, help="0 library default, 1 two-kernel path, 2 single-read kernel")
    ap.add_argument("--separate-update", action="store_true",
                    help="apply the update step with a separate adasd_update_thresholds call")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step of each input set in a HIP graph once and time replays "
                         "(the round counter then lives in device memory and is advanced inside the graph)")
    ap.add_argument("--shards", type=int, default=0,
                    help="also time one holder's calls of the column-sharded path with this many holders "
                         "(its V/G columns of the same workload; the other holders' records are computed "
                         "beforehand), reported under 'sharded'")
    ap.add_argument("--no-running-sums", action="store_true",
                    help="state without adasd_state.mom: the decision stage adds the history lists up in every call")
    ap.add_argument("--literal", action="store_true",
                    help="time the variant that follows Algorithm 1's loop as written (options base_test=1, "
                         "list_update=1) instead of the default readings")
    ap.add_argument("--list-cap", type=int, default=LIST_CAP,
                    help="capacity of the per-sequence history lists (the lists themselves hold 64+64 entries)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device-to-device copy of known size (counter calibration for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (sequences are independent, so the "
                 "path shards by sequence with no communication); use --gpus 1")

    B, K, V, n_sets = WORKLOADS[args.workload]
    large = args.workload == "large"
    if args.sets > 0:
        n_sets = args.sets

    import numpy as np
    import torch

    import paper_2512_11280_amd as am
    from paper_2512_11280_amd import workloads as wl

    am.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload == "closed_loop":
        return closed_loop(args, am, torch, B, K, V)

    # ---- seeded synthetic inputs, resident in HBM before any timing
    sets = []
    host0 = None
    for i in range(n_sets):
        if large:
            batch = wl.config_large(seed=wl.DEFAULT_SEED + 3 + 100 * i, B=B, k=K, V=V, cap=args.list_cap)
            print(f"input set {i} generated", file=sys.stderr, flush=True)
        else:
            batch = wl.config_batched(seed=wl.DEFAULT_SEED + 2 + 100 * i, B=B, k=K, V=V, cap=args.list_cap)
        if i == 0:
            host0 = batch
        sets.append((batch.target.cuda(), batch.draft.cuda(), batch.draft_tokens.cuda(), batch.seed))
    ws = am.Workspace(B, K, V, torch.bfloat16)
    state = am.State(B, args.list_cap, running_sums=not args.no_running_sums).load(host0.state)
    out = am.binding.alloc_verify_result(B, K)
    torch.cuda.synchronize()

    opts = am.Options(stats_path=args.stats_path, apply_update=0 if args.separate_update else 1,
                      base_test=1 if args.literal else 0, list_update=1 if args.literal else 0)
    if args.calibrate_copy:
        src = sets[0][0]
        dst = torch.empty_like(src)
        dst.copy_(src)                      # one elementwise copy kernel: reads and writes src.nbytes
        torch.cuda.synchronize()
        print(f"calibration copy: {src.numel() * src.element_size()} bytes read and written", file=sys.stderr)

    def eager_step(i, rounds=None):
        t, d, x, seed = sets[i % len(sets)]
        am.verify(t, d, x, ws, state=state, seed=seed, round0=i, rounds=rounds, options=opts, out=out)
        if args.separate_update:
            am.update_thresholds(state, K, out.n_accept, out.H_q, out.d_js)

    step = eager_step
    if args.graph:
        rounds = torch.zeros(B, dtype=torch.int32, device="cuda")
        one = torch.ones(B, dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(len(sets)):
                eager_step(i, rounds)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for i in range(len(sets)):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                eager_step(i, rounds)
                rounds.add_(one)             # every replay, of whichever set, is one round later
            graphs.append(gph)
        state.load(host0.state)
        rounds.zero_()
        torch.cuda.synchronize()

        def step(i):                         # noqa: F811
            graphs[i % len(sets)].replay()

    # ---- side measurements first (drafting calls, the single-stream configuration, the plain streaming read):
    #      they need nothing of the timed loop, and with them in front the chip has been under load for some
    #      tens of milliseconds when the warm-up starts, however few warm-up steps the caller asks for
    names = ["row_stats", "jsd", "decide", "sample", "update", "draft_entropy"]
    # ---- draft-side call (one [B, V] row block per drafted token), reported on the side
    rows = sets[0][1][:, 0]
    H = torch.empty(B, dtype=torch.float32, device="cuda")
    stop = torch.empty(B, dtype=torch.uint8, device="cuda")
    for _ in range(10):
        am.draft_entropy(rows, ws, T_G=state.T_G, step=0, k_max=20, H_out=H, stop_out=stop)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(200):
        am.draft_entropy(sets[i % len(sets)][1][:, i % K], ws, T_G=state.T_G, step=0, k_max=20,
                         H_out=H, stop_out=stop)
    torch.cuda.synchronize()
    draft_us = (time.perf_counter() - t1) / 200 * 1e6
    # the same call with the token draw (x_i ~ q_i) in the same pass
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    dst = torch.empty(B, dtype=torch.int32, device="cuda")
    for _ in range(10):
        am.draft_step(rows, ws, T_G=state.T_G, step=0, k_max=20, seed=1, H_out=H, stop_out=stop,
                      token_out=tok, status_out=dst)
    torch.cuda.synchronize()

    def draft_steps():
        for i in range(200):
            am.draft_step(sets[i % len(sets)][1][:, i % K], ws, T_G=state.T_G, step=i % K, k_max=20, seed=1,
                          round0=i, H_out=H, stop_out=stop, token_out=tok, status_out=dst)
        torch.cuda.synchronize()

    t1 = time.perf_counter()
    draft_steps()
    draft_step_us = (time.perf_counter() - t1) / 200 * 1e6
    am.profile_enable(2 * 200 + 8)          # once more with the launches carrying events: kernel time only
    draft_steps()
    ms, n = am.profile_read(5)
    draft_step_kernels_us = ms / 200 * 1e3 if n else None
    am.profile_disable()

    # ---- the single-stream configuration (B=1, k=8, V=128256 bf16, history lists of 64+64): latency of one call
    single = None
    if not large:
        one = wl.config_single_stream()
        t1_, d1_, x1_ = one.target.cuda(), one.draft.cuda(), one.draft_tokens.cuda()
        st1 = am.State(1, one.state["LA"].shape[1]).load(one.state)
        out1 = am.binding.alloc_verify_result(1, one.k)
        o1 = am.Options(apply_update=1)

        def single_calls(n):
            for i in range(n):
                am.verify(t1_, d1_, x1_, ws, state=st1, seed=one.seed, round0=i, options=o1, out=out1)
            torch.cuda.synchronize()

        single_calls(20)
        t1 = time.perf_counter()
        single_calls(200)
        single_wall = (time.perf_counter() - t1) / 200 * 1e6
        am.profile_enable(3 * 200 + 8)
        st1.load(one.state)
        single_calls(200)
        single_kern = {}
        for c, name in enumerate(names):
            ms, n = am.profile_read(c)
            if n:
                single_kern[name] = ms / 200 * 1e3
        am.profile_disable()
        single = {"workload": "single stream B=1 k=8 V=128256 bf16 (resident in the caches between calls)",
                  "us_per_call": single_wall, "kernel_us": single_kern}

    # ---- practical ceiling: the same logits streamed by a kernel that does no arithmetic (one 32 KiB
    #      piece per workgroup, all loads of a thread in flight at once), rotating over the input sets
    #      (one launch per set over a contiguous copy of exactly the rows the statistics stage reads)
    copies = [torch.cat([t[:, :K].reshape(-1), d.reshape(-1)]) for t, d, _, _ in sets]
    sink = torch.empty(copies[0].numel() * 2 // 32768 + 1, dtype=torch.int32, device="cuda")
    reps_stream = 40
    for c in copies:
        am.stream_read(c, sink)
    torch.cuda.synchronize()
    am.profile_enable(reps_stream + 8)
    stream_bytes = 0
    for i in range(reps_stream):
        c = copies[i % len(copies)]
        am.stream_read(c, sink)
        stream_bytes += c.numel() * c.element_size()
    torch.cuda.synchronize()
    ms, n = am.profile_read(6)
    am.profile_disable()
    stream_gbps = stream_bytes / (ms * 1e-3) / 1e9 if n and ms > 0 else None
    del copies

    state.load(host0.state)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    positions_per_s = B * K * args.steps / elapsed

    # ---- the same steps once more, each between two HIP events on the launch stream (the binding launches
    #      on torch's current stream): distribution of the step time on the device, launch gaps included
    state.load(host0.state)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i in range(args.steps):
        ev[i][0].record()
        step(args.warmup + i)
        ev[i][1].record()
    torch.cuda.synchronize()
    ev_us = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    step_events = {"median": ev_us[len(ev_us) // 2], "p10": ev_us[len(ev_us) // 10], "p90": ev_us[(len(ev_us) * 9) // 10],
                   "what": "one step between two HIP events on the launch stream, microseconds"}

    # ---- the same steps again with HIP events carried by the kernel launches themselves (library
    #      side, on the launch stream; the dispatch stamps them at its start and end): per-kernel
    #      durations for the roofline figure
    am.profile_enable(2 * args.steps + 8)
    state.load(host0.state)
    torch.cuda.synchronize()
    for i in range(args.steps):
        eager_step(args.warmup + i)          # (kernel timing needs the launches themselves, not a replay)
    torch.cuda.synchronize()
    kern_us = {}
    for c, name in enumerate(names):
        ms, n = am.profile_read(c)
        if n:
            kern_us[name] = ms / args.steps * 1e3       # per step (a class may hold two kernels)
    am.profile_disable()
    mean_accept = float(out.n_accept.float().mean().item())

    # Algorithmic bytes of one launch of the statistics stage: every target and draft logit of the
    # B*k verified positions once (513 024 B per position).  The single-read kernel streams them once; the
    # two-kernel path (normalisers, then JS distance) streams them twice and is still priced against ONE
    # read.  Each kernel alone is also given against the bytes it streams.
    algo_bytes = 2 * V * 2 * B * K
    stats_us = kern_us.get("row_stats", 0.0) + kern_us.get("jsd", 0.0)
    achieved = algo_bytes / (stats_us * 1e-6) / 1e9 if stats_us > 0 else 0.0
    per_kernel = {name: {"kernel_us": kern_us[name], "streamed_bytes": algo_bytes,
                         "GBps": algo_bytes / (kern_us[name] * 1e-6) / 1e9,
                         "frac": algo_bytes / (kern_us[name] * 1e-6) / 1e9 / HBM_PEAK_GBS}
                  for name in ("row_stats", "jsd") if name in kern_us}

    # ---- one holder's share of the column-sharded path (its V/G columns, the replicated stages in full)
    sharded = None
    if args.shards > 0:
        n_sh = args.shards
        cuts = [V * g // n_sh // 8 * 8 for g in range(n_sh)] + [V]
        t, d, x, seed = sets[0]
        shards = [am.Shard(n_sh, g, V, cuts[g]) for g in range(n_sh)]
        views = [(t[:, :, cuts[g]:cuts[g + 1]], d[:, :, cuts[g]:cuts[g + 1]]) for g in range(n_sh)]
        tri = torch.empty(n_sh, B * K * 2, 4, device="cuda")
        pos = torch.empty(n_sh, B * K, 4, device="cuda")
        top = torch.empty(n_sh, B, 4, device="cuda")
        cand = torch.empty(n_sh, B, am.binding.SHARD_CAND_BYTES, dtype=torch.uint8, device="cuda")
        tau = torch.empty(B, dtype=torch.float32, device="cuda")
        state.load(host0.state)

        def holder(g, r):
            """The calls holder g makes in one round, in order (the gathers between them are the caller's)."""
            am.verify_shard_stats(views[g][0], views[g][1], x, ws, shards[g], triples_out=tri[g])
            am.verify_shard_jsd(views[g][0], views[g][1], x, ws, shards[g], tri, pos_out=pos[g])
            am.verify_shard_decide(B, K, torch.bfloat16, x, ws, shards[g], tri, pos, state=state, seed=seed,
                                   round0=r, options=am.Options(apply_update=1), out=out)
            am.verify_shard_sample(views[g][0], views[g][1], x, ws, shards[g], seed=seed, round0=r, top_out=top[g])
            am.verify_shard_pick(B, K, torch.bfloat16, x, ws, shards[g], top, out, tau_out=tau)
            am.verify_shard_refine(views[g][0], views[g][1], x, ws, shards[g], tau, seed=seed, round0=r,
                                   cand_out=cand[g])
            am.verify_shard_settle(B, K, torch.bfloat16, x, ws, shards[g], tau, cand, out, seed=seed, round0=r)

        for g in range(n_sh):                 # fill every holder's records once
            holder(g, 0)
        torch.cuda.synchronize()
        reps = 100
        t1 = time.perf_counter()
        for r in range(reps):
            holder(0, r)
        torch.cuda.synchronize()
        sharded = {"holders": n_sh, "columns_per_holder": cuts[1] - cuts[0],
                   "us_per_round_one_holder": (time.perf_counter() - t1) / reps * 1e6,
                   "exchange_bytes_per_holder": (B * K * 2 + B * K + B) * 16 + B * am.binding.SHARD_CAND_BYTES}
        state.load(host0.state)

    # ---- CPU oracle on the same workload (baseline, not a target)
    cpu = None
    if not args.no_cpu_baseline and not large:
        from oracle import load_oracle
        ora = load_oracle()
        s = host0.state
        reps = 12                      # about 10 s of CPU work over the threads
        c0 = time.perf_counter()
        for r in range(reps):
            ora.verify(host0.target, host0.draft, host0.draft_tokens.numpy(), LA=s["LA"], LR=s["LR"],
                       nA=s["nA"], nR=s["nR"], seed=host0.seed, round0=r,
                       base_test=opts.base_test, list_update=opts.list_update)
        c1 = time.perf_counter()
        cpu = {"value": B * K * reps / (c1 - c0), "unit": "verified positions/s",
               "cores": ora.num_threads(), "kind": "oracle",
               "sample": f"full workload batch 0 (B={B}, k={K}, V={V}: {B * K} positions + {B} sampled "
                         f"tokens), {reps} repetitions, float64 C oracle with OpenMP over sequences"}
        # the same oracle on one thread (a B=1 slice: its parallel loop runs over sequences), a few seconds
        nb = 3
        c0 = time.perf_counter()
        for b in range(nb):
            ora.verify(host0.target[b:b + 1], host0.draft[b:b + 1], host0.draft_tokens[b:b + 1].numpy(),
                       LA=s["LA"][b:b + 1], LR=s["LR"][b:b + 1], nA=s["nA"][b:b + 1], nR=s["nR"][b:b + 1],
                       seed=host0.seed, seq_id=np.array([b]), round0=0,
                       base_test=opts.base_test, list_update=opts.list_update)
        c1 = time.perf_counter()
        cpu["single_thread"] = {"value": K * nb / (c1 - c0), "unit": "verified positions/s",
                                "sample": f"{nb} one-sequence calls ({K} positions + 1 sampled token each): the "
                                          f"oracle's only parallel loop is over sequences, so these run on one thread"}

    two_kernel = "jsd" in kern_us
    traffic, traffic_src = (STAGE_TRAFFIC["two_kernel" if two_kernel else "single_read"]
                            if args.workload == "headline" else (None, None))
    frac = achieved / HBM_PEAK_GBS
    line = {
        "metric": "verified positions/sec and achieved HBM GB/s (% peak) at B=32,k=8,V=128256 bf16",
        "value": positions_per_s,
        "unit": "verified positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"batched verify B={B} k={K} V={V} bf16 logits, "
                               f"{len(sets)} rotating seeded input sets, history lists 64+64 per sequence "
                               f"(capacity {args.list_cap})",
                   "step": "adasd_verify + adasd_update_thresholds" if args.separate_update
                           else "adasd_verify with options.apply_update (update step in the decision kernel)",
                   "launch": "replay of a captured HIP graph per input set" if args.graph else "eager launches",
                   "readings": "Algorithm 1's loop as written (base_test=1, list_update=1)" if args.literal
                               else "defaults (ratio test + residual, lists as of the round's start)"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": frac,
                     "target_frac": TARGET_FRAC,
                     "target": (f"met: {frac:.2f}" if frac >= TARGET_FRAC else
                                f"target {TARGET_FRAC:.2f} not met: {frac:.2f} (the stage is bound by its vector "
                                f"arithmetic, not by HBM; the plain read below is the ceiling a kernel without "
                                f"arithmetic reaches)"),
                     "traffic": traffic,
                     "traffic_kind": (None if traffic is None else
                                      "L2-miss traffic per launch (FETCH_SIZE + WRITE_SIZE count at the L2 and cannot "
                                      "tell HBM from the 256 MB Infinity Cache): a stored constant from " + traffic_src +
                                      ", valid for this workload and this statistics path only"),
                     "traffic_GBps": traffic / (stats_us * 1e-6) / 1e9 if traffic and stats_us > 0 else None,
                     "kernel": "k_rowstats + k_jsd" if two_kernel else "k_stats_fused",
                     "algorithmic_bytes": algo_bytes,
                     "kernel_us": stats_us,
                     "per_kernel": per_kernel,
                     "stream_read": {"GBps": stream_gbps, "frac": stream_gbps / HBM_PEAK_GBS if stream_gbps else None,
                                     "what": "adasd_stream_read over the same logits: loads only, no arithmetic"}},
        "cpu_baseline": cpu,
        "kernel_us": kern_us,
        "step_us_events": step_events,
        "single_stream": single,
        "draft_entropy_us_per_call": draft_us,
        "draft_step_us_per_call": draft_step_us,
        "draft_step_kernels_us": draft_step_kernels_us,
        "mean_accepted_length": mean_accept,
        "sharded": sharded,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
