#!/usr/bin/env python3
"""Throughput of the ShadowSync hot path on one MI355X.

Workload (default): the Mid CTR model -- 13 dense features, 8 tables x 1e6 rows x dim 64
fp32, ids Zipf(1.05), bag length Poisson(20)+1, bottom MLP 13-256-128-64, top MLP
100-512-256-1 with bf16 MFMA GEMMs over fp32 master weights, batch 2048, K=4 replicas each
fed by 2 lock-free worker streams (one host thread per stream), Shadow EASGD (alpha 0.1) enqueued
on a separate stream once per 5 trainer iterations of a replica.  One bench "step" = one
ss_train_step on one batch (forward, loss, backward, SGD on the replica, sort + segmented
reduction + row-wise Adagrad on the tables); steps go round-robin over the K replicas.
Inputs are seeded synthetic batches already resident in HBM when the clock starts.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant single memory-bound kernel (largest summed time of the gather
                and the row-update chunk pass), timed with HIP events inside the timed region
  kernels       the same event timing for every kernel class
  sync_isolation  the three shadow rules on K=8 x 50M-parameter replicas (GB/s vs HBM peak)
  cpu_baseline  the numpy oracle on the host cores, on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X datasheet

# HBM bytes per launch measured with `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` on the
# Mid and Large workloads (KiB per dispatch * 1024; FETCH_SIZE reads 0.50x and WRITE_SIZE 1.00x the
# known size of a plain streaming kernel, so fetches are scaled by 2.00).  Sources:
# profiles/mid_hbm_traffic.txt, profiles/large_hbm_traffic.txt.  None = not measured.
MEASURED_TRAFFIC = {
    "mid": {"gather": 52.9e6, "row_update_chunk": 125.2e6},
    "large": {"gather": 601e6, "row_update_chunk": 1357e6},
}
# Average kernel duration (us) reported by `rocprofv3 --kernel-trace --stats` with ONE stream
# active (profiles/mid_single_stream_kernel_stats.txt): the event brackets of the same run read
# about 5.5 us more per launch.  Quoted next to the live event figures, never instead of them.
PROFILER_ALONE_US = {
    "mid": {"gather": 14.73, "row_update_chunk": 32.42},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="mid", choices=["mid", "tiny", "hogwild", "large"])
    ap.add_argument("--batches", type=int, default=16, help="distinct batches cycled through")
    ap.add_argument("--foreground", type=int, default=0, metavar="K",
                    help="foreground variant (FR-EASGD-k): every worker stream exchanges its "
                         "replica with the centre copy on ITS OWN stream every k of its steps")
    ap.add_argument("--foreground-rule", default="easgd", choices=["easgd", "ma", "bmuf"],
                    help="with --foreground: easgd = per-worker exchange (FR-EASGD-k); ma / bmuf "
                         "= every k steps all worker streams meet, one S-MA / S-BMUF round runs "
                         "after all of them and all of them wait for it (FR-MA / FR-BMUF)")
    ap.add_argument("--continuous-shadow", action="store_true",
                    help="loop shadow rounds back to back (ss_shadow_start) instead of pacing them")
    ap.add_argument("--workers-per-replica", type=int, default=6,
                    help="Hogwild worker streams per replica")
    ap.add_argument("--replicas", type=int, default=0, metavar="K",
                    help="number of dense replicas (default: the workload's)")
    ap.add_argument("--no-shadow", action="store_true", help="run without the shadow stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sync-isolation", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket kernels with events in the timed region")
    ap.add_argument("--single-thread", action="store_true",
                    help="enqueue all streams from one host thread")
    return ap.parse_args()


def algorithmic_bytes(kernel, wl, batch_np, n_unique):
    """Bytes the method itself must move per launch of `kernel` on this batch."""
    n = int(batch_np.offsets[-1])
    B, T, d = wl.batch, wl.num_tables, wl.emb_dim
    if kernel == "gather":
        # per id: one row (4d) + its index (4) + sort key and pooled-vector id written (8);
        # per bag: pooled vector written (4d) + its offset (4)
        return n * (4 * d + 4 + 8) + B * T * (4 * d + 4)
    if kernel == "row_update_chunk":
        # per occurrence: gradient row (4d) + sorted key and bag id (8); per distinct row:
        # row read + written (8d) + accumulator read + written (8)
        return n * (4 * d + 8) + n_unique * (8 * d + 8)
    raise KeyError(kernel)


def cpu_baseline(wl, gen, seconds=20.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from paper_2003_03477_amd import synth
    batches = [gen.batch(10_000 + s) for s in range(3)]
    cp = synth.compact_problem(wl, batches)
    row_base = np.concatenate(([0], np.cumsum(cp.rows)))
    orc = oracle.OracleTrainer(wl.bot_dims, wl.top_dims, row_base, cp.h0, synth.dense_w0(wl),
                               wl.num_replicas, wl.lr_dense, wl.lr_emb, wl.adagrad_eps,
                               bf16=wl.bf16)
    t0 = time.perf_counter()
    steps = 0
    while True:
        orc.train_step(steps % wl.num_replicas, *cp.batches[steps % len(cp.batches)].as_tuple())
        steps += 1
        if steps % (wl.sync_gap * wl.num_replicas) == 0:
            orc.shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu)
        if time.perf_counter() - t0 > seconds or steps >= 64:
            break
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    return {"value": wl.batch * steps / dt, "unit": "examples/s", "cores": cores,
            "kind": "oracle",
            "sample": f"{steps} train steps of batch {wl.batch} (+ sync rounds) of the fp64 "
                      f"numpy oracle, tables compacted to the {sum(cp.rows)} touched rows, "
                      f"{dt:.1f} s; BLAS may use up to `cores` threads, the rest is one thread"}


def sync_isolation(binding, torch, rounds=20):
    """K=8 replicas of 50M fp32 parameters + centre copy: rounds of each rule back to back."""
    K, P = 8, 50_000_000
    g = torch.Generator(device="cuda").manual_seed(4)
    W = torch.randn(K * P, device="cuda", generator=g) * 0.02
    ps = torch.randn(P, device="cuda", generator=g) * 0.02
    wg = ps.clone()
    v = torch.zeros(P, device="cuda")
    st = torch.cuda.Stream()
    out = {}
    per_param = {"easgd": 8 * (K + 1), "ma": 8 * K + 4, "bmuf": 8 * K + 16}
    args = {"easgd": dict(alpha=0.05), "ma": dict(alpha=0.5), "bmuf": dict(alpha=0.5, eta=1.0, momentum=0.9)}
    for algo in ("easgd", "ma", "bmuf"):
        with torch.cuda.stream(st):
            for _ in range(3):
                binding.ss_sync_round(algo, K, P, P, W, ps, wg, v, stream=st, **args[algo])
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(rounds):
                binding.ss_sync_round(algo, K, P, P, W, ps, wg, v, stream=st, **args[algo])
            e1.record(st)
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / rounds
        gbs = per_param[algo] * P / us / 1e3
        out[algo] = {"us_per_round": us, "algorithmic_bytes": per_param[algo] * P,
                     "GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    out["config"] = f"K={K} replicas x {P} fp32 parameters, {rounds} rounds per rule back to back"
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K replicas share its HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2003_03477_amd import binding, synth

    wl = synth.WORKLOADS[args.workload]()
    if args.replicas:
        wl = wl.scaled(num_replicas=args.replicas)
    K = wl.num_replicas
    WPR = args.workers_per_replica
    NS = K * WPR                           # worker streams = worker slots
    gen = synth.BatchGenerator(wl)
    host_batches = [gen.batch(s) for s in range(args.batches)]
    max_ids = max(int(b.offsets[-1]) for b in host_batches) + 4096
    gpu = binding.from_workload(wl, num_worker_slots=NS, max_ids=max_ids)
    gpu.ss_init_tables_hash()
    gpu.ss_init_dense(synth.dense_w0(wl))
    dev_batches = [binding.upload_batch(b) for b in host_batches]
    streams = [torch.cuda.Stream() for _ in range(NS)]
    shadow = torch.cuda.Stream()
    losses = torch.zeros(NS, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def run(total_steps, first_step):
        """Step s runs on worker stream s % NS, which trains replica (s % NS) % K."""
        def one(s):
            w = s % NS
            gpu.ss_train_step(w % K, w, dev_batches[s % len(dev_batches)], streams[w],
                              losses[w:w + 1])

        r0_steps = [0]
        r0_lock = threading.Lock()

        fg_collective = args.foreground and args.foreground_rule != "easgd"
        meet = threading.Barrier(NS)
        arrive = [torch.cuda.Event() for _ in range(NS)]
        done = [torch.cuda.Event()]

        def foreground_collective(w):
            """All worker streams stop, one averaging round runs, all resume (the foreground
            form of Algorithms 3 and 4): stream order is enforced with events, host threads
            only meet to enqueue them."""
            arrive[w].record(streams[w])
            meet.wait()
            if w == 0:
                for e in arrive:
                    shadow.wait_event(e)
                mu = wl.mu if args.foreground_rule == "bmuf" else 0.0
                gpu.ss_shadow_sync(args.foreground_rule, wl.alpha, wl.eta, mu, shadow)
                done[0] = torch.cuda.Event()
                done[0].record(shadow)
            meet.wait()
            streams[w].wait_event(done[0])

        def worker(w):
            for j, s in enumerate(range(first_step + w, first_step + total_steps, NS)):
                one(s)
                if args.foreground and (j + 1) % args.foreground == 0:
                    if fg_collective:
                        # every worker must come to every meeting: none after the step count
                        # that all workers reach
                        if j + 1 <= total_steps // NS:
                            foreground_collective(w)
                    else:
                        gpu.ss_easgd_exchange(w % K, wl.alpha, streams[w])
                    continue
                # one shadow round per sync_gap iterations of replica 0 (all its workers)
                if w % K == 0 and not args.no_shadow and not args.continuous_shadow \
                        and not args.foreground:
                    with r0_lock:
                        r0_steps[0] += 1
                        due = r0_steps[0] % wl.sync_gap == 0
                    if due:
                        gpu.ss_shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
        if args.single_thread:
            for s in range(first_step, first_step + total_steps):
                one(s)
                if not args.no_shadow and not args.continuous_shadow and \
                        (s + 1 - first_step) % (wl.sync_gap * K) == 0:
                    gpu.ss_shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
            return
        ts = [threading.Thread(target=worker, args=(w,)) for w in range(NS)]
        for t in ts:
            t.start()
        for t in ts:
            t.join()

    if args.continuous_shadow and not args.no_shadow:
        gpu.ss_shadow_start(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
    run(args.warmup, 0)
    torch.cuda.synchronize()
    # Inside the timed region only the two roofline candidates are bracketed (two event pairs
    # per step); the other classes are timed in a short extra pass after the clock stops.
    classes = {"gather": binding.K_GATHER, "row_update_chunk": binding.K_ROW_UPDATE_CHUNK}
    extra = {"row_update_all": binding.K_ROW_UPDATE, "sort_and_segments": binding.K_SORT,
             "mlp_groups": binding.K_MLP, "interaction_fwd": binding.K_INTERACT_FWD,
             "interaction_bwd": binding.K_INTERACT_BWD, "sync_round": binding.K_SYNC}
    if not args.no_kernel_events:
        # every 8th launch of each class is bracketed: enough samples for the average, and the
        # cost of recording events stays out of the throughput being measured
        gpu.ss_profile_sample(8)
        gpu.ss_profile_arm(*classes.values())
    steps0, rounds0, _ = gpu.ss_get_counters()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    steps1, rounds1, _ = gpu.ss_get_counters()
    last_losses = losses.cpu().numpy().astype(float)   # mean log-loss of each stream's last batch

    kernels, roofline = {}, None
    if not args.no_kernel_events:
        for name, kid in classes.items():
            n, ms = gpu.ss_profile_read(kid)
            if n:
                kernels[name] = {"brackets": n, "avg_us": ms / n * 1e3, "total_ms": ms,
                                 "where": "timed region, every 8th launch bracketed"}
        # the two roofline candidates once more with ONE stream active (no queueing behind, and
        # no bandwidth shared with, other streams' kernels): comparable with a profiler's figure
        gpu.ss_profile_sample(1)
        gpu.ss_profile_arm(*classes.values())
        for s in range(24):
            gpu.ss_train_step(0, 0, dev_batches[s % len(dev_batches)], streams[0], losses[0:1])
        alone = {name: gpu.ss_profile_read(kid) for name, kid in classes.items()}
        gpu.ss_profile_arm(*extra.values())
        run(min(args.steps, 10 * wl.sync_gap * K), args.warmup + args.steps)
        for name, kid in extra.items():
            n, ms = gpu.ss_profile_read(kid)
            if n:
                kernels[name] = {"brackets": n, "avg_us": ms / n * 1e3, "total_ms": ms,
                                 "where": "extra pass after the timed region"}
        uniq = [sum(len(np.unique(b.indices[b.offsets[t * wl.batch]:b.offsets[(t + 1) * wl.batch]]))
                    for t in range(wl.num_tables)) for b in host_batches]
        for name in ("gather", "row_update_chunk"):
            if name not in kernels:
                continue
            per = [algorithmic_bytes(name, wl, b, uniq[k]) for k, b in enumerate(host_batches)]
            bpl = float(np.mean(per))
            ach = bpl / (kernels[name]["avg_us"] * 1e-6) / 1e9
            kernels[name].update({"algorithmic_bytes_per_launch": bpl, "GBps": ach,
                                  "frac_of_hbm_peak": ach / HBM_PEAK_GBS})
            n1, ms1 = alone[name]
            if n1:
                us1 = ms1 / n1 * 1e3
                kernels[name].update({"alone_avg_us": us1, "alone_GBps": bpl / us1 / 1e3,
                                      "alone_frac_of_hbm_peak": bpl / us1 / 1e3 / HBM_PEAK_GBS})
        cand = [k for k in ("gather", "row_update_chunk") if k in kernels]
        if cand:
            dom = max(cand, key=lambda k: kernels[k]["total_ms"])
            kd = kernels[dom]
            traffic = MEASURED_TRAFFIC.get(wl.name, {}).get(dom)
            roofline = {"bound": "hbm", "kernel": dom, "achieved": kd["GBps"],
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kd["frac_of_hbm_peak"],
                        "traffic": traffic, "avg_launch_us": kd["avg_us"],
                        "launches": kd["brackets"],
                        "algorithmic_bytes_per_launch": kd["algorithmic_bytes_per_launch"],
                        "alone_avg_launch_us": kd.get("alone_avg_us"),
                        "alone_achieved": kd.get("alone_GBps"),
                        "alone_frac": kd.get("alone_frac_of_hbm_peak"),
                        "profiler_alone_avg_launch_us": PROFILER_ALONE_US.get(wl.name, {}).get(dom),
                        "profiler_alone_frac": (
                            kd["algorithmic_bytes_per_launch"] /
                            (PROFILER_ALONE_US[wl.name][dom] * 1e-6) / 1e9 / HBM_PEAK_GBS
                            if dom in PROFILER_ALONE_US.get(wl.name, {}) else None),
                        "note": "achieved/frac: HIP events inside the timed region, where "
                                f"{NS + 1} streams share the GPU (includes queueing and shared "
                                "bandwidth); alone_*: the same kernel with one stream active; "
                                "profiler_alone_*: rocprofv3's duration of that kernel in a "
                                "one-stream run (committed profile, not measured in this run)"}

    if args.continuous_shadow and not args.no_shadow:
        gpu.ss_shadow_stop()
    rounds = rounds1 - rounds0
    shadow_txt = (f"FOREGROUND {args.foreground_rule.upper()} alpha={wl.alpha}: all worker "
                  f"streams stop for one averaging round every {args.foreground} of their steps"
                  if args.foreground and args.foreground_rule != "easgd" else
                  f"FOREGROUND EASGD alpha={wl.alpha}: every worker stream exchanges with the "
                  f"centre copy on its own stream every {args.foreground} of its steps"
                  if args.foreground else
                  "no shadow sync" if args.no_shadow else
                  f"S-{wl.algo.upper()} alpha={wl.alpha} looping continuously on a shadow stream"
                  if args.continuous_shadow else
                  f"S-{wl.algo.upper()} alpha={wl.alpha} on a shadow stream every {wl.sync_gap} "
                  f"trainer steps")
    out = {
        "metric": "train examples/s on 1 GPU with background sync",
        "value": wl.batch * args.steps / dt,
        "unit": "examples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.batch}, {wl.num_tables} tables, {sum(wl.rows)} "
                               f"rows x d{wl.emb_dim} fp32, Zipf({wl.zipf_s}), bag Poisson("
                               f"{wl.bag_lambda:g})+1, K={K} replicas x {WPR} worker stream(s), "
                               f"{shadow_txt}",
                   "shadow_rounds": int(rounds),
                   "last_batch_logloss": float(last_losses.mean()),
                   "avg_sync_gap": (float((steps1 - steps0).mean()) / rounds) if rounds else None,
                   "host_threads": 1 if args.single_thread else NS},
        "roofline": roofline,
        "kernels": kernels,
    }
    gpu.close()
    del gpu
    torch.cuda.empty_cache()
    if not args.no_sync_isolation:
        out["sync_isolation"] = sync_isolation(binding, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, gen)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
