#!/usr/bin/env python3
"""Throughput of the ShadowSync hot path on one MI355X.

Workload (default): the Mid CTR model -- 13 dense features, 8 tables x 1e6 rows x dim 64
fp32, ids Zipf(1.05), bag length Poisson(20)+1, bottom MLP 13-256-128-64, top MLP
100-512-256-1 with bf16 MFMA GEMMs over fp32 master weights, batch 2048, K=4 replicas each
fed by its own worker stream, Shadow EASGD (alpha 0.1) enqueued on a separate stream once per
5 trainer iterations of a replica.  One bench "step" = one ss_train_step on one batch; steps
go round-robin over the K replicas.  Inputs are seeded synthetic batches already resident in
HBM when the clock starts.

Prints ONE JSON line (see README for the fields).
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="mid", choices=["mid", "tiny", "hogwild"])
    ap.add_argument("--batches", type=int, default=16, help="distinct batches cycled through")
    ap.add_argument("--no-shadow", action="store_true", help="run without the shadow stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-kernel", default="gather",
                    choices=["gather", "sort", "row_update", "mlp", "interact", "none"])
    ap.add_argument("--single-thread", action="store_true",
                    help="enqueue all replicas from one host thread")
    return ap.parse_args()


def algorithmic_bytes(kernel, wl, batch_np, n_unique=None):
    """Bytes the method itself must move per launch of `kernel` on this batch."""
    n = int(batch_np.offsets[-1])
    B, T, d = wl.batch, wl.num_tables, wl.emb_dim
    if kernel == "gather":
        # per id: one row (4d) + its index (4) + sort key and pooled-vector id written (8);
        # per bag: pooled vector written (4d) + its offset (4)
        return n * (4 * d + 4 + 8) + B * T * (4 * d + 4)
    if kernel == "row_update":
        # per occurrence: de row (4d) + sorted position and bag id (8); per distinct row:
        # row read + written (8d) + accumulator read + written (8) + key and segment start (8)
        return n * (4 * d + 8) + n_unique * (8 * d + 16)
    if kernel == "sort":
        passes = 3
        return n * 16 * passes + n * 4  # key+value read and written per pass, + segment scan
    return None


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
        if steps % (5 * wl.num_replicas) == 0:
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
            "sample": f"{steps} train steps of batch {wl.batch} (fp64 numpy oracle, tables "
                      f"compacted to the {sum(cp.rows)} touched rows) in {dt:.1f} s"}


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
    K = wl.num_replicas
    gen = synth.BatchGenerator(wl)
    host_batches = [gen.batch(s) for s in range(args.batches)]
    max_ids = max(int(b.offsets[-1]) for b in host_batches) + 4096
    gpu = binding.from_workload(wl, num_worker_slots=K, max_ids=max_ids)
    gpu.ss_init_tables_hash()
    gpu.ss_init_dense(synth.dense_w0(wl))
    dev_batches = [binding.upload_batch(b) for b in host_batches]
    streams = [torch.cuda.Stream() for _ in range(K)]
    shadow = torch.cuda.Stream()
    losses = torch.zeros(K, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def run(total_steps, first_step):
        """Round-robin: step s trains replica s % K on stream s % K (one host thread per
        replica, as a trainer's worker threads would)."""
        def worker(i):
            mine = range(first_step + i, first_step + total_steps, K)
            for j, s in enumerate(mine):
                gpu.ss_train_step(i, i, dev_batches[s % len(dev_batches)], streams[i],
                                  losses[i:i + 1])
                if i == 0 and not args.no_shadow and (j + 1) % wl.sync_gap == 0:
                    gpu.ss_shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
        if args.single_thread:
            for s in range(first_step, first_step + total_steps):
                i = s % K
                gpu.ss_train_step(i, i, dev_batches[s % len(dev_batches)], streams[i],
                                  losses[i:i + 1])
                if not args.no_shadow and (s + 1) % (wl.sync_gap * K) == 0:
                    gpu.ss_shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
            return
        ts = [threading.Thread(target=worker, args=(i,)) for i in range(K)]
        for t in ts:
            t.start()
        for t in ts:
            t.join()

    run(args.warmup, 0)
    torch.cuda.synchronize()
    kid = {"gather": binding.K_GATHER, "sort": binding.K_SORT, "row_update": binding.K_ROW_UPDATE,
           "mlp": binding.K_MLP, "interact": binding.K_INTERACT, "none": binding.K_NONE}[args.profile_kernel]
    if kid:
        gpu.ss_profile_arm(kid)
    steps0, rounds0, _ = gpu.ss_get_counters()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    steps1, rounds1, _ = gpu.ss_get_counters()
    launches, kernel_ms = gpu.ss_profile_read() if kid else (0, 0.0)

    roofline = None
    if kid and launches and args.profile_kernel in ("gather", "row_update", "sort"):
        # average algorithmic bytes over the batches cycled through
        uniq = None
        if args.profile_kernel == "row_update":
            uniq = [sum(len(np.unique(b.indices[b.offsets[t * wl.batch]:b.offsets[(t + 1) * wl.batch]]))
                        for t in range(wl.num_tables)) for b in host_batches]
        per = [algorithmic_bytes(args.profile_kernel, wl, b, None if uniq is None else uniq[k])
               for k, b in enumerate(host_batches)]
        bytes_per_launch = float(np.mean(per))
        avg_s = kernel_ms / launches / 1e3
        achieved = bytes_per_launch / avg_s / 1e9
        roofline = {"bound": "hbm", "kernel": args.profile_kernel, "achieved": achieved,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": None, "avg_launch_us": avg_s * 1e6, "launches": launches,
                    "algorithmic_bytes_per_launch": bytes_per_launch}
    elif kid and launches:
        roofline = {"bound": "mfma" if args.profile_kernel == "mlp" else "hbm",
                    "kernel": args.profile_kernel, "achieved": None, "peak": None, "unit": None,
                    "frac": None, "traffic": None, "avg_launch_us": kernel_ms / launches * 1e3,
                    "launches": launches}

    rounds = rounds1 - rounds0
    out = {
        "metric": "train examples/s on 1 GPU with background sync",
        "value": wl.batch * args.steps / dt,
        "unit": "examples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.batch}, {wl.num_tables} tables x {wl.rows[0]} "
                               f"rows x d{wl.emb_dim} fp32, Zipf({wl.zipf_s}), bag Poisson("
                               f"{wl.bag_lambda:g})+1, K={K} replicas on {K} worker streams, "
                               f"{'no shadow sync' if args.no_shadow else 'S-' + wl.algo.upper() + ' alpha=' + str(wl.alpha) + ' on a shadow stream every ' + str(wl.sync_gap) + ' trainer steps'}",
                   "shadow_rounds": int(rounds),
                   "avg_sync_gap": (float((steps1 - steps0).mean()) / rounds) if rounds else None,
                   "host_threads": 1 if args.single_thread else K},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, gen)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
