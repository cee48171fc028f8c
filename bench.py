#!/usr/bin/env python3
"""Throughput of the ShadowSync hot path on one MI355X.

Headline workload (default): the Large CTR model -- 13 dense features, 26 tables of about
1.8e8 rows x dim 64 fp32 (46 GB) filled on the device, ids Zipf(1.1), bag length Poisson(30)+1,
bottom MLP 13-512-256-64, top MLP 415-1024-1024-512-256-1 with bf16 MFMA GEMMs over fp32 master
weights, batch 8192, K=4 dense replicas, Shadow BMUF (block momentum 0.9, block lr 1.0) looping
on its own stream beside the worker streams.  `--workload mid|hogwild|tiny` selects the others.

One bench STEP = one SWEEP: every worker stream runs one ss_train_step (forward, loss,
backward, SGD on its replica, sort + segmented reduction + row-wise Adagrad on the tables) on
a batch of its own, so a step trains (worker streams x batch) examples; `--steps K` times
exactly K sweeps.  Worker threads exist and every stream is warm before the clock starts.
Inputs are seeded synthetic batches (>= 64 distinct ones, each owned by one stream) resident in
HBM before the clock starts.

Prints ONE JSON line.  Besides the contract fields:
  no_shadow       the same K sweeps with the shadow stream off, and value / that (Section 3.2:
                  training is not stalled by the synchronisation)
  roofline        the kernel class a step spends most time in (all classes ranked, MLP kernels
                  against the bf16 MFMA peak, memory-bound ones against HBM peak), timed with
                  HIP events on the launching streams inside the timed region; the largest
                  MFMA class is reported beside it
  kernels         event timing of every kernel class
  sync_isolation  the three shadow rules on K=8 x 50M-parameter replicas, GB/s vs HBM peak, and
                  the streaming ceiling of this GPU (a plain 800 MB device copy); every
                  HBM-bound figure of the line is also given as a fraction of that ceiling
  cpu_baseline    the numpy oracle on the host cores, on a bounded sample of the same workload
  secondary       the Mid workload's throughput measured the same way (when the headline is Large)
`--sweep widths|gap` adds the Hogwild width sweep (Section 4.4) / the sync gap against the
number of replicas (Section 4.2) as a table inside the JSON.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X datasheet
MFMA_BF16_PEAK_TFLOPS = 2500.0

# worker streams per replica when --workers-per-replica is not given
# worker streams per replica tried by --sweep widths (a Large batch is 50 MB, and no stream
# may see a batch twice: fewer widths there)
WIDTHS = {"large": (1, 2, 3, 4, 6), "mid": (1, 2, 4, 6, 8, 12, 16), "tiny": (1, 2, 4, 8),
          "hogwild": (1, 2, 4, 6, 8, 12, 16)}
DEFAULT_WORKERS = {"large": "1", "mid": "6", "tiny": "2", "hogwild": "8,1,1,1"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30, help="timed sweeps over all worker streams")
    ap.add_argument("--warmup", type=int, default=5, help="untimed sweeps")
    ap.add_argument("--workload", default="large", choices=["large", "mid", "tiny", "hogwild"])
    ap.add_argument("--batches", type=int, default=64, help="distinct batches (at least)")
    ap.add_argument("--workers-per-replica", default=None, metavar="W | W0,W1,..",
                    help="Hogwild worker streams per replica (one number, or one per replica)")
    ap.add_argument("--replicas", type=int, default=0, metavar="K")
    ap.add_argument("--shadow", default="auto", choices=["auto", "paced", "continuous", "off"],
                    help="paced: one round per sync_gap iterations of a replica, enqueued by its "
                         "workers; continuous: the library's shadow thread loops rounds; auto: "
                         "the workload's own (Large, Hogwild: continuous; Mid, Tiny: paced)")
    ap.add_argument("--shadow-period-us", type=int, default=-1,
                    help="continuous shadow loop: rounds start at least this far apart "
                         "(default: 1000 for Large -- about one round per trainer iteration of a "
                         "replica --, 0 = back to back otherwise)")
    ap.add_argument("--foreground", type=int, default=0, metavar="k",
                    help="foreground variant: every k iterations a worker syncs on ITS OWN "
                         "stream (FR-EASGD-k), or all workers stop for a round (ma / bmuf)")
    ap.add_argument("--foreground-rule", default="easgd", choices=["easgd", "ma", "bmuf"])
    ap.add_argument("--sweep", default="none", choices=["none", "widths", "gap", "foreground"])
    ap.add_argument("--mlp-path", default="auto", choices=["auto", "layerwise"],
                    help="bf16 MLP kernels: auto = fused per-sample-tile kernels for widths <= 512")
    ap.add_argument("--sort-digit-bits", type=int, default=0, choices=[0, 8, 9, 10],
                    help="widest digit of a pass of the backward's radix sort (0: library default)")
    ap.add_argument("--serial-warmup", type=int, default=2,
                    help="warm-up sweeps run one stream at a time (at most warmup - 1)")
    ap.add_argument("--no-shadow-off", action="store_true", help="skip the shadow-off region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sync-isolation", action="store_true")
    ap.add_argument("--no-secondary", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--no-fork", action="store_true",
                    help="generate the batches in this process (for runs under a profiler)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------
# inputs
_GEN = None   # the generator the forked workers inherit (its Zipf tables are far too large to
              # send with every task)


_GEN_DIR = None   # hand-off directory (memory-backed where the system has one): a worker leaves
                  # a batch's arrays there instead of pushing 28 MB through the result pipe


def _gen_one(s):
    import numpy as np
    from paper_2003_03477_amd import synth
    bt = _GEN.batch(s)
    if _GEN_DIR is None:
        return bt
    paths = []
    for k, a in enumerate(bt.as_tuple()):
        path = os.path.join(_GEN_DIR, f"b{s}_{k}.npy")
        np.save(path, a)
        paths.append(path)
    return paths


def _collect(item):
    import numpy as np
    from paper_2003_03477_amd import synth
    if not isinstance(item, list):
        return item
    arrays = []
    for path in item:
        arrays.append(np.load(path))
        os.unlink(path)
    return synth.Batch(*arrays)


def progress(msg):
    """One line on stderr per finished stage of the run."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def make_batches(wl, n, fork=True):
    """n seeded batches; large jobs are generated in forked worker processes (the generator's
    Zipf tables are built once, before the fork), which must happen before anything
    initialises the GPU: pass fork=False afterwards."""
    from paper_2003_03477_amd import synth
    gen = synth.BatchGenerator(wl)
    if not fork or wl.mean_ids * n < 5e6:
        return gen, [gen.batch(s) for s in range(n)]
    import multiprocessing as mp
    procs = min(16, n, max(1, (os.cpu_count() or 1)))
    # close + join: the workers leave through their normal exit (terminating them by signal
    # runs whatever handler a profiler preloaded into the process, which can block)
    global _GEN, _GEN_DIR
    import shutil
    import tempfile
    _GEN = gen
    _GEN_DIR = tempfile.mkdtemp(prefix="ss_bench_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
    pool = mp.get_context("fork").Pool(procs)
    try:
        out = []
        for k, item in enumerate(pool.imap(_gen_one, range(n), chunksize=1)):
            out.append(_collect(item))
            if (k + 1) % 32 == 0:
                progress(f"{k + 1} of {n} batches generated")
    finally:
        pool.close()
        pool.join()
        shutil.rmtree(_GEN_DIR, ignore_errors=True)
        _GEN_DIR = None
    return gen, out


# ------------------------------------------------------------------------------------------
# algorithmic work per launch
def mlp_flops(wl):
    """Multiply-add flops per step of the MFMA kernel classes (the one-unit output layer runs
    outside them and is left out: 2*B*256 flops)."""
    layers = [(wl.bot_dims[i], wl.bot_dims[i + 1]) for i in range(len(wl.bot_dims) - 1)]
    first_top = len(layers)
    layers += [(wl.top_dims[i], wl.top_dims[i + 1]) for i in range(len(wl.top_dims) - 2)]
    B = wl.batch
    fwd = sum(2.0 * B * i * o for i, o in layers)
    dgrad = sum(2.0 * B * i * o for k, (i, o) in enumerate(layers) if k != 0)
    return {"mlp_fwd": fwd, "mlp_dgrad": dgrad, "mlp_wgrad": fwd}, first_top


def hbm_bytes(kernel, wl, n_ids, n_unique):
    """Bytes the method itself must move per launch (per id / per bag / per distinct row)."""
    B, T, d = wl.batch, wl.num_tables, wl.emb_dim
    if kernel == "gather":            # per id: row + index; per bag: pooled vector + offset
        return n_ids * (4 * d + 4) + B * T * (4 * d + 4)
    if kernel == "row_update_chunk":  # per occurrence: gradient row + sorted pair;
        return n_ids * (4 * d + 8) + n_unique * (8 * d + 8)   # per row: row r/w + state r/w
    if kernel == "interaction_bwd":   # per sample: df row, V tile read, dV tile written
        F = d + T * (T + 1) // 2
        return B * (4 * F + 2 * (T + 1) * d * 4)
    raise KeyError(kernel)


def measured_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (a line
    `traffic_bytes_per_launch <kernel> <bytes>` in profiles/<workload>_hbm_traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            m = re.match(r"\s*traffic_bytes_per_launch\s+(\S+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == kernel:
                return float(m.group(2))
    except OSError:
        pass
    return None


def profiler_in_region_us(workload, kernel):
    """A profiler's average duration of the class's launches inside the timed region of the same
    command, from the committed rocprofv3 summary (a line `in_region_avg_us <class> <us>` in
    profiles/<workload>_bench_kernel_stats.txt), or None."""
    path = os.path.join(ROOT, "profiles", f"{workload}_bench_kernel_stats.txt")
    try:
        for line in open(path):
            m = re.match(r"\s*in_region_avg_us\s+(\S+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == kernel:
                return float(m.group(2))
    except OSError:
        pass
    return None


# ------------------------------------------------------------------------------------------
def run_workload(args, wl, workers, shadow_mode, steps, warmup, host_batches, events=True,
                 shadow_off=True, tag=""):
    """Build a context, run warm-up + timed sweeps (shadow on, then shadow off), return the
    measurements as a dict.  `workers` = worker streams per replica (list of K ints).
    The first two warm-up sweeps run stream after stream: row-wise Adagrad starts from empty
    accumulators, where every update moves a row by about lr whatever the gradient, and several
    stale workers (of one replica or of several: the tables are shared) doing that to the same
    hot rows at once is the one moment a lock-free run can blow up (it did in the oracle's
    max-staleness schedule too).  A trainer spends a vanishing share of its life there; the
    remaining warm-up sweeps and everything timed run fully concurrent."""
    import numpy as np
    import torch
    from paper_2003_03477_amd import binding, synth

    K = wl.num_replicas
    replica_of = [r for r in range(K) for _ in range(workers[r])]
    NS = len(replica_of)
    assert len(host_batches) >= NS
    max_ids = max(int(b.offsets[-1]) for b in host_batches) + 4096
    gpu = binding.from_workload(wl, num_worker_slots=NS, max_ids=max_ids, mlp_path=args.mlp_path,
                                sort_digit_bits=args.sort_digit_bits)
    gpu.ss_init_tables_hash()
    gpu.ss_init_dense(synth.dense_w0(wl))
    progress(f"{wl.name}{tag}: context ready, {NS} worker streams")
    dev_batches = [binding.upload_batch(b) for b in host_batches]
    # every stream owns a disjoint set of batches: no two streams ever hold the same one
    own = [list(range(w, len(dev_batches), NS)) for w in range(NS)]
    streams = [torch.cuda.Stream() for _ in range(NS)]
    shadow = torch.cuda.Stream()
    total_sweeps = warmup + steps * (2 if shadow_off else 1) + 64
    losses = torch.zeros(NS, total_sweeps, dtype=torch.float32, device="cuda")
    done = [0] * NS                       # sweeps each worker has run so far
    torch.cuda.synchronize()

    fg = args.foreground
    fg_collective = fg and args.foreground_rule != "easgd"
    state = {"shadow_on": shadow_mode != "off" and not fg}
    r_lock = threading.Lock()
    r_steps = [0]
    meet = threading.Barrier(NS)
    arrive = [torch.cuda.Event() for _ in range(NS)]
    release = [torch.cuda.Event()]

    def foreground_collective(w):
        """All worker streams stop, one averaging round runs, all resume (foreground form of
        Algorithms 3 and 4): stream order through events, host threads meet to enqueue them."""
        arrive[w].record(streams[w])
        meet.wait()
        if w == 0:
            for e in arrive:
                shadow.wait_event(e)
            mu = wl.mu if args.foreground_rule == "bmuf" else 0.0
            gpu.ss_shadow_sync(args.foreground_rule, wl.alpha, wl.eta, mu, shadow)
            release[0] = torch.cuda.Event()
            release[0].record(shadow)
        meet.wait()
        streams[w].wait_event(release[0])

    turn = threading.Condition()
    turn_of = [0]

    def worker(w, sweeps, gate, serial=0):
        gate.wait()
        r = replica_of[w]
        for i in range(sweeps):
            j = done[w]
            if i < serial:
                # cold start: the first sweeps run stream after stream (see run_workload's doc)
                with turn:
                    turn.wait_for(lambda: turn_of[0] == i * NS + w)
            gpu.ss_train_step(r, w, dev_batches[own[w][j % len(own[w])]], streams[w],
                              losses[w, j:j + 1])
            if i < serial:
                streams[w].synchronize()
                with turn:
                    turn_of[0] += 1
                    turn.notify_all()
            done[w] = j + 1
            if fg:
                if (j + 1) % fg == 0:
                    if fg_collective:
                        foreground_collective(w)
                    else:
                        gpu.ss_easgd_exchange(r, wl.alpha, streams[w])
            elif shadow_mode == "paced" and state["shadow_on"] and r == 0:
                # one round per sync_gap iterations of replica 0 (all its workers together)
                with r_lock:
                    r_steps[0] += 1
                    due = r_steps[0] % wl.sync_gap == 0
                if due:
                    gpu.ss_shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)

    def region(sweeps, serial=0):
        """Run `sweeps` sweeps on all streams (the first `serial` of them one stream at a time);
        threads are created and parked at a barrier before the clock starts.  Returns seconds."""
        gate = threading.Barrier(NS + 1)
        turn_of[0] = 0
        ts = [threading.Thread(target=worker, args=(w, sweeps, gate, serial)) for w in range(NS)]
        for t in ts:
            t.start()
        torch.cuda.synchronize()
        gate.wait()
        clk = [time.clock_gettime_ns(time.CLOCK_MONOTONIC), time.clock_gettime_ns(time.CLOCK_BOOTTIME)]
        t0 = time.perf_counter()
        for t in ts:
            t.join()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # host clocks at both ends (a profiler's kernel time stamps can be cut to this window)
        state["clock_ns"] = {"monotonic": [clk[0], time.clock_gettime_ns(time.CLOCK_MONOTONIC)],
                             "boottime": [clk[1], time.clock_gettime_ns(time.CLOCK_BOOTTIME)]}
        return dt

    def shadow_loop(on):
        if shadow_mode != "continuous" or fg:
            state["shadow_on"] = on and shadow_mode != "off" and not fg
            return
        if on:
            gpu.ss_shadow_pace(args.shadow_period_us)
            gpu.ss_shadow_start(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
        else:
            gpu.ss_shadow_stop()
        state["shadow_on"] = on

    one = {"gather": binding.K_GATHER, "row_update_chunk": binding.K_ROW_UPDATE_CHUNK,
           "mlp_fwd": binding.K_MLP_FWD, "mlp_dgrad": binding.K_MLP_DGRAD,
           "mlp_wgrad": binding.K_MLP_WGRAD, "interaction_bwd": binding.K_INTERACT_BWD}
    groups = {"row_update_all": binding.K_ROW_UPDATE, "sort_all_passes": binding.K_SORT,
              "mlp_all_kernels_of_a_stage": binding.K_MLP,
              "interaction_fwd": binding.K_INTERACT_FWD, "sync_round": binding.K_SYNC}

    # ---- warm-up: every stream, every kernel, the shadow loop
    shadow_loop(True)
    region(warmup, serial=min(args.serial_warmup, max(warmup - 1, 0)) if NS > 1 else 0)
    progress(f"{wl.name}{tag}: warm-up done")
    # ---- timed region, shadow on
    # brackets cost a few per cent of a step when every launch carries one: every class gets
    # about a hundred over the region (a step launches the gather once and GEMMs a dozen times)
    every = max(1, (steps * NS) // 96)
    if events:
        gpu.ss_profile_sample(every)
        for kid in (binding.K_MLP_FWD, binding.K_MLP_DGRAD):
            gpu.ss_profile_sample_class(kid, max(1, (steps * NS * (7 if wl.name == "large" else 2)) // 96))
        gpu.ss_profile_arm(*one.values())
    per_step_guess = {"mlp_fwd": 7 if wl.name == "large" else 2, "mlp_dgrad": 6 if wl.name == "large" else 2}
    steps0, rounds0, _ = gpu.ss_get_counters()
    dt_on = region(steps)
    clock_on = state.get("clock_ns")
    progress(f"{wl.name}{tag}: timed region done, {wl.batch * NS * steps / dt_on:.4g} examples/s")
    steps1, rounds1, _ = gpu.ss_get_counters()
    kernels = {}
    if events:
        for name, kid in one.items():
            n, ms = gpu.ss_profile_read(kid)
            if n:
                kernels[name] = {"brackets": n, "avg_us": ms / n * 1e3,
                                 "where": "timed region, about one launch in "
                                          f"{max(1, round(steps * NS * per_step_guess.get(name, 1) / max(n, 1)))} bracketed"}
    shadow_loop(False)
    train_ne = gpu.ss_metrics_read(0)
    # ---- the same sweeps with the shadow stream off
    dt_off = None
    if shadow_off and not fg and shadow_mode != "off":
        if events:   # the same brackets as in the shadow-on region, so that the ratio of the
            gpu.ss_profile_arm(*one.values())   # two is the cost of the shadow loop alone
        dt_off = region(steps)
        if events:
            for kid in one.values():
                gpu.ss_profile_read(kid)
    rounds = rounds1 - rounds0
    per_replica = (steps1 - steps0).astype(float)

    # ---- structure of a step (launches per class) and the remaining classes, after the clock
    if events:
        gpu.ss_profile_sample(1)
        gpu.ss_profile_arm(*one.values())
        gpu.ss_train_step(0, 0, dev_batches[own[0][0]], streams[0], losses[0, -1:])
        per_step = {name: gpu.ss_profile_read(kid)[0] for name, kid in one.items()}
        # every one-kernel class once more with ONE stream active (no queueing behind, and no
        # bandwidth or CUs shared with, other streams' kernels)
        gpu.ss_profile_arm(*one.values())
        for j in range(12):
            gpu.ss_train_step(0, 0, dev_batches[own[0][j % len(own[0])]], streams[0], losses[0, -1:])
        alone = {name: gpu.ss_profile_read(kid) for name, kid in one.items()}
        gpu.ss_profile_arm(*groups.values())
        state["shadow_on"] = shadow_mode != "off"
        saved_mode = shadow_mode
        if shadow_mode == "continuous":
            for _ in range(8):
                gpu.ss_shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu, shadow)
        region(min(steps, 8))
        for name, kid in groups.items():
            n, ms = gpu.ss_profile_read(kid)
            if n:
                kernels[name] = {"brackets": n, "avg_us": ms / n * 1e3,
                                 "where": "extra sweeps after the timed regions"}
        flops, _ = mlp_flops(wl)
        n_ids = float(np.mean([int(b.offsets[-1]) for b in host_batches]))
        sample = host_batches[:8]
        n_uniq = float(np.mean([sum(len(np.unique(b.indices[b.offsets[t * wl.batch]:b.offsets[(t + 1) * wl.batch]]))
                                    for t in range(wl.num_tables)) for b in sample]))
        train_steps = steps * NS
        for name, kd in kernels.items():
            if name not in one:
                continue
            lps = max(per_step.get(name, 1), 1)
            kd["launches_per_step"] = lps
            kd["total_ms_in_timed_region"] = kd["avg_us"] * lps * train_steps * 1e-3
            n1, ms1 = alone.get(name, (0, 0.0))
            kd["alone_avg_us"] = (ms1 / n1 * 1e3) if n1 else None
            # (from the committed profile of the same command, not measured in this run: an
            # event pair under several streams also spans queueing, the profiler's does not)
            kd["profiler_in_region_avg_us"] = profiler_in_region_us(wl.name, name)
            if name in flops:
                work = flops[name] / lps
                ach = work / (kd["avg_us"] * 1e-6) / 1e12
                kd.update({"bound": "mfma", "algorithmic_flops_per_launch": work, "TFLOPps": ach,
                           "frac_of_bf16_mfma_peak": ach / MFMA_BF16_PEAK_TFLOPS})
                if kd["alone_avg_us"]:
                    kd["alone_TFLOPps"] = work / (kd["alone_avg_us"] * 1e-6) / 1e12
                    kd["alone_frac_of_bf16_mfma_peak"] = kd["alone_TFLOPps"] / MFMA_BF16_PEAK_TFLOPS
            else:
                work = hbm_bytes(name, wl, n_ids, n_uniq)
                ach = work / (kd["avg_us"] * 1e-6) / 1e9
                tr = measured_traffic(wl.name, name)
                kd.update({"bound": "hbm", "algorithmic_bytes_per_launch": work, "GBps": ach,
                           "frac_of_hbm_peak": ach / HBM_PEAK_GBS,
                           "counter_bytes_per_launch": tr,
                           "counter_frac_of_hbm_peak":
                               (tr / (kd["avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS) if tr else None})
                if kd["alone_avg_us"]:
                    kd["alone_GBps"] = work / (kd["alone_avg_us"] * 1e-6) / 1e9
                    kd["alone_frac_of_hbm_peak"] = kd["alone_GBps"] / HBM_PEAK_GBS
                    kd["alone_counter_frac_of_hbm_peak"] = \
                        (tr / (kd["alone_avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS) if tr else None

    # ---- loss windows
    host_losses = losses.cpu().numpy().astype(float)
    last_j = warmup + steps
    first_win = float(host_losses[:, :max(1, min(warmup, 2))].mean()) if warmup else float(host_losses[:, 0].mean())
    last_win = float(host_losses[:, max(0, last_j - 2):last_j].mean())
    diverged = (not math.isfinite(last_win)) or last_win > 1.5 * max(first_win, math.log(2.0))

    examples = wl.batch * NS * steps
    res = {
        "value": examples / dt_on, "ms_per_step": dt_on / steps * 1e3, "seconds": dt_on,
        "worker_streams": NS, "workers_per_replica": workers, "examples_per_step": wl.batch * NS,
        "shadow_rounds": int(rounds),
        "avg_sync_gap": (float(per_replica.mean()) / rounds) if rounds else None,
        "no_shadow_value": (examples / dt_off) if dt_off else None,
        "shadow_on_over_off": (dt_off / dt_on) if dt_off else None,
        "first_window_logloss": first_win, "last_window_logloss": last_win,
        "diverged": bool(diverged),
        "logloss_per_sweep": [float(v) for v in host_losses[:, :last_j].mean(axis=0)],
        "train_ne": {"examples": train_ne[0], "logloss": train_ne[1], "ctr": train_ne[2],
                     "ne": train_ne[3]},
        "kernels": kernels, "timed_region_host_clock_ns": clock_on,
    }
    gpu.close()
    del gpu, dev_batches, losses
    torch.cuda.empty_cache()
    return res


def pick_roofline(kernels, NS):
    cand = {k: v for k, v in kernels.items() if "total_ms_in_timed_region" in v}
    if not cand:
        return None
    # Ranked by the time a step spends in the class with one stream active (launches per step
    # x duration alone, where an event pair and the profiler agree): with several streams an
    # event pair also spans the launch's wait for free CUs, which inflates a class of many short
    # launches far more than one long kernel (GEMM launches x2.4, the row update x1.25 against
    # the profiler inside the same region) and would rank the classes differently from the
    # profile of the same command.
    def per_step_us(k):
        v = cand[k]
        return (v.get("alone_avg_us") or v["avg_us"]) * v["launches_per_step"]
    dom = max(cand, key=per_step_us)
    kd = cand[dom]
    mfma = kd["bound"] == "mfma"
    mf = {k: v for k, v in cand.items() if v["bound"] == "mfma"}
    top_mfma = max(mf, key=per_step_us) if mf else None
    return {"bound": kd["bound"], "kernel": dom,
            "ranking_us_per_step_one_stream": {k: per_step_us(k) for k in cand},
            "largest_mfma_class": None if top_mfma is None else {
                "kernel": top_mfma, "frac": mf[top_mfma]["frac_of_bf16_mfma_peak"],
                "alone_frac": mf[top_mfma].get("alone_frac_of_bf16_mfma_peak"),
                "avg_launch_us": mf[top_mfma]["avg_us"],
                "alone_avg_launch_us": mf[top_mfma].get("alone_avg_us"),
                "profiler_in_region_avg_launch_us": mf[top_mfma].get("profiler_in_region_avg_us")},
            "achieved": kd["TFLOPps"] if mfma else kd["GBps"],
            "peak": MFMA_BF16_PEAK_TFLOPS if mfma else HBM_PEAK_GBS,
            "unit": "TFLOP/s" if mfma else "GB/s",
            "frac": kd["frac_of_bf16_mfma_peak"] if mfma else kd["frac_of_hbm_peak"],
            "traffic": kd.get("counter_bytes_per_launch"),
            "avg_launch_us": kd["avg_us"], "launches": kd["brackets"],
            "launches_per_step": kd["launches_per_step"],
            "work_per_launch": kd["algorithmic_flops_per_launch"] if mfma else kd["algorithmic_bytes_per_launch"],
            "alone_avg_launch_us": kd.get("alone_avg_us"),
            "profiler_in_region_avg_launch_us": kd.get("profiler_in_region_avg_us"),
            "alone_achieved": kd.get("alone_TFLOPps") if mfma else kd.get("alone_GBps"),
            "alone_frac": kd.get("alone_frac_of_bf16_mfma_peak") if mfma else kd.get("alone_frac_of_hbm_peak"),
            "note": "the one-kernel class a step spends most time in (all classes ranked by "
                    "launches per step x duration with one stream active); achieved / frac: HIP "
                    f"events on the launching streams while {NS} worker streams (+ shadow) share "
                    "the GPU, so queueing and shared bandwidth are included; alone_*: the same "
                    "class with one stream active, measured after the timed regions; MFMA classes "
                    "average over the layers' GEMM shapes (total flops / total time)"}


# ------------------------------------------------------------------------------------------
def cpu_baseline(wl, seconds=20.0):
    """The oracle as it stands on the host cores, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from paper_2003_03477_amd import synth
    B = min(wl.batch, 2048)
    swl = wl.scaled(batch=B)
    gen = synth.BatchGenerator(swl)
    batches = [gen.batch(20_000 + s) for s in range(2)]
    cp = synth.compact_problem(swl, batches)
    row_base = np.concatenate(([0], np.cumsum(cp.rows)))
    orc = oracle.OracleTrainer(wl.bot_dims, wl.top_dims, row_base, cp.h0, synth.dense_w0(wl),
                               wl.num_replicas, wl.lr_dense, wl.lr_emb, wl.adagrad_eps,
                               bf16=wl.bf16)
    t0 = time.perf_counter()
    n = 0
    while True:
        orc.train_step(n % wl.num_replicas, *cp.batches[n % len(cp.batches)].as_tuple())
        n += 1
        if n % (wl.sync_gap * wl.num_replicas) == 0:
            orc.shadow_sync(wl.algo, wl.alpha, wl.eta, wl.mu)
        if time.perf_counter() - t0 > seconds or n >= 64:
            break
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    out = {"value": B * n / dt, "unit": "examples/s", "cores": cores, "kind": "oracle",
           "sample": f"{n} train steps of batch {B} (the workload's batch is {wl.batch}) + sync "
                     f"rounds of the fp64 numpy oracle, tables compacted to the {sum(cp.rows)} "
                     f"touched rows, {dt:.1f} s; BLAS uses up to `cores` threads, the rest one"}
    # the three sync rules on the host: K=8 replicas of 5M parameters (a tenth of the isolation
    # workload), one round each after a warm-up round, algorithmic bytes as counted for the GPU
    from oracle import sync as osync
    Kh, Ph = 8, 5_000_000
    rng = np.random.default_rng(4)
    W = rng.standard_normal((Kh, Ph)) * 0.02
    ps, wg, v = W[0].copy(), W[1].copy(), np.zeros(Ph)
    rules = {"easgd": (lambda: osync.easgd_round(W, ps, 0.05), 8 * (Kh + 1)),
             "ma": (lambda: osync.ma_round(W, wg, 0.5), 8 * Kh),
             "bmuf": (lambda: osync.bmuf_round(W, wg, v, 0.5, 1.0, 0.9), 8 * Kh + 16)}
    host = {}
    for name, (fn, per_param) in rules.items():
        fn()
        t0 = time.perf_counter()
        fn()
        d = time.perf_counter() - t0
        host[name] = {"ms_per_round": d * 1e3, "GBps_algorithmic": per_param * Ph / d / 1e9}
    out["sync_rules_on_host"] = {"config": f"K={Kh} x {Ph} parameters, fp64 numpy, one thread",
                                 **host}
    return out


def sync_isolation(rounds=50):
    """K=8 replicas of 50M fp32 parameters + centre copy: rounds of each rule back to back."""
    import torch
    from paper_2003_03477_amd import binding
    K, P = 8, 50_000_000
    g = torch.Generator(device="cuda").manual_seed(4)
    W = torch.randn(K * P, device="cuda", generator=g) * 0.02
    ps = torch.randn(P, device="cuda", generator=g) * 0.02
    wg = ps.clone()
    v = torch.zeros(P, device="cuda")
    st = torch.cuda.Stream()
    out = {}
    per_param = {"easgd": 8 * (K + 1), "ma": 8 * K, "bmuf": 8 * K + 16}
    kw = {"easgd": dict(alpha=0.05), "ma": dict(alpha=0.5),
          "bmuf": dict(alpha=0.5, eta=1.0, momentum=0.9)}
    for algo in ("easgd", "ma", "bmuf"):
        with torch.cuda.stream(st):
            for _ in range(3):
                binding.ss_sync_round(algo, K, P, P, W, ps, wg, v, stream=st, **kw[algo])
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(rounds):
                binding.ss_sync_round(algo, K, P, P, W, ps, wg, v, stream=st, **kw[algo])
            e1.record(st)
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / rounds
        gbs = per_param[algo] * P / us / 1e3
        out[algo] = {"us_per_round": us, "algorithmic_bytes": per_param[algo] * P,
                     "GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    # the streaming ceiling of this GPU, measured: a plain device-to-device copy of 800 MB
    # (read + write counted), the figure the 8 TB/s datasheet peak is to be read against
    half = K // 2 * P
    with torch.cuda.stream(st):
        for _ in range(3):
            W[half:].copy_(W[:half])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(20):
            W[half:].copy_(W[:half])
        e1.record(st)
    e1.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / 20
    ceiling = 2 * 4 * half / us / 1e3
    out["copy_ceiling"] = {"GBps": ceiling, "frac_of_hbm_peak": ceiling / HBM_PEAK_GBS,
                           "what": f"torch device-to-device copy of {4 * half} bytes, read + write "
                                   "counted, 20 copies back to back"}
    for algo in ("easgd", "ma", "bmuf"):
        out[algo]["frac_of_copy_ceiling"] = out[algo]["GBps"] / ceiling
    out["config"] = f"K={K} replicas x {P} fp32 parameters, {rounds} rounds per rule back to back"
    del W, ps, wg, v
    torch.cuda.empty_cache()
    return out


def annotate_copy_ceiling(out, ceiling):
    """Every HBM-bound figure of the line also as a fraction of the measured copy ceiling."""
    def one(kd):
        if kd and kd.get("bound") == "hbm":
            g = kd.get("GBps", kd.get("achieved"))
            if g is not None:
                kd["frac_of_copy_ceiling"] = g / ceiling
            a = kd.get("alone_GBps", kd.get("alone_achieved"))
            if a is not None:
                kd["alone_frac_of_copy_ceiling"] = a / ceiling
    one(out.get("roofline"))
    for kd in out.get("kernels", {}).values():
        one(kd)
    mid = out.get("secondary", {}).get("mid")
    if mid:
        one(mid.get("roofline"))
        for kd in mid.get("kernels", {}).values():
            one(kd)


def parse_workers(text, K):
    parts = [int(p) for p in str(text).split(",")]
    if len(parts) == 1:
        parts = parts * K
    if len(parts) != K or min(parts) < 0 or sum(parts) < 1:
        raise SystemExit(f"--workers-per-replica needs one number or {K} comma-separated ones")
    return parts


def shadow_mode_of(args, wl):
    if args.shadow != "auto":
        return args.shadow
    return "continuous" if wl.name in ("large", "hogwild") else "paced"


def shadow_text(args, wl, mode):
    if args.foreground and args.foreground_rule != "easgd":
        return (f"FOREGROUND {args.foreground_rule.upper()} alpha={wl.alpha}: all worker streams "
                f"stop for one averaging round every {args.foreground} of their steps")
    if args.foreground:
        return (f"FOREGROUND EASGD alpha={wl.alpha}: every worker exchanges with the centre copy "
                f"on its own stream every {args.foreground} of its steps")
    if mode == "off":
        return "no shadow sync"
    rule = f"S-{wl.algo.upper()} alpha={wl.alpha}" + (f" eta={wl.eta} mu={wl.mu}" if wl.algo == "bmuf" else "")
    if mode == "continuous":
        pace = f", rounds at least {args.shadow_period_us} us apart" if args.shadow_period_us else " back to back"
        return f"{rule} looping on the library's shadow thread and stream{pace}"
    return f"{rule} on a shadow stream, one round per {wl.sync_gap} iterations of a replica"


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K replicas share its HBM); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    from paper_2003_03477_amd import synth

    wl = synth.WORKLOADS[args.workload]()
    if args.replicas:
        wl = wl.scaled(num_replicas=args.replicas)
    K = wl.num_replicas
    workers = parse_workers(args.workers_per_replica or DEFAULT_WORKERS[wl.name], K)
    NS = sum(workers)
    mode = shadow_mode_of(args, wl)
    if args.shadow_period_us < 0:
        args.shadow_period_us = 1000 if wl.name == "large" else 0
    n_batches = max(args.batches, NS)
    # no stream sees a batch twice in the warm-up and the timed region: the loss and NE columns
    # are progressive validation on fresh data (the later regions -- shadow off, one stream
    # alone -- run over the same batches again)
    n_batches = max(n_batches, NS * (args.warmup + args.steps))
    if args.sweep != "none":
        # sweeps compare the loss reached, so no stream may see a batch twice: enough distinct
        # batches for the widest configuration (16 workers on each replica, or 8 replicas x 4)
        gap_w = int(args.workers_per_replica) if (args.workers_per_replica or "").isdigit() else 4
        widest = {"widths": max(WIDTHS[wl.name]) * K, "gap": 8 * gap_w, "foreground": NS}[args.sweep]
        n_batches = max(n_batches, widest * (args.warmup + args.steps))
    n_batches = (n_batches + NS - 1) // NS * NS
    # inputs first: batch generation forks worker processes, which must precede any GPU use
    t_gen = time.perf_counter()
    _, host_batches = make_batches(wl, n_batches, fork=not args.no_fork)
    mid_batches = None
    secondary = wl.name == "large" and not args.no_secondary and args.sweep == "none"
    if secondary:
        mid_wl = synth.mid()
        mid_workers = parse_workers(DEFAULT_WORKERS["mid"], mid_wl.num_replicas)
        _, mid_batches = make_batches(mid_wl, max(64, sum(mid_workers) * (args.warmup + args.steps)),
                                      fork=not args.no_fork)
    t_gen = time.perf_counter() - t_gen
    progress(f"inputs generated in {t_gen:.1f} s")

    res = run_workload(args, wl, workers, mode, args.steps, args.warmup, host_batches,
                       events=not args.no_kernel_events, shadow_off=not args.no_shadow_off)
    out = {
        "metric": "train examples/s on 1 GPU with background sync",
        "value": res["value"], "unit": "examples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.bf16 else "f32", "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: B={wl.batch}, {wl.num_tables} tables, {sum(wl.rows)} rows x "
                        f"d{wl.emb_dim} fp32, Zipf({wl.zipf_s}), bag Poisson({wl.bag_lambda:g})+1, "
                        f"MLP {'-'.join(map(str, wl.bot_dims))} / {'-'.join(map(str, wl.top_dims))}, "
                        f"K={K} replicas, worker streams per replica {workers}, "
                        f"{shadow_text(args, wl, mode)}",
            "step": f"one sweep = one ss_train_step on each of the {NS} worker streams = "
                    f"{res['examples_per_step']} examples",
            "global_batch": res["examples_per_step"], "worker_streams": NS,
            "host_threads": NS, "distinct_batches": n_batches,
            "timed_seconds": res["seconds"],
            "shadow_rounds": res["shadow_rounds"], "avg_sync_gap": res["avg_sync_gap"],
            "first_window_logloss": res["first_window_logloss"],
            "last_window_logloss": res["last_window_logloss"], "diverged": res["diverged"],
            "logloss_per_sweep": res["logloss_per_sweep"],
            "train_ne": res["train_ne"], "input_generation_seconds": t_gen,
            "timed_region_host_clock_ns": res["timed_region_host_clock_ns"],
        },
        "no_shadow": {"value": res["no_shadow_value"], "shadow_on_over_off": res["shadow_on_over_off"],
                      "note": "the same sweeps with the shadow stream idle; Section 3.2 claims "
                              "background sync leaves training throughput unchanged"},
        "roofline": pick_roofline(res["kernels"], NS),
        "kernels": res["kernels"],
    }
    if args.sweep == "widths":
        table = []
        for w in WIDTHS[wl.name]:
            ws = [w] * K
            need = sum(ws)
            hb = host_batches if len(host_batches) >= need else None
            if hb is None:
                _, hb = make_batches(wl, need, fork=False)
            r = run_workload(args, wl, ws, mode, args.steps, args.warmup, hb, events=False,
                             shadow_off=False)
            table.append({"workers_per_replica": w, "worker_streams": need,
                          "examples_per_s": r["value"], "avg_sync_gap": r["avg_sync_gap"],
                          "first_window_logloss": r["first_window_logloss"],
                          "last_window_logloss": r["last_window_logloss"],
                          "train_ne": r["train_ne"]["ne"]})
        out["width_sweep"] = {"what": "Hogwild width (Section 4.4): lock-free worker streams per "
                                      "replica against throughput and the loss reached over the "
                                      "same number of sweeps", "rows": table}
    if args.sweep == "gap":
        table = []
        for k in (2, 4, 8):
            wk = wl.scaled(num_replicas=k)
            ws = parse_workers(str(gap_w), k)
            for period in (0, 200, 1000):
                args.shadow_period_us = period
                r = run_workload(args, wk, ws, "continuous", args.steps, args.warmup, host_batches,
                                 events=False, shadow_off=False)
                table.append({"replicas": k, "shadow_period_us": period,
                              "examples_per_s": r["value"], "shadow_rounds": r["shadow_rounds"],
                              "avg_sync_gap": r["avg_sync_gap"]})
        out["sync_gap_table"] = {"what": "average sync gap (Section 4.2: trainer iterations per "
                                         "sync) against the number of replicas, shadow loop back "
                                         "to back and paced", "rows": table}
    if args.sweep == "foreground":
        table = []
        variants = [("shadow", 0, "easgd"), ("no sync", 0, "easgd"), ("FR-EASGD", 1, "easgd"),
                    ("FR-EASGD", 5, "easgd"), ("FR-EASGD", 30, "easgd"), ("FR-MA", 5, "ma"),
                    ("FR-MA", 1, "ma"), ("FR-BMUF", 5, "bmuf")]
        for name, k, rule in variants:
            args.foreground, args.foreground_rule = k, rule
            m = "off" if name == "no sync" else mode
            r = run_workload(args, wl, workers, m, args.steps, args.warmup, host_batches,
                             events=False, shadow_off=False)
            table.append({"variant": name if not k else f"{name}-{k}", "examples_per_s": r["value"],
                          "shadow_rounds": r["shadow_rounds"], "avg_sync_gap": r["avg_sync_gap"],
                          "last_window_logloss": r["last_window_logloss"],
                          "train_ne": r["train_ne"]["ne"]})
        args.foreground = 0
        out["foreground_table"] = {
            "what": "background (shadow) synchronisation against the foreground variants of "
                    "Section 4 (FR-EASGD-k: every worker exchanges with the centre copy on its own "
                    "stream every k iterations; FR-MA / FR-BMUF: all workers stop for one averaging "
                    "round every k iterations) and against no synchronisation", "rows": table}
    if secondary:
        r = run_workload(args, mid_wl, mid_workers, "paced", args.steps, args.warmup, mid_batches,
                         events=not args.no_kernel_events, shadow_off=not args.no_shadow_off)
        out["secondary"] = {"mid": {
            "value": r["value"], "unit": "examples/s", "ms_per_step": r["ms_per_step"],
            "worker_streams": r["worker_streams"], "examples_per_step": r["examples_per_step"],
            "no_shadow_value": r["no_shadow_value"], "shadow_on_over_off": r["shadow_on_over_off"],
            "avg_sync_gap": r["avg_sync_gap"], "first_window_logloss": r["first_window_logloss"],
            "last_window_logloss": r["last_window_logloss"], "diverged": r["diverged"],
            "roofline": pick_roofline(r["kernels"], r["worker_streams"]), "kernels": r["kernels"]}}
    if not args.no_sync_isolation:
        out["sync_isolation"] = sync_isolation()
        annotate_copy_ceiling(out, out["sync_isolation"]["copy_ceiling"]["GBps"])
        progress("sync isolation done")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
