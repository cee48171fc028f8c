"""Hogwild mode: several lock-free worker streams on one replica plus a continuously looping
shadow stream.  The racy run has no unique result, so the check is statistical: the
window-averaged log-loss curve of the device run must stay within 1 % of the oracle's curve over
the same batches, sync rounds spread evenly at the device run's measured rate of rounds per
step.  The oracle's curve is taken for the two extreme interleavings of a lock-free run (fully
serialised workers; workers of a replica that all start a round from the same state), which
differ by about half a percent themselves; the device run has to lie within 1 % of that band."""
import threading

import numpy as np
import pytest

import oracle
from paper_2003_03477_amd import binding, synth

pytestmark = pytest.mark.gpu


def test_hogwild_logloss_curve_tracks_serialised_oracle():
    import torch
    # Mid architecture, heavy row contention (Zipf 1.3), shrunk so the oracle runs in seconds
    wl = synth.hogwild().scaled(batch=256, rows=(20_000,) * 8, bag_lambda=6.0, num_replicas=2)
    W0, W1 = 4, 1                      # worker streams on replica 0 / replica 1
    S = 30                             # steps per worker
    NW = W0 + W1
    gen = synth.BatchGenerator(wl)
    batches = [[gen.batch(s * NW + w) for s in range(S)] for w in range(NW)]
    max_ids = max(int(b.offsets[-1]) for bs in batches for b in bs) + 64
    # first launches of every kernel (code loading) happen on a throw-away context, so that the
    # measured run starts with all workers moving at their steady pace
    warm = binding.from_workload(wl, num_worker_slots=1, max_ids=max_ids)
    warm.ss_init_tables_hash()
    warm.ss_init_dense(synth.dense_w0(wl))
    wb = binding.upload_batch(batches[0][0])
    for _ in range(3):
        warm.ss_train_step(0, 0, wb, None, None)
    warm.ss_shadow_sync(wl.algo, wl.alpha)
    torch.cuda.synchronize()
    warm.close()
    gpu = binding.from_workload(wl, num_worker_slots=NW, max_ids=max_ids)
    gpu.ss_init_tables_hash()
    w0 = synth.dense_w0(wl)
    gpu.ss_init_dense(w0)
    dev = [[binding.upload_batch(b) for b in bs] for bs in batches]
    streams = [torch.cuda.Stream() for _ in range(NW)]
    shadow = torch.cuda.Stream()
    losses = torch.zeros(NW, S, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    go = threading.Barrier(NW)

    def worker(w):
        replica = 0 if w < W0 else 1
        go.wait()
        for s in range(S):
            gpu.ss_train_step(replica, w, dev[w][s], streams[w], losses[w, s:s + 1])

    gpu.ss_shadow_start(wl.algo, wl.alpha, stream=shadow)
    ts = [threading.Thread(target=worker, args=(w,)) for w in range(NW)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    torch.cuda.synchronize()
    gpu.ss_shadow_stop()
    steps, rounds, examples = gpu.ss_get_counters()
    assert steps.tolist() == [W0 * S, W1 * S] and examples == NW * S * wl.batch
    assert rounds >= 1
    got = losses.cpu().numpy().astype(np.float64)          # [worker, step]
    assert np.all(np.isfinite(got)) and np.all(got > 0)

    # Oracle, two interleavings of the same lock-free run on the same batches, sync rounds
    # spread evenly at the measured rate:
    #   serial:     worker 0's batch, worker 1's batch, ... each on the fully updated state;
    #   concurrent: the W0 workers of replica 0 start every round from the SAME state and
    #               their changes (dense replica, touched rows, Adagrad accumulators) are summed,
    #               i.e. every worker computes on weights that miss its peers' current updates.
    # A real run lies between the two: how far depends on how the streams happen to overlap.
    per_step = rounds / float(NW * S)      # sync rounds per global step (either side of 1)

    def make_oracle():
        return oracle.OracleTrainer(wl.bot_dims, wl.top_dims, wl.row_base,
                                    synth.full_tables_h0(wl), w0, wl.num_replicas, wl.lr_dense,
                                    wl.lr_emb, wl.adagrad_eps, bf16=wl.bf16)

    def run_oracle(concurrent):
        orc = make_oracle()
        out = np.zeros_like(got)
        due = 0.0
        for s in range(S):
            if concurrent:
                rows = np.unique(np.concatenate([
                    oracle.dlrm.global_rows(wl.row_base, batches[w][s].indices, batches[w][s].offsets,
                                            wl.batch) for w in range(W0)]))
                W_s, h_s, G_s = orc.W[0].copy(), orc.h[rows].copy(), orc.G[rows].copy()
                dW, dh, dG = np.zeros_like(W_s), np.zeros_like(h_s), np.zeros_like(G_s)
                for w in range(W0):
                    orc.W[0][:] = W_s; orc.h[rows] = h_s; orc.G[rows] = G_s
                    out[w, s] = orc.train_step(0, *batches[w][s].as_tuple())
                    dW += orc.W[0] - W_s; dh += orc.h[rows] - h_s; dG += orc.G[rows] - G_s
                orc.W[0][:] = W_s + dW; orc.h[rows] = h_s + dh; orc.G[rows] = G_s + dG
                for w in range(W0, NW):
                    out[w, s] = orc.train_step(1, *batches[w][s].as_tuple())
            else:
                for w in range(NW):
                    out[w, s] = orc.train_step(0 if w < W0 else 1, *batches[w][s].as_tuple())
            for _ in range(NW):
                due += per_step
                while due >= 1.0:
                    orc.shadow_sync(wl.algo, wl.alpha)
                    due -= 1.0
        return out

    win = 10                               # windows of 10 steps = 50 batches, all workers

    def curve(x):
        return x.mean(axis=0).reshape(S // win, win).mean(axis=1)

    gc, sc, cc = curve(got), curve(run_oracle(False)), curve(run_oracle(True))
    lo, hi = np.minimum(sc, cc), np.maximum(sc, cc)
    print(f"hogwild windows: device {gc}, oracle serial {sc}, oracle concurrent {cc}, "
          f"rel to serial {(gc - sc) / sc}, rounds {rounds}")
    # within 1 % of the oracle's curve, the oracle's curve being the band between its two
    # interleavings
    assert np.all(gc > 0.99 * lo) and np.all(gc < 1.01 * hi), \
        f"log-loss curves differ: device {gc}, oracle serial {sc}, concurrent {cc}"
    assert np.all(np.abs(cc - sc) / sc < 0.01)              # the band itself is narrow
    assert sc[-1] < sc[0] and gc[-1] < gc[0]                # the model is actually learning
    gpu.close()
