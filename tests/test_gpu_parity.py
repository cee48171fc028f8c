"""Parity of the HIP path (through the C ABI) against the CPU oracle on seeded inputs."""
import functools

import numpy as np
import pytest

from paper_2003_03477_amd import binding, synth
import gpu_harness as H
from oracle import sync as osync

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


# ----------------------------------------------------------------------------- sync rules
@pytest.mark.parametrize("K", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("algo", ["easgd", "easgd_literal", "ma", "bmuf", "bmuf_nesterov"])
def test_sync_round_matches_oracle(K, algo):
    torch = _torch()
    P, stride = 4 * 12345, 4 * 12345 + 256      # several blocks, a ragged last block, padded stride
    rng = np.random.default_rng(100 + K)
    W = (rng.standard_normal((K, stride)) * 0.02).astype(np.float32)
    ps, wg, v = [(rng.standard_normal(P) * 0.02).astype(np.float32) for _ in range(3)]
    dW, dps, dwg, dv = [torch.from_numpy(a.copy()).cuda() for a in (W, ps, wg, v)]
    oW, ops, owg, ov = [a.astype(np.float64) for a in (W[:, :P], ps, wg, v)]
    for r in range(3):
        binding.ss_sync_round(algo, K, P, stride, dW, dps, dwg, dv, alpha=0.3, eta=0.7, momentum=0.9)
        if algo == "easgd":
            osync.easgd_round(oW, ops, 0.3)
        elif algo == "easgd_literal":
            osync.easgd_round_literal(oW, ops, 0.3)
        elif algo == "ma":
            osync.ma_round(oW, owg, 0.3)
        elif algo == "bmuf_nesterov":
            osync.bmuf_nesterov_round(oW, owg, ov, 0.3, 0.7, 0.9)
        else:
            osync.bmuf_round(oW, owg, ov, 0.3, 0.7, 0.9)
    torch.cuda.synchronize()
    gW = dW.cpu().numpy()
    H.close(gW[:, :P], oW, H.FP32_RTOL, "replicas")
    assert np.array_equal(gW[:, P:], W[:, P:]), "padding between replicas was written"
    H.close(dps.cpu().numpy(), ops, H.FP32_RTOL, "w_ps")
    H.close(dwg.cpu().numpy(), owg, H.FP32_RTOL, "w_global")
    H.close(dv.cpu().numpy(), ov, H.FP32_RTOL, "v", scale=0.02)


def test_sync_invariants_on_device():
    """Conservation under S-EASGD and replicas == mean under S-MA(alpha=1), measured on the
    device results themselves (fp32 round-off only)."""
    torch = _torch()
    K, P = 8, 1 << 16
    rng = np.random.default_rng(7)
    W = torch.from_numpy((rng.standard_normal((K, P)) * 0.02).astype(np.float32)).cuda()
    ps = torch.from_numpy((rng.standard_normal(P) * 0.02).astype(np.float32)).cuda()
    total0 = W.double().sum(0) + ps.double()
    for _ in range(5):
        binding.ss_sync_round("easgd", K, P, P, W, ps, None, None, alpha=0.05)
    total1 = W.double().sum(0) + ps.double()
    assert float((total1 - total0).abs().max()) < 4 * 2 ** -24 * (K + 1) * 0.1
    wg = torch.zeros(P, device="cuda")
    mean0 = W.double().mean(0)
    binding.ss_sync_round("ma", K, P, P, W, None, wg, None, alpha=1.0)
    assert float((W.double() - mean0).abs().max()) < 1e-7
    assert float((W - W[0]).abs().max()) == 0.0


@pytest.mark.parametrize("algo", ["easgd", "easgd_literal", "ma", "bmuf", "bmuf_nesterov"])
def test_sync_round_streaming_size_matches_oracle(algo):
    """A working set beyond the memory-side cache (K=8 x 8.4M parameters + centre copy, 300 MB):
    the round then runs through the kernel's streaming (non-temporal) instantiation, the one
    the sync-isolation benchmark times.  Every element against the oracle, two rounds."""
    torch = _torch()
    K, P = 8, 8_400_000
    stride = P + 1024
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((K, stride)) * 0.02).astype(np.float32)
    ps, wg, v = [(rng.standard_normal(P) * 0.02).astype(np.float32) for _ in range(3)]
    dW, dps, dwg, dv = [torch.from_numpy(a.copy()).cuda() for a in (W, ps, wg, v)]
    oW, ops, owg, ov = [a.astype(np.float64) for a in (W[:, :P], ps, wg, v)]
    fn = {"easgd": lambda: osync.easgd_round(oW, ops, 0.05),
          "easgd_literal": lambda: osync.easgd_round_literal(oW, ops, 0.05),
          "ma": lambda: osync.ma_round(oW, owg, 0.5),
          "bmuf": lambda: osync.bmuf_round(oW, owg, ov, 0.5, 1.0, 0.9),
          "bmuf_nesterov": lambda: osync.bmuf_nesterov_round(oW, owg, ov, 0.5, 1.0, 0.9)}[algo]
    alpha = 0.05 if algo.startswith("easgd") else 0.5
    for r in range(2):
        binding.ss_sync_round(algo, K, P, stride, dW, dps, dwg, dv, alpha=alpha, eta=1.0, momentum=0.9)
        fn()
    torch.cuda.synchronize()
    gW = dW.cpu().numpy()
    H.close(gW[:, :P], oW, H.FP32_RTOL, "replicas")
    assert np.array_equal(gW[:, P:], W[:, P:]), "padding between replicas was written"
    H.close(dps.cpu().numpy(), ops, H.FP32_RTOL, "w_ps")
    H.close(dwg.cpu().numpy(), owg, H.FP32_RTOL, "w_global")
    H.close(dv.cpu().numpy(), ov, H.FP32_RTOL, "v", scale=0.02)


# ----------------------------------------------------------------------------- table init
def test_hash_table_init_is_bit_identical():
    wl = synth.tiny().scaled(rows=(1000, 37, 4096, 5))
    gpu = binding.from_workload(wl)
    gpu.ss_init_tables_hash()
    for t, n in enumerate(wl.rows):
        rows = np.arange(n)
        vals, acc = gpu.ss_read_rows(t, rows)
        assert np.array_equal(vals, synth.table_rows_h0(wl.seed, t, rows, wl.emb_dim))
        assert not acc.any()


# ----------------------------------------------------------------------------- end to end
def test_tiny_config_deterministic_schedule():
    """Tiny CTR model, fp32, K=2, S-MA(alpha=1) after every sweep, 20 sweeps."""
    wl = synth.tiny()
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(40)]
    gpu, orc = H.make_pair(wl, batches)
    H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha)
    H.compare_state(gpu, orc, H.FP32_RTOL, "after 20 sweeps", wl.row_base)
    steps, rounds, examples = gpu.ss_get_counters()
    assert steps.tolist() == [20, 20] and rounds == 20 and examples == 40 * wl.batch
    # progressive Train NE over the 40 batches (each scored before the model trained on it)
    n, mean, ctr, ne = gpu.ss_metrics_read(0)
    on, omean, octr, one = orc.ne("train")
    assert n == on == 40 * wl.batch and abs(ctr - octr) < 1e-12
    assert abs(mean - omean) <= H.FP32_RTOL * omean and abs(ne - one) <= H.FP32_RTOL * one


@pytest.mark.parametrize("algo,alpha,eta,mu,gap", [("easgd", 0.1, 1.0, 0.0, 2),
                                                   ("bmuf", 0.5, 1.0, 0.9, 1),
                                                   ("bmuf_nesterov", 0.5, 0.8, 0.7, 2),
                                                   ("easgd_literal", 0.2, 1.0, 0.0, 3)])
def test_fp32_other_rules_and_ragged_shapes(algo, alpha, eta, mu, gap):
    """d=64, 3 unequal tables, batch not a multiple of anything, several sort passes."""
    wl = synth.tiny().scaled(batch=203, rows=(70001, 13, 2500), emb_dim=64, bag_lambda=6.0,
                             bot_dims=(13, 40, 64), top_dims=(64 + 6, 33, 17, 1),
                             num_replicas=3, algo=algo, alpha=alpha, eta=eta, mu=mu,
                             sync_gap=gap, zipf_s=1.2)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(12)]
    cp = synth.compact_problem(wl, batches)
    # keep the original (sparse) row ids for the large table so the sort sees wide keys
    gpu, orc = H.make_pair(wl, batches, h0=synth.full_tables_h0(wl))
    H.run_lockstep(gpu, orc, batches, gap, algo, alpha, eta, mu)
    H.compare_state(gpu, orc, H.FP32_RTOL, algo, wl.row_base)
    assert len(cp.touched[0]) > 500


@pytest.mark.parametrize("d", [32, 128])
def test_fp32_other_embedding_widths(d):
    """d = 32 and d = 128: the other lane groupings of the gather, interaction and row-update
    kernels (8 and 32 lanes per row), with hot rows (Zipf 1.3) and long bags."""
    T = 5
    wl = synth.tiny().scaled(batch=150, rows=(4000, 7, 900, 25000, 64), emb_dim=d, bag_lambda=9.0,
                             bot_dims=(13, 24, d), top_dims=(d + T * (T + 1) // 2, 40, 1),
                             num_replicas=2, algo="ma", alpha=0.5, sync_gap=2, zipf_s=1.3)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(8)]
    gpu, orc = H.make_pair(wl, batches, h0=synth.full_tables_h0(wl))
    H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha)
    H.compare_state(gpu, orc, H.FP32_RTOL, f"d={d}", wl.row_base)


@pytest.mark.parametrize("bf16", [False, True])
def test_mean_pooling(bf16):
    """Mean pooling (the pooling of the paper's Section 3.1 example): pooled vectors divided
    by the bag length, member gradients scaled by 1 / length; empty bags included."""
    wl = synth.tiny().scaled(batch=97, rows=(5000, 11, 800), emb_dim=32, bag_lambda=5.0,
                             bot_dims=(13, 48, 32), top_dims=(32 + 6, 64, 24, 1),
                             num_replicas=2, algo="easgd", alpha=0.2, sync_gap=2, zipf_s=1.2,
                             pooling="mean", bf16=bf16)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(8)]
    # empty a few bags of the first batch
    b0 = batches[0]
    lens = np.diff(b0.offsets).copy()
    lens[[0, 5, 97, 200]] = 0
    keep = np.concatenate([np.arange(b0.offsets[i], b0.offsets[i] + lens[i]) for i in range(len(lens))])
    batches[0] = synth.Batch(b0.dense, b0.labels, b0.indices[keep.astype(np.int64)],
                             np.concatenate(([0], np.cumsum(lens))).astype(np.int32))
    gpu, orc = H.make_pair(wl, batches, h0=synth.full_tables_h0(wl))
    if bf16:
        H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha, rtol=H.BF16_RTOL,
                       resync_row_base=wl.row_base)
    else:
        H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha)
        H.compare_state(gpu, orc, H.FP32_RTOL, "mean pooling", wl.row_base)


@pytest.mark.parametrize("bf16", [False, True])
def test_adam_on_the_tables(bf16):
    """Adam as the table optimiser (Section 3.2 names it beside Adagrad): moments per element
    and a step count per row kept beside the rows, rows updated only in the steps that touch
    them; hot rows (Zipf 1.3) take the chunk, stitch and long-run passes.  Every step is checked
    from a common state, in both precisions: m / (sqrt(v) + eps) turns the RELATIVE error of a
    gradient element into an absolute error of the row, however small the element, so free-
    running trajectories separate beyond any bound relative to the table's scale.  eps = 1e-4
    (the gradients here are 1e-4 .. 1e-3) keeps a single step well conditioned."""
    wl = synth.tiny().scaled(batch=160, rows=(5000, 9, 700), emb_dim=32, bag_lambda=7.0,
                             bot_dims=(13, 48, 32), top_dims=(32 + 6, 64, 24, 1),
                             num_replicas=2, algo="ma", alpha=0.5, sync_gap=2, zipf_s=1.3,
                             bf16=bf16, emb_optimizer="adam", adam_betas=(0.9, 0.99),
                             lr_emb=0.003, adagrad_eps=1e-4)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(10)]
    gpu, orc = H.make_pair(wl, batches, h0=synth.full_tables_h0(wl))
    H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha,
                   rtol=H.BF16_RTOL if bf16 else H.FP32_RTOL, resync_row_base=wl.row_base)
    assert orc.G.max() >= 5                      # some row was updated in many steps


@pytest.mark.parametrize("pooling,d", [("sum", 64), ("mean", 16)])
def test_partial_pooling_over_row_shards(pooling, d):
    """Tables split into three row ranges (Section 3.1, "Embedding PS"): every range pools the
    rows it owns, the partial vectors are compared one by one with the oracle's, and their sum
    feeds the rest of the step as usual."""
    T = 3
    wl = synth.tiny().scaled(batch=120, rows=(4001, 5, 700), emb_dim=d, bag_lambda=6.0,
                             bot_dims=(13, 32, d), top_dims=(d + T * (T + 1) // 2, 24, 1),
                             num_replicas=2, algo="ma", alpha=0.5, sync_gap=2, zipf_s=1.2,
                             pooling=pooling, emb_row_shards=3)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(6)]
    gpu, orc = H.make_pair(wl, batches, h0=synth.full_tables_h0(wl))
    H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha)
    H.compare_state(gpu, orc, H.FP32_RTOL, "partial pooling", wl.row_base)


def test_empty_bags_single_sample_and_hot_row():
    """Edge cases: empty bags, batch of one, one row owning a very long segment."""
    wl = synth.tiny().scaled(batch=64, rows=(50, 1000), emb_dim=16, bot_dims=(13, 16),
                             top_dims=(16 + 3, 8, 1), num_replicas=1)
    rng = np.random.default_rng(3)
    B, T = 64, 2

    def make(B, lens_fn, hot=None):
        lengths = np.array([[lens_fn(t, b) for b in range(B)] for t in range(T)])
        offsets = np.concatenate(([0], np.cumsum(lengths.ravel()))).astype(np.int32)
        idx = np.empty(offsets[-1], dtype=np.int32)
        for t in range(T):
            lo, hi = offsets[t * B], offsets[(t + 1) * B]
            idx[lo:hi] = rng.integers(0, wl.rows[t], hi - lo)
            if hot is not None and t == 1:
                idx[lo:hi][rng.random(hi - lo) < 0.9] = hot
        x = rng.standard_normal((B, 13)).astype(np.float32)
        y = (rng.random(B) < 0.3).astype(np.float32)
        return synth.Batch(x, y, idx, offsets)

    batches = [
        make(64, lambda t, b: 0 if (b + t) % 3 == 0 else 2),     # many empty bags
        make(64, lambda t, b: 0),                                # no ids at all
        make(1, lambda t, b: 5),                                 # single sample
        make(64, lambda t, b: 40, hot=7),                        # ~2300 hits on one row
        make(64, lambda t, b: 130 if b == 0 else 1),             # a bag longer than a wave
    ]
    gpu, orc = H.make_pair(wl, batches)
    H.run_lockstep(gpu, orc, batches, 1, "ma", 1.0)
    H.compare_state(gpu, orc, H.FP32_RTOL, "edge cases", wl.row_base)


# The two bf16 MLP code paths: "auto" picks the per-sample-tile fused kernels for these
# widths, "layerwise" forces one 128x128-tile GEMM per layer and pass (also what models
# outside the fused kernels' limits get: test_bf16_no_hidden_top_layer, the Large architecture).
@pytest.mark.parametrize("path", ["auto", "layerwise"])
def test_bf16_mid_scaled(path):
    """Mid CTR architecture (bf16 MLP GEMMs, fp32 master weights) on a compacted table set,
    step by step from a common state, every element of every tensor within the bf16 bound."""
    wl = synth.mid().scaled(batch=500, num_replicas=2, sync_gap=2)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(8)]
    cp = synth.compact_problem(wl, batches)
    gpu, orc = H.make_pair(wl, cp.batches, h0=cp.h0, rows=cp.rows, mlp_path=path)
    row_base = np.concatenate(([0], np.cumsum(cp.rows)))
    H.run_lockstep(gpu, orc, cp.batches, wl.sync_gap, wl.algo, wl.alpha, rtol=H.BF16_RTOL,
                   resync_row_base=row_base)
    print("gates taken the other way:", H.GATE_STATS)


@pytest.mark.parametrize("path", ["auto", "layerwise"])
def test_bf16_odd_widths(path):
    """bf16 with layer widths that are not multiples of the MFMA tile (guards, padding)."""
    wl = synth.tiny().scaled(batch=77, rows=(3000, 17, 900), emb_dim=64, bag_lambda=4.0,
                             bot_dims=(13, 40, 64), top_dims=(64 + 6, 72, 24, 1),
                             num_replicas=1, bf16=True, algo="ma", alpha=1.0)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(4)]
    gpu, orc = H.make_pair(wl, batches, mlp_path=path)
    H.run_lockstep(gpu, orc, batches, 1, "ma", 1.0, rtol=H.BF16_RTOL,
                   resync_row_base=wl.row_base)


def test_bf16_no_hidden_top_layer():
    """A bf16 model whose top MLP is a single linear unit: layer-wise kernels for the bottom
    stack; the output unit reads the interaction output and hands back an fp32, ungated
    gradient w.r.t. it."""
    wl = synth.tiny().scaled(batch=130, rows=(3000, 17, 900), emb_dim=32, bag_lambda=4.0,
                             bot_dims=(13, 72, 40, 32), top_dims=(32 + 6, 1),
                             num_replicas=2, bf16=True, algo="easgd", alpha=0.2, sync_gap=2)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(6)]
    gpu, orc = H.make_pair(wl, batches)
    H.run_lockstep(gpu, orc, batches, wl.sync_gap, wl.algo, wl.alpha, rtol=H.BF16_RTOL,
                   resync_row_base=wl.row_base)


def test_bf16_free_running_mid_scaled():
    """Mid architecture, K=4, S-EASGD every 5 sweeps, 20 sweeps WITHOUT resynchronising the two
    sides: every loss within the bf16 bound of the oracle's, and the final replicas within it
    in the Frobenius norm.  (Element-wise bounds do not survive a free run: row-wise Adagrad
    turns a 1 % gradient difference into a step difference of 1e-4 on rows of magnitude 0.05,
    and undecidable ReLU gates are taken differently; the per-step tests above cover the
    elements.)"""
    wl = synth.mid().scaled(batch=500, num_replicas=4, sync_gap=5)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(80)]
    cp = synth.compact_problem(wl, batches)
    gpu, orc = H.make_pair(wl, cp.batches, h0=cp.h0, rows=cp.rows)
    dev = [binding.upload_batch(b) for b in cp.batches]
    K = 4
    worst = 0.0
    for s in range(20):
        for i in range(K):
            k = s * K + i
            lg = float(gpu.ss_train_step(i, 0, dev[k]).cpu()[0])
            lo = orc.train_step(i, *cp.batches[k].as_tuple())
            worst = max(worst, abs(lg - lo) / lo)
            assert abs(lg - lo) <= H.BF16_RTOL * lo, f"step {k}: loss {lg} vs {lo}"
        if (s + 1) % wl.sync_gap == 0:
            orc.shadow_sync(wl.algo, wl.alpha)
            gpu.ss_shadow_sync(wl.algo, wl.alpha)
    for i in range(K):
        got, want = gpu.ss_read_dense(i).astype(np.float64), orc.W[i]
        fro = np.linalg.norm(got - want) / np.linalg.norm(want)
        assert fro <= H.BF16_RTOL, f"replica {i}: relative Frobenius error {fro}"
    got, want = gpu.ss_read_dense(-1).astype(np.float64), orc.w_ps
    assert np.linalg.norm(got - want) / np.linalg.norm(want) <= H.BF16_RTOL
    print(f"free run: worst relative loss difference {worst:.2e}")


def test_bf16_large_architecture_lockstep_bmuf():
    """The Large architecture (26 tables, 1024-wide top MLP, layer-wise MFMA GEMMs) with ITS
    schedule -- K=4 replicas, S-BMUF alpha 0.5, block lr 1, block momentum 0.9, a round after
    every sweep -- at a reduced batch on compacted tables, two sweeps, every step and every
    round checked element by element from a common state."""
    wl = synth.large().scaled(batch=256)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(8)]
    cp = synth.compact_problem(wl, batches)
    gpu, orc = H.make_pair(wl, cp.batches, h0=cp.h0, rows=cp.rows)
    row_base = np.concatenate(([0], np.cumsum(cp.rows)))
    H.run_lockstep(gpu, orc, cp.batches, wl.sync_gap, wl.algo, wl.alpha, wl.eta, wl.mu,
                   rtol=H.BF16_RTOL, resync_row_base=row_base)
    assert gpu.ss_get_counters()[1] == 2                      # two S-BMUF rounds ran
    print("gates taken the other way:", H.GATE_STATS)


def test_validation_errors_through_the_abi():
    wl = synth.tiny()
    gen = synth.BatchGenerator(wl)
    b = gen.batch(0)
    gpu, _ = H.make_pair(wl, [b])
    dev = binding.upload_batch(b)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_train_step(5, 0, dev)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_train_step(0, 3, dev)
    big = binding.DeviceBatch(dev.dense, dev.labels, dev.indices, dev.offsets, dev.batch, 10 ** 7)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_train_step(0, 0, big)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_shadow_sync(9, 0.1)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_read_dense(17)


# ----------------------------------------------------------------------------- full sizes
def _full_size_step_check(wl, n_batches, rtol):
    """Full-size tables filled by the device hash, the bench's launch configuration; the
    oracle works on the rows the batches touch (order-preserving relabelling), so every
    per-step output can be compared element by element and the touched rows one by one."""
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(n_batches)]
    cp = synth.compact_problem(wl, batches)
    row_base_c = np.concatenate(([0], np.cumsum(cp.rows)))
    gpu = binding.from_workload(wl, num_worker_slots=1,
                                max_ids=max(int(b.offsets[-1]) for b in batches) + 64)
    gpu.ss_init_tables_hash()
    w0 = synth.dense_w0(wl)
    gpu.ss_init_dense(w0)
    import oracle
    orc = oracle.OracleTrainer(wl.bot_dims, wl.top_dims, row_base_c, cp.h0, w0, wl.num_replicas,
                               wl.lr_dense, wl.lr_emb, wl.adagrad_eps, bf16=wl.bf16)
    B = wl.batch
    for k, (b, cb) in enumerate(zip(batches, cp.batches)):
        dev = binding.upload_batch(b)
        lg = float(gpu.ss_train_step(0, 0, dev).cpu()[0])
        lo, flipped = H.oracle_step(gpu, orc, 0, 0, cb.as_tuple())
        print(f"{wl.name} step {k}: undecidable ReLU gates taken the other way: {flipped}")
        assert abs(lg - lo) <= rtol * abs(lo), f"step {k}: loss {lg} vs {lo}"
        last = orc.last
        # sort order: positions bit-exact; keys equal after mapping compact ids back
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SORTED_POS).astype(np.int64),
                              last["sorted_pos"])
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SORTED_BAG).astype(np.int64),
                              np.asarray(last["bag_of_pos"], dtype=np.int64)[last["sorted_pos"]])
        glob = np.concatenate([wl.row_base[t] + cp.touched[t] for t in range(wl.num_tables)])
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SORTED_ROWS).astype(np.int64),
                              glob[last["sorted_keys"]])
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SEG_STARTS).astype(np.int64),
                              last["seg_starts"])
        H.close(gpu.ss_read_debug(0, binding.DBG_POOLED), last["e"],
                H.FP32_RTOL if k == 0 else rtol, f"step {k}: pooled e")
        H.close(gpu.ss_read_debug(0, binding.DBG_LOGITS), last["logit"], rtol, f"step {k}: logits")
        H.close_dense(gpu.ss_read_debug(0, binding.DBG_DENSE_GRAD), last["g"], rtol,
                      f"step {k}: dense grad", orc.layout)
        H.close(gpu.ss_read_debug(0, binding.DBG_POOLED_GRAD), last["de"], rtol, f"step {k}: de")
        H.close_dense(gpu.ss_read_dense(0), orc.W[0], rtol, f"step {k}: replica 0", orc.layout)
        for t in range(wl.num_tables):
            vals, acc = gpu.ss_read_rows(t, cp.touched[t])
            H.close(vals, orc.h[row_base_c[t]:row_base_c[t + 1]], rtol, f"step {k}: table {t} rows")
            # (the accumulator is quadratic in the row gradient: twice its relative error)
            H.close(acc, orc.G[row_base_c[t]:row_base_c[t + 1]], 2 * rtol, f"step {k}: table {t} G")
        # a sample of untouched rows is still the hash value, accumulator still zero
        rng = np.random.default_rng(k)
        for t in range(0, wl.num_tables, 3):
            cand = rng.integers(0, wl.rows[t], 64)
            cand = np.setdiff1d(cand, cp.touched[t])
            vals, acc = gpu.ss_read_rows(t, cand)
            assert np.array_equal(vals, synth.table_rows_h0(wl.seed, t, cand, wl.emb_dim))
            assert not acc.any()
        if k + 1 < len(batches):
            H.push_oracle_state_sparse(gpu, orc, cp, row_base_c)
    gpu.close()


def test_mid_full_size_steps():
    """Mid config at its real sizes (B=2048, 8 x 1e6 x 64 tables, ~344k ids per step)."""
    _full_size_step_check(synth.mid(), 2, H.BF16_RTOL)


def test_large_full_size_step():
    """Large config at its real sizes: 26 tables, ~1.8e8 rows x 64 (46 GB) filled on the
    device, B=8192 (~6.6M ids), 1024-wide top MLP through the layer-wise MFMA GEMMs."""
    _full_size_step_check(synth.large(), 1, H.BF16_RTOL)


# ----------------------------------------------------------------------------- extras
def test_single_trainer_easgd_exchange_and_eval_ne():
    """Algorithm 2 for one trainer (the unit the foreground variant enqueues on a worker
    stream), and the forward-only evaluation whose loss, divided by the label entropy, is the
    paper's normalised entropy."""
    wl = synth.tiny().scaled(num_replicas=3)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(4)]
    gpu, orc = H.make_pair(wl, batches)
    dev = [binding.upload_batch(b) for b in batches]
    for i in range(3):                      # make the replicas differ
        orc.train_step(i, *batches[i].as_tuple())
        gpu.ss_train_step(i, 0, dev[i])
    from oracle import sync as osync
    osync.easgd_round(orc.W[1:2], orc.w_ps, 0.3)
    gpu.ss_easgd_exchange(1, 0.3)
    osync.easgd_round_literal(orc.W[2:3], orc.w_ps, 0.2)
    gpu.ss_easgd_exchange(2, 0.2, algo="easgd_literal")
    H.compare_state(gpu, orc, H.FP32_RTOL, "after single-trainer exchanges", wl.row_base)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_easgd_exchange(1, 0.3, algo="ma")
    # eval: nothing changes, loss matches, NE = loss / H(ctr)
    before = gpu.ss_read_dense(0)
    lg = float(gpu.ss_eval_step(0, 0, dev[3]).cpu()[0])
    lo = orc.eval_logloss(0, *batches[3].as_tuple())
    assert abs(lg - lo) <= H.FP32_RTOL * lo
    assert np.array_equal(before, gpu.ss_read_dense(0))
    # NE (Section 4): the library's running accumulators against the oracle's
    n, mean, ctr, ne = gpu.ss_metrics_read(1)
    on, omean, octr, one = orc.ne("eval")
    assert n == on and abs(ctr - octr) < 1e-12
    assert abs(mean - omean) <= H.FP32_RTOL * omean and abs(ne - one) <= H.FP32_RTOL * one
    n, mean, ctr, ne = gpu.ss_metrics_read(0)           # the three training steps above
    on, omean, octr, one = orc.ne("train")
    assert n == on == 3 * wl.batch and abs(ctr - octr) < 1e-12
    assert abs(ne - one) <= H.FP32_RTOL * one
    gpu.ss_metrics_reset(0)
    assert gpu.ss_metrics_read(0)[0] == 0 and np.isnan(gpu.ss_metrics_read(0)[3])
    assert gpu.ss_metrics_read(1)[0] == wl.batch            # eval accumulator untouched by the reset


@pytest.mark.parametrize("path", ["auto", "layerwise"])
def test_eval_step_bf16_paths(path):
    """Forward-only evaluation through the fused and the layer-wise bf16 kernels: loss and
    logits against the oracle's, nothing updated, and the sorted arrays of the last TRAINING
    step stay readable afterwards although the evaluated batch has another size."""
    wl = synth.mid().scaled(batch=300, num_replicas=2)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(3)]
    small = synth.BatchGenerator(wl.scaled(batch=100)).batch(7)
    cp = synth.compact_problem(wl, batches)
    row_base = np.concatenate(([0], np.cumsum(cp.rows)))
    gpu, orc = H.make_pair(wl, cp.batches, h0=cp.h0, rows=cp.rows, mlp_path=path)
    dev = [binding.upload_batch(b) for b in cp.batches]
    gpu.ss_train_step(1, 0, dev[0])
    H.oracle_step(gpu, orc, 0, 1, cp.batches[0].as_tuple())
    H.push_oracle_state(gpu, orc, row_base)
    sorted_rows = gpu.ss_read_debug(0, binding.DBG_SORTED_ROWS).copy()
    seg = gpu.ss_read_debug(0, binding.DBG_SEG_STARTS).copy()
    before_w = gpu.ss_read_dense(1)
    before_rows = gpu.ss_read_rows(0, np.arange(cp.rows[0]))
    for k in (1, 2):
        lg = float(gpu.ss_eval_step(1, 0, dev[k]).cpu()[0])
        lo = orc.eval_logloss(1, *cp.batches[k].as_tuple())
        assert abs(lg - lo) <= H.BF16_RTOL * lo, f"eval loss {lg} vs {lo}"
        orc.train_step(1, *cp.batches[k].as_tuple(), update=False)
        H.close(gpu.ss_read_debug(0, binding.DBG_LOGITS), orc.last["logit"], H.BF16_RTOL, "eval logits")
        H.close(gpu.ss_read_debug(0, binding.DBG_POOLED), orc.last["e"], H.FP32_RTOL, "eval pooled e")
    # a smaller batch (rows of the same compacted tables: ids folded into range)
    idx = small.indices.copy()
    for t in range(wl.num_tables):
        lo_, hi_ = small.offsets[t * 100], small.offsets[(t + 1) * 100]
        idx[lo_:hi_] %= cp.rows[t]
    sb = synth.Batch(small.dense, small.labels, idx, small.offsets)
    lg = float(gpu.ss_eval_step(1, 0, binding.upload_batch(sb)).cpu()[0])
    lo = orc.eval_logloss(1, *sb.as_tuple())
    assert abs(lg - lo) <= H.BF16_RTOL * lo
    assert np.array_equal(before_w, gpu.ss_read_dense(1))
    after_rows = gpu.ss_read_rows(0, np.arange(cp.rows[0]))
    assert np.array_equal(before_rows[0], after_rows[0]) and np.array_equal(before_rows[1], after_rows[1])
    assert np.array_equal(sorted_rows, gpu.ss_read_debug(0, binding.DBG_SORTED_ROWS))
    assert np.array_equal(seg, gpu.ss_read_debug(0, binding.DBG_SEG_STARTS))


def test_profile_brackets_and_sampling():
    """Event brackets: every launch of an armed class by default, about 1 in n with sampling."""
    import torch
    wl = synth.tiny()
    gen = synth.BatchGenerator(wl)
    b = gen.batch(0)
    gpu = binding.from_workload(wl, num_worker_slots=1, max_ids=int(b.offsets[-1]) + 64)
    gpu.ss_init_tables_hash()
    gpu.ss_init_dense(synth.dense_w0(wl))
    db = binding.upload_batch(b)
    for every, lo, hi in ((1, 64, 64), (4, 6, 32), (8, 2, 20)):
        # sampled launches are picked by a hash of their running number: about 1 in `every`
        gpu.ss_profile_sample(every)
        gpu.ss_profile_arm(binding.K_GATHER, binding.K_ROW_UPDATE)
        for _ in range(64):
            gpu.ss_train_step(0, 0, db, None, None)
        torch.cuda.synchronize()
        n, ms = gpu.ss_profile_read(binding.K_GATHER)
        assert lo <= n <= hi and ms > 0.0, (every, n)
        n2, ms2 = gpu.ss_profile_read(binding.K_ROW_UPDATE)
        assert lo <= n2 <= hi and ms2 > 0.0, (every, n2)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_profile_sample(0)
    gpu.close()


def test_many_small_tables():
    """33 small tables of 60 rows (561 interaction pairs per sample, every row hit many times
    per step): the fp32 lockstep on a shape far from the configured workloads."""
    T = 33
    wl = synth.tiny().scaled(batch=40, rows=(60,) * T, emb_dim=16, bag_lambda=2.0,
                             bot_dims=(13, 24, 16), top_dims=(16 + T * (T + 1) // 2, 32, 1),
                             num_replicas=1, algo="ma", alpha=1.0)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(3)]
    gpu, orc = H.make_pair(wl, batches)
    H.run_lockstep(gpu, orc, batches, 1, "ma", 1.0)
    H.compare_state(gpu, orc, H.FP32_RTOL, "33 tables", wl.row_base)


_SORT_ROWS = (1, 2, 300, 70_000, 600_000, (1 << 20) + 1)


@functools.lru_cache(maxsize=1)
def _sort_width_problem():
    rows = _SORT_ROWS
    T = len(rows)
    wl = synth.tiny().scaled(batch=512, rows=rows, emb_dim=16, bag_lambda=25.0,
                             bot_dims=(13, 24, 16), top_dims=(16 + T * (T + 1) // 2, 32, 1),
                             num_replicas=1, algo="ma", alpha=1.0)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(2)]
    for b in batches:   # every table's last row (the top bit of its widest digit) is hit
        for t in range(T):
            lo, hi = int(b.offsets[t * wl.batch]), int(b.offsets[(t + 1) * wl.batch])
            b.indices[lo + (hi - lo) // 3] = rows[t] - 1
            b.indices[hi - 1] = rows[t] - 1
    return wl, batches, synth.full_tables_h0(wl)


@pytest.mark.parametrize("digit_bits", [8, 9, 10])
def test_sort_digit_widths(digit_bits):
    """The stable sort with every permitted digit width, on tables whose local rows need 1 to
    21 bits (one to three passes each, widths 1 to 10), ~80k ids per step (tiles of 512
    elements, several per table, ragged ends): sorted rows, positions, segment starts and the
    updated rows against the oracle."""
    wl, batches, h0 = _sort_width_problem()
    assert min(int(b.offsets[-1]) for b in batches) > 65536
    gpu, orc = H.make_pair(wl, batches, h0=h0.copy(), sort_digit_bits=digit_bits)
    H.run_lockstep(gpu, orc, batches, 1, "ma", 1.0)
    H.compare_state(gpu, orc, H.FP32_RTOL, f"sort digits of {digit_bits} bits", wl.row_base)
    gpu.close()


@pytest.mark.parametrize("T,d", [(13, 32), (40, 16), (1, 16)])
def test_interaction_shapes(T, d):
    """Shapes that drive the interaction kernels' other branches: 91 pairs in 4x4 blocks shared
    by four lanes (T=13, d=32), 66 blocks in two rounds of the wave (T=40), a single pair
    (T=1); fp32 lockstep against the oracle."""
    wl = synth.tiny().scaled(batch=24, rows=(50,) * T, emb_dim=d, bag_lambda=2.0,
                             bot_dims=(13, 24, d), top_dims=(d + T * (T + 1) // 2, 32, 1),
                             num_replicas=1, algo="ma", alpha=1.0)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(3)]
    gpu, orc = H.make_pair(wl, batches)
    H.run_lockstep(gpu, orc, batches, 1, "ma", 1.0)
    H.compare_state(gpu, orc, H.FP32_RTOL, f"T={T} d={d}", wl.row_base)
    gpu.close()
