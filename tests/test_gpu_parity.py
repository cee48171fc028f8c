"""Parity of the HIP path (through the C ABI) against the CPU oracle on seeded inputs."""
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


def _select_mlp_path(path, monkeypatch):
    """fused: per-sample-tile kernels; wide: one 128x128-tile GEMM per layer and pass;
    generic: the layout-agnostic GEMM that serves every remaining bf16 model."""
    if path in ("wide", "generic"):
        monkeypatch.setenv("SS_NO_FUSED_MLP", "1")
    if path == "generic":
        monkeypatch.setenv("SS_NO_WIDE_GEMM", "1")


@pytest.mark.parametrize("path", ["fused", "wide", "generic"])
def test_bf16_mid_scaled(path, monkeypatch):
    """Mid CTR architecture (bf16 MLP GEMMs, fp32 master weights) on a compacted table set,
    through each of the three bf16 MLP code paths."""
    _select_mlp_path(path, monkeypatch)
    wl = synth.mid().scaled(batch=500, num_replicas=2, sync_gap=2)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(8)]
    cp = synth.compact_problem(wl, batches)
    gpu, orc = H.make_pair(wl, cp.batches, h0=cp.h0, rows=cp.rows)
    row_base = np.concatenate(([0], np.cumsum(cp.rows)))
    H.run_lockstep(gpu, orc, cp.batches, wl.sync_gap, wl.algo, wl.alpha, rtol=H.BF16_RTOL,
                   resync_row_base=row_base)


@pytest.mark.parametrize("path", ["fused", "wide", "generic"])
def test_bf16_odd_widths(path, monkeypatch):
    """bf16 with layer widths that are not multiples of the MFMA tile (guards, padding)."""
    _select_mlp_path(path, monkeypatch)
    wl = synth.tiny().scaled(batch=77, rows=(3000, 17, 900), emb_dim=64, bag_lambda=4.0,
                             bot_dims=(13, 40, 64), top_dims=(64 + 6, 72, 24, 1),
                             num_replicas=1, bf16=True, algo="ma", alpha=1.0)
    gen = synth.BatchGenerator(wl)
    batches = [gen.batch(s) for s in range(4)]
    gpu, orc = H.make_pair(wl, batches)
    H.run_lockstep(gpu, orc, batches, 1, "ma", 1.0, rtol=H.BF16_RTOL,
                   resync_row_base=wl.row_base)


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
        lo = orc.train_step(0, *cb.as_tuple())
        lg = float(gpu.ss_train_step(0, 0, dev).cpu()[0])
        assert abs(lg - lo) <= rtol * abs(lo), f"step {k}: loss {lg} vs {lo}"
        last = orc.last
        # sort order: positions bit-exact; keys equal after mapping compact ids back
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SORTED_POS).astype(np.int64),
                              last["sorted_pos"])
        glob = np.concatenate([wl.row_base[t] + cp.touched[t] for t in range(wl.num_tables)])
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SORTED_ROWS).astype(np.int64),
                              glob[last["sorted_keys"]])
        assert np.array_equal(gpu.ss_read_debug(0, binding.DBG_SEG_STARTS).astype(np.int64),
                              last["seg_starts"])
        H.close(gpu.ss_read_debug(0, binding.DBG_POOLED), last["e"],
                H.FP32_RTOL if k == 0 else rtol, f"step {k}: pooled e")
        H.close(gpu.ss_read_debug(0, binding.DBG_LOGITS), last["logit"], rtol, f"step {k}: logits")
        H.close(gpu.ss_read_debug(0, binding.DBG_DENSE_GRAD), last["g"], rtol, f"step {k}: dense grad")
        H.close(gpu.ss_read_debug(0, binding.DBG_POOLED_GRAD), last["de"], rtol, f"step {k}: de")
        H.close(gpu.ss_read_dense(0), orc.W[0], rtol, f"step {k}: replica 0")
        for t in range(wl.num_tables):
            vals, acc = gpu.ss_read_rows(t, cp.touched[t])
            H.close(vals, orc.h[row_base_c[t]:row_base_c[t + 1]], rtol, f"step {k}: table {t} rows")
            H.close(acc, orc.G[row_base_c[t]:row_base_c[t + 1]], rtol, f"step {k}: table {t} G")
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
    ctr = float(batches[3].labels.mean())
    ne_gpu = binding.normalized_entropy(lg, ctr)
    ent = -(ctr * np.log(ctr) + (1 - ctr) * np.log(1 - ctr))
    assert abs(ne_gpu - lo / ent) < 1e-5


def test_profile_brackets_and_sampling():
    """Event brackets: every launch of an armed class by default, every n-th with sampling."""
    import torch
    wl = synth.tiny()
    gen = synth.BatchGenerator(wl)
    b = gen.batch(0)
    gpu = binding.from_workload(wl, num_worker_slots=1, max_ids=int(b.offsets[-1]) + 64)
    gpu.ss_init_tables_hash()
    gpu.ss_init_dense(synth.dense_w0(wl))
    db = binding.upload_batch(b)
    for every, want in ((1, 16), (4, 4), (5, 4)):
        gpu.ss_profile_sample(every)
        gpu.ss_profile_arm(binding.K_GATHER, binding.K_ROW_UPDATE)
        for _ in range(16):
            gpu.ss_train_step(0, 0, db, None, None)
        torch.cuda.synchronize()
        n, ms = gpu.ss_profile_read(binding.K_GATHER)
        assert n == want and ms > 0.0
        n2, ms2 = gpu.ss_profile_read(binding.K_ROW_UPDATE)
        assert n2 == want and ms2 > 0.0
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_profile_sample(0)
    gpu.close()
