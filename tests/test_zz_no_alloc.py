"""ss_eval_step_static (forward pass in the library's static scratch array, for callers that
cannot allocate) against ss_eval_step (worker slot in the caller's workspace): same loss and
logits, on two calls in a row, the second with a smaller batch; sizes beyond the array are
rejected with an error."""
import numpy as np
import pytest

from paper_2003_03477_amd import binding, synth

pytestmark = pytest.mark.gpu


def _ctx(wl, batches, mlp_path="auto", max_batch=None):
    rows = wl.rows
    max_ids = max(int(b.offsets[-1]) for b in batches) + 64
    gpu = binding.ShadowSync(rows, wl.emb_dim, wl.bot_dims, wl.top_dims, wl.num_replicas,
                             max_batch or max(b.dense.shape[0] for b in batches), max_ids, 1,
                             wl.bf16, wl.lr_dense, wl.lr_emb, wl.adagrad_eps, wl.seed,
                             pooling=wl.pooling, mlp_path=mlp_path)
    gpu.ss_init_tables_hash()
    gpu.ss_init_dense(synth.dense_w0(wl))
    return gpu


@pytest.mark.parametrize("kind", ["fp32", "bf16_fused", "bf16_layerwise", "bf16_mean_pool"])
def test_static_scratch_eval_matches_slot_eval(kind):
    import torch
    if kind == "fp32":
        wl = synth.tiny().scaled(batch=300, rows=(3000, 17, 900, 64))
        path = "auto"
    else:
        wl = synth.mid().scaled(batch=300, rows=(20_000,) * 8, num_replicas=2,
                                pooling="mean" if kind == "bf16_mean_pool" else "sum")
        path = "layerwise" if kind == "bf16_layerwise" else "auto"
    big = synth.BatchGenerator(wl).batch(0)
    small = synth.BatchGenerator(wl.scaled(batch=100)).batch(1)
    train = synth.BatchGenerator(wl).batch(2)
    gpu = _ctx(wl, [big, small, train], mlp_path=path)
    gpu.ss_train_step(1, 0, binding.upload_batch(train))        # replica 1 differs from w0
    loss_s = torch.zeros(1, device="cuda")
    for b in (big, small):                                       # second call: smaller batch
        dev = binding.upload_batch(b)
        B = b.dense.shape[0]
        want_loss = float(gpu.ss_eval_step(1, 0, dev).cpu()[0])
        want_logits = gpu.ss_read_debug(0, binding.DBG_LOGITS).copy()
        logits_s = torch.full((B,), 7.0, device="cuda")
        gpu.ss_eval_step_static(1, dev, loss_s, logits_s)
        torch.cuda.synchronize()
        got_loss = float(loss_s.cpu()[0])
        # same kernels on the same inputs: only the order of the loss's atomic adds may differ
        assert abs(got_loss - want_loss) <= 1e-6 * abs(want_loss), (kind, B, got_loss, want_loss)
        assert np.array_equal(logits_s.cpu().numpy(), want_logits), (kind, B)
    n, mean, ctr, ne = gpu.ss_metrics_read(1)
    assert n == 2 * (300 + 100)                                  # both entry points feed the eval NE
    gpu.close()


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    wl = synth.mid().scaled(batch=4096, rows=(20_000,) * 8, num_replicas=1, bag_lambda=2.0)
    b = synth.BatchGenerator(wl).batch(0)
    gpu = _ctx(wl, [b])
    loss = torch.zeros(1, device="cuda")
    with pytest.raises(binding.ShadowSyncError, match="static array"):
        gpu.ss_eval_step_static(0, binding.upload_batch(b), loss)
    with pytest.raises(binding.ShadowSyncError):
        gpu.ss_eval_step_static(3, binding.upload_batch(b), loss)   # bad replica
    gpu.close()
