"""Drive the HIP library and the CPU oracle side by side on the same seeded inputs."""
import numpy as np

import oracle
from paper_2003_03477_amd import binding, synth

FP32_RTOL = 1e-5   # spec bound for fp32 values
BF16_RTOL = 2e-2   # spec bound for values that passed through bf16 MLP GEMMs


def close(got, want, rtol, what, scale=None):
    """|got - want| <= rtol * (|want| + scale), scale = largest magnitude in `want`: the
    bound is relative to each element where that element is large and to the tensor's own
    scale where cancellation made it small.

    fp32 (rtol 1e-5): every element must satisfy it.  bf16 (rtol 2e-2): a ReLU gate is a
    floating-point comparison with zero, and operands that differ in the last fp32 bit can
    round to different bfloat16 values, so a handful of gates per step open on one side and
    not on the other; each flips one hidden unit of one sample.  There the bound must hold
    for all but 0.5 % of the elements and, for the tensor as a whole, in the Frobenius norm."""
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if want.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    sc = float(np.max(np.abs(want))) if scale is None else scale
    err = np.abs(got - want)
    bound = rtol * (np.abs(want) + sc)
    bad = err > bound
    allowed = 0 if rtol <= FP32_RTOL else int(0.005 * want.size)
    if int(bad.sum()) > allowed:
        k = int(np.argmax(err - bound))
        raise AssertionError(f"{what}: {int(bad.sum())}/{want.size} outside rtol {rtol}: worst at "
                             f"{k}: got {got[k]!r} want {want[k]!r} (scale {sc:.3g})")
    if allowed:
        fro = float(np.linalg.norm(got - want)) / max(float(np.linalg.norm(want)), 1e-300)
        assert fro <= rtol, f"{what}: relative Frobenius error {fro:.3g} > {rtol}"


def make_pair(wl, batches, h0=None, rows=None, slots=1, dtype=np.float64):
    """(gpu context, oracle trainer) holding the same initial state."""
    rows = tuple(rows if rows is not None else wl.rows)
    row_base = np.concatenate(([0], np.cumsum(rows)))
    if h0 is None:
        h0 = synth.full_tables_h0(wl)
    w0 = synth.dense_w0(wl)
    max_ids = max(int(b.offsets[-1]) for b in batches) + 64
    gpu = binding.ShadowSync(rows, wl.emb_dim, wl.bot_dims, wl.top_dims, wl.num_replicas,
                             max(b.dense.shape[0] for b in batches), max_ids, slots, wl.bf16,
                             wl.lr_dense, wl.lr_emb, wl.adagrad_eps, wl.seed, pooling=wl.pooling)
    for t in range(len(rows)):
        gpu.ss_write_rows(t, 0, h0[row_base[t]:row_base[t + 1]])
    gpu.ss_init_dense(w0)
    orc = oracle.OracleTrainer(wl.bot_dims, wl.top_dims, row_base, h0, w0, wl.num_replicas,
                               wl.lr_dense, wl.lr_emb, wl.adagrad_eps, dtype=dtype,
                               bf16=wl.bf16, pooling=wl.pooling)
    return gpu, orc


def compare_step(gpu, orc, slot, rtol, step_name, tables_exact=False):
    """Element-wise comparison of one step's intermediates (index work bit-exact).  The
    pooled embeddings are pure fp32 work, so they are held to the fp32 bound whenever the
    tables they read are known to match to that bound (always in fp32 runs; in bf16 runs only
    before the first table update, since later rows carry bf16-level gradient differences)."""
    last = orc.last
    B = last["e"].shape[0]
    for item, key in ((binding.DBG_SORTED_ROWS, "sorted_keys"), (binding.DBG_SORTED_POS, "sorted_pos"),
                      (binding.DBG_SEG_STARTS, "seg_starts"), (binding.DBG_BAG_OF_POS, "bag_of_pos")):
        got = gpu.ss_read_debug(slot, item).astype(np.int64)
        assert np.array_equal(got, np.asarray(last[key], dtype=np.int64)), f"{step_name}: {key} differs"
    assert int(gpu.ss_read_debug(slot, binding.DBG_NUM_UNIQUE)[0]) == len(last["seg_starts"])
    close(gpu.ss_read_debug(slot, binding.DBG_POOLED), last["e"],
          FP32_RTOL if (tables_exact or rtol <= FP32_RTOL) else rtol, f"{step_name}: pooled e")
    close(gpu.ss_read_debug(slot, binding.DBG_INTERACT), last["f"], rtol, f"{step_name}: interaction f")
    close(gpu.ss_read_debug(slot, binding.DBG_LOGITS), last["logit"], rtol, f"{step_name}: logits")
    close(gpu.ss_read_debug(slot, binding.DBG_DENSE_GRAD), last["g"], rtol, f"{step_name}: dense grad")
    close(gpu.ss_read_debug(slot, binding.DBG_POOLED_GRAD), last["de"], rtol, f"{step_name}: de")


def compare_state(gpu, orc, rtol, name, row_base):
    K = orc.W.shape[0]
    for i in range(K):
        close(gpu.ss_read_dense(i), orc.W[i], rtol, f"{name}: replica {i}")
    close(gpu.ss_read_dense(-4), orc.W.mean(axis=0), rtol, f"{name}: replica average")
    close(gpu.ss_read_dense(-1), orc.w_ps, rtol, f"{name}: w_ps")
    close(gpu.ss_read_dense(-2), orc.w_global, rtol, f"{name}: w_global")
    close(gpu.ss_read_dense(-3), orc.v, rtol, f"{name}: v", scale=max(1e-30, float(np.max(np.abs(orc.w_global)))))
    for t in range(len(row_base) - 1):
        n = int(row_base[t + 1] - row_base[t])
        vals, acc = gpu.ss_read_rows(t, np.arange(n))
        close(vals, orc.h[row_base[t]:row_base[t + 1]], rtol, f"{name}: table {t}")
        close(acc, orc.G[row_base[t]:row_base[t + 1]], rtol, f"{name}: adagrad state {t}")


def push_oracle_state(gpu, orc, row_base):
    """Overwrite the device state with the oracle's (rounded to fp32)."""
    for i in range(orc.W.shape[0]):
        gpu.ss_write_dense(i, orc.W[i])
    gpu.ss_write_dense(-1, orc.w_ps)
    gpu.ss_write_dense(-2, orc.w_global)
    gpu.ss_write_dense(-3, orc.v)
    for t in range(len(row_base) - 1):
        gpu.ss_write_rows(t, 0, orc.h[row_base[t]:row_base[t + 1]])
        gpu.ss_write_adagrad(t, 0, orc.G[row_base[t]:row_base[t + 1]])


def push_oracle_state_sparse(gpu, orc, cp, row_base_c):
    """Same, for a full-size device table set against a compacted oracle: only the touched
    rows (contiguous runs of original ids are written in one call)."""
    for i in range(orc.W.shape[0]):
        gpu.ss_write_dense(i, orc.W[i])
    for t, touched in enumerate(cp.touched):
        h = orc.h[row_base_c[t]:row_base_c[t + 1]]
        G = orc.G[row_base_c[t]:row_base_c[t + 1]]
        breaks = np.flatnonzero(np.diff(touched) != 1) + 1
        starts = np.concatenate(([0], breaks))
        ends = np.concatenate((breaks, [len(touched)]))
        for a, b in zip(starts, ends):
            gpu.ss_write_rows(t, int(touched[a]), h[a:b])
            gpu.ss_write_adagrad(t, int(touched[a]), G[a:b])


def run_lockstep(gpu, orc, batches, gap, algo, alpha, eta=1.0, mu=0.0, rtol=FP32_RTOL,
                 check_every=1, loss_rtol=None, resync_row_base=None):
    """The deterministic schedule (one worker per replica, sync at fixed steps) on both.

    With resync_row_base set, every step and every round is checked from a COMMON state: the
    full state is compared after each of them and the device state is then overwritten with
    the oracle's.  bf16 runs need this: row-wise Adagrad's update has magnitude ~lr whatever
    the gradient's scale, so a 1 % gradient difference (bf16 rounding, a flipped ReLU gate)
    becomes a 1e-4 difference in the row and the two trajectories separate beyond the 2e-2
    bound within a few steps, although each single step meets it."""
    K = orc.W.shape[0]
    dev = [binding.upload_batch(b) for b in batches]
    losses = []
    for s in range(len(batches) // K):
        for i in range(K):
            k = s * K + i
            lo = orc.train_step(i, *batches[k].as_tuple())
            lg = float(gpu.ss_train_step(i, 0, dev[k]).cpu()[0])
            losses.append((lg, lo))
            assert abs(lg - lo) <= (loss_rtol or rtol) * abs(lo), f"step {k}: loss {lg} vs {lo}"
            if k % check_every == 0:
                compare_step(gpu, orc, 0, rtol, f"step {k}",
                             tables_exact=(k == 0 or resync_row_base is not None))
            if resync_row_base is not None:
                compare_state(gpu, orc, rtol, f"after step {k}", resync_row_base)
                push_oracle_state(gpu, orc, resync_row_base)
        if (s + 1) % gap == 0:
            orc.shadow_sync(algo, alpha, eta, mu)
            gpu.ss_shadow_sync(algo, alpha, eta, mu)
            if resync_row_base is not None:
                compare_state(gpu, orc, FP32_RTOL, f"after round at sweep {s}", resync_row_base)
                push_oracle_state(gpu, orc, resync_row_base)
    return losses
