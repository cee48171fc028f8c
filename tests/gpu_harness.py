"""Drive the HIP library and the CPU oracle side by side on the same seeded inputs."""
import numpy as np

import oracle
from paper_2003_03477_amd import binding, synth

FP32_RTOL = 1e-5   # spec bound for fp32 values
BF16_RTOL = 2e-2   # spec bound for values that passed through bf16 MLP GEMMs


def close(got, want, rtol, what, scale=None):
    """Every element: |got - want| <= rtol * max(|want|, floor), floor = the largest magnitude
    in `want` (or `scale`): relative to the element where it is the tensor's largest, and
    relative to the tensor's own scale where cancellation made an element small.  No element
    is exempt, in either precision: in bf16 runs the ReLU gates that fp32 accumulation cannot
    decide are aligned first (align_gates), everything that remains is continuous."""
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if want.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    floor = float(np.max(np.abs(want))) if scale is None else scale
    err = np.abs(got - want)
    bound = rtol * np.maximum(np.abs(want), floor)
    bad = err > bound
    if bad.any():
        k = int(np.argmax(err - bound))
        raise AssertionError(f"{what}: {int(bad.sum())}/{want.size} outside rtol {rtol}: worst at "
                             f"{k}: got {got[k]!r} want {want[k]!r} (floor {floor:.3g})")


def close_dense(got, want, rtol, what, layout):
    """The dense vector layer by layer (each weight matrix and each bias vector against its own
    scale: gradients of different layers differ by orders of magnitude)."""
    pos = 0
    for li, (o, i) in enumerate(layout.layer_shapes()):
        wmax = float(np.max(np.abs(want[pos:pos + o * i])))
        close(got[pos:pos + o * i], want[pos:pos + o * i], rtol, f"{what}: layer {li} W")
        pos += o * i
        # a bias (gradient) is a sum over the batch with heavy cancellation (for the output
        # unit: sum of p - y); its floor is the larger of its own and its layer's weight scale
        bmax = float(np.max(np.abs(want[pos:pos + o])))
        close(got[pos:pos + o], want[pos:pos + o], rtol, f"{what}: layer {li} b",
              scale=max(bmax, wmax))
        pos += o
    assert pos == len(want)


GATE_STATS = {"steps": 0, "flipped": 0}


def align_gates(gpu, orc, slot, replica, x):
    """bf16 runs.  The oracle has just run the step's forward pass (orc.last, no update) on the
    batch whose dense features are x.  Read the device's stored activation of every ReLU
    layer, compare it with the oracle's element by element (bf16 bound), and list the units
    whose gate (activation > 0) the device took the other way.  A ReLU gate is a floating-point
    comparison with zero, so the device's decision is checked for VALIDITY, not for equality:
    it must be the right decision for the device's own input row of that layer (the stored
    bf16 activation of the layer below, itself just checked against the oracle) unless the
    exact pre-activation z' = sum_k a_k w_k + b of that row lies within the worst-case error of
    accumulating its n exact bf16 x bf16 products in fp32 in any order,
        |z'| <= n * 2^-24 * (sum_k |a_k w_k| + |b|).
    (The device's input row may differ from the oracle's in the last bfloat16 bit of isolated
    elements whose fp32 values straddle a rounding boundary; deeper layers inherit more of
    those, which is why the decision is judged on the device's row.)  Anything else fails.
    Returns the flips for OracleTrainer.train_step(gate_flips=...) and their number."""
    import oracle.dlrm as D
    L = orc.layout
    last = orc.last
    layers = L.unpack(orc.W[replica])
    nb = L.n_bot
    n_layers = len(layers)
    acts = [last["acts_bot"][i + 1] for i in range(nb)] + \
           [last["acts_top"][i + 1] for i in range(n_layers - nb)]
    flips = {}
    total = 0
    dev_in = np.asarray(x, dtype=np.float32)
    for l in range(n_layers - 1):
        item = binding.DBG_Z0 if l == nb - 1 else binding.DBG_HIDDEN_ACT + l
        want = acts[l]
        got = gpu.ss_read_debug(slot, item).reshape(want.shape)
        close(got, want, BF16_RTOL, f"activation of layer {l}")
        if l == nb:
            dev_in = gpu.ss_read_debug(slot, binding.DBG_INTERACT).reshape(want.shape[0], -1)
        diff = (got > 0) != (want > 0)
        if diff.any():
            bb, uu = np.nonzero(diff)
            W, bias = layers[l]
            a = D.bf16_round(dev_in[bb]).astype(np.float64)          # [m, in]
            w = D.bf16_round(W[uu]).astype(np.float64)               # [m, in]
            terms = np.abs(a * w)
            z = (a * w).sum(axis=1) + bias[uu]
            tol = W.shape[1] * 2.0 ** -24 * (terms.sum(axis=1) + np.abs(bias[uu]))
            wrong = ((z > 0) != (got[bb, uu] > 0)) & (np.abs(z) > tol)
            assert not wrong.any(), (
                f"layer {l}: {int(wrong.sum())} ReLU gate(s) decided against the device's own "
                f"input beyond fp32 accumulation error, e.g. sample {bb[wrong][0]} unit "
                f"{uu[wrong][0]}: z' = {z[wrong][0]:.3e}, tolerance {tol[wrong][0]:.3e}")
            flips[l] = (bb, uu)
            total += len(bb)
        dev_in = got
    GATE_STATS["steps"] += 1
    GATE_STATS["flipped"] += total
    return flips, total


def oracle_step(gpu, orc, slot, replica, batch_tuple):
    """The oracle's train step for a batch the device has just trained on `slot`.  bf16: the
    undecidable ReLU gates are taken the way the device took them (after checking that they
    are undecidable)."""
    if not orc.bf16:
        return orc.train_step(replica, *batch_tuple), 0
    orc.train_step(replica, *batch_tuple, update=False)
    flips, n = align_gates(gpu, orc, slot, replica, batch_tuple[0])
    return orc.train_step(replica, *batch_tuple, gate_flips=flips), n


def make_pair(wl, batches, h0=None, rows=None, slots=1, dtype=np.float64, mlp_path="auto",
              sort_digit_bits=0):
    """(gpu context, oracle trainer) holding the same initial state."""
    rows = tuple(rows if rows is not None else wl.rows)
    row_base = np.concatenate(([0], np.cumsum(rows)))
    if h0 is None:
        h0 = synth.full_tables_h0(wl)
    w0 = synth.dense_w0(wl)
    max_ids = max(int(b.offsets[-1]) for b in batches) + 64
    gpu = binding.ShadowSync(rows, wl.emb_dim, wl.bot_dims, wl.top_dims, wl.num_replicas,
                             max(b.dense.shape[0] for b in batches), max_ids, slots, wl.bf16,
                             wl.lr_dense, wl.lr_emb, wl.adagrad_eps, wl.seed, pooling=wl.pooling,
                             mlp_path=mlp_path, emb_optimizer=wl.emb_optimizer,
                             adam_betas=wl.adam_betas, emb_row_shards=wl.emb_row_shards,
                             sort_digit_bits=sort_digit_bits)
    for t in range(len(rows)):
        gpu.ss_write_rows(t, 0, h0[row_base[t]:row_base[t + 1]])
    gpu.ss_init_dense(w0)
    orc = oracle.OracleTrainer(wl.bot_dims, wl.top_dims, row_base, h0, w0, wl.num_replicas,
                               wl.lr_dense, wl.lr_emb, wl.adagrad_eps, dtype=dtype,
                               bf16=wl.bf16, pooling=wl.pooling, emb_optimizer=wl.emb_optimizer,
                               adam_betas=wl.adam_betas, emb_row_shards=wl.emb_row_shards)
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
    # the values the step's sort carries: the pooled-vector id of every sorted entry
    want_bag = np.asarray(last["bag_of_pos"], dtype=np.int64)[np.asarray(last["sorted_pos"], dtype=np.int64)]
    assert np.array_equal(gpu.ss_read_debug(slot, binding.DBG_SORTED_BAG).astype(np.int64), want_bag), \
        f"{step_name}: sorted pooled-vector ids differ"
    assert int(gpu.ss_read_debug(slot, binding.DBG_NUM_UNIQUE)[0]) == len(last["seg_starts"])
    close(gpu.ss_read_debug(slot, binding.DBG_POOLED), last["e"],
          FP32_RTOL if (tables_exact or rtol <= FP32_RTOL) else rtol, f"{step_name}: pooled e")
    if last.get("e_parts") is not None:
        close(gpu.ss_read_debug(slot, binding.DBG_POOLED_PARTIALS), last["e_parts"],
              FP32_RTOL if (tables_exact or rtol <= FP32_RTOL) else rtol,
              f"{step_name}: partial pooling results per row shard")
    close(gpu.ss_read_debug(slot, binding.DBG_INTERACT), last["f"], rtol, f"{step_name}: interaction f")
    close(gpu.ss_read_debug(slot, binding.DBG_LOGITS), last["logit"], rtol, f"{step_name}: logits")
    close_dense(gpu.ss_read_debug(slot, binding.DBG_DENSE_GRAD), last["g"], rtol,
                f"{step_name}: dense grad", orc.layout)
    close(gpu.ss_read_debug(slot, binding.DBG_POOLED_GRAD), last["de"], rtol, f"{step_name}: de")


def compare_state(gpu, orc, rtol, name, row_base):
    K = orc.W.shape[0]
    for i in range(K):
        close_dense(gpu.ss_read_dense(i), orc.W[i], rtol, f"{name}: replica {i}", orc.layout)
    close_dense(gpu.ss_read_dense(-4), orc.W.mean(axis=0), rtol, f"{name}: replica average", orc.layout)
    close_dense(gpu.ss_read_dense(-1), orc.w_ps, rtol, f"{name}: w_ps", orc.layout)
    close_dense(gpu.ss_read_dense(-2), orc.w_global, rtol, f"{name}: w_global", orc.layout)
    close(gpu.ss_read_dense(-3), orc.v, rtol, f"{name}: v", scale=max(1e-30, float(np.max(np.abs(orc.w_global)))))
    for t in range(len(row_base) - 1):
        n = int(row_base[t + 1] - row_base[t])
        vals, acc = gpu.ss_read_rows(t, np.arange(n))
        close(vals, orc.h[row_base[t]:row_base[t + 1]], rtol, f"{name}: table {t}")
        # the accumulator is quadratic in the row gradient: twice its relative error
        if orc.emb_optimizer == "adam":
            assert np.array_equal(acc, orc.G[row_base[t]:row_base[t + 1]]), f"{name}: step counts {t}"
            m, v = gpu.ss_read_adam_state(t, np.arange(n))
            close(m, orc.M[row_base[t]:row_base[t + 1]], rtol, f"{name}: Adam m {t}")
            # (the second moment is quadratic in the row gradient: twice its relative error)
            close(v, orc.V[row_base[t]:row_base[t + 1]], 2 * rtol if rtol > FP32_RTOL else rtol,
                  f"{name}: Adam v {t}")
            continue
        close(acc, orc.G[row_base[t]:row_base[t + 1]], 2 * rtol if rtol > FP32_RTOL else rtol,
              f"{name}: adagrad state {t}")


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
        if orc.emb_optimizer == "adam":
            gpu.ss_write_adam_state(t, 0, orc.M[row_base[t]:row_base[t + 1]],
                                    orc.V[row_base[t]:row_base[t + 1]])


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
            lg = float(gpu.ss_train_step(i, 0, dev[k]).cpu()[0])
            lo, _ = oracle_step(gpu, orc, 0, i, batches[k].as_tuple())
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
