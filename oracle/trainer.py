"""Oracle state machine: Algorithm 1 with K replicas on one host (test infrastructure).

Holds the single copy of the tables h (+ Adagrad accumulators), the K dense replicas
w^(i), the centre copy w^PS, the aggregated copy w^global and the momentum buffer v,
all initialised as Algorithm 1 states (h <- h0, w^PS <- w0, w^(i) <- w0; Algorithms 3
and 4 initialise w^global <- w0).  train_step is one pass of a worker thread's loop
body for one batch; shadow_sync is one pass of the shadow threads' loop body.
"""

from __future__ import annotations

import numpy as np

from . import dlrm, sync


class OracleTrainer:
    def __init__(self, bot_dims, top_dims, row_base, h0, w0, num_replicas,
                 lr_dense=0.01, lr_emb=0.01, adagrad_eps=1e-8, dtype=np.float64,
                 bf16=False, pooling="sum", emb_optimizer="rowwise_adagrad",
                 adam_betas=(0.9, 0.999), emb_row_shards=1):
        self.layout = dlrm.DenseLayout(tuple(bot_dims), tuple(top_dims))
        self.row_base = np.asarray(row_base, dtype=np.int64)
        self.T = len(self.row_base) - 1
        self.d = h0.shape[1]
        assert h0.shape[0] == self.row_base[-1]
        assert self.layout.top_dims[0] == self.d + self.T * (self.T + 1) // 2
        assert w0.shape == (self.layout.num_params,)
        self.dtype = dtype
        self.bf16 = bf16
        assert pooling in ("sum", "mean")
        self.pooling = pooling
        self.row_shards = max(1, int(emb_row_shards))
        assert emb_optimizer in ("rowwise_adagrad", "adam")
        self.emb_optimizer = emb_optimizer
        self.adam_betas = adam_betas
        self.h = h0.astype(dtype).copy()
        # per row: the Adagrad accumulator, or (Adam) the row's own step count
        self.G = np.zeros(h0.shape[0], dtype=dtype)
        self.M = np.zeros_like(self.h) if emb_optimizer == "adam" else None
        self.V = np.zeros_like(self.h) if emb_optimizer == "adam" else None
        self.W = np.tile(w0.astype(dtype), (num_replicas, 1))
        self.w_ps = w0.astype(dtype).copy()
        self.w_global = w0.astype(dtype).copy()
        self.v = np.zeros_like(self.w_ps)
        self.lr_dense, self.lr_emb, self.eps = lr_dense, lr_emb, adagrad_eps
        self.steps = np.zeros(num_replicas, dtype=np.int64)
        self.rounds = 0
        self.last = None
        # running sums behind the normalised entropy (Section 4, "Evaluation Metrics"):
        # [sum of per-example log-loss, positive labels, examples] for training and evaluation
        self.metrics = {"train": np.zeros(3), "eval": np.zeros(3)}

    # ------------------------------------------------------------------ worker thread
    def train_step(self, replica, x, y, indices, offsets, update=True, gate_flips=None):
        """One worker iteration (Algorithm 1, worker loop; Section 3.1 "Trainer"):
        forward, loss, backward, then "update h" and "update local param w^(i)".
        Returns the mean log-loss of the batch BEFORE the update.
        gate_flips: undecidable ReLU gates to take the other way (dlrm.mlp_backward)."""
        B = x.shape[0]
        L = self.layout
        w = self.W[replica]
        fw = dlrm.dlrm_forward(L, w, self.h, self.row_base, x, indices, offsets,
                               bf16=self.bf16, pooling=self.pooling, row_shards=self.row_shards)
        loss, g, de = dlrm.dlrm_backward(L, fw, y.astype(self.dtype), gate_flips)
        keys = dlrm.global_rows(self.row_base, indices, offsets, B)
        bag = dlrm.bag_of_position(offsets, B, self.T)
        scale = None
        if self.pooling == "mean":
            scale = 1.0 / np.maximum(dlrm.bag_lengths(offsets, B, self.T), 1)
        rows, g_rows, sk, perm, heads = dlrm.embedding_row_gradients(
            de.reshape(B * self.T, self.d), keys, bag, scale)
        self.last = dict(e=fw["e"], f=fw["f"], logit=fw["logit"], z0=fw["z0"], g=g,
                         acts_bot=fw["acts_bot"], acts_top=fw["acts_top"], e_parts=fw["e_parts"],
                         de=de, sorted_keys=sk, sorted_pos=perm, seg_starts=heads,
                         rows=rows, g_rows=g_rows, bag_of_pos=bag)
        if update:
            # the loss is the one BEFORE the update: every example is scored by a model that
            # has not trained on it yet (the progressive Train NE of Section 4)
            self.metrics["train"] += (loss * B, float(np.sum(y)), B)
            self.W[replica] = w - self.lr_dense * g
            if self.emb_optimizer == "adam":
                dlrm.adam_update(self.h, self.M, self.V, self.G, rows, g_rows, self.lr_emb,
                                 self.eps, *self.adam_betas)
            else:
                dlrm.rowwise_adagrad_update(self.h, self.G, rows, g_rows, self.lr_emb,
                                            self.eps)
            self.steps[replica] += 1
        return loss

    def eval_logloss(self, replica, x, y, indices, offsets):
        fw = dlrm.dlrm_forward(self.layout, self.W[replica], self.h, self.row_base, x,
                               indices, offsets, bf16=self.bf16, pooling=self.pooling,
                               row_shards=self.row_shards)
        loss = dlrm.bce_with_logits(fw["logit"], y.astype(self.dtype))[0]
        self.metrics["eval"] += (loss * x.shape[0], float(np.sum(y)), x.shape[0])
        return loss

    def ne(self, which):
        """(examples, mean log-loss, click rate, NE) of the "train" or "eval" accumulator:
        NE = mean log-loss / entropy of the click rate of the same examples (Section 4)."""
        s, pos, n = self.metrics[which]
        mean, p = s / n, pos / n
        return n, mean, p, mean / -(p * np.log(p) + (1 - p) * np.log(1 - p))

    # ------------------------------------------------------------------ shadow thread
    def shadow_sync(self, algo, alpha, eta=1.0, mu=0.0):
        """One round of Algorithm 2 ("easgd"), 3 ("ma") or 4 ("bmuf")."""
        if algo == "easgd":
            sync.easgd_round(self.W, self.w_ps, alpha)
        elif algo == "easgd_literal":
            sync.easgd_round_literal(self.W, self.w_ps, alpha)
        elif algo == "ma":
            sync.ma_round(self.W, self.w_global, alpha)
        elif algo == "bmuf":
            sync.bmuf_round(self.W, self.w_global, self.v, alpha, eta, mu)
        elif algo == "bmuf_nesterov":
            sync.bmuf_nesterov_round(self.W, self.w_global, self.v, alpha, eta, mu)
        else:
            raise ValueError(algo)
        self.rounds += 1

    # ------------------------------------------------------------------ schedules
    def run_deterministic(self, batches, gap, algo, alpha, eta=1.0, mu=0.0):
        """One worker per replica, sync at fixed steps: for s = 0, 1, ...: replica
        i = 0..K-1 trains batch s*K+i in turn (the tables are one shared copy, so
        replica i+1 sees replica i's row updates), and after every `gap` such sweeps one
        sync round runs.  Returns the list of per-batch losses."""
        K = self.W.shape[0]
        losses = []
        for s in range(len(batches) // K):
            for i in range(K):
                losses.append(self.train_step(i, *batches[s * K + i]))
            if (s + 1) % gap == 0:
                self.shadow_sync(algo, alpha, eta, mu)
        return losses

    def avg_sync_gap(self):
        """Average sync gap (Section 4.1): trainer iterations per sync, i.e. iterations
        of one trainer divided by the number of syncs it took part in."""
        return float(self.steps.mean()) / max(self.rounds, 1)


def normalized_entropy(p_hat, y):
    """NE (Section 4, "Evaluation Metrics"): mean cross-entropy of the predictions
    divided by the entropy of the empirical click rate."""
    p_hat = np.asarray(p_hat, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    ce = -(y * np.log(p_hat) + (1 - y) * np.log(1 - p_hat)).mean()
    p = y.mean()
    return ce / -(p * np.log(p) + (1 - p) * np.log(1 - p))
