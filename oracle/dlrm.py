"""Oracle for one trainer's model step (test infrastructure only).

The paper (Section 3.1, "Trainer") fixes the ORDER of a step: bottom MLP, embedding
look-ups (pooled where the table lives, Section 3.1 "Embedding PS"), interaction,
top MLP, backward, embedding gradients pushed to the tables (lock-free optimiser
update with co-located Adagrad state, Section 3.2 "Embedding Tables: Hogwild
Updates"), dense parameters updated in place (Section 3.2 "Interactions and MLPs").
It defers the model itself to the DLRM paper, so the concrete formulas below are the
readings this implementation takes: sum pooling (mean pooling, the paper's own example, as an
option), pairwise-dot interaction over the
bottom output and the T pooled vectors (strictly lower triangle, row-major, appended
after the bottom output), ReLU everywhere except the last top layer, mean binary
cross-entropy on the logit, plain SGD on dense weights, row-wise Adagrad on tables.

Data layout used throughout:
  dense parameter vector w (P,)   : bottom layers then top layers, each W[out][in]
                                    row-major followed by b[out]
  tables h (R, d)                 : all tables stacked; table t owns rows
                                    row_base[t] .. row_base[t+1]-1
  batch: x (B, n_dense), y (B,), indices (n,) row ids local to their table,
         offsets (T*B+1,) : bag (t, b) = indices[offsets[t*B+b] : offsets[t*B+b+1]]
         (table-major CSR, so a flat position `pos` identifies table and sample)
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- layout
@dataclass(frozen=True)
class DenseLayout:
    """Where each layer lives inside the flat dense vector (bottom first, W then b)."""

    bot_dims: Tuple[int, ...]
    top_dims: Tuple[int, ...]

    def layer_shapes(self) -> List[Tuple[int, int]]:
        dims = []
        for d in (self.bot_dims, self.top_dims):
            dims += [(d[i + 1], d[i]) for i in range(len(d) - 1)]  # (out, in)
        return dims

    @property
    def n_bot(self) -> int:
        return len(self.bot_dims) - 1

    @property
    def num_params(self) -> int:
        return sum(o * i + o for o, i in self.layer_shapes())

    def unpack(self, w: np.ndarray) -> List[Tuple[np.ndarray, np.ndarray]]:
        """Views (W[out,in], b[out]) into w, in layer order."""
        out, p = [], 0
        for o, i in self.layer_shapes():
            W = w[p : p + o * i].reshape(o, i)
            p += o * i
            b = w[p : p + o]
            p += o
            out.append((W, b))
        assert p == w.shape[0]
        return out


# --------------------------------------------------------------------------- bf16
def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned as float32 values.

    bfloat16 keeps the top 16 bits of an IEEE binary32, so rounding is done on the
    integer image: add 0x7FFF plus the lowest kept bit, then clear the low half.
    Inputs are first rounded to float32 (that is what the device holds).
    """
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def _identity(x):
    return x


def _quantiser(bf16: bool, dtype) -> Callable[[np.ndarray], np.ndarray]:
    if not bf16:
        return _identity
    return lambda a: bf16_round(a).astype(dtype)


# --------------------------------------------------------------------------- MLP
def mlp_forward(x, layers, relu_last: bool, q=_identity):
    """a_0 = x; a_l = ReLU(q(a_{l-1}) q(W_l)^T + b_l); the last layer is linear unless
    relu_last.  Returns the list of activations [a_0 .. a_L].  q rounds GEMM inputs
    (identity for fp32/fp64, bf16 rounding for the mixed-precision reading)."""
    acts = [x]
    n = len(layers)
    for li, (W, b) in enumerate(layers):
        z = q(acts[-1]) @ q(W).T + b
        if li < n - 1 or relu_last:
            z = np.maximum(z, 0)
        acts.append(z)
    return acts


def mlp_backward(acts, layers, d_out, relu_last: bool, q=_identity, gate_flips=None):
    """Back-propagation through mlp_forward.  d_out is dL/d(a_L).  Returns
    (list of (dW, db) per layer, dL/d(a_0)).  ReLU passes gradient where its output
    is positive.

    gate_flips (optional): {layer index: (sample indices, unit indices)} of ReLU units whose
    gate decision is to be INVERTED.  A gate is a floating-point comparison with zero; for a
    pre-activation that is zero to within the accumulation error of the precision the product
    was formed in, both outcomes are valid results of this definition.  The parity harness
    uses this to take such undecidable decisions the way the device's fp32 accumulation took
    them (it only ever lists units whose pre-activation here is that close to zero)."""
    n = len(layers)
    grads = [None] * n
    d = d_out
    for li in range(n - 1, -1, -1):
        W, _ = layers[li]
        if li < n - 1 or relu_last:
            gate = acts[li + 1] > 0
            if gate_flips and li in gate_flips:
                bb, uu = gate_flips[li]
                gate[bb, uu] = ~gate[bb, uu]
            d = d * gate
        dW = q(d).T @ q(acts[li])
        db = d.sum(axis=0)
        grads[li] = (dW, db)
        d = q(d) @ q(W)
    return grads, d


# --------------------------------------------------------------------------- embedding
def embedding_bag_forward(h, row_base, indices, offsets, B: int, pooling: str = "sum"):
    """Pooling (Section 3.1, done where the table lives).  Sum:
    e[b, t, :] = sum over j in bag(t, b), in j order, of h[row_base[t] + indices[j], :].
    Mean (the pooling of the paper's own example in Section 3.1): the same sum divided by the
    bag's length.  A row that occurs twice in a bag counts twice; an empty bag gives zeros."""
    assert pooling in ("sum", "mean")
    T = len(row_base) - 1
    d = h.shape[1]
    e = np.zeros((B, T, d), dtype=h.dtype)
    for t in range(T):
        for b in range(B):
            lo, hi = offsets[t * B + b], offsets[t * B + b + 1]
            for j in range(lo, hi):
                e[b, t, :] += h[row_base[t] + indices[j], :]
            if pooling == "mean" and hi > lo:
                e[b, t, :] /= (hi - lo)
    return e


def embedding_bag_forward_fast(h, row_base, indices, offsets, B: int, pooling: str = "sum"):
    """Same definition as embedding_bag_forward with the inner loop handed to numpy's
    row gather + sum (used at sizes where the triple loop is too slow; the two are
    compared in the CPU tests)."""
    assert pooling in ("sum", "mean")
    T = len(row_base) - 1
    d = h.shape[1]
    e = np.zeros((B, T, d), dtype=h.dtype)
    for t in range(T):
        base = row_base[t]
        for b in range(B):
            lo, hi = offsets[t * B + b], offsets[t * B + b + 1]
            if hi > lo:
                e[b, t, :] = h[base + indices[lo:hi]].sum(axis=0)
                if pooling == "mean":
                    e[b, t, :] /= (hi - lo)
    return e


def embedding_bag_forward_sharded(h, row_base, indices, offsets, B: int, n_shards: int,
                                  pooling: str = "sum"):
    """Partial pooling (Section 3.1, "Embedding PS"): table t is split into n_shards equal row
    ranges of ceil(rows_t / n_shards) rows; every range pools, in bag order, the rows of a bag
    that it owns; the trainer adds the partial vectors in range order (and divides by the bag
    length under mean pooling).  Returns (e (B, T, d), partials (n_shards, B, T, d))."""
    assert pooling in ("sum", "mean")
    T = len(row_base) - 1
    d = h.shape[1]
    parts = np.zeros((n_shards, B, T, d), dtype=h.dtype)
    for t in range(T):
        rows_t = int(row_base[t + 1] - row_base[t])
        per = -(-rows_t // n_shards)
        for b in range(B):
            lo, hi = offsets[t * B + b], offsets[t * B + b + 1]
            for j in range(lo, hi):
                s = int(indices[j]) // per
                parts[s, b, t, :] += h[row_base[t] + indices[j], :]
    e = parts[0].copy()
    for s in range(1, n_shards):
        e += parts[s]
    if pooling == "mean":
        lens = np.maximum(bag_lengths(offsets, B, T), 1).reshape(B, T)
        e = e / lens[:, :, None]
    return e, parts


def bag_lengths(offsets, B: int, T: int):
    """Length of the bag behind pooled vector b*T + t."""
    off = np.asarray(offsets, dtype=np.int64)
    return (off[1:] - off[:-1]).reshape(T, B).T.reshape(B * T)


def global_rows(row_base, indices, offsets, B: int):
    """Sort key of every flat position: row_base[table(pos)] + indices[pos]."""
    T = len(row_base) - 1
    keys = np.empty(len(indices), dtype=np.int64)
    for t in range(T):
        lo, hi = offsets[t * B], offsets[(t + 1) * B]
        keys[lo:hi] = row_base[t] + indices[lo:hi].astype(np.int64)
    return keys


def bag_of_position(offsets, B: int, T: int):
    """For each flat position the index b*T + t of the pooled vector it fed."""
    n = offsets[-1]
    out = np.empty(n, dtype=np.int64)
    for t in range(T):
        for b in range(B):
            out[offsets[t * B + b] : offsets[t * B + b + 1]] = b * T + t
    return out


def stable_sort_by_row(keys):
    """Stable sort of (key, position) pairs by key: equal keys keep ascending position.
    Returns (sorted_keys, sorted_positions, segment_starts) where segment_starts lists
    the index in the sorted order at which each distinct key begins."""
    perm = np.argsort(keys, kind="stable")
    sk = keys[perm]
    if len(sk) == 0:
        return sk, perm, np.zeros(0, dtype=np.int64)
    heads = np.flatnonzero(np.concatenate(([True], sk[1:] != sk[:-1])))
    return sk, perm, heads


def embedding_row_gradients(de, keys, bag_of_pos, bag_scale=None):
    """Gradient of every touched table row: g_r = sum, over the occurrences of r in
    ascending flat position, of de[bag that occurrence fed] (times bag_scale[bag] if given:
    1 / bag length under mean pooling, the derivative of the mean w.r.t. each member).
    de is (B*T, d).  Duplicates inside one bag and across the batch are all summed before any
    update.  Returns (unique_rows, g (U, d), sorted_keys, sorted_pos, segment_starts)."""
    sk, perm, heads = stable_sort_by_row(keys)
    if len(sk) == 0:
        return sk, np.zeros((0, de.shape[1]), de.dtype), sk, perm, heads
    contrib = de[bag_of_pos[perm]]
    if bag_scale is not None:
        contrib = contrib * np.asarray(bag_scale, dtype=de.dtype)[bag_of_pos[perm]][:, None]
    g = np.add.reduceat(contrib, heads, axis=0)
    return sk[heads], g, sk, perm, heads


def rowwise_adagrad_update(h, G, rows, g, lr: float, eps: float):
    """Row-wise Adagrad (one accumulator per row, co-located with the row,
    Section 3.2): G_r += mean_c g_r[c]^2 ;  h[r,:] -= lr * g_r / (sqrt(G_r) + eps).
    Each row in `rows` is distinct and gets exactly one update.  In place."""
    ms = (g * g).sum(axis=1) / g.shape[1]
    G[rows] = G[rows] + ms
    h[rows] = h[rows] - lr * g / (np.sqrt(G[rows]) + eps)[:, None]


def adam_update(h, M, V, T, rows, g, lr: float, eps: float, beta1: float, beta2: float):
    """Adam on the touched rows only, with its state kept beside the rows (Section 3.2 names
    Adam next to Adagrad as a table optimiser with co-located auxiliary state): per row r in
    `rows` (each distinct, one update per step)
        T_r += 1;  M_r = beta1 M_r + (1-beta1) g_r;  V_r = beta2 V_r + (1-beta2) g_r^2;
        h[r,:] -= lr * (M_r / (1-beta1^T_r)) / (sqrt(V_r / (1-beta2^T_r)) + eps).
    M, V are per element, T is the row's own step count: a row that a batch does not touch
    keeps all of its state.  In place."""
    T[rows] = T[rows] + 1
    M[rows] = beta1 * M[rows] + (1 - beta1) * g
    V[rows] = beta2 * V[rows] + (1 - beta2) * g * g
    t = T[rows][:, None]
    m_hat = M[rows] / (1 - beta1 ** t)
    v_hat = V[rows] / (1 - beta2 ** t)
    h[rows] = h[rows] - lr * m_hat / (np.sqrt(v_hat) + eps)


# --------------------------------------------------------------------------- interaction
def lower_pairs(T: int):
    """(r, c) with 1 <= r <= T, 0 <= c < r, row-major: the strictly lower triangle of
    the (T+1)x(T+1) Gram matrix."""
    return [(r, c) for r in range(1, T + 1) for c in range(r)]


def interaction_forward(z0, e):
    """V_b = [z0_b; e[b,0]; ...; e[b,T-1]];  f_b = concat(z0_b, <V_b[r], V_b[c]> for the
    strictly-lower (r, c) in row-major order).  Width d + T(T+1)/2."""
    B, T, d = e.shape
    V = np.concatenate([z0[:, None, :], e], axis=1)
    pairs = lower_pairs(T)
    f = np.empty((B, d + len(pairs)), dtype=z0.dtype)
    f[:, :d] = z0
    for p, (r, c) in enumerate(pairs):
        f[:, d + p] = (V[:, r, :] * V[:, c, :]).sum(axis=1)
    return f


def interaction_backward(z0, e, df):
    """d<V_r,V_c>/dV_r = V_c and /dV_c = V_r, accumulated over all pairs; the first d
    columns of df pass straight through to z0.  Returns (dz0, de)."""
    B, T, d = e.shape
    V = np.concatenate([z0[:, None, :], e], axis=1)
    dV = np.zeros_like(V)
    for p, (r, c) in enumerate(lower_pairs(T)):
        s = df[:, d + p][:, None]
        dV[:, r, :] += s * V[:, c, :]
        dV[:, c, :] += s * V[:, r, :]
    dz0 = df[:, :d] + dV[:, 0, :]
    return dz0, dV[:, 1:, :]


# --------------------------------------------------------------------------- loss
def bce_with_logits(logit, y):
    """Mean binary cross-entropy of p = sigmoid(logit) against y in {0,1} (the
    numerator of the normalised entropy of Section 4, "Evaluation Metrics"), computed
    from the logit as max(l,0) - l*y + log(1 + exp(-|l|)).  Returns (L, dL/dlogit)."""
    B = logit.shape[0]
    per = np.maximum(logit, 0) - logit * y + np.log1p(np.exp(-np.abs(logit)))
    t = np.exp(-np.abs(logit))                     # sigmoid without overflow
    p = np.where(logit >= 0, 1.0 / (1.0 + t), t / (1.0 + t))
    return per.sum() / B, (p - y) / B


# --------------------------------------------------------------------------- whole model
def dlrm_forward(layout: DenseLayout, w, h, row_base, x, indices, offsets, bf16=False,
                 fast=True, pooling="sum", row_shards=1):
    """Forward pass in the paper's order (Section 3.1 "Trainer").  Returns a dict of
    every intermediate the backward pass needs."""
    dtype = w.dtype
    q = _quantiser(bf16, dtype)
    layers = layout.unpack(w)
    bot, top = layers[: layout.n_bot], layers[layout.n_bot :]
    B = x.shape[0]
    acts_bot = mlp_forward(x.astype(dtype), bot, relu_last=True, q=q)
    z0 = acts_bot[-1]
    e_parts = None
    if row_shards > 1:
        e, e_parts = embedding_bag_forward_sharded(h, row_base, indices, offsets, B, row_shards,
                                                   pooling)
    else:
        bag = embedding_bag_forward_fast if fast else embedding_bag_forward
        e = bag(h, row_base, indices, offsets, B, pooling)
    f = interaction_forward(z0, e)
    acts_top = mlp_forward(f, top, relu_last=False, q=q)
    logit = acts_top[-1][:, 0]
    return dict(acts_bot=acts_bot, z0=z0, e=e, f=f, acts_top=acts_top, logit=logit,
                bot=bot, top=top, q=q, e_parts=e_parts)


def dlrm_backward(layout: DenseLayout, fw, y, gate_flips=None):
    """Loss and gradients.  Returns (L, dense gradient vector laid out like w,
    de (B, T, d)).  gate_flips: see mlp_backward; keys are layer indices counted over the
    whole model (bottom layers first)."""
    L, dlogit = bce_with_logits(fw["logit"], y)
    q = fw["q"]
    nb = layout.n_bot
    flips_bot = flips_top = None
    if gate_flips:
        flips_bot = {l: v for l, v in gate_flips.items() if l < nb}
        flips_top = {l - nb: v for l, v in gate_flips.items() if l >= nb}
    g_top, df = mlp_backward(fw["acts_top"], fw["top"], dlogit[:, None], False, q, flips_top)
    dz0, de = interaction_backward(fw["z0"], fw["e"], df)
    g_bot, _ = mlp_backward(fw["acts_bot"], fw["bot"], dz0, True, q, flips_bot)
    parts = []
    for dW, db in g_bot + g_top:
        parts += [dW.ravel(), db.ravel()]
    return L, np.concatenate(parts), de
