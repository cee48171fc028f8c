"""Oracle for the three shadow synchronisation rules (test infrastructure only).

One call = one ROUND: what the K shadow threads of Algorithms 2-4 do in one pass of
their loop, taken with the replicas i = 0..K-1 in ascending order, element-wise over
the P dense parameters.  All functions update their arguments in place.

  W        (K, P)  the replicas w^(i)
  w_ps     (P,)    the centre copy on the sync parameter server (Algorithm 2)
  w_global (P,)    the aggregated copy of Algorithms 3 and 4
  v        (P,)    block-momentum buffer (the "momentum update" remark in Algorithm 4)
"""

from __future__ import annotations

import numpy as np


def easgd_round(W, w_ps, alpha):
    """Shadow EASGD (Algorithm 2), reading both assignments with the values held
    before the exchange, i.e. the symmetric elastic move of the original EASGD (the
    discussion after Algorithm 4 likens the rule to it):
        delta = alpha * (w^(i) - w^PS);  w^PS += delta;  w^(i) -= delta.
    This reading conserves sum_i w^(i) + w^PS.  Replicas exchange one after another,
    so replica i+1 meets the centre already moved by replica i."""
    for i in range(W.shape[0]):
        delta = alpha * (W[i] - w_ps)
        w_ps += delta
        W[i] -= delta


def easgd_round_literal(W, w_ps, alpha):
    """Shadow EASGD with Algorithm 2's two assignments executed strictly one after the
    other, so the second line sees the centre that the first line just produced:
        w^PS <- (1-alpha) w^PS + alpha w^(i);  w^(i) <- (1-alpha) w^(i) + alpha w^PS.
    Kept as a variant; each exchange changes w^(i) + w^PS by alpha^2 (w^(i) - w^PS)."""
    for i in range(W.shape[0]):
        w_ps[:] = (1 - alpha) * w_ps + alpha * W[i]
        W[i] = (1 - alpha) * W[i] + alpha * w_ps


def ma_round(W, w_global, alpha):
    """Shadow MA (Algorithm 3): every trainer copies its replica, the copies are
    all-reduced and divided by n, and each replica is pulled towards the mean:
        w^global = (1/K) sum_i w^(i);  w^(i) <- (1-alpha) w^(i) + alpha w^global.
    On one device the snapshot and the replica it is mixed with are the same values."""
    K = W.shape[0]
    m = W[0].copy()
    for i in range(1, K):
        m += W[i]
    m /= K
    w_global[:] = m
    for i in range(K):
        W[i] = (1 - alpha) * W[i] + alpha * m


def bmuf_round(W, w_global, v, alpha, eta, mu):
    """Shadow BMUF (Algorithm 4) with the block-momentum form of the surrogate-gradient
    step that the algorithm's comment allows:
        m = (1/K) sum_i w^(i);  desc = m - w^global;  v <- mu v + eta desc;
        w^global <- w^global + v;  w^(i) <- (1-alpha) w^(i) + alpha w^global.
    mu = 0 is Algorithm 4 as printed; mu = 0 and eta = 1 make w^global the mean, i.e.
    Shadow MA.  All trainers' w^global copies start equal and receive the same
    all-reduced value, so one shared copy is kept."""
    K = W.shape[0]
    m = W[0].copy()
    for i in range(1, K):
        m += W[i]
    m /= K
    desc = m - w_global
    v[:] = mu * v + eta * desc
    w_global += v
    for i in range(K):
        W[i] = (1 - alpha) * W[i] + alpha * w_global


def bmuf_nesterov_round(W, w_global, v, alpha, eta, mu):
    """Shadow BMUF with Nesterov block momentum, the second option named in Algorithm 4's
    comment (the paper gives no formula; this is the block-momentum form of the BMUF paper it
    cites): v and w^global advance exactly as in bmuf_round, but the replicas are pulled
    towards the look-ahead point w^global + mu v instead of w^global:
        w^(i) <- (1-alpha) w^(i) + alpha (w^global + mu v).
    mu = 0 is bmuf_round."""
    K = W.shape[0]
    m = W[0].copy()
    for i in range(1, K):
        m += W[i]
    m /= K
    desc = m - w_global
    v[:] = mu * v + eta * desc
    w_global += v
    ahead = w_global + mu * v
    for i in range(K):
        W[i] = (1 - alpha) * W[i] + alpha * ahead

