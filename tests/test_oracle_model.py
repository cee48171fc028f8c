"""Pins for the model-step oracle: each test checks it against a fact that does not come
from the oracle itself (finite differences, torch autograd, dense matrix products,
Python's own stable sort, closed forms, hand-computed values)."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import dlrm
from helpers import random_problem

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _loss(p, w=None, h=None, pooling="sum"):
    L = dlrm.DenseLayout(p["bot"], p["top"])
    fw = dlrm.dlrm_forward(L, p["w"] if w is None else w, p["h"] if h is None else h,
                           p["row_base"], p["x"], p["indices"], p["offsets"], fast=False,
                           pooling=pooling)
    return dlrm.bce_with_logits(fw["logit"], p["y"])[0]


def _grads(p, pooling="sum"):
    L = dlrm.DenseLayout(p["bot"], p["top"])
    fw = dlrm.dlrm_forward(L, p["w"], p["h"], p["row_base"], p["x"], p["indices"],
                           p["offsets"], fast=False, pooling=pooling)
    loss, g, de = dlrm.dlrm_backward(L, fw, p["y"])
    keys = dlrm.global_rows(p["row_base"], p["indices"], p["offsets"], p["B"])
    bag = dlrm.bag_of_position(p["offsets"], p["B"], p["T"])
    scale = None
    if pooling == "mean":
        scale = 1.0 / np.maximum(dlrm.bag_lengths(p["offsets"], p["B"], p["T"]), 1)
    rows, g_rows, sk, perm, heads = dlrm.embedding_row_gradients(
        de.reshape(p["B"] * p["T"], p["d"]), keys, bag, scale)
    dh = np.zeros_like(p["h"])
    dh[rows] = g_rows
    return loss, g, de, dh


# ----------------------------------------------------------------------------- gradients
@pytest.mark.parametrize("seed,pooling", [(0, "sum"), (1, "sum"), (2, "sum"), (3, "mean"),
                                          (4, "mean")])
def test_dense_and_table_gradients_match_finite_differences(seed, pooling):
    rng = np.random.default_rng(seed)
    p = random_problem(rng)
    _, g, _, dh = _grads(p, pooling)
    eps = 1e-6
    num = np.zeros_like(g)
    for k in range(len(g)):
        wp, wm = p["w"].copy(), p["w"].copy()
        wp[k] += eps
        wm[k] -= eps
        num[k] = (_loss(p, w=wp, pooling=pooling) - _loss(p, w=wm, pooling=pooling)) / (2 * eps)
    assert np.max(np.abs(num - g)) < 1e-6 * max(1.0, np.max(np.abs(g)))
    numh = np.zeros_like(dh)
    for r in range(dh.shape[0]):
        for c in range(dh.shape[1]):
            hp, hm = p["h"].copy(), p["h"].copy()
            hp[r, c] += eps
            hm[r, c] -= eps
            numh[r, c] = (_loss(p, h=hp, pooling=pooling) - _loss(p, h=hm, pooling=pooling)) / (2 * eps)
    assert np.max(np.abs(numh - dh)) < 1e-6 * max(1.0, np.max(np.abs(dh)))


@pytest.mark.parametrize("seed", [3, 4])
def test_matches_torch_autograd(seed):
    """Same model written with torch ops (embedding_bag, linear, relu, BCE-with-logits)
    and differentiated by autograd."""
    rng = np.random.default_rng(seed)
    p = random_problem(rng, B=6, T=3, d=4, rows=(9, 4, 6), bot=(3, 8, 4), top_hidden=(7, 5),
                       max_len=4, allow_empty=True)
    loss, g, de, dh = _grads(p)
    B, T, d = p["B"], p["T"], p["d"]
    w = torch.tensor(p["w"], requires_grad=True)
    h = torch.tensor(p["h"], requires_grad=True)
    L = dlrm.DenseLayout(p["bot"], p["top"])
    layers, pos = [], 0
    for o, i in L.layer_shapes():
        W = w[pos:pos + o * i].view(o, i); pos += o * i
        b = w[pos:pos + o]; pos += o
        layers.append((W, b))
    z = torch.tensor(p["x"])
    for W, b in layers[:L.n_bot]:
        z = torch.relu(torch.nn.functional.linear(z, W, b))
    vecs = [z]
    for t in range(T):
        lo, hi = p["offsets"][t * B], p["offsets"][(t + 1) * B]
        tab = h[p["row_base"][t]:p["row_base"][t + 1]]
        idx = torch.tensor(p["indices"][lo:hi])
        off = torch.tensor(p["offsets"][t * B:(t + 1) * B] - lo)
        vecs.append(torch.nn.functional.embedding_bag(idx, tab, off, mode="sum"))
    V = torch.stack(vecs, dim=1)
    Gm = V @ V.transpose(1, 2)
    rr, cc = torch.tril_indices(T + 1, T + 1, offset=-1)
    f = torch.cat([z, Gm[:, rr, cc]], dim=1)
    a = f
    top = layers[L.n_bot:]
    for li, (W, b) in enumerate(top):
        a = torch.nn.functional.linear(a, W, b)
        if li < len(top) - 1:
            a = torch.relu(a)
    tl = torch.nn.functional.binary_cross_entropy_with_logits(a[:, 0], torch.tensor(p["y"]))
    tl.backward()
    assert abs(tl.item() - loss) < 1e-12
    np.testing.assert_allclose(w.grad.numpy(), g, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(h.grad.numpy(), dh, rtol=1e-10, atol=1e-13)


def test_gate_flips_equal_autograd_with_the_other_gate_decision():
    """mlp_backward's gate_flips: inverting the ReLU decision of listed units equals autograd
    through the same model in which each activation is its forward value times a CONSTANT
    0/1 gate, that gate being (pre-activation > 0) inverted at the listed units."""
    rng = np.random.default_rng(11)
    p = random_problem(rng, B=5, T=2, d=4, rows=(9, 4), bot=(3, 6, 4), top_hidden=(7, 5), max_len=3)
    L = dlrm.DenseLayout(p["bot"], p["top"])
    flips = {0: (np.array([0, 3]), np.array([2, 5])),      # bottom hidden layer
             1: (np.array([1]), np.array([3])),            # bottom output (z0)
             2: (np.array([4, 2]), np.array([0, 6])),      # top hidden layers
             3: (np.array([0]), np.array([1]))}
    fw = dlrm.dlrm_forward(L, p["w"], p["h"], p["row_base"], p["x"], p["indices"], p["offsets"],
                           fast=False)
    loss0, g0, de0 = dlrm.dlrm_backward(L, fw, p["y"])
    loss, g, de = dlrm.dlrm_backward(L, fw, p["y"], gate_flips=flips)
    assert loss == loss0 and not np.allclose(g, g0)
    B, T, d = p["B"], p["T"], p["d"]
    w = torch.tensor(p["w"], requires_grad=True)
    layers, pos = [], 0
    for o, i in L.layer_shapes():
        W = w[pos:pos + o * i].view(o, i); pos += o * i
        b = w[pos:pos + o]; pos += o
        layers.append((W, b))
    e_t = torch.tensor(fw["e"], requires_grad=True)

    def gated(pre, li):
        gate = (pre.detach() > 0)
        if li in flips:
            bb, uu = flips[li]
            gate[torch.tensor(bb), torch.tensor(uu)] ^= True
        # forward value unchanged (the oracle keeps its forward pass), gradient through the gate
        return (torch.relu(pre) - pre * gate.double()).detach() + pre * gate.double()

    z = torch.tensor(p["x"])
    for li in range(L.n_bot):
        W, b = layers[li]
        z = gated(torch.nn.functional.linear(z, W, b), li)
    V = torch.cat([z[:, None, :], e_t], dim=1)
    Gm = V @ V.transpose(1, 2)
    rr, cc = torch.tril_indices(T + 1, T + 1, offset=-1)
    a = torch.cat([z, Gm[:, rr, cc]], dim=1)
    n_layers = len(layers)
    for li in range(L.n_bot, n_layers):
        W, b = layers[li]
        a = torch.nn.functional.linear(a, W, b)
        if li < n_layers - 1:
            a = gated(a, li)
    tl = torch.nn.functional.binary_cross_entropy_with_logits(a[:, 0], torch.tensor(p["y"]))
    tl.backward()
    np.testing.assert_allclose(w.grad.numpy(), g, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(e_t.grad.numpy(), de, rtol=1e-10, atol=1e-13)


# ----------------------------------------------------------------------------- embedding
def _multiplicity(p):
    B, T = p["B"], p["T"]
    R = p["row_base"][-1]
    C = np.zeros((B * T, R))
    for t in range(T):
        for b in range(B):
            for j in range(p["offsets"][t * B + b], p["offsets"][t * B + b + 1]):
                C[b * T + t, p["row_base"][t] + p["indices"][j]] += 1
    return C


@pytest.mark.parametrize("allow_empty", [False, True])
def test_embedding_bag_is_multiplicity_matrix_product(allow_empty):
    rng = np.random.default_rng(5)
    p = random_problem(rng, B=9, T=3, d=4, rows=(6, 3, 11), bot=(3, 4), max_len=5,
                       allow_empty=allow_empty)
    C = _multiplicity(p)
    ref = (C @ p["h"]).reshape(p["B"], p["T"], p["d"])
    for fn in (dlrm.embedding_bag_forward, dlrm.embedding_bag_forward_fast):
        e = fn(p["h"], p["row_base"], p["indices"], p["offsets"], p["B"])
        np.testing.assert_allclose(e, ref, rtol=0, atol=1e-14)


@pytest.mark.parametrize("allow_empty", [False, True])
def test_mean_pooling_is_row_normalised_multiplicity_product(allow_empty):
    """Mean pooling and its gradient through the row-normalised multiplicity matrix
    N = diag(1/len) C (rows of empty bags stay zero): e = N h, dL/dh = N^T de."""
    rng = np.random.default_rng(15)
    p = random_problem(rng, B=11, T=3, d=4, rows=(6, 3, 11), bot=(3, 4), max_len=5,
                       allow_empty=allow_empty)
    C = _multiplicity(p)
    lens = C.sum(axis=1)
    N = C / np.maximum(lens, 1)[:, None]
    ref = (N @ p["h"]).reshape(p["B"], p["T"], p["d"])
    for fn in (dlrm.embedding_bag_forward, dlrm.embedding_bag_forward_fast):
        e = fn(p["h"], p["row_base"], p["indices"], p["offsets"], p["B"], "mean")
        np.testing.assert_allclose(e, ref, rtol=0, atol=1e-14)
    assert np.array_equal(dlrm.bag_lengths(p["offsets"], p["B"], p["T"]), lens.astype(np.int64))
    de = rng.standard_normal((p["B"] * p["T"], p["d"]))
    keys = dlrm.global_rows(p["row_base"], p["indices"], p["offsets"], p["B"])
    bag = dlrm.bag_of_position(p["offsets"], p["B"], p["T"])
    rows, g, _, _, _ = dlrm.embedding_row_gradients(de, keys, bag, 1.0 / np.maximum(lens, 1))
    touched = np.flatnonzero(C.sum(axis=0))
    assert np.array_equal(rows, touched)
    np.testing.assert_allclose(g, (N.T @ de)[touched], rtol=0, atol=1e-13)


def test_embedding_row_gradients_is_transposed_product_and_sort_is_stable():
    rng = np.random.default_rng(6)
    p = random_problem(rng, B=16, T=3, d=4, rows=(6, 3, 11), bot=(3, 4), max_len=5)
    C = _multiplicity(p)
    de = rng.standard_normal((p["B"] * p["T"], p["d"]))
    keys = dlrm.global_rows(p["row_base"], p["indices"], p["offsets"], p["B"])
    bag = dlrm.bag_of_position(p["offsets"], p["B"], p["T"])
    rows, g, sk, perm, heads = dlrm.embedding_row_gradients(de, keys, bag)
    ref = C.T @ de
    touched = np.flatnonzero(C.sum(axis=0))
    assert np.array_equal(rows, touched)
    np.testing.assert_allclose(g, ref[touched], rtol=0, atol=1e-13)
    # Python's sorted() is stable: an independent statement of the required order
    want = sorted(range(len(keys)), key=lambda j: keys[j])
    assert perm.tolist() == want
    assert np.all(np.diff(sk) >= 0)
    same = sk[1:] == sk[:-1]
    assert np.all(np.diff(perm)[same] > 0)
    assert sorted(perm.tolist()) == list(range(len(keys)))
    assert heads.tolist() == [j for j in range(len(sk)) if j == 0 or sk[j] != sk[j - 1]]
    # keys really are table-offset rows and bag ids really are b*T+t
    B, T = p["B"], p["T"]
    for t in range(T):
        for b in range(B):
            for j in range(p["offsets"][t * B + b], p["offsets"][t * B + b + 1]):
                assert keys[j] == p["row_base"][t] + p["indices"][j]
                assert bag[j] == b * T + t


def test_rowwise_adagrad_first_step_closed_form():
    rng = np.random.default_rng(7)
    h = rng.standard_normal((10, 8))
    h0 = h.copy()
    G = np.zeros(10)
    rows = np.array([1, 4, 7])
    g = rng.standard_normal((3, 8))
    lr, eps = 0.01, 1e-8
    dlrm.rowwise_adagrad_update(h, G, rows, g, lr, eps)
    for k, r in enumerate(rows):
        ms = sum(v * v for v in g[k]) / 8
        assert abs(G[r] - ms) < 1e-15
        for c in range(8):
            assert abs(h[r, c] - (h0[r, c] - lr * g[k, c] / (math.sqrt(ms) + eps))) < 1e-15
    untouched = np.setdiff1d(np.arange(10), rows)
    assert np.array_equal(h[untouched], h0[untouched]) and np.all(G[untouched] == 0)
    # a second step accumulates: G = ms1 + ms2
    G1 = G.copy()
    dlrm.rowwise_adagrad_update(h, G, rows, g, lr, eps)
    np.testing.assert_allclose(G[rows], 2 * G1[rows], rtol=1e-15)
    # scale invariance of the first step: |delta| = lr * |g| / rms(g), so rms(delta) = lr
    hh = np.zeros((1, 8)); GG = np.zeros(1)
    dlrm.rowwise_adagrad_update(hh, GG, np.array([0]), 1e3 * g[:1], lr, 0.0)
    assert abs(np.sqrt((hh ** 2).mean()) - lr) < 1e-12


def test_duplicate_rows_get_one_update_with_summed_gradient():
    """A row that occurs in two bags (and twice in one bag) is updated once with the sum."""
    bot, top = (2, 2), (2 + 1, 1)
    row_base = np.array([0, 3])
    rng = np.random.default_rng(8)
    h0 = rng.uniform(-1, 1, (3, 2))
    w0 = rng.uniform(-1, 1, 2 * 2 + 2 + 3 + 1)
    tr = oracle.OracleTrainer(bot, top, row_base, h0, w0, 1, lr_emb=0.1)
    x = rng.standard_normal((2, 2))
    y = np.array([1.0, 0.0])
    indices = np.array([1, 1, 2, 1])         # bag(0,0) = {1,1,2}, bag(0,1) = {1}
    offsets = np.array([0, 3, 4])
    tr.train_step(0, x, y, indices, offsets)
    de = tr.last["de"].reshape(2, 2)
    g1 = 2 * de[0] + de[1]
    g2 = de[0]
    for r, g in ((1, g1), (2, g2)):
        ms = (g * g).mean()
        np.testing.assert_allclose(tr.G[r], ms, rtol=1e-14)
        np.testing.assert_allclose(tr.h[r], h0[r] - 0.1 * g / (math.sqrt(ms) + 1e-8),
                                   rtol=1e-13)
    assert np.array_equal(tr.h[0], h0[0]) and tr.G[0] == 0
    assert tr.last["sorted_pos"].tolist() == [0, 1, 3, 2]
    assert tr.last["seg_starts"].tolist() == [0, 3]


@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_partial_pooling_over_row_shards(pooling):
    """Each shard's partial vector is the multiplicity matrix restricted to the rows the shard
    owns times those rows; the partials add up to the unsharded pooling (then divided by the bag
    length under mean pooling)."""
    rng = np.random.default_rng(9)
    p = random_problem(rng, B=5, T=3, d=4, rows=(10, 3, 7), bot=(3, 5, 4), top_hidden=(6,),
                       max_len=4, allow_empty=True)
    S = 3
    e, parts = dlrm.embedding_bag_forward_sharded(p["h"], p["row_base"], p["indices"], p["offsets"],
                                                  p["B"], S, pooling)
    Cm = _multiplicity(p)
    for s in range(S):
        own = np.zeros(p["row_base"][-1], dtype=bool)
        for t in range(p["T"]):
            rows_t = p["row_base"][t + 1] - p["row_base"][t]
            per = -(-rows_t // S)
            own[p["row_base"][t] + s * per: p["row_base"][t] + min(rows_t, (s + 1) * per)] = True
        want = (Cm[:, own] @ p["h"][own]).reshape(p["B"], p["T"], p["d"])
        np.testing.assert_allclose(parts[s], want, rtol=1e-12, atol=1e-14)
    ref = dlrm.embedding_bag_forward(p["h"], p["row_base"], p["indices"], p["offsets"], p["B"], pooling)
    np.testing.assert_allclose(e, ref, rtol=1e-12, atol=1e-14)


def test_adam_first_step_closed_form_and_untouched_rows():
    """First Adam step from zero state: m_hat = g and v_hat = g^2 exactly, so the row moves by
    lr * g / (|g| + eps) -- about lr * sign(g) -- whatever the betas; rows that are not listed
    keep their values, moments and step counts bit for bit."""
    rng = np.random.default_rng(0)
    h = rng.standard_normal((9, 4)); h0 = h.copy()
    M, V, T = np.zeros_like(h), np.zeros_like(h), np.zeros(9)
    rows = np.array([1, 4, 7])
    g = rng.standard_normal((3, 4))
    dlrm.adam_update(h, M, V, T, rows, g, 0.05, 1e-8, 0.9, 0.999)
    np.testing.assert_allclose(h[rows], h0[rows] - 0.05 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    np.testing.assert_allclose(M[rows], 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(V[rows], 0.001 * g * g, rtol=1e-12)
    others = np.setdiff1d(np.arange(9), rows)
    assert np.array_equal(h[others], h0[others]) and not M[others].any() and not V[others].any()
    assert T.tolist() == [0, 1, 0, 0, 1, 0, 0, 1, 0]


def test_adam_equals_torch_adam_when_every_row_is_touched_every_step():
    """With all rows listed in every step the lazy per-row step count equals the global one and
    the update is plain Adam: compared with torch.optim.Adam over 7 steps of random gradients."""
    rng = np.random.default_rng(1)
    h = rng.standard_normal((5, 3))
    p = torch.tensor(h.copy(), requires_grad=True)
    opt = torch.optim.Adam([p], lr=0.02, betas=(0.8, 0.95), eps=1e-6)
    M, V, T = np.zeros_like(h), np.zeros_like(h), np.zeros(5)
    for _ in range(7):
        g = rng.standard_normal((5, 3))
        dlrm.adam_update(h, M, V, T, np.arange(5), g, 0.02, 1e-6, 0.8, 0.95)
        p.grad = torch.tensor(g.copy())
        opt.step()
    np.testing.assert_allclose(h, p.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_adam_is_lazy_per_row():
    """A row touched in steps 1 and 3 only sees two updates with step counts 1 and 2 -- the same
    as a one-row Adam run on those two gradients alone."""
    rng = np.random.default_rng(2)
    h = rng.standard_normal((3, 2)); ref = h[1:2].copy()
    M, V, T = np.zeros_like(h), np.zeros_like(h), np.zeros(3)
    Mr, Vr, Tr = np.zeros((1, 2)), np.zeros((1, 2)), np.zeros(1)
    gs = [rng.standard_normal((1, 2)) for _ in range(3)]
    dlrm.adam_update(h, M, V, T, np.array([1]), gs[0], 0.1, 1e-8, 0.9, 0.999)
    dlrm.adam_update(h, M, V, T, np.array([0]), gs[1], 0.1, 1e-8, 0.9, 0.999)
    dlrm.adam_update(h, M, V, T, np.array([1]), gs[2], 0.1, 1e-8, 0.9, 0.999)
    for g in (gs[0], gs[2]):
        dlrm.adam_update(ref, Mr, Vr, Tr, np.array([0]), g, 0.1, 1e-8, 0.9, 0.999)
    np.testing.assert_allclose(h[1], ref[0], rtol=1e-14)
    assert T.tolist() == [1, 2, 0]


# ----------------------------------------------------------------------------- interaction
def _golden_lines(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        return [ln.split("#")[0].strip() for ln in fh if ln.split("#")[0].strip()]


def test_interaction_hand_example_and_widths():
    lines = _golden_lines("interaction.txt")
    widths = {}
    for ln in lines:
        k, v = ln.split(":")
        widths[k.strip()] = [float(t) for t in v.split()]
    # widths d + T(T+1)/2 of the three configured models
    for (d, T), F in zip(((16, 4), (64, 8), (64, 26)), widths["widths"]):
        z = np.zeros((1, d)); e = np.zeros((1, T, d))
        assert dlrm.interaction_forward(z, e).shape[1] == int(F)
    z = np.array([[1.0, 2.0]])
    e = np.array([[[3.0, 4.0], [5.0, 6.0]]])
    assert dlrm.interaction_forward(z, e)[0].tolist() == widths["example"]


def test_interaction_T1_is_a_single_dot_product_and_backward_is_product_rule():
    rng = np.random.default_rng(9)
    z = rng.standard_normal((5, 3)); e = rng.standard_normal((5, 1, 3))
    f = dlrm.interaction_forward(z, e)
    assert f.shape == (5, 4)
    np.testing.assert_allclose(f[:, 3], np.einsum("bi,bi->b", z, e[:, 0]), rtol=1e-14)
    df = rng.standard_normal((5, 4))
    dz, de = dlrm.interaction_backward(z, e, df)
    np.testing.assert_allclose(dz, df[:, :3] + df[:, 3:] * e[:, 0], rtol=1e-14)
    np.testing.assert_allclose(de[:, 0], df[:, 3:] * z, rtol=1e-14)


# ----------------------------------------------------------------------------- loss
def test_loss_closed_forms():
    y = np.array([0.0, 1.0, 1.0, 0.0])
    L, dl = dlrm.bce_with_logits(np.zeros(4), y)
    assert abs(L - math.log(2)) < 1e-15
    np.testing.assert_allclose(dl, (0.5 - y) / 4)
    l = np.array([-3.0, 0.7, 2.5, -0.2])
    p = 1 / (1 + np.exp(-l))
    naive = -(y * np.log(p) + (1 - y) * np.log(1 - p)).mean()
    assert abs(dlrm.bce_with_logits(l, y)[0] - naive) < 1e-14
    big = dlrm.bce_with_logits(np.array([800.0, -800.0]), np.array([0.0, 1.0]))[0]
    assert big == 800.0


def test_zero_last_layer_gives_ln2():
    rng = np.random.default_rng(10)
    p = random_problem(rng)
    L = dlrm.DenseLayout(p["bot"], p["top"])
    o, i = L.layer_shapes()[-1]
    p["w"][-(o * i + o):] = 0
    assert abs(_loss(p) - math.log(2)) < 1e-15


def test_normalized_entropy_of_constant_predictor_is_one():
    y = (np.random.default_rng(11).random(1000) < 0.3).astype(float)
    assert abs(oracle.normalized_entropy(np.full(1000, y.mean()), y) - 1.0) < 1e-12


# ----------------------------------------------------------------------------- bf16
def test_bf16_round_ties_to_even_and_matches_torch():
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20,
                  -1 - 2.0 ** -8, 3.0e-39, 65504.0, 0.1], dtype=np.float32)
    got = oracle.bf16_round(x)
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == np.float32(1 + 2.0 ** -6)
    assert got[3] == np.float32(1 + 2.0 ** -7) and got[4] == -1.0
    r = np.random.default_rng(12).standard_normal(10000).astype(np.float32)
    r = np.concatenate([x, r, r * 1e-20, r * 1e20])
    want = torch.tensor(r).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.bf16_round(r), want)


def test_bf16_mode_stays_close_to_full_precision():
    rng = np.random.default_rng(13)
    p = random_problem(rng, B=32, T=2, d=8, rows=(20, 30), bot=(3, 16, 8), top_hidden=(16,))
    L = dlrm.DenseLayout(p["bot"], p["top"])
    out = []
    for bf in (False, True):
        fw = dlrm.dlrm_forward(L, p["w"], p["h"], p["row_base"], p["x"], p["indices"],
                               p["offsets"], bf16=bf)
        out.append(dlrm.dlrm_backward(L, fw, p["y"]))
    assert abs(out[0][0] - out[1][0]) < 2e-2 * out[0][0]
    err = np.linalg.norm(out[0][1] - out[1][1]) / np.linalg.norm(out[0][1])
    assert 1e-5 < err < 5e-2          # rounding is really applied, and stays small


# ----------------------------------------------------------------------------- schedule
def test_fixed_gap_schedule_reports_its_gap_and_shares_tables():
    rng = np.random.default_rng(14)
    p = random_problem(rng)
    tr = oracle.OracleTrainer(p["bot"], p["top"], p["row_base"], p["h"], p["w"], 2)
    batch = (p["x"], p["y"], p["indices"], p["offsets"])
    tr.run_deterministic([batch] * 12, gap=3, algo="ma", alpha=1.0)
    assert tr.steps.tolist() == [6, 6] and tr.rounds == 2
    assert tr.avg_sync_gap() == 3.0
    # alpha = 1 model averaging right after the last sweep: both replicas hold the mean
    assert np.array_equal(tr.W[0], tr.W[1])


def test_running_ne_equals_ne_of_all_predictions_together():
    """OracleTrainer.ne: the running accumulators over several batches give the NE of the
    concatenated predictions (normalized_entropy, itself pinned by the constant predictor),
    for the progressive train metric (losses before each update) and for evaluation."""
    rng = np.random.default_rng(5)
    p = random_problem(rng, B=6, T=2, d=4, rows=(9, 4), bot=(3, 5, 4), top_hidden=(6,))
    tr = oracle.OracleTrainer(p["bot"], p["top"], p["row_base"], p["h"], p["w"], 1, 0.1, 0.1)
    preds, labels = [], []
    for k in range(4):
        q = random_problem(np.random.default_rng(50 + k), B=5 + k, T=2, d=4, rows=(9, 4),
                           bot=(3, 5, 4), top_hidden=(6,))
        tr.train_step(0, q["x"], q["y"], q["indices"], q["offsets"])
        preds.append(1 / (1 + np.exp(-tr.last["logit"])))     # scored before the update
        labels.append(q["y"])
    n, mean, ctr, ne = tr.ne("train")
    assert n == sum(len(y) for y in labels)
    assert abs(ne - oracle.normalized_entropy(np.concatenate(preds), np.concatenate(labels))) < 1e-12
    assert abs(ctr - np.concatenate(labels).mean()) < 1e-15
    ev_p, ev_y = [], []
    for k in range(3):
        q = random_problem(np.random.default_rng(80 + k), B=4 + k, T=2, d=4, rows=(9, 4),
                           bot=(3, 5, 4), top_hidden=(6,))
        tr.eval_logloss(0, q["x"], q["y"], q["indices"], q["offsets"])
        fw = dlrm.dlrm_forward(tr.layout, tr.W[0], tr.h, tr.row_base, q["x"], q["indices"], q["offsets"])
        ev_p.append(1 / (1 + np.exp(-fw["logit"])))
        ev_y.append(q["y"])
    assert abs(tr.ne("eval")[3] - oracle.normalized_entropy(np.concatenate(ev_p), np.concatenate(ev_y))) < 1e-12
    assert tr.ne("train")[0] == n                              # evaluation left the train sums alone
