"""Shared test helpers: small random problems for the oracle and the HIP path."""
import numpy as np


def random_problem(rng, B=4, T=2, d=4, rows=(7, 5), n_dense=3, bot=(3, 5, 4), top_hidden=(6,),
                   max_len=3, allow_empty=False):
    assert len(rows) == T and bot[-1] == d and bot[0] == n_dense
    F = d + T * (T + 1) // 2
    top = (F,) + tuple(top_hidden) + (1,)
    row_base = np.concatenate(([0], np.cumsum(rows)))
    h = rng.uniform(-0.5, 0.5, size=(row_base[-1], d))
    lo = 0 if allow_empty else 1
    lengths = rng.integers(lo, max_len + 1, size=(T, B))
    offsets = np.concatenate(([0], np.cumsum(lengths.ravel()))).astype(np.int64)
    indices = np.empty(offsets[-1], dtype=np.int64)
    for t in range(T):
        a, b = offsets[t * B], offsets[(t + 1) * B]
        indices[a:b] = rng.integers(0, rows[t], size=b - a)
    x = rng.standard_normal((B, n_dense))
    y = (rng.random(B) < 0.4).astype(np.float64)
    P = sum(bot[i + 1] * (bot[i] + 1) for i in range(len(bot) - 1)) + \
        sum(top[i + 1] * (top[i] + 1) for i in range(len(top) - 1))
    w = rng.uniform(-0.7, 0.7, size=P)
    return dict(bot=bot, top=top, row_base=row_base, h=h, w=w, x=x, y=y,
                indices=indices, offsets=offsets, B=B, T=T, d=d)
