"""Oracle for the placement of embedding tables on parameter servers (test infrastructure only).

Section 3.1, "Embedding PS": the look-up cost of every table is profiled, and the tables are
assigned to the embedding PSs by solving a bin-packing problem so that the PSs carry similar
costs; a table too large for one PS is partitioned and its parts pool what they own.  The
paper does not name the packing heuristic; the reading taken is the longest-processing-time
rule (items by decreasing cost, each to the currently least loaded PS), with row partitioning
of tables above a row limit and a part's cost proportional to its share of the rows.
"""
from __future__ import annotations


def plan_placement(rows, cost, num_ps, max_rows_per_shard=0):
    """Returns (shards, ps_cost): shards = list of (table, first_row, n_rows, cost, ps) in
    (table, first_row) order."""
    shards = []
    for t, (r, c) in enumerate(zip(rows, cost)):
        parts = 1 if max_rows_per_shard <= 0 else -(-r // max_rows_per_shard)
        per = -(-r // parts)
        first = 0
        while first < r:
            n = min(per, r - first)
            shards.append([t, first, n, c * n / r, -1])
            first += per
    order = sorted(range(len(shards)), key=lambda i: -shards[i][3])   # stable: ties keep order
    load = [0.0] * num_ps
    for i in order:
        p = min(range(num_ps), key=lambda q: load[q])                 # first of the least loaded
        shards[i][4] = p
        load[p] += shards[i][3]
    return [tuple(s) for s in shards], load
