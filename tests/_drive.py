"""Test helpers: drive a tree builder level by level with a toy draft model.

`build` is any callable with the oracle's signature build(rows, TT, d, k, root_token) ->
dict(n_nodes, tokens, parents, depth, src_row, ...), so the same driver serves the oracle
and (in GPU tests) the HIP path.
"""
import numpy as np


def node_strings(tree):
    """Token string (tuple) of every node; the root is ()."""
    out = []
    for i in range(tree["n_nodes"]):
        s, j = [], i
        while j > 0:
            s.append(int(tree["tokens"][j]))
            j = int(tree["parents"][j])
        out.append(tuple(reversed(s)))
    return out


def rows_from_fn(build, draft_fn, V, d, k):
    """Fill the draft-row array the way a real draft model would: one level at a time,
    each expanded node's row computed from its own token string."""
    rows = np.zeros((1 + (d - 1) * k, V), np.float32)
    rows[0] = draft_fn(())
    for l in range(1, d):
        P = k + l * k * k
        assert 1 + P <= 128, "driver needs the whole pool to be emitted"
        t = build(rows, 1 + P, l + 1, k, 0)
        strs = node_strings(t)
        for i in range(t["n_nodes"]):
            if t["depth"][i] == l and t["src_row"][i] >= 0:
                rows[t["src_row"][i]] = draft_fn(strs[i])
    return rows
