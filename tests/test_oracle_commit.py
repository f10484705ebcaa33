"""Pins of the oracle's input update (KV commit after verification).

Paper, Appendix "System Profiling and Overhead Analysis": the input update keeps the accepted tokens in
the KV cache and discards the rejected ones.  The pins tie ref.commit_rows to things other than itself:
element-by-element Python loops, the tree's ancestor sets (built by different oracle code), and the
attention definition (attending over the committed cache must equal tree attention of the accepted leaf).
"""
import numpy as np
import pytest

import dt_synth
from oracle import ref
from tests._drive import rows_from_fn


def _rand_bf16(rng, shape):
    return dt_synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("head_major", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_commit_matches_plain_loops(head_major, dtype):
    rng = np.random.default_rng(5)
    N, Hkv, D, cap, L = 9, 3, 8, 20, 11
    mk = (lambda sh: rng.standard_normal(sh).astype(np.float32)) if dtype == "f32" else (lambda sh: _rand_bf16(rng, sh))
    tree = mk((N, Hkv, D))
    cache = mk((Hkv, cap, D) if head_major else (cap, Hkv, D))
    before = cache.copy()
    path = np.array([0, 2, 5, 7, -1, -1, -1, -1, -1], np.int32)
    new_len = ref.commit_rows(cache, L, tree, path, 3, head_major=head_major)
    assert new_len == L + 4
    for t in range(cap):
        for g in range(Hkv):
            got = cache[g, t] if head_major else cache[t, g]
            old = before[g, t] if head_major else before[t, g]
            want = tree[path[t - L], g] if L <= t < L + 4 else old
            assert np.array_equal(got, want), (t, g)


def test_commit_respects_the_capacity_and_rejects_bad_paths():
    rng = np.random.default_rng(6)
    tree = rng.standard_normal((5, 2, 4)).astype(np.float32)
    cache = np.zeros((6, 2, 4), np.float32)
    path = np.array([0, 1, 3, 4], np.int32)
    assert ref.commit_rows(cache, 4, tree, path, 3) == 6                 # rows 4, 5 fit; the rest do not
    assert np.array_equal(cache[4], tree[0]) and np.array_equal(cache[5], tree[1])
    assert not cache[:4].any()
    full = np.ones((4, 2, 4), np.float32)
    assert ref.commit_rows(full, 4, tree, path, 0) == 4 and (full == 1).all()   # full cache: nothing written
    with pytest.raises(RuntimeError):
        ref.commit_rows(cache, 0, tree, np.array([0, 5], np.int32), 1)   # node outside the tree
    with pytest.raises(RuntimeError):
        ref.commit_rows(cache, 7, tree, path, 0)                         # prefix longer than the cache


def test_committed_rows_are_exactly_the_ancestor_set_of_the_accepted_leaf():
    # tree from build_tree, acceptance from accept; the committed rows must be the rows whose bits are set
    # in anc_mask[best] (the mask is produced by code that knows nothing of path_nodes), in depth order
    rng = np.random.default_rng(11)
    V, TT, d, k = 200, 24, 4, 3
    rows = rng.standard_normal((1 + (d - 1) * k, V)).astype(np.float32) * 2
    t = ref.build_tree(rows, TT, d, k)
    N = t["n_nodes"]
    target = rng.standard_normal((N, V)).astype(np.float32)
    for i in range(1, N):                                   # make a good share of the nodes acceptable
        if rng.random() < 0.7:
            target[t["parents"][i], t["tokens"][i]] = 50.0
    acc = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
    assert acc["accept_len"] >= 1
    Hkv, D, L, cap = 2, 4, 5, 16
    tree_k = rng.standard_normal((N, Hkv, D)).astype(np.float32)
    cache = np.zeros((cap, Hkv, D), np.float32)
    new_len = ref.commit_rows(cache, L, tree_k, acc["path_nodes"], acc["accept_len"])
    mask = t["anc_mask"][acc["best_node"]]
    members = [j for j in range(N) if (int(mask[j // 64]) >> (j % 64)) & 1]
    assert new_len == L + len(members)
    assert [int(t["depth"][j]) for j in members] == list(range(len(members)))
    for s, j in enumerate(members):
        assert np.array_equal(cache[L + s], tree_k[j])
    assert not cache[new_len:].any()


def test_attention_over_the_committed_cache_equals_tree_attention_of_the_leaf():
    # keys visible to the accepted leaf = prefix + its ancestors + itself.  After the commit the same keys
    # are cache rows 0 .. new_len-1; attending with the leaf's query over them (the last one supplied as
    # a one-node tree) must give the leaf's tree-attention output.
    rng = np.random.default_rng(12)
    Hq, Hkv, D, L, N = 4, 2, 16, 7, 6
    parents = np.array([-1, 0, 0, 1, 3, 2], np.int32)
    depth = np.array([0, 1, 1, 2, 3, 2], np.int32)
    masks = np.zeros((N, 2), np.uint64)
    for i in range(N):
        m = (1 << i) | (int(masks[parents[i], 0]) if parents[i] >= 0 else 0)
        masks[i, 0] = m
    q = _rand_bf16(rng, (N, Hq, D)); kt = _rand_bf16(rng, (N, Hkv, D)); vt = _rand_bf16(rng, (N, Hkv, D))
    kp = _rand_bf16(rng, (L, Hkv, D)); vp = _rand_bf16(rng, (L, Hkv, D))
    scale = D ** -0.5
    full = ref.tree_attention(q, kt, vt, kp, vp, masks, scale)
    leaf, path = 4, np.array([0, 1, 3, 4], np.int32)
    kc = np.zeros((L + 8, Hkv, D), np.uint16); vc = np.zeros_like(kc)
    kc[:L], vc[:L] = kp, vp
    n1 = ref.commit_rows(kc, L, kt, path, 3)
    n2 = ref.commit_rows(vc, L, vt, path, 3)
    assert n1 == n2 == L + 4
    one = np.zeros((1, 2), np.uint64); one[0, 0] = 1
    again = ref.tree_attention(q[leaf:leaf + 1], kc[n1 - 1:n1], vc[n1 - 1:n1], kc[:n1 - 1], vc[:n1 - 1], one, scale)
    assert np.array_equal(again[0], full[leaf])
