"""Pins of the oracle's tree build (A2-A4): brute force on token strings, special cases that
have a closed form, and structural invariants of the outputs."""
import itertools

import numpy as np
import pytest

import dt_synth
from oracle import ref
from tests._brute import brute_frontiers, brute_min_margin, brute_tree, toy_logits
from tests._drive import node_strings, rows_from_fn


def closure_by_matrix_squaring(parents):
    """Reflexive-transitive closure of the parent relation, by boolean matrix squaring."""
    n = len(parents)
    A = np.eye(n, dtype=bool)
    for i in range(1, n):
        A[i, parents[i]] = True
    for _ in range(8):
        A = (A.astype(np.int32) @ A.astype(np.int32)) > 0
    return A


def mask_to_matrix(mask, n):
    M = np.zeros((n, n), bool)
    for i in range(n):
        for j in range(n):
            M[i, j] = (int(mask[i, j // 64]) >> (j % 64)) & 1
    return M


def check_invariants(t, TT, d, k):
    n = t["n_nodes"]
    assert 1 <= n <= TT
    assert t["parents"][0] == -1 and t["depth"][0] == 0
    assert (t["depth"][:n] <= d).all()
    assert (np.diff(t["depth"][:n]) >= 0).all()                 # level-major node order
    for i in range(1, n):
        p = t["parents"][i]
        assert 0 <= p < i and t["depth"][i] == t["depth"][p] + 1
        assert t["score"][i] <= t["score"][p] + 0.0             # log-probs are <= 0
    M = mask_to_matrix(t["anc_mask"], n)
    assert np.array_equal(M, closure_by_matrix_squaring(t["parents"][:n]))
    assert np.array_equal(M.sum(1), t["depth"][:n] + 1)         # popcount = depth + 1
    for p in range(n):
        kids = [i for i in range(1, n) if t["parents"][i] == p]
        assert len(kids) <= k
        toks = [int(t["tokens"][i]) for i in kids]
        assert len(set(toks)) == len(toks)                      # sibling tokens distinct
    # bits above n are never set
    for i in range(n):
        for j in range(n, t["anc_mask"].shape[1] * 64):
            assert not (int(t["anc_mask"][i, j // 64]) >> (j % 64)) & 1


CASES = [(V, TT, d, k) for V in (4, 8) for d in (1, 2, 3) for k in (1, 2, 3)
         for TT in (1, 2, 4, 7, 12, 40)]


@pytest.mark.parametrize("V,TT,d,k", CASES)
def test_tree_matches_brute_force_on_strings(V, TT, d, k):
    for seed in range(3):
        fn = lambda s: toy_logits(seed * 1000 + V, s, V)
        rows = rows_from_fn(ref.build_tree, fn, V, d, k)
        t = ref.build_tree(rows, TT, d, k, 5)
        kept, score, own = brute_tree(fn, V, TT, d, k)
        strs = node_strings(t)
        assert strs[0] == () and t["tokens"][0] == 5 and t["logp"][0] == 0.0 and t["score"][0] == 0.0
        assert set(strs[1:]) == kept
        assert len(strs) == len(set(strs))
        for i in range(1, t["n_nodes"]):
            assert abs(t["score"][i] - score[strs[i]]) < 1e-5
            # the node's own log-probability (the P_d of the acceptance ratio): the brute force's logit minus
            # the float64 log-sum-exp of the row of the node's string prefix, and the one float add per level
            assert abs(t["logp"][i] - own[strs[i]]) < 2e-6 * max(1.0, abs(own[strs[i]]))
            par = t["parents"][i]
            assert t["score"][i] == np.float32(t["score"][par] + t["logp"][i])
            assert strs[t["parents"][i]] == strs[i][:-1]         # parent = string prefix
            assert t["depth"][i] == len(strs[i])
        check_invariants(t, TT, d, k)
        assert t["min_margin"] > 1e-6                            # the brute force assumes no near-ties


def test_k1_is_the_greedy_chain():
    V, d = 16, 5
    fn = lambda s: toy_logits(11, s, V)
    rows = rows_from_fn(ref.build_tree, fn, V, d, 1)
    for TT in (1, 3, 6, 10):
        t = ref.build_tree(rows, TT, d, 1, 0)
        n = min(d, TT - 1) + 1
        assert t["n_nodes"] == n
        s = ()
        for i in range(1, n):
            tok = int(np.argmax(fn(s)))
            assert t["tokens"][i] == tok and t["parents"][i] == i - 1
            s += (tok,)


def test_d1_is_a_star_of_the_root_topk():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((1, 50)).astype(np.float32)
    order = np.lexsort((np.arange(50), -x[0].astype(np.float64)))
    for TT, k in [(4, 8), (20, 8), (9, 8)]:
        t = ref.build_tree(x, TT, 1, k, 0)
        n = min(k, TT - 1) + 1
        assert t["n_nodes"] == n
        assert (t["parents"][1:] == 0).all() and (t["depth"][1:] == 1).all()
        assert sorted(t["tokens"][1:].tolist()) == sorted(order[:n - 1].tolist())
        # node order is ascending pool index = descending logit
        assert t["tokens"][1:].tolist() == order[:n - 1].tolist()


def test_tt1_is_root_only_and_large_tt_keeps_whole_pool():
    rows = dt_synth.draft_rows(dt_synth.config(1), 0)
    t = ref.build_tree(rows, 1, 3, 2, 9)
    assert t["n_nodes"] == 1 and t["tokens"][0] == 9 and t["anc_mask"][0, 0] == 1
    t = ref.build_tree(rows, 100, 3, 2, 9)
    assert t["n_nodes"] == 1 + 2 + 2 * 4                         # P = k + (d-1) k^2 = 10
    check_invariants(t, 100, 3, 2)


def test_src_row_is_the_row_layout_the_header_documents():
    cfg = dt_synth.config(1)
    rows = dt_synth.draft_rows(cfg, 0)
    TT, d, k = 100, 3, 2
    t = ref.build_tree(rows, TT, d, k, 0)
    assert t["src_row"][0] == 0
    for l in range(1, d):
        owned = [t["src_row"][i] for i in range(t["n_nodes"]) if t["depth"][i] == l and t["src_row"][i] >= 0]
        assert owned == list(range(1 + (l - 1) * k, 1 + (l - 1) * k + len(owned)))   # ascending pool index
    assert all(t["src_row"][i] == -1 for i in range(t["n_nodes"]) if t["depth"][i] == d)


def test_no_viable_candidates_stops_expansion():
    V, d, k = 6, 3, 2
    rows = np.full((1 + (d - 1) * k, V), -np.inf, np.float32)
    rows[0, [1, 4]] = [0.5, 0.25]          # root has two viable children
    rows[1, 2] = 1.0                        # first child has one viable child, second has none
    t = ref.build_tree(rows, 16, d, k, 0)
    strs = node_strings(t)
    assert set(strs) == {(), (1,), (4,), (1, 2)}
    rows[1, :] = -np.inf
    t = ref.build_tree(rows, 16, d, k, 0)
    assert set(node_strings(t)) == {(), (1,), (4,)}
    rows[0, :] = -np.inf
    t = ref.build_tree(rows, 16, d, k, 0)
    assert t["n_nodes"] == 1


@pytest.mark.parametrize("ci", [1, 2, 3])
def test_invariants_on_benchmark_shaped_inputs(ci):
    cfg = dt_synth.config(ci)
    TT, d, k = cfg.params[0]
    t = ref.build_tree(dt_synth.draft_rows(cfg, 0), TT, d, k, 1)
    assert t["n_nodes"] == TT
    check_invariants(t, TT, d, k)


def test_invariants_random_sweep():
    rng = np.random.default_rng(5)
    for _ in range(40):
        V = int(rng.integers(33, 400))
        d, k = int(rng.integers(1, 9)), int(rng.integers(1, 13))
        TT = int(rng.integers(1, 129))
        rows = (rng.standard_normal((1 + (d - 1) * k, V)) * 3).astype(np.float32)
        if rng.random() < 0.5:
            rows = dt_synth.f32_to_bf16_bits(rows)
        t = ref.build_tree(rows, TT, d, k, 0)
        assert t["n_nodes"] == min(TT, 1 + k + (d - 1) * k * k)
        check_invariants(t, TT, d, k)


def test_bad_arguments_are_rejected():
    rows = np.zeros((5, 64), np.float32)
    for TT, d, k in [(0, 3, 2), (129, 3, 2), (8, 0, 2), (8, 9, 2), (8, 3, 0), (8, 3, 33), (8, 4, 2)]:
        with pytest.raises(RuntimeError):
            ref.build_tree(rows, TT, d, k, 0)


def test_exact_score_ties_across_rows_go_to_the_lowest_pool_index():
    """All-equal rows: every candidate of a level has the same score, so both the level cut and
    the rerank are decided by the tie-break alone (lowest pool index = earlier parent, lower rank)."""
    V, d, k = 8, 3, 2
    rows = np.zeros((1 + (d - 1) * k, V), np.float32)
    t = ref.build_tree(rows, 6, d, k, 0)
    assert set(node_strings(t)) == {(), (0,), (1,), (0, 0), (0, 1), (1, 0)}
    t = ref.build_tree(rows, 9, d, k, 0)
    # level 2 is complete (4 nodes); its expanded set is the two lowest pool indices = children of
    # the first level-1 node; the two level-3 nodes kept are the children of the first of those.
    assert set(node_strings(t)) == {(), (0,), (1,), (0, 0), (0, 1), (1, 0), (1, 1), (0, 0, 0), (0, 0, 1)}
    assert t["min_margin"] == 0.0          # such an input is exactly what the margin guard flags


@pytest.mark.parametrize("V,TT,d,k", [(8, 6, 3, 2), (8, 3, 3, 3), (6, 12, 4, 2), (7, 5, 2, 3), (5, 9, 3, 3)])
def test_level_outputs_match_the_brute_force_frontiers(V, TT, d, k):
    # what a draft model between the levels is handed: the expanded nodes of every level, in slot order.
    # The brute force works on token strings only; TT is small on purpose (the rerank may later drop
    # expanded nodes from the tree, the level outputs must not care).
    for seed in range(6):
        fn = lambda s: toy_logits(100 + seed, s, V)
        rows = rows_from_fn(ref.build_tree, fn, V, d, k)
        t = ref.build_tree(rows, TT, d, k, with_levels=True)
        want = brute_frontiers(fn, V, d, k)
        strings = {0: [()]}
        for l in range(1, d):
            lv = t["levels"][l]
            mine = []
            for s in range(len(lv["tokens"])):
                par = () if lv["parent_slot"][s] < 0 else strings[l - 1][lv["parent_slot"][s]]
                assert (lv["parent_slot"][s] < 0) == (l == 1)
                mine.append(par + (int(lv["tokens"][s]),))
            strings[l] = mine
            assert mine == want[l], (seed, l)
            for s in range(len(mine)):
                # draft-side mask: own row, the parent's mask, nothing else
                bits = {r for r in range(256) if (int(lv["mask"][s][r // 64]) >> (r % 64)) & 1}
                up = {0} if l == 1 else {r for r in range(256)
                                         if (int(t["levels"][l - 1]["mask"][lv["parent_slot"][s]][r // 64]) >> (r % 64)) & 1}
                assert bits == up | {int(lv["rows"][s])} and len(bits) == l + 1


def test_level_outputs_survive_a_rerank_that_drops_expanded_nodes_and_stop_without_candidates():
    V, d, k = 8, 4, 3
    fn = lambda s: toy_logits(7, s, V)
    rows = rows_from_fn(ref.build_tree, fn, V, d, k)
    small = ref.build_tree(rows, 2, d, k, with_levels=True)        # the tree keeps one node only
    big = ref.build_tree(rows, 40, d, k, with_levels=True)
    for l in range(1, d):
        assert np.array_equal(small["levels"][l]["tokens"], big["levels"][l]["tokens"])
        assert np.array_equal(small["levels"][l]["parent_slot"], big["levels"][l]["parent_slot"])
    assert small["n_nodes"] == 2
    one = ref.build_tree(rows, 1, d, k, with_levels=True)          # TT = 1: nothing is drafted at all
    assert all(len(one["levels"][l]["tokens"]) == 0 for l in range(1, d))
    rows2 = rows.copy()
    rows2[1:1 + k] = -np.inf                                         # level-1 nodes propose nothing
    t = ref.build_tree(rows2, 40, d, k, with_levels=True)
    assert len(t["levels"][1]["tokens"]) == k and len(t["levels"][2]["tokens"]) == 0 and len(t["levels"][3]["tokens"]) == 0


@pytest.mark.parametrize("V,TT,d,k", [(8, 4, 2, 2), (8, 7, 3, 2), (8, 12, 3, 3), (6, 5, 3, 3), (8, 30, 3, 3), (8, 3, 1, 3)])
def test_min_margin_is_the_smallest_cross_row_gap_of_any_cut(V, TT, d, k):
    """The decision margin the parity tests rely on: recomputed on token strings in float64 (every chosen /
    passed-over pair of every cut, pairs proposed by the same string left out)."""
    finite = 0
    for seed in range(12):
        fn = lambda s: toy_logits(300 + seed, s, V)
        rows = rows_from_fn(ref.build_tree, fn, V, d, k)
        got = ref.build_tree(rows, TT, d, k, 0)["min_margin"]
        want = brute_min_margin(fn, V, TT, d, k)
        if np.isinf(want):
            assert np.isinf(got)
        else:
            assert abs(got - want) < 1e-5, (seed, got, want)
            finite += 1
    assert finite > 0 or d == 1            # d = 1: one row only, nothing crosses rows


def test_min_margin_of_a_constructed_gap():
    # two level-1 nodes, both expanded; their rows put exactly one known gap across the final cut
    V, d, k = 4, 2, 2
    rows = np.full((3, V), -30.0, np.float32)
    rows[0, [0, 1]] = [0.0, 0.0]                 # children a=(0), b=(1): lp = -log 2 each (others negligible)
    rows[1, [2, 3]] = [0.0, -1.0]                # under a: lp ~ -0.3133, -1.3133
    rows[2, [2, 3]] = [0.0, -0.75]               # under b: lp ~ -0.3869, -1.1369
    # pool scores: a, b = -0.693; (a,2) -1.006, (b,2) -1.080, (b,3) -1.830, (a,3) -2.006
    t = ref.build_tree(rows, 5, d, k, 0)         # keeps a, b, (a,2), (b,2); passes over (b,3), (a,3)
    assert sorted(node_strings(t)) == [(), (0,), (0, 2), (1,), (1, 2)]
    from scipy.special import logsumexp
    l0, l1, l2 = (logsumexp(rows[i].astype(np.float64)) for i in range(3))
    kept = {"a2": -l0 + 0.0 - l1, "b2": -l0 + 0.0 - l2}
    gone = {"a3": -l0 - 1.0 - l1, "b3": -l0 - 0.75 - l2}
    # cross-row pairs only: (a2, b3), (b2, a3) -- and a/b (root row) against both
    want = min(kept["a2"] - gone["b3"], kept["b2"] - gone["a3"], -l0 - gone["a3"], -l0 - gone["b3"])
    assert abs(t["min_margin"] - want) < 1e-6
    assert abs(want - (kept["b2"] - gone["b3"])) > 1e-3     # the same-row pair (b2, b3) would have been smaller: it is not counted


# ---- the token-count exit of the expansion loop (Algorithm 2), applied on request -----------------------

def levels_expanded(TT, d, k):
    """Closed form with every candidate viable: the root proposes k, every later expansion k*k; level l is
    expanded iff 1 + k + (l-1) k^2 < TT."""
    n = 0
    for l in range(1, d):
        if 1 + k + (l - 1) * k * k >= TT:
            break
        n += 1
    return n


@pytest.mark.parametrize("V,TT,d,k", [(8, 4, 4, 2), (8, 6, 4, 2), (8, 8, 4, 2), (8, 12, 4, 2), (6, 5, 3, 3), (6, 14, 3, 3),
                                      (7, 3, 3, 2), (8, 2, 3, 2), (5, 1, 3, 2), (8, 40, 3, 3)])
def test_early_stop_matches_brute_force_and_the_closed_form_level_count(V, TT, d, k):
    for seed in range(4):
        fn = lambda s: toy_logits(500 + seed, s, V)
        rows = rows_from_fn(ref.build_tree, fn, V, d, k)
        t = ref.build_tree(rows, TT, d, k, 3, with_levels=True, early_stop=True)
        kept, score, _ = brute_tree(fn, V, TT, d, k, early_stop=True)
        strs = node_strings(t)
        assert set(strs[1:]) == kept and len(strs) == len(set(strs))
        for i in range(1, t["n_nodes"]):
            assert abs(t["score"][i] - score[strs[i]]) < 1e-5
        check_invariants(t, TT, d, k)
        n_lv = levels_expanded(TT, d, k) if TT > 1 else 0
        assert [len(t["levels"][l]["tokens"]) > 0 for l in range(1, d)] == [l <= n_lv for l in range(1, d)]
        assert t["n_nodes"] == 1 or t["depth"].max() <= n_lv + 1
        want = brute_frontiers(fn, V, d, k, stop_at=TT)
        for l in range(1, d):
            assert len(t["levels"][l]["tokens"]) == len(want[l])
        # the rows of levels that are never expanded are not read: poison them
        bad = rows.copy()
        bad[1 + n_lv * k:] = np.nan
        t2 = ref.build_tree(bad, TT, d, k, 3, early_stop=True)
        assert t2["n_nodes"] == t["n_nodes"] and (t2["tokens"] == t["tokens"]).all() and (t2["score"] == t["score"]).all()


def test_early_stop_changes_nothing_when_the_budget_outlasts_the_levels_and_cuts_deep_chains_otherwise():
    V, d, k = 8, 4, 2
    # a draft that always continues its own string with near certainty: the best tree is one deep chain
    def chain(s):
        x = np.full(V, -9.0, np.float32)
        x[(len(s) * 3 + 1) % V] = 9.0
        x[(len(s) * 3 + 2) % V] = 0.0
        return x
    rows = rows_from_fn(ref.build_tree, chain, V, d, k)
    late = 1 + k + (d - 2) * k * k + 1                      # first budget the count never reaches before the last level
    a = ref.build_tree(rows, late, d, k)
    b = ref.build_tree(rows, late, d, k, early_stop=True)
    assert a["n_nodes"] == b["n_nodes"] and (a["tokens"] == b["tokens"]).all() and (a["parents"] == b["parents"]).all()
    # TT = 4: without the exit the rerank keeps the chain down to depth 3; with it 1 + 2 + 4 >= 4 stops after level 1
    a = ref.build_tree(rows, 4, d, k)
    b = ref.build_tree(rows, 4, d, k, early_stop=True)
    assert a["depth"].max() == 3 and b["depth"].max() == 2
    assert b["n_nodes"] == 4 and set(node_strings(b)) <= {(), (1,), (2,), (1, 4), (1, 5), (2, 4), (2, 5)}
