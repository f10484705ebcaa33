"""Pins of the oracle's acceptance (A6-A7) and of its Philox generator."""
import os

import numpy as np
import pytest
from scipy.special import log_softmax

import dt_synth
from oracle import ref
from tests._brute import brute_greedy_accept, toy_logits
from tests._drive import node_strings, rows_from_fn

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Philox

def philox_py(ctr, key):
    """Independent statement of Philox4x32-10 with Python integers."""
    c, k = list(ctr), list(key)
    for _ in range(10):
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return tuple(c)


def test_philox_known_answer_vectors():
    n = 0
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        assert ref.philox4x32(w[0:4], w[4:6]) == tuple(w[6:10])
        assert philox_py(w[0:4], w[4:6]) == tuple(w[6:10])
        n += 1
    assert n == 3


def test_philox_two_implementations_agree_and_uniform_mapping():
    rng = np.random.default_rng(0)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 2 ** 32, 4)]
        key = [int(x) for x in rng.integers(0, 2 ** 32, 2)]
        assert ref.philox4x32(ctr, key) == philox_py(ctr, key)
    seed, step = 0x123456789ABCDEF, 0xFEDCBA9876543
    for seq, node in [(0, 1), (3, 77), (2, 0xFFFFFFFF)]:
        x0 = philox_py([node, seq, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])[0]
        u = ref.uniform(seed, step, seq, node)
        assert u == (x0 >> 8) / 2.0 ** 24 and 0.0 <= u < 1.0


# ------------------------------------------------------------------ greedy

def tree_and_target(seed, V, TT, d, k):
    dfn = lambda s: toy_logits(seed, s, V)
    tfn = lambda s: toy_logits(seed, s, V) + toy_logits(seed + 77, s, V, sigma=1.0)   # correlated target
    rows = rows_from_fn(ref.build_tree, dfn, V, d, k)
    t = ref.build_tree(rows, TT, d, k, 0)
    strs = node_strings(t)
    target = np.stack([tfn(s) for s in strs])
    return t, strs, target, tfn


@pytest.mark.parametrize("V,TT,d,k", [(4, 6, 2, 2), (4, 12, 3, 2), (6, 16, 3, 3), (8, 30, 3, 3), (3, 20, 3, 3)])
def test_greedy_matches_brute_force_over_all_paths(V, TT, d, k):
    hits = 0
    for seed in range(25):
        t, strs, target, tfn = tree_and_target(seed, V, TT, d, k)
        a = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
        path, bonus = brute_greedy_accept(set(strs[1:]), tfn)
        assert a["accept_len"] == len(path)
        assert strs[a["best_node"]] == path
        assert a["out_tokens"][: len(path) + 1].tolist() == list(path) + [bonus]
        assert (a["out_tokens"][len(path) + 1:] == -1).all()
        assert [strs[i] for i in a["path_nodes"][: len(path) + 1]] == [path[:j] for j in range(len(path) + 1)]
        assert np.array_equal(a["node_argmax"], np.argmax(target, axis=1))
        hits += len(path) > 0
    assert hits > 0


def test_speculative_greedy_decoding_equals_sequential_greedy_decoding():
    """Multi-step decode with a random (TT, d, k) per step emits the target's own greedy
    sequence (the paper's lossless / byte-identical claim at temperature 0)."""
    V, steps = 6, 12
    rng = np.random.default_rng(9)
    dfn_ctx = lambda ctx: (lambda s: toy_logits(1, ctx + s, V))
    tfn = lambda s: toy_logits(1, s, V) + toy_logits(2, s, V, sigma=1.5)
    want, s = [], ()
    for _ in range(60):
        tok = int(np.argmax(tfn(s)))
        want.append(tok)
        s += (tok,)
    ctx, emitted, lens = (), [], []
    for _ in range(steps):
        TT, d, k = int(rng.integers(1, 25)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        rows = rows_from_fn(ref.build_tree, dfn_ctx(ctx), V, d, k)
        t = ref.build_tree(rows, TT, d, k, 0)
        strs = node_strings(t)
        target = np.stack([tfn(ctx + st) for st in strs])
        a = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
        new = a["out_tokens"][: a["accept_len"] + 1].tolist()
        emitted += new
        ctx += tuple(new)
        lens.append(a["accept_len"])
    assert emitted == want[: len(emitted)]
    assert max(lens) > 0


def test_target_equal_to_draft_accepts_the_top1_chain():
    cfg = dt_synth.config(1)
    rows = dt_synth.draft_rows(cfg, 0)
    TT, d, k = 11, 3, 2
    t = ref.build_tree(rows, TT, d, k, 0)
    target = np.stack([rows[r] if r >= 0 else np.zeros(cfg.V, np.float32) for r in t["src_row"]])
    a = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
    assert a["accept_len"] == d
    p = a["path_nodes"][: d + 1]
    for j in range(1, d + 1):                     # each step takes the parent's top-1 child
        assert t["tokens"][p[j]] == np.argmax(rows[t["src_row"][p[j - 1]]])


def test_target_argmax_outside_the_tree_accepts_nothing():
    cfg = dt_synth.config(1)
    rows = dt_synth.draft_rows(cfg, 0)
    t = ref.build_tree(rows, 8, 3, 2, 0)
    target = np.zeros((t["n_nodes"], cfg.V), np.float32)
    outside = [v for v in range(cfg.V) if v not in set(t["tokens"].tolist())][0]
    target[:, outside] = 1.0
    a = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
    assert a["accept_len"] == 0 and a["best_node"] == 0 and a["out_tokens"][0] == outside
    assert a["path_nodes"][0] == 0 and (a["path_nodes"][1:] == -1).all()


def test_deepest_wins_and_ties_go_to_lowest_index():
    # root -> {1, 2}; 1 -> {3}; 2 -> {4}; all accepted: depth-2 nodes 3 and 4 tie -> 3.
    tokens = np.array([0, 5, 6, 7, 8], np.int32)
    parents = np.array([-1, 0, 0, 1, 2], np.int32)
    depth = np.array([0, 1, 1, 2, 2], np.int32)
    V = 16
    target = np.zeros((5, V), np.float32)
    logp = np.full(5, -50.0, np.float32)          # draft prob tiny -> alpha = 1 for every node
    a = ref.accept(ref.STOCHASTIC, target, tokens, parents, depth, logp=logp, seed=1, step=2)
    assert a["accepted"].all() and a["best_node"] == 3 and a["accept_len"] == 2
    assert a["out_tokens"][:2].tolist() == [5, 7]


# -------------------------------------------------------------- stochastic

def test_stochastic_with_one_hot_target_reduces_to_greedy():
    for seed in range(10):
        t, strs, target, tfn = tree_and_target(seed, 6, 16, 3, 3)
        g = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
        hot = np.full_like(target, -1e4)
        hot[np.arange(len(target)), np.argmax(target, 1)] = 0.0
        s = ref.accept(ref.STOCHASTIC, hot, t["tokens"], t["parents"], t["depth"], logp=t["logp"],
                       seed=seed, step=3)
        assert s["best_node"] == g["best_node"] and s["accept_len"] == g["accept_len"]
        assert np.array_equal(s["out_tokens"], g["out_tokens"])


def test_stochastic_alpha_one_when_target_equals_draft():
    cfg = dt_synth.config(1)
    rows = dt_synth.draft_rows(cfg, 0)
    t = ref.build_tree(rows, 11, 3, 2, 0)
    target = np.stack([rows[r] if r >= 0 else np.zeros(cfg.V, np.float32) for r in t["src_row"]])
    # make P_T >= P_d certain despite the float rounding of logp
    a = ref.accept(ref.STOCHASTIC, target, t["tokens"], t["parents"], t["depth"], logp=t["logp"] - 1e-3,
                   seed=4, step=0)
    assert a["accepted"].all()
    deepest = int(np.flatnonzero(t["depth"] == t["depth"].max())[0])
    assert a["best_node"] == deepest


def test_stochastic_acceptance_frequency_matches_alpha():
    V = 5
    rng = np.random.default_rng(0)
    tokens = np.array([0, 1, 2, 3], np.int32)
    parents = np.array([-1, 0, 0, 1], np.int32)
    depth = np.array([0, 1, 1, 2], np.int32)
    target = rng.standard_normal((4, V)).astype(np.float32)
    T = 0.8
    lpT = log_softmax(target.astype(np.float64) / T, axis=1)
    logp = np.array([0.0, lpT[0, 1] + 0.7, lpT[0, 2] - 0.2, lpT[1, 3] + 1.5], np.float32)
    alpha = np.minimum(1.0, np.exp([lpT[0, 1] - logp[1], lpT[0, 2] - logp[2], lpT[1, 3] - logp[3]]))
    n = 20000
    cnt = np.zeros(3)
    bonus_hist = np.zeros(V)
    for step in range(n):
        a = ref.accept(ref.STOCHASTIC, target, tokens, parents, depth, logp=logp, temperature=T, seed=42, step=step)
        cnt += a["accepted"][1:]
        if a["best_node"] == 2:
            bonus_hist[a["out_tokens"][1]] += 1
    sigma = np.sqrt(alpha * (1 - alpha) / n)
    assert (np.abs(cnt / n - alpha) < 4.5 * sigma + 1e-9).all()
    assert alpha[1] == 1.0 and cnt[1] == n
    # when node 1 is rejected the walk ends at node 2: the bonus follows softmax(target[2]/T)
    m = bonus_hist.sum()
    p0 = np.exp(lpT[2])
    assert m > 1000 and (np.abs(bonus_hist / m - p0) < 4.5 * np.sqrt(p0 * (1 - p0) / m)).all()


def test_bonus_is_the_inverse_cdf_of_the_target_distribution():
    V = 7
    tokens, parents, depth = np.array([0], np.int32), np.array([-1], np.int32), np.array([0], np.int32)
    target = np.array([[0.1, 2.0, -1.0, 0.5, 0.5, 3.0, -2.0]], np.float32)
    p = np.exp(log_softmax(target[0].astype(np.float64) / 1.3))
    cdf = np.cumsum(p)
    for step in range(300):
        a = ref.accept(ref.STOCHASTIC, target, tokens, parents, depth, logp=np.zeros(1, np.float32),
                       temperature=1.3, seed=7, step=step)
        u = ref.uniform(7, step, 0, 0xFFFFFFFF)
        assert a["out_tokens"][0] == int(np.searchsorted(cdf, u, side="right"))
        assert a["accept_len"] == 0


def test_argmax_ties_go_to_the_lowest_token_id():
    rng = np.random.default_rng(12)
    V = 40
    tokens = np.array([0, 3, 4], np.int32)
    parents = np.array([-1, 0, 0], np.int32)
    depth = np.array([0, 1, 1], np.int32)
    for _ in range(20):
        target = rng.integers(0, 3, size=(3, V)).astype(np.float32)     # every row has many maxima
        a = ref.accept(ref.GREEDY, target, tokens, parents, depth)
        assert np.array_equal(a["node_argmax"], np.argmax(target, axis=1))   # numpy: first occurrence
        assert a["out_tokens"][a["accept_len"]] == np.argmax(target[a["best_node"]])
    target = np.zeros((3, V), np.float32)
    target[0, [4, 3]] = 1.0                       # tie between the two children: token 3 wins
    a = ref.accept(ref.GREEDY, target, tokens, parents, depth)
    assert a["best_node"] == 1 and a["out_tokens"][:2].tolist() == [3, 0]
    bits = dt_synth.f32_to_bf16_bits(target)
    b = ref.accept(ref.GREEDY, bits, tokens, parents, depth)
    assert b["best_node"] == 1 and np.array_equal(a["out_tokens"], b["out_tokens"])


# ------------------------------------------------- target-sampled (distribution-preserving) mode

def _ar_sample(tfn, ctx, n, T, seed, step, seq):
    """The target's own autoregressive sampling with the uniforms of one speculative step: position j of the
    step uses the uniform of depth j.  numpy cumsum / searchsorted, no oracle code."""
    out, s = [], ctx
    for j in range(n):
        x = tfn(s).astype(np.float64) / T
        p = np.exp(x - x.max()); p /= p.sum()
        u = ref.uniform(seed, step, seq, 0x80000000 + j)
        tok = int(np.searchsorted(np.cumsum(p), u, side="right"))
        out.append(min(tok, len(p) - 1))
        s += (out[-1],)
    return out


def test_sampled_verification_emits_the_targets_own_samples_token_for_token():
    """One speculative step in mode 2 returns exactly the leading tokens of the autoregressive sample drawn
    with the same uniforms: as many as form a path of the tree, plus one (the bonus)."""
    V = 6
    rng = np.random.default_rng(21)
    lens = []
    for trial in range(150):
        TT, d, k = int(rng.integers(1, 30)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        T = float(rng.choice([0.7, 1.0, 1.6]))
        dfn = lambda s: toy_logits(40 + trial % 7, s, V)
        tfn = lambda s: toy_logits(40 + trial % 7, s, V) + toy_logits(90, s, V, sigma=0.7)   # close to the draft
        rows = rows_from_fn(ref.build_tree, dfn, V, d, k)
        t = ref.build_tree(rows, TT, d, k, 0)
        strs = node_strings(t)
        target = np.stack([tfn(st) for st in strs])
        a = ref.accept(ref.SAMPLED, target, t["tokens"], t["parents"], t["depth"], temperature=T, seed=5, step=trial, seq=3)
        if a["min_margin"] < 1e-9:
            continue
        ar = _ar_sample(tfn, (), d + 1, T, 5, trial, 3)
        n = 0
        while n < d and tuple(ar[: n + 1]) in set(strs):
            n += 1
        assert a["accept_len"] == n, trial
        assert a["out_tokens"][: n + 1].tolist() == ar[: n + 1], trial
        assert strs[a["best_node"]] == tuple(ar[:n])
        lens.append(n)
    assert max(lens) >= 2 and min(lens) == 0


def test_sampled_verification_preserves_the_target_distribution():
    """Whatever the tree, the first emitted token is distributed as softmax(target(root)/T), and the second,
    given the first, as the target's next-token distribution after it."""
    V, T = 5, 1.3
    dfn = lambda s: toy_logits(3, s, V)
    tfn = lambda s: toy_logits(3, s, V) * 0.5 + toy_logits(4, s, V, sigma=1.0)
    rows = rows_from_fn(ref.build_tree, dfn, V, 3, 2)
    t = ref.build_tree(rows, 7, 3, 2, 0)
    strs = node_strings(t)
    target = np.stack([tfn(st) for st in strs])
    steps = 20000
    first = np.zeros(V)
    pair = np.zeros((V, V))
    n_two = 0
    for step in range(steps):
        a = ref.accept(ref.SAMPLED, target, t["tokens"], t["parents"], t["depth"], temperature=T, seed=8, step=step)
        out = a["out_tokens"]
        first[out[0]] += 1
        if a["accept_len"] >= 1:
            pair[out[0], out[1]] += 1
            n_two += 1
    sm = lambda x: np.exp(x / T - np.max(x / T)) / np.exp(x / T - np.max(x / T)).sum()
    p1 = sm(tfn(()).astype(np.float64))
    assert np.abs(first / steps - p1).max() < 4 * np.sqrt(0.25 / steps)
    assert n_two > 2000
    for tok in range(V):
        if pair[tok].sum() > 1500:                       # first tokens that are in the tree and drawn often
            p2 = sm(tfn((tok,)).astype(np.float64))
            assert np.abs(pair[tok] / pair[tok].sum() - p2).max() < 4.5 * np.sqrt(0.25 / pair[tok].sum())


def test_sampled_verification_with_a_one_hot_target_is_greedy():
    V = 7
    rng = np.random.default_rng(4)
    dfn = lambda s: toy_logits(6, s, V)
    rows = rows_from_fn(ref.build_tree, dfn, V, 3, 3)
    t = ref.build_tree(rows, 12, 3, 3, 0)
    target = np.full((t["n_nodes"], V), -30.0, np.float32)
    for i in range(t["n_nodes"]):
        target[i, rng.integers(0, V)] = 30.0
    g = ref.accept(ref.GREEDY, target, t["tokens"], t["parents"], t["depth"])
    for step in range(20):
        s = ref.accept(ref.SAMPLED, target, t["tokens"], t["parents"], t["depth"], temperature=1.0, seed=1, step=step)
        assert s["accept_len"] == g["accept_len"] and np.array_equal(s["out_tokens"], g["out_tokens"])
        assert np.array_equal(s["node_argmax"], g["node_argmax"])


# ---------------------------------------------- the decision margins the parity tests rely on

def _small_tree_and_target(seed, V=9, TT=14, d=3, k=3):
    t, strs, target, _ = tree_and_target(seed, V, TT, d, k)
    return t, target


def test_stochastic_min_margin_is_recomputed_in_float64():
    """min over nodes with alpha < 1 of |u - alpha|, and the distance of the bonus uniform to the edges of its
    CDF bin (lower edge only when the bonus is not token 0): numpy/scipy float64 from the same uniforms."""
    seen_alpha, seen_bonus = 0, 0
    for seed in range(30):
        t, target = _small_tree_and_target(seed)
        T = float(np.float32([0.7, 1.0, 1.9][seed % 3]))     # the temperature crosses the C interface as a float
        a = ref.accept(ref.STOCHASTIC, target, t["tokens"], t["parents"], t["depth"], logp=t["logp"], temperature=T,
                       seed=11, step=seed, seq=2)
        lpT = log_softmax(target.astype(np.float64) / T, axis=1)
        m_alpha = np.inf
        acc = [True]
        for i in range(1, t["n_nodes"]):
            alpha = min(1.0, float(np.exp(lpT[t["parents"][i], t["tokens"][i]] - np.float64(t["logp"][i]))))
            u = ref.uniform(11, seed, 2, i)
            acc.append(u < alpha)
            if alpha < 1.0:
                m_alpha = min(m_alpha, abs(u - alpha))
        assert a["accepted"].tolist() == acc
        cdf = np.cumsum(np.exp(lpT[a["best_node"]]))
        u = ref.uniform(11, seed, 2, 0xFFFFFFFF)
        bonus = int(np.searchsorted(cdf, u, side="right"))
        assert a["out_tokens"][a["accept_len"]] == bonus
        m_bonus = cdf[bonus] - u
        if bonus > 0:
            m_bonus = min(m_bonus, u - cdf[bonus - 1])
        want = min(m_alpha, m_bonus)
        assert abs(a["min_margin"] - want) <= 1e-6 * want + 1e-12, (seed, a["min_margin"], want)
        seen_alpha += m_alpha < m_bonus
        seen_bonus += m_bonus < m_alpha
    assert seen_alpha > 3 and seen_bonus > 3          # both terms decide the minimum in some case


def test_sampled_node_margins_and_min_margin_are_recomputed_in_float64():
    for seed in range(30):
        t, target = _small_tree_and_target(seed)
        T = float(np.float32([0.7, 1.0, 1.9][seed % 3]))
        a = ref.accept(ref.SAMPLED, target, t["tokens"], t["parents"], t["depth"], temperature=T, seed=12, step=seed, seq=1)
        p = np.exp(log_softmax(target.astype(np.float64) / T, axis=1))
        want_node, draw = [], []
        for i in range(t["n_nodes"]):
            cdf = np.cumsum(p[i])
            u = ref.uniform(12, seed, 1, 0x80000000 + int(t["depth"][i]))
            y = int(np.searchsorted(cdf, u, side="right"))
            draw.append(y)
            m = cdf[y] - u
            if y > 0:
                m = min(m, u - cdf[y - 1])
            want_node.append(m)
        assert a["node_argmax"].tolist() == draw
        assert np.allclose(a["node_margin"], want_node, rtol=1e-6, atol=1e-12)
        # the sequence's margin: the nodes whose draw decides the output (all ancestors accepted)
        ok = [True]
        for i in range(1, t["n_nodes"]):
            ok.append(ok[t["parents"][i]] and t["tokens"][i] == draw[t["parents"][i]])
        want = min(m for m, o in zip(want_node, ok) if o)
        assert abs(a["min_margin"] - want) <= 1e-6 * want + 1e-12
        assert want >= min(want_node)


def test_a_uniform_of_exactly_zero_skips_tokens_without_mass():
    """u = 0 is reachable (probability 2^-24 per draw).  The inverse CDF is "first id with cdf > u", so tokens of
    zero probability in front of the first token with mass are never drawn (a ">=" test would draw token 0)."""
    BONUS_STEP, DEPTH0_STEP = 657078, 2169497        # found by search; the asserts below re-check them
    assert ref.uniform(0, BONUS_STEP, 0, 0xFFFFFFFF) == 0.0
    assert philox_py([0xFFFFFFFF, 0, BONUS_STEP, 0], [0, 0])[0] >> 8 == 0
    assert ref.uniform(0, DEPTH0_STEP, 0, 0x80000000) == 0.0
    assert philox_py([0x80000000, 0, DEPTH0_STEP, 0], [0, 0])[0] >> 8 == 0
    V = 6
    target = np.array([[-np.inf, -np.inf, 0.5, 1.0, -np.inf, 0.0]], np.float32)
    one = (np.array([0], np.int32), np.array([-1], np.int32), np.array([0], np.int32))
    a = ref.accept(ref.STOCHASTIC, target, *one, logp=np.zeros(1, np.float32), seed=0, step=BONUS_STEP, seq=0)
    assert a["out_tokens"][0] == 2
    a = ref.accept(ref.SAMPLED, target, *one, seed=0, step=DEPTH0_STEP, seq=0)
    assert a["out_tokens"][0] == 2 and a["node_argmax"][0] == 2
    target[0, 0] = -3.0                               # token 0 with mass: u = 0 draws it
    a = ref.accept(ref.STOCHASTIC, target, *one, logp=np.zeros(1, np.float32), seed=0, step=BONUS_STEP, seq=0)
    assert a["out_tokens"][0] == 0
