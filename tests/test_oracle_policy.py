"""Pins of the oracle's action selection: action table, policy MLP, action cache (Algorithm 1)."""
import math
import os

import numpy as np
import pytest

from oracle import ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def golden_sets():
    gold = dict(l.split(None, 1) for l in open(os.path.join(ROOT, "tests", "golden", "action_space.txt"))
                if not l.startswith("#"))
    return [list(map(int, gold[key].split())) for key in ("TT", "d", "k")]


def test_action_table_is_the_printed_space_after_the_printed_filter():
    TTs, ds, ks = golden_sets()
    table = ref.action_table()
    brute = [(TT, d, k) for TT in TTs for d in ds for k in ks if TT <= k ** (d - 1)]   # exact integer power
    assert [tuple(r) for r in table] == brute
    dropped = sorted(set((TT, d, k) for TT in TTs for d in ds for k in ks) - set(brute))
    assert dropped == [(80, 3, 8), (96, 3, 8), (128, 3, 8)] and len(table) == 177
    assert len(set(map(tuple, table))) == len(table)


def rand_net(rng, F, H, A):
    W1 = (rng.standard_normal((F, H)) / np.sqrt(F)).astype(np.float32)
    W2 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float32)
    W3 = (rng.standard_normal((H, A)) / np.sqrt(H)).astype(np.float32)
    b1, b2, b3 = (rng.standard_normal(n).astype(np.float32) * 0.1 for n in (H, H, A))
    return W1, b1, W2, b2, W3, b3


@pytest.mark.parametrize("F,H,A", [(12, 5, 7), (300, 64, 20), (1536, 128, 177)])
def test_policy_logits_match_numpy_float64(F, H, A):
    rng = np.random.default_rng(F)
    net = rand_net(rng, F, H, A)
    x = rng.standard_normal(F).astype(np.float32)
    W1, b1, W2, b2, W3, b3 = (a.astype(np.float64) for a in net)
    want = np.tanh(np.tanh(x.astype(np.float64) @ W1 + b1) @ W2 + b2) @ W3 + b3
    got = ref.policy_logits(x, *net)
    assert np.abs(got - want).max() < 1e-12


def test_policy_logits_closed_forms_and_operand_orientation():
    rng = np.random.default_rng(1)
    F, H, A = 9, 4, 6
    W1, b1, W2, b2, W3, b3 = rand_net(rng, F, H, A)
    x = rng.standard_normal(F).astype(np.float32)
    # no signal path: the logits are the last bias
    assert np.allclose(ref.policy_logits(x, W1, b1, W2, b2, np.zeros_like(W3), b3), b3, atol=0)
    # scalar chain
    one = lambda v: np.array([[v]], np.float32)
    g = ref.policy_logits(np.array([0.7], np.float32), one(1.5), np.array([0.2], np.float32), one(-0.8),
                          np.array([0.1], np.float32), one(2.0), np.array([-0.3], np.float32))
    f = np.float32
    want = float(f(2.0)) * math.tanh(float(f(-0.8)) * math.tanh(float(f(1.5)) * float(f(0.7)) + float(f(0.2))) + float(f(0.1))) + float(f(-0.3))
    assert abs(g[0] - want) < 1e-14
    # [in][out] orientation: a single weight W2[i][j] carries hidden unit i of layer 1 to unit j of layer 2 only
    W2s = np.zeros((H, H), np.float32); W2s[1, 3] = 1.0
    W3s = np.zeros((H, A), np.float32); W3s[3, 2] = 1.0; W3s[1, 4] = 1.0      # unit 3 -> action 2, unit 1 -> action 4
    W1s = np.zeros((F, H), np.float32); W1s[5, 1] = 1.0                        # feature 5 -> unit 1
    z = np.zeros(H, np.float32)
    g = ref.policy_logits(x, W1s, z, W2s, z, W3s, np.zeros(A, np.float32))
    want2 = math.tanh(math.tanh(float(x[5])))
    assert abs(g[2] - want2) < 1e-14 and abs(g[4]) < 1e-300 and np.count_nonzero(g) == 1


def test_action_cache_queries_the_policy_once_per_interval():
    rng = np.random.default_rng(2)
    A = 11
    for N in (1, 2, 10, 30):
        cs, ca = 0, -1
        used, queried_at = [], []
        per_step_logits = rng.standard_normal((95, A))
        for t in range(95):
            r = ref.policy_step(cs, ca, per_step_logits[t], N)
            cs, ca = r["cache_step"], r["cached_action"]
            used.append(r["action"])
            if r["queried"]:
                queried_at.append(t)
                assert r["action"] == int(np.argmax(per_step_logits[t]))
        assert queried_at == list(range(0, 95, N))                   # ceil(T/N) queries, at the interval starts
        for t in range(95):
            assert used[t] == used[(t // N) * N]                     # an action persists for N decision points
    # between queries the logits are not even looked at
    r = ref.policy_step(3, 5, None, 10)
    assert r["action"] == 5 and not r["queried"] and r["cache_step"] == 4
    r = ref.policy_step(9, 5, None, 10)
    assert r["cache_step"] == 0                                      # interval over: next point queries again
    r = ref.policy_step(4, -1, np.array([0.0, 2.0, 1.0]), 10)        # nothing cached yet: query
    assert r["queried"] and r["action"] == 1 and r["cache_step"] == 1


def test_greedy_ties_go_to_the_lowest_action_and_margin_is_the_top2_gap():
    r = ref.policy_step(0, -1, np.array([1.0, 3.0, 3.0, -2.0]), 5)
    assert r["action"] == 1 and r["margin"] == 0.0
    r = ref.policy_step(0, -1, np.array([1.0, 3.5, 3.0, -2.0]), 5)
    assert r["action"] == 1 and abs(r["margin"] - 0.5) < 1e-15


def test_sampled_actions_follow_the_softmax_and_the_inverse_cdf():
    logits = np.array([0.3, -1.0, 2.0, 0.0, 1.2])
    p = np.exp(logits - logits.max()); p /= p.sum()
    cdf = np.cumsum(p)
    counts = np.zeros(5)
    T = 20000
    for step in range(T):
        r = ref.policy_step(0, -1, logits, 3, mode=1, seed=77, step=step, seq=4)
        u = ref.uniform(77, step, 4, 0xFFFFFFFE)
        if r["margin"] > 1e-12:
            assert r["action"] == int(np.searchsorted(cdf, u, side="right"))
        counts[r["action"]] += 1
    assert np.abs(counts / T - p).max() < 4 * np.sqrt(0.25 / T)


# ------------------------------------------------------- reward averaged over the cache interval

def _run_intervals(N, steps, tokens, elapsed, start=(0, -1)):
    """Drive the action cache and the reward bookkeeping together for `steps` decision points."""
    cs, ca = start
    acc = dict(sum=0.0, steps=0)
    out = []
    lg = np.array([0.0, 1.0, 0.5])
    for t in range(steps):
        r = ref.policy_step(cs, ca, lg, N)
        cs, ca = r["cache_step"], r["cached_action"]
        done, avg = ref.reward_step(cs, tokens[t], elapsed[t], acc)
        out.append((r["queried"], done, avg))
    return out, acc


@pytest.mark.parametrize("N", [1, 3, 10, 30])
def test_reward_is_the_mean_of_tokens_per_second_over_each_cache_interval(N):
    rng = np.random.default_rng(N)
    steps = 3 * N + (N // 2)
    tokens = rng.integers(1, 9, steps).astype(np.float64)
    elapsed = rng.uniform(0.004, 0.03, steps)
    out, acc = _run_intervals(N, steps, tokens, elapsed)
    per_step = tokens / elapsed
    for t, (queried, done, avg) in enumerate(out):
        assert queried == (t % N == 0)                       # an interval opens with a policy query ...
        assert done == (t % N == N - 1)                      # ... and closes N decision points later
        if done:
            want = per_step[t - N + 1:t + 1].mean()          # the averaged reward: 1/N sum tokens_i / seconds_i
            assert abs(avg - want) <= 1e-12 * want
        else:
            assert np.isnan(avg)                             # nothing reported inside an interval
    # the open interval at the end keeps its partial sum
    tail = steps % N
    assert acc["steps"] == tail and abs(acc["sum"] - per_step[steps - tail:].sum()) < 1e-9


def test_reward_closed_forms_and_bad_arguments():
    N = 10
    # constant speed: the average is that speed; tokens 1..N in one second each: (N+1)/2
    out, _ = _run_intervals(N, N, np.full(N, 4.0), np.full(N, 0.02))
    assert out[-1][1] and abs(out[-1][2] - 200.0) < 1e-9
    out, _ = _run_intervals(N, N, np.arange(1, N + 1, dtype=np.float64), np.ones(N))
    assert abs(out[-1][2] - (N + 1) / 2) < 1e-12
    # a generation that starts in the middle of an interval (4 of 10 steps already used by a cached action)
    out, _ = _run_intervals(N, 6, np.full(6, 3.0), np.full(6, 0.5), start=(4, 2))
    assert [d for _, d, _ in out] == [False] * 5 + [True] and abs(out[-1][2] - 6.0) < 1e-12   # mean over the 6 seen
    acc = dict(sum=0.0, steps=0)
    for bad in (0.0, -1.0):
        with pytest.raises(RuntimeError):
            ref.reward_step(1, 2.0, bad, acc)
