"""Brute-force statements of the tree build and of greedy acceptance, on token STRINGS.

No pool indices, slots or row arithmetic here: a candidate is the tuple of tokens from
the root to it, its parent is the tuple without the last token, sets are Python sets and
orders are Python tuple sorts.  A toy "draft model" maps a token string to a logit row.
Used to pin the oracle's bookkeeping on tiny inputs (V <= 8, d <= 3, k <= 3).
"""
import numpy as np
from scipy.special import logsumexp


def toy_logits(seed, string, V, sigma=2.0):
    """Deterministic float32 logit row of a token string (a toy draft or target model)."""
    h = np.random.SeedSequence([seed, len(string)] + [int(t) + 1 for t in string])
    return (np.random.Generator(np.random.PCG64(h)).standard_normal(V) * sigma).astype(np.float32)


def brute_tree(draft_fn, V, TT, d, k, early_stop=False):
    """Returns (set of kept strings, cumulative score of every candidate string, own log-probability
    of every candidate string = its logit minus the log-sum-exp of the row that proposed it).
    early_stop: no level is expanded once the root and all strings proposed so far number TT or more."""
    def topk(string):
        x = draft_fn(string).astype(np.float64)
        lse = logsumexp(x)
        order = sorted(range(V), key=lambda t: (-x[t], t))[:k]
        return [(t, x[t] - lse) for t in order if x[t] > -np.inf]

    score, own = {}, {}
    levels = []
    frontier = [()]          # strings to expand at this level
    for level in range(1, d + 1):
        cands = []
        for s in frontier:
            for t, lp in topk(s):
                c = s + (t,)
                score[c] = (score[s] if s else 0.0) + lp
                own[c] = lp
                cands.append(c)
        levels.append(cands)
        if not cands:
            break
        if early_stop and 1 + sum(len(lv) for lv in levels) >= TT:
            break
        ranked = sorted(cands, key=lambda c: -score[c])
        frontier = ranked[:k]
    everyone = [c for lv in levels for c in lv]
    ranked = sorted(everyone, key=lambda c: -score[c])
    kept = set(ranked[:max(TT - 1, 0)])
    return kept, score, own


def brute_frontiers(draft_fn, V, d, k, stop_at=None):
    """The strings expanded at levels 1..d-1, each level as an ORDERED list: a level's chosen strings are
    listed parent by parent (in the order the parents were listed one level up) and, under one parent, in
    the order of that parent's top-k list.  Returns [None, level 1, ..., level d-1].
    stop_at: a token budget; a level is expanded only while the root and the strings proposed so far number
    fewer than it."""
    def topk(string):
        x = draft_fn(string).astype(np.float64)
        lse = logsumexp(x)
        order = sorted(range(V), key=lambda t: (-x[t], t))[:k]
        return [(t, x[t] - lse) for t in order if x[t] > -np.inf]

    score = {(): 0.0}
    out = [None]
    frontier = [()]
    for level in range(1, d):
        cands = []                      # in (parent order, rank under the parent) order
        for s in frontier:
            for t, lp in topk(s):
                score[s + (t,)] = score[s] + lp
                cands.append(s + (t,))
        if stop_at is not None and len(score) >= stop_at:      # score holds the root and every proposed string
            break
        chosen = set(sorted(cands, key=lambda c: -score[c])[:k])
        frontier = [c for c in cands if c in chosen]
        out.append(frontier)
        if not frontier:
            break
    while len(out) < max(d, 1):
        out.append([])
    return out


def brute_greedy_accept(strings, target_fn):
    """strings: set of kept token strings (the tree without the root).

    Enumerates every root-to-node path; the accepted path is the longest one all of whose
    tokens equal the target arg max after the preceding string.  Returns (path string, bonus).
    """
    def amax(s):
        x = target_fn(s)
        return int(np.flatnonzero(x == x.max())[0])

    best = ()
    for s in sorted(strings, key=lambda c: (len(c), c)):
        if all(s[:j] in strings or j == 0 for j in range(len(s))) and \
           all(s[j] == amax(s[:j]) for j in range(len(s))):
            if len(s) > len(best):
                best = s
    return best, amax(best)


def brute_min_margin(draft_fn, V, TT, d, k):
    """Smallest score gap between a chosen and a passed-over candidate that were proposed by different
    token strings (different draft rows), over every cut of the build: the choice of the k strings to expand
    at levels 1..d-1 and the final cut to TT-1.  float64 scores on token strings; inf if no such pair."""
    def topk(string):
        x = draft_fn(string).astype(np.float64)
        lse = logsumexp(x)
        order = sorted(range(V), key=lambda t: (-x[t], t))[:k]
        return [(t, x[t] - lse) for t in order if x[t] > -np.inf]

    def gap(chosen, passed):
        g = [score[a] - score[b] for a in chosen for b in passed if a[:-1] != b[:-1]]
        return min(g) if g else np.inf

    score = {(): 0.0}
    margin = np.inf
    everyone = []
    frontier = [()]
    for level in range(1, d + 1):
        cands = [s + (t,) for s in frontier for t, _ in topk(s)]
        for s in frontier:
            for t, lp in topk(s):
                score[s + (t,)] = score[s] + lp
        everyone += cands
        if level == d or TT == 1:
            break
        ranked = sorted(cands, key=lambda c: -score[c])
        margin = min(margin, gap(ranked[:k], ranked[k:]))
        frontier = ranked[:k]
        if not frontier:
            break
    if TT > 1:
        ranked = sorted(everyone, key=lambda c: -score[c])
        margin = min(margin, gap(ranked[:TT - 1], ranked[TT - 1:]))
    return margin
