"""ctypes front end of the CPU oracle (oracle/dt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The product package never imports it.

Arrays are numpy: float32 for fp32 data, uint16 (raw bf16 bit patterns) for bf16 data.
Every function handles ONE sequence; callers loop over a batch.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dt_oracle.c")
_LIB = os.path.join(_HERE, "libdt_oracle.so")

TT_MAX, D_MAX, K_MAX = 128, 8, 32
F32, BF16 = 0, 1
GREEDY, STOCHASTIC, SAMPLED = 0, 1, 2


def build(force=False):
    """Compile the oracle with gcc (plain C, -O2, OpenMP over independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ref_uniform.restype = C.c_float
        _lib.ref_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
    return _lib


def _dt(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle arrays are float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _check(rc, what):
    if rc < 0:
        raise RuntimeError("%s failed with code %d" % (what, rc))
    return rc


def topk_rows(logits, k):
    """A1: per-row top-k (logit desc, id asc) and log-sum-exp.  logits [R, V]."""
    logits = np.ascontiguousarray(logits)
    R, V = logits.shape
    val = np.empty((R, k), np.float32)
    idx = np.empty((R, k), np.int32)
    lse = np.empty(R, np.float32)
    _check(lib().ref_topk_rows(_p(logits), _dt(logits), C.c_int64(R), V, C.c_int64(V), k,
                               _p(val), _p(idx), _p(lse)), "ref_topk_rows")
    return val, idx, lse


def build_tree(rows, TT, d, k, root_token=0, TT_cap=TT_MAX, with_levels=False, early_stop=False):
    """A1-A4 for one sequence.  rows [>= 1+(d-1)k, V].  Returns a dict of node arrays.

    with_levels: also "levels", a list indexed by level l = 1..d-1 of dicts (tokens, parent_slot, rows, mask)
    describing the nodes expanded at that level -- what a draft model between the levels is handed.
    early_stop: leave the expansion loop once the root plus the candidates proposed so far number TT or more
    (the token-count exit of Algorithm 2's expansion loop)."""
    rows = np.ascontiguousarray(rows)
    R, V = rows.shape
    W = (TT_cap + 63) // 64
    n = C.c_int32(0)
    tokens = np.full(TT_cap, -1, np.int32)
    parents = np.full(TT_cap, -1, np.int32)
    depth = np.zeros(TT_cap, np.int32)
    score = np.zeros(TT_cap, np.float32)
    logp = np.zeros(TT_cap, np.float32)
    src_row = np.full(TT_cap, -1, np.int32)
    mask = np.zeros((TT_cap, W), np.uint64)
    margin = C.c_float(0)
    ecnt = np.zeros(D_MAX, np.int32) if with_levels else None
    etok = np.full((D_MAX, K_MAX), -1, np.int32) if with_levels else None
    epar = np.full((D_MAX, K_MAX), -1, np.int32) if with_levels else None
    emask = np.zeros((D_MAX, K_MAX, 4), np.uint64) if with_levels else None
    _check(lib().ref_build_tree(_p(rows), _dt(rows), V, C.c_int64(V), R, TT, d, k, root_token, TT_cap,
                                C.byref(n), _p(tokens), _p(parents), _p(depth), _p(score), _p(logp),
                                _p(src_row), _p(mask), C.byref(margin), _p(ecnt), _p(etok), _p(epar), _p(emask),
                                1 if early_stop else 0),
           "ref_build_tree")
    N = n.value
    out = dict(n_nodes=N, tokens=tokens[:N], parents=parents[:N], depth=depth[:N], score=score[:N],
               logp=logp[:N], src_row=src_row[:N], anc_mask=mask[:N], min_margin=margin.value)
    if with_levels:
        out["levels"] = [None] + [dict(tokens=etok[l, :ecnt[l]], parent_slot=epar[l, :ecnt[l]],
                                       rows=1 + (l - 1) * k + np.arange(ecnt[l]), mask=emask[l, :ecnt[l]])
                                  for l in range(1, max(d, 1))]
    return out


def tree_attention(q, k_tree, v_tree, k_prefix, v_prefix, anc_mask, scale, samples=None, TT_cap=TT_MAX):
    """A5 for one sequence.  q [N,Hq,D]; k_tree/v_tree [N,Hkv,D]; k_prefix/v_prefix [L,Hkv,D].

    samples: optional int array [n,2] of (node, head) pairs -> output [n, D]; else [N,Hq,D].
    Output float32 (on the bf16 grid for bf16 inputs).
    """
    q = np.ascontiguousarray(q)
    k_tree, v_tree = np.ascontiguousarray(k_tree), np.ascontiguousarray(v_tree)
    k_prefix, v_prefix = np.ascontiguousarray(k_prefix), np.ascontiguousarray(v_prefix)
    N, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    L = k_prefix.shape[0]
    anc_mask = np.ascontiguousarray(anc_mask, np.uint64)
    assert anc_mask.shape == (N, (TT_cap + 63) // 64)
    if samples is not None:
        samples = np.asarray(samples, np.int32).reshape(-1, 2)
        sn, sh = np.ascontiguousarray(samples[:, 0]), np.ascontiguousarray(samples[:, 1])
        out = np.empty((len(sn), D), np.float32)
        ns = len(sn)
    else:
        sn = sh = None
        out = np.empty((N, Hq, D), np.float32)
        ns = 0
    _check(lib().ref_tree_attention(_dt(q), Hq, Hkv, D, C.c_float(scale), _p(q), _p(k_tree), _p(v_tree), N,
                                    _p(k_prefix), _p(v_prefix), L, C.c_int64(Hkv * D), C.c_int64(D),
                                    _p(anc_mask), TT_cap, _p(sn), _p(sh), ns, _p(out)), "ref_tree_attention")
    return out


def accept(mode, target, tokens, parents, depth, logp=None, temperature=1.0, d_cap=D_MAX,
           seed=0, step=0, seq=0):
    """A6-A7 for one sequence.  target [N, V] (row i = target logits after node i)."""
    target = np.ascontiguousarray(target)
    N, V = target.shape
    tokens = np.ascontiguousarray(tokens, np.int32)
    parents = np.ascontiguousarray(parents, np.int32)
    depth = np.ascontiguousarray(depth, np.int32)
    logp = None if logp is None else np.ascontiguousarray(logp, np.float32)
    alen, best = C.c_int32(0), C.c_int32(0)
    path = np.empty(d_cap + 1, np.int32)
    out_tok = np.empty(d_cap + 1, np.int32)
    amax = np.empty(N, np.int32)
    accepted = np.empty(N, np.uint8)
    margin = C.c_float(0)
    nmargin = np.full(N, np.inf, np.float32)
    _check(lib().ref_accept(mode, C.c_float(temperature), _p(target), _dt(target), V, C.c_int64(V), N,
                            _p(tokens), _p(parents), _p(depth), _p(logp), d_cap,
                            C.c_uint64(seed), C.c_uint64(step), C.c_uint32(seq),
                            C.byref(alen), C.byref(best), _p(path), _p(out_tok), _p(amax), _p(accepted),
                            C.byref(margin), _p(nmargin)), "ref_accept")
    return dict(accept_len=alen.value, best_node=best.value, path_nodes=path, out_tokens=out_tok,
                node_argmax=amax, accepted=accepted.astype(bool), min_margin=margin.value, node_margin=nmargin)


def commit_rows(cache, L, tree, path_nodes, accept_len, head_major=False):
    """Input update for one sequence and one cache tensor, in place.

    cache: [cap, Hkv, D] (or [Hkv, cap, D] with head_major), rows 0..L-1 valid; tree: [N, Hkv, D].
    Returns the new length."""
    assert cache.flags.c_contiguous and cache.dtype == tree.dtype
    tree = np.ascontiguousarray(tree)
    N, Hkv, D = tree.shape
    if head_major:
        assert cache.shape[0] == Hkv and cache.shape[2] == D
        cap, st, sh = cache.shape[1], D, cache.shape[1] * D
    else:
        assert cache.shape[1] == Hkv and cache.shape[2] == D
        cap, st, sh = cache.shape[0], Hkv * D, D
    path = np.ascontiguousarray(path_nodes, np.int32)
    new_len = C.c_int64(0)
    _check(lib().ref_commit_rows(_p(cache), _dt(cache), C.c_int64(cap), C.c_int64(L), C.c_int64(st), C.c_int64(sh),
                                 Hkv, D, _p(tree), N, _p(path), int(accept_len), C.byref(new_len)), "ref_commit_rows")
    return new_len.value


def action_table():
    """Appendix A action table after the TT <= k^(d-1) filter: int32 [n, 3] rows (TT, d, k)."""
    out = np.zeros((256, 3), np.int32)
    n = lib().ref_action_table(_p(out), 256)
    return out[:n].copy()


def policy_logits(feat, W1, b1, W2, b2, W3, b3):
    """MLP logits in float64.  feat [F] float32; W1 [F,H], W2 [H,H], W3 [H,A] float32 ([in][out])."""
    f32 = lambda a: np.ascontiguousarray(a, np.float32)
    feat, W1, b1, W2, b2, W3, b3 = map(f32, (feat, W1, b1, W2, b2, W3, b3))
    F, H = W1.shape
    A = W3.shape[1]
    assert feat.shape == (F,) and W2.shape == (H, H) and W3.shape[0] == H
    out = np.zeros(A, np.float64)
    _check(lib().ref_policy_logits(_p(feat), F, H, A, _p(W1), _p(b1), _p(W2), _p(b2), _p(W3), _p(b3), _p(out)),
           "ref_policy_logits")
    return out


def policy_step(cache_step, cached_action, logits, N, mode=0, seed=0, step=0, seq=0):
    """One decision point of Algorithm 1.  Returns dict(action, cache_step, cached_action, queried, margin)."""
    cs, ca, q = C.c_int(cache_step), C.c_int(cached_action), C.c_int(0)
    margin = C.c_double(np.inf)
    lg = None if logits is None else np.ascontiguousarray(logits, np.float64)
    act = _check(lib().ref_policy_step(C.byref(cs), C.byref(ca), _p(lg), 1 if lg is None else len(lg), N, mode,
                                       C.c_uint64(seed), C.c_uint64(step), C.c_uint32(seq), C.byref(q),
                                       C.byref(margin)), "ref_policy_step")
    return dict(action=act, cache_step=cs.value, cached_action=ca.value, queried=bool(q.value), margin=margin.value)


def reward_step(cache_step, tokens, elapsed, acc):
    """Reward bookkeeping of one decoding step.  acc: dict(sum, steps), updated in place.
    Returns (done, avg): avg is the interval's average reward when the interval ended with this step."""
    s, n = C.c_double(acc["sum"]), C.c_int(acc["steps"])
    avg, done = C.c_double(float("nan")), C.c_int(0)
    _check(lib().ref_reward_step(int(cache_step), C.c_double(tokens), C.c_double(elapsed), C.byref(s), C.byref(n),
                                 C.byref(avg), C.byref(done)), "ref_reward_step")
    acc["sum"], acc["steps"] = s.value, n.value
    return bool(done.value), avg.value


def philox4x32(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().ref_philox4x32(c, k, o)
    return tuple(int(x) for x in o)


def uniform(seed, step, seq, node):
    return float(lib().ref_uniform(seed, step, seq, node))
