"""Oracle side of a parity case: trees, targets and acceptance of a StepConfig, with the margin guard.

A case whose oracle decisions hinge on a score gap below the guard (a cross-row cut that a
last-bit difference in a log-sum-exp could flip, or a uniform within 1e-5 of its acceptance
probability) is deterministically regenerated with seed+1; the replacement is printed.
"""
import numpy as np

import dt_synth
from oracle import ref

TREE_MARGIN = 1e-4
ACCEPT_MARGIN = 1e-5


class OracleCase:
    pass


def oracle_case(ci, seed=0, cfg=None, philox_step=0, max_bumps=20, early_stop=False):
    for bump in range(max_bumps):
        c = dt_synth.config(ci, seed + bump) if cfg is None else cfg
        if cfg is not None:
            c.seed = seed + bump
        case = OracleCase()
        case.cfg = c
        case.early_stop = early_stop
        case.drafts = [dt_synth.draft_rows(c, b) for b in range(c.B)]
        case.trees = []
        for b in range(c.B):
            TT, d, k = c.params[b]
            case.trees.append(ref.build_tree(case.drafts[b], TT, d, k, dt_synth.root_token(c, b), early_stop=early_stop))
        margin = min(t["min_margin"] for t in case.trees)
        if margin < TREE_MARGIN:
            print("margin guard: %s seed %d tree margin %.3g -> seed %d" % (c.name, c.seed, margin, c.seed + 1))
            continue
        case.targets = [dt_synth.target_rows(c, b, case.trees[b]["src_row"], case.drafts[b]) for b in range(c.B)]
        case.accepts = []
        for b in range(c.B):
            t = case.trees[b]
            case.accepts.append(ref.accept(c.mode, case.targets[b], t["tokens"], t["parents"], t["depth"],
                                           logp=t["logp"], temperature=c.temperature, seed=c.philox_seed,
                                           step=philox_step, seq=b))
        if c.mode != dt_synth.GREEDY:
            am = min(a["min_margin"] for a in case.accepts)
            if am < ACCEPT_MARGIN:
                print("margin guard: %s seed %d accept margin %.3g -> seed %d" % (c.name, c.seed, am, c.seed + 1))
                continue
        return case
    raise RuntimeError("margin guard: no acceptable seed found")


def make_step(case, TT_cap=None, kv_head_major=False):
    """Device buffers of the case with draft rows, Q/K/V and (oracle-tree-derived) targets uploaded."""
    import torch
    from paper_2601_12212_amd.step import Step
    c = case.cfg
    st = Step(c.params, c.prefix_len, c.Hq, c.Hkv, c.D, c.V,
              dtype=torch.float32 if c.dtype == "f32" else torch.bfloat16, mode=c.mode,
              temperature=c.temperature, TT_cap=TT_cap, philox_seed=c.philox_seed,
              tree_flags=1 if getattr(case, "early_stop", False) else 0, kv_head_major=kv_head_major)
    dt_synth.fill_draft_and_qkv(st, c, case.drafts)
    for b in range(c.B):
        st.set_target(b, case.targets[b])
    return st


def assert_tree_equal(got, want, tag=""):
    assert got["n_nodes"] == want["n_nodes"], tag
    for key in ("tokens", "parents", "depth", "src_row"):
        assert np.array_equal(got[key], want[key]), (tag, key)
    assert np.array_equal(got["anc_mask"], want["anc_mask"]), (tag, "anc_mask")
    # cumulative fp32 log-probabilities: a few ulp of the score per level plus the lse rounding
    tol = 2e-5 + 4e-6 * np.abs(want["score"])
    assert (np.abs(got["score"] - want["score"]) <= tol).all(), (tag, "score", np.abs(got["score"] - want["score"]).max())
    assert (np.abs(got["logp"] - want["logp"]) <= 1e-5 + 2e-6 * np.abs(want["logp"])).all(), (tag, "logp")


def assert_accept_equal(got, want, tag=""):
    assert got["accept_len"] == want["accept_len"], tag
    assert got["best_node"] == want["best_node"], tag
    assert np.array_equal(got["path_nodes"], want["path_nodes"]), tag
    assert np.array_equal(got["out_tokens"], want["out_tokens"]), tag
    # per-node draws of the target-sampled mode are compared where their own margin allows it
    sure = want["node_margin"] >= ACCEPT_MARGIN if "node_margin" in want else np.ones(len(want["node_argmax"]), bool)
    assert np.array_equal(got["node_argmax"][sure], want["node_argmax"][sure]), tag
