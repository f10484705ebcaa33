"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, sizes its workspace, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

import paper_2601_12212_amd as dt
from paper_2601_12212_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dt_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = dt.load_library()
    names = declared_symbols()
    assert {"dt_build_tree", "dt_tree_attention", "dt_accept", "dt_topk_rows", "dt_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings_and_limits_match_header():
    text = open(os.path.join(ROOT, "include", "dt.h")).read()
    for name, val in [("DT_TT_MAX", binding.DT_TT_MAX), ("DT_D_MAX", binding.DT_D_MAX), ("DT_K_MAX", binding.DT_K_MAX)]:
        assert int(re.search(r"#define %s (\d+)" % name, text).group(1)) == val
    assert dt.dt_status_string(0) == "ok"
    assert "workspace" in dt.dt_status_string(-3)
    # the caps are the maxima of the action space printed in the paper's appendix
    gold = dict(l.split(None, 1) for l in open(os.path.join(ROOT, "tests", "golden", "action_space.txt"))
                if not l.startswith("#"))
    assert max(map(int, gold["TT"].split())) == binding.DT_TT_MAX
    assert max(map(int, gold["d"].split())) == binding.DT_D_MAX
    assert max(map(int, gold["k"].split())) == binding.DT_K_MAX
    assert len(gold["TT"].split()) * len(gold["d"].split()) * len(gold["k"].split()) == int(gold["combinations"])


def test_workspace_bytes():
    small = dt.dt_workspace_bytes(1, 5, 1024, 8, 4, 64)
    big = dt.dt_workspace_bytes(16, 16 * 85, 128256, 96, 32, 128)
    assert 0 < small < big < (1 << 31)
    with pytest.raises(dt.DtError) as e:
        dt.dt_workspace_bytes(1, 5, 1024, 129, 4, 64)
    assert e.value.status == -2
    with pytest.raises(dt.DtError):
        dt.dt_workspace_bytes(1, 5, 600000, 8, 4, 64)          # vocabulary beyond the row-kernel limit


def test_bad_arguments_are_rejected_before_any_launch():
    lib = dt.load_library()
    one = C.c_void_p(256)       # non-null, aligned, never dereferenced on the host
    ws = C.c_void_p(4096)
    # null pointers
    assert lib.dt_topk_rows(None, None, 1, 4, 1024, 1024, 4, one, one, one, ws, 1 << 20) == -1
    # k out of range / above V
    assert lib.dt_topk_rows(None, one, 1, 4, 1024, 1024, 0, one, one, one, ws, 1 << 20) == -2
    assert lib.dt_topk_rows(None, one, 1, 4, 1024, 1024, 33, one, one, one, ws, 1 << 20) == -2
    assert lib.dt_topk_rows(None, one, 1, 4, 8, 8, 9, one, one, one, ws, 1 << 20) == -2
    # row stride shorter than the row, bad dtype
    assert lib.dt_topk_rows(None, one, 1, 4, 1024, 1000, 4, one, one, one, ws, 1 << 20) == -1
    assert lib.dt_topk_rows(None, one, 7, 4, 1024, 1024, 4, one, one, one, ws, 1 << 20) == -1
    # workspace missing / too small / misaligned
    assert lib.dt_topk_rows(None, one, 1, 4, 1024, 1024, 4, one, one, one, None, 0) == -3
    assert lib.dt_topk_rows(None, one, 1, 4, 1024, 1024, 4, one, one, one, ws, 16) == -3
    assert lib.dt_topk_rows(None, one, 1, 4, 1024, 1024, 4, one, one, one, C.c_void_p(4100), 1 << 20) == -3
    # build_tree: TT_cap over the limit, null params, too few rows, small workspace
    args = lambda **kw: [kw.get("stream"), kw.get("batch", 1), kw.get("params", one), one, 1, 1024, 1024, one,
                         kw.get("rows", 5), one, kw.get("TT_cap", 8)] + [one] * 8 + [ws, kw.get("wsb", 1 << 24), kw.get("flags", 0)]
    assert lib.dt_build_tree(*args(TT_cap=129)) == -2
    assert lib.dt_build_tree(*args(TT_cap=0)) == -2
    assert lib.dt_build_tree(*args(params=None)) == -1
    assert lib.dt_build_tree(*args(batch=4, rows=3)) == -1
    assert lib.dt_build_tree(*args(wsb=64)) == -3
    assert lib.dt_build_tree(*args(batch=0)) == 0
    assert lib.dt_build_tree(*args(flags=2)) == -1          # an unknown flag bit
    # attention: Hq not a multiple of Hkv, head dim over the limit, non-positive scale
    att = lambda **kw: [None, 1, 1, kw.get("Hq", 32), kw.get("Hkv", 8), kw.get("D", 128), kw.get("scale", 0.1),
                        one, one, one, one, one, one, one, 1024, 1024, 128, one, 60, one, ws, 1 << 24]
    assert lib.dt_tree_attention(*att(Hq=30)) == -1
    assert lib.dt_tree_attention(*att(D=256)) == -2
    assert lib.dt_tree_attention(*att(scale=0.0)) == -1
    # accept: bad mode, stochastic without logp or with T <= 0
    acc = lambda **kw: [None, 1, kw.get("mode", 0), kw.get("T", 1.0), one, 1, 1024, 1024, one, one, one, one,
                        kw.get("logp", one), one, 8, 0, 0, one, one, one, one, None, ws, kw.get("wsb", 1 << 24)]
    assert lib.dt_accept(*acc(mode=3)) == -1
    assert lib.dt_accept(*acc(mode=2, T=0.0)) == -1
    assert lib.dt_accept(*acc(mode=1, logp=None)) == -1
    assert lib.dt_accept(*acc(mode=1, T=0.0)) == -1
    assert lib.dt_accept(*acc(wsb=8)) == -3
    # level-at-a-time build: level / rows-per-sequence out of range, misaligned state, null outputs
    lev = lambda **kw: [None, kw.get("batch", 1), kw.get("level", 1), one, one, 1, 1024, 1024, kw.get("rps", 8), None, 60,
                        kw.get("state", ws), kw.get("nexp", one), one, one, one, one, one, ws, kw.get("wsb", 1 << 24),
                        kw.get("flags", 0)]
    assert lib.dt_expand_level(*lev(level=0)) == -1
    assert lib.dt_expand_level(*lev(level=9)) == -1
    assert lib.dt_expand_level(*lev(rps=33)) == -1
    assert lib.dt_expand_level(*lev(state=C.c_void_p(4100))) == -1
    assert lib.dt_expand_level(*lev(nexp=None)) == -1
    assert lib.dt_expand_level(*lev(wsb=16)) == -3
    assert lib.dt_expand_level(*lev(batch=0)) == 0
    assert lib.dt_expand_level(*lev(flags=4)) == -1
    fin = lambda **kw: [None, kw.get("batch", 1), one, 1024, one, kw.get("TT_cap", 60), kw.get("state", ws)] + [one] * 8 + \
                       [kw.get("flags", 0)]
    assert lib.dt_finish_tree(*fin(TT_cap=0)) == -2
    assert lib.dt_finish_tree(*fin(state=None)) == -1
    assert lib.dt_finish_tree(*fin(batch=0)) == 0
    assert lib.dt_finish_tree(*fin(flags=3)) == -1
    nbytes = C.c_size_t(0)
    assert lib.dt_level_state_bytes(3, C.byref(nbytes)) == 0 and nbytes.value >= 3 * 225 * (32 * 8 + 4)
    # policy: hidden size / action count over the limits, bad interval, small workspace
    pol = lambda **kw: [None, kw.get("batch", 1), 1, one, 12288, 12288, kw.get("H", 128), kw.get("A", 177)] + [one] * 7 + \
                       [kw.get("N", 30), kw.get("sample", 0), 0, 0, one, one, one, None, None, None, ws, kw.get("wsb", 1 << 24)]
    assert lib.dt_policy_step(*pol(H=100)) == -2
    assert lib.dt_policy_step(*pol(A=300)) == -2
    assert lib.dt_policy_step(*pol(N=0)) == -1
    assert lib.dt_policy_step(*pol(sample=2)) == -1
    assert lib.dt_policy_step(*pol(wsb=64)) == -3
    assert lib.dt_policy_step(*pol(batch=0)) == 0
    # commit: null pointers, new length aliasing the old one, TT_cap over the limit, nothing to do
    other = C.c_void_p(512)
    com = lambda **kw: [None, kw.get("batch", 1), kw.get("layers", 2), 1, 8, 128, one, one, kw.get("kp", one), one, one,
                        one, 1024, 128, one, one, one, one, kw.get("TT_cap", 60), kw.get("new", other), None]
    assert lib.dt_commit(*com(kp=None)) == -1
    assert lib.dt_commit(*com(new=one)) == -1
    assert lib.dt_commit(*com(TT_cap=129)) == -2
    assert lib.dt_commit(*com(batch=0)) == 0
    assert lib.dt_commit(*com(layers=0)) == 0
    # reward bookkeeping: null accumulators, a bonus count that is not 0/1, no positive time
    rew = lambda **kw: [None, kw.get("batch", 2), one, kw.get("bonus", 1), kw.get("secs", 0.01), kw.get("per_seq"), one,
                        kw.get("acc", one), one, one, one]
    assert lib.dt_reward_step(*rew(acc=None)) == -1
    assert lib.dt_reward_step(*rew(bonus=2)) == -1
    assert lib.dt_reward_step(*rew(secs=0.0)) == -1
    assert lib.dt_reward_step(*rew(batch=0)) == 0


def test_launch_grid_limits_are_checked_on_the_host():
    """Rows ride in the y and z dimensions of the streaming grids and in x of the selection grid: row counts
    beyond 65,535 are ordinary, and a call with more than 2^31 - 1 rows returns DT_ERR_LIMIT before the
    workspace is even looked at.  Sequences ride in the z dimension of the attention grid (with up to 8 key
    splits)."""
    lib = dt.load_library()
    one, ws = C.c_void_p(256), C.c_void_p(4096)
    # 70,000 rows: past the limit check (the tiny workspace is what is refused)
    assert lib.dt_topk_rows(None, one, 1, 70000, 1024, 1024, 4, one, one, one, ws, 16) == -3
    assert lib.dt_topk_rows(None, one, 1, 1 << 31, 1024, 1024, 4, one, one, one, ws, 1 << 40) == -2
    assert lib.dt_topk_rows(None, one, 1, (1 << 31) - 1, 1024, 1024, 4, one, one, one, ws, 16) == -3
    acc = lambda batch, TT_cap, wsb: [None, batch, 0, 1.0, one, 1, 1024, 1024, one, one, one, one, one, one, TT_cap, 0, 0,
                                       one, one, one, one, None, ws, wsb]
    assert lib.dt_accept(*acc(512, 128, 16)) == -3              # 65,536 rows: fine
    assert lib.dt_accept(*acc(1 << 24, 128, 1 << 40)) == -2     # 2^31 rows
    bt = lambda rows: [None, 1, one, one, 1, 1024, 1024, one, rows, one, 8] + [one] * 8 + [ws, 16, 0]
    assert lib.dt_build_tree(*bt(70000)) == -3
    assert lib.dt_build_tree(*bt(1 << 31)) == -2
    att = lambda batch, Hq: [None, batch, 1, Hq, 8, 128, 0.1, one, one, one, one, one, one, one, 1024, 1024, 128, one, 60,
                             one, ws, 1 << 24]
    assert lib.dt_tree_attention(*att(8192, 32)) == -2
    assert lib.dt_tree_attention(*att(1, 8 * 8192)) == -2


def test_action_table_matches_the_oracle_and_the_golden_sets():
    from oracle import ref
    table = dt.dt_action_table()
    assert table == [tuple(int(v) for v in r) for r in ref.action_table()]
    assert len(table) == 177 and dt.dt_policy_workspace_bytes(4, 12288, 128) >= 192 * 4 * 128 * 4


def test_binding_argument_lists_have_the_length_of_the_header_prototypes():
    """A parameter added to a prototype and forgotten in the ctypes argument list would shift every later
    argument silently: the binding's argtypes of each function it declares must be as long as the header's
    parameter list."""
    text = open(os.path.join(ROOT, "include", "dt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    protos = re.findall(r"\b(?:int|const char \*|void)\s*(dt_[a-z_0-9]+)\s*\(([^;{]*?)\)\s*;", text, flags=re.S)
    assert len(protos) >= 20
    lib = dt.load_library()
    checked = 0
    for name, args in protos:
        args = args.strip()
        want = 0 if args in ("", "void") else len(args.split(","))
        fn = getattr(lib, name)
        if fn.argtypes is None:
            assert want == 0 or name.startswith("dt_profile") or name.endswith("_string") or name == "dt_last_hip_error", name
            continue
        assert len(fn.argtypes) == want, (name, len(fn.argtypes), want)
        checked += 1
    assert checked >= 12
