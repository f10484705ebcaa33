"""GPU parity of the input update (dt_commit) against the oracle: byte-exact caches, lengths and next roots."""
import numpy as np
import pytest

import dt_synth
from oracle import ref
from tests._cases import oracle_case

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _dev(a, dtype):
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def _host(t, dtype):
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def run_commit(case, dtype, Hkv, D, n_layers, head_major, slack, seed):
    import paper_2601_12212_amd as dt
    c = case.cfg
    B, TT_cap = c.B, max(p[0] for p in c.params)
    rng = np.random.default_rng(seed)
    mk = (lambda sh: rng.standard_normal(sh).astype(np.float32)) if dtype == "f32" else \
         (lambda sh: dt_synth.f32_to_bf16_bits(rng.standard_normal(sh).astype(np.float32)))
    L = [int(x) for x in c.prefix_len]
    cap = [L[b] + slack[b % len(slack)] for b in range(B)]
    tree_k = [mk((B, TT_cap, Hkv, D)) for _ in range(n_layers)]
    tree_v = [mk((B, TT_cap, Hkv, D)) for _ in range(n_layers)]
    shape = lambda b: (Hkv, max(cap[b], 1), D) if head_major else (max(cap[b], 1), Hkv, D)
    cache_k = [[mk(shape(b)) for b in range(B)] for _ in range(n_layers)]
    cache_v = [[mk(shape(b)) for b in range(B)] for _ in range(n_layers)]
    if head_major and len(set(cap)) > 1:
        pytest.skip("one head stride per call: head-major caches need equal capacities")
    d_tk = [_dev(a, dtype) for a in tree_k]; d_tv = [_dev(a, dtype) for a in tree_v]
    d_ck = [[_dev(a, dtype) for a in row] for row in cache_k]; d_cv = [[_dev(a, dtype) for a in row] for row in cache_v]
    i64 = dict(dtype=torch.int64, device="cuda")
    i32 = dict(dtype=torch.int32, device="cuda")
    ptrs = lambda rows: torch.tensor([[t.data_ptr() for t in row] for row in rows], **i64)
    n_nodes = torch.tensor([t["n_nodes"] for t in case.trees], **i32)
    path = torch.tensor(np.stack([a["path_nodes"] for a in case.accepts]), **i32)
    alen = torch.tensor([a["accept_len"] for a in case.accepts], **i32)
    otok = torch.tensor(np.stack([a["out_tokens"] for a in case.accepts]), **i32)
    new_len = torch.full((B,), -7, **i32)
    next_root = torch.full((B,), -7, **i32)
    st, sh = (D, max(cap[0], 1) * D) if head_major else (Hkv * D, D)
    dt.dt_commit(d_tk[0], Hkv, D, torch.tensor([t.data_ptr() for t in d_tk], **i64),
                 torch.tensor([t.data_ptr() for t in d_tv], **i64), ptrs(d_ck), ptrs(d_cv),
                 torch.tensor(L, **i32), torch.tensor(cap, **i32), st, sh, n_nodes, path, alen, otok, TT_cap,
                 new_len, next_root)
    torch.cuda.synchronize()
    for b in range(B):
        a = case.accepts[b]
        N = case.trees[b]["n_nodes"]
        want_len = None
        for l in range(n_layers):
            for tree, cache, dcache in ((tree_k, cache_k, d_ck), (tree_v, cache_v, d_cv)):
                want = cache[l][b].copy()
                if cap[b] >= 1:
                    want_len = ref.commit_rows(want, L[b], tree[l][b, :N], a["path_nodes"], a["accept_len"],
                                               head_major=head_major)
                else:
                    want_len = 0
                assert np.array_equal(_host(dcache[l][b], dtype), want), (b, l)
        assert int(new_len[b]) == want_len, (b, int(new_len[b]), want_len)
        assert int(next_root[b]) == int(a["out_tokens"][a["accept_len"]])


def _case(params, plen, seed=0):
    cfg = dt_synth.StepConfig("commit", "bf16", 8, 2, 128, 1500, params, plen, seed=seed)
    return oracle_case(0, cfg=cfg)


def test_commit_bf16_vector_path_several_layers():
    case = _case([(24, 4, 3), (60, 6, 4), (1, 1, 1), (40, 8, 2), (33, 3, 5)], [5, 130, 64, 0, 17])
    assert max(a["accept_len"] for a in case.accepts) >= 1
    run_commit(case, "bf16", Hkv=2, D=128, n_layers=3, head_major=False, slack=[9, 20, 1, 3, 0], seed=1)


def test_commit_head_major_cache_and_fp32():
    case = _case([(24, 4, 3), (60, 6, 4), (16, 5, 2)], [40, 40, 40])
    run_commit(case, "bf16", Hkv=4, D=64, n_layers=2, head_major=True, slack=[12], seed=2)
    run_commit(case, "f32", Hkv=2, D=64, n_layers=2, head_major=False, slack=[12, 2], seed=3)


def test_commit_scalar_path_for_odd_head_sizes():
    case = _case([(24, 4, 3), (50, 7, 3)], [3, 77])
    run_commit(case, "bf16", Hkv=3, D=20, n_layers=1, head_major=False, slack=[10], seed=4)   # 40-byte rows
    run_commit(case, "f32", Hkv=1, D=7, n_layers=2, head_major=False, slack=[10], seed=5)
