"""Pins of the oracle's tree attention (A5) against library softmax / einsum in float64 and
against special cases with a textbook meaning (ordinary decode, causal attention)."""
import numpy as np
import pytest
from scipy.special import softmax

import dt_synth
from oracle import ref


def rand_case(rng, N, Hq, Hkv, D, L, bf16=False):
    mk = lambda *s: rng.standard_normal(s).astype(np.float32)
    arrs = [mk(N, Hq, D), mk(N, Hkv, D), mk(N, Hkv, D), mk(L, Hkv, D), mk(L, Hkv, D)]
    if bf16:
        arrs = [dt_synth.f32_to_bf16_bits(a) for a in arrs]
    return arrs


def random_parents(rng, N):
    return np.array([-1] + [int(rng.integers(0, i)) for i in range(1, N)], np.int32)


def mask_from_parents(parents, TT_cap=128):
    N = len(parents)
    m = np.zeros((N, (TT_cap + 63) // 64), np.uint64)
    for i in range(N):
        j = i
        while j >= 0:
            m[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
            j = parents[j]
    return m


def dense_reference(q, kt, vt, kp, vp, parents, scale):
    """float64 attention with an explicit dense boolean mask, via einsum + scipy softmax."""
    q, kt, vt, kp, vp = [dt_synth.as_f32(a).astype(np.float64) for a in (q, kt, vt, kp, vp)]
    N, Hq, D = q.shape
    Hkv, L = kt.shape[1], kp.shape[0]
    G = Hq // Hkv
    K = np.concatenate([kp, kt], 0).repeat(G, axis=1)       # [L+N, Hq, D]
    Vv = np.concatenate([vp, vt], 0).repeat(G, axis=1)
    s = np.einsum("ihd,thd->iht", q, K) * scale
    vis = np.zeros((N, L + N), bool)
    vis[:, :L] = True
    for i in range(N):
        j = i
        while j >= 0:
            vis[i, L + j] = True
            j = parents[j]
    s = np.where(vis[:, None, :], s, -np.inf)
    p = softmax(s, axis=-1)
    return np.einsum("iht,thd->ihd", p, Vv)


@pytest.mark.parametrize("N,Hq,Hkv,D,L", [(8, 4, 4, 64, 128), (13, 8, 2, 32, 77), (5, 6, 3, 16, 0), (70, 2, 1, 8, 9)])
def test_matches_dense_mask_float64(N, Hq, Hkv, D, L):
    rng = np.random.default_rng(N * 100 + L)
    q, kt, vt, kp, vp = rand_case(rng, N, Hq, Hkv, D, L)
    parents = random_parents(rng, N)
    scale = 1.0 / np.sqrt(D)
    out = ref.tree_attention(q, kt, vt, kp, vp, mask_from_parents(parents), scale)
    want = dense_reference(q, kt, vt, kp, vp, parents, scale)
    assert np.abs(out - want).max() < 1e-6


def test_tt1_is_ordinary_decode_over_L_plus_1_keys():
    rng = np.random.default_rng(1)
    Hq, Hkv, D, L = 8, 2, 32, 50
    q, kt, vt, kp, vp = rand_case(rng, 1, Hq, Hkv, D, L)
    out = ref.tree_attention(q, kt, vt, kp, vp, mask_from_parents(np.array([-1])), 0.3)
    K = np.concatenate([kp, kt], 0).astype(np.float64)
    Vv = np.concatenate([vp, vt], 0).astype(np.float64)
    for h in range(Hq):
        g = h // (Hq // Hkv)
        p = softmax(0.3 * K[:, g] @ q[0, h].astype(np.float64))
        assert np.abs(out[0, h] - p @ Vv[:, g]).max() < 1e-6


def test_chain_tree_is_causal_attention_of_a_suffix():
    rng = np.random.default_rng(2)
    N, H, D, L = 6, 2, 16, 10
    q, kt, vt, kp, vp = rand_case(rng, N, H, H, D, L)
    parents = np.arange(-1, N - 1, dtype=np.int32)
    out = ref.tree_attention(q, kt, vt, kp, vp, mask_from_parents(parents), 0.25)
    K = np.concatenate([kp, kt], 0).astype(np.float64)
    Vv = np.concatenate([vp, vt], 0).astype(np.float64)
    for i in range(N):
        for h in range(H):
            p = softmax(0.25 * K[: L + i + 1, h] @ q[i, h].astype(np.float64))   # causal: keys 0..L+i
            assert np.abs(out[i, h] - p @ Vv[: L + i + 1, h]).max() < 1e-6


def test_equal_values_give_that_value_and_prefix_permutation_is_invisible():
    rng = np.random.default_rng(3)
    N, Hq, Hkv, D, L = 9, 4, 2, 8, 20
    q, kt, vt, kp, vp = rand_case(rng, N, Hq, Hkv, D, L)
    parents = random_parents(rng, N)
    m = mask_from_parents(parents)
    row = rng.standard_normal(D).astype(np.float32)
    out = ref.tree_attention(q, kt, np.broadcast_to(row, vt.shape).copy(), kp, np.broadcast_to(row, vp.shape).copy(), m, 0.5)
    assert np.abs(out - row).max() < 1e-6
    perm = rng.permutation(L)
    a = ref.tree_attention(q, kt, vt, kp, vp, m, 0.5)
    b = ref.tree_attention(q, kt, vt, kp[perm], vp[perm], m, 0.5)
    assert np.abs(a - b).max() < 1e-6


def test_sibling_keys_are_invisible():
    """Changing K/V of a node that is not an ancestor of i must not change output i."""
    rng = np.random.default_rng(4)
    N, H, D, L = 7, 2, 8, 5
    q, kt, vt, kp, vp = rand_case(rng, N, H, H, D, L)
    parents = np.array([-1, 0, 0, 1, 1, 2, 2], np.int32)
    m = mask_from_parents(parents)
    a = ref.tree_attention(q, kt, vt, kp, vp, m, 0.5)
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[2] += 5.0
    vt2[2] -= 3.0
    b = ref.tree_attention(q, kt2, vt2, kp, vp, m, 0.5)
    changed = [i for i in range(N) if np.abs(a[i] - b[i]).max() > 0]
    assert changed == [2, 5, 6]            # node 2 and its descendants only


def test_bf16_inputs_upcast_exactly_and_output_on_bf16_grid_and_samples():
    rng = np.random.default_rng(5)
    N, Hq, Hkv, D, L = 10, 8, 2, 128, 40
    q, kt, vt, kp, vp = rand_case(rng, N, Hq, Hkv, D, L, bf16=True)
    parents = random_parents(rng, N)
    m = mask_from_parents(parents)
    scale = 1.0 / np.sqrt(D)
    out = ref.tree_attention(q, kt, vt, kp, vp, m, scale)
    want = dense_reference(q, kt, vt, kp, vp, parents, scale)
    assert np.abs(out - want).max() < 2.0 ** -8 * np.abs(want).max() + 1e-6   # half a bf16 ulp
    assert np.array_equal(dt_synth.bf16_bits_to_f32(dt_synth.f32_to_bf16_bits(out)), out)
    samples = np.array([[0, 0], [9, 7], [4, 3]], np.int32)
    sub = ref.tree_attention(q, kt, vt, kp, vp, m, scale, samples=samples)
    for r, (i, h) in enumerate(samples):
        assert np.array_equal(sub[r], out[i, h])
