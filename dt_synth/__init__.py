"""Seeded synthetic inputs for one draft-tree speculative step.

This module is shared by the tests, the oracle-timing leg and the GPU benchmark.  It
holds NO arithmetic of the method (no top-k, no softmax, no tree logic): only shapes,
random draws and dtype rounding.  Arrays are numpy; bf16 data is carried as uint16 bit
patterns (numpy has no bf16).

The shapes stand in for the workloads the paper evaluates on (LLaMA-3.1-8B, Vicuna-13B,
LLaMA-3.3-70B on chat/code/math/summarisation prompts): head counts, head dim and vocab
size of those models, contexts of 128..8192 tokens, (TT, d, k) inside the ranges of the
paper's action space.  No prompt, weight or dataset item is reproduced.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

GREEDY, STOCHASTIC, SAMPLED = 0, 1, 2


def f32_to_bf16_bits(x):
    """float32 -> bf16 bit pattern (uint16), round to nearest even.  Finite inputs."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def as_f32(a):
    """Exact float32 view of a config-dtype array (float32 or bf16 bits)."""
    return a if a.dtype == np.float32 else bf16_bits_to_f32(a)


@dataclass
class StepConfig:
    name: str
    dtype: str                      # "f32" | "bf16"
    Hq: int
    Hkv: int
    D: int
    V: int
    params: List[Tuple[int, int, int]]   # per sequence (TT, d, k)
    prefix_len: List[int]
    mode: int = GREEDY
    temperature: float = 1.0
    sigma_draft: float = 3.0
    coupled_target: bool = True     # target row = draft row of the node + N(0,1)
    seed: int = 0
    philox_seed: int = 0x5EED
    extra: dict = field(default_factory=dict)

    @property
    def B(self):
        return len(self.params)

    def n_rows(self, b):
        TT, d, k = self.params[b]
        return 1 + (d - 1) * k

    def row_off(self):
        off = [0]
        for b in range(self.B):
            off.append(off[-1] + self.n_rows(b))
        return np.asarray(off, np.int64)

    def node_off(self):
        off = [0]
        for b in range(self.B):
            off.append(off[-1] + self.params[b][0])
        return np.asarray(off, np.int64)

    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2


def config(i, seed=0):
    """The five benchmark configurations (1-based, as numbered in the design notes)."""
    if i == 1:
        return StepConfig("cfg1_tiny_fp32", "f32", 4, 4, 64, 1024, [(8, 3, 2)], [128], sigma_draft=2.0,
                          coupled_target=False, seed=seed)
    if i == 2:
        return StepConfig("cfg2_llama3_8b_tt60", "bf16", 32, 8, 128, 128256, [(60, 6, 10)], [1024], seed=seed)
    if i == 3:
        return StepConfig("cfg3_vicuna_13b_tt64", "bf16", 40, 40, 128, 32000, [(64, 7, 8)], [2048], seed=seed)
    if i == 4:
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 4, 0xC0F])))
        params, plen = [], []
        for _ in range(16):
            TT = int(rng.choice([32, 48, 64, 80, 96]))
            d = int(rng.integers(4, 9))
            k = int(rng.integers(4, 13))
            params.append((TT, d, k))
            plen.append(int(rng.integers(256, 4097)))
        return StepConfig("cfg4_llama3_8b_b16_ragged", "bf16", 32, 8, 128, 128256, params, plen, seed=seed)
    if i == 5:
        return StepConfig("cfg5_llama3_70b_b4_stochastic", "bf16", 64, 8, 128, 128256, [(96, 8, 12)] * 4,
                          [8192] * 4, mode=STOCHASTIC, temperature=1.0, seed=seed)
    raise ValueError("config index 1..5")


def _rng(cfg, b, stream):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, b, stream, 0xD7])))


def _round(cfg, x):
    x = np.ascontiguousarray(x, np.float32)
    return x if cfg.dtype == "f32" else f32_to_bf16_bits(x)


def draft_rows(cfg, b):
    """Draft logits of sequence b: [1+(d-1)k, V], rows ~ N(0, sigma_draft) in the config dtype."""
    rng = _rng(cfg, b, 1)
    x = rng.standard_normal((cfg.n_rows(b), cfg.V), dtype=np.float32) * np.float32(cfg.sigma_draft)
    return _round(cfg, x)


def target_rows(cfg, b, src_row, draft=None):
    """Target logits [N, V] of sequence b given the tree's src_row (length N).

    coupled: row i = draft row src_row[i] + N(0,1); nodes never handed a draft row
    (src_row < 0) get a fresh N(0, sigma_draft) row + N(0,1).  uncoupled: N(0, sigma_draft).
    """
    src_row = np.asarray(src_row)
    N = len(src_row)
    rng = _rng(cfg, b, 2)
    sig = np.float32(cfg.sigma_draft)
    if not cfg.coupled_target:
        return _round(cfg, rng.standard_normal((N, cfg.V), dtype=np.float32) * sig)
    if draft is None:
        draft = draft_rows(cfg, b)
    out = np.empty((N, cfg.V), np.float32)
    for i in range(N):
        fresh = rng.standard_normal(cfg.V, dtype=np.float32) * sig
        noise = rng.standard_normal(cfg.V, dtype=np.float32)
        base = as_f32(draft[src_row[i]]) if src_row[i] >= 0 else fresh
        out[i] = base + noise
    return _round(cfg, out)


def qkv(cfg, b):
    """q [TT,Hq,D], k_tree/v_tree [TT,Hkv,D], k_prefix/v_prefix [L,Hkv,D], all ~ N(0,1).

    Only the first n_nodes rows of the tree-sized arrays are used by a step.
    """
    TT = cfg.params[b][0]
    L = cfg.prefix_len[b]
    rng = _rng(cfg, b, 3)
    q = _round(cfg, rng.standard_normal((TT, cfg.Hq, cfg.D), dtype=np.float32))
    kt = _round(cfg, rng.standard_normal((TT, cfg.Hkv, cfg.D), dtype=np.float32))
    vt = _round(cfg, rng.standard_normal((TT, cfg.Hkv, cfg.D), dtype=np.float32))
    kp = _round(cfg, rng.standard_normal((L, cfg.Hkv, cfg.D), dtype=np.float32))
    vp = _round(cfg, rng.standard_normal((L, cfg.Hkv, cfg.D), dtype=np.float32))
    return q, kt, vt, kp, vp


def root_token(cfg, b):
    return int(_rng(cfg, b, 4).integers(0, cfg.V))


# ---- filling a device-side step object (anything with set_draft/set_root_token/set_qkv/set_target)

def fill_draft_and_qkv(step, cfg, drafts=None):
    """Upload draft rows, root tokens and Q/K/V of every sequence.  Returns the draft rows."""
    drafts = drafts or [draft_rows(cfg, b) for b in range(cfg.B)]
    for b in range(cfg.B):
        step.set_draft(b, drafts[b])
        step.set_root_token(b, root_token(cfg, b))
        step.set_qkv(b, *qkv(cfg, b))
    return drafts


def fill_target(step, cfg, src_rows, drafts=None):
    """Upload target rows built from each sequence's src_row array.  Returns them."""
    targets = []
    for b in range(cfg.B):
        t = target_rows(cfg, b, src_rows[b], None if drafts is None else drafts[b])
        step.set_target(b, t)
        targets.append(t)
    return targets
