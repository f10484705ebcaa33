"""Device buffers of one speculative step for a batch, and the three library calls on them.

Plumbing only: allocation with torch, host->device copies of caller-provided arrays, and
calls into the binding.  No arithmetic of the method happens here.
"""
import numpy as np
import torch

from . import binding as B


def _to_torch(a, dtype, device):
    """numpy float32 / uint16(bf16 bits) -> device tensor of `dtype`."""
    if dtype == torch.bfloat16:
        assert a.dtype == np.uint16
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    assert a.dtype == np.float32
    return torch.from_numpy(a).to(device)


class Step:
    def __init__(self, params, prefix_len, Hq, Hkv, D, V, dtype=torch.bfloat16, mode=B.DT_ACCEPT_GREEDY,
                 temperature=1.0, TT_cap=None, philox_seed=0, device="cuda", tree_flags=0, kv_head_major=False):
        """kv_head_major: the prefix caches are laid out [kv head, token, D] (every head's keys contiguous,
        one common token capacity) instead of [token, kv head, D]; the library takes either through its two
        strides."""
        self.device, self.dtype = device, dtype
        self.Bsz = len(params)
        self.Hq, self.Hkv, self.D, self.V = Hq, Hkv, D, V
        self.mode, self.temperature, self.philox_seed = mode, float(temperature), int(philox_seed)
        self.tree_flags = int(tree_flags)
        self.TT_cap = int(TT_cap if TT_cap is not None else max(p[0] for p in params))
        self.host_params = [tuple(int(x) for x in p) for p in params]
        self.host_prefix_len = [int(x) for x in prefix_len]
        rows = [1 + (d - 1) * k for (_, d, k) in self.host_params]
        self.host_row_off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int64)
        self.total_rows = int(self.host_row_off[-1])
        dev, i32 = device, torch.int32
        Bz, TC = self.Bsz, self.TT_cap
        self.params = torch.tensor(self.host_params, dtype=i32, device=dev)
        self.row_off = torch.from_numpy(self.host_row_off).to(dev)
        self.root_token = torch.zeros(Bz, dtype=i32, device=dev)
        self.draft_logits = torch.empty((self.total_rows, V), dtype=dtype, device=dev)
        self.target_logits = torch.zeros((Bz, TC, V), dtype=dtype, device=dev)
        self.n_nodes = torch.zeros(Bz, dtype=i32, device=dev)
        self.tokens = torch.full((Bz, TC), -1, dtype=i32, device=dev)
        self.parents = torch.full((Bz, TC), -1, dtype=i32, device=dev)
        self.depth = torch.zeros((Bz, TC), dtype=i32, device=dev)
        self.src_row = torch.full((Bz, TC), -1, dtype=i32, device=dev)
        self.score = torch.zeros((Bz, TC), dtype=torch.float32, device=dev)
        self.logp = torch.zeros((Bz, TC), dtype=torch.float32, device=dev)
        self.anc_mask = torch.zeros((Bz, TC, B.DT_MASK_WORDS), dtype=torch.int64, device=dev)
        self.q = torch.zeros((Bz, TC, Hq, D), dtype=dtype, device=dev)
        self.k_tree = torch.zeros((Bz, TC, Hkv, D), dtype=dtype, device=dev)
        self.v_tree = torch.zeros((Bz, TC, Hkv, D), dtype=dtype, device=dev)
        self.out = torch.zeros((Bz, TC, Hq, D), dtype=dtype, device=dev)
        self.kv_head_major = bool(kv_head_major)
        if self.kv_head_major:
            cap = max(max(self.host_prefix_len), 1)
            shapes = [(Hkv, cap, D)] * Bz
            self.kv_stride_tok, self.kv_stride_head = D, cap * D
        else:
            shapes = [(max(L, 1), Hkv, D) for L in self.host_prefix_len]
            self.kv_stride_tok, self.kv_stride_head = Hkv * D, D
        self.k_prefix = [torch.zeros(s, dtype=dtype, device=dev) for s in shapes]
        self.v_prefix = [torch.zeros(s, dtype=dtype, device=dev) for s in shapes]
        self.k_prefix_ptrs = torch.tensor([t.data_ptr() for t in self.k_prefix], dtype=torch.int64, device=dev)
        self.v_prefix_ptrs = torch.tensor([t.data_ptr() for t in self.v_prefix], dtype=torch.int64, device=dev)
        self.prefix_len = torch.tensor(self.host_prefix_len, dtype=i32, device=dev)
        self.accept_len = torch.zeros(Bz, dtype=i32, device=dev)
        self.best_node = torch.zeros(Bz, dtype=i32, device=dev)
        self.path_nodes = torch.zeros((Bz, B.DT_D_MAX + 1), dtype=i32, device=dev)
        self.out_tokens = torch.zeros((Bz, B.DT_D_MAX + 1), dtype=i32, device=dev)
        self.node_argmax = torch.zeros((Bz, TC), dtype=i32, device=dev)
        nbytes = B.dt_workspace_bytes(Bz, self.total_rows, V, TC, Hq, D)
        self.ws = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        self.scale = 1.0 / float(np.sqrt(D))

    # ---- uploads (numpy float32 or bf16 bit patterns) ----------------------------------------
    def set_draft(self, b, rows):
        r0 = int(self.host_row_off[b])
        self.draft_logits[r0:r0 + rows.shape[0]].copy_(_to_torch(rows, self.dtype, self.device))

    def set_root_token(self, b, tok):
        self.root_token[b] = int(tok)

    def set_target(self, b, rows):
        self.target_logits[b, :rows.shape[0]].copy_(_to_torch(rows, self.dtype, self.device))

    def set_qkv(self, b, q, kt, vt, kp, vp):
        n = q.shape[0]
        self.q[b, :n].copy_(_to_torch(q, self.dtype, self.device))
        self.k_tree[b, :n].copy_(_to_torch(kt, self.dtype, self.device))
        self.v_tree[b, :n].copy_(_to_torch(vt, self.dtype, self.device))
        if kp.shape[0]:
            kd, vd = _to_torch(kp, self.dtype, self.device), _to_torch(vp, self.dtype, self.device)
            if self.kv_head_major:
                self.k_prefix[b][:, :kp.shape[0]].copy_(kd.permute(1, 0, 2))
                self.v_prefix[b][:, :vp.shape[0]].copy_(vd.permute(1, 0, 2))
            else:
                self.k_prefix[b][:kp.shape[0]].copy_(kd)
                self.v_prefix[b][:vp.shape[0]].copy_(vd)

    # ---- the three calls ------------------------------------------------------------------------
    def build_tree(self):
        B.dt_build_tree(self.params, self.draft_logits, self.row_off, self.total_rows, self.root_token, self.TT_cap,
                        self.n_nodes, self.tokens, self.parents, self.depth, self.score, self.logp, self.src_row,
                        self.anc_mask, self.ws, self.tree_flags)

    def tree_attention(self):
        B.dt_tree_attention(self.q, self.k_tree, self.v_tree, self.n_nodes, self.k_prefix_ptrs, self.v_prefix_ptrs,
                            self.prefix_len, max(self.host_prefix_len), self.kv_stride_tok, self.kv_stride_head,
                            self.anc_mask, self.scale, self.out, self.ws)

    def accept(self, philox_step=0):
        B.dt_accept(self.mode, self.temperature, self.target_logits, self.n_nodes, self.tokens, self.parents,
                    self.depth, self.logp, self.anc_mask, self.philox_seed, int(philox_step), self.accept_len,
                    self.best_node, self.path_nodes, self.out_tokens, self.node_argmax, self.ws)

    def run(self, philox_step=0):
        self.build_tree()
        self.tree_attention()
        self.accept(philox_step)

    # ---- the same three calls with the argument lists marshalled once ---------------------------
    def prepare(self):
        """Marshal the (fixed) pointer arguments once; run_prepared() then costs three foreign calls."""
        p = lambda t: None if t is None else t.data_ptr()
        dtc = B._dtype(self.draft_logits)
        wsb = self.ws.numel()
        self._lib = B.load_library()
        self._a_build = (self.Bsz, p(self.params), p(self.draft_logits), dtc, self.V, self.draft_logits.stride(0),
                         p(self.row_off), self.total_rows, p(self.root_token), self.TT_cap, p(self.n_nodes),
                         p(self.tokens), p(self.parents), p(self.depth), p(self.score), p(self.logp),
                         p(self.src_row), p(self.anc_mask), p(self.ws), wsb, self.tree_flags)
        self._a_attn = (self.Bsz, dtc, self.Hq, self.Hkv, self.D, self.scale, p(self.q), p(self.k_tree),
                        p(self.v_tree), p(self.n_nodes), p(self.k_prefix_ptrs), p(self.v_prefix_ptrs),
                        p(self.prefix_len), max(self.host_prefix_len), self.kv_stride_tok, self.kv_stride_head,
                        p(self.anc_mask), self.TT_cap, p(self.out), p(self.ws), wsb)
        self._a_acc_head = (self.Bsz, self.mode, self.temperature, p(self.target_logits), dtc, self.V,
                            self.target_logits.stride(1), p(self.n_nodes), p(self.tokens), p(self.parents),
                            p(self.depth), p(self.logp), p(self.anc_mask), self.TT_cap, self.philox_seed)
        self._a_acc_tail = (p(self.accept_len), p(self.best_node), p(self.path_nodes), p(self.out_tokens),
                            p(self.node_argmax), p(self.ws), wsb)
        return self

    def run_prepared(self, stream, philox_step=0):
        lib = self._lib
        rc = lib.dt_build_tree(stream, *self._a_build)
        rc = rc or lib.dt_tree_attention(stream, *self._a_attn)
        rc = rc or lib.dt_accept(stream, *self._a_acc_head, philox_step, *self._a_acc_tail)
        if rc:
            raise B.DtError("step", rc)

    # ---- downloads ----------------------------------------------------------------------------------
    def tree(self, b):
        n = int(self.n_nodes[b].item())
        g = lambda t: t[b, :n].cpu().numpy()
        return dict(n_nodes=n, tokens=g(self.tokens), parents=g(self.parents), depth=g(self.depth),
                    score=g(self.score), logp=g(self.logp), src_row=g(self.src_row),
                    anc_mask=self.anc_mask[b, :n].cpu().numpy().view(np.uint64))

    def accepted(self, b):
        n = int(self.n_nodes[b].item())
        return dict(accept_len=int(self.accept_len[b].item()), best_node=int(self.best_node[b].item()),
                    path_nodes=self.path_nodes[b].cpu().numpy(), out_tokens=self.out_tokens[b].cpu().numpy(),
                    node_argmax=self.node_argmax[b, :n].cpu().numpy())

    def attention_out(self, b):
        n = int(self.n_nodes[b].item())
        return self.out[b, :n].float().cpu().numpy()
