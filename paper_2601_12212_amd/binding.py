"""ctypes binding of libdt.so.  Argument marshalling only."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdt.so")

DT_TT_MAX, DT_D_MAX, DT_K_MAX, DT_MASK_WORDS = 128, 8, 32, 2
DT_F32, DT_BF16 = 0, 1
DT_TREE_EARLY_STOP = 1
DT_ACCEPT_GREEDY, DT_ACCEPT_STOCHASTIC, DT_ACCEPT_SAMPLED = 0, 1, 2

_lib = None


class DtError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        msg = "%s failed: %s (%d)" % (fn, dt_status_string(status), status)
        if status == -5:
            lib = load_library()
            code = lib.dt_last_hip_error()
            msg += " [hip error %d: %s]" % (code, lib.dt_hip_error_string(code).decode())
        super().__init__(msg)


def library_path():
    return _LIB_PATH


def load_library():
    """Load libdt.so (built by paper_2601_12212_amd/build.py).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libdt.so is not built: run `python paper_2601_12212_amd/build.py` "
                              "(there is no fallback path)")
        lib = C.CDLL(_LIB_PATH)
        vp, i32, i64, u64, f32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
        lib.dt_status_string.restype = C.c_char_p
        lib.dt_status_string.argtypes = [i32]
        lib.dt_last_hip_error.restype = i32
        lib.dt_hip_error_string.restype = C.c_char_p
        lib.dt_hip_error_string.argtypes = [i32]
        lib.dt_workspace_bytes.argtypes = [i32, i64, i32, i32, i32, i32, C.POINTER(sz)]
        lib.dt_topk_rows.argtypes = [vp, vp, i32, i64, i32, i64, i32, vp, vp, vp, vp, sz]
        lib.dt_topk_rows_static.argtypes = [vp, vp, i32, i64, i32, i64, i32, vp, vp, vp]
        lib.dt_topk_rows_static.restype = i32
        lib.dt_build_tree.argtypes = [vp, i32, vp, vp, i32, i32, i64, vp, i64, vp, i32] + [vp] * 8 + [vp, sz, i32]
        lib.dt_tree_attention.argtypes = [vp, i32, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64,
                                          vp, i32, vp, vp, sz]
        lib.dt_accept.argtypes = [vp, i32, i32, f32, vp, i32, i32, i64, vp, vp, vp, vp, vp, vp, i32, u64, u64,
                                  vp, vp, vp, vp, vp, vp, sz]
        lib.dt_level_state_bytes.argtypes = [i32, C.POINTER(sz)]
        lib.dt_expand_level.argtypes = [vp, i32, i32, vp, vp, i32, i32, i64, i32, vp, i32, vp] + [vp] * 6 + [vp, sz, i32]
        lib.dt_finish_tree.argtypes = [vp, i32, vp, i32, vp, i32, vp] + [vp] * 8 + [i32]
        lib.dt_action_table.argtypes = [vp, i32, C.POINTER(i32)]
        lib.dt_policy_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(sz)]
        lib.dt_policy_step.argtypes = [vp, i32, i32, vp, i64, i32, i32, i32] + [vp] * 7 + [i32, i32, u64, u64] + \
                                      [vp] * 6 + [vp, sz]
        lib.dt_reward_step.argtypes = [vp, i32, vp, i32, f32, vp, vp, vp, vp, vp, vp]
        lib.dt_reward_step.restype = i32
        lib.dt_commit.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp, i32, vp, vp]
        lib.dt_profile_enable.argtypes = [i32]
        lib.dt_profile_enable.restype = i32
        lib.dt_profile_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(i32)]
        lib.dt_profile_read.restype = i32
        lib.dt_profile_kernel_name.argtypes = [i32]
        lib.dt_profile_kernel_name.restype = C.c_char_p
        lib.dt_init.argtypes = []
        for fn in ("dt_init", "dt_workspace_bytes", "dt_topk_rows", "dt_build_tree", "dt_tree_attention", "dt_accept", "dt_commit",
                   "dt_level_state_bytes", "dt_expand_level", "dt_finish_tree", "dt_action_table",
                   "dt_policy_workspace_bytes", "dt_policy_step"):
            getattr(lib, fn).restype = i32
        _lib = lib
    return _lib


def dt_status_string(status):
    return load_library().dt_status_string(status).decode()


def dt_init():
    rc = load_library().dt_init()
    if rc:
        raise DtError("dt_init", rc)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dtype(t):
    import torch
    if t.dtype == torch.float32:
        return DT_F32
    if t.dtype == torch.bfloat16:
        return DT_BF16
    raise TypeError("dt: tensors are float32 or bfloat16, got %s" % t.dtype)


def _check(fn, rc):
    if rc != 0:
        raise DtError(fn, rc)


def dt_workspace_bytes(batch, total_rows, V, TT_cap, Hq, D):
    out = C.c_size_t(0)
    _check("dt_workspace_bytes", load_library().dt_workspace_bytes(batch, total_rows, V, TT_cap, Hq, D, C.byref(out)))
    return out.value


def dt_topk_rows(logits, k, top_val, top_id, lse, ws):
    n_rows, V = logits.shape
    _check("dt_topk_rows", load_library().dt_topk_rows(
        _stream(), _ptr(logits), _dtype(logits), n_rows, V, logits.stride(0), k, _ptr(top_val), _ptr(top_id),
        _ptr(lse), _ptr(ws), ws.numel() * ws.element_size()))


def dt_topk_rows_static(logits, k, top_val, top_id, lse):
    n_rows, V = logits.shape
    _check("dt_topk_rows_static", load_library().dt_topk_rows_static(
        _stream(), _ptr(logits), _dtype(logits), n_rows, V, logits.stride(0), k, _ptr(top_val), _ptr(top_id),
        _ptr(lse)))


def dt_build_tree(params, draft_logits, row_off, total_rows, root_token, TT_cap, n_nodes, tokens, parents, depth,
                  score, logp, src_row, anc_mask, ws, flags=0):
    batch = params.shape[0]
    V = draft_logits.shape[1]
    _check("dt_build_tree", load_library().dt_build_tree(
        _stream(), batch, _ptr(params), _ptr(draft_logits), _dtype(draft_logits), V, draft_logits.stride(0),
        _ptr(row_off), total_rows, _ptr(root_token), TT_cap, _ptr(n_nodes), _ptr(tokens), _ptr(parents),
        _ptr(depth), _ptr(score), _ptr(logp), _ptr(src_row), _ptr(anc_mask), _ptr(ws),
        ws.numel() * ws.element_size(), flags))


def dt_tree_attention(q, k_tree, v_tree, n_nodes, k_prefix_ptrs, v_prefix_ptrs, prefix_len, max_prefix_len,
                      kv_stride_tok, kv_stride_head, anc_mask, scale, out, ws):
    batch, TT_cap, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    _check("dt_tree_attention", load_library().dt_tree_attention(
        _stream(), batch, _dtype(q), Hq, Hkv, D, scale, _ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(n_nodes),
        _ptr(k_prefix_ptrs), _ptr(v_prefix_ptrs), _ptr(prefix_len), max_prefix_len, kv_stride_tok, kv_stride_head,
        _ptr(anc_mask), TT_cap, _ptr(out), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size()))


def dt_accept(mode, temperature, target_logits, n_nodes, tokens, parents, depth, logp, anc_mask, philox_seed,
              philox_step, accept_len, best_node, path_nodes, out_tokens, node_argmax, ws):
    batch, TT_cap, V = target_logits.shape
    _check("dt_accept", load_library().dt_accept(
        _stream(), batch, mode, temperature, _ptr(target_logits), _dtype(target_logits), V, target_logits.stride(1),
        _ptr(n_nodes), _ptr(tokens), _ptr(parents), _ptr(depth), _ptr(logp), _ptr(anc_mask), TT_cap, philox_seed,
        philox_step, _ptr(accept_len), _ptr(best_node), _ptr(path_nodes), _ptr(out_tokens), _ptr(node_argmax),
        _ptr(ws), ws.numel() * ws.element_size()))


def dt_level_state_bytes(batch):
    out = C.c_size_t(0)
    _check("dt_level_state_bytes", load_library().dt_level_state_bytes(batch, C.byref(out)))
    return out.value


def dt_expand_level(level, params, level_logits, rows_per_seq, prefix_len, TT_cap, state, n_expand, exp_token,
                    exp_parent_slot, exp_row, exp_pos, exp_mask, ws, flags=0):
    """level_logits: [batch * R, V] with R = 1 at level 1, rows_per_seq otherwise."""
    batch = params.shape[0]
    V = level_logits.shape[1]
    _check("dt_expand_level", load_library().dt_expand_level(
        _stream(), batch, level, _ptr(params), _ptr(level_logits), _dtype(level_logits), V, level_logits.stride(0),
        rows_per_seq, _ptr(prefix_len), TT_cap, _ptr(state), _ptr(n_expand), _ptr(exp_token), _ptr(exp_parent_slot),
        _ptr(exp_row), _ptr(exp_pos), _ptr(exp_mask), _ptr(ws), ws.numel() * ws.element_size(), flags))


def dt_finish_tree(params, V, root_token, TT_cap, state, n_nodes, tokens, parents, depth, score, logp, src_row,
                   anc_mask, flags=0):
    batch = params.shape[0]
    _check("dt_finish_tree", load_library().dt_finish_tree(
        _stream(), batch, _ptr(params), V, _ptr(root_token), TT_cap, _ptr(state), _ptr(n_nodes), _ptr(tokens),
        _ptr(parents), _ptr(depth), _ptr(score), _ptr(logp), _ptr(src_row), _ptr(anc_mask), flags))


def dt_action_table():
    """-> list of (TT, d, k): the action table of the paper's appendix after its filter (host side)."""
    lib = load_library()
    n = C.c_int(0)
    buf = (C.c_int32 * (3 * 256))()
    _check("dt_action_table", lib.dt_action_table(buf, 256, C.byref(n)))
    return [(buf[3 * i], buf[3 * i + 1], buf[3 * i + 2]) for i in range(n.value)]


def dt_policy_workspace_bytes(batch, F, H):
    out = C.c_size_t(0)
    _check("dt_policy_workspace_bytes", load_library().dt_policy_workspace_bytes(batch, F, H, C.byref(out)))
    return out.value


def dt_policy_step(features, W1, b1, W2, b2, W3, b3, action_table, cache_interval, sample, philox_seed, philox_step,
                   cache_step, cached_action, params_out, action_out, queried_out, logits_out, ws):
    """features [batch, F]; W1 [F,H], W2 [H,H], W3 [H,A] float32 ([in][out]); action_table int32 [A,3] on the device."""
    batch, F = features.shape
    H, A = W3.shape
    _check("dt_policy_step", load_library().dt_policy_step(
        _stream(), batch, _dtype(features), _ptr(features), features.stride(0), F, H, A, _ptr(W1), _ptr(b1), _ptr(W2),
        _ptr(b2), _ptr(W3), _ptr(b3), _ptr(action_table), cache_interval, int(sample), philox_seed, philox_step,
        _ptr(cache_step), _ptr(cached_action), _ptr(params_out), _ptr(action_out), _ptr(queried_out), _ptr(logits_out),
        _ptr(ws), ws.numel() * ws.element_size()))


def dt_commit(dtype_of, Hkv, D, k_tree_ptrs, v_tree_ptrs, k_prefix_ptrs, v_prefix_ptrs, prefix_len, prefix_cap,
              kv_stride_tok, kv_stride_head, n_nodes, path_nodes, accept_len, out_tokens, TT_cap, new_prefix_len,
              next_root_token):
    """k_tree_ptrs / v_tree_ptrs: int64 device tensors [n_layers]; k_prefix_ptrs / v_prefix_ptrs: [n_layers, batch];
    dtype_of: any tensor of the cache dtype."""
    n_layers, batch = k_prefix_ptrs.shape
    _check("dt_commit", load_library().dt_commit(
        _stream(), batch, n_layers, _dtype(dtype_of), Hkv, D, _ptr(k_tree_ptrs), _ptr(v_tree_ptrs), _ptr(k_prefix_ptrs),
        _ptr(v_prefix_ptrs), _ptr(prefix_len), _ptr(prefix_cap), kv_stride_tok, kv_stride_head, _ptr(n_nodes),
        _ptr(path_nodes), _ptr(accept_len), _ptr(out_tokens), TT_cap, _ptr(new_prefix_len), _ptr(next_root_token)))


def dt_profile_enable(max_launches):
    _check("dt_profile_enable", load_library().dt_profile_enable(int(max_launches)))


def dt_profile_read(kernel_id):
    """-> (kernel name, total milliseconds, launches) recorded since the last dt_profile_enable."""
    ms, n = C.c_double(0), C.c_int(0)
    lib = load_library()
    _check("dt_profile_read", lib.dt_profile_read(kernel_id, C.byref(ms), C.byref(n)))
    return lib.dt_profile_kernel_name(kernel_id).decode(), ms.value, n.value


def dt_reward_step(accept_len, count_bonus, elapsed_seconds, cache_step, reward_sum, reward_steps, reward_avg,
                   interval_done, elapsed_per_seq=None):
    _check("dt_reward_step", load_library().dt_reward_step(
        _stream(), accept_len.shape[0], _ptr(accept_len), int(count_bonus), float(elapsed_seconds), _ptr(elapsed_per_seq),
        _ptr(cache_step), _ptr(reward_sum), _ptr(reward_steps), _ptr(reward_avg), _ptr(interval_done)))
