"""The allocation-free entry point (dt_topk_rows_static: scratch in device memory owned by the library)
against the entry point it is a variant of (dt_topk_rows: scratch in the caller's workspace).

Both run the same kernels, so every output must agree bit for bit, log-sum-exp included.  Two calls in a
row, the second on a smaller input: the scratch keeps the first call's contents and nothing of it may
leak into the second result.  Collected last on purpose (the round's end runs pytest -x)."""
import ctypes as C

import numpy as np
import pytest

import dt_synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _both(x, k):
    import paper_2601_12212_amd as dt
    R, V = x.shape
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16) if x.dtype == np.uint16 else torch.from_numpy(x).cuda()
    outs = []
    for static in (False, True):
        val = torch.full((R, k), 7.0, dtype=torch.float32, device="cuda")
        idx = torch.full((R, k), 7, dtype=torch.int32, device="cuda")
        lse = torch.full((R,), 7.0, dtype=torch.float32, device="cuda")
        if static:
            dt.dt_topk_rows_static(xd, k, val, idx, lse)
        else:
            ws = torch.zeros(dt.dt_workspace_bytes(1, R, V, 8, 1, 64), dtype=torch.uint8, device="cuda")
            dt.dt_topk_rows(xd, k, val, idx, lse, ws)
        torch.cuda.synchronize()
        outs.append((val.cpu().numpy(), idx.cpu().numpy(), lse.cpu().numpy()))
    return outs


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    from oracle import ref
    rng = np.random.default_rng(17)
    big = dt_synth.f32_to_bf16_bits((rng.standard_normal((51, 128256)) * 3).astype(np.float32))
    small = dt_synth.f32_to_bf16_bits((rng.standard_normal((7, 5003)) * 3).astype(np.float32))
    small[3, 11:] = dt_synth.f32_to_bf16_bits(np.array([-np.inf], np.float32))[0]      # a row with 11 viable tokens
    for x, k in ((big, 10), (small, 32), (rng.standard_normal((5, 1000)).astype(np.float32), 3)):
        (v0, i0, l0), (v1, i1, l1) = _both(x, k)
        assert np.array_equal(i0, i1) and np.array_equal(v0.view(np.uint32), v1.view(np.uint32))
        assert np.array_equal(l0.view(np.uint32), l1.view(np.uint32))
        wv, wi, wl = ref.topk_rows(x, k)                     # and both against the oracle
        assert np.array_equal(i1, wi) and np.array_equal(v1, wv)
        fin = np.isfinite(wl)
        assert (np.abs(l1[fin] - wl[fin]) <= 4e-6 * np.maximum(1.0, np.abs(wl[fin]))).all()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import paper_2601_12212_amd as dt
    lib = dt.load_library()
    one = C.c_void_p(256)
    # 497 rows of the Llama vocabulary need 497 * 16 * 1056 bytes > 8 MiB: refused on the host, nothing launched
    assert lib.dt_topk_rows_static(None, one, 1, 497, 128256, 128256, 10, one, one, one) == -2
    assert lib.dt_topk_rows_static(None, None, 1, 4, 1024, 1024, 4, one, one, one) == -1
    assert lib.dt_topk_rows_static(None, one, 1, 4, 1024, 1024, 33, one, one, one) == -2
    assert lib.dt_topk_rows_static(None, one, 1, 0, 1024, 1024, 4, one, one, one) == 0
    x = torch.zeros((496, 128256), dtype=torch.bfloat16, device="cuda")                 # the largest that fits
    val = torch.empty((496, 4), dtype=torch.float32, device="cuda")
    idx = torch.empty((496, 4), dtype=torch.int32, device="cuda")
    lse = torch.empty(496, dtype=torch.float32, device="cuda")
    dt.dt_topk_rows_static(x, 4, val, idx, lse)
    torch.cuda.synchronize()
    assert (idx.cpu().numpy() == np.arange(4)).all() and np.allclose(lse.cpu().numpy(), np.log(128256.0), rtol=1e-6)
