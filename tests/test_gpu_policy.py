"""GPU parity of the action selection (dt_policy_step) against the oracle: logits within fp32 accumulation
error of the float64 MLP, actions / cache state / emitted (TT, d, k) exact wherever the oracle's deciding gap
is above the guard."""
import numpy as np
import pytest

import dt_synth
from oracle import ref

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

LOGIT_TOL = 3e-4
GREEDY_GUARD = 3e-3      # top-2 logit gap below which the chosen action is not compared
SAMPLE_GUARD = 1e-4      # distance of the uniform to a CDF edge


def run_policy(B, F, H, bf16, N, sample, steps, seed):
    import paper_2601_12212_amd as dt
    rng = np.random.default_rng(seed)
    table = np.array(dt.dt_action_table(), np.int32)
    A = len(table)
    W1 = (rng.standard_normal((F, H)) / np.sqrt(F)).astype(np.float32)
    W2 = (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float32)
    W3 = (rng.standard_normal((H, A)) * (3.0 / np.sqrt(H))).astype(np.float32)
    b1, b2, b3 = (rng.standard_normal(n).astype(np.float32) * 0.1 for n in (H, H, A))
    dev = lambda a: torch.from_numpy(a).cuda()
    dW = [dev(a) for a in (W1, b1, W2, b2, W3, b3)]
    d_table = dev(table)
    i32 = dict(dtype=torch.int32, device="cuda")
    cache_step = torch.zeros(B, **i32)
    cached = torch.full((B,), -1, **i32)
    # sequence 1 starts in the middle of an interval with a cached action (if there is a sequence 1)
    o_cs, o_ca = [0] * B, [-1] * B
    if B > 1 and N > 3:
        cache_step[1], cached[1] = 2, 5
        o_cs[1], o_ca[1] = 2, 5
    params_out = torch.zeros((B, 3), **i32)
    action_out = torch.zeros(B, **i32)
    queried = torch.zeros(B, **i32)
    logits_out = torch.zeros((B, A), dtype=torch.float32, device="cuda")
    ws = torch.empty(dt.dt_policy_workspace_bytes(B, F, H), dtype=torch.uint8, device="cuda")
    compared = close_calls = 0
    for t in range(steps):
        x = rng.standard_normal((B, F)).astype(np.float32)
        if bf16:
            bits = dt_synth.f32_to_bf16_bits(x)
            x = dt_synth.bf16_bits_to_f32(bits)
            feat = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        else:
            feat = dev(x)
        logits_out.fill_(-77.0)
        dt.dt_policy_step(feat, *dW, d_table, N, sample, 99, t, cache_step, cached, params_out, action_out, queried,
                          logits_out, ws)
        torch.cuda.synchronize()
        for b in range(B):
            lg = ref.policy_logits(x[b], W1, b1, W2, b2, W3, b3)
            r = ref.policy_step(o_cs[b], o_ca[b], lg, N, mode=sample, seed=99, step=t, seq=b)
            assert int(queried[b]) == int(r["queried"]), (t, b)
            if r["queried"]:
                got = logits_out[b].cpu().numpy()
                assert np.abs(got - lg).max() < LOGIT_TOL, (t, b, np.abs(got - lg).max())
                if r["margin"] < (SAMPLE_GUARD if sample else GREEDY_GUARD):
                    # too close to call across precisions: both neighbours of the deciding gap are correct.
                    # The device's choice must be one of them (greedy: a logit within the guard of the
                    # oracle's best; sampling: the chosen CDF bin or one next to it); the checker then
                    # continues from that choice, and such steps are counted.
                    dev_act = int(action_out[b])
                    if sample:
                        assert abs(dev_act - r["action"]) <= 1, (t, b, dev_act, r["action"])
                    else:
                        assert lg.max() - lg[dev_act] < GREEDY_GUARD, (t, b, dev_act, r["action"])
                    assert int(cached[b]) == dev_act and int(cache_step[b]) == r["cache_step"]
                    o_cs[b], o_ca[b] = r["cache_step"], dev_act
                    close_calls += 1
                    continue
            else:
                assert (logits_out[b] == -77.0).all()             # nothing evaluated for a cached action
            o_cs[b], o_ca[b] = r["cache_step"], r["cached_action"]
            assert int(action_out[b]) == r["action"], (t, b)
            assert int(cache_step[b]) == r["cache_step"] and int(cached[b]) == r["cached_action"]
            assert tuple(int(v) for v in params_out[b]) == tuple(int(v) for v in table[r["action"]])
            compared += 1
    print("policy parity: %d decisions compared exactly, %d inside the guard" % (compared, close_calls))
    assert compared > 0.8 * B * steps and close_calls <= 0.1 * B * steps


def test_policy_llama_features_greedy_with_interval():
    run_policy(B=3, F=3 * 4096, H=128, bf16=True, N=4, sample=0, steps=10, seed=1)


def test_policy_sampling_small_net_and_odd_feature_size():
    run_policy(B=11, F=1000, H=64, bf16=False, N=2, sample=1, steps=8, seed=2)


def test_policy_every_step_and_one_sequence():
    run_policy(B=1, F=3 * 5120, H=128, bf16=True, N=1, sample=0, steps=5, seed=3)


@pytest.mark.parametrize("N,bonus,per_seq", [(4, 1, False), (10, 0, True), (1, 1, False)])
def test_reward_averaged_over_the_cache_interval(N, bonus, per_seq):
    """dt_policy_step and dt_reward_step driven together over several intervals: the device accumulators,
    the interval-closed flags and the averaged reward against the oracle's (float against double)."""
    import paper_2601_12212_amd as dt
    B, F, H, steps = 5, 256, 64, 3 * N + 2
    rng = np.random.default_rng(100 + N)
    table = np.array(dt.dt_action_table(), np.int32)
    A = len(table)
    dev = lambda a: torch.from_numpy(a).cuda()
    Wts = [dev((rng.standard_normal(sh) * sc).astype(np.float32)) for sh, sc in
           (((F, H), F ** -0.5), ((H,), 0.1), ((H, H), H ** -0.5), ((H,), 0.1), ((H, A), 1.0), ((A,), 0.1))]
    i32 = dict(dtype=torch.int32, device="cuda")
    cache_step, cached = torch.zeros(B, **i32), torch.full((B,), -1, **i32)
    cache_step[1], cached[1] = (2 % N), (5 if N > 2 else -1)          # one sequence starts inside an interval
    params_out = torch.zeros((B, 3), **i32)
    ws = torch.empty(dt.dt_policy_workspace_bytes(B, F, H), dtype=torch.uint8, device="cuda")
    r_sum = torch.zeros(B, dtype=torch.float32, device="cuda")
    r_steps = torch.zeros(B, **i32)
    r_avg = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
    r_done = torch.full((B,), -1, **i32)
    acc = [dict(sum=0.0, steps=0) for _ in range(B)]
    closed = 0
    for t in range(steps):
        feat = dev(rng.standard_normal((B, F)).astype(np.float32))
        dt.dt_policy_step(feat, *Wts, dev(table), N, 0, 7, t, cache_step, cached, params_out, None, None, None, ws)
        accept_len = rng.integers(0, 9, B).astype(np.int32)
        secs = rng.uniform(0.003, 0.02, B).astype(np.float32)
        if per_seq:
            dt.dt_reward_step(dev(accept_len), bonus, 0.0, cache_step, r_sum, r_steps, r_avg, r_done, elapsed_per_seq=dev(secs))
        else:
            secs[:] = secs[0]
            dt.dt_reward_step(dev(accept_len), bonus, float(secs[0]), cache_step, r_sum, r_steps, r_avg, r_done)
        torch.cuda.synchronize()
        cs = cache_step.cpu().numpy()
        for b in range(B):
            done, avg = ref.reward_step(int(cs[b]), float(accept_len[b] + bonus), float(secs[b]), acc[b])
            assert int(r_done[b]) == int(done), (t, b)
            assert int(r_steps[b]) == acc[b]["steps"]
            assert abs(float(r_sum[b]) - acc[b]["sum"]) <= 2e-6 * max(1.0, acc[b]["sum"])
            if done:
                assert abs(float(r_avg[b]) - avg) <= 2e-6 * avg, (t, b, float(r_avg[b]), avg)
                closed += 1
    assert closed >= 2 * B
