"""Pins of oracle/policy.py: the paper's worked example, a library interpolator, closed forms on a linear
profile, brute force."""
import os

import numpy as np
import pytest
from scipy.interpolate import RegularGridInterpolator

from oracle import policy as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _profile(rng=None):
    b = [1, 4, 16, 64, 256]
    k = [1024, 16384, 65536, 262144]
    if rng is None:     # T = 2 + 0.01 B + 1e-5 KV, exactly bilinear
        ms = [[2 + 0.01 * x + 1e-5 * y for y in k] for x in b]
    else:
        ms = np.cumsum(np.cumsum(rng.uniform(0.1, 1.0, (len(b), len(k))), axis=0), axis=1).tolist()
    return b, k, ms


def test_lookup_is_bilinear_clamped_below_and_linear_beyond():
    rng = np.random.default_rng(0)
    b, k, ms = _profile(rng)
    pr = op.Profile(b, k, ms)
    for i, x in enumerate(b):
        for j, y in enumerate(k):
            assert pr.lookup(x, y) == pytest.approx(ms[i][j], rel=0, abs=1e-12)
    ref = RegularGridInterpolator((np.array(b, float), np.array(k, float)), np.array(ms), method="linear")
    for _ in range(200):
        x, y = rng.uniform(b[0], b[-1]), rng.uniform(k[0], k[-1])
        assert pr.lookup(x, y) == pytest.approx(float(ref([[x, y]])[0]), rel=1e-12)
    assert pr.lookup(0, 10) == ms[0][0] and pr.lookup(1, 500) == ms[0][0]              # below the first point
    ext = RegularGridInterpolator((np.array(b, float), np.array(k, float)), np.array(ms), method="linear", bounds_error=False, fill_value=None)
    for x, y in ((300, 70000), (100, 400000), (1000, 1e6)):                            # beyond the last point
        assert pr.lookup(x, y) == pytest.approx(float(ext([[x, y]])[0]), rel=1e-12)
    lin = op.Profile(*_profile())
    assert lin.lookup(100, 50000) == pytest.approx(2 + 1.0 + 0.5, rel=1e-12)
    assert lin.lookup(512, 524288) == pytest.approx(2 + 5.12 + 5.24288, rel=1e-12)


def test_future_kv_closed_forms_and_brute_force():
    # n equal requests: all finish together, the last iteration is the largest
    assert op.max_future_kv([(100, 0)] * 5, None, 40) == (5 * 140, 40)
    assert op.max_future_kv([(100, 30)] * 5, None, 40) == (5 * 110, 10)
    assert op.max_future_kv([(100, 70)], None, 40) == (101, 1)          # past the average: one more token
    # one long and one short request: the maximum is either when the short one ends or at the very end
    assert op.max_future_kv([(1000, 0), (10, 35)], None, 40)[0] == max(1005 + 15, 1040)
    rng = np.random.default_rng(1)
    for _ in range(50):
        run = [(int(rng.integers(1, 3000)), int(rng.integers(0, 300))) for _ in range(int(rng.integers(0, 20)))]
        new, avg = int(rng.integers(1, 3000)), int(rng.integers(1, 400))
        reqs = [[kv, max(1, avg - g)] for kv, g in run] + [[new, avg]]
        best = 0
        while reqs:                               # a literal simulation, one generated token at a time
            for r in reqs:
                r[0] += 1
                r[1] -= 1
            best = max(best, sum(r[0] for r in reqs))
            reqs = [r for r in reqs if r[1] > 0]
        assert op.max_future_kv(run, new, avg)[0] == best


def test_admission_uses_batch_size_future_kv_and_wait_time():
    pr = op.Profile(*_profile())               # T = 2 + 0.01 B + 1e-5 KV
    run = [(2000, 10)] * 15
    ok, t, kv = op.predict_admit(pr, run, 1000, 110, tpot_ms=5.0)
    # the 15 running requests end after 100 more tokens (KV 2100 each); the new one is at 1000 + 100 then
    assert kv == 15 * 2100 + 1100 and t == pytest.approx(2 + 0.16 + 1e-5 * kv) and ok
    ok2, t2, _ = op.predict_admit(pr, run, 1000, 110, tpot_ms=5.0, wait_ms=3.0)
    assert t2 == pytest.approx(t + 3.0) and not ok2
    assert not op.predict_admit(pr, run, 1000, 110, tpot_ms=t)[0]       # strictly below the TPOT


def test_dynamic_chunking_worked_example():
    prompt, patterns = None, []
    for line in open(os.path.join(GOLDEN, "dynamic_chunking_example.txt")):
        f = line.split()
        if f and f[0] == "prompt":
            prompt = int(f[1])
        elif f and f[0] == "pattern":
            patterns.append([int(v) for v in f[1:]])
    sizes = lambda plan: [sum(t for _, t in it) for it in plan]
    assert sizes(op.chunk_plan([prompt], 1024, dynamic=False)) == [1024, 1024, 2] and [1024, 1024, 2] in patterns
    assert sizes(op.chunk_plan([prompt], 1024, dynamic=False, first_iteration_used=1023)) == [1, 1024, 1024, 1] and [1, 1024, 1024, 1] in patterns
    assert sizes(op.chunk_plan([prompt], 1024, dynamic=True)) == [1024, 1026] and [1024, 1026] in patterns
    assert sizes(op.chunk_plan([prompt], 1024, dynamic=True, first_iteration_used=1023)) == [1, 1024, 1025]   # one cycle less than four
    assert sizes(op.chunk_plan([prompt], 4096, dynamic=False)) == [2050] and [2050] in patterns


def test_chunk_plan_invariants():
    rng = np.random.default_rng(2)
    for _ in range(200):
        prompts = [int(v) for v in rng.integers(1, 5000, size=int(rng.integers(1, 12)))]
        budget, dyn, used0 = int(rng.integers(1, 2048)), bool(rng.integers(0, 2)), 0
        if rng.integers(0, 2):
            used0 = int(rng.integers(0, budget + 1))
        plan = op.chunk_plan(prompts, budget, dyn, used0)
        got = [0] * len(prompts)
        order = []
        for n, it in enumerate(plan):
            tot = sum(t for _, t in it) + (used0 if n == 0 else 0)
            assert tot <= budget or (dyn and tot < 2 * budget)
            assert all(t >= 1 for _, t in it)
            for r, t in it:
                got[r] += t
                order.append(r)
            # an iteration that went over the budget did so by finishing its last request
            if tot > budget:
                r, _ = it[-1]
                assert got[r] == prompts[r]
        assert got == prompts and order == sorted(order)                 # everything served, first come first served
        if not dyn:
            assert len(plan) >= -(-(sum(prompts) + used0) // budget)
        assert len(op.chunk_plan(prompts, budget, True, used0)) <= len(op.chunk_plan(prompts, budget, False, used0))


def test_chunked_prefill_prediction_on_a_linear_profile():
    pr = op.Profile(*_profile())               # T = 2 + 0.01 B + 1e-5 KV
    run = [(4000, 0)] * 32
    T = lambda b, kv: 2 + 0.01 * b + 1e-5 * kv

    def keeps(c, prompt, tpot):      # the definition, iteration by iteration: 32 decodes grow by one token each time
        done, j = 0, 0
        while done < prompt:
            cc = min(c, prompt - done)
            if not T(32 + cc, 32 * (4001 + j) + done + cc) < tpot:
                return False
            done, j = done + cc, j + 1
        return True

    want = max(c for c in range(1, 2001) if keeps(c, 2000, 4.0))
    # the chunk that fits the first iteration alone, c < (4 - 2 - 0.32 - 1.28032) / 0.01001, cannot be kept: the prefix
    # it attends and the decodes grow, so the prediction settles on a smaller one
    first_only = int(np.ceil((4 - 2 - 0.32 - 1.28032) / 0.01001) - 1)
    assert not keeps(first_only, 2000, 4.0) and want < first_only
    ok, c, n, total = op.predict_chunked_prefill(pr, run, 2000, avg_decode=500, tpot_ms=4.0, ttft_ms=1e9)
    assert ok and c == want and n == -(-2000 // c)
    times = [pr.lookup(32 + min(c, 2000 - j * c), 32 * (4001 + j) + min((j + 1) * c, 2000)) for j in range(n)]
    assert total == pytest.approx(sum(times)) and max(times) < 4.0
    ok2, c2, n2, total2 = op.predict_chunked_prefill(pr, run, 30, avg_decode=500, tpot_ms=4.0, ttft_ms=1e9)
    assert ok2 and c2 == 30 and n2 == 1 and total2 == pytest.approx(pr.lookup(62, 32 * 4001 + 30))
    assert not op.predict_chunked_prefill(pr, run, 30, 500, 4.0, ttft_ms=total2)[0]           # TTFT is a strict bound, wait time counts
    assert not op.predict_chunked_prefill(pr, run, 30, 500, 4.0, ttft_ms=total2 + 1.0, wait_ms=1.5)[0]
    assert op.predict_chunked_prefill(pr, run, 30, 500, 1.0, 1e9) == (False, 0, 0, float("inf"))
    # decodes that are predicted to finish during the prefill stop counting: with 2 tokens left each, the third
    # iteration runs without them
    short = [(4000, 498)] * 32
    ok3, c3, n3, total3 = op.predict_chunked_prefill(pr, short, 600, avg_decode=500, tpot_ms=4.2, ttft_ms=1e9)
    assert ok3 and n3 >= 3
    t_last = pr.lookup(min(c3, 600 - (n3 - 1) * c3), 600)
    assert total3 == pytest.approx(sum(pr.lookup(32 + c3, 32 * (4001 + j) + (j + 1) * c3) for j in range(2))
                                   + sum(pr.lookup(min(c3, 600 - j * c3), min((j + 1) * c3, 600)) for j in range(2, n3)))
    assert t_last < 4.2


def test_batch_limits_on_a_linear_profile():
    pr = op.Profile(*_profile())
    p, d, tpot = 1000, 200, 6.0
    # T(B, B (p + d/2)) = 2 + B (0.01 + 1e-5 * 1100) < 6  ->  B < 4 / 0.021
    assert op.batch_limit_pd(pr, p, d, tpot, capacity=1e12) == int(np.ceil(4 / 0.021) - 1)
    assert op.batch_limit_pd(pr, p, d, tpot, capacity=50 * 1100 + 1) == 50          # memory-bound
    assert op.batch_limit_pd(pr, p, d, 2.0, 1e12) == 0
    # co-location: T_iter = 2 + 0.01 B + 1e-5 (d/(p+d) B (p + d/2) + p)
    f = lambda b: 2 + 0.01 * b + 1e-5 * (d / (p + d) * b * (p + d / 2) + p)
    want = max(b for b in range(1, 4097) if f(b) < tpot)
    assert op.batch_limit_co(pr, p, d, tpot, ttft_ms=1e12, capacity=1e12) == want
    # a tight TTFT needs few iterations, i.e. a large batch: the limit is an interval's upper end or nothing
    tight = (p + d) / want * f(want)
    assert op.batch_limit_co(pr, p, d, tpot, ttft_ms=tight, capacity=1e12) == 0


def test_cost_of_a_request_by_hand():
    # T = 2 + 0.01 B + 1e-5 KV with KV knots from 0: GEMM(B) = 2 + 0.01 B, DcAttn(kv) = 1e-5 kv
    pr = op.Profile([1, 4096], [0, 10 ** 7], [[2.01, 102.01], [42.96, 142.96]])
    assert op.gemm_time(pr, 100) == pytest.approx(3.0) and op.attn_time(pr, 220000) == pytest.approx(2.2)
    # co-located, p = 1000, d = 200, B = 100: 1200 * 3 / 100 + 0.01 + 1e-5 * 200 * 1100 = 36 + 0.01 + 2.2
    assert op.cost_co(pr, 1000, 200, 100) == pytest.approx(38.21)
    # disaggregated, B_pf = 2000, B_dc = 50: 1000 * 22 / 2000 + 0.01 + 200 * 2.5 / 50 + 2.2 = 11 + 0.01 + 10 + 2.2
    assert op.cost_pd(pr, 1000, 200, 2000, 50) == pytest.approx(23.21)
    # larger batches share the fixed 2 ms of an iteration among more tokens: the cost falls with B and tends to the
    # per-token slope, 0.01 (p + d) + attention
    costs = [op.cost_co(pr, 1000, 200, b) for b in (10, 100, 1000, 4000)]
    assert all(x > y for x, y in zip(costs, costs[1:])) and costs[-1] > 0.01 * 1200 + 2.21
    # at the batch limits: decode batch limit for TPOT 6 is ceil(4 / 0.021) - 1 = 190 (see the batch-limit test)
    assert op.optimal_cost_pd(pr, 1000, 200, 6.0, 1e12, 2000) == pytest.approx(op.cost_pd(pr, 1000, 200, 2000, 190))
    assert op.optimal_cost_pd(pr, 1000, 200, 2.0, 1e12, 2000) == float("inf")
    b = op.batch_limit_co(pr, 1000, 200, 6.0, 1e12, 1e12)
    assert op.optimal_cost_co(pr, 1000, 200, 6.0, 1e12, 1e12) == pytest.approx((1200 * (2 + 0.01 * b) / b) + 0.01 + 2.2)
    # a looser TPOT allows a larger batch and so a lower cost (the paper's Fig. on cost vs TPOT)
    assert op.optimal_cost_co(pr, 1000, 200, 12.0, 1e12, 1e12) < op.optimal_cost_co(pr, 1000, 200, 6.0, 1e12, 1e12)
