"""polysched (C++ behind the C ABI) against oracle/policy.py: integers and decisions bit-exact, times to
rounding; plus argument errors and exported symbols."""
import math
import os
import re

import numpy as np
import pytest

from oracle import policy as op
from paper_2507_17769_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _tables(rng):
    b = sorted(set(int(v) for v in rng.integers(1, 600, size=int(rng.integers(1, 7)))))
    k = sorted(set(int(v) for v in rng.integers(0, 2_000_000, size=int(rng.integers(1, 7)))))
    ms = np.cumsum(np.cumsum(rng.uniform(0.05, 2.0, (len(b), len(k))), axis=0), axis=1).astype(np.float32)
    return b, k, ms


def test_exports_every_declared_symbol():
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "polysched.h")).read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(ps_[a-z_]+)\s*\(", text)))
    assert declared == B.SCHED_EXPORTS, (declared, B.SCHED_EXPORTS)


def test_lookup_matches_oracle_everywhere():
    rng = np.random.default_rng(0)
    for _ in range(30):
        b, k, ms = _tables(rng)
        pr, want = B.Profile(b, k, ms), op.Profile(b, k, ms.tolist())
        pts = [(x, y) for x in b for y in k] + [(rng.uniform(-5, 900), rng.uniform(-10, 3e6)) for _ in range(60)]
        for x, y in pts:
            assert pr.lookup(x, y) == want.lookup(x, y)        # same double arithmetic in the same order
        pr.close()
    assert math.isnan(B.lib.ps_profile_lookup(None, 1.0, 1.0))


def test_future_kv_and_admission_match_oracle():
    rng = np.random.default_rng(1)
    b, k, ms = _tables(rng)
    pr, want = B.Profile(b, k, ms), op.Profile(b, k, ms.tolist())
    for _ in range(300):
        run = [(int(rng.integers(0, 5000)), int(rng.integers(0, 400))) for _ in range(int(rng.integers(0, 40)))]
        new, avg = int(rng.integers(0, 5000)), int(rng.integers(1, 500))
        assert B.max_future_kv(run, new, avg) == op.max_future_kv(run, new, avg)
        assert B.max_future_kv(run, None, avg) == op.max_future_kv(run, None, avg)
        tpot, wait = float(rng.uniform(0.1, 30)), float(rng.uniform(0, 5))
        assert pr.predict_admit(run, new, avg, tpot, wait) == op.predict_admit(want, run, new, avg, tpot, wait)
    pr.close()


def test_chunk_plan_matches_oracle_and_the_worked_example():
    sizes = lambda plan: [sum(t for _, t in it) for it in plan]
    assert sizes(B.chunk_plan([2050], 1024, False)) == [1024, 1024, 2]
    assert sizes(B.chunk_plan([2050], 1024, False, 1023)) == [1, 1024, 1024, 1]
    assert sizes(B.chunk_plan([2050], 1024, True)) == [1024, 1026]
    assert sizes(B.chunk_plan([2050], 1024, True, 1023)) == [1, 1024, 1025]
    rng = np.random.default_rng(2)
    for _ in range(300):
        prompts = [int(v) for v in rng.integers(1, 5000, size=int(rng.integers(0, 12)))]
        budget = int(rng.integers(1, 2048))
        used0 = int(rng.integers(0, budget + 1)) if rng.integers(0, 2) else 0
        for dyn in (False, True):
            assert B.chunk_plan(prompts, budget, dyn, used0) == op.chunk_plan(prompts, budget, dyn, used0)


def test_chunked_prefill_prediction_and_limits_match_oracle():
    rng = np.random.default_rng(3)
    for _ in range(12):
        b, k, ms = _tables(rng)
        pr, want = B.Profile(b, k, ms), op.Profile(b, k, ms.tolist())
        for _ in range(15):
            run = [(int(rng.integers(0, 5000)), int(rng.integers(0, 400))) for _ in range(int(rng.integers(0, 40)))]
            prompt, avg = int(rng.integers(1, 3000)), int(rng.integers(1, 500))
            tpot, ttft, wait = float(rng.uniform(0.1, 40)), float(rng.uniform(1, 400)), float(rng.uniform(0, 5))
            assert pr.predict_chunked_prefill(run, prompt, avg, tpot, ttft, wait) == op.predict_chunked_prefill(want, run, prompt, avg, tpot, ttft, wait)
        p, d = float(rng.integers(1, 4000)), float(rng.integers(1, 1000))
        tpot, ttft, cap = float(rng.uniform(0.5, 40)), float(rng.uniform(5, 2000)), float(rng.uniform(1e4, 3e6))
        assert pr.batch_limit_pd(p, d, tpot, cap, 600) == op.batch_limit_pd(want, p, d, tpot, cap, 600)
        assert pr.batch_limit_co(p, d, tpot, ttft, cap, 600) == op.batch_limit_co(want, p, d, tpot, ttft, cap, 600)
        pr.close()


def test_costs_match_oracle():
    rng = np.random.default_rng(5)
    for _ in range(20):
        b, k, ms = _tables(rng)
        pr, want = B.Profile(b, k, ms), op.Profile(b, k, ms.tolist())
        for _ in range(10):
            p, d = float(rng.integers(1, 8192)), float(rng.integers(1, 2048))
            bpf, bdc, bb = float(rng.integers(1, 4096)), float(rng.integers(1, 512)), float(rng.integers(1, 4096))
            tpot, ttft, cap = float(rng.uniform(1, 60)), float(rng.uniform(50, 2000)), float(rng.uniform(1e4, 3e6))
            assert pr.cost_pd(p, d, bpf, bdc) == op.cost_pd(want, p, d, bpf, bdc)      # same double arithmetic in the same order
            assert pr.cost_co(p, d, bb) == op.cost_co(want, p, d, bb)
            assert pr.optimal_cost_pd(p, d, tpot, cap, bpf, 600) == op.optimal_cost_pd(want, p, d, tpot, cap, bpf, 600)
            assert pr.optimal_cost_co(p, d, tpot, ttft, cap, 600) == op.optimal_cost_co(want, p, d, tpot, ttft, cap, 600)
        pr.close()
    assert math.isnan(B.lib.ps_cost_co(None, 1.0, 1.0, 1.0))


def test_argument_errors():
    with pytest.raises(B.PolystepError):
        B.Profile([4, 4], [1], [[1.0], [2.0]])            # batch sizes not strictly ascending
    with pytest.raises(B.PolystepError):
        B.Profile([1], [5, 2], [[1.0, 2.0]])
    with pytest.raises(B.PolystepError):
        B.Profile([1], [5], [[float("nan")]])
    with pytest.raises(B.PolystepError):
        B.chunk_plan([0], 16, True)                        # empty prompt
    with pytest.raises(B.PolystepError):
        B.chunk_plan([5], 16, True, 17)                    # more than the budget already used
    with pytest.raises(B.PolystepError):
        B.max_future_kv([(-1, 0)], 5, 10)
    with pytest.raises(B.PolystepError):
        B.max_future_kv([(1, 0)], 5, 0)
