"""ps_sim_run (C++, through the C ABI) against the simulator oracle: every per-request output and every counter
identical, on traces that reach queueing, drops, promotion, parking and scale-down."""
import numpy as np
import pytest

from oracle import policy as opol
from oracle import sim as osim
from oracle import sim_pd as osim_pd
from paper_2507_17769_amd import binding as B
from paper_2507_17769_amd import workloads as W

BS = (1, 16, 64, 256, 1024, 4096)
KS = (16, 4096, 65536, 1048576)


def tables(fn):
    ms = np.array([[fn(b, k) for k in KS] for b in BS], dtype=np.float32)  # the C table stores float32
    return B.Profile(BS, KS, ms), opol.Profile(BS, KS, ms.astype(np.float64).tolist())


def compare(got, want, n):
    for name in ("end_ms", "cost_ms", "scale_ups", "scale_downs", "promotions", "dropped"):
        assert got[name] == want[name], (name, got[name], want[name])
    assert got["attained"].tolist() == want["attained"]
    if "server" in want:   # co-located: one instance does both phases
        assert got["server"].tolist() == want["server"] and got["decode_server"].tolist() == want["server"]
    else:
        assert got["server"].tolist() == want["prefill_server"] and got["decode_server"].tolist() == want["decode_server"]
    assert got["first_token_ms"].tolist() == want["first_token_ms"]   # doubles, bit for bit
    assert got["finish_ms"].tolist() == want["finish_ms"]


@pytest.mark.parametrize("seed,n_servers,rate,max_prompt,max_output,avg,period,cap,burst", [
    (0, 4, 0.03, 1024, 256, 128, 200, 2e6, False),
    (1, 2, 0.5, 1024, 256, 128, 200, 2e6, False),       # overloaded: queues and drops
    (2, 8, 0.06, 1024, 256, 128, 50, 2e6, True),        # frequent scale-down checks, tier mix flips half way
    (3, 3, 0.01, 1024, 256, 128, 100, 2500.0, False), # long prompts in several chunks, KV capacity binds
    (4, 20, 0.25, 1024, 256, 128, 1000, 2e6, False),
    (5, 6, 0.01, 4096, 128, 64, 300, 2e6, False),       # prompts that need several chunks under the tight tiers
])
def test_simulator_matches_the_oracle(seed, n_servers, rate, max_prompt, max_output, avg, period, cap, burst):
    gp, op = tables(lambda b, k: 4.0 + 0.012 * b + 2e-5 * k)
    n = 300 if cap > 1e5 else 100   # queued requests are tried again every step: the capacity-bound case is slow in the oracle
    tr = W.sim_trace(seed, n, rate, max_prompt, max_output, burst=burst)
    args = (tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], list(W.SIM_TPOTS_MS), n_servers, avg, cap, period)
    want = osim.simulate(op, *args)
    got = gp.simulate(*args)
    print({k: v for k, v in want.items() if not isinstance(v, list)}, "attained", sum(want["attained"]))
    compare(got, want, n)
    gp.close()


@pytest.mark.parametrize("seed,n_servers,rate,max_prompt,max_output,avg,period,cap,budget,burst", [
    (0, 4, 0.03, 1024, 256, 128, 200, 2e6, 1024, False),
    (1, 3, 0.5, 1024, 256, 128, 200, 2e6, 1024, False),       # overloaded: queues and drops on both sides
    (2, 8, 0.06, 1024, 256, 128, 50, 2e6, 512, True),         # frequent scale-down checks, tier mix flips half way
    (3, 4, 0.02, 8192, 512, 256, 100, 60000.0, 2048, False),  # long prompts in several chunks, KV capacity binds
    (4, 20, 0.25, 1024, 256, 128, 1000, 2e6, 2048, False),
])
def test_disaggregated_simulator_matches_the_oracle(seed, n_servers, rate, max_prompt, max_output, avg, period, cap, budget, burst):
    gp, op = tables(lambda b, k: 4.0 + 0.012 * b + 2e-5 * k)
    n = 300
    tr = W.sim_trace(seed, n, rate, max_prompt, max_output, burst=burst)
    args = (tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], list(W.SIM_TPOTS_MS), n_servers, avg, cap)
    want = osim_pd.simulate(op, *args, budget, period)
    got = gp.simulate(*args, period, disaggregated=True, prefill_budget=budget)
    print({k: v for k, v in want.items() if not isinstance(v, list)}, "attained", sum(want["attained"]))
    compare(got, want, n)
    gp.close()


def test_disaggregated_paths_are_all_reached_by_the_comparison_cases():
    _, op = tables(lambda b, k: 4.0 + 0.012 * b + 2e-5 * k)
    seen = {"dropped": 0, "promotions": 0, "scale_downs": 0, "multi_chunk": 0}
    for seed, n_servers, rate, mp, mo, avg, period, cap, budget, burst in ((1, 3, 0.5, 1024, 256, 128, 200, 2e6, 1024, False),
                                                                        (3, 4, 0.02, 8192, 512, 256, 100, 60000.0, 2048, False)):
        tr = W.sim_trace(seed, 300, rate, mp, mo, burst=burst)
        res = osim_pd.simulate(op, tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], list(W.SIM_TPOTS_MS), n_servers, avg, cap, budget, period)
        for k in ("dropped", "promotions", "scale_downs"):
            seen[k] += res[k]
        seen["multi_chunk"] += sum(1 for p, f in zip(tr["prompt"], res["first_token_ms"]) if p >= 2 * budget and f > 0)
    assert all(v > 0 for v in seen.values()), seen


def test_simulator_paths_are_all_reached_by_the_comparison_cases():
    """The cases above are only worth something if they reach the branches; checked on the oracle."""
    _, op = tables(lambda b, k: 4.0 + 0.012 * b + 2e-5 * k)
    seen = {"dropped": 0, "promotions": 0, "scale_downs": 0}
    for seed, n_servers, rate, burst, period in ((1, 2, 0.5, False, 200), (2, 8, 0.06, True, 50)):
        tr = W.sim_trace(seed, 300, rate, 1024, 256, burst=burst)
        res = osim.simulate(op, tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], list(W.SIM_TPOTS_MS), n_servers, 128, 2e6, period)
        for k in seen:
            seen[k] += res[k]
    assert all(v > 0 for v in seen.values()), seen


def test_simulator_stops_at_max_steps_and_rejects_malformed_input():
    gp, op = tables(lambda b, k: 7.0)
    args = ([0.0, 5.0], [100, 100], [1000, 1000], [300.0, 300.0], [0, 1], [20.0, 50.0], 2, 100, 1e9, 100)
    got, want = gp.simulate(*args, max_steps=500), osim.simulate(op, *args, max_steps=500)
    assert got["end_ms"] == 500
    compare(got, want, 2)
    with pytest.raises(B.PolystepError):
        gp.simulate([5.0, 0.0], [1, 1], [1, 1], [300.0, 300.0], [0, 0], [20.0], 1, 1, 1e9)      # arrivals not sorted
    with pytest.raises(B.PolystepError):
        gp.simulate([0.0], [1], [1], [300.0], [1], [20.0], 1, 1, 1e9)                            # tier out of range
    with pytest.raises(B.PolystepError):
        gp.simulate([0.0], [1], [1], [300.0], [0], [50.0, 20.0], 1, 1, 1e9)                      # tiers not ascending
    with pytest.raises(B.PolystepError):
        gp.simulate([0.0], [1], [1], [300.0], [0], [20.0], 1, 1, 1e9, disaggregated=True)        # no prefill budget
    gp.close()


def test_random_configurations_match_the_oracle():
    """Seeded random tables, cluster sizes, rates, length mixes, check periods, capacities and budgets, either deployment."""
    rng = np.random.default_rng(1)
    for it in range(12):
        a, bb, cc = float(rng.uniform(2, 8)), float(rng.uniform(0.004, 0.03)), float(rng.uniform(5e-6, 5e-5))
        gp, op = tables(lambda b, k: a + bb * b + cc * k)
        n_servers, rate = int(rng.integers(1, 12)), float(rng.choice([0.005, 0.02, 0.05, 0.15, 0.4]))
        max_prompt, max_output, avg = int(rng.choice([256, 1024, 4096])), int(rng.choice([64, 256])), int(rng.choice([32, 128]))
        period, cap, burst = int(rng.choice([50, 200, 1000])), float(rng.choice([3000.0, 30000.0, 2e6])), bool(rng.integers(0, 2))
        budget = int(rng.choice([256, 1024, 2048]))
        tr = W.sim_trace(int(rng.integers(0, 10000)), 120, rate, max_prompt, max_output, burst=burst)
        args = (tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], list(W.SIM_TPOTS_MS), n_servers, avg, cap)
        if rng.integers(0, 2):
            want = osim_pd.simulate(op, *args, budget, period)
            got = gp.simulate(*args, period, disaggregated=True, prefill_budget=budget)
        else:
            want = osim.simulate(op, *args, period)
            got = gp.simulate(*args, period)
        compare(got, want, 120)
        gp.close()
