"""Pins of the cluster simulator's oracle: hand-computed timelines, capacity bounds that follow from
the admission formulas, the placement order of Sec. 4.3/4.4 on constructed clusters, and invariants
of the deadline-based SLO (Sec. 2.3) on random traces."""
import math

import numpy as np
import pytest

from oracle import policy, sim
from paper_2507_17769_amd import workloads as W


def table(fn, bs=(1, 64, 4096), ks=(1, 65536, 10 ** 7)):
    return policy.Profile(bs, ks, [[fn(b, k) for k in ks] for b in bs])


def run(prof, reqs, tpots, n_servers, avg, period=1000, cap=10 ** 12, max_steps=10 ** 9):
    a, p, o, t, tier = (list(c) for c in zip(*reqs))
    return sim.simulate(prof, a, p, o, t, tier, tpots, n_servers, avg, cap, period, max_steps)


def test_single_request_timeline_by_hand():
    # constant 7.3 ms iterations; arrival 0.4 is seen at step 1 and the idle instance starts the prefill there: 1 -> 8.3;
    # iterations then run back to back: 8.3 -> 15.6 -> 22.9 (third token, done), noticed at step 23; the run ends after it
    res = run(table(lambda b, k: 7.3), [(0.4, 100, 3, 300.0, 0)], [20.0], 1, 3)
    assert res["first_token_ms"] == [1 + 7.3] and res["finish_ms"] == [1 + 7.3 + 7.3 + 7.3]
    assert res["attained"] == [1] and res["server"] == [0]
    assert res["end_ms"] == 24 and res["cost_ms"] == 23.0 and res["scale_ups"] == 1 and res["scale_downs"] == 0


def test_token_i_is_due_at_ttft_plus_i_tpot():
    # T = 1 + kv/100 ms: a 1000-token prompt (prefill 0 -> 11) decodes back to back at 11 + 0.01 i ms for token i, which
    # the average-length prediction (10 tokens) did not foresee: token i comes at 11 + 11 i + 0.005 i (i + 1) and is due at
    # 1000 + 20 i, so the first late one is the smallest i with 0.005 i^2 - 8.995 i - 989 > 0
    prof = policy.Profile([1, 4096], [0, 10 ** 6], [[1.0, 1.0 + 10 ** 4]] * 2)
    first_late = math.floor((8.995 + math.sqrt(8.995 ** 2 + 4 * 0.005 * 989)) / 0.01) + 1
    assert first_late == 1903            # the positive root is 1902.9
    for output, ok in ((first_late, 1), (first_late + 1, 0)):     # tokens 0 .. output - 1
        res = run(prof, [(0.0, 1000, output, 1000.0, 0)], [20.0], 1, 10)
        assert res["attained"] == [ok]
        i = output - 1
        assert res["finish_ms"][0] == pytest.approx(11 + 11 * i + 0.005 * i * (i + 1), rel=1e-9)


def test_scale_down_returns_the_empty_instance_and_cost_counts_time_outside_the_pool():
    # as above with one output token: done at step 9; the check at step 30 returns the instance (out of the pool 1..30);
    # the second request takes it again at step 100, first token at 107.3, seen at step 108, run ends at 109
    res = run(table(lambda b, k: 7.3), [(0.4, 100, 1, 300.0, 0), (100.0, 50, 1, 300.0, 0)], [20.0], 1, 3, period=10)
    assert res["first_token_ms"] == [8.3, 107.3] and res["finish_ms"] == [8.3, 107.3]
    assert res["scale_ups"] == 2 and res["scale_downs"] == 1
    assert res["end_ms"] == 109 and res["cost_ms"] == (10 - 1) + (109 - 100)


def test_deadlines_follow_the_token_index_when_the_output_outgrows_the_prediction():
    # the same request, checked token by token with a plain loop: iterations chained end to start
    prof = policy.Profile([1, 4096], [0, 10 ** 6], [[1.0, 1.0 + 10 ** 4]] * 2)

    def expect(output):
        t = 0 + prof.lookup(1000, 1000)           # prefill starts at step 0
        late = t > 1000.0
        for i in range(1, output):
            t = t + prof.lookup(1, 1000 + i)
            late = late or t > 1000.0 + 20.0 * i
        return t, late

    for output, want_late in ((1000, False), (4000, True)):
        res = run(prof, [(0.0, 1000, output, 1000.0, 0)], [20.0], 1, 10)
        t, late = expect(output)
        assert late == want_late
        assert res["finish_ms"] == [t] and res["attained"] == [int(not late)]


def test_highest_load_first_fills_an_instance_to_the_bound_of_the_admission_formula():
    # T(B) = B ms, TPOT 20: an instance with n decodes admits one more while T(n + 1) < 20, i.e. holds 19
    prof = table(lambda b, k: float(b), bs=(1, 4096))
    reqs = [(30.0 * i, 1, 2000, 300.0, 0) for i in range(25)]
    res = run(prof, reqs, [20.0], 3, 2000, max_steps=800)
    assert res["server"] == [0] * 19 + [1] * 6
    assert res["scale_ups"] == 2 and res["promotions"] == 0


def test_among_instances_with_room_the_highest_load_one_is_taken():
    # as above, but the first request ends after 150 tokens (before step 3000): at step 5000 instance 0 holds 18
    # requests and instance 1 holds 6, both have room, and the new request goes to instance 0
    prof = table(lambda b, k: float(b), bs=(1, 4096))
    reqs = [(30.0 * i, 1, 150 if i == 0 else 10 ** 5, 300.0, 0) for i in range(25)] + [(5000.0, 1, 5, 300.0, 0)]
    res = run(prof, reqs, [20.0], 3, 2000, max_steps=5010)
    assert res["finish_ms"][0] < 3000 and res["server"] == [0] * 19 + [1] * 6 + [0]


def test_admission_looks_at_the_largest_future_kv_size():
    # T = kv / 1000 ms, TPOT 18, prompts of 1000 tokens predicted to grow by 3000: four requests peak below 16 000
    # KV tokens, five above 19 000, so the fifth request opens the next instance although the iteration it would join
    # now takes 5 ms
    prof = policy.Profile([1, 4096], [0, 10 ** 6], [[0.0, 1000.0]] * 2)
    reqs = [(50.0 * i, 1000, 10 ** 5, 300.0, 0) for i in range(9)]
    res = run(prof, reqs, [18.0], 3, 3000, max_steps=500)
    assert res["server"] == [0] * 4 + [1] * 4 + [2]


def test_admission_respects_the_kv_capacity():
    # constant iterations; every request is predicted to end at 1000 + 100 KV tokens: four fit below 5000, five do not
    reqs = [(50.0 * i, 1000, 10 ** 5, 300.0, 0) for i in range(6)]
    res = run(table(lambda b, k: 7.3), reqs, [20.0], 2, 100, cap=5000, max_steps=400)
    assert res["server"] == [0] * 4 + [1] * 2


def test_lazy_promotion_only_when_the_own_cluster_is_full_and_before_scaling_up():
    # tiers 20 / 50 ms, T(B) = B.  The tier-0 request opens instance 0; the first tier-1 request finds no cluster of
    # its own and no room rule against it on instance 0 (T(2) < 20): it is promoted there rather than opening instance 1.
    prof = table(lambda b, k: float(b), bs=(1, 4096))
    reqs = [(0.0, 1, 2000, 300.0, 0), (40.0, 1, 2000, 300.0, 1)]
    res = run(prof, reqs, [20.0, 50.0], 2, 2000, max_steps=100)
    assert res["server"] == [0, 0] and res["promotions"] == 1 and res["scale_ups"] == 1
    # Instance 0 full for tier 0 (19 requests): a tier-1 request cannot be promoted and opens instance 1 for tier 1;
    # later tier-1 requests go to their own cluster, not to tier 0's
    reqs = [(30.0 * i, 1, 2000, 300.0, 0) for i in range(19)] + [(600.0, 1, 2000, 300.0, 1), (700.0, 1, 2000, 300.0, 1)]
    res = run(prof, reqs, [20.0, 50.0], 2, 2000, max_steps=800)
    assert res["server"] == [0] * 19 + [1, 1] and res["promotions"] == 0 and res["scale_ups"] == 2


def test_promoted_request_keeps_its_own_tpot_in_its_deadlines():
    # tiers 20 / 50 ms, T = 1 + kv/100.  r1 (tier 1) is promoted onto r0's tier-0 instance once r0's prefill (0 -> 11) is
    # over.  With both decoding, an iteration takes about 12 + 0.02 g ms after g tokens: slower than 20 ms from g = 400
    # on, which makes r0 late, but r1's 2500 tokens stay ahead of 1005 + 50 i (they would not stay ahead of 1005 + 20 i)
    prof = policy.Profile([1, 4096], [0, 10 ** 6], [[1.0, 1.0 + 10 ** 4]] * 2)
    reqs = [(0.0, 1000, 3000, 1000.0, 0), (5.0, 100, 2500, 1000.0, 1)]
    res = run(prof, reqs, [20.0, 50.0], 1, 10)
    assert res["server"] == [0, 0] and res["promotions"] == 1
    assert res["attained"] == [0, 1]
    i = 2499
    assert res["finish_ms"][1] > 1005 + 20 * i and res["finish_ms"][1] < 1005 + 50 * i


def test_wait_for_the_iteration_in_flight_counts_against_the_first_token_deadline():
    # 50 ms iterations; at step 60 instance 0 is inside the iteration 50 -> 100: a request with 80 ms to its first token
    # would wait 40 ms and prefill for 50, so it goes to a fresh instance instead
    reqs = [(0.0, 10, 100, 1000.0, 0), (60.0, 10, 2, 80.0, 0)]
    res = run(table(lambda b, k: 50.0), reqs, [100.0], 2, 100, max_steps=200)
    assert res["server"] == [0, 1] and res["first_token_ms"][1] == 110.0


def test_time_already_spent_queueing_counts_against_the_first_token_deadline():
    # one instance, 50 ms iterations; r1 arrives at 1 while r0's prefill runs and can only be looked at again at step 50:
    # with TTFT 120 it still makes it (first token at 100 <= 121), with TTFT 90 it cannot any more and is dropped
    for ttft, served in ((120.0, True), (90.0, False)):
        res = run(table(lambda b, k: 50.0), [(0.0, 10, 1, 1000.0, 0), (1.0, 10, 1, ttft, 0)], [100.0], 1, 1)
        assert (res["server"][1], res["dropped"], res["attained"][1]) == ((0, 0, 1) if served else (-1, 1, 0))
        assert res["first_token_ms"][1] == (100.0 if served else -1.0)


def test_later_chunks_attend_the_prompt_prefix():
    # T = tokens/100 + kv/10000: a 3000-token prompt on an empty instance keeps the largest chunk with T < 20, 1980 tokens
    # (19.998 ms; the second iteration, 1020 tokens attending all 3000, takes 10.5 ms), back to back
    prof = policy.Profile([0, 4096], [0, 10 ** 6], [[0.0, 100.0], [40.96, 140.96]])
    res = run(prof, [(0.0, 3000, 1, 300.0, 0)], [20.0], 1, 1)
    assert prof.lookup(1980, 1980) < 20.0 <= prof.lookup(1981, 1981)
    assert res["first_token_ms"] == [prof.lookup(1980, 1980) + prof.lookup(1020, 3000)]


def test_pending_instance_joins_the_tier_of_its_requests():
    # r0 (tier 0, 3 tokens) opens instance 0; r1 (tier 1, long) is promoted onto it; r0 finishes; the check at step 50
    # finds no tier-0 request on the instance and parks it; r2 (tier 1) at step 60 cannot use a parked instance as a
    # tighter cluster, asks to scale up, and gets the parked instance, which joins tier 1; instance 1 is never used
    prof = table(lambda b, k: float(b), bs=(1, 4096))
    reqs = [(0.0, 1, 3, 300.0, 0), (5.0, 1, 2000, 300.0, 1), (60.0, 1, 2000, 300.0, 1)]
    res = run(prof, reqs, [20.0, 50.0], 2, 2000, period=50, max_steps=200)
    assert res["server"] == [0, 0, 0]
    assert res["promotions"] == 1 and res["scale_ups"] == 2 and res["scale_downs"] == 0
    assert res["cost_ms"] == 200.0  # one instance outside the pool from step 0 to the end


def test_request_that_cannot_make_its_first_token_any_more_is_dropped():
    # one instance, 60 ms prefills, TTFT 100: the second request would wait 60 ms and need 60 more
    prof = table(lambda b, k: 60.0 if b > 1 else 5.0, bs=(1, 2, 4096))
    res = run(prof, [(0.0, 500, 2, 100.0, 0), (1.0, 500, 2, 100.0, 0)], [100.0], 1, 2)
    assert res["attained"] == [1, 0] and res["dropped"] == 1 and res["server"] == [0, -1]
    assert res["first_token_ms"][1] == -1.0


def _random_trace(seed, n, rate_per_ms, max_prompt, max_output):
    return W.sim_trace(seed, n, rate_per_ms, max_prompt, max_output)


def test_invariants_on_random_traces():
    prof = table(lambda b, k: 4.0 + 0.012 * b + 2e-5 * k, bs=(1, 16, 64, 256, 1024, 4096), ks=(16, 4096, 65536, 1048576))
    tpots = [20.0, 30.0, 50.0, 100.0]
    drops = []
    for seed, n_servers, rate in ((0, 4, 0.03), (1, 2, 0.5), (2, 8, 0.06)):
        tr = _random_trace(seed, 250, rate, 1024, 256)
        res = sim.simulate(prof, tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, n_servers, 128, 2 * 10 ** 6, 200)
        served = 0
        for i in range(250):
            a, ft, fin = tr["arrival"][i], res["first_token_ms"][i], res["finish_ms"][i]
            if res["server"][i] < 0:
                assert res["attained"][i] == 0 and ft == -1.0 and fin == -1.0
                continue
            served += 1
            assert a < ft <= fin
            # an iteration takes at least the table's smallest value; tokens come one per iteration
            assert fin - ft >= (tr["output"][i] - 1) * 4.0
            if res["attained"][i]:
                assert ft <= a + tr["ttft"][i] and fin <= a + tr["ttft"][i] + (tr["output"][i] - 1) * tpots[tr["tier"][i]]
        assert served + res["dropped"] == 250
        assert 0 < res["cost_ms"] <= n_servers * res["end_ms"]
        assert res["scale_downs"] <= res["scale_ups"] <= res["scale_downs"] + n_servers
        drops.append(res["dropped"])
    # the overloaded two-instance run exercises the drop path, the roomy ones do not
    assert drops[0] == 0 and drops[1] > 0 and drops[2] == 0, drops
