"""Pins of the prefill-decode disaggregated simulator's oracle: hand-computed timelines for dynamic chunking
(Sec. 4.7), deadline order of the prefill queue (Sec. 4.2), load-based choice of the prefill instance, the
wait-time-aware decode admission (Sec. 4.6), the hand-over, and invariants on random traces."""
import numpy as np

from oracle import policy, sim_pd
from paper_2507_17769_amd import workloads as W


def table(fn, bs=(1, 64, 4096), ks=(1, 65536, 10 ** 7)):
    return policy.Profile(bs, ks, [[fn(b, k) for k in ks] for b in bs])


def run(prof, reqs, tpots, n_servers, avg, budget, period=1000, cap=10 ** 12, max_steps=10 ** 9):
    a, p, o, t, tier = (list(c) for c in zip(*reqs))
    return sim_pd.simulate(prof, a, p, o, t, tier, tpots, n_servers, avg, cap, budget, period, max_steps)


def test_dynamic_chunking_timeline_and_hand_over_by_hand():
    # the paper's example: 2050 tokens, budget 1024 -> iterations of 1024 and 1026 tokens (not three).  10.5 ms
    # iterations back to back: prefill 0 -> 10.5 -> 21 (first token); the decode side sees the request at step 21, takes
    # an instance from the pool, decodes 21 -> 31.5, noticed at step 32; the run ends after it
    res = run(table(lambda b, k: 10.5), [(0.0, 2050, 2, 300.0, 0)], [20.0], 2, 2, 1024)
    assert res["first_token_ms"] == [21.0] and res["finish_ms"] == [31.5] and res["attained"] == [1]
    assert res["prefill_server"] == [0] and res["decode_server"] == [1]
    assert res["end_ms"] == 33 and res["cost_ms"] == 33.0 + (33 - 21) and res["scale_ups"] == 2


def test_prefill_prediction_plans_with_dynamic_chunking():
    # same request with 25 ms to its first token: two iterations (21 ms) are predicted and it is admitted; three
    # iterations of plain chunking (31.5 ms) would not fit
    res = run(table(lambda b, k: 10.5), [(0.0, 2050, 1, 25.0, 0)], [20.0], 1, 1, 1024)
    assert res["first_token_ms"] == [21.0] and res["attained"] == [1] and res["dropped"] == 0


def test_later_chunks_attend_the_prompt_prefix():
    # T = tokens/100 + kv/10000; 3000 tokens with budget 1024: 1024 tokens, then the remaining 1976 (< 2 x 1024) at once,
    # attending all 3000, back to back
    prof = policy.Profile([0, 4096], [0, 10 ** 6], [[0.0, 100.0], [40.96, 140.96]])
    res = run(prof, [(0.0, 3000, 1, 300.0, 0)], [50.0], 1, 1, 1024)
    assert res["first_token_ms"] == [prof.lookup(1024, 1024) + prof.lookup(1976, 3000)]


def test_decode_admission_respects_the_kv_capacity():
    # every request is predicted to end near 1000 + 100 KV tokens: four fit below 5000 on a decode instance, five do not
    reqs = [(50.0 * i, 1000, 10 ** 5, 300.0, 0) for i in range(6)]
    res = run(table(lambda b, k: 7.3), reqs, [20.0], 4, 100, 2048, cap=5000, max_steps=400)
    assert res["prefill_server"] == [0] * 6 and res["decode_server"] == [1] * 4 + [2] * 2


def test_decode_iterations_attend_the_prompt_plus_the_generated_tokens():
    # T = kv / 100 ms: prefill of 1000 tokens 0 -> 10; the decode instance starts at step 10 and attends 1001, then 1002
    # tokens: 10 -> 20.01 -> 30.03
    prof = policy.Profile([1, 4096], [0, 10 ** 6], [[0.0, 10.0 ** 4]] * 2)
    res = run(prof, [(0.0, 1000, 3, 300.0, 0)], [20.0], 2, 3, 2048)
    assert res["first_token_ms"] == [10.0] and res["finish_ms"] == [10 + prof.lookup(1, 1001) + prof.lookup(1, 1002)]
    assert 30.02 < res["finish_ms"][0] < 30.04


def test_token_i_is_due_at_ttft_plus_i_tpot():
    # T = 1 + kv/100 ms: prefill of 1000 tokens 0 -> 11, decode from step 11 at 11 + 0.01 i ms for token i (the prediction
    # assumed 10 tokens): token i comes at 11 + 11 i + 0.005 i (i + 1), is due at 1000 + 20 i, first late one: i = 1903
    prof = policy.Profile([1, 4096], [0, 10 ** 6], [[1.0, 1.0 + 10 ** 4]] * 2)
    for output, ok in ((1903, 1), (1904, 0)):     # tokens 0 .. output - 1
        res = run(prof, [(0.0, 1000, output, 1000.0, 0)], [20.0], 2, 10, 2048)
        i = output - 1
        assert res["attained"] == [ok] and abs(res["finish_ms"][0] - (11 + 11 * i + 0.005 * i * (i + 1))) < 1e-6


def test_prefill_queue_is_served_in_deadline_order():
    # both requests are seen at step 1; the one that arrived later has the nearer first-token deadline and is
    # prefilled first (one 2048-token request per iteration, 50 ms each)
    reqs = [(0.2, 2048, 1, 1000.0, 0), (0.5, 2048, 1, 300.0, 0)]
    res = run(table(lambda b, k: 50.0), reqs, [100.0], 1, 1, 2048)
    assert res["prefill_server"] == [0, 0]
    assert res["first_token_ms"] == [101.0, 51.0]


def test_prefill_goes_to_the_most_loaded_instance_that_still_meets_the_deadline():
    # 50 ms per 2048-token iteration.  r1 (TTFT 300) can wait behind r0 on instance 0; r2 (TTFT 120) cannot wait for both
    # (48 + 50 + 50 > 118) and opens instance 1; r3 (TTFT 1000) fits on both and takes the one with more queued tokens
    reqs = [(0.0, 2048, 1, 300.0, 0), (1.0, 2048, 1, 300.0, 0), (2.0, 2048, 1, 120.0, 0), (3.0, 2048, 1, 1000.0, 0)]
    res = run(table(lambda b, k: 50.0), reqs, [100.0], 3, 1, 2048)
    assert res["prefill_server"] == [0, 0, 1, 0]
    assert res["first_token_ms"] == [50.0, 100.0, 52.0, 150.0]


def test_a_request_joins_only_if_those_already_queued_still_make_their_deadlines():
    # T = tokens / 100 ms, budget 1024.  r0 (1024 tokens) runs 0 -> 10.24; ra (600 tokens, 17 ms to its first token) is
    # queued behind it at step 1: 9.24 + 6 = 15.24 ms, in time.  rb (300 tokens) at step 2 would share ra's iteration
    # (900 tokens, 9 ms) and push ra's first token to 19.24, past its deadline at 18: rb takes a fresh instance instead
    prof = policy.Profile([0, 4096], [1, 10 ** 7], [[0.0, 0.0], [40.96, 40.96]])
    reqs = [(0.0, 1024, 1, 300.0, 0), (1.0, 600, 1, 17.0, 0), (2.0, 300, 1, 300.0, 0)]
    res = run(prof, reqs, [100.0], 2, 1, 1024)
    assert res["prefill_server"] == [0, 0, 1]
    assert res["first_token_ms"] == [prof.lookup(1024, 1), prof.lookup(1024, 1) + prof.lookup(600, 1), 2 + prof.lookup(300, 1)]
    assert res["attained"] == [1, 1, 1]


def test_decode_admission_counts_the_wait_for_the_iteration_in_flight():
    # decode iterations 18 ms, prefill iterations 25 ms, TPOT 20.  r0 decodes on instance 1 in cycles 25 -> 43 -> 61 ...
    # r1's first token comes at 55 with its second due at 30 + TTFT + 20.  With TTFT 26 there are 21 ms left: waiting
    # 6 ms for instance 1's cycle and 18 ms of iteration is too late, so a fresh instance is taken; with TTFT 40 (35 ms
    # left) the request joins instance 1
    prof = policy.Profile([1, 8, 64, 4096], [1, 10 ** 7], [[18.0] * 2, [18.0] * 2, [25.0] * 2, [25.0] * 2])
    for ttft, want in ((26.0, 2), (40.0, 1)):
        reqs = [(0.0, 100, 1000, 1000.0, 0), (30.0, 100, 5, ttft, 0)]
        res = run(prof, reqs, [20.0], 3, 1000, 2048, max_steps=200)
        assert res["first_token_ms"][:2] == [25.0, 55.0]
        assert res["prefill_server"] == [0, 0] and res["decode_server"] == [1, want]


def test_scale_down_of_both_kinds_of_instance():
    # one request; at the check of step 50 the prefill instance (idle since 10.5) and the decode instance (idle since
    # 21.5) go back to the pool; a second request at step 100 takes instance 0 again for its prefill
    res = run(table(lambda b, k: 10.5), [(0.0, 100, 2, 300.0, 0), (100.0, 100, 1, 300.0, 0)], [20.0], 2, 2, 1024, period=50)
    assert res["scale_ups"] == 3 and res["scale_downs"] == 2
    assert res["prefill_server"] == [0, 0] and res["decode_server"] == [1, -1]
    assert res["finish_ms"] == [11 + 10.5, 110.5] and res["end_ms"] == 112
    assert res["cost_ms"] == 50.0 + (50 - 11) + (112 - 100)


def test_request_without_a_chance_is_dropped_before_and_after_prefill():
    # before prefill: one instance, 60 ms prefills, TTFT 100: the second request would wait 59 ms and need 60 more
    prof = table(lambda b, k: 60.0 if b > 1 else 5.0, bs=(1, 2, 4096))
    res = run(prof, [(0.0, 500, 1, 100.0, 0), (1.0, 500, 1, 100.0, 0)], [100.0], 1, 1, 2048)
    assert res["attained"] == [1, 0] and res["dropped"] == 1 and res["prefill_server"] == [0, -1]
    # after prefill: a single instance does the prefill and there is none for decoding: the request keeps its place while
    # an empty instance could still deliver its second token (due at 0 + 20 + 10), then is dropped: first token but no end
    res = run(table(lambda b, k: 5.0), [(0.0, 100, 3, 20.0, 0)], [10.0], 1, 3, 2048, period=10 ** 6)
    assert res["first_token_ms"] == [5.0] and res["finish_ms"] == [-1.0] and res["dropped"] == 1 and res["attained"] == [0]
    assert res["end_ms"] == 26  # dropped at step 25: 5 ms of iteration are no longer strictly less than the 5 ms left


def test_invariants_on_random_traces():
    prof = table(lambda b, k: 4.0 + 0.012 * b + 2e-5 * k, bs=(1, 16, 64, 256, 1024, 4096), ks=(16, 4096, 65536, 1048576))
    tpots = list(W.SIM_TPOTS_MS)
    drops = []
    for seed, n_servers, rate in ((0, 4, 0.03), (1, 3, 0.5), (2, 8, 0.06)):
        tr = W.sim_trace(seed, 250, rate, 1024, 256)
        res = sim_pd.simulate(prof, tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, n_servers, 128, 2 * 10 ** 6, 1024, 200)
        finished = 0
        for i in range(250):
            a, ft, fin = tr["arrival"][i], res["first_token_ms"][i], res["finish_ms"][i]
            if fin < 0:
                assert res["attained"][i] == 0
                assert (ft < 0) == (res["prefill_server"][i] < 0) and res["decode_server"][i] < 0
                continue
            finished += 1
            assert a < ft <= fin and res["prefill_server"][i] >= 0
            assert (res["decode_server"][i] >= 0) == (tr["output"][i] > 1)
            assert res["decode_server"][i] != res["prefill_server"][i]
            assert fin - ft >= (tr["output"][i] - 1) * 4.0
            if res["attained"][i]:
                assert ft <= a + tr["ttft"][i] and fin <= a + tr["ttft"][i] + (tr["output"][i] - 1) * tpots[tr["tier"][i]]
        assert finished + res["dropped"] == 250
        assert 0 < res["cost_ms"] <= n_servers * res["end_ms"]
        drops.append(res["dropped"])
    assert drops[0] == 0 and drops[1] > 0 and drops[2] == 0, drops
