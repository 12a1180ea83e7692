"""Cluster simulator for the paper's policy on co-located (chunked-prefill) instances
(test infrastructure; plain and slow on purpose).

What is simulated (Sec. 5.1): serving instances whose iteration times come from the
(batch size, KV cache size) -> time table, advanced in 1 ms steps, under the router of Sec. 4:
one cluster of instances per TPOT tier (4.2 request binning), requests sent to the highest-load
instance that still meets the SLO so that a load gradient forms (4.3), looser-tier requests
allowed onto tighter-tier instances only when their own cluster is full (4.4 lazy promotion),
instances taken from and returned to a shared idle pool (4.3), the admission test by simulated
future KV size (4.5) and by the chunk size that can be kept for the whole prefill with the wait
for the instance's current iteration included (4.6, 4.7), and the deadline-based SLO of Sec. 2.3:
token i of a request (i = 0 the first token) is due at arrival + TTFT + i * TPOT.

Readings fixed where the text is loose:
  * time advances in whole milliseconds; in each step, in this order: (A) iterations whose end time
    has been reached deliver their tokens at that (fractional) end time, (B) requests that have
    arrived join the queue of their tier, (C) every `check_period` steps the scale-down check runs,
    (D) the queues are served, tightest tier first, first come first served, stopping at the first
    request of a queue that cannot be placed but could still make its first-token deadline on an
    empty instance (one that no longer could is dropped: it counts as not attained and is never
    served), (E) every instance that is not inside an iteration
    and has requests starts one: at the end time of its previous iteration if that ended within this
    step (iterations run back to back; only the router works on the 1 ms grid), else at the step;
  * an iteration holds one token of every request in decode and the next chunk of the one request
    in prefill (an instance takes a new request only while no prefill is in progress on it); its
    duration is the table's value for (tokens, sum of KV sizes attended): a decode attends its KV
    length plus the new token, the chunk attends the prompt tokens up to its own end;
  * the prefill's last chunk produces token 0; a request with output length d then takes d - 1
    decode iterations; its KV length after prefill is the prompt length;
  * "load" of an instance = number of requests on it; candidates are tried from the highest load
    down (ties: the instance that joined the cluster first);
  * placement order: own cluster, then the clusters of tighter tiers from the nearest one (lazy
    promotion; the instance's own, tighter, TPOT bounds its iterations), then scale-up (a pending
    instance holding requests of this tier first, then the idle pool), else the request stays queued;
  * an instance admits a request if (a) the chunked-prefill prediction admits it against the
    instance's TPOT and the time left to the request's first-token deadline, (b) the iteration time
    predicted for the largest future KV size with the request added stays below the instance's TPOT,
    (c) that KV size stays below the capacity;
  * scale-down check, per cluster: its lowest-load instance (ties: joined last) goes back to the
    idle pool if it is empty, and into the pending state if none of its requests belongs to the
    cluster's tier; a pending instance takes no requests, joins the tier of its tightest request
    when that tier scales up, and goes to the idle pool once empty (checked at every step);
  * cost = time instances spend outside the idle pool (Sec. 5.4: instances x seconds).
"""
import math

from . import policy


class Request:
    __slots__ = ("arrival", "prompt", "output", "ttft", "tier", "server", "chunk", "prefilled", "generated",
                 "kv_len", "violated", "first_token", "finish", "phase")

    def __init__(self, arrival, prompt, output, ttft, tier):
        self.arrival, self.prompt, self.output, self.ttft, self.tier = float(arrival), int(prompt), int(output), float(ttft), int(tier)
        self.server, self.chunk, self.prefilled, self.generated, self.kv_len = -1, 0, 0, 0, 0
        self.violated, self.first_token, self.finish = False, -1.0, -1.0
        self.phase = 0  # 0 not arrived / queued, 1 prefill, 2 decode, 3 done


POOL, ACTIVE, PENDING = 0, 1, 2


class Server:
    def __init__(self, sid):
        self.sid, self.state, self.tier, self.joined = sid, POOL, -1, -1
        self.reqs = []          # request indices in admission order
        self.busy_until = None  # end time of the iteration in flight
        self.free_at = None     # end time of an iteration that ended in the current step
        self.batch = []         # (request index, tokens) of the iteration in flight
        self.since = 0.0        # when it last left the idle pool


def simulate(profile, arrival, prompt, output, ttft, tier, tpots, n_servers, avg_decode, kv_capacity, check_period=1000,
             max_steps=10 ** 9):
    """Returns a dict: per-request lists `attained`, `first_token_ms`, `finish_ms`, `server`; `end_ms`;
    `cost_ms` (instance-milliseconds outside the idle pool); `scale_ups`, `scale_downs`, `promotions`, `dropped`."""
    n = len(arrival)
    reqs = [Request(arrival[i], prompt[i], output[i], ttft[i], tier[i]) for i in range(n)]
    assert all(r.prompt >= 1 and r.output >= 1 and 0 <= r.tier < len(tpots) for r in reqs)
    assert all(x <= y for x, y in zip(arrival, arrival[1:])), "arrivals must be sorted"
    servers = [Server(s) for s in range(n_servers)]
    queues = [[] for _ in tpots]
    first_server = [-1] * n
    stats = {"scale_ups": 0, "scale_downs": 0, "promotions": 0, "dropped": 0}
    cost = 0.0
    join_counter = 0
    next_arrival = 0
    done = 0

    def running_decodes(s):
        return [(reqs[i].kv_len, reqs[i].generated) for i in s.reqs if reqs[i].phase == 2]

    def admits(s, r, now):
        if any(reqs[i].phase == 1 for i in s.reqs):
            return 0
        run = running_decodes(s)
        tpot = tpots[s.tier]
        wait = max(0.0, s.busy_until - now) if s.busy_until is not None else 0.0
        ok, chunk, _, _ = policy.predict_chunked_prefill(profile, run, r.prompt, avg_decode, tpot, r.arrival + r.ttft - now, wait)
        if not ok:
            return 0
        ok2, _, kv = policy.predict_admit(profile, run, r.prompt, avg_decode, tpot, 0.0)
        if not ok2 or not kv < kv_capacity:
            return 0
        return chunk

    def by_load(cands):
        return sorted(cands, key=lambda s: (-len(s.reqs), s.joined))

    def place(ri, now):
        nonlocal join_counter
        r = reqs[ri]
        for t in range(r.tier, -1, -1):  # own cluster, then tighter ones
            for s in by_load([s for s in servers if s.state == ACTIVE and s.tier == t]):
                c = admits(s, r, now)
                if c:
                    if t != r.tier:
                        stats["promotions"] += 1
                    return s, c
        # scale up: a pending instance whose tightest request is of this tier, else the idle pool
        cand = [s for s in servers if s.state == PENDING and min(reqs[i].tier for i in s.reqs) == r.tier]
        cand = by_load(cand) + [s for s in servers if s.state == POOL]
        for s in cand:
            was = s.state
            s_tier, s_state = s.tier, s.state
            s.tier, s.state = r.tier, ACTIVE
            c = admits(s, r, now)
            if c:
                if was == POOL:
                    s.since = now
                s.joined = join_counter
                join_counter += 1
                stats["scale_ups"] += 1
                return s, c
            s.tier, s.state = s_tier, s_state
            if was == POOL:
                break  # every idle instance gives the same answer
        return None, 0

    def to_pool(s, now):
        nonlocal cost
        cost += now - s.since
        s.state, s.tier, s.joined = POOL, -1, -1
        stats["scale_downs"] += 1

    now = 0
    while done < n and now < max_steps:
        # (A) iterations that have ended
        for s in servers:
            if s.busy_until is not None and s.busy_until <= now:
                t_end = s.busy_until
                for ri, tok in s.batch:
                    r = reqs[ri]
                    if r.phase == 1:
                        r.prefilled += tok
                        if r.prefilled < r.prompt:
                            continue
                        r.phase, r.kv_len, r.generated, r.first_token = 2, r.prompt, 1, t_end
                    else:
                        r.kv_len += 1
                        r.generated += 1
                    if t_end > r.arrival + r.ttft + (r.generated - 1) * tpots[r.tier]:
                        r.violated = True
                    if r.generated == r.output:
                        r.phase, r.finish = 3, t_end
                        s.reqs.remove(ri)
                        done += 1
                s.busy_until, s.batch, s.free_at = None, [], t_end
        for s in servers:
            if s.state == PENDING and not s.reqs:
                to_pool(s, now)
        # (B) arrivals
        while next_arrival < n and reqs[next_arrival].arrival <= now:
            queues[reqs[next_arrival].tier].append(next_arrival)
            next_arrival += 1
        # (C) scale-down check
        if now % check_period == 0:
            for t in range(len(tpots)):
                cl = [s for s in servers if s.state == ACTIVE and s.tier == t]
                if not cl:
                    continue
                last = sorted(cl, key=lambda s: (len(s.reqs), -s.joined))[0]
                if not last.reqs:
                    to_pool(last, now)
                elif all(reqs[i].tier != t for i in last.reqs):
                    last.state = PENDING
        # (D) routing
        for q in queues:
            while q:
                s, c = place(q[0], now)
                if s is None:
                    r = reqs[q[0]]
                    if policy.predict_chunked_prefill(profile, [], r.prompt, avg_decode, tpots[r.tier], r.arrival + r.ttft - now, 0.0)[0]:
                        break
                    q.pop(0)
                    r.phase, r.violated = 3, True
                    stats["dropped"] += 1
                    done += 1
                    continue
                ri = q.pop(0)
                r = reqs[ri]
                r.server, r.chunk, r.phase = s.sid, c, 1
                first_server[ri] = s.sid
                s.reqs.append(ri)
        # (E) start iterations
        for s in servers:
            if s.busy_until is None and s.reqs:
                tokens, kv, batch = 0, 0, []
                for ri in s.reqs:
                    r = reqs[ri]
                    if r.phase == 2:
                        batch.append((ri, 1))
                        tokens += 1
                        kv += r.kv_len + 1
                    else:
                        c = min(r.chunk, r.prompt - r.prefilled)
                        batch.append((ri, c))
                        tokens += c
                        kv += r.prefilled + c
                s.batch = batch
                s.busy_until = (s.free_at if s.free_at is not None else now) + profile.lookup(tokens, kv)
        for s in servers:
            s.free_at = None
        now += 1
    for s in servers:
        if s.state != POOL:
            cost += now - s.since
    return {
        "attained": [int(r.phase == 3 and not r.violated) for r in reqs],
        "first_token_ms": [r.first_token for r in reqs],
        "finish_ms": [r.finish for r in reqs],
        "server": first_server,
        "end_ms": now,
        "cost_ms": cost,
        **stats,
    }
