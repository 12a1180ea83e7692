"""Cluster simulator for the paper's policy on prefill-decode disaggregated instances
(test infrastructure; plain and slow on purpose).  The co-located variant is in sim.py; the clock,
the deadline-based SLO (Sec. 2.3), the decode clusters per TPOT tier with highest-load-first
placement, lazy promotion, idle pool and parking (Sec. 4.2-4.4) are the same here.  What differs:

  * prefill runs on a cluster of its own that serves all tiers; queued requests are taken in order
    of their first-token deadline, arrival + TTFT (Sec. 4.2); a prefill instance forms its
    iterations by dynamic chunking with a token budget (Sec. 4.7: a request whose remaining length
    is below twice the budget is finished at once and closes the iteration); a request goes to the
    prefill instance with most queued prompt tokens that is still predicted to deliver its first
    token in time, counting the iterations of the requests already there and the wait for the one
    in flight (Sec. 4.7), else to a new instance from the idle pool;
  * when its prefill ends the request has its first token and its KV cache and queues for a decode
    instance of its tier (the transfer itself takes no time here: the paper gives none);
  * a decode instance admits it if the iteration time predicted for the largest future KV size
    stays below the instance's TPOT, that KV size is below the capacity (Sec. 4.5), and the wait for
    the iteration in flight plus that iteration time still meets the deadline of the request's
    second token, arrival + TTFT + TPOT (Sec. 4.6).

Readings fixed where the text is loose (beyond those of sim.py):
  * step order: ended iterations, arrivals, scale-down check, decode queues (tightest first, first
    come first served), prefill queue (nearest deadline first), iteration starts;
  * a chunk attends the prompt tokens up to its own end; an iteration's duration is the table's
    value for (tokens in it, KV tokens attended);
  * a request joins a prefill instance only if the requests already queued there still get their
    first tokens in time with it in the plan (dynamic chunking lets a later request share the
    iteration of an earlier one's last chunk and so lengthens it);
  * load of a prefill instance = prompt tokens not yet processed on it; the scale-down check returns
    the prefill instance with the lowest load to the pool if it holds no request;
  * a queued request that could no longer meet its next deadline even on an empty instance is
    dropped (before prefill: the first token; between prefill and decode: the second token).
"""
from . import policy

POOL, ACTIVE, PENDING = 0, 1, 2
PREFILL_CLUSTER = -2


class Request:
    def __init__(self, arrival, prompt, output, ttft, tier):
        self.arrival, self.prompt, self.output, self.ttft, self.tier = float(arrival), int(prompt), int(output), float(ttft), int(tier)
        self.prefilled, self.generated, self.kv_len = 0, 0, 0
        self.violated, self.first_token, self.finish = False, -1.0, -1.0
        self.phase = 0  # 0 queued for prefill, 1 in prefill, 4 queued for decode, 2 in decode, 3 done
        self.prefill_server, self.decode_server = -1, -1


class Server:
    def __init__(self, sid):
        self.sid, self.state, self.tier, self.joined = sid, POOL, -1, -1
        self.reqs, self.busy_until, self.batch, self.since, self.free_at = [], None, [], 0.0, None


def simulate(profile, arrival, prompt, output, ttft, tier, tpots, n_servers, avg_decode, kv_capacity, prefill_budget,
             check_period=1000, max_steps=10 ** 9):
    """Returns a dict: per-request lists `attained`, `first_token_ms`, `finish_ms`, `prefill_server`, `decode_server`;
    `end_ms`, `cost_ms`, `scale_ups`, `scale_downs`, `promotions`, `dropped`."""
    n = len(arrival)
    reqs = [Request(arrival[i], prompt[i], output[i], ttft[i], tier[i]) for i in range(n)]
    assert all(r.prompt >= 1 and r.output >= 1 and 0 <= r.tier < len(tpots) for r in reqs)
    assert all(x <= y for x, y in zip(arrival, arrival[1:])), "arrivals must be sorted"
    servers = [Server(s) for s in range(n_servers)]
    prefill_queue = []
    decode_queues = [[] for _ in tpots]
    stats = {"scale_ups": 0, "scale_downs": 0, "promotions": 0, "dropped": 0}
    cost, join_counter, next_arrival, done = 0.0, 0, 0, 0

    def wait_of(s, now):
        return max(0.0, s.busy_until - now) if s.busy_until is not None else 0.0

    def left(s, ri):
        """prompt tokens of request ri not yet processed or in the iteration in flight"""
        r = reqs[ri]
        return r.prompt - r.prefilled - sum(tok for i, tok in s.batch if i == ri)

    def prefill_load(s):
        return sum(reqs[i].prompt - reqs[i].prefilled for i in s.reqs)

    def prefill_admits(s, r, now):
        """would r, queued behind the requests already on s, get its first token in time, and would they still get theirs"""
        ids = [i for i in s.reqs if left(s, i) > 0]
        rem = [left(s, i) for i in ids] + [r.prompt]
        at = [reqs[i].prompt - left(s, i) for i in ids] + [0]
        whole = [reqs[i].prompt for i in ids] + [r.prompt]
        due = [reqs[i].arrival + reqs[i].ttft - now for i in ids] + [r.arrival + r.ttft - now]
        t = wait_of(s, now)
        for it in policy.chunk_plan(rem, prefill_budget, True, 0):
            tokens = kv = 0
            for idx, tok in it:
                at[idx] += tok
                tokens += tok
                kv += at[idx]
            t += profile.lookup(tokens, kv)
            for idx, _ in it:
                if at[idx] == whole[idx] and not t < due[idx]:
                    return False
        return True

    def decode_admits(s, r, now):
        run = [(reqs[i].kv_len, reqs[i].generated) for i in s.reqs]
        ok, t, kv = policy.predict_admit(profile, run, r.kv_len, avg_decode, tpots[s.tier], 0.0)
        return ok and kv < kv_capacity and wait_of(s, now) + t < r.arrival + r.ttft + tpots[r.tier] - now

    def by_load(cands):
        return sorted(cands, key=lambda s: (-len(s.reqs), s.joined))

    def join(s, tier, now):
        nonlocal join_counter
        if s.state == POOL:
            s.since = now
        s.state, s.tier, s.joined = ACTIVE, tier, join_counter
        join_counter += 1
        stats["scale_ups"] += 1

    def place_decode(r, now):
        for t in range(r.tier, -1, -1):
            for s in by_load([s for s in servers if s.state == ACTIVE and s.tier == t]):
                if decode_admits(s, r, now):
                    if t != r.tier:
                        stats["promotions"] += 1
                    return s
        cand = by_load([s for s in servers if s.state == PENDING and min(reqs[i].tier for i in s.reqs) == r.tier])
        for s in cand + [s for s in servers if s.state == POOL]:
            was, old_tier = s.state, s.tier
            s.tier = r.tier
            ok = decode_admits(s, r, now)
            s.tier = old_tier
            if ok:
                join(s, r.tier, now)
                return s
            if was == POOL:
                break
        return None

    def place_prefill(r, now):
        cl = [s for s in servers if s.state == ACTIVE and s.tier == PREFILL_CLUSTER]
        for s in sorted(cl, key=lambda s: (-prefill_load(s), s.joined)):
            if prefill_admits(s, r, now):
                return s
        for s in servers:
            if s.state == POOL:
                if prefill_admits(s, r, now):
                    join(s, PREFILL_CLUSTER, now)
                    return s
                break
        return None

    def to_pool(s, now):
        nonlocal cost
        cost += now - s.since
        s.state, s.tier, s.joined = POOL, -1, -1
        stats["scale_downs"] += 1

    def drop(r):
        nonlocal done
        r.phase, r.violated = 3, True
        stats["dropped"] += 1
        done += 1

    now = 0
    while done < n and now < max_steps:
        # ended iterations
        for s in servers:
            if s.busy_until is None or s.busy_until > now:
                continue
            t_end = s.busy_until
            for ri, tok in s.batch:
                r = reqs[ri]
                if r.phase == 1:
                    r.prefilled += tok
                    if r.prefilled < r.prompt:
                        continue
                    r.kv_len, r.generated, r.first_token = r.prompt, 1, t_end
                else:
                    r.kv_len += 1
                    r.generated += 1
                if t_end > r.arrival + r.ttft + (r.generated - 1) * tpots[r.tier]:
                    r.violated = True
                if r.generated == r.output:
                    s.reqs.remove(ri)
                    r.phase, r.finish = 3, t_end
                    done += 1
                elif r.phase == 1:  # prefill done: hand over to the decode side
                    s.reqs.remove(ri)
                    r.phase = 4
                    decode_queues[r.tier].append(ri)
            s.busy_until, s.batch, s.free_at = None, [], t_end
        for s in servers:
            if s.state == PENDING and not s.reqs:
                to_pool(s, now)
        # arrivals, kept in order of first-token deadline
        while next_arrival < n and reqs[next_arrival].arrival <= now:
            prefill_queue.append(next_arrival)
            next_arrival += 1
        prefill_queue.sort(key=lambda i: (reqs[i].arrival + reqs[i].ttft, i))
        # scale-down check
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
            cl = [s for s in servers if s.state == ACTIVE and s.tier == PREFILL_CLUSTER]
            if cl:
                last = sorted(cl, key=lambda s: (prefill_load(s), -s.joined))[0]
                if not last.reqs:
                    to_pool(last, now)
        # decode queues
        for q in decode_queues:
            while q:
                r = reqs[q[0]]
                s = place_decode(r, now)
                if s is None:
                    if profile.lookup(1, r.kv_len + 1) < r.arrival + r.ttft + tpots[r.tier] - now:
                        break
                    q.pop(0)
                    drop(r)
                    continue
                s.reqs.append(q.pop(0))
                r.phase, r.decode_server = 2, s.sid
        # prefill queue
        while prefill_queue:
            r = reqs[prefill_queue[0]]
            s = place_prefill(r, now)
            if s is None:
                if prefill_admits(Server(-1), r, now):
                    break
                prefill_queue.pop(0)
                drop(r)
                continue
            s.reqs.append(prefill_queue.pop(0))
            r.phase, r.prefill_server = 1, s.sid
        # iteration starts
        for s in servers:
            if s.busy_until is not None or not s.reqs:
                continue
            tokens = kv = 0
            if s.tier == PREFILL_CLUSTER:
                plan = policy.chunk_plan([reqs[i].prompt - reqs[i].prefilled for i in s.reqs], prefill_budget, True, 0)
                s.batch = [(s.reqs[idx], tok) for idx, tok in plan[0]]
                for ri, tok in s.batch:
                    tokens += tok
                    kv += reqs[ri].prefilled + tok
            else:
                s.batch = [(ri, 1) for ri in s.reqs]
                for ri in s.reqs:
                    tokens += 1
                    kv += reqs[ri].kv_len + 1
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
        "prefill_server": [r.prefill_server for r in reqs],
        "decode_server": [r.decode_server for r in reqs],
        "end_ms": now,
        "cost_ms": cost,
        **stats,
    }
