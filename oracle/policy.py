"""Consumers of the latency profile: what the paper's router does with the table this repository
measures (test infrastructure; plain and slow on purpose).

Sec. 4.5 ("Profile-Based Batch Formation"): iteration time is looked up in a map
(batch size, KV cache size) -> time; when routing, future iterations are simulated with every
request's output predicted as the average decode length, the largest KV cache size reached is
taken, and the request is admitted when the time looked up for (current token batch size, that KV
size) is below the TPOT.  Sec. 4.6 ("Wait-Time-Aware Scheduling"): the time the request waits for
the server's current iteration is added to the predicted iteration time.  Sec. 4.7 ("Handling
TTFT"): dynamic chunking for a prefill instance (a request whose remaining length is below twice
the token budget is finished at once and nothing else is admitted into that enlarged iteration),
and, for co-location, admitting a prefill only if the chunk size predicted at scheduling time can
be kept for the whole prefill while the decodes' KV grows.  Sec. 3.4: batch-size limits.
Sec. 3.5: the cost of serving one request at those batch sizes.

Readings fixed where the text is loose (each is one sentence of the paper made executable):
  * table lookup: bilinear interpolation between profiled points; below the first point of an axis
    the first point's value is used, beyond the last one the last interval is extended linearly;
  * a running request that has generated g tokens is predicted to generate max(1, avg - g) more;
    in future iteration i (0-based) every request still running attends its current KV length + i + 1;
  * "current token batch size" = number of running requests + the new one;
  * dynamic chunking: iterations are filled first-come first-served; a request is finished in the
    current iteration if it fits the room left, or (dynamic) if the iteration then stays below
    twice the budget, in which case the iteration is closed; otherwise it gets the room left;
  * co-location: the chunk size predicted at scheduling time is the largest c that can be kept for
    all ceil(prompt / c) iterations of the prefill, i.e. every one of them stays below the TPOT while
    the chunks attend a growing prefix and the decodes grow by one token per iteration (and leave
    when predicted finished); the request is admitted if such a c exists and the sum of those
    iterations plus the wait time stays below the TTFT.  (Taking the largest c that fits the first
    iteration and rejecting when a later one does not would turn away every multi-chunk prompt on a
    table that grows with the KV size at all, even on an empty instance.)
  * cost (Sec. 3.5): the table is the only profile there is, so its two axes are taken apart as the
    paper's cost model does (Sec. 3.4): GEMM(B) = T(B, smallest profiled KV size) and
    DcAttn(kv) = T(smallest profiled batch, kv) - T(smallest profiled batch, smallest profiled KV
    size); PF(p), the prefill attention of a whole prompt, is taken as DcAttn(p), the paper's own
    simplification ("comparable to decode attention with the same existing KV length").
"""
import math


class Profile:
    """(batch size, KV cache size) -> time.  batch_sizes and kv_sizes ascending; ms[i][j] for
    (batch_sizes[i], kv_sizes[j])."""

    def __init__(self, batch_sizes, kv_sizes, ms):
        self.b = [float(v) for v in batch_sizes]
        self.k = [float(v) for v in kv_sizes]
        self.ms = [[float(v) for v in row] for row in ms]
        assert len(self.ms) == len(self.b) and all(len(r) == len(self.k) for r in self.ms)
        assert all(x < y for x, y in zip(self.b, self.b[1:])) and all(x < y for x, y in zip(self.k, self.k[1:]))

    @staticmethod
    def _segment(knots, x):
        """(index of the interval's left knot, position in it): 0 below the first knot, > 1 beyond the last."""
        if len(knots) == 1 or x <= knots[0]:
            return 0, 0.0
        i = len(knots) - 2
        for j in range(len(knots) - 1):
            if x < knots[j + 1]:
                i = j
                break
        return i, (x - knots[i]) / (knots[i + 1] - knots[i])

    def lookup(self, batch, kv):
        i, tb = self._segment(self.b, float(batch))
        j, tk = self._segment(self.k, float(kv))
        i1 = min(i + 1, len(self.b) - 1)
        j1 = min(j + 1, len(self.k) - 1)
        v00, v01, v10, v11 = self.ms[i][j], self.ms[i][j1], self.ms[i1][j], self.ms[i1][j1]
        lo = v00 + (v01 - v00) * tk
        hi = v10 + (v11 - v10) * tk
        return lo + (hi - lo) * tb


def max_future_kv(running, new_prompt, avg_decode):
    """running: list of (kv_len, generated).  Simulate iterations until every request has finished;
    return (largest total KV cache size attended in an iteration, iterations simulated)."""
    reqs = [(int(kv), max(1, int(avg_decode) - int(g))) for kv, g in running]
    if new_prompt is not None:
        reqs.append((int(new_prompt), max(1, int(avg_decode))))
    best, it = 0, 0
    while any(rem > it for _, rem in reqs):
        total = sum(kv + it + 1 for kv, rem in reqs if rem > it)
        best = max(best, total)
        it += 1
    return best, it


def predict_admit(profile, running, new_prompt, avg_decode, tpot_ms, wait_ms=0.0):
    """(admit?, predicted time = iteration time + wait time, largest future KV size)."""
    kv, _ = max_future_kv(running, new_prompt, avg_decode)
    t = profile.lookup(len(running) + 1, kv) + float(wait_ms)
    return t < float(tpot_ms), t, kv


def chunk_plan(prompts, budget, dynamic, first_iteration_used=0):
    """prompts: remaining prompt lengths in arrival order.  Returns the iterations, each a list of
    (request index, tokens).  first_iteration_used: tokens of other work already in the first one."""
    remaining = [int(p) for p in prompts]
    budget = int(budget)
    assert budget >= 1 and all(p >= 1 for p in remaining) and 0 <= first_iteration_used <= budget
    out, head, used = [], 0, int(first_iteration_used)
    while head < len(remaining):
        it, open_ = [], True
        while open_ and head < len(remaining):
            r, room = remaining[head], budget - used
            if r <= room:
                take = r
            elif dynamic and used + r < 2 * budget:
                take, open_ = r, False
            elif room > 0:
                take, open_ = room, False
            else:
                break
            it.append((head, take))
            used += take
            remaining[head] -= take
            if remaining[head] == 0:
                head += 1
            if used >= budget:
                open_ = False
        out.append(it)
        used = 0
    return out


def predict_chunked_prefill(profile, running, prompt, avg_decode, tpot_ms, ttft_ms, wait_ms=0.0):
    """Co-location.  Returns (admit?, chunk size, iterations, predicted time to first token)."""
    prompt = int(prompt)
    decs = [(int(kv), max(1, int(avg_decode) - int(g))) for kv, g in running]

    def iteration_times(chunk):
        """times of the ceil(prompt / chunk) iterations if this chunk size is kept, or None if one reaches the TPOT"""
        times, done, j = [], 0, 0
        while done < prompt:
            c = min(chunk, prompt - done)
            active = [(kv, rem) for kv, rem in decs if rem > j]
            kv = sum(kv + j + 1 for kv, _ in active) + done + c
            t = profile.lookup(len(active) + c, kv)
            if not t < tpot_ms:
                return None
            times.append(t)
            done += c
            j += 1
        return times

    for chunk in range(prompt, 0, -1):
        times = iteration_times(chunk)
        if times is not None:
            total = float(wait_ms)
            for t in times:
                total += t
            return total < ttft_ms, chunk, len(times), total
    return False, 0, 0, math.inf


def batch_limit_pd(profile, p, d, tpot_ms, capacity, b_max=4096):
    """Sec. 3.4, decode instance of a disaggregated deployment: the largest batch size B with
    T(B, B (p + d/2)) < TPOT and B (p + d/2) < C; 0 if none."""
    best = 0
    for b in range(1, int(b_max) + 1):
        kv = b * (p + d / 2.0)
        if kv < capacity and profile.lookup(b, kv) < tpot_ms:
            best = b
    return best


def batch_limit_co(profile, p, d, tpot_ms, ttft_ms, capacity, b_max=4096):
    """Sec. 3.4, co-location with chunked prefill: the largest token batch size B with
    T_iter = T(B, d/(p+d) B (p + d/2) + p) < TPOT, N_iter T_iter < TTFT with N_iter = (p+d)/B,
    and the KV size below C; 0 if none."""
    best = 0
    for b in range(1, int(b_max) + 1):
        kv = d / (p + d) * b * (p + d / 2.0) + p
        t = profile.lookup(b, kv)
        if kv < capacity and t < tpot_ms and (p + d) / b * t < ttft_ms:
            best = b
    return best


def gemm_time(profile, batch):
    """GEMM(B) of the paper's cost model: the table's time at the smallest profiled KV size."""
    return profile.lookup(batch, profile.k[0])


def attn_time(profile, kv):
    """DcAttn(kv): what the table adds over its smallest profiled KV size, at the smallest profiled batch."""
    return profile.lookup(profile.b[0], kv) - profile.lookup(profile.b[0], profile.k[0])


def cost_pd(profile, p, d, b_pf, b_dc):
    """Sec. 3.5, disaggregated: p GEMM(B_pf)/B_pf + PF(p) + d GEMM(B_dc)/B_dc + DcAttn(d (p + d/2)), in instance-ms."""
    return p * gemm_time(profile, b_pf) / b_pf + attn_time(profile, p) + d * gemm_time(profile, b_dc) / b_dc + attn_time(profile, d * (p + d / 2.0))


def cost_co(profile, p, d, b):
    """Sec. 3.5, co-located: (p + d) GEMM(B)/B + PF(p) + DcAttn(d (p + d/2)), in instance-ms."""
    return (p + d) * gemm_time(profile, b) / b + attn_time(profile, p) + attn_time(profile, d * (p + d / 2.0))


def optimal_cost_pd(profile, p, d, tpot_ms, capacity, b_pf, b_max=4096):
    """Cost at the largest decode batch the TPOT and the memory allow (Sec. 3.4, 3.5); inf if none."""
    b = batch_limit_pd(profile, p, d, tpot_ms, capacity, b_max)
    return cost_pd(profile, p, d, b_pf, b) if b > 0 else math.inf


def optimal_cost_co(profile, p, d, tpot_ms, ttft_ms, capacity, b_max=4096):
    """Cost at the largest token batch the TPOT, the TTFT and the memory allow (Sec. 3.4, 3.5); inf if none."""
    b = batch_limit_co(profile, p, d, tpot_ms, ttft_ms, capacity, b_max)
    return cost_co(profile, p, d, b) if b > 0 else math.inf
