// Host-side consumers of the latency profile (see include/polysched.h for the passages).
#include "../../include/polysched.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <new>
#include <vector>

struct ps_profile {
    std::vector<double> b, k, ms;  // ms[i * k.size() + j]
};

namespace {

// index of the interval's left knot and the position inside it: 0 below the first knot, > 1 beyond the last
void segment(const std::vector<double>& knots, double x, size_t* idx, double* t) {
    if (knots.size() == 1 || x <= knots[0]) { *idx = 0; *t = 0.0; return; }
    size_t i = knots.size() - 2;
    for (size_t j = 0; j + 1 < knots.size(); j++)
        if (x < knots[j + 1]) { i = j; break; }
    *idx = i;
    *t = (x - knots[i]) / (knots[i + 1] - knots[i]);
}

struct Req { int64_t kv; int64_t rem; };

std::vector<Req> predicted(const ps_running_req* running, int32_t n, int32_t avg) {
    std::vector<Req> v;
    v.reserve((size_t)n + 1);
    for (int32_t i = 0; i < n; i++) v.push_back(Req{running[i].kv_len, std::max<int64_t>(1, (int64_t)avg - running[i].generated)});
    return v;
}

bool bad_running(const ps_running_req* running, int32_t n) {
    if (n < 0 || (n > 0 && !running)) return true;
    for (int32_t i = 0; i < n; i++)
        if (running[i].kv_len < 0 || running[i].generated < 0) return true;
    return false;
}

}  // namespace

extern "C" ps_status ps_profile_create(const int32_t* batch_sizes, int32_t n_batch, const int64_t* kv_sizes, int32_t n_kv,
                                       const float* ms, ps_profile** out) {
    if (!batch_sizes || !kv_sizes || !ms || !out || n_batch < 1 || n_kv < 1) return PS_EINVAL;
    for (int32_t i = 1; i < n_batch; i++)
        if (batch_sizes[i] <= batch_sizes[i - 1]) return PS_EINVAL;
    for (int32_t j = 1; j < n_kv; j++)
        if (kv_sizes[j] <= kv_sizes[j - 1]) return PS_EINVAL;
    for (int64_t i = 0; i < (int64_t)n_batch * n_kv; i++)
        if (!std::isfinite(ms[i])) return PS_EINVAL;
    ps_profile* p = new (std::nothrow) ps_profile;
    if (!p) return PS_ENOMEM;
    p->b.assign(batch_sizes, batch_sizes + n_batch);
    p->k.assign(kv_sizes, kv_sizes + n_kv);
    p->ms.assign(ms, ms + (size_t)n_batch * n_kv);
    *out = p;
    return PS_OK;
}

extern "C" void ps_profile_destroy(ps_profile* p) { delete p; }

extern "C" double ps_profile_lookup(const ps_profile* p, double batch, double kv) {
    if (!p) return std::numeric_limits<double>::quiet_NaN();
    size_t i, j;
    double tb, tk;
    segment(p->b, batch, &i, &tb);
    segment(p->k, kv, &j, &tk);
    const size_t nk = p->k.size();
    const size_t i1 = std::min(i + 1, p->b.size() - 1), j1 = std::min(j + 1, nk - 1);
    const double v00 = p->ms[i * nk + j], v01 = p->ms[i * nk + j1], v10 = p->ms[i1 * nk + j], v11 = p->ms[i1 * nk + j1];
    const double lo = v00 + (v01 - v00) * tk;
    const double hi = v10 + (v11 - v10) * tk;
    return lo + (hi - lo) * tb;
}

// The total KV size in iteration i is  sum over requests with rem > i of (kv + i + 1).  Between two
// finishing times it only grows, so the maximum is reached in the last iteration before some request
// finishes: i = rem_r - 1 for some r.  Sorted by rem, a suffix sum gives each candidate in O(1).
extern "C" ps_status ps_max_future_kv(const ps_running_req* running, int32_t n_running, int32_t new_prompt_len,
                                      int32_t avg_decode_len, int64_t* max_kv, int32_t* n_iters) {
    if (!max_kv || !n_iters || avg_decode_len < 1 || bad_running(running, n_running)) return PS_EINVAL;
    std::vector<Req> v = predicted(running, n_running, avg_decode_len);
    if (new_prompt_len >= 0) v.push_back(Req{new_prompt_len, std::max<int64_t>(1, avg_decode_len)});
    std::sort(v.begin(), v.end(), [](const Req& a, const Req& b) { return a.rem < b.rem; });
    int64_t best = 0, suffix_kv = 0;
    for (size_t r = v.size(); r-- > 0;) {
        suffix_kv += v[r].kv;                       // requests r.. are still running in iteration v[r].rem - 1
        const int64_t active = (int64_t)(v.size() - r);
        best = std::max(best, suffix_kv + active * v[r].rem);   // each attends kv + (rem - 1) + 1
    }
    *max_kv = best;
    *n_iters = v.empty() ? 0 : (int32_t)v.back().rem;
    return PS_OK;
}

extern "C" ps_status ps_predict_admit(const ps_profile* p, const ps_running_req* running, int32_t n_running, int32_t new_prompt_len,
                                      int32_t avg_decode_len, double tpot_ms, double wait_ms, int32_t* admit, double* predicted_ms,
                                      int64_t* max_kv) {
    if (!p || !admit || !predicted_ms || !max_kv || new_prompt_len < 0) return PS_EINVAL;
    int64_t kv = 0;
    int32_t iters = 0;
    const ps_status st = ps_max_future_kv(running, n_running, new_prompt_len, avg_decode_len, &kv, &iters);
    if (st != PS_OK) return st;
    const double t = ps_profile_lookup(p, (double)(n_running + 1), (double)kv) + wait_ms;
    *admit = t < tpot_ms ? 1 : 0;
    *predicted_ms = t;
    *max_kv = kv;
    return PS_OK;
}

extern "C" ps_status ps_chunk_plan(const int32_t* prompts, int32_t n, int32_t budget, int32_t dynamic, int32_t first_iteration_used,
                                   int32_t* chunks, int32_t cap, int32_t* n_chunks, int32_t* n_iterations) {
    if (!prompts || !n_chunks || !n_iterations || n < 0 || budget < 1 || cap < 0 || (cap > 0 && !chunks) ||
        first_iteration_used < 0 || first_iteration_used > budget)
        return PS_EINVAL;
    for (int32_t i = 0; i < n; i++)
        if (prompts[i] < 1) return PS_EINVAL;
    int32_t head = 0, iter = 0, count = 0;
    int64_t used = first_iteration_used, rem = n > 0 ? prompts[0] : 0;
    while (head < n) {
        bool open = true;
        while (open && head < n) {
            const int64_t room = budget - used;
            int64_t take;
            if (rem <= room) take = rem;
            else if (dynamic && used + rem < 2 * (int64_t)budget) { take = rem; open = false; }
            else if (room > 0) { take = room; open = false; }
            else break;
            if (count < cap) { chunks[3 * count] = iter; chunks[3 * count + 1] = head; chunks[3 * count + 2] = (int32_t)take; }
            count++;
            used += take;
            rem -= take;
            if (rem == 0 && ++head < n) rem = prompts[head];
            if (used >= budget) open = false;
        }
        iter++;
        used = 0;
    }
    *n_chunks = count;
    *n_iterations = iter;
    return PS_OK;
}

extern "C" ps_status ps_predict_chunked_prefill(const ps_profile* p, const ps_running_req* running, int32_t n_running,
                                                int32_t prompt_len, int32_t avg_decode_len, double tpot_ms, double ttft_ms,
                                                double wait_ms, int32_t* admit, int32_t* chunk, int32_t* n_iters,
                                                double* first_token_ms) {
    if (!p || !admit || !chunk || !n_iters || !first_token_ms || prompt_len < 1 || avg_decode_len < 1 || bad_running(running, n_running))
        return PS_EINVAL;
    const std::vector<Req> decs = predicted(running, n_running, avg_decode_len);
    // sum of the iteration times if chunk size c is kept, or a negative value as soon as one reaches the TPOT
    // decodes still running in iteration j and the KV tokens they attend there, computed once per j
    std::vector<int64_t> act_j, kv_j;
    auto decodes_in = [&](int32_t j) {
        while ((int32_t)act_j.size() <= j) {
            const int64_t jj = (int64_t)act_j.size();
            int64_t active = 0, kv = 0;
            for (const Req& r : decs)
                if (r.rem > jj) { active++; kv += r.kv + jj + 1; }
            act_j.push_back(active);
            kv_j.push_back(kv);
        }
    };
    auto kept = [&](int32_t c_fit, int32_t* n_out) {
        double total = wait_ms;
        int64_t done = 0;
        int32_t j = 0;
        for (; done < prompt_len; j++) {
            const int64_t c = std::min<int64_t>(c_fit, prompt_len - done);
            decodes_in(j);
            const int64_t active = act_j[j];
            int64_t kv = kv_j[j];
            kv += done + c;
            const double t = ps_profile_lookup(p, (double)(active + c), (double)kv);
            if (!(t < tpot_ms)) return -1.0;
            total += t;
            done += c;
        }
        *n_out = j;
        return total;
    };
    for (int32_t c = prompt_len; c >= 1; c--) {
        int32_t n = 0;
        const double total = kept(c, &n);
        if (total < 0.0) continue;
        *admit = total < ttft_ms ? 1 : 0;
        *chunk = c;
        *n_iters = n;
        *first_token_ms = total;
        return PS_OK;
    }
    *admit = 0; *chunk = 0; *n_iters = 0;
    *first_token_ms = std::numeric_limits<double>::infinity();
    return PS_OK;
}

extern "C" int32_t ps_batch_limit_pd(const ps_profile* prof, double p, double d, double tpot_ms, double capacity, int32_t b_max) {
    if (!prof) return 0;
    int32_t best = 0;
    for (int32_t b = 1; b <= b_max; b++) {
        const double kv = b * (p + d / 2.0);
        if (kv < capacity && ps_profile_lookup(prof, (double)b, kv) < tpot_ms) best = b;
    }
    return best;
}

extern "C" int32_t ps_batch_limit_co(const ps_profile* prof, double p, double d, double tpot_ms, double ttft_ms, double capacity,
                                     int32_t b_max) {
    if (!prof) return 0;
    int32_t best = 0;
    for (int32_t b = 1; b <= b_max; b++) {
        const double kv = d / (p + d) * b * (p + d / 2.0) + p;
        const double t = ps_profile_lookup(prof, (double)b, kv);
        if (kv < capacity && t < tpot_ms && (p + d) / b * t < ttft_ms) best = b;
    }
    return best;
}

// Sec. 3.5.  The table's two axes taken apart as in the cost model of Sec. 3.4: GEMM(B) is the time at the smallest
// profiled KV size, DcAttn(kv) what the KV size adds at the smallest profiled batch; PF(p) is taken as DcAttn(p).
static double gemm_time(const ps_profile* p, double batch) { return ps_profile_lookup(p, batch, p->k[0]); }
static double attn_time(const ps_profile* p, double kv) { return ps_profile_lookup(p, p->b[0], kv) - ps_profile_lookup(p, p->b[0], p->k[0]); }

extern "C" double ps_cost_pd(const ps_profile* prof, double p, double d, double b_pf, double b_dc) {
    if (!prof || !(b_pf > 0.0) || !(b_dc > 0.0)) return std::numeric_limits<double>::quiet_NaN();
    return p * gemm_time(prof, b_pf) / b_pf + attn_time(prof, p) + d * gemm_time(prof, b_dc) / b_dc + attn_time(prof, d * (p + d / 2.0));
}

extern "C" double ps_cost_co(const ps_profile* prof, double p, double d, double b) {
    if (!prof || !(b > 0.0)) return std::numeric_limits<double>::quiet_NaN();
    return (p + d) * gemm_time(prof, b) / b + attn_time(prof, p) + attn_time(prof, d * (p + d / 2.0));
}

extern "C" double ps_optimal_cost_pd(const ps_profile* prof, double p, double d, double tpot_ms, double capacity, double b_pf, int32_t b_max) {
    if (!prof) return std::numeric_limits<double>::quiet_NaN();
    const int32_t b = ps_batch_limit_pd(prof, p, d, tpot_ms, capacity, b_max);
    return b > 0 ? ps_cost_pd(prof, p, d, b_pf, (double)b) : std::numeric_limits<double>::infinity();
}

extern "C" double ps_optimal_cost_co(const ps_profile* prof, double p, double d, double tpot_ms, double ttft_ms, double capacity, int32_t b_max) {
    if (!prof) return std::numeric_limits<double>::quiet_NaN();
    const int32_t b = ps_batch_limit_co(prof, p, d, tpot_ms, ttft_ms, capacity, b_max);
    return b > 0 ? ps_cost_co(prof, p, d, (double)b) : std::numeric_limits<double>::infinity();
}
