// Cluster simulator for the paper's router on co-located (chunked-prefill) serving instances
// (Sec. 5.1: instances advance in 1 ms steps with iteration times taken from the
// (batch size, KV cache size) -> time table; Sec. 4.2-4.7: one cluster per TPOT tier, highest-load
// instance first, lazy promotion onto tighter tiers, scaling from and to an idle pool, admission by
// predicted future KV size and by the chunk size that can be kept for the whole prefill with the wait
// for the iteration in flight; Sec. 2.3: token i of a request is due at arrival + TTFT + i * TPOT).
// A second simulator does the same for prefill-decode disaggregated instances: a prefill cluster shared by
// all tiers that takes requests in first-token-deadline order and forms iterations by dynamic chunking
// (Sec. 4.2, 4.7), and decode clusters per tier with the wait-time-aware admission of Sec. 4.6.
// Host only.  The decisions themselves are the ones exported by policy.cpp.
#include <algorithm>
#include <cstdint>
#include <deque>
#include <new>
#include <utility>
#include <vector>

#include "../../include/polysched.h"

namespace {

enum Phase { QUEUED = 0, PREFILL = 1, DECODE = 2, DONE = 3, HANDED_OVER = 4 };
constexpr int32_t PREFILL_CLUSTER = -2;  // "tier" of an instance that serves the prefill cluster
enum State { POOL = 0, ACTIVE = 1, PENDING = 2 };

struct Request {
    double arrival, ttft;
    int32_t prompt, output, tier;
    int32_t chunk = 0, prefilled = 0, generated = 0, kv_len = 0;
    int32_t first_server = -1, decode_server = -1;
    int phase = QUEUED;
    bool violated = false;
    double first_token = -1.0, finish = -1.0;
};

struct Instance {
    int32_t id = 0;
    int state = POOL;
    int32_t tier = -1;
    int64_t joined = -1;              // order of joining a cluster: the tie-break of the load order
    std::vector<int32_t> reqs;        // in admission order
    bool in_iteration = false;
    double busy_until = 0.0;
    std::vector<std::pair<int32_t, int32_t>> batch;  // (request, tokens) of the iteration in flight
    double since = 0.0;               // when it last left the idle pool
    bool just_ended = false;          // an iteration ended in the current step, at free_at: the next one starts there
    double free_at = 0.0;
};

// State and steps that both deployments share.
struct Cluster {
    const ps_profile* prof;
    const ps_sim_config& cfg;
    std::vector<Request> reqs;
    std::vector<Instance> inst;
    ps_sim_summary sum{};
    double cost = 0.0;
    int64_t join_counter = 0;
    int32_t done = 0;
    std::vector<ps_running_req> run;   // scratch: the decodes of the instance under test
    std::vector<Instance*> cand;       // scratch: candidate list

    Cluster(const ps_profile* p, const ps_sim_config& c) : prof(p), cfg(c) {}

    static double wait_of(const Instance& s, int64_t now) { return s.in_iteration ? std::max(0.0, s.busy_until - (double)now) : 0.0; }

    // highest load first; among equals the instance that joined its cluster first
    static void by_load(std::vector<Instance*>& v) {
        std::stable_sort(v.begin(), v.end(), [](const Instance* a, const Instance* b) {
            if (a->reqs.size() != b->reqs.size()) return a->reqs.size() > b->reqs.size();
            return a->joined < b->joined;
        });
    }

    void join(Instance& s, int32_t tier, int64_t now) {
        if (s.state == POOL) s.since = (double)now;
        s.state = ACTIVE;
        s.tier = tier;
        s.joined = join_counter++;
        sum.scale_ups++;
    }

    void to_pool(Instance& s, int64_t now) {
        cost += (double)now - s.since;
        s.state = POOL;
        s.tier = -1;
        s.joined = -1;
        sum.scale_downs++;
    }

    void drop(Request& r) {
        r.phase = DONE;
        r.violated = true;
        sum.dropped++;
        done++;
    }

    // Sec. 4.3, 4.4: the request's own cluster, then the clusters of tighter tiers from the nearest one (lazy promotion),
    // each from the most loaded instance down; then scale-up: a parked instance whose tightest request is of this tier,
    // else one from the idle pool.  admit(instance, tier it would serve, request) returns 0 for "no", else a value that
    // is handed back through *granted.
    template <class Admit>
    Instance* place_in_tiers(const Request& r, int64_t now, Admit admit, int32_t* granted) {
        for (int32_t t = r.tier; t >= 0; t--) {
            cand.clear();
            for (Instance& s : inst)
                if (s.state == ACTIVE && s.tier == t) cand.push_back(&s);
            by_load(cand);
            for (Instance* s : cand) {
                const int32_t g = admit(*s, t, r);
                if (g) {
                    if (t != r.tier) sum.promotions++;
                    *granted = g;
                    return s;
                }
            }
        }
        cand.clear();
        for (Instance& s : inst) {
            if (s.state != PENDING) continue;
            int32_t tightest = INT32_MAX;
            for (int32_t i : s.reqs) tightest = std::min(tightest, reqs[i].tier);
            if (tightest == r.tier) cand.push_back(&s);
        }
        by_load(cand);
        for (Instance& s : inst)
            if (s.state == POOL) cand.push_back(&s);
        for (Instance* s : cand) {
            const int32_t g = admit(*s, r.tier, r);
            if (g) {
                join(*s, r.tier, now);
                *granted = g;
                return s;
            }
            if (s->state == POOL) break;  // every idle instance gives the same answer
        }
        return nullptr;
    }

    // Iterations that have ended deliver their tokens at their end time (Sec. 2.3: token i is due at
    // arrival + TTFT + i * TPOT).  prefill_done(instance, request index) is called for a request whose last chunk
    // has just produced token 0 and that has more tokens to generate.
    template <class PrefillDone>
    void deliver_ended(int64_t now, PrefillDone prefill_done) {
        for (Instance& s : inst) {
            if (!s.in_iteration || !(s.busy_until <= (double)now)) continue;
            const double t_end = s.busy_until;
            for (const auto& bt : s.batch) {
                Request& r = reqs[bt.first];
                const bool was_prefill = r.phase == PREFILL;
                if (was_prefill) {
                    r.prefilled += bt.second;
                    if (r.prefilled < r.prompt) continue;
                    r.phase = DECODE;
                    r.kv_len = r.prompt;
                    r.generated = 1;
                    r.first_token = t_end;
                } else {
                    r.kv_len++;
                    r.generated++;
                }
                if (t_end > r.arrival + r.ttft + (double)(r.generated - 1) * cfg.tpot_ms[r.tier]) r.violated = true;
                if (r.generated == r.output) {
                    s.reqs.erase(std::find(s.reqs.begin(), s.reqs.end(), bt.first));
                    r.phase = DONE;
                    r.finish = t_end;
                    done++;
                } else if (was_prefill) {
                    prefill_done(s, bt.first);
                }
            }
            s.in_iteration = false;
            s.batch.clear();
            s.just_ended = true;
            s.free_at = t_end;
            sum.iterations++;
        }
        for (Instance& s : inst)
            if (s.state == PENDING && s.reqs.empty()) to_pool(s, now);
    }

    // Scale-down check of the decode (or co-located) clusters: the least loaded instance of each returns to the idle
    // pool if empty and is parked if none of its requests is of the cluster's tier.
    void check_tier_clusters(int64_t now) {
        for (int32_t t = 0; t < cfg.n_tiers; t++) {
            Instance* last = nullptr;
            for (Instance& s : inst) {
                if (s.state != ACTIVE || s.tier != t) continue;
                if (!last || s.reqs.size() < last->reqs.size() || (s.reqs.size() == last->reqs.size() && s.joined > last->joined))
                    last = &s;
            }
            if (!last) continue;
            if (last->reqs.empty()) {
                to_pool(*last, now);
            } else {
                bool own = false;
                for (int32_t i : last->reqs) own = own || reqs[i].tier == t;
                if (!own) last->state = PENDING;
            }
        }
    }

    // The batch in s.batch starts: at the end of the previous iteration if that ended within this step (iterations run
    // back to back; only the router works on the 1 ms grid), else at the step.
    void start_iteration(Instance& s, int64_t now, int64_t tokens, int64_t kv) {
        s.busy_until = (s.just_ended ? s.free_at : (double)now) + ps_profile_lookup(prof, (double)tokens, (double)kv);
        s.in_iteration = true;
    }

    void end_step() {
        for (Instance& s : inst) s.just_ended = false;
    }

    void close(int64_t now) {
        for (Instance& s : inst)
            if (s.state != POOL) cost += (double)now - s.since;
        sum.end_ms = now;
        sum.cost_ms = cost;
    }
};

// ---------------------------------------------------------------------------------------------------
// Co-location with chunked prefill
// ---------------------------------------------------------------------------------------------------
struct Sim : Cluster {
    std::vector<std::deque<int32_t>> queues;
    using Cluster::Cluster;

    // chunk size the instance would keep for the request's prefill if it served `tier`, 0 = not admitted
    int32_t admits(const Instance& s, int32_t tier, const Request& r, int64_t now) {
        run.clear();
        for (int32_t i : s.reqs) {
            if (reqs[i].phase == PREFILL) return 0;  // one prefill at a time
            run.push_back(ps_running_req{reqs[i].kv_len, reqs[i].generated});
        }
        const double tpot = cfg.tpot_ms[tier];
        int32_t ok = 0, chunk = 0, n_it = 0;
        double t_first = 0.0;
        sum.admission_tests++;
        if (ps_predict_chunked_prefill(prof, run.data(), (int32_t)run.size(), r.prompt, cfg.avg_decode_len, tpot,
                                       r.arrival + r.ttft - (double)now, wait_of(s, now), &ok, &chunk, &n_it, &t_first) != PS_OK || !ok)
            return 0;
        int32_t ok2 = 0;
        double predicted = 0.0;
        int64_t kv = 0;
        if (ps_predict_admit(prof, run.data(), (int32_t)run.size(), r.prompt, cfg.avg_decode_len, tpot, 0.0, &ok2, &predicted, &kv) != PS_OK ||
            !ok2 || !((double)kv < cfg.kv_capacity))
            return 0;
        return chunk;
    }

    void run_all() {
        const int32_t n = (int32_t)reqs.size();
        int32_t next_arrival = 0;
        int64_t now = 0;
        queues.resize(cfg.n_tiers);
        while (done < n && now < cfg.max_steps) {
            deliver_ended(now, [](Instance&, int32_t) {});  // the request stays where it is and decodes
            while (next_arrival < n && reqs[next_arrival].arrival <= (double)now) {
                queues[reqs[next_arrival].tier].push_back(next_arrival);
                next_arrival++;
            }
            if (now % cfg.check_period_ms == 0) check_tier_clusters(now);
            // routing: tightest tier first, first come first served
            for (auto& q : queues) {
                while (!q.empty()) {
                    Request& r = reqs[q.front()];
                    int32_t chunk = 0;
                    Instance* s = place_in_tiers(r, now, [&](const Instance& c, int32_t tier, const Request& rr) { return admits(c, tier, rr, now); }, &chunk);
                    if (!s) {
                        int32_t ok = 0, c = 0, n_it = 0;
                        double t_first = 0.0;
                        ps_predict_chunked_prefill(prof, nullptr, 0, r.prompt, cfg.avg_decode_len, cfg.tpot_ms[r.tier],
                                                   r.arrival + r.ttft - (double)now, 0.0, &ok, &c, &n_it, &t_first);
                        if (ok) break;  // it can still make its first token on an empty instance: keep its place
                        q.pop_front();
                        drop(r);
                        continue;
                    }
                    r.first_server = r.decode_server = s->id;
                    r.chunk = chunk;
                    r.phase = PREFILL;
                    s->reqs.push_back(q.front());
                    q.pop_front();
                }
            }
            // instances outside an iteration that hold requests start one: a token of every decode, the next chunk of the prefill
            for (Instance& s : inst) {
                if (s.in_iteration || s.reqs.empty()) continue;
                int64_t tokens = 0, kv = 0;
                for (int32_t i : s.reqs) {
                    const Request& r = reqs[i];
                    if (r.phase == DECODE) {
                        s.batch.emplace_back(i, 1);
                        tokens += 1;
                        kv += r.kv_len + 1;
                    } else {
                        const int32_t c = std::min(r.chunk, r.prompt - r.prefilled);
                        s.batch.emplace_back(i, c);
                        tokens += c;
                        kv += r.prefilled + c;
                    }
                }
                start_iteration(s, now, tokens, kv);
            }
            end_step();
            now++;
        }
        close(now);
    }
};

// ---------------------------------------------------------------------------------------------------
// Prefill-decode disaggregation
// ---------------------------------------------------------------------------------------------------
struct SimPD : Cluster {
    std::vector<int32_t> prefill_queue;
    std::vector<std::deque<int32_t>> decode_queues;
    std::vector<int32_t> rem, at, whole, plan;
    std::vector<double> due;
    using Cluster::Cluster;

    // prompt tokens of request i neither processed nor in the iteration in flight
    int32_t left(const Instance& s, int32_t i) const {
        int32_t v = reqs[i].prompt - reqs[i].prefilled;
        for (const auto& bt : s.batch)
            if (bt.first == i) v -= bt.second;
        return v;
    }

    int64_t prefill_load(const Instance& s) const {
        int64_t v = 0;
        for (int32_t i : s.reqs) v += reqs[i].prompt - reqs[i].prefilled;
        return v;
    }

    // dynamic-chunking plan of `rem` as {iteration, request, tokens} triples in `plan`; returns the number of chunks
    int32_t make_plan() {
        int32_t n_chunks = 0, n_iters = 0;
        if (plan.size() < 3 * (rem.size() + 8)) plan.resize(3 * (rem.size() + 8));
        for (;;) {
            ps_chunk_plan(rem.data(), (int32_t)rem.size(), cfg.prefill_budget, 1, 0, plan.data(), (int32_t)(plan.size() / 3), &n_chunks, &n_iters);
            if ((size_t)n_chunks * 3 <= plan.size()) return n_chunks;
            plan.resize((size_t)n_chunks * 3);
        }
    }

    // Would r, queued behind the requests already on s, get its first token in time, and would they still get theirs
    // (Sec. 4.7: the iterations of the requests already there and the wait for the one in flight count; dynamic
    // chunking lets a later request share the iteration of an earlier one's last chunk and so lengthens it)?
    bool prefill_admits(const Instance& s, const Request& r, int64_t now) {
        rem.clear();
        at.clear();
        whole.clear();
        due.clear();
        for (int32_t i : s.reqs) {
            const int32_t l = left(s, i);
            if (l <= 0) continue;
            rem.push_back(l);
            at.push_back(reqs[i].prompt - l);
            whole.push_back(reqs[i].prompt);
            due.push_back(reqs[i].arrival + reqs[i].ttft - (double)now);
        }
        rem.push_back(r.prompt);
        at.push_back(0);
        whole.push_back(r.prompt);
        due.push_back(r.arrival + r.ttft - (double)now);
        const int32_t n_chunks = make_plan();
        sum.admission_tests++;
        double t = wait_of(s, now);
        int32_t c = 0;
        while (c < n_chunks) {
            const int32_t it = plan[3 * c], first = c;
            int64_t tokens = 0, kv = 0;
            for (; c < n_chunks && plan[3 * c] == it; c++) {
                at[plan[3 * c + 1]] += plan[3 * c + 2];
                tokens += plan[3 * c + 2];
                kv += at[plan[3 * c + 1]];
            }
            t += ps_profile_lookup(prof, (double)tokens, (double)kv);
            for (int32_t e = first; e < c; e++) {
                const int32_t idx = plan[3 * e + 1];
                if (at[idx] == whole[idx] && !(t < due[idx])) return false;
            }
        }
        return true;
    }

    // Sec. 4.5, 4.6: the largest future KV size keeps the iteration below the TPOT of the tier served, fits the memory,
    // and the wait for the iteration in flight plus that iteration still meets the request's second-token deadline
    bool decode_admits(const Instance& s, int32_t tier, const Request& r, int64_t now) {
        run.clear();
        for (int32_t i : s.reqs) run.push_back(ps_running_req{reqs[i].kv_len, reqs[i].generated});
        int32_t ok = 0;
        double t = 0.0;
        int64_t kv = 0;
        sum.admission_tests++;
        if (ps_predict_admit(prof, run.data(), (int32_t)run.size(), r.kv_len, cfg.avg_decode_len, cfg.tpot_ms[tier], 0.0, &ok, &t, &kv) != PS_OK)
            return false;
        return ok && (double)kv < cfg.kv_capacity && wait_of(s, now) + t < r.arrival + r.ttft + cfg.tpot_ms[r.tier] - (double)now;
    }

    // the prefill instance with most unprocessed prompt tokens that admits the request, else one from the idle pool
    Instance* place_prefill(const Request& r, int64_t now) {
        cand.clear();
        for (Instance& s : inst)
            if (s.state == ACTIVE && s.tier == PREFILL_CLUSTER) cand.push_back(&s);
        std::stable_sort(cand.begin(), cand.end(), [this](const Instance* a, const Instance* b) {
            const int64_t la = prefill_load(*a), lb = prefill_load(*b);
            if (la != lb) return la > lb;
            return a->joined < b->joined;
        });
        for (Instance* s : cand)
            if (prefill_admits(*s, r, now)) return s;
        for (Instance& s : inst) {
            if (s.state != POOL) continue;
            if (prefill_admits(s, r, now)) {
                join(s, PREFILL_CLUSTER, now);
                return &s;
            }
            break;
        }
        return nullptr;
    }

    void run_all() {
        const int32_t n = (int32_t)reqs.size();
        int32_t next_arrival = 0;
        int64_t now = 0;
        const Instance empty_instance{};
        decode_queues.resize(cfg.n_tiers);
        while (done < n && now < cfg.max_steps) {
            deliver_ended(now, [this](Instance& s, int32_t i) {  // prefill done: hand over to the decode side
                s.reqs.erase(std::find(s.reqs.begin(), s.reqs.end(), i));
                reqs[i].phase = HANDED_OVER;
                decode_queues[reqs[i].tier].push_back(i);
            });
            // arrivals, kept in order of first-token deadline (Sec. 4.2)
            while (next_arrival < n && reqs[next_arrival].arrival <= (double)now) prefill_queue.push_back(next_arrival++);
            std::sort(prefill_queue.begin(), prefill_queue.end(), [this](int32_t a, int32_t b) {
                const double da = reqs[a].arrival + reqs[a].ttft, db = reqs[b].arrival + reqs[b].ttft;
                return da != db ? da < db : a < b;
            });
            if (now % cfg.check_period_ms == 0) {
                check_tier_clusters(now);
                Instance* last = nullptr;  // the least loaded prefill instance goes back if it holds no request
                int64_t last_load = 0;
                for (Instance& s : inst) {
                    if (s.state != ACTIVE || s.tier != PREFILL_CLUSTER) continue;
                    const int64_t l = prefill_load(s);
                    if (!last || l < last_load || (l == last_load && s.joined > last->joined)) { last = &s; last_load = l; }
                }
                if (last && last->reqs.empty()) to_pool(*last, now);
            }
            for (auto& q : decode_queues) {
                while (!q.empty()) {
                    Request& r = reqs[q.front()];
                    int32_t yes = 0;
                    Instance* s = place_in_tiers(r, now, [&](const Instance& c, int32_t tier, const Request& rr) { return decode_admits(c, tier, rr, now) ? 1 : 0; }, &yes);
                    if (!s) {
                        // an empty instance could still deliver the second token in time: keep the place in the queue
                        if (ps_profile_lookup(prof, 1.0, (double)(r.kv_len + 1)) < r.arrival + r.ttft + cfg.tpot_ms[r.tier] - (double)now) break;
                        q.pop_front();
                        drop(r);
                        continue;
                    }
                    s->reqs.push_back(q.front());
                    q.pop_front();
                    r.phase = DECODE;
                    r.decode_server = s->id;
                }
            }
            while (!prefill_queue.empty()) {
                Request& r = reqs[prefill_queue.front()];
                Instance* s = place_prefill(r, now);
                if (!s) {
                    if (prefill_admits(empty_instance, r, now)) break;
                    prefill_queue.erase(prefill_queue.begin());
                    drop(r);
                    continue;
                }
                s->reqs.push_back(prefill_queue.front());
                prefill_queue.erase(prefill_queue.begin());
                r.phase = PREFILL;
                r.first_server = s->id;
            }
            for (Instance& s : inst) {
                if (s.in_iteration || s.reqs.empty()) continue;
                int64_t tokens = 0, kv = 0;
                if (s.tier == PREFILL_CLUSTER) {
                    rem.clear();
                    for (int32_t i : s.reqs) rem.push_back(reqs[i].prompt - reqs[i].prefilled);
                    const int32_t n_chunks = make_plan();
                    for (int32_t c = 0; c < n_chunks && plan[3 * c] == 0; c++) {
                        const int32_t i = s.reqs[plan[3 * c + 1]], tok = plan[3 * c + 2];
                        s.batch.emplace_back(i, tok);
                        tokens += tok;
                        kv += reqs[i].prefilled + tok;
                    }
                } else {
                    for (int32_t i : s.reqs) {
                        s.batch.emplace_back(i, 1);
                        tokens += 1;
                        kv += reqs[i].kv_len + 1;
                    }
                }
                start_iteration(s, now, tokens, kv);
            }
            end_step();
            now++;
        }
        close(now);
    }
};

}  // namespace

template <class S>
static void run_and_report(S& sim, const ps_sim_config* cfg, const ps_sim_request* requests, int32_t n, uint8_t* attained,
                           double* first_token_ms, double* finish_ms, int32_t* server, int32_t* decode_server, ps_sim_summary* summary) {
    sim.reqs.resize(n);
    for (int32_t i = 0; i < n; i++) {
        Request& r = sim.reqs[i];
        r.arrival = requests[i].arrival_ms;
        r.ttft = requests[i].ttft_ms;
        r.prompt = requests[i].prompt_len;
        r.output = requests[i].output_len;
        r.tier = requests[i].tier;
    }
    sim.inst.resize(cfg->n_servers);
    for (int32_t s = 0; s < cfg->n_servers; s++) sim.inst[s].id = s;
    sim.run_all();
    for (int32_t i = 0; i < n; i++) {
        const Request& r = sim.reqs[i];
        if (attained) attained[i] = (r.phase == DONE && !r.violated) ? 1 : 0;
        if (first_token_ms) first_token_ms[i] = r.first_token;
        if (finish_ms) finish_ms[i] = r.finish;
        if (server) server[i] = r.first_server;
        if (decode_server) decode_server[i] = r.decode_server;
    }
    *summary = sim.sum;
}

extern "C" ps_status ps_sim_run(const ps_profile* profile, const ps_sim_config* cfg, const ps_sim_request* requests, int32_t n,
                                uint8_t* attained, double* first_token_ms, double* finish_ms, int32_t* server,
                                int32_t* decode_server, ps_sim_summary* summary) {
    if (!profile || !cfg || n < 0 || (n > 0 && !requests) || !summary) return PS_EINVAL;
    if (cfg->n_servers < 1 || cfg->n_tiers < 1 || !cfg->tpot_ms || cfg->avg_decode_len < 1 || cfg->check_period_ms < 1 || cfg->max_steps < 0)
        return PS_EINVAL;
    if (cfg->mode != PS_SIM_COLOCATED && cfg->mode != PS_SIM_DISAGGREGATED) return PS_EINVAL;
    if (cfg->mode == PS_SIM_DISAGGREGATED && cfg->prefill_budget < 1) return PS_EINVAL;
    for (int32_t t = 0; t < cfg->n_tiers; t++)
        if (!(cfg->tpot_ms[t] > 0.0) || (t > 0 && !(cfg->tpot_ms[t - 1] < cfg->tpot_ms[t]))) return PS_EINVAL;
    for (int32_t i = 0; i < n; i++) {
        const ps_sim_request& q = requests[i];
        if (q.prompt_len < 1 || q.output_len < 1 || q.tier < 0 || q.tier >= cfg->n_tiers || !(q.ttft_ms > 0.0) || !(q.arrival_ms >= 0.0))
            return PS_EINVAL;
        if (i > 0 && q.arrival_ms < requests[i - 1].arrival_ms) return PS_EINVAL;
    }
    try {
        if (cfg->mode == PS_SIM_COLOCATED) {
            Sim sim(profile, *cfg);
            run_and_report(sim, cfg, requests, n, attained, first_token_ms, finish_ms, server, decode_server, summary);
        } else {
            SimPD sim(profile, *cfg);
            run_and_report(sim, cfg, requests, n, attained, first_token_ms, finish_ms, server, decode_server, summary);
        }
    } catch (const std::bad_alloc&) {
        return PS_ENOMEM;
    }
    return PS_OK;
}
