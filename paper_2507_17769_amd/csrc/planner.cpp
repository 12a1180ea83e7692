// Host-side step planner (no HIP calls): validates a batch, builds the integer arrays of a
// step and the attention work list.  A batch holds every running decode request (one new token
// each) and a chunk of prefill tokens in the capacity that is left (Sec. 2.4); each sequence
// carries its own page table into the 16-token paged KV cache.
#include "planner.h"

#include <algorithm>
#include <unordered_set>

namespace ps {

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

ps_status validate_batch(const ps_seq* seqs, int n_seqs, const PlanConfig& cfg, std::vector<uint8_t>& page_seen,
                         std::string& err) {
    if (n_seqs < 0) { err = "n_seqs is negative"; return PS_EINVAL; }
    if (n_seqs > 0 && !seqs) { err = "seqs is null"; return PS_EINVAL; }
    const bool have_pool = cfg.n_pool_pages >= 0;
    if (have_pool && (int)page_seen.size() < cfg.n_pool_pages) page_seen.assign(cfg.n_pool_pages, 0);
    std::unordered_set<int32_t> pages_nopool;
    static thread_local std::vector<int32_t> marked;  // pages flagged in page_seen, cleared again before returning
    static thread_local std::vector<int64_t> ids;
    marked.clear();
    ids.clear();
    int64_t tokens = 0;
    ps_status rc = PS_OK;
    auto who = [&](int s) { return "seq " + std::to_string(s) + " (req " + std::to_string(seqs[s].req_id) + "): "; };
    for (int s = 0; s < n_seqs && rc == PS_OK; s++) {
        const ps_seq& q = seqs[s];
        if (q.n_new < 1) { err = who(s) + "n_new must be >= 1"; rc = PS_EINVAL; break; }
        if (q.kv_len < q.n_new) { err = who(s) + "kv_len is smaller than n_new"; rc = PS_EINVAL; break; }
        if (q.kv_len > cfg.max_position) { err = who(s) + "kv_len exceeds max_position"; rc = PS_ERANGE; break; }
        if (!q.page_table) { err = who(s) + "page_table is null"; rc = PS_EINVAL; break; }
        if (q.n_pages < ceil_div(q.kv_len, PS_PAGE_SIZE)) { err = who(s) + "page_table is shorter than ceil(kv_len/16)"; rc = PS_EINVAL; break; }
        ids.push_back(q.req_id);
        tokens += q.n_new;
        if (tokens > (1 << 24)) { err = "batch has more than 2^24 new tokens"; rc = PS_ERANGE; break; }
        for (int i = 0; i < q.n_pages; i++) {
            const int32_t pg = q.page_table[i];
            if (pg < 0 || (have_pool && pg >= cfg.n_pool_pages)) {
                err = who(s) + "page id " + std::to_string(pg) + " outside the pool";
                rc = PS_ERANGE;
                break;
            }
            bool dup;
            if (have_pool) {
                dup = page_seen[pg] != 0;
                if (!dup) { page_seen[pg] = 1; marked.push_back(pg); }
            } else {
                dup = !pages_nopool.insert(pg).second;
            }
            if (dup) {
                err = who(s) + "page id " + std::to_string(pg) + " appears twice in the batch";
                rc = PS_EINVAL;
                break;
            }
        }
    }
    for (int32_t pg : marked) page_seen[pg] = 0;
    if (rc == PS_OK && n_seqs > 1) {
        std::sort(ids.begin(), ids.end());
        const auto dup = std::adjacent_find(ids.begin(), ids.end());
        if (dup != ids.end()) {
            int s = 0, seen = 0;
            for (int i = 0; i < n_seqs; i++)
                if (seqs[i].req_id == *dup && ++seen == 2) { s = i; break; }
            err = who(s) + "duplicate req_id in batch";
            rc = PS_EINVAL;
        }
    }
    return rc;
}

void build_indices(const ps_seq* seqs, int n_seqs, StepPlan& plan) {
    plan.n_seqs = n_seqs;
    plan.cu_seqlens.assign(n_seqs + 1, 0);
    plan.seqs.resize(n_seqs);
    plan.pages.clear();
    plan.total_kv = 0;
    int T = 0;
    for (int s = 0; s < n_seqs; s++) {
        const int used = ceil_div(seqs[s].kv_len, PS_PAGE_SIZE);
        plan.seqs[s] = SeqInfo{T, seqs[s].n_new, seqs[s].kv_len, (int32_t)plan.pages.size()};
        plan.pages.insert(plan.pages.end(), seqs[s].page_table, seqs[s].page_table + used);
        T += seqs[s].n_new;
        plan.cu_seqlens[s + 1] = T;
        plan.total_kv += seqs[s].kv_len;
    }
    plan.n_tokens = T;
    plan.positions.resize(T);
    plan.slots.resize(T);
    for (int s = 0; s < n_seqs; s++) {
        const int prefix = seqs[s].kv_len - seqs[s].n_new;
        int32_t* pos = plan.positions.data() + plan.cu_seqlens[s];
        int32_t* slot = plan.slots.data() + plan.cu_seqlens[s];
        for (int i = 0; i < seqs[s].n_new; i++) {
            const int p = prefix + i;
            pos[i] = p;
            slot[i] = seqs[s].page_table[p / PS_PAGE_SIZE] * PS_PAGE_SIZE + p % PS_PAGE_SIZE;
        }
    }
}

// Attention plan.  The KV stream of every (sequence, kv head, query block) is a segment of page
// pairs; a decode token's cost is the bytes of its KV span (Sec. 2.2, 3.4: decode attention does
// not batch, it scales with the KV tokens read).  Instead of fixed-size splits handed out
// dynamically, the concatenation of all segments is cut into runs of equal weight, one per worker,
// so that all workers stream for the same time and the launch has no tail.  A run that ends inside
// a segment leaves a partial; a merge pass combines the partials.
//
// There are two kinds of worker, each with its own pool of segments.  Query blocks of more than one
// tile (prefill chunks, Sec. 2.4) go to teams: a block of four wavefronts that shares every pair of
// pages through LDS and is bound by the matrix units.  Single-tile blocks (decodes) go to single
// wavefronts, which are bound by HBM.  All blocks of the launch are resident at once; how many of
// them work as teams: all of them in a step without decodes; otherwise one per CU, and more only if
// the teams would outlast the streams (a team's time is its page pairs times a cost that grows once
// two teams share a CU, the wavefronts' time is the larger of the HBM time of all their pairs and of
// the per-wavefront time when few wavefronts are left).
void build_attention_plan(const PlanConfig& cfg, StepPlan& plan) {
    plan.items.clear();
    plan.groups.clear();
    plan.worker_begin.clear();
    plan.n_partial_slots = 0;
    plan.n_partial_items = 0;
    plan.n_team_workers = 0;
    const int TQ = 16 / cfg.group;                 // tokens per 16-row query tile
    const int multi_nt = cfg.prefill_tokens / TQ;  // tiles a team item always reserves
    const int W_SINGLE = 2, W_MULTI = 3;           // nominal weight of a page pair (the pools are cut separately)

    struct Segment { int seq, q0, qn, np, w; };
    std::vector<Segment> segs_team, segs_wave;
    int64_t units_team = 0, units_wave = 0;
    for (int si = 0; si < plan.n_seqs; si++) {
        const SeqInfo& sq = plan.seqs[si];
        const int prefix = sq.kv_len - sq.n_new;
        const int qb = sq.n_new <= TQ ? TQ : cfg.prefill_tokens;
        for (int q0 = 0; q0 < sq.n_new; q0 += qb) {
            const int qn = std::min(qb, sq.n_new - q0);
            const int np = ceil_div(prefix + q0 + qn, PS_PAGE_SIZE);
            if (sq.n_new <= TQ) {
                segs_wave.push_back(Segment{si, q0, qn, np, W_SINGLE});
                units_wave += (int64_t)ceil_div(np, 2) * W_SINGLE * cfg.n_kv_heads;
            } else {
                segs_team.push_back(Segment{si, q0, qn, np, W_MULTI});
                units_team += (int64_t)ceil_div(np, 2) * W_MULTI * cfg.n_kv_heads;
            }
        }
    }
    plan.worker_begin.push_back(0);
    if (segs_team.empty() && segs_wave.empty()) return;

    // how many workers each pool gets
    int n_team = 0, n_wave = 0;
    if (cfg.n_workers > 0) {
        n_team = segs_team.empty() ? 0 : cfg.n_workers;
        n_wave = segs_wave.empty() ? 0 : cfg.n_workers;
    } else {
        const int B = std::max(1, cfg.block_slots);
        const double pairs_team = (double)units_team / W_MULTI, pairs_wave = (double)units_wave / W_SINGLE;
        if (segs_team.empty()) {
            n_wave = 4 * B;
        } else if (segs_wave.empty()) {
            n_team = B;
        } else if (cfg.n_teams > 0) {
            n_team = std::min(cfg.n_teams, B - 1);
            n_wave = 4 * (B - n_team);
        } else {
            // One team per CU, next to a block of streaming wavefronts: half the blocks' wavefronts already keep HBM busy,
            // and a team that finishes early costs nothing.  More teams (two on some CUs, which slows both) only when the
            // teams would otherwise outlast the streams.
            auto cost = [&](int t) {
                const double crowd = t <= B / 2 ? 0.0 : (double)(t - B / 2) / (B / 2);
                const double t_team = pairs_team * cfg.team_pair_ns * (1.0 + cfg.team_crowding * crowd) / t;
                const double t_wave = std::max(pairs_wave * cfg.hbm_pair_ns, pairs_wave * cfg.wave_pair_ns / (4.0 * (B - t)));
                return std::max(t_team, t_wave);
            };
            n_team = std::max(1, B / 2);
            double best = cost(n_team);
            for (int t = n_team + 1; t < B; t++)
                if (cost(t) < 0.98 * best) { best = cost(t); n_team = t; }
            n_wave = 4 * (B - n_team);
            // Few decodes beside a large chunk: no more wavefronts than keep the streams inside the teams' time with a
            // margin, so that a short stream is not cut into hundreds of pieces for the merge to put together again.
            const double crowd = n_team <= B / 2 ? 0.0 : (double)(n_team - B / 2) / (B / 2);
            const double t_team = pairs_team * cfg.team_pair_ns * (1.0 + cfg.team_crowding * crowd) / n_team;
            const double need = 2.0 * pairs_wave * cfg.wave_pair_ns / std::max(t_team, 1.0);
            if (need < n_wave) n_wave = std::max(8, (int)need);
        }
    }
    // do not spread thinner than ~4 page pairs per worker
    if (n_team > 0) n_team = (int)std::max<int64_t>(1, std::min<int64_t>(n_team, units_team / (4 * W_MULTI)));
    if (n_wave > 0) n_wave = (int)std::max<int64_t>(1, std::min<int64_t>(n_wave, units_wave / (4 * W_SINGLE)));
    plan.n_team_workers = n_team;
    plan.worker_begin.reserve(n_team + n_wave + 1);
    plan.items.reserve(n_team + n_wave + (segs_team.size() + segs_wave.size()) * cfg.n_kv_heads);

    auto cut_pool = [&](const std::vector<Segment>& segs, int64_t units, int n_workers) {
        if (segs.empty()) return;
        const int base = (int)plan.worker_begin.size() - 1;   // global id of the pool's first worker
        // worker w ends where the cumulative weight reaches (w+1) * units / n_workers, so rounding
        // to whole pairs never accumulates
        const int64_t q_units = units / n_workers, r_units = units % n_workers;
        auto boundary = [&](int w) { return q_units * (w + 1) + r_units * (w + 1) / n_workers; };
        int worker = 0;
        int64_t done = 0;                // cumulative weight handed out so far
        int64_t left = boundary(0);      // weight the current worker may still take
        auto next_worker = [&]() {
            if (worker + 1 < n_workers) {
                worker++;
                plan.worker_begin.push_back((int32_t)plan.items.size());
                left = boundary(worker) - done;
            } else {
                left = INT64_MAX / 4;  // whatever is left belongs to the last worker
            }
        };
        // KV-head-major order: every head carries the same total weight, so with n_kv_heads a multiple of
        // the number of L2 domains each domain's contiguous share of the workers (see attn_kernel) streams
        // whole heads, and the query blocks of a prefill chunk that re-read one head's keys share an L2.
        for (int h = 0; h < cfg.n_kv_heads; h++) {
            for (const Segment& sg : segs) {
                const SeqInfo& sq = plan.seqs[sg.seq];
                const int n_pairs = ceil_div(sg.np, 2);
                const int nt_alloc = sq.n_new <= TQ ? 1 : multi_nt;
                const int n_tiles = ceil_div(sg.qn, TQ);
                const size_t first = plan.items.size();
                int pair = 0;
                while (pair < n_pairs) {
                    int take = (int)std::min<int64_t>(n_pairs - pair, left / sg.w);
                    if (take <= 0) {
                        // quota smaller than one pair: hand over, unless the worker is still empty
                        if ((int)plan.items.size() > plan.worker_begin.back()) { next_worker(); continue; }
                        take = 1;
                    }
                    plan.items.push_back(AttnItem{sg.seq, h, sg.q0, sg.qn, 2 * pair, std::min(sg.np, 2 * (pair + take)), -1,
                                                  base + worker, sq.tok0 + sg.q0, sq.kv_len - sq.n_new + sg.q0, sq.page_off,
                                                  plan.pages[sq.page_off + 2 * pair],
                                                  plan.pages[sq.page_off + std::min(2 * pair + 1, sg.np - 1)], 0, 0, 0});
                    pair += take;
                    left -= (int64_t)take * sg.w;
                    done += (int64_t)take * sg.w;
                    if (left < sg.w && pair < n_pairs) next_worker();
                }
                const int n_splits = (int)(plan.items.size() - first);
                if (n_splits > 1) {
                    const int slot0 = plan.n_partial_slots;
                    for (int t = 0; t < n_tiles; t++)
                        plan.groups.push_back(MergeGroup{sq.tok0 + sg.q0 + t * TQ, std::min(TQ, sg.qn - t * TQ), h, slot0 + t,
                                                         n_splits, nt_alloc, 0, 0});
                    for (int j = 0; j < n_splits; j++) plan.items[first + j].partial = slot0 + j * nt_alloc;
                    plan.n_partial_slots += n_splits * nt_alloc;
                    plan.n_partial_items += n_splits;
                }
            }
        }
        // workers that received nothing (possible only through rounding) get empty ranges
        while ((int)plan.worker_begin.size() < base + n_workers + 1) plan.worker_begin.push_back((int32_t)plan.items.size());
        plan.worker_begin.back() = (int32_t)plan.items.size();
    };
    cut_pool(segs_team, units_team, n_team);
    cut_pool(segs_wave, units_wave, n_wave);
}

}  // namespace ps
