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
    std::unordered_set<int64_t> ids;
    std::unordered_set<int32_t> pages_nopool;
    std::vector<int32_t> marked;  // pages flagged in page_seen, cleared again before returning
    ids.reserve(n_seqs * 2);
    int64_t tokens = 0;
    ps_status rc = PS_OK;
    for (int s = 0; s < n_seqs && rc == PS_OK; s++) {
        const ps_seq& q = seqs[s];
        const std::string who = "seq " + std::to_string(s) + " (req " + std::to_string(q.req_id) + "): ";
        if (q.n_new < 1) { err = who + "n_new must be >= 1"; rc = PS_EINVAL; break; }
        if (q.kv_len < q.n_new) { err = who + "kv_len is smaller than n_new"; rc = PS_EINVAL; break; }
        if (q.kv_len > cfg.max_position) { err = who + "kv_len exceeds max_position"; rc = PS_ERANGE; break; }
        if (!q.page_table) { err = who + "page_table is null"; rc = PS_EINVAL; break; }
        if (q.n_pages < ceil_div(q.kv_len, PS_PAGE_SIZE)) { err = who + "page_table is shorter than ceil(kv_len/16)"; rc = PS_EINVAL; break; }
        if (!ids.insert(q.req_id).second) { err = who + "duplicate req_id in batch"; rc = PS_EINVAL; break; }
        tokens += q.n_new;
        if (tokens > (1 << 24)) { err = "batch has more than 2^24 new tokens"; rc = PS_ERANGE; break; }
        for (int i = 0; i < q.n_pages; i++) {
            const int32_t pg = q.page_table[i];
            if (pg < 0 || (have_pool && pg >= cfg.n_pool_pages)) {
                err = who + "page id " + std::to_string(pg) + " outside the pool";
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
                err = who + "page id " + std::to_string(pg) + " appears twice in the batch";
                rc = PS_EINVAL;
                break;
            }
        }
    }
    for (int32_t pg : marked) page_seen[pg] = 0;
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

void build_attention_plan(const PlanConfig& cfg, StepPlan& plan) {
    plan.items.clear();
    plan.groups.clear();
    plan.n_partial_slots = 0;
    plan.n_partial_items = 0;
    const int TQ = 16 / cfg.group;                 // tokens per 16-row query tile
    const int multi_nt = cfg.prefill_tokens / TQ;  // tiles a multi-tile item always reserves

    // total KV pages the launch will stream, to pick the split size
    int split = cfg.split_pages;
    if (split <= 0) {
        int64_t page_heads = 0;
        for (const SeqInfo& sq : plan.seqs) {
            const int qb = sq.n_new <= TQ ? TQ : cfg.prefill_tokens;
            const int prefix = sq.kv_len - sq.n_new;
            for (int q0 = 0; q0 < sq.n_new; q0 += qb)
                page_heads += (int64_t)ceil_div(prefix + std::min(sq.n_new, q0 + qb), PS_PAGE_SIZE) * cfg.n_kv_heads;
        }
        int64_t s = (page_heads + 4095) / 4096;
        s = std::max<int64_t>(8, std::min<int64_t>(64, s));
        split = (int)s;
    }
    split = std::max(2, split + (split & 1));  // even: pages are consumed in pairs

    for (int si = 0; si < plan.n_seqs; si++) {
        const SeqInfo& sq = plan.seqs[si];
        const int prefix = sq.kv_len - sq.n_new;
        const int qb = sq.n_new <= TQ ? TQ : cfg.prefill_tokens;
        for (int q0 = 0; q0 < sq.n_new; q0 += qb) {
            const int qn = std::min(qb, sq.n_new - q0);
            const int nt_alloc = qn <= TQ ? 1 : multi_nt;
            const int n_tiles = ceil_div(qn, TQ);
            const int np = ceil_div(prefix + q0 + qn, PS_PAGE_SIZE);
            int n_splits = ceil_div(np, split);
            int pps = ceil_div(np, n_splits);
            pps += pps & 1;
            n_splits = ceil_div(np, pps);
            for (int h = 0; h < cfg.n_kv_heads; h++) {
                if (n_splits == 1) {
                    plan.items.push_back(AttnItem{si, h, q0, qn, 0, np, -1, -1});
                    continue;
                }
                const int base = plan.n_partial_slots;
                const int g0 = (int)plan.groups.size();
                for (int t = 0; t < n_tiles; t++)
                    plan.groups.push_back(MergeGroup{sq.tok0 + q0 + t * TQ, std::min(TQ, qn - t * TQ), h, base + t,
                                                     n_splits, nt_alloc, 0, 0});
                for (int j = 0; j < n_splits; j++)
                    plan.items.push_back(AttnItem{si, h, q0, qn, j * pps, std::min(np, (j + 1) * pps),
                                                  base + j * nt_alloc, g0});
                plan.n_partial_slots += n_splits * nt_alloc;
                plan.n_partial_items += n_splits;
            }
        }
    }
    // longest first, so the tail of the launch is made of short items
    auto weight = [&](const AttnItem& it) { return (it.page_end - it.page_begin) * (it.q_ntok <= TQ ? 1 : 2 * multi_nt); };
    std::stable_sort(plan.items.begin(), plan.items.end(),
                     [&](const AttnItem& x, const AttnItem& y) { return weight(x) > weight(y); });
}

}  // namespace ps
