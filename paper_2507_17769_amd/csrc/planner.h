// Host-side step planner: batch validation, index arrays and the attention work list.
// Pure C++ (no HIP calls), so it also serves host-only contexts.
#pragma once
#include <string>
#include <vector>

#include "ps_common.h"

namespace ps {

struct StepPlan {
    int n_seqs = 0;
    int n_tokens = 0;
    int64_t total_kv = 0;
    std::vector<int32_t> cu_seqlens;  // [n_seqs + 1]
    std::vector<int32_t> positions;   // [T]
    std::vector<int32_t> slots;       // [T]
    std::vector<SeqInfo> seqs;        // [n_seqs]
    std::vector<int32_t> pages;       // flat page lists (only the ceil(kv_len/16) pages in use)
    std::vector<AttnItem> items;        // grouped by worker, in worker order
    std::vector<int32_t> worker_begin;  // [n_workers + 1]
    std::vector<MergeGroup> groups;
    int n_partial_slots = 0;
    int n_partial_items = 0;
};

struct PlanConfig {
    int n_kv_heads = 1;
    int group = 1;             // n_q_heads / n_kv_heads
    int max_position = 0;
    int n_pool_pages = -1;     // < 0: unknown (host-only context without a pool)
    int n_workers = 0;         // attention workers; 0 = one per resident wavefront slot
    int worker_slots = 2048;   // wavefronts of the attention kernel resident at once
    int prefill_tokens = 8;    // query tokens per multi-tile attention item
    int prefill_weight = 3;    // cost of a page pair of a multi-tile item; a single-tile (decode) pair costs 2
};

// Validates the batch (see ps_seq in polystep.h).  On failure returns PS_EINVAL / PS_ERANGE
// with a message in err and leaves plan unspecified.  page_seen is scratch of n_pool_pages
// bytes (all zero on entry and on exit) used to detect shared pages.
ps_status validate_batch(const ps_seq* seqs, int n_seqs, const PlanConfig& cfg, std::vector<uint8_t>& page_seen,
                         std::string& err);

// Fills cu_seqlens / positions / slots / seqs / pages of the plan.  Batch must be valid.
void build_indices(const ps_seq* seqs, int n_seqs, StepPlan& plan);

// Fills items / groups / partial counts.  Requires build_indices.
void build_attention_plan(const PlanConfig& cfg, StepPlan& plan);

}  // namespace ps
