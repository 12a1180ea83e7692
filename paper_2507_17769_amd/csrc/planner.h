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
    std::vector<int32_t> worker_begin;  // [n_workers + 1]; the first n_team_workers workers are teams (blocks of four
                                        // wavefronts), the others single wavefronts
    int n_team_workers = 0;
    std::vector<MergeGroup> groups;
    int n_partial_slots = 0;
    int n_partial_items = 0;
};

struct PlanConfig {
    int n_kv_heads = 1;
    int group = 1;             // n_q_heads / n_kv_heads
    int max_position = 0;
    int n_pool_pages = -1;     // < 0: unknown (host-only context without a pool)
    int n_workers = 0;         // workers of each kind; 0 = share the resident blocks between the kinds by cost
    int n_teams = 0;           // > 0: this many teams when a step has both kinds of work (0 = by cost)
    int block_slots = 512;     // blocks (of four wavefronts) of the attention kernel resident at once
    int prefill_tokens = 32;   // query tokens per team item (all its tiles)
    // cost model behind the split of the blocks: nanoseconds a team spends on a pair of pages while it has its CU's
    // matrix units to itself and the streams keep HBM busy, the relative growth of that when two teams share every CU, HBM time of a pair streamed
    // by a single wavefront (all of them together), time a lone wavefront needs for a pair
    double team_pair_ns = 2200.0, team_crowding = 0.85, hbm_pair_ns = 2.75, wave_pair_ns = 2000.0;
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
