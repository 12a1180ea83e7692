// Host code of the library (step planner, profile consumers, cluster simulator) replayed on inputs that the test
// wrote to a file, in a build with AddressSanitizer and UndefinedBehaviorSanitizer (test_host_sanitizers.py).
// Results go to stdout as numbers; the test compares them with what the regular library returns for the same inputs.
//   driver plan <file>     batches -> status, counts and checksums of the index arrays and the attention work list
//   driver sim <file>      table, configuration and trace -> summary and checksums of the per-request outputs
#include <cinttypes>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "planner.h"
#include "../../include/polysched.h"

static uint64_t mix(uint64_t h, uint32_t v) { return h * 1000003ull + v; }

static int run_plan(FILE* f) {
    int n_cases = 0;
    if (fscanf(f, "%d", &n_cases) != 1) return 2;
    std::vector<uint8_t> page_seen;
    ps::StepPlan plan;
    for (int c = 0; c < n_cases; c++) {
        ps::PlanConfig pc;
        int n_seqs = 0, team_weight = 0;
        if (fscanf(f, "%d %d %d %d %d %d %d %d %d", &pc.n_kv_heads, &pc.group, &pc.max_position, &pc.n_pool_pages, &pc.n_workers,
                   &pc.block_slots, &pc.prefill_tokens, &team_weight, &n_seqs) != 9) return 2;
        pc.team_pair_ns = 100.0 * team_weight;
        std::vector<ps_seq> seqs(n_seqs);
        std::vector<std::vector<int32_t>> tables(n_seqs);
        for (int s = 0; s < n_seqs; s++) {
            long long id;
            int n_new, kv_len, n_pages;
            if (fscanf(f, "%lld %d %d %d", &id, &n_new, &kv_len, &n_pages) != 4) return 2;
            tables[s].resize(n_pages > 0 ? n_pages : 0);
            for (int i = 0; i < n_pages; i++)
                if (fscanf(f, "%d", &tables[s][i]) != 1) return 2;
            seqs[s] = ps_seq{id, n_new, kv_len, tables[s].data(), n_pages};
        }
        page_seen.assign(pc.n_pool_pages > 0 ? pc.n_pool_pages : 0, 0);
        std::string err;
        const ps_status st = ps::validate_batch(seqs.data(), n_seqs, pc, page_seen, err);
        if (st != PS_OK) { printf("%d\n", (int)st); continue; }
        ps::build_indices(seqs.data(), n_seqs, plan);
        ps::build_attention_plan(pc, plan);
        uint64_t h_idx = 0, h_items = 0;
        for (int32_t v : plan.cu_seqlens) h_idx = mix(h_idx, (uint32_t)v);
        for (int32_t v : plan.positions) h_idx = mix(h_idx, (uint32_t)v);
        for (int32_t v : plan.slots) h_idx = mix(h_idx, (uint32_t)v);
        for (const ps::AttnItem& it : plan.items) {
            int32_t w[8];
            memcpy(w, &it, sizeof(w));
            for (int i = 0; i < 8; i++) h_items = mix(h_items, (uint32_t)w[i]);
        }
        printf("0 %d %lld %zu %" PRIu64 " %" PRIu64 "\n", plan.n_tokens, (long long)plan.total_kv, plan.items.size(), h_idx, h_items);
    }
    return 0;
}

static int run_sim(FILE* f) {
    int nb = 0, nk = 0;
    if (fscanf(f, "%d %d", &nb, &nk) != 2) return 2;
    std::vector<int32_t> bs(nb);
    std::vector<int64_t> ks(nk);
    std::vector<float> ms((size_t)nb * nk);
    for (auto& v : bs) if (fscanf(f, "%d", &v) != 1) return 2;
    for (auto& v : ks) { long long t; if (fscanf(f, "%lld", &t) != 1) return 2; v = t; }
    for (auto& v : ms) if (fscanf(f, "%f", &v) != 1) return 2;
    ps_profile* prof = nullptr;
    if (ps_profile_create(bs.data(), nb, ks.data(), nk, ms.data(), &prof) != PS_OK) return 3;
    int n_runs = 0;
    if (fscanf(f, "%d", &n_runs) != 1) return 2;
    for (int r = 0; r < n_runs; r++) {
        ps_sim_config cfg{};
        long long max_steps;
        if (fscanf(f, "%d %d %d", &cfg.mode, &cfg.n_servers, &cfg.n_tiers) != 3) return 2;
        std::vector<double> tpots(cfg.n_tiers);
        for (auto& v : tpots) if (fscanf(f, "%lf", &v) != 1) return 2;
        cfg.tpot_ms = tpots.data();
        if (fscanf(f, "%d %lf %d %lld %d", &cfg.avg_decode_len, &cfg.kv_capacity, &cfg.check_period_ms, &max_steps, &cfg.prefill_budget) != 5) return 2;
        cfg.max_steps = max_steps;
        int n = 0;
        if (fscanf(f, "%d", &n) != 1) return 2;
        std::vector<ps_sim_request> reqs(n);
        for (auto& q : reqs)
            if (fscanf(f, "%lf %d %d %lf %d", &q.arrival_ms, &q.prompt_len, &q.output_len, &q.ttft_ms, &q.tier) != 5) return 2;
        std::vector<uint8_t> att(n);
        std::vector<double> first(n), fin(n);
        std::vector<int32_t> srv(n), dsrv(n);
        ps_sim_summary sm{};
        const ps_status st = ps_sim_run(prof, &cfg, reqs.data(), n, att.data(), first.data(), fin.data(), srv.data(), dsrv.data(), &sm);
        if (st != PS_OK) { printf("%d\n", (int)st); continue; }
        uint64_t h = 0;
        for (int i = 0; i < n; i++) {
            uint64_t a, b;
            memcpy(&a, &first[i], 8);
            memcpy(&b, &fin[i], 8);
            h = mix(mix(mix(mix(mix(mix(mix(h, att[i]), (uint32_t)a), (uint32_t)(a >> 32)), (uint32_t)b), (uint32_t)(b >> 32)), (uint32_t)srv[i]), (uint32_t)dsrv[i]);
        }
        printf("0 %lld %.17g %lld %lld %lld %lld %lld %lld %" PRIu64 "\n", (long long)sm.end_ms, sm.cost_ms, (long long)sm.scale_ups, (long long)sm.scale_downs,
               (long long)sm.promotions, (long long)sm.dropped, (long long)sm.iterations, (long long)sm.admission_tests, h);
        // the decisions the router takes one at a time, on this run's first requests
        for (int i = 0; i < n && i < 8; i++) {
            ps_running_req run[3] = {{reqs[i].prompt_len + 5, 5}, {1000, 100}, {17, 1}};
            int32_t admit = 0, chunk = 0, iters = 0;
            double pred = 0, ft = 0;
            int64_t kv = 0;
            ps_predict_admit(prof, run, 3, reqs[i].prompt_len, cfg.avg_decode_len, tpots[reqs[i].tier], 1.5, &admit, &pred, &kv);
            printf("%d %.17g %lld ", admit, pred, (long long)kv);
            ps_predict_chunked_prefill(prof, run, 3, reqs[i].prompt_len, cfg.avg_decode_len, tpots[reqs[i].tier], reqs[i].ttft_ms, 0.5, &admit, &chunk, &iters, &ft);
            printf("%d %d %d %.17g\n", admit, chunk, iters, ft);
        }
    }
    ps_profile_destroy(prof);
    return 0;
}

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* f = fopen(argv[2], "r");
    if (!f) return 2;
    const int rc = !strcmp(argv[1], "plan") ? run_plan(f) : !strcmp(argv[1], "sim") ? run_sim(f) : 2;
    fclose(f);
    return rc;
}
