/* polysched: host-side consumers of the latency profile that polystep measures.
 *
 * These are the decisions the paper's router takes with the (batch size, KV cache size) -> time
 * table (Sec. 4.5 "Profile-Based Batch Formation", Sec. 4.6 "Wait-Time-Aware Scheduling",
 * Sec. 4.7 "Handling TTFT", Sec. 3.4 batch-size limits, Sec. 3.5 cost of a request), and the cluster
 * simulation the paper evaluates its router with (Sec. 5.1).  Plain C, host memory only, no GPU work,
 * no global state; a profile object is immutable after creation and may be shared by threads.
 * All times are milliseconds.  Functions return PS_OK or PS_EINVAL (null pointer, malformed
 * argument) and leave their outputs untouched on error. */
#ifndef POLYSCHED_H
#define POLYSCHED_H

#include "polystep.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ps_profile ps_profile;

/* Build the table: batch_sizes [n_batch] and kv_sizes [n_kv] strictly ascending, ms [n_batch][n_kv]
 * row-major (ms[i * n_kv + j] for batch_sizes[i], kv_sizes[j]).  The arrays are copied.
 * PS_EINVAL for empty or unsorted axes or a non-finite time; PS_ENOMEM. */
ps_status ps_profile_create(const int32_t* batch_sizes, int32_t n_batch, const int64_t* kv_sizes, int32_t n_kv,
                            const float* ms, ps_profile** out);
void ps_profile_destroy(ps_profile* p);

/* (batch size, KV cache size) -> time (Sec. 4.5): bilinear interpolation between profiled points;
 * below the first point of an axis the first point's value, beyond the last point the last
 * interval extended linearly.  Returns NaN for a null profile. */
double ps_profile_lookup(const ps_profile* p, double batch, double kv);

/* A request running on a server: its KV cache length now and the tokens it has generated. */
typedef struct {
    int32_t kv_len;
    int32_t generated;
} ps_running_req;

/* Sec. 4.5: simulate future iterations with every request predicted to generate avg_decode_len
 * tokens in total (a request at or past that is predicted to generate one more), each growing
 * by one token per iteration until it finishes; *max_kv = the largest total KV cache size attended
 * in one iteration, *n_iters = iterations simulated.  new_prompt_len < 0: no new request. */
ps_status ps_max_future_kv(const ps_running_req* running, int32_t n_running, int32_t new_prompt_len, int32_t avg_decode_len,
                           int64_t* max_kv, int32_t* n_iters);

/* Sec. 4.5 + 4.6: *predicted_ms = T(n_running + 1, largest future KV size) + wait_ms (the time the
 * request would wait for the server's current iteration); *admit = predicted < tpot_ms. */
ps_status ps_predict_admit(const ps_profile* p, const ps_running_req* running, int32_t n_running, int32_t new_prompt_len,
                           int32_t avg_decode_len, double tpot_ms, double wait_ms, int32_t* admit, double* predicted_ms,
                           int64_t* max_kv);

/* Sec. 4.7, prefill instance.  prompts [n]: remaining prompt lengths in arrival order; budget:
 * token budget of an iteration; first_iteration_used: tokens of other work already in the first
 * iteration (0..budget).  Iterations are filled first come first served; a request is finished in
 * the current iteration if it fits the room left, or (dynamic != 0) if the iteration then stays
 * below twice the budget, which closes the iteration to further requests; otherwise it gets the
 * room left.  Output: chunks as triples {iteration, request, tokens} in order, at most cap triples
 * written, *n_chunks = the number there are, *n_iterations = iterations used. */
ps_status ps_chunk_plan(const int32_t* prompts, int32_t n, int32_t budget, int32_t dynamic, int32_t first_iteration_used,
                        int32_t* chunks, int32_t cap, int32_t* n_chunks, int32_t* n_iterations);

/* Sec. 4.7, co-location.  The chunk size predicted at scheduling time is the largest c in [1, prompt_len]
 * that can be kept for all ceil(prompt / c) iterations of the prefill: every one of them stays below tpot_ms
 * while the chunks attend a growing prefix and every running decode grows by one token per iteration (and
 * leaves when predicted finished).  *admit = such a c exists and wait_ms + the sum of those iteration times
 * (= *first_token_ms) stays below ttft_ms.  No chunk size can be kept: *admit = 0, *chunk = *n_iters = 0,
 * *first_token_ms = +inf. */
ps_status ps_predict_chunked_prefill(const ps_profile* p, const ps_running_req* running, int32_t n_running, int32_t prompt_len,
                                     int32_t avg_decode_len, double tpot_ms, double ttft_ms, double wait_ms, int32_t* admit,
                                     int32_t* chunk, int32_t* n_iters, double* first_token_ms);

/* Sec. 3.4.  Decode instance of a prefill-decode disaggregated deployment: the largest batch size
 * B <= b_max with T(B, B (p + d/2)) < tpot_ms and B (p + d/2) < capacity (KV tokens); 0 if none. */
int32_t ps_batch_limit_pd(const ps_profile* prof, double p, double d, double tpot_ms, double capacity, int32_t b_max);
/* Co-location with chunked prefill: the largest token batch size B <= b_max with
 * T_iter = T(B, d/(p+d) B (p + d/2) + p) < tpot_ms, (p+d)/B * T_iter < ttft_ms and that KV size
 * below capacity; 0 if none. */
int32_t ps_batch_limit_co(const ps_profile* prof, double p, double d, double tpot_ms, double ttft_ms, double capacity, int32_t b_max);

/* Sec. 3.5: cost of serving one request (prompt p, output d), in instance-milliseconds.  The table's two axes are
 * taken apart as in the cost model of Sec. 3.4: GEMM(B) = T(B, smallest profiled KV size), DcAttn(kv) =
 * T(smallest profiled batch, kv) - T(smallest profiled batch, smallest profiled KV size), PF(p) = DcAttn(p).
 *   disaggregated: p GEMM(b_pf)/b_pf + PF(p) + d GEMM(b_dc)/b_dc + DcAttn(d (p + d/2))
 *   co-located:    (p + d) GEMM(b)/b + PF(p) + DcAttn(d (p + d/2))
 * NaN for a null profile or a non-positive batch size. */
double ps_cost_pd(const ps_profile* prof, double p, double d, double b_pf, double b_dc);
double ps_cost_co(const ps_profile* prof, double p, double d, double b);
/* The same at the batch limits above (the minimal cost of Sec. 3.5); +inf if no batch size satisfies them. */
double ps_optimal_cost_pd(const ps_profile* prof, double p, double d, double tpot_ms, double capacity, double b_pf, int32_t b_max);
double ps_optimal_cost_co(const ps_profile* prof, double p, double d, double tpot_ms, double ttft_ms, double capacity, int32_t b_max);

/* ---- Cluster simulation (Sec. 5.1) of the router of Sec. 4 on co-located instances --------------
 *
 * Instances advance in steps of 1 ms; an iteration's duration is the profile's value for (tokens in the
 * iteration, KV tokens attended).  In every step, in this order: iterations whose end time has been
 * reached deliver their tokens at that end time; arrived requests join the queue of their tier; every
 * check_period_ms steps the scale-down check runs; the queues are served, tightest tier first, first come
 * first served; instances outside an iteration that hold requests start one, at the end time of their
 * previous iteration if that ended within this step (iterations run back to back; only the router works on
 * the 1 ms grid), else at the step.
 * An iteration holds one token per request in decode and the next chunk of the one request in prefill (an
 * instance takes a new request only while no prefill is in progress on it); the prefill's last chunk
 * produces token 0, a request with output_len d then takes d - 1 decode iterations.  Token i is due at
 * arrival + TTFT + i * (the request's own TPOT) (Sec. 2.3); a request is attained if every token is.
 * Placement (Sec. 4.3, 4.4): the request's own cluster, then the clusters of tighter tiers from the
 * nearest one (lazy promotion), each from the instance with most requests down, then scale-up (a parked
 * instance whose tightest request is of this tier, else an instance from the idle pool); an instance
 * admits the request if ps_predict_chunked_prefill admits it against the instance's TPOT, the time left to
 * the first-token deadline and the wait for the iteration in flight, ps_predict_admit keeps the largest
 * future KV size's iteration below that TPOT, and that KV size is below kv_capacity.  A request that cannot
 * be placed keeps its place in the queue while it could still make its first token on an empty instance
 * and is dropped (not attained, never served) once it could not.
 * Scale-down check, per cluster: the instance with fewest requests returns to the idle pool if empty and
 * is parked if none of its requests is of the cluster's tier; a parked instance takes no requests and
 * returns to the pool once empty.  cost_ms = instance time outside the idle pool (Sec. 5.4).
 *
 * PS_SIM_DISAGGREGATED differs as follows.  Prefill runs on a cluster of its own, shared by all tiers:
 * queued requests are taken in order of arrival + TTFT (Sec. 4.2); a prefill instance forms its iterations
 * with ps_chunk_plan (dynamic, prefill_budget) over its requests in admission order; a request goes to the
 * prefill instance with most unprocessed prompt tokens on which the plan with the request added (the wait
 * for the iteration in flight plus the planned iterations) gives the request its first token before its
 * deadline and still gives every request already queued there its own in time, else to an instance from
 * the idle pool.  The prefill's end delivers token 0
 * and queues the request for decoding (the transfer takes no time); decode clusters work as above except
 * that an instance admits the request if ps_predict_admit keeps the largest future KV size's iteration
 * below the instance's TPOT, that KV size is below kv_capacity, and the wait for the iteration in flight
 * plus that iteration time is before the second token's deadline, arrival + TTFT + TPOT (Sec. 4.6).  Step
 * order: ended iterations, arrivals, scale-down check (also returning the least loaded prefill instance if
 * it holds no request), decode queues, prefill queue, iteration starts.  A queued request is dropped once
 * an empty instance could no longer meet its next deadline (first token before prefill, second after). */
enum { PS_SIM_COLOCATED = 0, PS_SIM_DISAGGREGATED = 1 };

typedef struct {
    int32_t mode;             /* PS_SIM_COLOCATED or PS_SIM_DISAGGREGATED */
    int32_t n_servers;
    int32_t n_tiers;
    const double* tpot_ms;    /* [n_tiers], strictly ascending */
    int32_t avg_decode_len;   /* the router's output-length prediction (Sec. 4.5) */
    double kv_capacity;       /* KV tokens per instance */
    int32_t check_period_ms;
    int64_t max_steps;        /* the run stops after this many steps even if requests are unfinished */
    int32_t prefill_budget;   /* disaggregated: token budget of a prefill iteration (Sec. 4.7) */
} ps_sim_config;

typedef struct {
    double arrival_ms;
    int32_t prompt_len, output_len;
    double ttft_ms;
    int32_t tier;
} ps_sim_request;

typedef struct {
    int64_t end_ms;           /* steps simulated */
    double cost_ms;
    int64_t scale_ups, scale_downs, promotions, dropped;
    int64_t iterations;       /* instance iterations completed */
    int64_t admission_tests;  /* (request, instance) pairs examined by the router */
} ps_sim_summary;

/* requests [n] sorted by arrival.  Per-request outputs (each may be null): attained (0/1), time of the
 * first token and of the last one (-1 if never produced), the instance that ran the prefill and the one
 * that ran the decode iterations (the same when co-located; -1 if never placed).  PS_EINVAL for malformed
 * arguments; PS_ENOMEM. */
ps_status ps_sim_run(const ps_profile* profile, const ps_sim_config* cfg, const ps_sim_request* requests, int32_t n,
                     uint8_t* attained, double* first_token_ms, double* finish_ms, int32_t* server, int32_t* decode_server,
                     ps_sim_summary* summary);

#ifdef __cplusplus
}
#endif
#endif
