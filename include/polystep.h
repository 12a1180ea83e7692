/*
 * polystep — one mixed-batch serving iteration of a decoder-only transformer on one
 * AMD MI355X (gfx950): a chunk of prefill tokens plus one token per running decode
 * request, over a paged KV cache with 16-token pages.
 *
 * This is the engine iteration that PolyServe's router profiles and schedules
 * (Sec. 2.1 "LLM Inference Workflow": the layer; Sec. 2.4: chunked prefill batches all
 * current decodes with a prefill chunk; Sec. 4.5 "Profile-Based Batch Formation": the
 * router consumes a (batch size, KV cache size) -> iteration time table measured on the
 * engine).  The paper's router owns the request queues and dispatches batches to the
 * engine (Sec. 6.1), which is the shape of this interface: the caller describes a batch,
 * the library runs it.
 *
 * Conventions
 *  - Every call returns ps_status; nothing throws or aborts across this boundary.
 *    ps_last_error() gives a human-readable reason for the last failure.
 *  - "device" pointers are HIP device memory on the context's GPU; "host" pointers are
 *    ordinary process memory.  The caller owns every buffer it passes in; the library owns
 *    the context, its repacked weight copies, the KV pool, allocator state and workspaces.
 *  - All floating-point tensors crossing the boundary are bfloat16 (bits of the upper half
 *    of an IEEE binary32), row-major.  Accumulation is fp32 on the device.
 *  - Calls that launch work are asynchronous on the stream given to ps_create unless
 *    stated otherwise; ps_sync() waits for it.  A context is not thread-safe.
 *  - A batch is validated completely on the host before anything is launched: a failing
 *    call leaves device state untouched.
 */
#ifndef POLYSTEP_H
#define POLYSTEP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ps_ctx ps_ctx;

typedef enum {
    PS_OK = 0,
    PS_EINVAL = 1,  /* null pointer, unsupported shape, malformed batch record          */
    PS_ERANGE = 2,  /* page id / position / layer index outside its range               */
    PS_ENOMEM = 3,  /* KV pool exhausted, or a host/device allocation failed            */
    PS_ESTATE = 4,  /* call out of order: layer not initialised, no KV pool, host-only  */
    PS_EDEVICE = 5  /* a HIP call failed; ps_last_error() carries HIP's message         */
} ps_status;

#define PS_PAGE_SIZE 16
#define PS_N_STAGES 8
#define PS_GRID_MAX_DRAWS 8

/* ps_model_desc.flags */
#define PS_FLAG_HOST_ONLY 1u /* no device is touched: allocator, index and planning calls only */

/* Layer shape (Sec. 5.1 "Model and GPU": a GQA decoder of the LLaMA family).
 * Supported: head_dim 64 or 128; n_q_heads / n_kv_heads in {1,2,4,8,16}; hidden (<= 8192),
 * ffn and n_q_heads*head_dim multiples of 64; page_size 16.  rms_eps <= 0 selects 1e-5. */
typedef struct {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn, n_layers;
    int32_t page_size;    /* must be 16 */
    int32_t max_position; /* largest kv_len any sequence may reach (rotary table size) */
    float rms_eps, rope_base;
    uint32_t flags;
} ps_model_desc;

/* One layer's weights: device pointers, bfloat16, math layout [in][out] row-major, no
 * biases.  w_qkv has the query, key and value column blocks in that order
 * ([hidden][(n_q + 2 n_kv) * head_dim]); w_o [n_q*head_dim][hidden]; w_gate, w_up
 * [hidden][ffn]; w_down [ffn][hidden]; g_attn, g_ffn [hidden] RMSNorm gains. */
typedef struct {
    const void *w_qkv, *w_o, *w_gate, *w_up, *w_down, *g_attn, *g_ffn;
} ps_layer_weights;

/* One sequence of a batch (Sec. 2.4): n_new tokens are fed this step (1 for a decode,
 * the chunk size for a prefill chunk); kv_len is the attended span AFTER the step, the
 * new tokens included, so the cached prefix is kv_len - n_new and a decode with
 * kv_len 1 attends to its own key only.  page_table (host, caller-owned) lists physical
 * page ids: logical position p lives in page page_table[p / 16], slot p % 16.
 * Requirements: n_new >= 1, n_new <= kv_len <= max_position, n_pages >= ceil(kv_len/16),
 * page ids inside the pool, no page shared by two sequences of one batch, req_ids unique. */
typedef struct {
    int64_t req_id;
    int32_t n_new;
    int32_t kv_len;
    const int32_t* page_table;
    int32_t n_pages;
} ps_seq;

/* Per-step measurements.  Stages, summed over layers:
 * 0 RMSNorm(attn)  1 QKV GEMM  2 split sum + RoPE + KV append  3 attention (+ split merge)
 * 4 O GEMM  5 split sum + residual + RMSNorm(ffn)  6 gate/up GEMM + SwiGLU
 * 7 down GEMM, split sum + residual (+ the next layer's RMSNorm) */
typedef struct {
    int32_t n_tokens;        /* sum of n_new */
    int64_t total_kv;        /* sum of kv_len */
    int32_t n_attn_items;    /* work items of the attention launch (per layer) */
    int32_t n_attn_partials; /* of which wrote a split partial */
    float ms_total;          /* first launch to last, HIP events */
    float ms_stage[PS_N_STAGES];
} ps_step_stats;

/* Optional copies of one layer's intermediates, for numerical checks.  Any pointer may be
 * null.  Device buffers, written during ps_step: xn, xn2 [T][hidden] bf16; q [T][n_q][d]
 * bf16 after rotation; attn [T][n_q*d] bf16; x1 [T][hidden] fp32 (input + attention
 * branch); act [T][ffn] bf16 (silu(gate)*up); x_in, x_out [T][hidden] fp32: the residual
 * stream entering and leaving the layer, as kept between layers (x_in is written only for
 * layers > 0, x_out for the last layer only while option "out_f32" is set).  x_in / x_out
 * let one layer of a deep stack be checked on its own: feed x_in and that layer's weights
 * and KV slot to a reference and compare with x_out. */
typedef struct {
    void *xn, *q, *attn, *x1, *xn2, *act, *x_in, *x_out;
} ps_taps;

/* ---- lifetime ------------------------------------------------------------------- */

/* Create a context for `desc` on the current HIP device.  hip_stream is a hipStream_t
 * (null = the default stream) on which all work is enqueued.  With PS_FLAG_HOST_ONLY no
 * HIP call is ever made and every call that needs the device returns PS_ESTATE.
 * Errors: PS_EINVAL (null, unsupported shape), PS_ENOMEM, PS_EDEVICE. */
ps_status ps_create(const ps_model_desc* desc, void* hip_stream, ps_ctx** out);

/* Wait for all work enqueued by this context. */
ps_status ps_sync(ps_ctx* ctx);

/* Free everything the context owns (waits for outstanding work first).  Null is a no-op. */
void ps_destroy(ps_ctx* ctx);

/* Reason for the most recent failing call on ctx (or, with ctx == NULL, of the most
 * recent failing ps_create on this thread).  Never null; valid until the next call. */
const char* ps_last_error(const ps_ctx* ctx);

/* Tuning knobs, mainly for tests: "attn_workers" (number of workers of either kind the attention
 * KV streams are cut across, 0 = share the resident blocks between the kinds; different values cut
 * the streams in different places and must give the same results within rounding),
 * "attn_teams" (> 0: this many four-wavefront teams for the prefill query blocks of a step that also has
 * decodes, the other resident blocks streaming the decodes' KV; 0 = one per CU, more if the teams would
 * outlast the streams), "attn_prefill_weight" (what the planner charges a team for a pair of pages, in
 * units of 100 ns, when it decides whether more than one team per CU is needed; it only moves the cuts),
 * "gemm_split_k" (0 = automatic; the weight-streaming kernel's K splits), "gemm_whole_tiles" (1: the tiled GEMM kernel gives
 * every tile to one block instead of cutting the K loops of a last, partial wave of tiles over all blocks; 2: it cuts
 * every such tail that can be cut, also where the cost model would not; same results up to fp32 summation order), "gemm_tile" (block tile edge of the tiled GEMM kernel, which
 * serves more than 64 tokens: 0 = automatic (the weight-streaming kernel stays in charge up to 96
 * tokens, up to 160 for all projections but the QKV one), 128 or 256), "out_f32" (1: ps_step writes x_out as fp32 [T][hidden],
 * the precision the residual stream is kept in, instead of rounding it to bf16).
 * "only_layer" (l >= 0: ps_step runs layer l alone, x_in -> x_out, as if it were the whole model;
 * -1 = the whole stack.  A benchmark of a single layer loads several copies of it as layers and
 * rotates through them, so that every step streams its weights from HBM and not from a cache
 * that a real stack of layers would have flushed).
 * "time_attention" (N >= 1: bracket the attention kernel launch of every Nth step with HIP
 * events, see ps_attention_times; the two event records cost a few microseconds of stream time),
 * "poison_workspaces" (1: before every step all of the library's workspaces are filled with bfloat16 NaN, so that a kernel
 * reading what the step has not written shows in the output; for tests),
 * "time_gemm" (N >= 1: the same around each of the four projection launches of every layer of every Nth step, see
 * ps_gemm_times).  PS_EINVAL for an unknown name or bad value. */
ps_status ps_set_option(ps_ctx* ctx, const char* name, int64_t value);

/* ---- weights (Sec. 2.1: attention module, O-projection, gated feed-forward) -------- */

/* Copy layer `layer`'s weights into the library's own MFMA-friendly layout (W^T for the
 * GEMMs; gate and up columns interleaved so SwiGLU runs in the GEMM epilogue).  The
 * caller may free its buffers once ps_sync() has returned.  May be called again to
 * replace a layer.  Errors: PS_ERANGE (layer), PS_EINVAL (null pointer), PS_ENOMEM. */
ps_status ps_init_layer(ps_ctx* ctx, int32_t layer, const ps_layer_weights* w);

/* ---- paged KV cache (Sec. 2.1: prefill fills the KV cache, decode extends it) --------- */

/* Allocate a pool of n_pages pages for n_kv_layers physical KV layer slots (layer l uses
 * slot l mod n_kv_layers), zero it, and seed the allocator: the free list is the
 * Fisher-Yates shuffle of 0..n_pages-1 driven by splitmix64(perm_seed) (i from n_pages-1
 * down to 1, j = next() mod (i+1), swap).  Replaces any previous pool and forgets all
 * reservations.  Errors: PS_EINVAL, PS_ENOMEM. */
ps_status ps_kv_alloc(ps_ctx* ctx, int32_t n_pages, int32_t n_kv_layers, uint64_t perm_seed);

/* Make request req_id own ceil(kv_len/16) pages, popping new ones from the front of the
 * free list; writes its whole page list to pages_out[0..*n_out).  All-or-nothing:
 * PS_ENOMEM if the pool cannot cover the growth, PS_ERANGE if cap is too small. */
ps_status ps_kv_reserve(ps_ctx* ctx, int64_t req_id, int32_t kv_len, int32_t* pages_out, int32_t cap, int32_t* n_out);

/* Return req_id's pages to the back of the free list, in hand-out order.  PS_EINVAL if unknown. */
ps_status ps_kv_release(ps_ctx* ctx, int64_t req_id);

/* Number of pages currently on the free list (negative if there is no pool). */
int32_t ps_kv_free_pages(const ps_ctx* ctx);

/* Store / fetch keys and values of logical positions pos0 .. pos0+n-1 of `seq` in KV layer
 * slot `layer mod n_kv_layers`.  k and v are device bf16 [n][n_kv_heads][head_dim], 16-byte aligned; keys
 * are stored as given (the cache holds keys after rotation).  Only seq->page_table and
 * n_pages are used.  Used to load a cached prefix, to snapshot, and as the payload of a
 * prefill->decode hand-off (Sec. 2.4).  Errors: PS_ERANGE (position or page id). */
ps_status ps_kv_write(ps_ctx* ctx, int32_t layer, const ps_seq* seq, int32_t pos0, int32_t n, const void* k, const void* v);
ps_status ps_kv_read(ps_ctx* ctx, int32_t layer, const ps_seq* seq, int32_t pos0, int32_t n, void* k, void* v);

/* ---- the step (Sec. 2.1 layer, Sec. 2.4 mixed batch) ------------------------------- */

/* Run all n_layers layers over the batch.  x_in, x_out: device bf16 [T][hidden] (x_out is
 * fp32 [T][hidden] while option "out_f32" is set),
 * T = sum of n_new, sequences concatenated in the order given; x_out may alias x_in.
 * Between layers, and between the two halves of a layer, the residual stream is kept in
 * fp32; queries, keys and values are rounded to bf16 once, after rotation.
 * Per layer: RMSNorm -> QKV -> rotary embedding on q,k -> append k,v to the pages ->
 * causal attention of each new token over cache positions 0..its own (Softmax(QK^T/sqrt d)V,
 * query head h reading KV head h / (n_q/n_kv)) -> O-projection + residual -> RMSNorm ->
 * silu(gate) * up -> down projection + residual.
 * n_seqs == 0 is a valid empty step (nothing is launched).  With stats != NULL the call
 * records HIP events per stage and returns only after the step has finished.
 * Errors: PS_EINVAL / PS_ERANGE for a malformed batch (see ps_seq), PS_ESTATE if a layer
 * or the pool is missing; on any error nothing has been launched. */
ps_status ps_step(ps_ctx* ctx, const ps_seq* seqs, int32_t n_seqs, const void* x_in, void* x_out, ps_step_stats* stats);

/* The same step for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  ps_step_static runs exactly the kernels of ps_step, but every buffer
 * beyond x_in and x_out (normalised activations, queries, attention output, gated activation, the fp32
 * residual stream, GEMM and attention split partials, the device copy of the step's integer metadata) is a
 * piece of one device array of PS_STATIC_SCRATCH_BYTES that is part of the library image: each GPU the
 * library runs on holds that array from the moment the library is loaded until the process ends.  The call
 * makes no hipMalloc / hipFree / hipHostMalloc and creates no stream or event (the pinned metadata ring and its
 * events are made by ps_create); host-side planning arrays live on the process heap.  Results are
 * bit-identical to ps_step's for the same batch and options.
 * Limits: the buffers of the step must fit the array and its metadata 512 KiB, otherwise PS_ERANGE and nothing
 * is launched (decode batches: an 8B-shaped layer fits 160 one-token sequences, a 70B-shaped one 96; steps with
 * a prefill chunk of hundreds of tokens do not fit; the message states the bytes needed).  No per-stage
 * statistics.  All contexts of a process on one GPU share that GPU's array, which keeps the previous call's
 * contents (the one piece that has to start at zero, the arrival counters of the tiled GEMM, the call clears
 * itself with a fill kernel): static
 * steps that overlap on one GPU -- two contexts on different streams -- race and must be serialised by the
 * caller; steps on one stream are ordered by the stream.  Other errors as ps_step. */
#define PS_STATIC_SCRATCH_BYTES (64u << 20)
ps_status ps_step_static(ps_ctx* ctx, const ps_seq* seqs, int32_t n_seqs, const void* x_in, void* x_out);

/* ---- whole model (Sec. 2.1: a request's tokens go in, the next token comes out) ----- */

/* What surrounds the layer stack.  Device pointers, bf16: embedding [vocab][hidden] (row = token
 * id), g_final [hidden] (gain of the RMS normalisation after the last layer), w_out
 * [hidden][vocab] (output matrix, input-major like the layer weights, no bias).  vocab: a
 * positive multiple of 64, at most 2^20, with vocab * hidden * 2 bytes below 4 GiB. */
typedef struct {
    const void* embedding;
    const void* g_final;
    const void* w_out;
    int32_t vocab;
} ps_head_weights;

/* Copy the head's weights into the library (w_out into the GEMM's operand layout).  The caller
 * may free its buffers once ps_sync() has returned.  May be called again.  Errors: PS_EINVAL,
 * PS_ERANGE, PS_ENOMEM, PS_ESTATE (host-only context). */
ps_status ps_init_head(ps_ctx* ctx, const ps_head_weights* w);

/* One full-model step: token_ids (HOST, [T], concatenated like x_in of ps_step) -> embedding rows
 * -> all layers (as ps_step) -> RMS normalisation of every sequence's LAST new token -> logits =
 * that row times w_out -> the index of the largest logit, the lowest index among equal ones.
 * Outputs are device buffers, any may be null: next_tokens int32 [n_seqs]; logits fp32
 * [n_seqs][vocab]; hidden fp32 [T][hidden] (output of the last layer, before the normalisation).
 * stats as in ps_step (layer stages only).  ms_parts: HOST float[3] or null; when given, HIP events
 * time the embedding gather, the layer stack and the head (normalisation + output projection +
 * greedy pick), and the call returns only after the step has finished.
 * Errors: as ps_step; PS_ESTATE without ps_init_head or while option "only_layer" is set;
 * PS_ERANGE for a token id outside [0, vocab). */
ps_status ps_step_tokens(ps_ctx* ctx, const ps_seq* seqs, int32_t n_seqs, const int32_t* token_ids, int32_t* next_tokens,
                         float* logits, float* hidden, ps_step_stats* stats, float* ms_parts);

/* Integer side of a step, host only, no launch: cu_seqlens [n_seqs+1] (exclusive scan of
 * n_new), positions [T] (kv_len - n_new + i), slot_mapping [T] (page id * 16 + position
 * % 16): the cache slots the step's KV append writes.  Output arrays are host memory; any
 * may be null.  Same validation as ps_step (the pool-size check is skipped when no pool exists). */
ps_status ps_step_indices(ps_ctx* ctx, const ps_seq* seqs, int32_t n_seqs, int32_t* cu_seqlens, int32_t* positions, int32_t* slot_mapping);

/* The attention work list the step would launch, host only.  Each item is 8 int32:
 * {seq index, kv head, first new-token index of its query block, number of query tokens,
 *  first KV page (logical), one past last KV page, partial slot or -1 when the item
 *  writes final output, worker}.  Items are listed worker by worker.  Query blocks of sequences with more
 * new tokens than one 16-row tile holds (16 / (n_q_heads / n_kv_heads)) belong to teams (blocks of four
 * wavefronts; twelve tiles per item), which come first; the others to single wavefronts.  Within either
 * kind every worker's items carry (nearly) the same number of KV pages.  Writes min(*n_items, cap) items. */
ps_status ps_plan_attention(ps_ctx* ctx, const ps_seq* seqs, int32_t n_seqs, int32_t* items, int32_t cap, int32_t* n_items);

/* Durations (ms) of the attention kernel launches (one per layer per step, split merge
 * excluded) recorded since the previous call while option "time_attention" was on; at most
 * 2048 are kept.  Waits for the stream.  Writes min(count, cap) values to ms (host) and the
 * number written to *n.  This is the kernel the roofline of a decode-heavy step is quoted on
 * (Sec. 2.2: decode attention does not batch; its cost follows the KV bytes read). */
ps_status ps_attention_times(ps_ctx* ctx, float* ms, int32_t cap, int32_t* n);

/* Durations (ms) of the four projection launches of a layer (QKV, O, gate/up + SwiGLU, down, in that order; the
 * kernels that sum their split partials are not included) recorded since the previous call while option
 * "time_gemm" was on: one record of four values per layer of every timed step, at most 1024 records are kept.
 * Waits for the stream.  Writes min(count, cap) records to ms (host, [cap][4]) and their number to *n.  These are
 * the kernels the roofline of a prefill-heavy step is quoted on (Sec. 2.2: large token batches make the
 * projections compute-bound). */
ps_status ps_gemm_times(ps_ctx* ctx, float* ms, int32_t cap, int32_t* n);

/* Measurement support, not a step of the path: what the device sustains while every SIMD issues
 * back-to-back dense bf16 MFMAs with no memory traffic.  The nominal matrix peak assumes the
 * maximum shader clock; under matrix load the power management settles lower, and the fractions
 * of peak reported for the projections (Sec. 2.2: prefill and large batches are compute-bound)
 * are quoted against both.  Launches blocks of four wavefronts, wavefronts_per_simd (1, 2 or 4)
 * blocks per compute unit; each wavefront issues mfma_per_wavefront (4096 .. 2^22, rounded down to
 * a multiple of 4) independent 32x32x16 MFMAs.  Allocates and frees a few hundred KiB of device
 * memory, runs on the context's stream and waits for it.  *out is host memory. */
typedef struct ps_clock_reading {
    double shader_mhz;      /* shader-clock ticks per microsecond of the constant-rate wall clock, mean over blocks */
    double ticks_per_mfma;  /* shader-clock ticks per MFMA as a wavefront saw them (32 = back to back, alone on its SIMD) */
    double mfma_tflops;     /* 2*32*32*16 flop x MFMAs issued on the device / elapsed time between HIP events */
    double elapsed_ms;
    int32_t compute_units;
    int32_t wavefronts_per_simd;
} ps_clock_reading;
ps_status ps_clock_under_load(ps_ctx* ctx, int32_t mfma_per_wavefront, int32_t wavefronts_per_simd, ps_clock_reading* out);

/* Measurement support, not a step of the path: the rate at which plain vector loads stream a
 * buffer of `bytes` (a multiple of 16 KiB, 1 GiB .. 8 GiB: several times the last-level cache, so
 * that every pass comes from HBM) -- the ceiling for decode attention, whose cost is the KV bytes
 * it reads (Sec. 2.2).  The buffer is allocated, filled once, read `passes` (1 .. 16) times
 * between two HIP events on the context's stream, and freed; *gb_per_s (host) = bytes * passes /
 * elapsed / 1e9. */
ps_status ps_hbm_read_rate(ps_ctx* ctx, int64_t bytes, int32_t passes, double* gb_per_s);

/* Ask subsequent steps to copy layer `layer`'s intermediates; taps == NULL switches it off. */
ps_status ps_set_taps(ps_ctx* ctx, int32_t layer, const ps_taps* taps);

/* ---- latency profile (Sec. 4.5: the (batch size, KV cache size) -> time map) -------- */

/* One cell of the grid: a prefill chunk of `chunk` tokens (0 = none) plus n_decode decode
 * tokens, timed for n_draws (<= PS_GRID_MAX_DRAWS) draws of the lengths: chunk_prefix
 * [n_draws] is the chunk's cached prefix, decode_kv [n_draws][n_decode] the decode KV
 * lengths after the step (host arrays drawn by the caller). */
typedef struct {
    int32_t chunk, n_decode, n_draws;
    const int32_t* chunk_prefix;
    const int32_t* decode_kv;
} ps_grid_cell_spec;

typedef struct {
    int32_t warmup; /* untimed steps per draw */
    int32_t iters;  /* timed steps per draw; the draw's time is their median */
} ps_grid_opts;

typedef struct {
    int32_t chunk, n_decode, n_tokens, n_draws;
    int64_t total_kv;               /* of the median draw */
    float median_ms;                /* median over draws of the per-draw median step time */
    float stage_ms[PS_N_STAGES];    /* per-stage times of the median draw */
    float draw_ms[PS_GRID_MAX_DRAWS];
    int64_t draw_total_kv[PS_GRID_MAX_DRAWS];
} ps_grid_cell;

/* Time every cell.  Pages for the synthetic requests come from the context's allocator
 * and are released again; x_in / x_out are device bf16 [max tokens of any cell][hidden]
 * scratch supplied by the caller (x_in's contents are the activations used).  Synchronous.
 * Errors: PS_ENOMEM if the free pages cannot hold a cell, plus ps_step's. */
ps_status ps_profile_grid(ps_ctx* ctx, const ps_grid_cell_spec* cells, int32_t n_cells, const ps_grid_opts* opts,
                          const void* x_in, void* x_out, ps_grid_cell* out);

#ifdef __cplusplus
}
#endif
#endif /* POLYSTEP_H */
