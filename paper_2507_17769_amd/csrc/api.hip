// C-ABI of libpolystep: context, weights, paged KV pool + allocator, the mixed-batch step and
// the latency-profile grid.  See include/polystep.h for the contract of every entry point.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>

#include "planner.h"
#include "ps_common.h"

namespace ps {

int attn_prefill_tokens_per_item(int G);

struct LayerWeights {
    bf16_t *wqkv_t = nullptr, *wo_t = nullptr, *wgu_t = nullptr, *wd_t = nullptr, *g_attn = nullptr, *g_ffn = nullptr;
    bool ready = false;
};

struct Staging {  // pinned host buffer for one step's metadata
    void* host = nullptr;
    size_t bytes = 0;
};

}  // namespace ps

using namespace ps;

struct ps_ctx {
    ps_model_desc desc{};
    bool host_only = false;
    hipStream_t stream = nullptr;
    std::string err;

    std::vector<LayerWeights> layers;
    float* rope_cs = nullptr;  // [max_position][d/2] (cos, sin)

    // KV pool + allocator
    bf16_t* pool = nullptr;
    int n_pool_pages = -1;
    int n_kv_slots = 0;
    size_t slot_elems = 0;  // elements per physical layer slot
    std::deque<int32_t> free_list;
    std::unordered_map<int64_t, std::vector<int32_t>> owned;
    std::vector<uint8_t> page_seen;

    // workspaces
    int cap_tokens = 0;
    bf16_t *ws_xn = nullptr, *ws_q = nullptr, *ws_attn = nullptr, *ws_act = nullptr;
    float *ws_x1 = nullptr, *ws_xmid = nullptr;
    // model head (ps_init_head): embedding table, final gain, repacked output matrix; its workspaces
    bf16_t *embedding = nullptr, *g_final = nullptr, *wout_t = nullptr;
    int vocab = 0;
    bool head_ready = false;
    bf16_t* ws_embed = nullptr;   // [cap_tokens][hidden] bf16: embedding rows of the step's tokens
    float* ws_final = nullptr;    // [cap_tokens][hidden] fp32: output of the last layer
    float* ws_logits = nullptr;   // fp32 partials of the output projection, [splits][n_seqs][vocab]
    size_t logits_bytes = 0;
    int32_t* ws_next = nullptr;   // [cap] greedy tokens when the caller passes none
    int next_cap = 0;
    hipEvent_t ev_head[4] = {nullptr, nullptr, nullptr, nullptr};
    float* ws_part = nullptr;  // fp32 GEMM partials [splits][T][N], shared by the three projections
    size_t part_bytes = 0;
    size_t act_bytes = 0;
    float *part_o = nullptr, *part_ml = nullptr;
    int cap_part_slots = 0;
    // tiled GEMM: parked accumulators of partial K runs and one counter per tile (zero between launches)
    float* ws_skfrag = nullptr;
    size_t skfrag_bytes = 0;
    int* ws_skcnt = nullptr;
    int skcnt_n = 0;
    // Device copies of the staging ring (same 8 slots).  The copy of step n+1's metadata runs on
    // copy_stream while step n's kernels execute; the main stream only waits for the slot's event.
    char* dev_meta = nullptr;
    size_t dev_meta_slot = 0;  // bytes per slot
    hipStream_t copy_stream = nullptr;
    hipEvent_t meta_ready[8] = {};
    // Ring of 8 pinned buffers in two halves.  One event per half, recorded after the half's last
    // copy has been enqueued, tells when all four buffers of that half may be overwritten: one
    // event record per four steps instead of one per step.
    Staging staging[8];
    hipEvent_t half_done[2] = {nullptr, nullptr};
    bool half_pending[2] = {false, false};
    int staging_next = 0;

    // options / debug
    int opt_attn_workers = 0;
    int opt_attn_teams = 0;
    int opt_attn_prefill_weight = 22;
    int worker_slots = 2048;
    int opt_gemm_split_k = 0;
    int opt_gemm_tile = 0;
    int opt_gemm_whole_tiles = 0;
    bool opt_poison = false;
    int opt_only_layer = -1;
    bool opt_out_f32 = false;
    int tap_layer = -1;
    ps_taps taps{};

    // optional event pairs around every attention launch (see ps_attention_times)
    int opt_time_attention = 0;   // 0 = off, N = bracket the attention launch of every Nth step
    int64_t step_counter = 0;
    std::vector<hipEvent_t> attn_ev;  // ring of 2 * ATTN_EV_PAIRS events
    int attn_ev_count = 0;            // pairs recorded since the last ps_attention_times

    // ps_step_static: this device's copy of the scratch array, a pinned ring for the metadata (allocated by ps_create)
    unsigned char* static_scratch = nullptr;
    char* static_host = nullptr;
    hipEvent_t static_ev[4] = {nullptr, nullptr, nullptr, nullptr};
    bool static_pending[4] = {false, false, false, false};
    int static_next = 0;

    // optional event pairs around the four projection launches of a layer (see ps_gemm_times)
    int opt_time_gemm = 0;            // 0 = off, N = bracket them in every Nth step
    std::vector<hipEvent_t> gemm_ev;  // ring of 8 * GEMM_EV_RECS events: record r holds pairs (qkv, o, gate/up, down)
    int gemm_ev_count = 0;            // records (one per layer of a timed step) since the last ps_gemm_times

    hipEvent_t ev[PS_N_STAGES * 2 + 2] = {};
    bool have_events = false;
    StepPlan plan;
};

static constexpr int ATTN_EV_PAIRS = 2048;
static constexpr int GEMM_EV_RECS = 1024;

// Scratch of ps_step_static: workspaces, GEMM and attention partials and the step's metadata, carved out of one
// file-scope device array instead of hipMalloc'ed buffers.  Every device the library runs on holds its own copy of
// the array at its own address; `scratch` itself is only a host-side handle, so the address is asked for once per
// device (ps_create, with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[PS_STATIC_SCRATCH_BYTES];
static constexpr int MAX_DEVICES = 64;
static void* g_scratch_addr[MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;
static constexpr size_t STATIC_META_SLOT = 512u << 10;  // bytes of step metadata one static step may carry
static constexpr int STATIC_META_SLOTS = 4;             // pinned host ring
static thread_local std::string g_create_err;

static ps_status fail(ps_ctx* c, ps_status s, const std::string& msg) {
    if (c) c->err = msg; else g_create_err = msg;
    return s;
}
static ps_status hip_fail(ps_ctx* c, hipError_t e, const char* what) {
    return fail(c, e == hipErrorOutOfMemory ? PS_ENOMEM : PS_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(c, call)                                   \
    do {                                                   \
        hipError_t e__ = (call);                           \
        if (e__ != hipSuccess) return hip_fail(c, e__, #call); \
    } while (0)

template <typename T>
static ps_status dev_alloc(ps_ctx* c, T** p, size_t bytes, const char* what) {
    *p = nullptr;
    if (bytes == 0) return PS_OK;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(p), bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *p = nullptr;
        return fail(c, PS_ENOMEM, std::string("device allocation failed for ") + what + " (" + std::to_string(bytes) + " bytes): " + hipGetErrorString(e));
    }
    return PS_OK;
}
template <typename T>
static void dev_free(T*& p) {
    if (p) (void)hipFree(p);
    p = nullptr;
}

static int qkv_cols(const ps_model_desc& d) { return (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim; }

static PlanConfig plan_config(const ps_ctx* c) {
    PlanConfig pc;
    pc.n_kv_heads = c->desc.n_kv_heads;
    pc.group = c->desc.n_q_heads / c->desc.n_kv_heads;
    pc.max_position = c->desc.max_position;
    pc.n_pool_pages = c->n_pool_pages;
    pc.n_workers = c->opt_attn_workers;
    pc.n_teams = c->opt_attn_teams;
    pc.team_pair_ns = 100.0 * c->opt_attn_prefill_weight;
    pc.block_slots = c->worker_slots / 4;
    pc.prefill_tokens = attn_prefill_tokens_per_item(pc.group);
    return pc;
}

// ------------------------------------------------------------------------------ lifetime
extern "C" ps_status ps_create(const ps_model_desc* desc, void* hip_stream, ps_ctx** out) {
    if (!desc || !out) return fail(nullptr, PS_EINVAL, "ps_create: null argument");
    *out = nullptr;
    const ps_model_desc& d = *desc;
    if (d.hidden <= 0 || d.n_q_heads <= 0 || d.n_kv_heads <= 0 || d.head_dim <= 0 || d.ffn <= 0 || d.n_layers <= 0 || d.max_position <= 0)
        return fail(nullptr, PS_EINVAL, "ps_create: every dimension must be positive");
    if (d.page_size != PS_PAGE_SIZE) return fail(nullptr, PS_EINVAL, "ps_create: page_size must be 16");
    if (d.head_dim != 64 && d.head_dim != 128) return fail(nullptr, PS_EINVAL, "ps_create: head_dim must be 64 or 128");
    if (d.n_q_heads % d.n_kv_heads) return fail(nullptr, PS_EINVAL, "ps_create: n_q_heads must be a multiple of n_kv_heads");
    const int G = d.n_q_heads / d.n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16) return fail(nullptr, PS_EINVAL, "ps_create: n_q_heads / n_kv_heads must be 1, 2, 4, 8 or 16");
    if (d.hidden % 64 || d.ffn % 64 || (d.n_q_heads * d.head_dim) % 64)
        return fail(nullptr, PS_EINVAL, "ps_create: hidden, ffn and n_q_heads*head_dim must be multiples of 64");
    if (!(d.rope_base > 1.0f)) return fail(nullptr, PS_EINVAL, "ps_create: rope_base must be > 1");
    if (d.max_position > (1 << 22)) return fail(nullptr, PS_ERANGE, "ps_create: max_position above 2^22");
    if (d.hidden > 8192) return fail(nullptr, PS_ERANGE, "ps_create: hidden above 8192");

    ps_ctx* c = new (std::nothrow) ps_ctx();
    if (!c) return fail(nullptr, PS_ENOMEM, "ps_create: out of host memory");
    c->desc = d;
    if (!(c->desc.rms_eps > 0.f)) c->desc.rms_eps = 1e-5f;
    c->host_only = (d.flags & PS_FLAG_HOST_ONLY) != 0;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->layers.resize(d.n_layers);
    if (c->host_only) {
        *out = c;
        return PS_OK;
    }
    // rotary table, angles in fp64: theta_j = base^(-2j/d), entry = (cos, sin)(pos * theta_j)
    const int half = d.head_dim / 2;
    std::vector<float> cs((size_t)d.max_position * half * 2);
    std::vector<double> theta(half);
    for (int j = 0; j < half; j++) theta[j] = std::pow((double)d.rope_base, -2.0 * j / d.head_dim);
    for (int p = 0; p < d.max_position; p++)
        for (int j = 0; j < half; j++) {
            const double phi = (double)p * theta[j];
            cs[((size_t)p * half + j) * 2] = (float)std::cos(phi);
            cs[((size_t)p * half + j) * 2 + 1] = (float)std::sin(phi);
        }
    ps_status st = dev_alloc(nullptr, &c->rope_cs, cs.size() * sizeof(float), "rotary table");
    if (st != PS_OK) { delete c; return st; }
    hipError_t e = hipMemcpy(c->rope_cs, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) { ps_destroy(c); return hip_fail(nullptr, e, "hipMemcpy(rotary table)"); }
    c->worker_slots = attention_worker_slots();
    {   // set-up for ps_step_static, so that the entry point itself never allocates
        int dev = 0;
        e = hipGetDevice(&dev);
        if (e != hipSuccess) { ps_destroy(c); return hip_fail(nullptr, e, "hipGetDevice"); }
        if (dev < 0 || dev >= MAX_DEVICES) { ps_destroy(c); return fail(nullptr, PS_ERANGE, "ps_create: device index above 63"); }
        {
            std::lock_guard<std::mutex> lock(g_scratch_mutex);
            if (!g_scratch_addr[dev]) {
                void* addr = nullptr;
                e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
                if (e != hipSuccess || !addr) { ps_destroy(c); return hip_fail(nullptr, e, "hipGetSymbolAddress(scratch)"); }
                g_scratch_addr[dev] = addr;
            }
            c->static_scratch = static_cast<unsigned char*>(g_scratch_addr[dev]);
        }
        e = hipHostMalloc(reinterpret_cast<void**>(&c->static_host), STATIC_META_SLOT * STATIC_META_SLOTS, hipHostMallocDefault);
        if (e != hipSuccess) { (void)hipGetLastError(); c->static_host = nullptr; ps_destroy(c); return fail(nullptr, PS_ENOMEM, "ps_create: pinned metadata ring"); }
        for (auto& ev : c->static_ev) {
            e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
            if (e != hipSuccess) { ps_destroy(c); return hip_fail(nullptr, e, "hipEventCreate"); }
        }
    }
    *out = c;
    return PS_OK;
}

extern "C" ps_status ps_sync(ps_ctx* c) {
    if (!c) return PS_EINVAL;
    if (c->host_only) return PS_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->half_pending[0] = c->half_pending[1] = false;
    for (bool& b : c->static_pending) b = false;
    return PS_OK;
}

static void free_workspaces(ps_ctx* c) {
    dev_free(c->ws_xn); dev_free(c->ws_q); dev_free(c->ws_attn); dev_free(c->ws_act);
    dev_free(c->ws_xmid); dev_free(c->ws_x1); dev_free(c->ws_part);
    dev_free(c->ws_embed); dev_free(c->ws_final);
    c->cap_tokens = 0;
    c->part_bytes = 0;
}

extern "C" void ps_destroy(ps_ctx* c) {
    if (!c) return;
    if (!c->host_only) {
        (void)hipStreamSynchronize(c->stream);
        for (auto& l : c->layers) {
            dev_free(l.wqkv_t); dev_free(l.wo_t); dev_free(l.wgu_t); dev_free(l.wd_t); dev_free(l.g_attn); dev_free(l.g_ffn);
        }
        dev_free(c->rope_cs);
        dev_free(c->pool);
        free_workspaces(c);
        dev_free(c->embedding); dev_free(c->g_final); dev_free(c->wout_t); dev_free(c->ws_logits); dev_free(c->ws_next);
        for (auto& e : c->ev_head) if (e) (void)hipEventDestroy(e);
        dev_free(c->part_o); dev_free(c->part_ml);
        dev_free(c->ws_skfrag); dev_free(c->ws_skcnt);
        if (c->dev_meta) (void)hipFree(c->dev_meta);
        for (auto& e : c->meta_ready)
            if (e) (void)hipEventDestroy(e);
        if (c->copy_stream) { (void)hipStreamSynchronize(c->copy_stream); (void)hipStreamDestroy(c->copy_stream); }
        for (auto& s : c->staging)
            if (s.host) (void)hipHostFree(s.host);
        for (auto& e : c->half_done)
            if (e) (void)hipEventDestroy(e);
        if (c->static_host) (void)hipHostFree(c->static_host);
        for (auto& e : c->static_ev) if (e) (void)hipEventDestroy(e);
        if (c->have_events) for (auto& e : c->ev) if (e) (void)hipEventDestroy(e);
        for (auto& e : c->attn_ev) if (e) (void)hipEventDestroy(e);
        for (auto& e : c->gemm_ev) if (e) (void)hipEventDestroy(e);
    }
    delete c;
}

extern "C" const char* ps_last_error(const ps_ctx* c) { return c ? c->err.c_str() : g_create_err.c_str(); }

extern "C" ps_status ps_set_option(ps_ctx* c, const char* name, int64_t value) {
    if (!c || !name) return fail(c, PS_EINVAL, "ps_set_option: null argument");
    if (!strcmp(name, "attn_prefill_weight")) {
        if (value < 1 || value > 64) return fail(c, PS_EINVAL, "attn_prefill_weight must be in [1, 64]");
        c->opt_attn_prefill_weight = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "attn_teams")) {
        if (value < 0 || value > (1 << 20)) return fail(c, PS_EINVAL, "attn_teams must be in [0, 2^20]");
        c->opt_attn_teams = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "attn_workers")) {
        if (value < 0 || value > (1 << 20)) return fail(c, PS_EINVAL, "attn_workers must be in [0, 2^20]");
        c->opt_attn_workers = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "only_layer")) {
        if (value < -1 || value >= c->desc.n_layers) return fail(c, PS_ERANGE, "only_layer must be -1 or a layer index");
        c->opt_only_layer = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "gemm_tile")) {
        if (value != 0 && value != 128 && value != 256) return fail(c, PS_EINVAL, "gemm_tile must be 0, 128 or 256");
        c->opt_gemm_tile = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "poison_workspaces")) {
        if (value != 0 && value != 1) return fail(c, PS_EINVAL, "poison_workspaces must be 0 or 1");
        c->opt_poison = value != 0;
        return PS_OK;
    }
    if (!strcmp(name, "gemm_whole_tiles")) {
        if (value < 0 || value > 2) return fail(c, PS_EINVAL, "gemm_whole_tiles must be 0, 1 or 2");
        c->opt_gemm_whole_tiles = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "gemm_split_k")) {
        if (value < 0 || value > 64) return fail(c, PS_EINVAL, "gemm_split_k must be in [0, 64]");
        c->opt_gemm_split_k = (int)value;
        return PS_OK;
    }
    if (!strcmp(name, "time_attention")) {
        if (value < 0 || value > 1024) return fail(c, PS_EINVAL, "time_attention must be in [0, 1024]");
        if (c->host_only) return fail(c, PS_ESTATE, "time_attention: host-only context");
        if (value && c->attn_ev.empty()) {
            c->attn_ev.assign(2 * ATTN_EV_PAIRS, nullptr);
            for (auto& e : c->attn_ev) HIP_TRY(c, hipEventCreate(&e));
        }
        c->opt_time_attention = (int)value;
        c->attn_ev_count = 0;
        return PS_OK;
    }
    if (!strcmp(name, "time_gemm")) {
        if (value < 0 || value > 1024) return fail(c, PS_EINVAL, "time_gemm must be in [0, 1024]");
        if (c->host_only) return fail(c, PS_ESTATE, "time_gemm: host-only context");
        if (value && c->gemm_ev.empty()) {
            c->gemm_ev.assign(8 * GEMM_EV_RECS, nullptr);
            for (auto& e : c->gemm_ev) HIP_TRY(c, hipEventCreate(&e));
        }
        c->opt_time_gemm = (int)value;
        c->gemm_ev_count = 0;
        return PS_OK;
    }
    if (!strcmp(name, "out_f32")) {
        if (value != 0 && value != 1) return fail(c, PS_EINVAL, "out_f32 must be 0 or 1");
        c->opt_out_f32 = value != 0;
        return PS_OK;
    }
    return fail(c, PS_EINVAL, std::string("unknown option ") + name);
}

// ------------------------------------------------------------------------------ weights
extern "C" ps_status ps_init_layer(ps_ctx* c, int32_t layer, const ps_layer_weights* w) {
    if (!c || !w) return fail(c, PS_EINVAL, "ps_init_layer: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_init_layer: host-only context");
    if (layer < 0 || layer >= c->desc.n_layers) return fail(c, PS_ERANGE, "ps_init_layer: layer index out of range");
    if (!w->w_qkv || !w->w_o || !w->w_gate || !w->w_up || !w->w_down || !w->g_attn || !w->g_ffn)
        return fail(c, PS_EINVAL, "ps_init_layer: null weight pointer");
    const ps_model_desc& d = c->desc;
    const int H = d.hidden, F = d.ffn, NQ = d.n_q_heads * d.head_dim, NQKV = qkv_cols(d);
    LayerWeights& L = c->layers[layer];
    ps_status st;
    if (!L.wqkv_t) {
        if ((st = dev_alloc(c, &L.wqkv_t, (size_t)NQKV * H * 2, "w_qkv")) != PS_OK) return st;
        if ((st = dev_alloc(c, &L.wo_t, (size_t)H * NQ * 2, "w_o")) != PS_OK) return st;
        if ((st = dev_alloc(c, &L.wgu_t, (size_t)2 * F * H * 2, "w_gate/up")) != PS_OK) return st;
        if ((st = dev_alloc(c, &L.wd_t, (size_t)H * F * 2, "w_down")) != PS_OK) return st;
        if ((st = dev_alloc(c, &L.g_attn, (size_t)H * 2, "g_attn")) != PS_OK) return st;
        if ((st = dev_alloc(c, &L.g_ffn, (size_t)H * 2, "g_ffn")) != PS_OK) return st;
    }
    L.ready = false;
    HIP_TRY(c, launch_repack_weight(static_cast<const bf16_t*>(w->w_qkv), L.wqkv_t, H, NQKV, 0, c->stream));
    HIP_TRY(c, launch_repack_weight(static_cast<const bf16_t*>(w->w_o), L.wo_t, NQ, H, 0, c->stream));
    HIP_TRY(c, launch_repack_weight(static_cast<const bf16_t*>(w->w_gate), L.wgu_t, H, F, 1, c->stream));
    HIP_TRY(c, launch_repack_weight(static_cast<const bf16_t*>(w->w_up), L.wgu_t, H, F, 2, c->stream));
    HIP_TRY(c, launch_repack_weight(static_cast<const bf16_t*>(w->w_down), L.wd_t, F, H, 0, c->stream));
    HIP_TRY(c, launch_copy_bytes(w->g_attn, L.g_attn, (size_t)H * 2, c->stream));
    HIP_TRY(c, launch_copy_bytes(w->g_ffn, L.g_ffn, (size_t)H * 2, c->stream));
    L.ready = true;
    return PS_OK;
}

extern "C" ps_status ps_init_head(ps_ctx* c, const ps_head_weights* w) {
    if (!c || !w) return fail(c, PS_EINVAL, "ps_init_head: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_init_head: host-only context");
    if (!w->embedding || !w->g_final || !w->w_out) return fail(c, PS_EINVAL, "ps_init_head: null weight pointer");
    if (w->vocab <= 0 || w->vocab % 64 || w->vocab > (1 << 20)) return fail(c, PS_EINVAL, "ps_init_head: vocab must be a positive multiple of 64, at most 2^20");
    const int H = c->desc.hidden, V = w->vocab;
    if ((size_t)V * H * 2 >= (1ull << 32)) return fail(c, PS_ERANGE, "ps_init_head: output matrix of 4 GiB or more");
    ps_status st;
    if (c->vocab != V) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        dev_free(c->embedding); dev_free(c->wout_t); dev_free(c->g_final);
        c->vocab = 0;
        if ((st = dev_alloc(c, &c->embedding, (size_t)V * H * 2, "embedding")) != PS_OK) return st;
        if ((st = dev_alloc(c, &c->wout_t, (size_t)V * H * 2, "w_out")) != PS_OK) return st;
        if ((st = dev_alloc(c, &c->g_final, (size_t)H * 2, "g_final")) != PS_OK) return st;
        c->vocab = V;
    }
    c->head_ready = false;
    HIP_TRY(c, launch_copy_bytes(w->embedding, c->embedding, (size_t)V * H * 2, c->stream));
    HIP_TRY(c, launch_repack_weight(static_cast<const bf16_t*>(w->w_out), c->wout_t, H, V, 0, c->stream));
    HIP_TRY(c, launch_copy_bytes(w->g_final, c->g_final, (size_t)H * 2, c->stream));
    c->head_ready = true;
    return PS_OK;
}

// ------------------------------------------------------------------------------ KV pool
static inline uint64_t splitmix64_next(uint64_t& s) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

extern "C" ps_status ps_kv_alloc(ps_ctx* c, int32_t n_pages, int32_t n_kv_layers, uint64_t perm_seed) {
    if (!c) return PS_EINVAL;
    if (n_pages <= 0 || n_kv_layers <= 0) return fail(c, PS_EINVAL, "ps_kv_alloc: n_pages and n_kv_layers must be positive");
    if (n_pages > (1 << 26)) return fail(c, PS_ERANGE, "ps_kv_alloc: more than 2^26 pages");
    const ps_model_desc& d = c->desc;
    const size_t slot_elems = (size_t)n_pages * d.n_kv_heads * 2 * PS_PAGE_SIZE * d.head_dim;
    if (!c->host_only) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        dev_free(c->pool);
        c->n_pool_pages = -1;
        ps_status st = dev_alloc(c, &c->pool, slot_elems * n_kv_layers * 2, "KV pool");
        if (st != PS_OK) return st;
        HIP_TRY(c, hipMemsetAsync(c->pool, 0, slot_elems * n_kv_layers * 2, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
    }
    c->n_pool_pages = n_pages;
    c->n_kv_slots = n_kv_layers;
    c->slot_elems = slot_elems;
    c->page_seen.assign(n_pages, 0);
    c->owned.clear();
    std::vector<int32_t> order(n_pages);
    for (int i = 0; i < n_pages; i++) order[i] = i;
    uint64_t s = perm_seed;
    for (int i = n_pages - 1; i >= 1; i--) {
        const uint64_t j = splitmix64_next(s) % (uint64_t)(i + 1);
        std::swap(order[i], order[(size_t)j]);
    }
    c->free_list.assign(order.begin(), order.end());
    return PS_OK;
}

extern "C" ps_status ps_kv_reserve(ps_ctx* c, int64_t req_id, int32_t kv_len, int32_t* pages_out, int32_t cap, int32_t* n_out) {
    if (!c || !n_out || (!pages_out && cap > 0)) return fail(c, PS_EINVAL, "ps_kv_reserve: null argument");
    if (c->n_pool_pages < 0) return fail(c, PS_ESTATE, "ps_kv_reserve: no KV pool (call ps_kv_alloc)");
    if (kv_len < 0 || kv_len > c->desc.max_position) return fail(c, PS_ERANGE, "ps_kv_reserve: kv_len outside [0, max_position]");
    const int want = (kv_len + PS_PAGE_SIZE - 1) / PS_PAGE_SIZE;
    auto it = c->owned.find(req_id);
    const int have = it == c->owned.end() ? 0 : (int)it->second.size();
    const int need = want - have;
    const int total = std::max(have, want);
    if (cap < total) return fail(c, PS_ERANGE, "ps_kv_reserve: pages_out too small");
    if (need > (int)c->free_list.size()) return fail(c, PS_ENOMEM, "ps_kv_reserve: KV pool exhausted");
    std::vector<int32_t>& v = c->owned[req_id];
    for (int i = 0; i < need; i++) {
        v.push_back(c->free_list.front());
        c->free_list.pop_front();
    }
    for (int i = 0; i < total; i++) pages_out[i] = v[i];
    *n_out = total;
    return PS_OK;
}

extern "C" ps_status ps_kv_release(ps_ctx* c, int64_t req_id) {
    if (!c) return PS_EINVAL;
    auto it = c->owned.find(req_id);
    if (it == c->owned.end()) return fail(c, PS_EINVAL, "ps_kv_release: unknown req_id");
    for (int32_t p : it->second) c->free_list.push_back(p);
    c->owned.erase(it);
    return PS_OK;
}

extern "C" int32_t ps_kv_free_pages(const ps_ctx* c) {
    if (!c || c->n_pool_pages < 0) return -1;
    return (int32_t)c->free_list.size();
}

// pinned staging: returns a host buffer of at least `bytes`, safe to overwrite
static ps_status staging_acquire(ps_ctx* c, size_t bytes, Staging** out, int* index) {
    const int idx = c->staging_next, half = idx / 4;
    c->staging_next = (idx + 1) % 8;
    *index = idx;
    Staging& s = c->staging[idx];
    if (idx % 4 == 0 && c->half_pending[half]) {  // entering a half: its previous copies must be done
        HIP_TRY(c, hipEventSynchronize(c->half_done[half]));
        c->half_pending[half] = false;
    }
    if (s.bytes < bytes) {
        if (s.host) (void)hipHostFree(s.host);
        s.host = nullptr;
        s.bytes = 0;
        const size_t want = std::max(bytes + bytes / 2, (size_t)1 << 16);
        hipError_t e = hipHostMalloc(&s.host, want, hipHostMallocDefault);
        if (e != hipSuccess) { (void)hipGetLastError(); s.host = nullptr; return fail(c, PS_ENOMEM, "pinned staging allocation failed"); }
        s.bytes = want;
    }
    *out = &s;
    return PS_OK;
}

// call after the last kernel that reads slot `index`'s device copy has been enqueued
static ps_status staging_commit(ps_ctx* c, int index) {
    if (index % 4 != 3) return PS_OK;
    const int half = index / 4;
    if (!c->half_done[half]) HIP_TRY(c, hipEventCreateWithFlags(&c->half_done[half], hipEventDisableTiming));
    HIP_TRY(c, hipEventRecord(c->half_done[half], c->stream));
    c->half_pending[half] = true;
    return PS_OK;
}

// Between staging_acquire and staging_commit a call may fail (a HIP error, an allocation) after copies and kernels
// that read the slot have been enqueued.  The guard then waits for both streams and forgets the pending halves, so
// that the next pass through the ring cannot overwrite buffers that are still being read.
struct StagingGuard {
    ps_ctx* c;
    bool committed = false;
    explicit StagingGuard(ps_ctx* ctx) : c(ctx) {}
    ~StagingGuard() {
        if (committed) return;
        (void)hipStreamSynchronize(c->stream);
        if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
        c->half_pending[0] = c->half_pending[1] = false;
        for (bool& b : c->static_pending) b = false;
    }
};

// Copy `bytes` of staging slot `index` to its device slot on the copy stream and make the main
// stream wait for it.  *dev receives the device address.
// Device slot `index` of the metadata ring, grown to hold `bytes`.
static ps_status dev_meta_slot(ps_ctx* c, int index, size_t bytes, char** dev) {
    if (c->dev_meta_slot < bytes) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        if (c->copy_stream) HIP_TRY(c, hipStreamSynchronize(c->copy_stream));
        if (c->dev_meta) (void)hipFree(c->dev_meta);
        c->dev_meta = nullptr;
        c->dev_meta_slot = 0;
        const size_t want = (std::max(bytes + bytes / 2, (size_t)1 << 16) + 255) & ~(size_t)255;
        ps_status st = dev_alloc(c, &c->dev_meta, want * 8, "step metadata");
        if (st != PS_OK) return st;
        c->dev_meta_slot = want;
    }
    *dev = c->dev_meta + (size_t)index * c->dev_meta_slot;
    return PS_OK;
}

static ps_status upload_meta(ps_ctx* c, const Staging* sg, int index, size_t bytes, const char** dev) {
    if (!c->copy_stream) {
        HIP_TRY(c, hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
        for (auto& e : c->meta_ready) HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }
    char* d = nullptr;
    ps_status st0 = dev_meta_slot(c, index, bytes, &d);
    if (st0 != PS_OK) return st0;
    HIP_TRY(c, hipMemcpyAsync(d, sg->host, bytes, hipMemcpyHostToDevice, c->copy_stream));
    HIP_TRY(c, hipEventRecord(c->meta_ready[index], c->copy_stream));
    HIP_TRY(c, hipStreamWaitEvent(c->stream, c->meta_ready[index], 0));
    *dev = d;
    return PS_OK;
}

static ps_status kv_copy(ps_ctx* c, bool to_pool, int32_t layer, const ps_seq* seq, int32_t pos0, int32_t n, void* k, void* v) {
    const char* name = to_pool ? "ps_kv_write" : "ps_kv_read";
    if (!c || !seq || !seq->page_table) return fail(c, PS_EINVAL, std::string(name) + ": null argument");
    if (c->host_only) return fail(c, PS_ESTATE, std::string(name) + ": host-only context");
    if (!c->pool) return fail(c, PS_ESTATE, std::string(name) + ": no KV pool (call ps_kv_alloc)");
    if (layer < 0 || layer >= c->desc.n_layers) return fail(c, PS_ERANGE, std::string(name) + ": layer index out of range");
    if (n == 0) return PS_OK;
    if (!k || !v) return fail(c, PS_EINVAL, std::string(name) + ": null k or v");
    if ((reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v)) & 15) return fail(c, PS_EINVAL, std::string(name) + ": k and v must be 16-byte aligned");
    if (n < 0 || pos0 < 0 || (int64_t)pos0 + n > (int64_t)seq->n_pages * PS_PAGE_SIZE)
        return fail(c, PS_ERANGE, std::string(name) + ": positions outside the sequence's pages");
    for (int p = pos0 / PS_PAGE_SIZE; p <= (pos0 + n - 1) / PS_PAGE_SIZE; p++)
        if (seq->page_table[p] < 0 || seq->page_table[p] >= c->n_pool_pages)
            return fail(c, PS_ERANGE, std::string(name) + ": page id outside the pool");
    Staging* s;
    int s_idx = 0;
    ps_status st = staging_acquire(c, (size_t)n * 4, &s, &s_idx);
    if (st != PS_OK) return st;
    StagingGuard guard(c);
    int32_t* slots = static_cast<int32_t*>(s->host);
    for (int i = 0; i < n; i++) {
        const int p = pos0 + i;
        slots[i] = seq->page_table[p / PS_PAGE_SIZE] * PS_PAGE_SIZE + p % PS_PAGE_SIZE;
    }
    const char* dslots = nullptr;
    if ((st = upload_meta(c, s, s_idx, (size_t)n * 4, &dslots)) != PS_OK) return st;
    bf16_t* slot_base = c->pool + (size_t)(layer % c->n_kv_slots) * c->slot_elems;
    HIP_TRY(c, launch_kv_copy(to_pool, slot_base, reinterpret_cast<const int32_t*>(dslots), n, pos0 & 3, c->desc.n_kv_heads,
                              c->desc.head_dim, static_cast<bf16_t*>(k), static_cast<bf16_t*>(v), c->stream));
    if ((st = staging_commit(c, s_idx)) == PS_OK) guard.committed = true;
    return st;
}

extern "C" ps_status ps_kv_write(ps_ctx* c, int32_t layer, const ps_seq* seq, int32_t pos0, int32_t n, const void* k, const void* v) {
    return kv_copy(c, true, layer, seq, pos0, n, const_cast<void*>(k), const_cast<void*>(v));
}
extern "C" ps_status ps_kv_read(ps_ctx* c, int32_t layer, const ps_seq* seq, int32_t pos0, int32_t n, void* k, void* v) {
    return kv_copy(c, false, layer, seq, pos0, n, k, v);
}

// ------------------------------------------------------------------------------ planning
static ps_status make_plan(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, bool with_attention) {
    const PlanConfig pc = plan_config(c);
    std::string err;
    ps_status st = validate_batch(seqs, n_seqs, pc, c->page_seen, err);
    if (st != PS_OK) return fail(c, st, err);
    build_indices(seqs, n_seqs, c->plan);
    if (with_attention) build_attention_plan(pc, c->plan);
    return PS_OK;
}

extern "C" ps_status ps_step_indices(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, int32_t* cu_seqlens, int32_t* positions, int32_t* slot_mapping) {
    if (!c) return PS_EINVAL;
    ps_status st = make_plan(c, seqs, n_seqs, false);
    if (st != PS_OK) return st;
    const StepPlan& p = c->plan;
    if (cu_seqlens) std::copy(p.cu_seqlens.begin(), p.cu_seqlens.end(), cu_seqlens);
    if (positions) std::copy(p.positions.begin(), p.positions.end(), positions);
    if (slot_mapping) std::copy(p.slots.begin(), p.slots.end(), slot_mapping);
    return PS_OK;
}

extern "C" ps_status ps_plan_attention(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, int32_t* items, int32_t cap, int32_t* n_items) {
    if (!c || !n_items || (!items && cap > 0)) return fail(c, PS_EINVAL, "ps_plan_attention: null argument");
    ps_status st = make_plan(c, seqs, n_seqs, true);
    if (st != PS_OK) return st;
    const StepPlan& p = c->plan;
    *n_items = (int32_t)p.items.size();
    const int n = std::min<int>(cap, (int)p.items.size());
    static_assert(sizeof(AttnItem) == 16 * sizeof(int32_t), "item is 16 int32, the first 8 are reported");
    for (int i = 0; i < n; i++) memcpy(items + (size_t)i * 8, &p.items[i], 8 * sizeof(int32_t));
    return PS_OK;
}

extern "C" ps_status ps_set_taps(ps_ctx* c, int32_t layer, const ps_taps* taps) {
    if (!c) return PS_EINVAL;
    if (!taps) { c->tap_layer = -1; return PS_OK; }
    if (layer < 0 || layer >= c->desc.n_layers) return fail(c, PS_ERANGE, "ps_set_taps: layer index out of range");
    c->tap_layer = layer;
    c->taps = *taps;
    return PS_OK;
}

// ------------------------------------------------------------------------------ the step
static size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

// What the tiled GEMM needs beside its output for a step of T tokens: the largest over the layer's four projections.
static void sk_need(const ps_ctx* c, int T, int head_rows, size_t* frag_bytes, int* n_counters) {
    const ps_model_desc& d = c->desc;
    const int H = d.hidden, F = d.ffn, NQ = d.n_q_heads * d.head_dim, NQKV = qkv_cols(d);
    const int shapes[4][3] = {{NQKV, H, GemmOut::PARTIAL_F32}, {H, NQ, GemmOut::PARTIAL_F32}, {2 * F, H, GemmOut::SWIGLU_BF16}, {H, F, GemmOut::PARTIAL_F32}};
    *frag_bytes = 0;
    *n_counters = 0;
    for (const auto& sh : shapes) {
        size_t fb = 0;
        int nc = 0;
        gemm_workspace(T, sh[0], sh[1], sh[2], c->opt_gemm_split_k, c->opt_gemm_tile, c->opt_gemm_whole_tiles, &fb, &nc);
        *frag_bytes = std::max(*frag_bytes, fb);
        *n_counters = std::max(*n_counters, nc);
    }
    if (head_rows > 0) {   // the output projection: one row per sequence
        size_t fb = 0;
        int nc = 0;
        gemm_workspace(head_rows, c->vocab, H, GemmOut::PARTIAL_F32, 1, c->opt_gemm_tile, c->opt_gemm_whole_tiles, &fb, &nc);
        *frag_bytes = std::max(*frag_bytes, fb);
        *n_counters = std::max(*n_counters, nc);
    }
}

static ps_status ensure_workspaces(ps_ctx* c, int T, int n_part_slots, int head_rows) {
    const ps_model_desc& d = c->desc;
    if (T > c->cap_tokens) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        free_workspaces(c);
        const int cap = std::max(T + T / 4, 64);
        const int cap16 = (cap + 15) & ~15;  // operand-order buffers hold whole 16-row tiles
        const int H = d.hidden, F = d.ffn, NQ = d.n_q_heads * d.head_dim, NQKV = qkv_cols(d);
        (void)NQKV;
        ps_status st;
        if ((st = dev_alloc(c, &c->ws_xn, (size_t)cap16 * H * 2, "xn")) != PS_OK) return st;
        if ((st = dev_alloc(c, &c->ws_q, (size_t)cap * NQ * 2, "q")) != PS_OK) return st;
        if ((st = dev_alloc(c, &c->ws_attn, (size_t)cap16 * NQ * 2, "attn")) != PS_OK) return st;
        c->act_bytes = gemm_out_bytes(cap, 2 * F, H, GemmOut::SWIGLU_BF16, 0, 0);  // whole row tiles of the GEMM
        if ((st = dev_alloc(c, &c->ws_act, c->act_bytes, "act")) != PS_OK) return st;
        if ((st = dev_alloc(c, &c->ws_x1, (size_t)cap * H * 4, "x1")) != PS_OK) return st;
        if (d.n_layers > 1 && (st = dev_alloc(c, &c->ws_xmid, (size_t)cap * H * 4, "inter-layer x")) != PS_OK) return st;
        if (c->head_ready) {
            if ((st = dev_alloc(c, &c->ws_embed, (size_t)cap * H * 2, "embedding rows")) != PS_OK) return st;
            if ((st = dev_alloc(c, &c->ws_final, (size_t)cap * H * 4, "final hidden states")) != PS_OK) return st;
        }
        c->cap_tokens = cap;
    }
    {   // GEMM partial buffer: sized for this step's T (the split count depends on T)
        const int H = d.hidden, F = d.ffn, NQ = d.n_q_heads * d.head_dim, NQKV = qkv_cols(d);
        size_t need = gemm_out_bytes(T, NQKV, H, GemmOut::PARTIAL_F32, c->opt_gemm_split_k, c->opt_gemm_tile);
        need = std::max(need, gemm_out_bytes(T, H, NQ, GemmOut::PARTIAL_F32, c->opt_gemm_split_k, c->opt_gemm_tile));
        need = std::max(need, gemm_out_bytes(T, H, F, GemmOut::PARTIAL_F32, c->opt_gemm_split_k, c->opt_gemm_tile));
        if (need > c->part_bytes) {
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            dev_free(c->ws_part);
            c->part_bytes = 0;
            const size_t want = std::max(need + need / 4, (size_t)16 << 20);
            ps_status st = dev_alloc(c, &c->ws_part, want, "GEMM partials");
            if (st != PS_OK) return st;
            c->part_bytes = want;
        }
    }
    {   // tiled GEMM workspace
        size_t fb = 0;
        int nc = 0;
        sk_need(c, T, head_rows, &fb, &nc);
        if (fb > c->skfrag_bytes) {
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            dev_free(c->ws_skfrag);
            c->skfrag_bytes = 0;
            ps_status st = dev_alloc(c, &c->ws_skfrag, fb, "GEMM parked accumulators");
            if (st != PS_OK) return st;
            c->skfrag_bytes = fb;
        }
        if (nc > c->skcnt_n) {
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            dev_free(c->ws_skcnt);
            c->skcnt_n = 0;
            const int want = (nc + nc / 2 + 255) & ~3;
            ps_status st = dev_alloc(c, &c->ws_skcnt, (size_t)want * sizeof(int), "GEMM tile counters");
            if (st != PS_OK) return st;
            HIP_TRY(c, launch_fill_zero(c->ws_skcnt, (size_t)want * sizeof(int), c->stream));   // the kernels leave them zero
            c->skcnt_n = want;
        }
    }
    if (n_part_slots > c->cap_part_slots) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        dev_free(c->part_o); dev_free(c->part_ml);
        c->cap_part_slots = 0;
        const int cap = n_part_slots + n_part_slots / 2 + 64;
        ps_status st;
        if ((st = dev_alloc(c, &c->part_o, (size_t)cap * 16 * d.head_dim * 4, "attention partials")) != PS_OK) return st;
        if ((st = dev_alloc(c, &c->part_ml, (size_t)cap * 16 * 2 * 4, "attention partial stats")) != PS_OK) return st;
        c->cap_part_slots = cap;
    }
    return PS_OK;
}

struct MetaLayout {
    size_t positions, slots, seqs, pages, items, workers, groups, tokens, last_rows, total;
};
static MetaLayout meta_layout(const StepPlan& p, bool with_tokens) {
    MetaLayout m;
    size_t at = 0;
    m.positions = at; at = align16(at + p.positions.size() * 4);
    m.slots = at;     at = align16(at + p.slots.size() * 4);
    m.seqs = at;      at = align16(at + p.seqs.size() * sizeof(SeqInfo));
    m.pages = at;     at = align16(at + p.pages.size() * 4);
    m.items = at;     at = align16(at + p.items.size() * sizeof(AttnItem));
    m.workers = at;   at = align16(at + p.worker_begin.size() * 4);
    m.groups = at;    at = align16(at + p.groups.size() * sizeof(MergeGroup));
    m.tokens = at;    if (with_tokens) at = align16(at + (size_t)p.n_tokens * 4);
    m.last_rows = at; if (with_tokens) at = align16(at + (size_t)p.n_seqs * 4);
    m.total = at;
    return m;
}

// Token side of a full-model step: host token ids in, greedy tokens (and optionally logits / final hidden
// states) out.  Null for ps_step, which takes and returns hidden states.
struct TokenIO {
    const int32_t* token_ids;  // host [T]
    int32_t* next_tokens;      // device [n_seqs] or null
    float* logits;             // device [n_seqs][vocab] or null
    float* hidden;             // device [T][hidden] fp32 or null
    float* ms;                 // host [3] or null: embedding, stack, head (needs stats-style synchronisation)
};

// Device buffers of one step besides its inputs and outputs: the library's growing workspaces (ps_step,
// ps_step_tokens) or pieces of the static scratch array (ps_step_static).
struct StepBufs {
    bf16_t *xn = nullptr, *q = nullptr, *attn = nullptr, *act = nullptr;
    float *x1 = nullptr, *xmid = nullptr, *part = nullptr, *part_o = nullptr, *part_ml = nullptr;
    size_t part_bytes = 0, act_bytes = 0;
    float* skfrag = nullptr;
    size_t skfrag_bytes = 0;
    int* skcnt = nullptr;
    int skcnt_n = 0;
    char* meta = nullptr;  // static steps only: device copy of the metadata
};

// Lay the buffers of a step of T tokens out in the static scratch array.  Nothing is allocated: a step whose buffers
// do not fit PS_STATIC_SCRATCH_BYTES is refused.
static ps_status carve_static(ps_ctx* c, int T, int n_part_slots, size_t meta_bytes, StepBufs* w) {
    const ps_model_desc& d = c->desc;
    const int H = d.hidden, F = d.ffn, NQ = d.n_q_heads * d.head_dim, NQKV = qkv_cols(d);
    const size_t T16 = (size_t)((T + 15) & ~15);
    size_t at = 0;
    auto take = [&](size_t bytes) { const size_t o = at; at = (at + bytes + 255) & ~(size_t)255; return o; };
    const size_t o_xn = take(T16 * H * 2), o_q = take((size_t)T * NQ * 2), o_attn = take(T16 * NQ * 2);
    w->act_bytes = gemm_out_bytes(T, 2 * F, H, GemmOut::SWIGLU_BF16, 0, 0);
    const size_t o_act = take(w->act_bytes), o_x1 = take((size_t)T * H * 4), o_xmid = take(d.n_layers > 1 ? (size_t)T * H * 4 : 0);
    w->part_bytes = gemm_out_bytes(T, NQKV, H, GemmOut::PARTIAL_F32, c->opt_gemm_split_k, c->opt_gemm_tile);
    w->part_bytes = std::max(w->part_bytes, gemm_out_bytes(T, H, NQ, GemmOut::PARTIAL_F32, c->opt_gemm_split_k, c->opt_gemm_tile));
    w->part_bytes = std::max(w->part_bytes, gemm_out_bytes(T, H, F, GemmOut::PARTIAL_F32, c->opt_gemm_split_k, c->opt_gemm_tile));
    const size_t o_part = take(w->part_bytes);
    const size_t o_po = take((size_t)n_part_slots * 16 * d.head_dim * 4), o_pml = take((size_t)n_part_slots * 16 * 2 * 4);
    const size_t o_meta = take(meta_bytes);
    int n_cnt = 0;
    sk_need(c, T, 0, &w->skfrag_bytes, &n_cnt);
    w->skcnt_n = (n_cnt + 3) & ~3;
    const size_t o_skfrag = take(w->skfrag_bytes), o_skcnt = take((size_t)w->skcnt_n * sizeof(int));
    if (meta_bytes > STATIC_META_SLOT)
        return fail(c, PS_ERANGE, "ps_step_static: the step's metadata (" + std::to_string(meta_bytes) + " bytes: positions, page lists, attention work list) exceeds " +
                                      std::to_string(STATIC_META_SLOT) + " bytes; use ps_step for batches of this size");
    if (at > (size_t)PS_STATIC_SCRATCH_BYTES)
        return fail(c, PS_ERANGE, "ps_step_static: the step needs " + std::to_string(at) + " bytes of scratch, the static array holds " +
                                      std::to_string((size_t)PS_STATIC_SCRATCH_BYTES) + "; use ps_step for batches of this size");
    unsigned char* b = c->static_scratch;
    w->xn = reinterpret_cast<bf16_t*>(b + o_xn); w->q = reinterpret_cast<bf16_t*>(b + o_q); w->attn = reinterpret_cast<bf16_t*>(b + o_attn);
    w->act = reinterpret_cast<bf16_t*>(b + o_act); w->x1 = reinterpret_cast<float*>(b + o_x1); w->xmid = reinterpret_cast<float*>(b + o_xmid);
    w->part = reinterpret_cast<float*>(b + o_part); w->part_o = reinterpret_cast<float*>(b + o_po); w->part_ml = reinterpret_cast<float*>(b + o_pml);
    w->meta = reinterpret_cast<char*>(b + o_meta);
    w->skfrag = reinterpret_cast<float*>(b + o_skfrag);
    w->skcnt = reinterpret_cast<int*>(b + o_skcnt);
    return PS_OK;
}

static ps_status step_impl(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, const void* x_in, void* x_out, ps_step_stats* stats,
                           const TokenIO* tio, bool use_static = false) {
    if (!c) return PS_EINVAL;
    if (c->host_only) return fail(c, PS_ESTATE, "ps_step: host-only context");
    if (!c->pool) return fail(c, PS_ESTATE, "ps_step: no KV pool (call ps_kv_alloc)");
    for (int l = 0; l < c->desc.n_layers; l++)
        if (!c->layers[l].ready) return fail(c, PS_ESTATE, "ps_step: layer " + std::to_string(l) + " has no weights (call ps_init_layer)");
    ps_status st = make_plan(c, seqs, n_seqs, true);
    if (st != PS_OK) return st;
    const StepPlan& p = c->plan;
    if (stats) {
        memset(stats, 0, sizeof(*stats));
        stats->n_tokens = p.n_tokens;
        stats->total_kv = p.total_kv;
        stats->n_attn_items = (int32_t)p.items.size();
        stats->n_attn_partials = p.n_partial_items;
    }
    if (n_seqs == 0) return PS_OK;
    if (!tio && (!x_in || !x_out)) return fail(c, PS_EINVAL, "ps_step: null activation pointer");
    if (tio) {
        if (!c->head_ready) return fail(c, PS_ESTATE, "ps_step_tokens: no model head (call ps_init_head)");
        if (c->opt_only_layer >= 0) return fail(c, PS_ESTATE, "ps_step_tokens: option only_layer is set");
        if (!tio->token_ids) return fail(c, PS_EINVAL, "ps_step_tokens: null token ids");
        for (int t = 0; t < p.n_tokens; t++)
            if (tio->token_ids[t] < 0 || tio->token_ids[t] >= c->vocab)
                return fail(c, PS_ERANGE, "ps_step_tokens: token " + std::to_string(t) + " has id " + std::to_string(tio->token_ids[t]) +
                                              " outside the vocabulary of " + std::to_string(c->vocab));
        if (!c->ws_embed && c->cap_tokens > 0) {  // workspaces were sized before the head existed
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            free_workspaces(c);
        }
    }

    c->step_counter++;
    const ps_model_desc& d = c->desc;
    const int T = p.n_tokens, H = d.hidden, F = d.ffn, NQ = d.n_q_heads * d.head_dim, NQKV = qkv_cols(d);
    const MetaLayout ml = meta_layout(p, tio != nullptr);
    StepBufs W;
    if (use_static) {
        if ((st = carve_static(c, T, p.n_partial_slots, ml.total, &W)) != PS_OK) return st;
    } else {
        if ((st = ensure_workspaces(c, T, p.n_partial_slots, tio ? p.n_seqs : 0)) != PS_OK) return st;
        W.xn = c->ws_xn; W.q = c->ws_q; W.attn = c->ws_attn; W.act = c->ws_act; W.x1 = c->ws_x1; W.xmid = c->ws_xmid;
        W.part = c->ws_part; W.part_o = c->part_o; W.part_ml = c->part_ml; W.part_bytes = c->part_bytes; W.act_bytes = c->act_bytes;
        W.skfrag = c->ws_skfrag; W.skfrag_bytes = c->skfrag_bytes; W.skcnt = c->ws_skcnt; W.skcnt_n = c->skcnt_n;
    }
    if (c->opt_poison) {
        // every buffer the step's kernels write before they read: bf16 NaN (0x7FC0) everywhere, which as fp32 words is a
        // NaN too.  A kernel that reads what no kernel of this step wrote carries it into the output.
        const uint32_t nan2 = 0x7FC07FC0u;
        const size_t T16 = (size_t)((T + 15) & ~15);
        HIP_TRY(c, launch_fill_words(W.xn, T16 * H * 2, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.q, (size_t)T * NQ * 2, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.attn, T16 * NQ * 2, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.act, W.act_bytes, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.x1, (size_t)T * H * 4, nan2, c->stream));
        if (W.xmid) HIP_TRY(c, launch_fill_words(W.xmid, (size_t)T * H * 4, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.part, W.part_bytes, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.part_o, (size_t)p.n_partial_slots * 16 * d.head_dim * 4, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.part_ml, (size_t)p.n_partial_slots * 16 * 2 * 4, nan2, c->stream));
        HIP_TRY(c, launch_fill_words(W.skfrag, W.skfrag_bytes, nan2, c->stream));
    }
    // the array of a static step keeps whatever the previous call left where this call's tile counters lie
    if (use_static && W.skcnt_n > 0) HIP_TRY(c, launch_fill_zero(W.skcnt, (size_t)W.skcnt_n * sizeof(int), c->stream));

    // one pinned buffer, one host-to-device copy for all of the step's integer metadata
    Staging* sg = nullptr;
    int sg_idx = 0;
    char* hb = nullptr;
    if (use_static) {
        // slot of the pinned ring made at ps_create; its previous copy (four static steps ago) must have been made
        sg_idx = c->static_next;
        c->static_next = (sg_idx + 1) % STATIC_META_SLOTS;
        if (c->static_pending[sg_idx]) {
            HIP_TRY(c, hipEventSynchronize(c->static_ev[sg_idx]));
            c->static_pending[sg_idx] = false;
        }
        hb = c->static_host + (size_t)sg_idx * STATIC_META_SLOT;
    } else {
        if ((st = staging_acquire(c, ml.total, &sg, &sg_idx)) != PS_OK) return st;
        hb = static_cast<char*>(sg->host);
    }
    StagingGuard guard(c);
    memcpy(hb + ml.positions, p.positions.data(), p.positions.size() * 4);
    memcpy(hb + ml.slots, p.slots.data(), p.slots.size() * 4);
    memcpy(hb + ml.seqs, p.seqs.data(), p.seqs.size() * sizeof(SeqInfo));
    memcpy(hb + ml.pages, p.pages.data(), p.pages.size() * 4);
    memcpy(hb + ml.items, p.items.data(), p.items.size() * sizeof(AttnItem));
    memcpy(hb + ml.workers, p.worker_begin.data(), p.worker_begin.size() * 4);
    if (!p.groups.empty()) memcpy(hb + ml.groups, p.groups.data(), p.groups.size() * sizeof(MergeGroup));
    if (tio) {
        memcpy(hb + ml.tokens, tio->token_ids, (size_t)p.n_tokens * 4);
        int32_t* lr = reinterpret_cast<int32_t*>(hb + ml.last_rows);  // last new token of every sequence
        for (int i = 0; i < p.n_seqs; i++) lr[i] = p.cu_seqlens[i + 1] - 1;
    }
    // How the metadata reaches the device.  A step on hidden states: extra blocks of its first kernel (the RMS
    // normalisation, which needs none of it) copy it out of the pinned buffer.  A step on token ids needs it in its
    // very first kernel (the embedding gather): copy engine, on the copy stream.
    const char* db = nullptr;
    const void* fetch_src = nullptr;
    void* fetch_dst = nullptr;
    if (use_static) {
        db = W.meta;
        fetch_src = hb; fetch_dst = W.meta;
    } else if (!tio) {
        char* dslot = nullptr;
        if ((st = dev_meta_slot(c, sg_idx, ml.total, &dslot)) != PS_OK) return st;
        db = dslot;
        fetch_src = hb; fetch_dst = dslot;
    } else if ((st = upload_meta(c, sg, sg_idx, ml.total, &db)) != PS_OK) return st;
    const int32_t* d_pos = reinterpret_cast<const int32_t*>(db + ml.positions);
    const int32_t* d_slots = reinterpret_cast<const int32_t*>(db + ml.slots);

    if (stats && !c->have_events) {
        for (auto& e : c->ev) HIP_TRY(c, hipEventCreate(&e));
        c->have_events = true;
    }
    // with stats, events bracket every stage of every layer; stage times are summed over layers
    std::vector<float> stage_ms(PS_N_STAGES, 0.f);
    float total_ms = 0.f;
    hipStream_t s = c->stream;

    // Full-model step: the stack's input is the embedding rows of the step's tokens, its output stays fp32
    const bool out_f32 = tio ? true : c->opt_out_f32 != 0;
    if (tio) {
        if (tio->ms && !c->ev_head[0])
            for (auto& e : c->ev_head) HIP_TRY(c, hipEventCreate(&e));
        if (tio->ms) HIP_TRY(c, hipEventRecord(c->ev_head[0], s));
        HIP_TRY(c, launch_embed_gather(c->embedding, reinterpret_cast<const int32_t*>(db + ml.tokens), c->ws_embed, T, H, s));
        if (tio->ms) HIP_TRY(c, hipEventRecord(c->ev_head[1], s));
        x_in = c->ws_embed;
        x_out = tio->hidden ? static_cast<void*>(tio->hidden) : static_cast<void*>(c->ws_final);
    }
    // The residual stream stays fp32 inside the stack: only x_in and x_out are bf16.  Every
    // projection leaves fp32 partial sums; the kernel that consumes them adds them up.
    const void* x_cur = x_in;
    bool x_cur_f32 = false;
    // only_layer: the step runs that one layer as a whole model (x_in -> x_out)
    const int l_begin = c->opt_only_layer >= 0 ? c->opt_only_layer : 0;
    const int l_end = c->opt_only_layer >= 0 ? c->opt_only_layer + 1 : d.n_layers;
    for (int l = l_begin; l < l_end; l++) {
        const LayerWeights& L = c->layers[l];
        const bool tap = (l == c->tap_layer);
        const bool last = (l == l_end - 1);
        bf16_t* pool_slot = c->pool + (size_t)(l % c->n_kv_slots) * c->slot_elems;
        int e = 0, n_splits = 1;
        // event pairs around this layer's four projection launches, when asked for and while the ring has room
        hipEvent_t* gev = nullptr;
        if (c->opt_time_gemm > 0 && c->gemm_ev_count < GEMM_EV_RECS && (c->step_counter % c->opt_time_gemm) == 0)
            gev = c->gemm_ev.data() + (size_t)8 * c->gemm_ev_count++;
        auto run_gemm = [&](const GemmArgs& ga, int* splits, int which) -> hipError_t {
            if (gev) (void)hipEventRecord(gev[2 * which], s);
            const hipError_t ge = launch_gemm(ga, splits, s);
            if (gev) (void)hipEventRecord(gev[2 * which + 1], s);
            return ge;
        };
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[e], s));
        // 0: RMSNorm of the layer input (layers after the first get it from the previous layer's last kernel)
        if (l == l_begin) HIP_TRY(c, launch_rmsnorm(x_cur, x_cur_f32, L.g_attn, W.xn, T, H, d.rms_eps, s, nullptr, fetch_src, fetch_dst, fetch_src ? ml.total : 0));
        if (tap && c->taps.xn) HIP_TRY(c, launch_untile(W.xn, static_cast<bf16_t*>(c->taps.xn), T, H, s));
        if (tap && c->taps.x_in && l > l_begin) HIP_TRY(c, launch_copy_bytes(x_cur, c->taps.x_in, (size_t)T * H * 4, s));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 1: QKV projection -> fp32 partials
        GemmArgs g{};
        g.A = W.xn; g.Wp = L.wqkv_t; g.M = T; g.N = NQKV; g.K = H; g.kind = GemmOut::PARTIAL_F32;
        g.out = W.part; g.out_bytes = W.part_bytes; g.split_k = c->opt_gemm_split_k; g.tile = c->opt_gemm_tile;
        g.sk_frag = W.skfrag; g.sk_frag_bytes = W.skfrag_bytes; g.sk_counters = W.skcnt; g.sk_n_counters = W.skcnt_n;
        g.sk_mode = c->opt_gemm_whole_tiles;
        HIP_TRY(c, run_gemm(g, &n_splits, 0));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 2: sum the partials, rotate, round once to bf16, append k/v to the pages
        HIP_TRY(c, launch_rope_append(W.part, n_splits, W.q, T, d.n_q_heads, d.n_kv_heads, d.head_dim, d_pos,
                                      d_slots, c->rope_cs, pool_slot, s));
        if (tap && c->taps.q) HIP_TRY(c, launch_copy_bytes(W.q, c->taps.q, (size_t)T * NQ * 2, s));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 3: attention
        AttnArgs a{};
        a.q = W.q; a.ldq = NQ; a.pool_slot = pool_slot;
        a.seqs = reinterpret_cast<const SeqInfo*>(db + ml.seqs);
        a.pages = reinterpret_cast<const int32_t*>(db + ml.pages);
        a.items = reinterpret_cast<const AttnItem*>(db + ml.items);
        a.n_items = (int)p.items.size();
        a.worker_begin = reinterpret_cast<const int32_t*>(db + ml.workers);
        a.n_workers = (int)p.worker_begin.size() - 1;
        a.n_team = p.n_team_workers;
        a.groups = reinterpret_cast<const MergeGroup*>(db + ml.groups);
        a.n_groups = (int)p.groups.size();
        a.max_splits = 0;
        a.max_merge_rows = 0;
        for (const MergeGroup& mg : p.groups) {
            a.max_splits = std::max(a.max_splits, (int)mg.n_splits);
            a.max_merge_rows = std::max(a.max_merge_rows, (int)mg.n_tok * (d.n_q_heads / d.n_kv_heads));
        }
        a.part_o = W.part_o; a.part_ml = W.part_ml; a.out = W.attn;
        a.n_q = d.n_q_heads; a.n_kv = d.n_kv_heads; a.d = d.head_dim;
        const bool time_attn = c->opt_time_attention > 0 && c->attn_ev_count < ATTN_EV_PAIRS &&
                               (c->step_counter % c->opt_time_attention) == 0;
        a.ev_begin = time_attn ? c->attn_ev[2 * c->attn_ev_count] : nullptr;
        a.ev_end = time_attn ? c->attn_ev[2 * c->attn_ev_count + 1] : nullptr;
        HIP_TRY(c, launch_attention(a, s));
        if (time_attn) c->attn_ev_count++;
        if (tap && c->taps.attn) HIP_TRY(c, launch_untile(W.attn, static_cast<bf16_t*>(c->taps.attn), T, NQ, s));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 4: O projection -> fp32 partials
        g.A = W.attn; g.Wp = L.wo_t; g.N = H; g.K = NQ;
        HIP_TRY(c, run_gemm(g, &n_splits, 1));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 5: x1 = x + sum(partials) (fp32), xn = RMSNorm(x1)
        ReduceAddNormArgs r{};
        r.resid = x_cur; r.resid_f32 = x_cur_f32; r.partials = W.part; r.n_splits = n_splits; r.T = T; r.H = H;
        r.x_f32 = W.x1; r.x_bf16 = nullptr; r.gain = L.g_ffn; r.xn = W.xn; r.eps = d.rms_eps;
        HIP_TRY(c, launch_reduce_add_norm(r, s));
        if (tap && c->taps.x1) HIP_TRY(c, launch_copy_bytes(W.x1, c->taps.x1, (size_t)T * H * 4, s));
        if (tap && c->taps.xn2) HIP_TRY(c, launch_untile(W.xn, static_cast<bf16_t*>(c->taps.xn2), T, H, s));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 6: gate/up + SwiGLU
        g.A = W.xn; g.Wp = L.wgu_t; g.N = 2 * F; g.K = H; g.kind = GemmOut::SWIGLU_BF16;
        g.out = W.act; g.out_bytes = W.act_bytes;
        HIP_TRY(c, run_gemm(g, nullptr, 2));
        if (tap && c->taps.act) HIP_TRY(c, launch_untile(W.act, static_cast<bf16_t*>(c->taps.act), T, F, s));
        if (stats) HIP_TRY(c, hipEventRecord(c->ev[++e], s));
        // 7: down projection -> fp32 partials; out = x1 + sum(partials); for an inner layer also the
        //    next layer's normalised input
        g.A = W.act; g.Wp = L.wd_t; g.N = H; g.K = F; g.kind = GemmOut::PARTIAL_F32;
        g.out = W.part; g.out_bytes = W.part_bytes;
        HIP_TRY(c, run_gemm(g, &n_splits, 3));
        r.resid = W.x1; r.resid_f32 = true; r.n_splits = n_splits;
        if (last) {
            r.x_f32 = out_f32 ? static_cast<float*>(x_out) : nullptr;
            r.x_bf16 = out_f32 ? nullptr : static_cast<bf16_t*>(x_out);
            r.gain = nullptr; r.xn = nullptr;
        } else {
            r.x_f32 = W.xmid; r.x_bf16 = nullptr;
            r.gain = c->layers[l + 1].g_attn; r.xn = W.xn;
        }
        HIP_TRY(c, launch_reduce_add_norm(r, s));
        void* x_next = last ? x_out : static_cast<void*>(W.xmid);
        if (tap && c->taps.x_out && (!last || out_f32))
            HIP_TRY(c, launch_copy_bytes(x_next, c->taps.x_out, (size_t)T * H * 4, s));
        if (stats) {
            HIP_TRY(c, hipEventRecord(c->ev[++e], s));
            HIP_TRY(c, hipEventSynchronize(c->ev[e]));
            for (int i = 0; i < PS_N_STAGES; i++) {
                float ms = 0.f;
                HIP_TRY(c, hipEventElapsedTime(&ms, c->ev[i], c->ev[i + 1]));
                stage_ms[i] += ms;
            }
            float ms = 0.f;
            HIP_TRY(c, hipEventElapsedTime(&ms, c->ev[0], c->ev[PS_N_STAGES]));
            total_ms += ms;
        }
        x_cur = x_next;
        x_cur_f32 = true;
    }
    if (stats) {
        stats->ms_total = total_ms;
        for (int i = 0; i < PS_N_STAGES; i++) stats->ms_stage[i] = stage_ms[i];
    }
    if (tio) {
        // head: RMS normalisation of every sequence's last new token, output projection, greedy token
        if (tio->ms) HIP_TRY(c, hipEventRecord(c->ev_head[2], s));
        const int M = p.n_seqs, V = c->vocab;
        float* logits = tio->logits;
        if (!logits) {
            const size_t need = (size_t)M * V * sizeof(float);
            if (need > c->logits_bytes) {
                HIP_TRY(c, hipStreamSynchronize(s));
                dev_free(c->ws_logits);
                c->logits_bytes = 0;
                if ((st = dev_alloc(c, &c->ws_logits, need + need / 4, "logits")) != PS_OK) return st;
                c->logits_bytes = need + need / 4;
            }
            logits = c->ws_logits;
        }
        int32_t* next = tio->next_tokens;
        if (!next) {
            if (M > c->next_cap) {
                HIP_TRY(c, hipStreamSynchronize(s));
                dev_free(c->ws_next);
                c->next_cap = 0;
                if ((st = dev_alloc(c, &c->ws_next, (size_t)(M + 64) * 4, "next tokens")) != PS_OK) return st;
                c->next_cap = M + 64;
            }
            next = c->ws_next;
        }
        HIP_TRY(c, launch_rmsnorm(x_out, true, c->g_final, W.xn, M, H, d.rms_eps, s, reinterpret_cast<const int32_t*>(db + ml.last_rows)));
        GemmArgs g{};
        g.A = W.xn; g.Wp = c->wout_t; g.M = M; g.N = V; g.K = H; g.kind = GemmOut::PARTIAL_F32;
        g.out = logits; g.out_bytes = (size_t)M * V * sizeof(float);
        g.split_k = 1;  // one partial buffer: it is the logits
        g.tile = c->opt_gemm_tile;
        g.sk_mode = c->opt_gemm_whole_tiles;
        g.sk_frag = W.skfrag; g.sk_frag_bytes = W.skfrag_bytes; g.sk_counters = W.skcnt; g.sk_n_counters = W.skcnt_n;
        int n_splits = 1;
        HIP_TRY(c, launch_gemm(g, &n_splits, s));
        if (n_splits != 1) return fail(c, PS_EDEVICE, "ps_step_tokens: output projection was split");
        HIP_TRY(c, launch_argmax_rows(logits, M, V, next, s));
        if (tio->ms) {
            HIP_TRY(c, hipEventRecord(c->ev_head[3], s));
            HIP_TRY(c, hipEventSynchronize(c->ev_head[3]));
            for (int i = 0; i < 3; i++) HIP_TRY(c, hipEventElapsedTime(&tio->ms[i], c->ev_head[i], c->ev_head[i + 1]));
        }
    }
    if (use_static) {   // the pinned slot may be refilled once the first kernel has read it; the step's end is a safe mark
        HIP_TRY(c, hipEventRecord(c->static_ev[sg_idx], c->stream));
        c->static_pending[sg_idx] = true;
        guard.committed = true;
        return PS_OK;
    }
    if ((st = staging_commit(c, sg_idx)) == PS_OK) guard.committed = true;
    return st;
}

extern "C" ps_status ps_step_static(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, const void* x_in, void* x_out) {
    if (c && !c->host_only && !c->static_scratch) return fail(c, PS_ESTATE, "ps_step_static: the context has no static scratch");
    return step_impl(c, seqs, n_seqs, x_in, x_out, nullptr, nullptr, true);
}

extern "C" ps_status ps_step(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, const void* x_in, void* x_out, ps_step_stats* stats) {
    return step_impl(c, seqs, n_seqs, x_in, x_out, stats, nullptr);
}

extern "C" ps_status ps_step_tokens(ps_ctx* c, const ps_seq* seqs, int32_t n_seqs, const int32_t* token_ids, int32_t* next_tokens,
                                    float* logits, float* hidden, ps_step_stats* stats, float* ms_parts) {
    const TokenIO tio{token_ids, next_tokens, logits, hidden, ms_parts};
    return step_impl(c, seqs, n_seqs, nullptr, nullptr, stats, &tio);
}

extern "C" ps_status ps_attention_times(ps_ctx* c, float* ms, int32_t cap, int32_t* n) {
    if (!c || !n || (!ms && cap > 0)) return fail(c, PS_EINVAL, "ps_attention_times: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_attention_times: host-only context");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const int cnt = std::min<int>(c->attn_ev_count, cap);
    for (int i = 0; i < cnt; i++) HIP_TRY(c, hipEventElapsedTime(&ms[i], c->attn_ev[2 * i], c->attn_ev[2 * i + 1]));
    *n = cnt;
    c->attn_ev_count = 0;
    return PS_OK;
}

extern "C" ps_status ps_gemm_times(ps_ctx* c, float* ms, int32_t cap, int32_t* n) {
    if (!c || !n || (!ms && cap > 0)) return fail(c, PS_EINVAL, "ps_gemm_times: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_gemm_times: host-only context");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const int cnt = std::min<int>(c->gemm_ev_count, cap);
    for (int i = 0; i < cnt; i++)
        for (int k = 0; k < 4; k++) HIP_TRY(c, hipEventElapsedTime(&ms[4 * i + k], c->gemm_ev[8 * i + 2 * k], c->gemm_ev[8 * i + 2 * k + 1]));
    *n = cnt;
    c->gemm_ev_count = 0;
    return PS_OK;
}

extern "C" ps_status ps_clock_under_load(ps_ctx* c, int32_t mfma_per_wavefront, int32_t wavefronts_per_simd, ps_clock_reading* out) {
    if (!c || !out) return fail(c, PS_EINVAL, "ps_clock_under_load: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_clock_under_load: host-only context");
    if (mfma_per_wavefront < 4096 || mfma_per_wavefront > (1 << 22)) return fail(c, PS_ERANGE, "ps_clock_under_load: mfma_per_wavefront outside [4096, 2^22]");
    if (wavefronts_per_simd != 1 && wavefronts_per_simd != 2 && wavefronts_per_simd != 4)
        return fail(c, PS_EINVAL, "ps_clock_under_load: wavefronts_per_simd must be 1, 2 or 4");
    int dev = 0, cus = 0, wall_khz = 0;
    HIP_TRY(c, hipGetDevice(&dev));
    HIP_TRY(c, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    HIP_TRY(c, hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, dev));
    if (cus <= 0 || wall_khz <= 0) return fail(c, PS_EDEVICE, "ps_clock_under_load: the device reports no compute units or no wall-clock rate");
    const int blocks = cus * wavefronts_per_simd, rounds = mfma_per_wavefront / 4;
    float* sink = nullptr;
    long long* ticks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ps_status st = PS_OK;
    hipError_t he = hipSuccess;
    float ms = 0.f;
    std::vector<long long> h((size_t)blocks * 2);
    if ((st = dev_alloc(c, &sink, (size_t)blocks * 256 * sizeof(float), "clock probe output")) != PS_OK) return st;
    if ((st = dev_alloc(c, &ticks, (size_t)blocks * 2 * sizeof(long long), "clock probe ticks")) != PS_OK) { dev_free(sink); return st; }
    // a short launch first, so that the timed one starts with the pipes and the clock already under load
    if ((he = hipEventCreate(&e0)) == hipSuccess && (he = hipEventCreate(&e1)) == hipSuccess &&
        (he = launch_mfma_clock_probe(blocks, 1024, sink, ticks, c->stream)) == hipSuccess &&
        (he = hipEventRecord(e0, c->stream)) == hipSuccess &&
        (he = launch_mfma_clock_probe(blocks, rounds, sink, ticks, c->stream)) == hipSuccess &&
        (he = hipEventRecord(e1, c->stream)) == hipSuccess && (he = hipStreamSynchronize(c->stream)) == hipSuccess &&
        (he = hipEventElapsedTime(&ms, e0, e1)) == hipSuccess)
        he = hipMemcpy(h.data(), ticks, h.size() * sizeof(long long), hipMemcpyDeviceToHost);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    dev_free(sink);
    dev_free(ticks);
    if (he != hipSuccess) return hip_fail(c, he, "ps_clock_under_load");
    double shader = 0, wall = 0;
    for (int b = 0; b < blocks; b++) { shader += (double)h[2 * b]; wall += (double)h[2 * b + 1]; }
    if (!(wall > 0) || !(ms > 0)) return fail(c, PS_EDEVICE, "ps_clock_under_load: the clocks did not advance");
    out->shader_mhz = shader / wall * (wall_khz / 1e3);
    out->ticks_per_mfma = shader / blocks / (4.0 * rounds);
    out->mfma_tflops = (double)blocks * 4 * (4.0 * rounds) * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
    out->elapsed_ms = ms;
    out->compute_units = cus;
    out->wavefronts_per_simd = wavefronts_per_simd;
    return PS_OK;
}

extern "C" ps_status ps_hbm_read_rate(ps_ctx* c, int64_t bytes, int32_t passes, double* gb_per_s) {
    if (!c || !gb_per_s) return fail(c, PS_EINVAL, "ps_hbm_read_rate: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_hbm_read_rate: host-only context");
    if (bytes < (1ll << 30) || bytes > (8ll << 30) || (bytes & 16383)) return fail(c, PS_ERANGE, "ps_hbm_read_rate: bytes must be a multiple of 16 KiB in [1 GiB, 8 GiB]");
    if (passes < 1 || passes > 16) return fail(c, PS_ERANGE, "ps_hbm_read_rate: passes outside [1, 16]");
    int dev = 0, cus = 0;
    HIP_TRY(c, hipGetDevice(&dev));
    HIP_TRY(c, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus <= 0) return fail(c, PS_EDEVICE, "ps_hbm_read_rate: the device reports no compute units");
    const int blocks = 2 * cus;  // eight wavefronts per compute unit
    uint8_t* buf = nullptr;
    uint32_t* out = nullptr;
    ps_status st = PS_OK;
    if ((st = dev_alloc(c, &buf, (size_t)bytes, "read-rate buffer")) != PS_OK) return st;
    if ((st = dev_alloc(c, &out, (size_t)blocks * 4 * sizeof(uint32_t), "read-rate output")) != PS_OK) { dev_free(buf); return st; }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t he = hipSuccess;
    float ms = 0.f;
    if ((he = hipEventCreate(&e0)) == hipSuccess && (he = hipEventCreate(&e1)) == hipSuccess &&
        (he = hipMemsetAsync(buf, 1, (size_t)bytes, c->stream)) == hipSuccess &&
        (he = launch_stream_read_probe(buf, (size_t)bytes, blocks, out, c->stream)) == hipSuccess &&  // untimed first pass
        (he = hipEventRecord(e0, c->stream)) == hipSuccess) {
        for (int i = 0; i < passes && he == hipSuccess; i++) he = launch_stream_read_probe(buf, (size_t)bytes, blocks, out, c->stream);
        if (he == hipSuccess && (he = hipEventRecord(e1, c->stream)) == hipSuccess && (he = hipStreamSynchronize(c->stream)) == hipSuccess)
            he = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (he != hipSuccess) (void)hipDeviceSynchronize();  // nothing may still be reading the buffer when it is freed
    dev_free(buf);
    dev_free(out);
    if (he != hipSuccess) return hip_fail(c, he, "ps_hbm_read_rate");
    if (!(ms > 0)) return fail(c, PS_EDEVICE, "ps_hbm_read_rate: no time elapsed");
    *gb_per_s = (double)bytes * passes / (ms * 1e-3) / 1e9;
    return PS_OK;
}

// ------------------------------------------------------------------------------ latency grid
static float median_of(std::vector<float> v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n == 0 ? 0.f : (n & 1 ? v[n / 2] : 0.5f * (v[n / 2 - 1] + v[n / 2]));
}

extern "C" ps_status ps_profile_grid(ps_ctx* c, const ps_grid_cell_spec* cells, int32_t n_cells, const ps_grid_opts* opts,
                                     const void* x_in, void* x_out, ps_grid_cell* out) {
    if (!c || !cells || !opts || !out || n_cells < 0) return fail(c, PS_EINVAL, "ps_profile_grid: null argument");
    if (c->host_only) return fail(c, PS_ESTATE, "ps_profile_grid: host-only context");
    if (opts->iters < 1 || opts->warmup < 0) return fail(c, PS_EINVAL, "ps_profile_grid: iters must be >= 1, warmup >= 0");
    hipEvent_t t0 = nullptr, t1 = nullptr;
    HIP_TRY(c, hipEventCreate(&t0));
    {
        const hipError_t e1 = hipEventCreate(&t1);
        if (e1 != hipSuccess) { (void)hipEventDestroy(t0); return hip_fail(c, e1, "hipEventCreate"); }
    }
    ps_status rc = PS_OK;
    const int64_t id_base = INT64_MIN / 2;  // request ids of the synthetic sequences
    for (int ci = 0; ci < n_cells && rc == PS_OK; ci++) {
        const ps_grid_cell_spec& cs = cells[ci];
        ps_grid_cell& oc = out[ci];
        memset(&oc, 0, sizeof(oc));
        oc.chunk = cs.chunk;
        oc.n_decode = cs.n_decode;
        oc.n_draws = cs.n_draws;
        oc.n_tokens = cs.chunk + cs.n_decode;
        if (cs.chunk < 0 || cs.n_decode < 0 || cs.n_draws < 1 || cs.n_draws > PS_GRID_MAX_DRAWS ||
            (cs.chunk > 0 && !cs.chunk_prefix) || (cs.n_decode > 0 && !cs.decode_kv)) {
            rc = fail(c, PS_EINVAL, "ps_profile_grid: malformed cell " + std::to_string(ci));
            break;
        }
        std::vector<float> draw_ms;
        std::vector<ps_step_stats> draw_stats(cs.n_draws);
        for (int dr = 0; dr < cs.n_draws && rc == PS_OK; dr++) {
            // build the batch: chunk first, then the decodes; pages from the allocator
            const int n_seqs = (cs.chunk > 0 ? 1 : 0) + cs.n_decode;
            std::vector<ps_seq> seqs(n_seqs);
            std::vector<std::vector<int32_t>> tables(n_seqs);
            int si = 0, reserved = 0;
            auto add = [&](int n_new, int kv_len) -> ps_status {
                std::vector<int32_t>& t = tables[si];
                t.resize((kv_len + PS_PAGE_SIZE - 1) / PS_PAGE_SIZE);
                int32_t n = 0;
                ps_status st = ps_kv_reserve(c, id_base + si, kv_len, t.data(), (int32_t)t.size(), &n);
                if (st != PS_OK) return st;
                reserved = si + 1;
                seqs[si] = ps_seq{id_base + si, n_new, kv_len, t.data(), n};
                si++;
                return PS_OK;
            };
            if (cs.chunk > 0) rc = add(cs.chunk, cs.chunk_prefix[dr] + cs.chunk);
            for (int j = 0; j < cs.n_decode && rc == PS_OK; j++) rc = add(1, cs.decode_kv[(size_t)dr * cs.n_decode + j]);
            if (rc == PS_OK) {
                for (int w = 0; w < opts->warmup && rc == PS_OK; w++) rc = ps_step(c, seqs.data(), n_seqs, x_in, x_out, nullptr);
                std::vector<float> it_ms;
                for (int it = 0; it < opts->iters && rc == PS_OK; it++) {
                    hipError_t e = hipEventRecord(t0, c->stream);
                    if (e == hipSuccess) rc = ps_step(c, seqs.data(), n_seqs, x_in, x_out, nullptr);
                    if (rc != PS_OK) break;
                    if (e == hipSuccess) e = hipEventRecord(t1, c->stream);
                    if (e == hipSuccess) e = hipEventSynchronize(t1);
                    float ms = 0.f;
                    if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
                    if (e != hipSuccess) { rc = hip_fail(c, e, "ps_profile_grid timing"); break; }
                    it_ms.push_back(ms);
                }
                if (rc == PS_OK) {
                    draw_ms.push_back(median_of(it_ms));
                    rc = ps_step(c, seqs.data(), n_seqs, x_in, x_out, &draw_stats[dr]);  // one more pass for the stage split
                }
            }
            for (int k = 0; k < reserved; k++) (void)ps_kv_release(c, id_base + k);
        }
        if (rc != PS_OK) break;
        // median draw = the one whose time is the (lower) median
        std::vector<int> order(cs.n_draws);
        for (int i = 0; i < cs.n_draws; i++) order[i] = i;
        std::sort(order.begin(), order.end(), [&](int a, int b) { return draw_ms[a] < draw_ms[b]; });
        const int med = order[(cs.n_draws - 1) / 2];
        oc.median_ms = median_of(draw_ms);
        oc.total_kv = draw_stats[med].total_kv;
        for (int i = 0; i < PS_N_STAGES; i++) oc.stage_ms[i] = draw_stats[med].ms_stage[i];
        for (int i = 0; i < cs.n_draws; i++) {
            oc.draw_ms[i] = draw_ms[i];
            oc.draw_total_kv[i] = draw_stats[i].total_kv;
        }
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    return rc;
}
