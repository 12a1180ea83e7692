// Internal declarations shared by the host code and the gfx950 kernels of libpolystep.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/polystep.h"

namespace ps {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

// ---------------------------------------------------------------------------------
// KV pool layout (one physical layer slot):  [page][kv_head][K|V][16 * head_dim] bf16.
// Inside a 16-token x head_dim chunk the elements are ordered so that a wavefront's
// 16-byte-per-lane loads are both contiguous (1 KiB per instruction) and already in
// MFMA operand order:
//   K chunk: [s = d/32][g = 4][tok = 16][8]      element (tok, dd): s = dd/32, g = (dd%32)/8
//   V chunk: [p = d/32][g = 4][dl = 16][h = 2][4] element (tok, dd): p = dd/32, h = (dd/16)%2,
//                                                 dl = dd%16, g = tok/4, i = tok%4
// ---------------------------------------------------------------------------------
__host__ __device__ inline int k_elem_offset(int tok, int dd) {
    return (((dd >> 5) * 4 + ((dd & 31) >> 3)) * 16 + tok) * 8 + (dd & 7);
}
__host__ __device__ inline int v_elem_offset(int tok, int dd) {
    return ((((dd >> 5) * 4 + (tok >> 2)) * 16 + (dd & 15)) * 2 + ((dd >> 4) & 1)) * 4 + (tok & 3);
}

// Activation matrices that feed a GEMM (normalised inputs, attention output, gated activation)
// are kept in MFMA operand order rather than row-major:
//   [m_tile = m/16][k_block = k/32][g = (k%32)/8][mm = m%16][8]          (1 KiB per tile-block)
// so that the consumer's operand load is one contiguous KiB per wavefront instruction (a
// row-major gather of 16 rows x 64 bytes costs twice the cache-line requests and measurably
// starves the weight stream).  Storage holds ceil(M/16)*16 rows; rows beyond M are never read
// into a stored result.
__host__ __device__ inline size_t act_offset(int m, int k, int K) {
    return ((((size_t)(m >> 4) * (K >> 5) + (k >> 5)) * 4 + ((k & 31) >> 3)) * 16 + (m & 15)) * 8 + (k & 7);
}

// Attention work item.  The first 8 fields are what ps_plan_attention reports; the rest is
// what the kernel needs so that it never has to look the sequence up.
struct AttnItem {
    int32_t seq;         // index into the step's sequence table
    int32_t kv_head;
    int32_t q_tok0;      // first new-token index (within the sequence) of the query block
    int32_t q_ntok;      // query tokens in the block
    int32_t page_begin;  // logical KV pages [page_begin, page_end)
    int32_t page_end;
    int32_t partial;     // first partial slot, or -1: the item covers its whole KV span
    int32_t worker;      // worker the item is assigned to: a team (block of four wavefronts) or a single wavefront
    int32_t tok_g0;      // global token index of the block's first query token
    int32_t pos0;        // cache position of that token
    int32_t page_off;    // offset of the sequence's page list in the flat page array
    int32_t page0, page1;  // physical ids of the item's first two pages: the first loads need no table lookup
    int32_t pad0, pad1, pad2;
};

// Split-KV merge group: one 16-row query tile of one (sequence, kv head).
struct MergeGroup {
    int32_t tok0;        // global token index of the tile's first token
    int32_t n_tok;       // valid tokens in the tile
    int32_t kv_head;
    int32_t first_slot;  // slot of split j is first_slot + j * stride
    int32_t n_splits;
    int32_t stride;
    int32_t pad0, pad1;
};

// Per-sequence record on the device.
struct SeqInfo {
    int32_t tok0;      // cu_seqlens
    int32_t n_new;
    int32_t kv_len;
    int32_t page_off;  // offset of its page list in the flat page array
};

struct GemmOut {
    enum Kind : int { PARTIAL_F32 = 0, SWIGLU_BF16 = 1 };
};

// ------------------------------------------------------------------ launchers (device side)
// All take the stream explicitly and return hipGetLastError() of the launch.
// out is written in operand order (act_offset)
// src_rows: output row i normalises input row src_rows[i].  meta_*: extra blocks of the launch copy meta_bytes (a multiple
// of 16) from device-visible host memory to device memory (the step's metadata, see rmsnorm_kernel)
hipError_t launch_rmsnorm(const void* x, bool x_is_f32, const bf16_t* gain, bf16_t* out, int T, int H, float eps,
                          hipStream_t st, const int32_t* src_rows = nullptr, const void* meta_src = nullptr, void* meta_dst = nullptr,
                          size_t meta_bytes = 0);
hipError_t launch_embed_gather(const bf16_t* table, const int32_t* ids, bf16_t* out, int T, int H, hipStream_t st);
hipError_t launch_argmax_rows(const float* x, int M, int N, int32_t* out, hipStream_t st);
// operand-order [M][K] bf16 matrix -> row-major (for the debug taps)
hipError_t launch_untile(const bf16_t* src, bf16_t* dst, int M, int K, hipStream_t st);
// qkv: fp32 partials [n_splits][T][(n_q + 2 n_kv) d] of the QKV projection (summed here)
hipError_t launch_rope_append(const float* qkv, int n_splits, bf16_t* q_out, int T, int n_q, int n_kv, int d,
                              const int32_t* positions, const int32_t* slots, const float* rope_cs, bf16_t* pool_slot,
                              hipStream_t st);
// x = resid + sum of n_splits fp32 partials [n_splits][T][H]; writes any of: x as fp32, x as bf16,
// rmsnorm(x) * gain as bf16 (gain == null: no normalisation)
struct ReduceAddNormArgs {
    const void* resid;
    bool resid_f32;
    const float* partials;
    int n_splits;
    int T, H;
    float* x_f32;          // may be null
    bf16_t* x_bf16;        // may be null
    const bf16_t* gain;    // may be null
    bf16_t* xn;            // required when gain != null; operand order (act_offset)
    float eps;
};
hipError_t launch_reduce_add_norm(const ReduceAddNormArgs& a, hipStream_t st);
hipError_t launch_kv_copy(bool to_pool, bf16_t* pool_slot, const int32_t* slots_dev, int n, int phase, int n_kv, int d, bf16_t* k,
                          bf16_t* v, hipStream_t st);
hipError_t launch_repack_weight(const bf16_t* w, bf16_t* wp, int K, int N, int interleave, hipStream_t st);
hipError_t launch_copy_bytes(const void* src, void* dst, size_t n, hipStream_t st);
// sink: blocks * 256 floats; ticks: blocks * 2 (shader-clock ticks, wall-clock ticks of wavefront 0 of each block)
hipError_t launch_mfma_clock_probe(int blocks, int rounds, float* sink, long long* ticks, hipStream_t st);
// reads the first bytes / 16 KiB whole 16 KiB chunks of buf; out: blocks * 4 words
hipError_t launch_stream_read_probe(const void* buf, size_t bytes, int blocks, uint32_t* out, hipStream_t st);

struct GemmArgs {
    const bf16_t* A;   // [M][K] activations in operand order (act_offset)
    const bf16_t* Wp;  // repacked weights (launch_repack_weight)
    int M, N, K;
    int kind;          // GemmOut::Kind
    void* out;         // PARTIAL_F32: fp32 [splits][M][N] row-major; SWIGLU_BF16: bf16 [M][N/2] in operand order
    size_t out_bytes;  // capacity of out; at least gemm_out_bytes(...)
    int split_k;       // 0 = choose
    int tile;          // M > 64: 0 = choose (streaming up to 96 tokens, then a tile), 128 or 256 = block tile edge
    // tiled kernel only (see gemm_workspace): parked accumulators of K runs that cover part of a tile, and one counter
    // per tile that must be zero on entry (the kernel leaves it zero)
    int sk_mode;       // 0 = the cost model decides whether the tail's K loops are cut, 1 = never (whole tiles only), 2 = wherever possible
    float* sk_frag;
    size_t sk_frag_bytes;
    int* sk_counters;
    int sk_n_counters;
};
// *n_splits receives the number of partial buffers written (1 for SWIGLU_BF16)
hipError_t launch_gemm(const GemmArgs& a, int* n_splits, hipStream_t st);
size_t gemm_out_bytes(int M, int N, int K, int kind, int split_k_opt, int tile_opt);
// what launch_gemm needs in sk_frag / sk_counters for this shape (both 0 where the streaming kernel serves it)
void gemm_workspace(int M, int N, int K, int kind, int split_k_opt, int tile_opt, int sk_mode, size_t* frag_bytes, int* n_counters);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);   // bytes: rounded down to a multiple of 16
hipError_t launch_fill_words(void* p, size_t bytes, uint32_t word, hipStream_t st);

struct AttnArgs {
    const bf16_t* q;   // rotated queries [T][n_q * d]: row stride ldq elements
    int ldq;
    const bf16_t* pool_slot;
    const SeqInfo* seqs;
    const int32_t* pages;
    const AttnItem* items;
    int n_items;
    const int32_t* worker_begin;  // [n_workers + 1]: items of worker w are [worker_begin[w], worker_begin[w+1])
    int n_workers;
    int n_team;        // the first n_team workers are teams (one block each), the rest single wavefronts
    int team_per_xcd, wave_blocks_per_xcd;   // set by launch_attention
    const MergeGroup* groups;
    int n_groups;
    int max_splits;    // largest n_splits of any group: sizes the merge kernel's blocks
    int max_merge_rows;   // largest n_tok * G over the merge groups (rows of a tile that are merged)
    float* part_o;     // [slot][16][d]
    float* part_ml;    // [slot][16][2]
    bf16_t* out;       // [T][n_q * d] in operand order (act_offset)
    int n_q, n_kv, d;
    hipEvent_t ev_begin, ev_end;  // optional: recorded right before / after the main kernel (not the merge)
};
hipError_t launch_attention(const AttnArgs& a, hipStream_t st);
int attention_worker_slots();  // wavefronts of the attention kernel that are resident at once on this device

}  // namespace ps
