// Paged-KV attention for a mixed batch in one launch (Sec. 2.1: Softmax(QK^T/sqrt(d))V over
// the keys and values of all previous tokens; Sec. 2.4: a prefill chunk against its cached
// prefix together with one-token decodes; Sec. 2.2: decode attention gets no batching
// benefit, its cost follows the KV bytes read).
//
// One wavefront per worker; a worker runs a short list of work items = (sequence, kv head, query
// block, KV page range) of equal total weight (see the planner), so all wavefronts stream for the
// same time.  Decode items keep the next pair of pages in flight in registers while the current
// pair is consumed.  A query
// tile is 16 rows = (16/G tokens) x (G query heads of the kv head), so every K/V byte is
// read once for the whole GQA group.  Per pair of 16-token pages:
//     S^T[key][row]  = K . Q^T      (MFMA 16x16x32, K chunk is the A operand)
//     online softmax over keys     (4 keys per lane in-register, 2 shuffles across lane groups)
//     O^T[d][row]   += V^T . P^T    (MFMA 16x16x32; the S^T accumulator layout is already
//                                    the B-operand layout, so P never leaves registers)
// The cache stores K and V chunks pre-ordered for these operands (see ps_common.h), so every
// load instruction of a wave fetches 1 KiB of contiguous memory.
// Items that cover only part of a KV span write (max, sum, unnormalised O) partials; a merge
// kernel combines them.
#include "ps_device.h"

#include <algorithm>

namespace ps {

constexpr float NEG_BIG = -1.0e30f;

// K and V chunks of a pair of pages, as loaded: 16 bytes per lane per register.
template <int KS>
struct PairRegs {
    uint4 ka[KS], kb[KS], va[KS], vb[KS];
};

template <int D>
__device__ __forceinline__ void load_pair(PairRegs<D / 32>& p, const bf16_t* pool_lane, size_t page_stride, int pa, int pb) {
    constexpr int KS = D / 32;
    const bf16_t* ca = pool_lane + (size_t)pa * page_stride;
    const bf16_t* cb = pool_lane + (size_t)pb * page_stride;
#pragma unroll
    for (int s = 0; s < KS; s++) {
        p.ka[s] = ldg16(ca + s * 512);
        p.kb[s] = ldg16(cb + s * 512);
    }
#pragma unroll
    for (int s = 0; s < KS; s++) {
        p.va[s] = ldg16(ca + 16 * D + s * 512);
        p.vb[s] = ldg16(cb + 16 * D + s * 512);
    }
}

// Running softmax state of NT query tiles against one KV stream.
template <int D, int NT>
struct TileState {
    f32x4_t o[NT][D / 16];
    float m[NT], lsum[NT];
};

// Maximum over the four lanes r, r+16, r+32, r+48 that share a query row, in the vector ALU:
// v_permlane16_swap (x, x) returns {rows 0,0,2,2 | rows 1,1,3,3} of x and v_permlane32_swap the
// {lower, lower | upper, upper} halves, so each step combines a lane with its partner in both.
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float row_quad_max(float v) {
    const u32x2_t a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
    const u32x2_t b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}

// One pair of pages (32 keys) for all NT query tiles.  kpos0 = position of the pair's first key;
// b_valid = the second page exists.  PV16 selects how P.V is issued: per page with 16x16x16 MFMAs
// (bandwidth-bound decode items) or per pair with one 16x16x32 MFMA (compute-bound prefill items).
template <int D, int NT, bool PV16>
__device__ __forceinline__ void compute_pair(TileState<D, NT>& st, const PairRegs<D / 32>& p, const bf16x8_t (&qf)[NT][D / 32],
                                             const int (&pq)[NT], int kpos0, bool b_valid, int g, float scale2) {
    constexpr int KS = D / 32, DT = D / 16;
    const int kpos_a = kpos0 + 4 * g, kpos_b = kpos_a + 16;
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; s++) {
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(p.ka[s]), qf[nt][s], sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(p.kb[s]), qf[nt][s], sb, 0, 0, 0);
        }
        // scores stay raw; the scale (> 0) goes into the running max and into the exponent's fma
        float sv[8];
        bool ok[8];
        float mx = NEG_BIG;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            ok[i] = kpos_a + i <= pq[nt];
            ok[4 + i] = b_valid && (kpos_b + i <= pq[nt]);
            sv[i] = sa[i];
            sv[4 + i] = sb[i];
        }
#pragma unroll
        for (int i = 0; i < 8; i++) mx = ok[i] ? fmaxf(mx, sv[i]) : mx;
        mx = row_quad_max(mx);
        const float m_new = fmaxf(st.m[nt], mx * scale2);
        const float alpha = __builtin_amdgcn_exp2f(st.m[nt] - m_new);
        st.m[nt] = m_new;
        float pv[8], ps = 0.f;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            pv[i] = ok[i] ? __builtin_amdgcn_exp2f(fmaf(sv[i], scale2, -m_new)) : 0.f;
            ps += pv[i];
        }
        st.lsum[nt] = st.lsum[nt] * alpha + ps;
        if constexpr (PV16) {
            // one 16x16x16 MFMA per page and d-tile: each 8-byte half of a loaded V register
            // quad is an operand as it stands, so no register moves sit between load and use
            const uint2 pwa = {pack_bf16(pv[0], pv[1]), pack_bf16(pv[2], pv[3])};
            const uint2 pwb = {pack_bf16(pv[4], pv[5]), pack_bf16(pv[6], pv[7])};
            const s16x4_t pfa = __builtin_bit_cast(s16x4_t, pwa), pfb = __builtin_bit_cast(s16x4_t, pwb);
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
                const int s = dt >> 1;
                const uint2 wa = (dt & 1) ? uint2{p.va[s].z, p.va[s].w} : uint2{p.va[s].x, p.va[s].y};
                const uint2 wb = (dt & 1) ? uint2{p.vb[s].z, p.vb[s].w} : uint2{p.vb[s].x, p.vb[s].y};
                f32x4_t acc = st.o[nt][dt];
                acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, wa), pfa, acc, 0, 0, 0);
                st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, wb), pfb, acc, 0, 0, 0);
            }
        } else {
            uint4 pw;
            pw.x = pack_bf16(pv[0], pv[1]);
            pw.y = pack_bf16(pv[2], pv[3]);
            pw.z = pack_bf16(pv[4], pv[5]);
            pw.w = pack_bf16(pv[6], pv[7]);
            const bf16x8_t pf = as_bf16x8(pw);
            // once the running max has settled alpha is exactly 1 in every lane: skip the D/4 multiplies
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int dt = 0; dt < DT; dt++) {
                    st.o[nt][dt][0] *= alpha; st.o[nt][dt][1] *= alpha; st.o[nt][dt][2] *= alpha; st.o[nt][dt][3] *= alpha;
                }
            }
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
                const int s = dt >> 1;
                uint4 vw;
                if (dt & 1) { vw.x = p.va[s].z; vw.y = p.va[s].w; vw.z = p.vb[s].z; vw.w = p.vb[s].w; }
                else        { vw.x = p.va[s].x; vw.y = p.va[s].y; vw.z = p.vb[s].x; vw.w = p.vb[s].y; }
                st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vw), pf, st.o[nt][dt], 0, 0, 0);
            }
        }
    }
}

// One work item on one wavefront.  PIPE = true keeps the next pair of pages in flight in a second
// register set while the current pair is consumed (decode items: the wave is bandwidth-bound).
template <int D, int G, int NT, bool PIPE>
__device__ __forceinline__ void attn_item(const AttnArgs& a, const AttnItem it) {
    constexpr int KS = D / 32;   // MFMA k-steps over head_dim
    constexpr int DT = D / 16;   // 16-row tiles of O^T
    constexpr int TQ = 16 / G;   // tokens per query tile
    const int lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;

    const int32_t* pages = a.pages + it.page_off;
    const int head = it.kv_head * G + (r % G);

    int qi[NT], pq[NT];  // global token index and cache position of this lane's query row, per tile
    bool rvalid[NT];
    bf16x8_t qf[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        const int ql = nt * TQ + r / G;  // token of the row within the block
        rvalid[nt] = ql < it.q_ntok;
        const int qc = min(ql, it.q_ntok - 1);
        qi[nt] = it.tok_g0 + qc;
        pq[nt] = it.pos0 + qc;
        const bf16_t* qrow = a.q + (size_t)qi[nt] * a.ldq + head * D + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; s++) qf[nt][s] = as_bf16x8(ldg16(qrow + 32 * s));
    }

    TileState<D, NT> st;
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        st.m[nt] = NEG_BIG;
        st.lsum[nt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; dt++) st.o[nt][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    const float scale2 = 1.4426950408889634f / sqrtf((float)D);  // log2(e)/sqrt(d): softmax in base 2
    const size_t page_stride = (size_t)a.n_kv * 2 * 16 * D;
    const bf16_t* pool_lane = a.pool_slot + (size_t)it.kv_head * 2 * 16 * D + (size_t)lane * 8;

    // Pages are consumed in blocks of up to 64: lane l keeps the id of the block's page l, and a
    // uniform readlane hands the ids out, so no load sits between a pair's id and its data.
    for (int blk = it.page_begin; blk < it.page_end; blk += 64) {
        const int n_pg = min(64, it.page_end - blk);
        const int my_pid = pages[blk + min(lane, n_pg - 1)];
        const int n_pairs = (n_pg + 1) >> 1;
        const bool first_blk = blk == it.page_begin;
        // the item carries its first two page ids, so the first pair's loads do not wait for my_pid
        auto pid = [&](int j) {
            if (j < 2 && first_blk) return j == 0 ? it.page0 : it.page1;
            return __builtin_amdgcn_readlane(my_pid, min(j, n_pg - 1));
        };
        if constexpr (PIPE) {
            // Two register sets; the steady-state body issues its loads unconditionally so that the
            // wait before each compute covers exactly the older set (a conditional load would force
            // a wait for everything at the join).
            PairRegs<KS> b0, b1;
            load_pair<D>(b0, pool_lane, page_stride, pid(0), pid(1));
            int i = 0;
            for (; i + 2 < n_pairs; i += 2) {
                // scheduling barriers: keep every batch of loads ahead of the previous batch's math
                load_pair<D>(b1, pool_lane, page_stride, pid(2 * i + 2), pid(2 * i + 3));
                __builtin_amdgcn_sched_barrier(0);
                compute_pair<D, NT, PIPE>(st, b0, qf, pq, (blk + 2 * i) * 16, true, g, scale2);
                __builtin_amdgcn_sched_barrier(0);
                load_pair<D>(b0, pool_lane, page_stride, pid(2 * i + 4), pid(2 * i + 5));
                __builtin_amdgcn_sched_barrier(0);
                compute_pair<D, NT, PIPE>(st, b1, qf, pq, (blk + 2 * i + 2) * 16, true, g, scale2);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (i + 2 == n_pairs) {
                load_pair<D>(b1, pool_lane, page_stride, pid(2 * i + 2), pid(2 * i + 3));
                compute_pair<D, NT, PIPE>(st, b0, qf, pq, (blk + 2 * i) * 16, true, g, scale2);
                compute_pair<D, NT, PIPE>(st, b1, qf, pq, (blk + 2 * i + 2) * 16, 2 * i + 3 < n_pg, g, scale2);
            } else {
                compute_pair<D, NT, PIPE>(st, b0, qf, pq, (blk + 2 * i) * 16, 2 * i + 1 < n_pg, g, scale2);
            }
        } else {
            PairRegs<KS> b0;
            for (int i = 0; i < n_pairs; i++) {
                load_pair<D>(b0, pool_lane, page_stride, pid(2 * i), pid(2 * i + 1));
                compute_pair<D, NT, PIPE>(st, b0, qf, pq, (blk + 2 * i) * 16, 2 * i + 1 < n_pg, g, scale2);
            }
        }
    }

#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        float l = st.lsum[nt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (it.partial < 0) {
            if (rvalid[nt]) {
                const float inv = 1.0f / l;
#pragma unroll
                for (int dt = 0; dt < DT; dt++) {
                    uint2 w;
                    w.x = pack_bf16(st.o[nt][dt][0] * inv, st.o[nt][dt][1] * inv);
                    w.y = pack_bf16(st.o[nt][dt][2] * inv, st.o[nt][dt][3] * inv);
                    *reinterpret_cast<uint2*>(a.out + act_offset(qi[nt], head * D + 16 * dt + 4 * g, a.n_q * D)) = w;
                }
            }
        } else if (rvalid[nt]) {  // rows beyond the block's tokens are never merged: do not store them
            const size_t slot = (size_t)it.partial + nt;
            float* po = a.part_o + (slot * 16 + r) * D + 4 * g;
#pragma unroll
            for (int dt = 0; dt < DT; dt++)
                *reinterpret_cast<float4*>(po + 16 * dt) = float4{st.o[nt][dt][0], st.o[nt][dt][1], st.o[nt][dt][2], st.o[nt][dt][3]};
            if (g == 0) {
                float* pm = a.part_ml + (slot * 16 + r) * 2;
                pm[0] = st.m[nt];
                pm[1] = l;
            }
        }
    }
}

constexpr int PREFILL_NT = 2;  // query tiles per wave for multi-tile (prefill) items

template <int D, int G>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_kernel(AttnArgs a) {
    // one wavefront = one worker: it runs the items the planner assigned to it, in order
    constexpr int TQ = 16 / G;
    // consecutive block ids go to different XCDs (one L2 each): XCD x runs the contiguous workers
    // [x * per_xcd, (x+1) * per_xcd), i.e. neighbouring parts of the work list share an L2
    const int per_xcd = (a.n_workers + 7) >> 3;
    const int w = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (w >= a.n_workers) return;
    const int i0 = a.worker_begin[w], i1 = a.worker_begin[w + 1];
    for (int i = i0; i < i1; i++) {
        const AttnItem it = a.items[i];
        if (it.q_ntok <= TQ)
            attn_item<D, G, 1, true>(a, it);
        else
            attn_item<D, G, PREFILL_NT, false>(a, it);
    }
}

// Combine split partials of one query tile: out = sum_j 2^(m_j - M) O_j / sum_j 2^(m_j - M) l_j.
// One block per merge group.  A tile is n_rows x D/4 float4 pieces, 64 pieces per pass and wavefront.  The block's
// wavefronts form a (pass, split) grid: wavefront (wp, ws) takes the passes wp, wp + NWP, ... and of each the splits
// ws, ws + NWS, ...  Passes are independent, so a 16-row prefill tile (eight passes) costs the latency of one;
// the NWS wavefronts of a pass (a sequence cut over hundreds of workers would otherwise be merged split after split)
// each reduce their share to (max, sum, O) against their own maximum, and the first of them combines the NWS results
// through LDS in a fixed order.
constexpr int MERGE_MAX_WAVES = 16;

template <int D, int G>
__global__ __launch_bounds__(64 * MERGE_MAX_WAVES) void attn_merge_kernel(AttnArgs a, int NWS) {
    __shared__ float4 s_acc[MERGE_MAX_WAVES][64];
    __shared__ float2 s_ml[MERGE_MAX_WAVES][64];
    const MergeGroup mg = a.groups[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
    const int NWP = NW / NWS, ws = wave % NWS, wp = wave / NWS;
    const int n_rows = mg.n_tok * G;  // valid rows are the first n_tok * G of the tile
    const int n_items = n_rows * (D / 4);
    for (int c0 = 0; c0 < n_items; c0 += 64 * NWP) {   // the same trip count for every wavefront: the barriers below
        const int c = c0 + wp * 64 + lane;
        const bool live = c < n_items;
        const int r = live ? c / (D / 4) : 0, col = live ? (c % (D / 4)) * 4 : 0;
        // this wavefront's splits, eight at a time with all loads of a batch issued together
        float M = NEG_BIG;
        for (int j0 = ws; j0 < mg.n_splits; j0 += 8 * NWS) {
            float mv[8];
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (j0 + j * NWS < mg.n_splits) mv[j] = a.part_ml[((size_t)(mg.first_slot + (j0 + j * NWS) * mg.stride) * 16 + r) * 2];
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (j0 + j * NWS < mg.n_splits) M = fmaxf(M, mv[j]);
        }
        float4 acc = {0.f, 0.f, 0.f, 0.f};
        float L = 0.f;
        for (int j0 = ws; j0 < mg.n_splits; j0 += 8 * NWS) {
            float2 ml[8];
            float4 v[8];
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (j0 + j * NWS < mg.n_splits) {
                    const size_t row = (size_t)(mg.first_slot + (j0 + j * NWS) * mg.stride) * 16 + r;
                    ml[j] = *reinterpret_cast<const float2*>(a.part_ml + row * 2);
                    v[j] = *reinterpret_cast<const float4*>(a.part_o + row * D + col);
                }
#pragma unroll
            for (int j = 0; j < 8; j++)
                if (j0 + j * NWS < mg.n_splits) {
                    const float w = __builtin_amdgcn_exp2f(ml[j].x - M);
                    L += w * ml[j].y;
                    acc.x += w * v[j].x; acc.y += w * v[j].y; acc.z += w * v[j].z; acc.w += w * v[j].w;
                }
        }
        if (NWS > 1) {
            s_acc[wave][lane] = acc;
            s_ml[wave][lane] = float2{M, L};
            __syncthreads();
            if (ws == 0) {
                for (int w = 1; w < NWS; w++) M = fmaxf(M, s_ml[wave + w][lane].x);
                acc = float4{0.f, 0.f, 0.f, 0.f};
                L = 0.f;
                for (int w = 0; w < NWS; w++) {
                    const float2 q = s_ml[wave + w][lane];
                    const float4 v = s_acc[wave + w][lane];
                    const float f = __builtin_amdgcn_exp2f(q.x - M);  // a wavefront without splits holds (NEG_BIG, 0, 0): f * 0
                    L += f * q.y;
                    acc.x += f * v.x; acc.y += f * v.y; acc.z += f * v.z; acc.w += f * v.w;
                }
            }
        }
        if (ws == 0 && live) {
            const float inv = 1.0f / L;
            const int head = mg.kv_head * G + r % G;
            uint2 w;
            w.x = pack_bf16(acc.x * inv, acc.y * inv);
            w.y = pack_bf16(acc.z * inv, acc.w * inv);
            *reinterpret_cast<uint2*>(a.out + act_offset(mg.tok0 + r / G, head * D + col, a.n_q * D)) = w;
        }
        if (NWS > 1) __syncthreads();  // the next pass overwrites the LDS slots
    }
}

int attn_prefill_tokens_per_item(int G) { return PREFILL_NT * (16 / G); }

template <int D, int G>
static hipError_t launch_dg(const AttnArgs& a, hipStream_t st) {
    if (a.ev_begin) (void)hipEventRecord(a.ev_begin, st);
    hipLaunchKernelGGL((attn_kernel<D, G>), dim3(((a.n_workers + 7) >> 3) * 8), dim3(64), 0, st, a);
    hipError_t e = hipGetLastError();
    if (a.ev_end) (void)hipEventRecord(a.ev_end, st);
    if (e != hipSuccess || a.n_groups == 0) return e;
    // wavefronts that share a pass's splits: about eight splits each (one batch of loads), a power of two up to 16;
    // the rest of the block's 16 wavefronts take different passes, as many as the largest tile has
    int nws = 1;
    while (nws < MERGE_MAX_WAVES && nws * 8 < a.max_splits) nws *= 2;
    const int passes = (std::max(1, a.max_merge_rows) * (D / 4) + 63) / 64;
    int nwp = 1;
    while (nwp * 2 * nws <= MERGE_MAX_WAVES && nwp < passes) nwp *= 2;
    hipLaunchKernelGGL((attn_merge_kernel<D, G>), dim3(a.n_groups), dim3(64 * nws * nwp), 0, st, a, nws);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const AttnArgs& a, hipStream_t st) {
    switch (a.n_q / a.n_kv) {
        case 1: return launch_dg<D, 1>(a, st);
        case 2: return launch_dg<D, 2>(a, st);
        case 4: return launch_dg<D, 4>(a, st);
        case 8: return launch_dg<D, 8>(a, st);
        case 16: return launch_dg<D, 16>(a, st);
    }
    return hipErrorInvalidValue;
}

// Resident wavefronts of the attention kernel: CUs x 4 SIMDs x 2 (the kernel is built for two
// wavefronts per SIMD).
int attention_worker_slots() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 2048;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 2048;
    return cus * 4 * 2;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
    if (a.n_items <= 0 || a.n_workers <= 0) return hipSuccess;
    if (a.d == 128) return launch_d<128>(a, st);
    if (a.d == 64) return launch_d<64>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace ps
