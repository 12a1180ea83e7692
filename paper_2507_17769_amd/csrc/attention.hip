// Paged-KV attention for a mixed batch in one launch (Sec. 2.1: Softmax(QK^T/sqrt(d))V over
// the keys and values of all previous tokens; Sec. 2.4: a prefill chunk against its cached
// prefix together with one-token decodes; Sec. 2.2: decode attention gets no batching
// benefit, its cost follows the KV bytes read).
//
// A worker runs a short list of work items = (sequence, kv head, query block, KV page range) of
// equal total weight (see the planner), so all workers of a kind run for the same time.  Decode
// items belong to single wavefronts, which keep the next pair of pages in flight in registers while
// the current pair is consumed.  The query blocks of a prefill chunk belong to teams: the four
// wavefronts of a block take TEAM_NT query tiles each and share every pair of pages through a ring
// in LDS that global_load_lds fills two pairs ahead, so a pair is fetched from L2 once per 4 TEAM_NT
// tiles and needs no registers while in flight (three tiles are what the register file holds: the
// accumulators of the tiles, their queries and one set of K and V operands).  A query
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

// Decode streams read every byte once: they load with the non-temporal hint (ldg16_stream), so that they do not push
// out of L2 what the teams of the same launch re-read (the keys and values of the prefill chunk's prefix).
template <int D>
__device__ __forceinline__ void load_pair(PairRegs<D / 32>& p, const bf16_t* pool_lane, size_t page_stride, int pa, int pb) {
    constexpr int KS = D / 32;
    const bf16_t* ca = pool_lane + (size_t)pa * page_stride;
    const bf16_t* cb = pool_lane + (size_t)pb * page_stride;
#pragma unroll
    for (int s = 0; s < KS; s++) {
        p.ka[s] = ldg16_stream(ca + s * 512);
        p.kb[s] = ldg16_stream(cb + s * 512);
    }
#pragma unroll
    for (int s = 0; s < KS; s++) {
        p.va[s] = ldg16_stream(ca + 16 * D + s * 512);
        p.vb[s] = ldg16_stream(cb + 16 * D + s * 512);
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

// End of an item: the NT tiles of a wavefront go to the output (normalised) or, for an item that covers only part
// of its KV span, to partial slots it.partial + slot0 + nt.
// st.lsum holds each row's complete sum (the same value in the four lanes that share the row).
template <int D, int G, int NT>
__device__ __forceinline__ void store_tiles(const AttnArgs& a, const AttnItem& it, TileState<D, NT>& st, const int (&qi)[NT],
                                            const bool (&rvalid)[NT], int slot0, int lane) {
    constexpr int DT = D / 16;
    const int r = lane & 15, g = lane >> 4;
    const int head = it.kv_head * G + (r % G);
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        const float l = st.lsum[nt];
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
            const size_t slot = (size_t)it.partial + slot0 + nt;
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

// One single-tile work item on one wavefront: the next pair of pages is in flight in a second register
// set while the current pair is consumed (the wavefront is bandwidth-bound).
template <int D, int G>
__device__ __forceinline__ void attn_item(const AttnArgs& a, const AttnItem it) {
    constexpr int NT = 1;
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
            compute_pair<D, NT, true>(st, b0, qf, pq, (blk + 2 * i) * 16, true, g, scale2);
            __builtin_amdgcn_sched_barrier(0);
            load_pair<D>(b0, pool_lane, page_stride, pid(2 * i + 4), pid(2 * i + 5));
            __builtin_amdgcn_sched_barrier(0);
            compute_pair<D, NT, true>(st, b1, qf, pq, (blk + 2 * i + 2) * 16, true, g, scale2);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (i + 2 == n_pairs) {
            load_pair<D>(b1, pool_lane, page_stride, pid(2 * i + 2), pid(2 * i + 3));
            compute_pair<D, NT, true>(st, b0, qf, pq, (blk + 2 * i) * 16, true, g, scale2);
            compute_pair<D, NT, true>(st, b1, qf, pq, (blk + 2 * i + 2) * 16, 2 * i + 3 < n_pg, g, scale2);
        } else {
            compute_pair<D, NT, true>(st, b0, qf, pq, (blk + 2 * i) * 16, 2 * i + 1 < n_pg, g, scale2);
        }
    }
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {   // each lane summed its own keys: add up the four lanes of a row
        float l = st.lsum[nt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        st.lsum[nt] = l;
    }
    store_tiles<D, G, NT>(a, it, st, qi, rvalid, 0, lane);
}

// ---- teams: the query blocks of a prefill chunk ---------------------------------------------------
constexpr int TEAM_WAVES = 4;
constexpr int TEAM_NT = 3;     // query tiles per wavefront
constexpr int TEAM_RING = 3;   // pairs of pages in LDS: the one in use, and two on their way

__device__ __forceinline__ u32x2_t lds_read8(uint32_t addr, int off) {
    u32x2_t v;
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(off) : "memory");
    return v;
}
// maximum of three without the quieting of signalling NaNs that fmaxf brings along
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Softmax update of one query tile for a pair of pages: raw scores sa (page a, keys 4g..4g+3 of this lane's query row) and
// sb (page b) -> P as a packed B operand, reference maximum updated, alpha = the factor the accumulators take.  The row
// sums are not taken here: the matrix unit adds up the rounded P it multiplies V with (see team_pair), so that the
// output is a weighted mean of V rows whose weights sum to one exactly as rounded.
// mask: keys beyond the row's position are taken out by setting their scores to -inf (the running maximum starts at a
// large finite negative number, so a row that has seen no key yet keeps it and gets P = 0, alpha = 1).
__device__ __forceinline__ bf16x8_t team_softmax(bool mask, const f32x4_t& sa, const f32x4_t& sb, float& m, float& alpha,
                                                 int pq, int kpos_a, float scale2) {
    float sv[8] = {sa[0], sa[1], sa[2], sa[3], sb[0], sb[1], sb[2], sb[3]};
    if (mask) {   // uniform: only the pairs that reach past the wavefront's first query position
        const float ninf = -__builtin_inff();
#pragma unroll
        for (int i = 0; i < 4; i++) {
            sv[i] = kpos_a + i <= pq ? sv[i] : ninf;
            sv[4 + i] = kpos_a + 16 + i <= pq ? sv[4 + i] : ninf;
        }
    }
    float mx = max3(max3(sv[0], sv[1], sv[2]), max3(sv[3], sv[4], sv[5]), max3(sv[6], sv[7], sv[7]));
    {   // over the four lanes r, r+16, r+32, r+48 that share the row (see row_quad_max)
        const u32x2_t x = __builtin_amdgcn_permlane16_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        const float y = max3(__uint_as_float(x.x), __uint_as_float(x.y), mx);
        const u32x2_t z = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
        mx = max3(__uint_as_float(z.x), __uint_as_float(z.y), y);
    }
    // The reference is the exact running maximum, so a row's largest P is exactly 1 and carries no rounding error into
    // P.V.  (A reference that follows lazily, moving only after the maximum has grown by some factor, saves most of the
    // accumulator rescaling: measured 6 % faster on long prefixes, with 10 % more rounding error in the layer's output.)
    const float cand = mx * scale2;
    const float m_new = cand > m ? cand : m;
    alpha = __builtin_amdgcn_exp2f(m - m_new);
    m = m_new;
    float pv[8];
#pragma unroll
    for (int i = 0; i < 8; i++) pv[i] = __builtin_amdgcn_exp2f(fmaf(sv[i], scale2, -m_new));
    uint4 pw;
    pw.x = pack_bf16(pv[0], pv[1]);
    pw.y = pack_bf16(pv[2], pv[3]);
    pw.z = pack_bf16(pv[4], pv[5]);
    pw.w = pack_bf16(pv[6], pv[7]);
    return as_bf16x8(pw);
}

// One pair of pages from ring slot `addr` (LDS byte address of this lane's 16 bytes of the slot's first KiB) for the
// wavefront's NT tiles.  The slot holds the pair as 4 KS KiB blocks [k-step s][K page a, K page b, V page a, V page b];
// the V operand of a d-tile is the same 8-byte half of the two V blocks, read as such, so no register is moved.
template <int D, int NT>
__device__ __forceinline__ void team_pair(TileState<D, NT>& st, f32x4_t (&lacc)[NT], uint32_t addr, const bf16x8_t (&qf)[NT][D / 32],
                                          int pos_row, int tok_step, int pos_max, int kpos_a, float scale2, bool mask) {
    constexpr int KS = D / 32, DT = D / 16;
    u32x4_t kk[2 * KS];
#pragma unroll
    for (int s = 0; s < KS; s++) {
        kk[2 * s] = lds_read16(addr, (4 * s + 0) * 1024);
        kk[2 * s + 1] = lds_read16(addr, (4 * s + 1) * 1024);
    }
    if constexpr (KS == 4)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kk[0]), "+v"(kk[1]), "+v"(kk[2]), "+v"(kk[3]), "+v"(kk[4]), "+v"(kk[5]), "+v"(kk[6]), "+v"(kk[7]));
    else
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kk[0]), "+v"(kk[1]), "+v"(kk[2]), "+v"(kk[3]));
    u32x2_t va[DT], vb[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++) {
        va[dt] = lds_read8(addr, (4 * (dt >> 1) + 2) * 1024 + 8 * (dt & 1));
        vb[dt] = lds_read8(addr, (4 * (dt >> 1) + 3) * 1024 + 8 * (dt & 1));
    }
    f32x4_t sa[NT], sb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        sa[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        sb[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; s++) {
            sa[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kk[2 * s]), qf[nt][s], sa[nt], 0, 0, 0);
            sb[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kk[2 * s + 1]), qf[nt][s], sb[nt], 0, 0, 0);
        }
    }
    bf16x8_t pf[NT];
    float alpha[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) pf[nt] = team_softmax(mask, sa[nt], sb[nt], st.m[nt], alpha[nt], min(pos_row + nt * tok_step, pos_max), kpos_a, scale2);
    if constexpr (DT == 8)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(va[0]), "+v"(va[1]), "+v"(va[2]), "+v"(va[3]), "+v"(va[4]), "+v"(va[5]), "+v"(va[6]), "+v"(va[7]),
                     "+v"(vb[0]), "+v"(vb[1]), "+v"(vb[2]), "+v"(vb[3]), "+v"(vb[4]), "+v"(vb[5]), "+v"(vb[6]), "+v"(vb[7]));
    else
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(va[0]), "+v"(va[1]), "+v"(va[2]), "+v"(va[3]), "+v"(vb[0]), "+v"(vb[1]), "+v"(vb[2]), "+v"(vb[3]));
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        // once the running max has settled alpha is exactly 1 in every lane: skip the D/4 multiplies
        if (__builtin_amdgcn_ballot_w64(alpha[nt] != 1.0f) != 0) {
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
                st.o[nt][dt][0] *= alpha[nt]; st.o[nt][dt][1] *= alpha[nt]; st.o[nt][dt][2] *= alpha[nt]; st.o[nt][dt][3] *= alpha[nt];
            }
            lacc[nt][0] *= alpha[nt]; lacc[nt][1] *= alpha[nt]; lacc[nt][2] *= alpha[nt]; lacc[nt][3] *= alpha[nt];
        }
        // row sums of P: a tile of ones in V's place; every accumulator row then holds its column's (= query row's) sum
        const u32x4_t ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
        lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ones), pf[nt], lacc[nt], 0, 0, 0);
#pragma unroll
        for (int dt = 0; dt < DT; dt++) {
            const u32x4_t vw = {va[dt].x, va[dt].y, vb[dt].x, vb[dt].y};
            st.o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vw), pf[nt], st.o[nt][dt], 0, 0, 0);
        }
    }
}

// One work item on a team.  Wavefront w holds the tiles TEAM_NT w .. TEAM_NT w + TEAM_NT - 1 of the query block.
// Pair i of the item's page range sits in ring slot i % 3.  Wavefront w copies the KS KiB blocks w KS .. w KS + KS - 1
// of every pair.  Per pair: wait for the own copies of this pair (the copies of the next pair may still be in flight),
// barrier (now every wavefront's part of the pair has landed, and every wavefront has finished with the pair before, whose
// slot is the one to refill), issue the copies of pair i + 2, compute.  Past the item's last pair the copies fetch that
// last pair again, into slots nobody reads, so that the wait counts are the same in every trip.
template <int D, int G>
__device__ __forceinline__ void team_item(const AttnArgs& a, const AttnItem it, uint8_t* ring, int wave) {
    constexpr int NT = TEAM_NT;
    constexpr int KS = D / 32, DT = D / 16, TQ = 16 / G;
    constexpr int PAIR_BYTES = 4 * KS * 1024;
    const int lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int32_t* pages = a.pages + it.page_off;
    const int head = it.kv_head * G + (r % G);

    // Row (lane r) of tile nt of this wavefront is token (wave NT + nt) TQ + r / G of the block, clamped to the block's
    // last token (rows past it compute on that token's data and are not stored).  Only the queries stay in registers:
    // positions for the masks and token indices for the stores are formed again where they are needed.
    const int tok_row = wave * NT * TQ + r / G;
    bf16x8_t qf[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        const int qc = min(tok_row + nt * TQ, it.q_ntok - 1);
        const bf16_t* qrow = a.q + (size_t)(it.tok_g0 + qc) * a.ldq + head * D + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; s++) qf[nt][s] = as_bf16x8(ldg16(qrow + 32 * s));
    }
    // positions of the wavefront's first and last valid token: pairs that end at or before the first need no mask,
    // pairs that begin after the last are skipped
    const int wave_tok0 = wave * NT * TQ;
    const bool wave_has_rows = wave_tok0 < it.q_ntok;
    const int pos_first = it.pos0 + min(wave_tok0, it.q_ntok - 1);
    const int pos_last = it.pos0 + min(wave_tok0 + NT * TQ, it.q_ntok) - 1;

    TileState<D, NT> st;
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        st.m[nt] = NEG_BIG;
        st.lsum[nt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; dt++) st.o[nt][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    f32x4_t lacc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) lacc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const float scale2 = 1.4426950408889634f / sqrtf((float)D);
    const size_t page_stride = (size_t)a.n_kv * 2 * 16 * D;
    const bf16_t* pool_lane = a.pool_slot + (size_t)it.kv_head * 2 * 16 * D + (size_t)lane * 8;
    const uint32_t ring0 = (uint32_t)(uintptr_t)ring;

    const int n_pg = it.page_end - it.page_begin;
    const int n_pairs = (n_pg + 1) >> 1;
    // ids of 64 pages at a time, lane l holding page tb0 + l of the item's range; the copies run ahead of the
    // computation, so the table follows the copies
    int tb0 = 0;
    int tbl = pages[it.page_begin + min(lane, n_pg - 1)];
    auto issue = [&](int j, int slot) {
        const int jj = min(j, n_pairs - 1);
        if (2 * jj >= tb0 + 64) {
            tb0 += 64;
            tbl = pages[it.page_begin + tb0 + min(lane, n_pg - tb0 - 1)];
            vm_wait<0>();   // here, so that the compiler does not wait for everything where the paths join
        }
        const int la = 2 * jj - tb0;
        const int pa = __builtin_amdgcn_readlane(tbl, la);
        const int pb = __builtin_amdgcn_readlane(tbl, min(la + 1, n_pg - tb0 - 1));
        const bf16_t* ca = pool_lane + (size_t)pa * page_stride;
        const bf16_t* cb = pool_lane + (size_t)pb * page_stride;
        uint8_t* dst = ring + slot * PAIR_BYTES;
#pragma unroll
        for (int k = 0; k < KS; k++) {
            const int c = wave * KS + k;            // KiB block of the pair: [k-step c / 4][c % 4: Ka, Kb, Va, Vb]
            const bf16_t* src = ((c & 1) ? cb : ca) + ((c >> 1) & 1) * 16 * D + (c >> 2) * 512;
            PS_GLOBAL_TO_LDS(src, dst + c * 1024);
        }
    };

    __builtin_amdgcn_s_barrier();   // every wavefront has finished with the ring (previous item)
    issue(0, 0);
    issue(1, 1);
    // the wavefront computes on the first n_mine pairs (those that begin at or before its last query position) and only
    // keeps copying and meeting the barriers for the rest; two loops, so that no accumulator is live across a branch
    const int n_mine = !wave_has_rows || (pos_last >> 4) < it.page_begin ? 0 : min(n_pairs, ((pos_last >> 4) - it.page_begin) / 2 + 1);
    int slot = 0;
    for (int i = 0; i < n_mine; i++) {
        vm_wait<KS>();
        __builtin_amdgcn_s_barrier();
        issue(i + 2, slot >= 1 ? slot - 1 : TEAM_RING - 1);     // (i + 2) % 3
        const int kpos0 = (it.page_begin + 2 * i) * 16;
        team_pair<D, NT>(st, lacc, ring0 + slot * PAIR_BYTES + lane * 16, qf, it.pos0 + tok_row, TQ, it.pos0 + it.q_ntok - 1, kpos0 + 4 * g, scale2,
                         kpos0 + 31 > pos_first);
        slot = slot + 1 == TEAM_RING ? 0 : slot + 1;
    }
    for (int i = n_mine; i < n_pairs; i++) {
        vm_wait<KS>();
        __builtin_amdgcn_s_barrier();
        issue(i + 2, slot >= 1 ? slot - 1 : TEAM_RING - 1);
        slot = slot + 1 == TEAM_RING ? 0 : slot + 1;
    }
    vm_wait<0>();   // the surplus copies have landed before the ring is used again
    int qi[NT];
    bool rvalid[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        st.lsum[nt] = lacc[nt][0];
        rvalid[nt] = tok_row + nt * TQ < it.q_ntok;
        qi[nt] = it.tok_g0 + min(tok_row + nt * TQ, it.q_ntok - 1);
    }
    if (wave_has_rows) store_tiles<D, G, NT>(a, it, st, qi, rvalid, wave * NT, lane);
}

template <int D, int G>
__global__ __launch_bounds__(64 * TEAM_WAVES) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_kernel(AttnArgs a) {
    __shared__ __attribute__((aligned(1024))) uint8_t ring[TEAM_RING * (D / 8) * 1024];
    // Consecutive block ids go to different XCDs (one L2 each).  XCD x runs the contiguous teams
    // [x * team_per_xcd, (x+1) * team_per_xcd) and after them a contiguous share of the single-wavefront workers,
    // i.e. neighbouring parts of either work list share an L2, and every XCD has the same mix of the two kinds.
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (j < a.team_per_xcd) {
        const int t = xcd * a.team_per_xcd + j;
        if (t >= a.n_team) return;
        const int i0 = a.worker_begin[t], i1 = a.worker_begin[t + 1];
        for (int i = i0; i < i1; i++) team_item<D, G>(a, a.items[i], ring, wave);
    } else {
        const int w = a.n_team + (xcd * a.wave_blocks_per_xcd + (j - a.team_per_xcd)) * TEAM_WAVES + wave;
        if (j - a.team_per_xcd >= a.wave_blocks_per_xcd || w >= a.n_workers) return;
        const int i0 = a.worker_begin[w], i1 = a.worker_begin[w + 1];
        for (int i = i0; i < i1; i++) attn_item<D, G>(a, a.items[i]);
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

int attn_prefill_tokens_per_item(int G) { return TEAM_WAVES * TEAM_NT * (16 / G); }

template <int D, int G>
static hipError_t launch_dg(const AttnArgs& a_in, hipStream_t st) {
    AttnArgs a = a_in;
    a.team_per_xcd = (a.n_team + 7) >> 3;
    a.wave_blocks_per_xcd = ((a.n_workers - a.n_team + TEAM_WAVES - 1) / TEAM_WAVES + 7) >> 3;
    if (a.ev_begin) (void)hipEventRecord(a.ev_begin, st);
    hipLaunchKernelGGL((attn_kernel<D, G>), dim3((a.team_per_xcd + a.wave_blocks_per_xcd) * 8), dim3(64 * TEAM_WAVES), 0, st, a);
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
// wavefronts per SIMD, i.e. two blocks of four per CU).
int attention_worker_slots() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 2048;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 2048;
    return cus * 4 * 2;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
    if (a.n_items <= 0 || a.n_workers <= 0) return hipSuccess;
    if (a.n_team < 0 || a.n_team > a.n_workers) return hipErrorInvalidValue;
    if (a.d == 128) return launch_d<128>(a, st);
    if (a.d == 64) return launch_d<64>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace ps
