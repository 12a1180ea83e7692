// Paged-KV attention for a mixed batch in one launch (Sec. 2.1: Softmax(QK^T/sqrt(d))V over
// the keys and values of all previous tokens; Sec. 2.4: a prefill chunk against its cached
// prefix together with one-token decodes; Sec. 2.2: decode attention gets no batching
// benefit, its cost follows the KV bytes read).
//
// One wavefront per work item = (sequence, kv head, query block, KV page range).  A query
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

namespace ps {

constexpr float NEG_BIG = -1.0e30f;

template <int D, int G, int NT>
__device__ __forceinline__ void attn_item(const AttnArgs& a, const AttnItem it) {
    constexpr int KS = D / 32;   // MFMA k-steps over head_dim
    constexpr int DT = D / 16;   // 16-row tiles of O^T
    constexpr int TQ = 16 / G;   // tokens per query tile
    const int lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;

    const SeqInfo sq = a.seqs[it.seq];
    const int prefix = sq.kv_len - sq.n_new;
    const int32_t* pages = a.pages + sq.page_off;
    const int q_last = it.q_tok0 + it.q_ntok - 1;
    const int head = it.kv_head * G + (r % G);

    int qi[NT], pq[NT];
    bool rvalid[NT];
    bf16x8_t qf[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        const int q = it.q_tok0 + nt * TQ + r / G;
        rvalid[nt] = q <= q_last;
        qi[nt] = min(q, q_last);
        pq[nt] = prefix + qi[nt];
        const bf16_t* qrow = a.q + (size_t)(sq.tok0 + qi[nt]) * a.ldq + head * D + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; s++) qf[nt][s] = as_bf16x8(ldg16(qrow + 32 * s));
    }

    f32x4_t o[NT][DT];
    float m[NT], lsum[NT];
#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        m[nt] = NEG_BIG;
        lsum[nt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; dt++) o[nt][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    const float scale2 = 1.4426950408889634f / sqrtf((float)D);  // log2(e)/sqrt(d): softmax in base 2
    const size_t chunk = (size_t)16 * D;                         // elements per K or V chunk
    const size_t page_stride = (size_t)a.n_kv * 2 * chunk;
    const bf16_t* pool_h = a.pool_slot + (size_t)it.kv_head * 2 * chunk + (size_t)lane * 8;

    for (int pp = it.page_begin; pp < it.page_end; pp += 2) {
        const bool b_valid = pp + 1 < it.page_end;
        const int pa = pages[pp];
        const int pb = b_valid ? pages[pp + 1] : pa;
        const bf16_t* ca = pool_h + (size_t)pa * page_stride;
        const bf16_t* cb = pool_h + (size_t)pb * page_stride;
        uint4 ka[KS], kb[KS], va[KS], vb[KS];
#pragma unroll
        for (int s = 0; s < KS; s++) {
            ka[s] = ldg16(ca + s * 512);
            kb[s] = ldg16(cb + s * 512);
        }
#pragma unroll
        for (int s = 0; s < KS; s++) {
            va[s] = ldg16(ca + chunk + s * 512);
            vb[s] = ldg16(cb + chunk + s * 512);
        }
        const int kpos_a = pp * 16 + 4 * g, kpos_b = kpos_a + 16;

#pragma unroll
        for (int nt = 0; nt < NT; nt++) {
            f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; s++) {
                sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka[s]), qf[nt][s], sa, 0, 0, 0);
                sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kb[s]), qf[nt][s], sb, 0, 0, 0);
            }
            float sv[8];
            bool ok[8];
            float mx = NEG_BIG;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                ok[i] = kpos_a + i <= pq[nt];
                ok[4 + i] = b_valid && (kpos_b + i <= pq[nt]);
                sv[i] = sa[i] * scale2;
                sv[4 + i] = sb[i] * scale2;
            }
#pragma unroll
            for (int i = 0; i < 8; i++) mx = ok[i] ? fmaxf(mx, sv[i]) : mx;
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m[nt], mx);
            const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
            m[nt] = m_new;
            float pv[8], ps = 0.f;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                pv[i] = ok[i] ? __builtin_amdgcn_exp2f(sv[i] - m_new) : 0.f;
                ps += pv[i];
            }
            lsum[nt] = lsum[nt] * alpha + ps;
            uint4 pw;
            pw.x = pack_bf16(pv[0], pv[1]);
            pw.y = pack_bf16(pv[2], pv[3]);
            pw.z = pack_bf16(pv[4], pv[5]);
            pw.w = pack_bf16(pv[6], pv[7]);
            const bf16x8_t pf = as_bf16x8(pw);
#pragma unroll
            for (int dt = 0; dt < DT; dt++) {
                const int s = dt >> 1;
                uint4 vw;
                if (dt & 1) { vw.x = va[s].z; vw.y = va[s].w; vw.z = vb[s].z; vw.w = vb[s].w; }
                else        { vw.x = va[s].x; vw.y = va[s].y; vw.z = vb[s].x; vw.w = vb[s].y; }
                f32x4_t acc = o[nt][dt];
                acc[0] *= alpha; acc[1] *= alpha; acc[2] *= alpha; acc[3] *= alpha;
                o[nt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vw), pf, acc, 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int nt = 0; nt < NT; nt++) {
        float l = lsum[nt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (it.partial < 0) {
            if (rvalid[nt]) {
                const float inv = 1.0f / l;
                bf16_t* orow = a.out + (size_t)(sq.tok0 + qi[nt]) * (a.n_q * D) + head * D + 4 * g;
#pragma unroll
                for (int dt = 0; dt < DT; dt++) {
                    uint2 w;
                    w.x = pack_bf16(o[nt][dt][0] * inv, o[nt][dt][1] * inv);
                    w.y = pack_bf16(o[nt][dt][2] * inv, o[nt][dt][3] * inv);
                    *reinterpret_cast<uint2*>(orow + 16 * dt) = w;
                }
            }
        } else {
            const size_t slot = (size_t)it.partial + nt;
            float* po = a.part_o + (slot * 16 + r) * D + 4 * g;
#pragma unroll
            for (int dt = 0; dt < DT; dt++)
                *reinterpret_cast<float4*>(po + 16 * dt) = float4{o[nt][dt][0], o[nt][dt][1], o[nt][dt][2], o[nt][dt][3]};
            if (g == 0) {
                float* pm = a.part_ml + (slot * 16 + r) * 2;
                pm[0] = m[nt];
                pm[1] = l;
            }
        }
    }
}

constexpr int PREFILL_NT = 2;  // query tiles per wave for multi-tile (prefill) items

template <int D, int G>
__global__ __launch_bounds__(64) void attn_kernel(AttnArgs a) {
    const AttnItem it = a.items[blockIdx.x];
    constexpr int TQ = 16 / G;
    if (it.q_ntok <= TQ)
        attn_item<D, G, 1>(a, it);
    else
        attn_item<D, G, PREFILL_NT>(a, it);
}

// Combine split partials of one query tile: out = sum_j 2^(m_j - M) O_j / sum_j 2^(m_j - M) l_j.
// One 64-thread block per merge group; thread = (row r = tid%16, quarter of d = tid/16).
template <int D, int G>
__global__ __launch_bounds__(64) void attn_merge_kernel(AttnArgs a) {
    const MergeGroup mg = a.groups[blockIdx.x];
    const int r = threadIdx.x & 15, part = threadIdx.x >> 4;
    const int tok = r / G;
    if (tok >= mg.n_tok) return;
    const int head = mg.kv_head * G + r % G;
    float M = NEG_BIG;
    for (int j = 0; j < mg.n_splits; j++)
        M = fmaxf(M, a.part_ml[((size_t)(mg.first_slot + j * mg.stride) * 16 + r) * 2]);
    float acc[D / 4];
#pragma unroll
    for (int i = 0; i < D / 4; i++) acc[i] = 0.f;
    float L = 0.f;
    for (int j = 0; j < mg.n_splits; j++) {
        const size_t slot = (size_t)(mg.first_slot + j * mg.stride);
        const float w = __builtin_amdgcn_exp2f(a.part_ml[(slot * 16 + r) * 2] - M);
        L += w * a.part_ml[(slot * 16 + r) * 2 + 1];
        const float4* po = reinterpret_cast<const float4*>(a.part_o + (slot * 16 + r) * D + part * (D / 4));
#pragma unroll
        for (int i = 0; i < D / 16; i++) {
            const float4 v = po[i];
            acc[4 * i + 0] += w * v.x; acc[4 * i + 1] += w * v.y; acc[4 * i + 2] += w * v.z; acc[4 * i + 3] += w * v.w;
        }
    }
    const float inv = 1.0f / L;
    bf16_t* orow = a.out + (size_t)(mg.tok0 + tok) * (a.n_q * D) + head * D + part * (D / 4);
#pragma unroll
    for (int i = 0; i < D / 8; i++)
        *reinterpret_cast<uint32_t*>(orow + 2 * i) = pack_bf16(acc[2 * i] * inv, acc[2 * i + 1] * inv);
}

int attn_prefill_tokens_per_item(int G) { return PREFILL_NT * (16 / G); }

template <int D, int G>
static hipError_t launch_dg(const AttnArgs& a, hipStream_t st) {
    if (a.ev_begin) (void)hipEventRecord(a.ev_begin, st);
    hipLaunchKernelGGL((attn_kernel<D, G>), dim3(a.n_items), dim3(64), 0, st, a);
    hipError_t e = hipGetLastError();
    if (a.ev_end) (void)hipEventRecord(a.ev_end, st);
    if (e != hipSuccess || a.n_groups == 0) return e;
    hipLaunchKernelGGL((attn_merge_kernel<D, G>), dim3(a.n_groups), dim3(64), 0, st, a);
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

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.d == 128) return launch_d<128>(a, st);
    if (a.d == 64) return launch_d<64>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace ps
