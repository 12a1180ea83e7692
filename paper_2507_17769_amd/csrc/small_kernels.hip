// Bandwidth-trivial kernels of the step: RMSNorm, rotary embedding + KV append, the fused
// split-reduce + residual + RMSNorm, and logical KV read/write.  (Sec. 2.1: each module is preceded by an RMS
// normalisation; the prefill pass fills the KV cache that later decode steps extend.)
#include <algorithm>

#include "ps_device.h"

namespace ps {

// ---------------------------------------------------------------------------- RMSNorm
// One block per token row, one thread per 8 consecutive elements (H <= 8192): out = x * rsqrt(mean(x^2) + eps) * gain,
// fp32 math, the row held in registers between the sum and the scaling.
// sum over the block of one value per thread; red: one float per wavefront
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); w++) tot += red[w];
    return tot;
}

// The step's first kernel also brings the step's integer metadata over: blocks past the n_rows normalising ones copy
// it from the pinned host buffer the planner filled (mapped into the device's address space) to its device slot, 16
// bytes per thread and trip.  The kernels that read it come later in the stream; a copy engine transfer in its place
// sat between two steps for some 16 us (it only started once the previous step's last kernel had ended).
template <bool X_F32>
__global__ __launch_bounds__(1024) void rmsnorm_kernel(const void* __restrict__ xin, const bf16_t* __restrict__ gain,
                                                       bf16_t* __restrict__ out, int H, float eps,
                                                       const int32_t* __restrict__ src_rows, int n_rows,
                                                       const uint4* __restrict__ meta_src, uint4* __restrict__ meta_dst, uint32_t meta_n16) {
    if ((int)blockIdx.x >= n_rows) {
        const uint32_t stride = (gridDim.x - n_rows) * blockDim.x;
        for (uint32_t i = (blockIdx.x - n_rows) * blockDim.x + threadIdx.x; i < meta_n16; i += stride) meta_dst[i] = meta_src[i];
        return;
    }
    const int orow = blockIdx.x;                            // output row
    const int row = src_rows ? src_rows[orow] : orow;       // input row (the head normalises selected rows only)
    const int c = threadIdx.x * 8;
    __shared__ float red[16];
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    uint4 gw = uint4{0u, 0u, 0u, 0u};
    if (c < H) {
        if (X_F32) {
            const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(xin) + (size_t)row * H + c);
            float4 a = p[0], b = p[1];
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        } else {
            uint4 w = ldg16(static_cast<const bf16_t*>(xin) + (size_t)row * H + c);
            v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x); v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
            v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z); v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
        }
        gw = ldg16(gain + c);
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) ss += v[i] * v[i];
    const float r = 1.0f / sqrtf(block_sum(ss, red) / (float)H + eps);
    if (c < H) {
        float g[8] = {bf16_lo(gw.x), bf16_hi(gw.x), bf16_lo(gw.y), bf16_hi(gw.y),
                      bf16_lo(gw.z), bf16_hi(gw.z), bf16_lo(gw.w), bf16_hi(gw.w)};
        uint4 o;
        o.x = pack_bf16(v[0] * r * g[0], v[1] * r * g[1]);
        o.y = pack_bf16(v[2] * r * g[2], v[3] * r * g[3]);
        o.z = pack_bf16(v[4] * r * g[4], v[5] * r * g[5]);
        o.w = pack_bf16(v[6] * r * g[6], v[7] * r * g[7]);
        *reinterpret_cast<uint4*>(out + act_offset(orow, c, H)) = o;
    }
}

hipError_t launch_rmsnorm(const void* x, bool x_is_f32, const bf16_t* gain, bf16_t* out, int T, int H, float eps,
                          hipStream_t st, const int32_t* src_rows, const void* meta_src, void* meta_dst, size_t meta_bytes) {
    if (T <= 0) return hipSuccess;
    if (H > 8192 || H % 8 || (meta_bytes & 15) || meta_bytes >= ((size_t)1 << 32)) return hipErrorInvalidValue;
    const int nt = ((H / 8 + 63) / 64) * 64;
    const uint32_t n16 = (uint32_t)(meta_bytes / 16);
    // enough copying blocks to have the whole buffer in flight at once (the reads cross the host link), 64 at most
    const int nc = n16 ? (int)std::min<uint32_t>(64, (n16 + nt - 1) / nt) : 0;
    const uint4* ms = static_cast<const uint4*>(meta_src);
    uint4* md = static_cast<uint4*>(meta_dst);
    if (x_is_f32)
        hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3(T + nc), dim3(nt), 0, st, x, gain, out, H, eps, src_rows, T, ms, md, n16);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(T + nc), dim3(nt), 0, st, x, gain, out, H, eps, src_rows, T, ms, md, n16);
    return hipGetLastError();
}

// --------------------------------------------------------------- embedding rows, greedy token
// (Sec. 2.1: tokens enter the layers as embedding vectors; every step ends by generating a token.)
// One 256-thread block per token: out[t][:] = table[ids[t]][:], 16 bytes per thread and trip.
__global__ __launch_bounds__(256) void embed_gather_kernel(const bf16_t* __restrict__ table, const int32_t* __restrict__ ids,
                                                           bf16_t* __restrict__ out, int H) {
    const uint4* src = reinterpret_cast<const uint4*>(table + (size_t)ids[blockIdx.x] * H);
    uint4* dst = reinterpret_cast<uint4*>(out + (size_t)blockIdx.x * H);
    for (int c = threadIdx.x; c < H / 8; c += 256) dst[c] = src[c];
}

hipError_t launch_embed_gather(const bf16_t* table, const int32_t* ids, bf16_t* out, int T, int H, hipStream_t st) {
    if (T <= 0) return hipSuccess;
    hipLaunchKernelGGL(embed_gather_kernel, dim3(T), dim3(256), 0, st, table, ids, out, H);
    return hipGetLastError();
}

// One 1024-thread block per row: index of the row's largest value, the lowest index among equal ones.
// A NaN never wins a comparison, so a row of NaNs yields 0.
__global__ __launch_bounds__(1024) void argmax_rows_kernel(const float* __restrict__ x, int N, int32_t* __restrict__ out) {
    const float* row = x + (size_t)blockIdx.x * N;
    float best = -INFINITY;
    int arg = 0x7fffffff;
    for (int c = threadIdx.x * 4; c < N; c += 4096) {   // N is a multiple of 4
        const float4 v = *reinterpret_cast<const float4*>(row + c);
        if (v.x > best) { best = v.x; arg = c; }
        if (v.y > best) { best = v.y; arg = c + 1; }
        if (v.z > best) { best = v.z; arg = c + 2; }
        if (v.w > best) { best = v.w; arg = c + 3; }
    }
    // (value, index) maximum with ties to the lower index: first inside the wavefront, then across the 16 wavefronts
    auto better = [](float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); };
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(arg, o, 64);
        if (better(ov, oi, best, arg)) { best = ov; arg = oi; }
    }
    __shared__ float sv[16];
    __shared__ int si[16];
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = arg; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; w++)
            if (better(sv[w], si[w], best, arg)) { best = sv[w]; arg = si[w]; }
        out[blockIdx.x] = arg == 0x7fffffff ? 0 : arg;
    }
}

hipError_t launch_argmax_rows(const float* x, int M, int N, int32_t* out, hipStream_t st) {
    if (M <= 0) return hipSuccess;
    if (N % 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(argmax_rows_kernel, dim3(M), dim3(1024), 0, st, x, N, out);
    return hipGetLastError();
}

// --------------------------------------------------------------- rotary + KV append
// grid (T, ceil((n_q + 2 n_kv) / heads per block)), 256 threads.  A head takes d/8 threads; a thread owns the four
// rotation pairs (j, j + d/2), j = 4 * (its index in the head) .. + 3, and moves them as 16-byte pieces.
// Input is the fp32 QKV projection as n_splits partial sums [n_splits][T][(n_q + 2 n_kv) d],
// added up here; every value is rounded to bf16 exactly once, after the rotation: query heads
// go to q_out [T][n_q][d], key heads (rotated) and value heads to their cache slot.  cs is the
// fp64-built table [position][d/2] of (cos, sin).
__global__ __launch_bounds__(256) void rope_append_kernel(const float* __restrict__ qkv, int n_splits, size_t split_stride,
                                                          bf16_t* __restrict__ q_out, int n_q, int n_kv, int d,
                                                          const int32_t* __restrict__ positions,
                                                          const int32_t* __restrict__ slots,
                                                          const float2* __restrict__ cs, bf16_t* __restrict__ pool) {
    const int t = blockIdx.x;
    const int tph = d >> 3;                       // threads per head
    const int hh = blockIdx.y * (256 / tph) + threadIdx.x / tph;
    if (hh >= n_q + 2 * n_kv) return;
    const int j = 4 * (threadIdx.x % tph);
    const int half = d >> 1;
    const int ld = (n_q + 2 * n_kv) * d;
    const float* row = qkv + (size_t)t * ld + (size_t)hh * d;
    // all split loads are issued before the first add (n_splits <= 8)
    float4 plo[8], phi[8];
#pragma unroll
    for (int s = 0; s < 8; s++)
        if (s < n_splits) {
            plo[s] = *reinterpret_cast<const float4*>(row + s * split_stride + j);
            phi[s] = *reinterpret_cast<const float4*>(row + s * split_stride + j + half);
        }
    float lo[4] = {0.f, 0.f, 0.f, 0.f}, hi[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 8; s++)
        if (s < n_splits) {
            lo[0] += plo[s].x; lo[1] += plo[s].y; lo[2] += plo[s].z; lo[3] += plo[s].w;
            hi[0] += phi[s].x; hi[1] += phi[s].y; hi[2] += phi[s].z; hi[3] += phi[s].w;
        }
    bf16_t blo[4], bhi[4];
    if (hh < n_q + n_kv) {
        const float4* cp = reinterpret_cast<const float4*>(cs + (size_t)positions[t] * half + j);
        const float4 c01 = cp[0], c23 = cp[1];    // (cos, sin) of pairs j, j+1 and j+2, j+3
        const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
            blo[e] = f32_to_bf16(lo[e] * co[e] - hi[e] * si[e]);
            bhi[e] = f32_to_bf16(hi[e] * co[e] + lo[e] * si[e]);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            blo[e] = f32_to_bf16(lo[e]);
            bhi[e] = f32_to_bf16(hi[e]);
        }
    }
    const uint2 plo4 = uint2{(uint32_t)blo[0] | ((uint32_t)blo[1] << 16), (uint32_t)blo[2] | ((uint32_t)blo[3] << 16)};
    const uint2 phi4 = uint2{(uint32_t)bhi[0] | ((uint32_t)bhi[1] << 16), (uint32_t)bhi[2] | ((uint32_t)bhi[3] << 16)};
    if (hh < n_q) {
        bf16_t* qr = q_out + ((size_t)t * n_q + hh) * d;
        *reinterpret_cast<uint2*>(qr + j) = plo4;
        *reinterpret_cast<uint2*>(qr + j + half) = phi4;
    } else if (hh < n_q + n_kv) {
        const int h = hh - n_q;
        const int slot = slots[t];
        bf16_t* kc = pool + (((size_t)(slot >> 4) * n_kv + h) * 2 + 0) * (size_t)(16 * d);
        // j is a multiple of 4: the four elements sit in one 8-element group of the key chunk
        *reinterpret_cast<uint2*>(kc + k_elem_offset(slot & 15, j)) = plo4;
        *reinterpret_cast<uint2*>(kc + k_elem_offset(slot & 15, j + half)) = phi4;
    } else {
        const int h = hh - n_q - n_kv;
        const int slot = slots[t];
        bf16_t* vc = pool + (((size_t)(slot >> 4) * n_kv + h) * 2 + 1) * (size_t)(16 * d);
#pragma unroll
        for (int e = 0; e < 4; e++) {
            vc[v_elem_offset(slot & 15, j + e)] = blo[e];
            vc[v_elem_offset(slot & 15, j + half + e)] = bhi[e];
        }
    }
}

hipError_t launch_rope_append(const float* qkv, int n_splits, bf16_t* q_out, int T, int n_q, int n_kv, int d,
                              const int32_t* positions, const int32_t* slots, const float* rope_cs, bf16_t* pool_slot,
                              hipStream_t st) {
    if (T <= 0) return hipSuccess;
    if (n_splits > 8 || d % 8 || d > 2048) return hipErrorInvalidValue;
    const size_t split_stride = (size_t)T * (n_q + 2 * n_kv) * d;
    const int heads_per_block = 256 / (d / 8);
    hipLaunchKernelGGL(rope_append_kernel, dim3(T, (n_q + 2 * n_kv + heads_per_block - 1) / heads_per_block), dim3(256), 0, st, qkv,
                       n_splits, split_stride, q_out, n_q, n_kv, d,
                       positions, slots, reinterpret_cast<const float2*>(rope_cs), pool_slot);
    return hipGetLastError();
}

// ------------------------------------------------------- logical KV write / read
// k, v are [n][n_kv][d] in logical order; slots[i] = page * 16 + position in the page of token i, the tokens being
// consecutive positions starting at a position whose remainder mod 4 is `phase`.  One thread per (group of four
// positions aligned to 4, kv head, 8 consecutive dd): in the cache a key keeps 8 consecutive dd of one token together
// (16 bytes) and a value keeps the four tokens of such a group together for one dd (8 bytes), so the thread moves
// whole 16-byte rows on the logical side and 16- or 8-byte pieces on the cache side, transposing the 4 x 8 value
// tile in registers.  Tokens of a group outside [0, n) are left alone (the first and last group may be partial).
template <bool TO_POOL>
__global__ __launch_bounds__(256) void kv_copy_kernel(bf16_t* __restrict__ pool, const int32_t* __restrict__ slots, int n,
                                                      int phase, int n_kv, int d, bf16_t* __restrict__ k, bf16_t* __restrict__ v) {
    const int gpd = d >> 3;  // 8-element groups per head
    const int n_quads = (phase + n + 3) >> 2;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= (long long)n_quads * n_kv * gpd) return;
    const int g = (int)(id % gpd), h = (int)((id / gpd) % n_kv), qi = (int)(id / ((long long)gpd * n_kv));
    const int dd0 = g * 8;
    const int i0 = 4 * qi - phase;                    // token index of the group's first position
    const int t_lo = max(0, -i0), t_hi = min(4, n - i0);   // valid positions of the group: t_lo <= t < t_hi
    const int slot = slots[i0 + t_lo] - t_lo;         // slot of the group's first position (same page: groups are aligned)
    bf16_t* kc = pool + (((size_t)(slot >> 4) * n_kv + h) * 2 + 0) * (size_t)(16 * d);
    bf16_t* vc = kc + 16 * d;
    const int tok0 = slot & 15;                       // a multiple of 4
    for (int t = t_lo; t < t_hi; t++) {
        uint4* kr = reinterpret_cast<uint4*>(k + ((size_t)(i0 + t) * n_kv + h) * d + dd0);
        uint4* kp = reinterpret_cast<uint4*>(kc + k_elem_offset(tok0 + t, dd0));
        if (TO_POOL) *kp = *kr;
        else *kr = *kp;
    }
    if (t_lo == 0 && t_hi == 4) {
        uint16_t tile[4][8];
        if (TO_POOL) {
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const uint4 r = *reinterpret_cast<const uint4*>(v + ((size_t)(i0 + t) * n_kv + h) * d + dd0);
                const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                for (int e = 0; e < 8; e++) tile[t][e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
#pragma unroll
            for (int e = 0; e < 8; e++)
                *reinterpret_cast<uint2*>(vc + v_elem_offset(tok0, dd0 + e)) =
                    uint2{(uint32_t)tile[0][e] | ((uint32_t)tile[1][e] << 16), (uint32_t)tile[2][e] | ((uint32_t)tile[3][e] << 16)};
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint2 r = *reinterpret_cast<const uint2*>(vc + v_elem_offset(tok0, dd0 + e));
                tile[0][e] = (uint16_t)r.x; tile[1][e] = (uint16_t)(r.x >> 16);
                tile[2][e] = (uint16_t)r.y; tile[3][e] = (uint16_t)(r.y >> 16);
            }
#pragma unroll
            for (int t = 0; t < 4; t++) {
                uint4 o;
                o.x = (uint32_t)tile[t][0] | ((uint32_t)tile[t][1] << 16);
                o.y = (uint32_t)tile[t][2] | ((uint32_t)tile[t][3] << 16);
                o.z = (uint32_t)tile[t][4] | ((uint32_t)tile[t][5] << 16);
                o.w = (uint32_t)tile[t][6] | ((uint32_t)tile[t][7] << 16);
                *reinterpret_cast<uint4*>(v + ((size_t)(i0 + t) * n_kv + h) * d + dd0) = o;
            }
        }
    } else {
        for (int t = t_lo; t < t_hi; t++)
            for (int e = 0; e < 8; e++) {
                bf16_t* vr = v + ((size_t)(i0 + t) * n_kv + h) * d + dd0 + e;
                bf16_t* vp = vc + v_elem_offset(tok0 + t, dd0 + e);
                if (TO_POOL) *vp = *vr;
                else *vr = *vp;
            }
    }
}

hipError_t launch_kv_copy(bool to_pool, bf16_t* pool_slot, const int32_t* slots_dev, int n, int phase, int n_kv, int d, bf16_t* k,
                          bf16_t* v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (d % 8 || phase < 0 || phase > 3) return hipErrorInvalidValue;
    const long long threads = (long long)((phase + n + 3) >> 2) * n_kv * (d >> 3);
    const int blocks = (int)((threads + 255) / 256);
    if (to_pool)
        hipLaunchKernelGGL(kv_copy_kernel<true>, dim3(blocks), dim3(256), 0, st, pool_slot, slots_dev, n, phase, n_kv, d, k, v);
    else
        hipLaunchKernelGGL(kv_copy_kernel<false>, dim3(blocks), dim3(256), 0, st, pool_slot, slots_dev, n, phase, n_kv, d, k, v);
    return hipGetLastError();
}

// ------------------------------------------------- split reduce + residual + RMSNorm
// One block per token row, one thread per 8 consecutive elements (H <= 8192).  x = resid + sum_s partials[s];
// optionally stored as fp32 and/or bf16; optionally followed by RMSNorm (x * rsqrt(mean(x^2) + eps) * gain) stored
// as bf16.  The row stays in registers between the two phases.
template <bool RESID_F32>
__global__ __launch_bounds__(1024) void reduce_add_norm_kernel(ReduceAddNormArgs a) {
    const int row = blockIdx.x;
    const int H = a.H, c = threadIdx.x * 8;
    const size_t split_stride = (size_t)a.T * H;
    __shared__ float red[16];
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    uint4 gw = uint4{0u, 0u, 0u, 0u};
    if (c < H) {
        // all loads are issued before the first add (n_splits <= 8)
        float4 q0[8], q1[8];
#pragma unroll
        for (int s = 0; s < 8; s++)
            if (s < a.n_splits) {
                const float4* p = reinterpret_cast<const float4*>(a.partials + s * split_stride + (size_t)row * H + c);
                q0[s] = p[0];
                q1[s] = p[1];
            }
        if (a.gain) gw = ldg16(a.gain + c);
        if (RESID_F32) {
            const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(a.resid) + (size_t)row * H + c);
            const float4 x0 = p[0], x1 = p[1];
            v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w;
            v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
        } else {
            const uint4 w = ldg16(static_cast<const bf16_t*>(a.resid) + (size_t)row * H + c);
            v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x); v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
            v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z); v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
        }
#pragma unroll
        for (int s = 0; s < 8; s++)
            if (s < a.n_splits) {
                v[0] += q0[s].x; v[1] += q0[s].y; v[2] += q0[s].z; v[3] += q0[s].w;
                v[4] += q1[s].x; v[5] += q1[s].y; v[6] += q1[s].z; v[7] += q1[s].w;
            }
        if (a.x_f32) {
            float4* o = reinterpret_cast<float4*>(a.x_f32 + (size_t)row * H + c);
            o[0] = float4{v[0], v[1], v[2], v[3]};
            o[1] = float4{v[4], v[5], v[6], v[7]};
        }
        if (a.x_bf16) {
            uint4 o;
            o.x = pack_bf16(v[0], v[1]); o.y = pack_bf16(v[2], v[3]);
            o.z = pack_bf16(v[4], v[5]); o.w = pack_bf16(v[6], v[7]);
            *reinterpret_cast<uint4*>(a.x_bf16 + (size_t)row * H + c) = o;
        }
    }
    if (!a.gain) return;
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) ss += v[i] * v[i];
    const float r = 1.0f / sqrtf(block_sum(ss, red) / (float)H + a.eps);
    if (c < H) {
        uint4 o;
        o.x = pack_bf16(v[0] * r * bf16_lo(gw.x), v[1] * r * bf16_hi(gw.x));
        o.y = pack_bf16(v[2] * r * bf16_lo(gw.y), v[3] * r * bf16_hi(gw.y));
        o.z = pack_bf16(v[4] * r * bf16_lo(gw.z), v[5] * r * bf16_hi(gw.z));
        o.w = pack_bf16(v[6] * r * bf16_lo(gw.w), v[7] * r * bf16_hi(gw.w));
        *reinterpret_cast<uint4*>(a.xn + act_offset(row, c, H)) = o;
    }
}

hipError_t launch_reduce_add_norm(const ReduceAddNormArgs& a, hipStream_t st) {
    if (a.T <= 0) return hipSuccess;
    if (a.H > 8192 || a.H % 8 || a.n_splits > 8) return hipErrorInvalidValue;
    const int nt = ((a.H / 8 + 63) / 64) * 64;
    if (a.resid_f32)
        hipLaunchKernelGGL(reduce_add_norm_kernel<true>, dim3(a.T), dim3(nt), 0, st, a);
    else
        hipLaunchKernelGGL(reduce_add_norm_kernel<false>, dim3(a.T), dim3(nt), 0, st, a);
    return hipGetLastError();
}

// Device-to-device copy of n bytes (n a multiple of 16, both pointers 16-byte aligned).
__global__ __launch_bounds__(256) void copy_bytes_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// operand order -> row-major, 16 bytes (8 elements of one row) per thread
__global__ __launch_bounds__(256) void untile_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int M, int K) {
    const size_t total = (size_t)M * (K / 8);
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int m = (int)(i / (K / 8)), k = (int)(i % (K / 8)) * 8;
        *reinterpret_cast<uint4*>(dst + (size_t)m * K + k) = *reinterpret_cast<const uint4*>(src + act_offset(m, k, K));
    }
}

hipError_t launch_untile(const bf16_t* src, bf16_t* dst, int M, int K, hipStream_t st) {
    const size_t total = (size_t)M * (K / 8);
    if (total == 0) return hipSuccess;
    const int blocks = (int)std::min<size_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(untile_kernel, dim3(blocks), dim3(256), 0, st, src, dst, M, K);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Clock-under-load probe.  Every wavefront issues `rounds` x 4 independent 32x32x16 bf16 MFMAs on
// operands made from a hash of its lane (finite, mixed signs and exponents) and reports how many
// shader-clock ticks and how many ticks of the constant-rate wall clock that took.  No memory
// traffic inside the loop: the rate is what the matrix pipes sustain at the clock the power
// management settles on, which is the ceiling the GEMM kernels can be priced against.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_clock_probe_kernel(int rounds, float* __restrict__ sink, long long* __restrict__ ticks) {
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u;
    uint32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        h = h * 1664525u + 1013904223u;
        // two bf16 values with exponents 2^-2 .. 2^1, random mantissa and sign
        const uint32_t lo = 0x3e80u + ((h >> 8) & 0x1ffu) + ((h & 1u) << 15), hi = 0x3e80u + ((h >> 20) & 0x1ffu) + ((h & 2u) << 14);
        w[i] = lo | (hi << 16);
    }
    const u32x4_t av = {w[0], w[1], w[2], w[3]}, bv = {w[4], w[5], w[6], w[7]};
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, av), b = __builtin_bit_cast(bf16x8_t, bv);
    f32x16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < rounds; i++) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    const long long t1 = clock64(), w1 = wall_clock64();
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 16; e++) acc += c0[e] + c1[e] + c2[e] + c3[e];
    sink[blockIdx.x * 256 + threadIdx.x] = acc;  // keeps the loop alive
    if (threadIdx.x == 0) {
        ticks[2 * blockIdx.x] = t1 - t0;
        ticks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

hipError_t launch_mfma_clock_probe(int blocks, int rounds, float* sink, long long* ticks, hipStream_t st) {
    hipLaunchKernelGGL(mfma_clock_probe_kernel, dim3(blocks), dim3(256), 0, st, rounds, sink, ticks);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Streaming-read probe: every wavefront reads whole 16 KiB chunks (8 loads of 16 B per lane in
// flight), chunk c going to wavefront c mod n_wavefronts; nothing is written unless the xor of
// everything read hits one particular value.  The rate over a buffer several times the
// last-level cache is what plain loads get out of HBM, the ceiling for the KV stream of decode
// attention.  n_chunks * 16 KiB must not exceed the buffer; out holds one word per wavefront.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_probe_kernel(const uint4* __restrict__ buf, long long n_chunks, uint32_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const long long wave = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6, n_waves = ((long long)gridDim.x * 256) >> 6;
    uint32_t acc = 0;
    for (long long c = wave; c < n_chunks; c += n_waves) {
        const uint4* p = buf + c * 1024 + lane;
#pragma unroll
        for (int j = 0; j < 16; j += 8) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) v[u] = p[(j + u) * 64];
#pragma unroll
            for (int u = 0; u < 8; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
    }
    if (acc == 0x12345678u) out[wave] = acc;
}

hipError_t launch_stream_read_probe(const void* buf, size_t bytes, int blocks, uint32_t* out, hipStream_t st) {
    hipLaunchKernelGGL(stream_read_probe_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const uint4*>(buf), (long long)(bytes >> 14), out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_words_kernel(uint4* __restrict__ p, size_t n16, uint32_t word) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = uint4{word, word, word, word};
}

hipError_t launch_fill_words(void* p, size_t bytes, uint32_t word, hipStream_t st) {
    const size_t n16 = bytes / 16;
    if (n16 == 0 || !p) return hipSuccess;
    const int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_words_kernel, dim3(blocks), dim3(256), 0, st, static_cast<uint4*>(p), n16, word);
    return hipGetLastError();
}
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) { return launch_fill_words(p, bytes, 0u, st); }

hipError_t launch_copy_bytes(const void* src, void* dst, size_t n, hipStream_t st) {
    const size_t n16 = n / 16;
    if (n16 == 0) return hipSuccess;
    const int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
    hipLaunchKernelGGL(copy_bytes_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), n16);
    return hipGetLastError();
}

}  // namespace ps
