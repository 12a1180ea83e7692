// Weight GEMMs of the layer (Sec. 2.1: query/key/value generation, O-projection, gate/up and
// down projections; Sec. 2.2: the only operations with a batching effect).
//
//   C[M][N] = A[M][K] * W[K][N],  A = activations (bf16, K contiguous),
//   Bt = W^T [N][K] (bf16, K contiguous; repacked once at layer init), fp32 accumulate.
//
// bf16 MFMA 32x32x16 tiles, operands staged through LDS in BK = 64 slices with a
// register-held prefetch of the next slice.  256 threads = 4 wavefronts per block.
// Epilogues: plain store; residual add (residual and output each bf16 or fp32); SwiGLU on
// interleaved gate/up columns (bf16 out).  Optional split-K writes fp32 partials and a
// small reduce kernel applies the epilogue.
#include "ps_device.h"

namespace ps {

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // +16 bytes per row: conflict-free 16-byte reads across 16 rows

struct GemmParams {
    const bf16_t* A;
    const bf16_t* Bt;
    int M, N, K;
    int kind;
    int resid_f32, out_f32;
    const void* resid;
    void* out;
    float* ws;       // split-K partials [split][M][N], or null
    int kb_per_split;  // BK-blocks per split
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// Apply the epilogue to one element pair location.  For SWIGLU, (g, u) are the gate and up
// pre-activations of feature f and the output row stride is N/2.
__device__ __forceinline__ void store_plain(const GemmParams& p, int m, int n, float v) {
    const size_t idx = (size_t)m * p.N + n;
    if (p.kind == GemmEpilogue::RESID)
        v += p.resid_f32 ? static_cast<const float*>(p.resid)[idx] : bf16_to_f32(static_cast<const bf16_t*>(p.resid)[idx]);
    if (p.out_f32)
        static_cast<float*>(p.out)[idx] = v;
    else
        static_cast<bf16_t*>(p.out)[idx] = f32_to_bf16(v);
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_kernel(GemmParams p) {
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wave
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "4 waves");
    constexpr int A_CHUNKS = BM * (BK / 8) / 256;  // 16-byte chunks per thread
    constexpr int B_CHUNKS = BN * (BK / 8) / 256;
    static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small");

    __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LDS_STRIDE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kb_total = p.K / BK;
    const int kb_begin = blockIdx.z * p.kb_per_split;
    const int kb_end = min(kb_total, kb_begin + p.kb_per_split);

    // global -> register staging assignments
    const bf16_t* a_src[A_CHUNKS];
    const bf16_t* b_src[B_CHUNKS];
    int a_dst[A_CHUNKS], b_dst[B_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; i++) {
        const int c = tid + 256 * i, r = c >> 3, kc = c & 7;
        const int gm = min(m0 + r, p.M - 1);
        a_src[i] = p.A + (size_t)gm * p.K + kc * 8;
        a_dst[i] = r * LDS_STRIDE + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; i++) {
        const int c = tid + 256 * i, r = c >> 3, kc = c & 7;
        const int gn = min(n0 + r, p.N - 1);
        b_src[i] = p.Bt + (size_t)gn * p.K + kc * 8;
        b_dst[i] = r * LDS_STRIDE + kc * 8;
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    uint4 ra[A_CHUNKS], rb[B_CHUNKS];
    if (kb_begin < kb_end) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; i++) ra[i] = ldg16(a_src[i] + (size_t)kb_begin * BK);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; i++) rb[i] = ldg16(b_src[i] + (size_t)kb_begin * BK);
    }

    const int a_rd = (wm * WTM + (lane & 31)) * LDS_STRIDE + (lane >> 5) * 8;
    const int b_rd = (wn * WTN + (lane & 31)) * LDS_STRIDE + (lane >> 5) * 8;

    for (int kb = kb_begin; kb < kb_end; kb++) {
        __syncthreads();  // previous slice fully consumed
#pragma unroll
        for (int i = 0; i < A_CHUNKS; i++) *reinterpret_cast<uint4*>(&sA[a_dst[i]]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_CHUNKS; i++) *reinterpret_cast<uint4*>(&sB[b_dst[i]]) = rb[i];
        __syncthreads();
        if (kb + 1 < kb_end) {
#pragma unroll
            for (int i = 0; i < A_CHUNKS; i++) ra[i] = ldg16(a_src[i] + (size_t)(kb + 1) * BK);
#pragma unroll
            for (int i = 0; i < B_CHUNKS; i++) rb[i] = ldg16(b_src[i] + (size_t)(kb + 1) * BK);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++) {
            bf16x8_t af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; i++)
                af[i] = as_bf16x8(*reinterpret_cast<const uint4*>(&sA[a_rd + i * 32 * LDS_STRIDE + ks * 16]));
#pragma unroll
            for (int j = 0; j < TN; j++)
                bfr[j] = as_bf16x8(*reinterpret_cast<const uint4*>(&sB[b_rd + j * 32 * LDS_STRIDE + ks * 16]));
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int j = 0; j < TN; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    }

    // epilogue: lane holds column n = lane%32, rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32 tile
    const int col = lane & 31, rbase = (lane >> 5) * 4;
    if (p.ws) {
        float* ws = p.ws + (size_t)blockIdx.z * p.M * p.N;
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const int m = m0 + wm * WTM + i * 32 + (e >> 2) * 8 + rbase + (e & 3);
                    const int n = n0 + wn * WTN + j * 32 + col;
                    if (m < p.M && n < p.N) ws[(size_t)m * p.N + n] = acc[i][j][e];
                }
        return;
    }
    if (p.kind == GemmEpilogue::SWIGLU_BF16) {
        if constexpr (TN % 2 == 0) {
            bf16_t* out = static_cast<bf16_t*>(p.out);
            const int F = p.N >> 1;
#pragma unroll
            for (int i = 0; i < TM; i++)
#pragma unroll
                for (int j = 0; j < TN; j += 2)
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        const int m = m0 + wm * WTM + i * 32 + (e >> 2) * 8 + rbase + (e & 3);
                        const int nb = n0 + wn * WTN + j * 32;  // multiple of 64: gate tile, then up tile
                        const int f = (nb >> 1) + col;
                        if (m < p.M && nb < p.N) out[(size_t)m * F + f] = f32_to_bf16(silu_f(acc[i][j][e]) * acc[i][j + 1][e]);
                    }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int m = m0 + wm * WTM + i * 32 + (e >> 2) * 8 + rbase + (e & 3);
                const int n = n0 + wn * WTN + j * 32 + col;
                if (m < p.M && n < p.N) store_plain(p, m, n, acc[i][j][e]);
            }
}

// Sum split-K partials and apply the epilogue.  One thread per output element
// (per feature pair for SwiGLU).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmParams p, int n_split) {
    const size_t MN = (size_t)p.M * p.N;
    if (p.kind == GemmEpilogue::SWIGLU_BF16) {
        const int F = p.N >> 1;
        const size_t total = (size_t)p.M * F;
        for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
            const int m = (int)(i / F), f = (int)(i % F);
            const int ng = (f >> 5) * 64 + (f & 31);
            float g = 0.f, u = 0.f;
            for (int s = 0; s < n_split; s++) {
                g += p.ws[s * MN + (size_t)m * p.N + ng];
                u += p.ws[s * MN + (size_t)m * p.N + ng + 32];
            }
            static_cast<bf16_t*>(p.out)[i] = f32_to_bf16(silu_f(g) * u);
        }
        return;
    }
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < MN; i += (size_t)gridDim.x * 256) {
        float v = 0.f;
        for (int s = 0; s < n_split; s++) v += p.ws[s * MN + i];
        store_plain(p, (int)(i / p.N), (int)(i % p.N), v);
    }
}

struct GemmPlan {
    int cfg;      // 0: 128x128 block, 1: 64x128 block
    int split_k;
    int kb_per_split;
};

static GemmPlan plan_gemm(int M, int N, int K, int split_opt) {
    GemmPlan g;
    g.cfg = (M <= 64) ? 1 : 0;
    const int bm = g.cfg == 1 ? 64 : 128;
    const int tiles = ((M + bm - 1) / bm) * ((N + 127) / 128);
    const int kb = K / BK;
    int s = 1;
    if (split_opt > 0) {
        s = split_opt;
    } else {
        const int target = (g.cfg == 1) ? 768 : 256;  // skinny GEMMs stream weights: want every CU busy several times over
        if (tiles < target) s = (target + tiles - 1) / tiles;
        if (s > 16) s = 16;
    }
    if (s > kb) s = kb;
    if (s < 1) s = 1;
    g.kb_per_split = (kb + s - 1) / s;
    g.split_k = (kb + g.kb_per_split - 1) / g.kb_per_split;
    return g;
}

size_t gemm_splitk_ws_bytes(int M, int N, int K, int split_opt) {
    GemmPlan g = plan_gemm(M, N, K, split_opt);
    return g.split_k > 1 ? (size_t)g.split_k * M * N * sizeof(float) : 0;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t st) {
    if (a.M <= 0) return hipSuccess;
    GemmPlan g = plan_gemm(a.M, a.N, a.K, a.split_k);
    if (g.split_k > 1 && (size_t)g.split_k * a.M * a.N * sizeof(float) > a.splitk_ws_bytes) {
        g.split_k = 1;  // workspace too small: fall back to a single pass
        g.kb_per_split = a.K / BK;
    }
    GemmParams p;
    p.A = a.A; p.Bt = a.Bt; p.M = a.M; p.N = a.N; p.K = a.K; p.kind = a.kind; p.resid = a.resid; p.out = a.out;
    p.resid_f32 = a.resid_f32 ? 1 : 0; p.out_f32 = a.out_f32 ? 1 : 0;
    p.ws = g.split_k > 1 ? a.splitk_ws : nullptr;
    p.kb_per_split = g.kb_per_split;
    if (g.cfg == 1) {
        dim3 grid((a.N + 127) / 128, (a.M + 63) / 64, g.split_k);
        hipLaunchKernelGGL((gemm_kernel<64, 128, 2, 2>), grid, dim3(256), 0, st, p);
    } else {
        dim3 grid((a.N + 127) / 128, (a.M + 127) / 128, g.split_k);
        hipLaunchKernelGGL((gemm_kernel<128, 128, 2, 2>), grid, dim3(256), 0, st, p);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (g.split_k > 1) {
        const size_t total = (a.kind == GemmEpilogue::SWIGLU_BF16) ? (size_t)a.M * (a.N / 2) : (size_t)a.M * a.N;
        const int blocks = (int)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, p, g.split_k);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace ps
