// Weight GEMMs of the layer (Sec. 2.1: query/key/value generation, O-projection, gate/up and
// down projections; Sec. 2.2: the operations with a batching effect -- at small token counts
// their cost is the weight bytes streamed, at large ones the MFMA work).
//
//   C[M][N] = A[M][K] * W[K][N],  A = activations (bf16, K contiguous), fp32 accumulate.
//
// Weights are repacked once at layer init into MFMA-tile-major order (see repack_weight_kernel):
//   Wp[n_tile = n/16][k_block = k/32][g = (k%32)/8][nn = n%16][8]        (1 KiB per tile-block)
// so that one 16-byte load per lane fetches a contiguous KiB that already is the operand of a
// 16x16x32 MFMA (lane = 16 g + nn holds W^T[n][k0 + 8g .. +7]).
//
// Two kernels:
//  * gemm_wstream_kernel (M <= 64): weight streaming.  A wavefront owns 64 output columns and a
//    K slice, loads weight operands straight from HBM into registers (no LDS hop), activation
//    operands (operand order, see act_offset) from L1/L2, two k-block groups in flight; the four wavefronts of a block split K among
//    themselves and reduce through LDS in a fixed order.
//  * gemm_tiled_kernel (M > 64): 128x128 block tile, bf16 MFMA 32x32x16, operands staged
//    through LDS in BK = 64 slices with a register-held prefetch of the next slice.
// Output is either fp32 partials [split][M][N] (the consumer kernel sums the splits, adds the
// residual, normalises, rotates ...) or, for the fused gate/up matrix, silu(gate) * up in bf16.
#include "ps_device.h"

namespace ps {

struct GemmParams {
    const bf16_t* A;
    const bf16_t* Wp;
    int M, N, K;
    int kind;          // GemmOut::Kind
    void* out;         // fp32 [split][M][N] row-major, or bf16 [M][N/2] in operand order
    int kb_per_split;  // tiled: BK-slices per block split; wstream: 32-wide k-blocks per wavefront slice
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// ------------------------------------------------------------------------------------------
// Weight streaming kernel.  grid (N/64, splits), 256 threads.
// ------------------------------------------------------------------------------------------
template <int MT>
struct WsFrags {
    uint4 w[4];   // weight operands of the 4 column tiles
    uint4 x[MT];  // activation operands of the MT row tiles
};

template <int MT>
__device__ __forceinline__ void ws_load(WsFrags<MT>& f, const bf16_t* w_lane, size_t w_tile_stride, const bf16_t* x_lane, int kb) {
#pragma unroll
    for (int j = 0; j < 4; j++) f.w[j] = ldg16(w_lane + j * w_tile_stride + (size_t)kb * 512);
#pragma unroll
    for (int mt = 0; mt < MT; mt++) f.x[mt] = ldg16(x_lane + mt * w_tile_stride + (size_t)kb * 512);
}

template <int MT>
__device__ __forceinline__ void ws_mma(f32x4_t (&acc)[MT][4], const WsFrags<MT>& f) {
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < 4; j++)
            acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(f.w[j]), as_bf16x8(f.x[mt]), acc[mt][j], 0, 0, 0);
}

template <int MT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_wstream_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(16))) float red[4 * MT * 4 * 64 * 4];  // [wave][mt][j][lane] float4
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int ng = blockIdx.x;  // 64-column group
    const int KB = p.K >> 5;
    const int slice = blockIdx.y * 4 + wave;
    const int b0 = min(KB, slice * p.kb_per_split), b1 = min(KB, b0 + p.kb_per_split);

    const size_t w_tile_stride = (size_t)KB * 512;  // elements between consecutive 16-column tiles
    const bf16_t* w_lane = p.Wp + (size_t)ng * 4 * w_tile_stride + (size_t)lane * 8;
    const bf16_t* x_lane = p.A + (size_t)lane * 8;  // activations are in operand order: same tile stride as the weights

    f32x4_t acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[mt][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // groups of two k-blocks, two groups in flight; loads in the steady-state body are unconditional
    const int n_grp = (b1 - b0) >> 1;
    if (n_grp > 0) {
        WsFrags<MT> a0, a1, c0, c1;
        ws_load<MT>(a0, w_lane, w_tile_stride, x_lane, b0);
        ws_load<MT>(a1, w_lane, w_tile_stride, x_lane, b0 + 1);
        int i = 0;
        for (; i + 2 < n_grp; i += 2) {
            // the scheduling barriers keep each batch of loads ahead of the MFMAs that consume the
            // previous batch; without them the compiler sinks the loads and drains the queue
            ws_load<MT>(c0, w_lane, w_tile_stride, x_lane, b0 + 2 * i + 2);
            ws_load<MT>(c1, w_lane, w_tile_stride, x_lane, b0 + 2 * i + 3);
            __builtin_amdgcn_sched_barrier(0);
            ws_mma<MT>(acc, a0);
            ws_mma<MT>(acc, a1);
            __builtin_amdgcn_sched_barrier(0);
            ws_load<MT>(a0, w_lane, w_tile_stride, x_lane, b0 + 2 * i + 4);
            ws_load<MT>(a1, w_lane, w_tile_stride, x_lane, b0 + 2 * i + 5);
            __builtin_amdgcn_sched_barrier(0);
            ws_mma<MT>(acc, c0);
            ws_mma<MT>(acc, c1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (i + 2 == n_grp) {
            ws_load<MT>(c0, w_lane, w_tile_stride, x_lane, b0 + 2 * i + 2);
            ws_load<MT>(c1, w_lane, w_tile_stride, x_lane, b0 + 2 * i + 3);
            ws_mma<MT>(acc, a0);
            ws_mma<MT>(acc, a1);
            ws_mma<MT>(acc, c0);
            ws_mma<MT>(acc, c1);
        } else {
            ws_mma<MT>(acc, a0);
            ws_mma<MT>(acc, a1);
        }
    }
    if ((b1 - b0) & 1) {
        WsFrags<MT> t;
        ws_load<MT>(t, w_lane, w_tile_stride, x_lane, b1 - 1);
        ws_mma<MT>(acc, t);
    }

    // fixed-order reduction over the block's four K slices: wave w finishes column tile w
    float4* red4 = reinterpret_cast<float4*>(red);
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < 4; j++)
            red4[((wave * MT + mt) * 4 + j) * 64 + lane] = float4{acc[mt][j][0], acc[mt][j][1], acc[mt][j][2], acc[mt][j][3]};
    __syncthreads();
    auto total = [&](int mt, int j) {
        float4 s = red4[((0 * MT + mt) * 4 + j) * 64 + lane];
#pragma unroll
        for (int w = 1; w < 4; w++) {
            const float4 v = red4[((w * MT + mt) * 4 + j) * 64 + lane];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        return s;
    };
    // lane holds C[m = 16 mt + r][n = 64 ng + 16 j + 4 g + 0..3]
    if (p.kind == GemmOut::SWIGLU_BF16) {
        if (wave >= 2) return;  // tiles 0,1 = gate, tiles 2,3 = up of the same 32 features
        bf16_t* out = static_cast<bf16_t*>(p.out);
        const int F = p.N >> 1;
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const int m = mt * 16 + r;
            const float4 gt = total(mt, wave), up = total(mt, wave + 2);
            if (m < p.M) {
                uint2 o;
                o.x = pack_bf16(silu_f(gt.x) * up.x, silu_f(gt.y) * up.y);
                o.y = pack_bf16(silu_f(gt.z) * up.z, silu_f(gt.w) * up.w);
                *reinterpret_cast<uint2*>(out + act_offset(m, ng * 32 + wave * 16 + 4 * g, F)) = o;
            }
        }
        return;
    }
    float* out = static_cast<float*>(p.out) + (size_t)blockIdx.y * p.M * p.N;
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int m = mt * 16 + r;
        const float4 s = total(mt, wave);
        if (m < p.M) *reinterpret_cast<float4*>(out + (size_t)m * p.N + ng * 64 + wave * 16 + 4 * g) = s;
    }
}

// ------------------------------------------------------------------------------------------
// Tiled kernel.  grid (N/128, ceil(M/128), splits), 256 threads = 2x2 wavefronts of 64x64.
// ------------------------------------------------------------------------------------------
constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // +16 bytes per row: conflict-free 16-byte reads across 16 rows

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmParams p) {
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wave
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1 && TN % 2 == 0, "4 waves, even column tiles");
    constexpr int A_CHUNKS = BM * (BK / 8) / 256;  // 16-byte chunks per thread
    constexpr int B_CHUNKS = BN * (BK / 8) / 256;

    __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LDS_STRIDE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kb_total = p.K / BK;
    const int kb_begin = blockIdx.z * p.kb_per_split;
    const int kb_end = min(kb_total, kb_begin + p.kb_per_split);
    const int KB32 = p.K >> 5;
    const int n_tiles = p.N >> 4;
    const bf16_t* a_src[A_CHUNKS];
    const bf16_t* b_src[B_CHUNKS];
    int a_dst[A_CHUNKS], b_dst[B_CHUNKS];
    const int m_tiles = (p.M + 15) >> 4;
#pragma unroll
    for (int i = 0; i < A_CHUNKS; i++) {
        // A and B slices are fetched in source (operand) order: 64 consecutive chunks = one KiB tile-block
        const int c = tid + 256 * i, blk = c >> 6, l = c & 63;
        const int mtl = blk >> 1, kbl = blk & 1;
        const int mt = min(m0 / 16 + mtl, m_tiles - 1);
        a_src[i] = p.A + (((size_t)mt * KB32 + kbl) * 64 + l) * 8;
        a_dst[i] = (mtl * 16 + (l & 15)) * LDS_STRIDE + kbl * 32 + (l >> 4) * 8;
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; i++) {
        // chunk c of the B slice in source (tile-major) order: 64 consecutive chunks = one KiB tile-block
        const int c = tid + 256 * i, blk = c >> 6, l = c & 63;
        const int ntl = blk >> 1, kbl = blk & 1;  // 16-column tile and 32-wide k-block inside the slice
        const int nt = min(n0 / 16 + ntl, n_tiles - 1);
        b_src[i] = p.Wp + (((size_t)nt * KB32 + kbl) * 64 + l) * 8;
        b_dst[i] = (ntl * 16 + (l & 15)) * LDS_STRIDE + kbl * 32 + (l >> 4) * 8;
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
        for (int i = 0; i < A_CHUNKS; i++) ra[i] = ldg16(a_src[i] + (size_t)kb_begin * 2 * 512);
#pragma unroll
        for (int i = 0; i < B_CHUNKS; i++) rb[i] = ldg16(b_src[i] + (size_t)kb_begin * 2 * 512);
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
            for (int i = 0; i < A_CHUNKS; i++) ra[i] = ldg16(a_src[i] + (size_t)(kb + 1) * 2 * 512);
#pragma unroll
            for (int i = 0; i < B_CHUNKS; i++) rb[i] = ldg16(b_src[i] + (size_t)(kb + 1) * 2 * 512);
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

    // lane holds column n = lane%32, rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32 tile
    const int col = lane & 31, rbase = (lane >> 5) * 4;
    if (p.kind == GemmOut::SWIGLU_BF16) {
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
                    if (m < p.M && nb < p.N) out[act_offset(m, (nb >> 1) + col, F)] = f32_to_bf16(silu_f(acc[i][j][e]) * acc[i][j + 1][e]);
                }
        return;
    }
    float* out = static_cast<float*>(p.out) + (size_t)blockIdx.z * p.M * p.N;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int m = m0 + wm * WTM + i * 32 + (e >> 2) * 8 + rbase + (e & 3);
                const int n = n0 + wn * WTN + j * 32 + col;
                if (m < p.M && n < p.N) out[(size_t)m * p.N + n] = acc[i][j][e];
            }
}

// ------------------------------------------------------------------------------------------
// Planning and launch
// ------------------------------------------------------------------------------------------
struct GemmPlan {
    bool wstream;
    int splits;        // partial buffers written (grid.y / grid.z)
    int kb_per_split;
};

static GemmPlan plan_gemm(int M, int N, int K, int kind, int split_opt) {
    GemmPlan g;
    g.wstream = M <= 64;
    int s = 1;
    if (g.wstream) {
        const int groups = N / 64, KB = K / 32;
        if (kind != GemmOut::SWIGLU_BF16) {
            s = split_opt > 0 ? split_opt : (512 + groups - 1) / groups;  // aim at two blocks per CU
            s = std::min(s, 8);
            s = std::min(s, std::max(1, KB / 8));  // keep at least two k-blocks per wavefront slice
            s = std::max(s, 1);
        }
        g.kb_per_split = (KB + 4 * s - 1) / (4 * s);
        g.splits = s;
    } else {
        const int tiles = ((M + 127) / 128) * ((N + 127) / 128), kb = K / BK;
        if (kind != GemmOut::SWIGLU_BF16) {
            s = split_opt > 0 ? split_opt : (tiles < 256 ? (256 + tiles - 1) / tiles : 1);
            s = std::max(1, std::min(std::min(s, 8), kb));
        }
        g.kb_per_split = (kb + s - 1) / s;
        g.splits = (kb + g.kb_per_split - 1) / g.kb_per_split;
    }
    return g;
}

size_t gemm_out_bytes(int M, int N, int K, int kind, int split_opt) {
    if (kind == GemmOut::SWIGLU_BF16) return 0;  // dense output: the caller sizes it
    return (size_t)plan_gemm(M, N, K, kind, split_opt).splits * M * N * sizeof(float);
}

hipError_t launch_gemm(const GemmArgs& a, int* n_splits, hipStream_t st) {
    if (n_splits) *n_splits = 1;
    if (a.M <= 0) return hipSuccess;
    if (a.N % 64 || a.K % 64) return hipErrorInvalidValue;
    const GemmPlan g = plan_gemm(a.M, a.N, a.K, a.kind, a.split_k);
    if (gemm_out_bytes(a.M, a.N, a.K, a.kind, a.split_k) > a.out_bytes) return hipErrorInvalidValue;
    GemmParams p;
    p.A = a.A; p.Wp = a.Wp; p.M = a.M; p.N = a.N; p.K = a.K; p.kind = a.kind; p.out = a.out;
    p.kb_per_split = g.kb_per_split;
    if (n_splits) *n_splits = g.splits;
    if (g.wstream) {
        const dim3 grid(a.N / 64, g.splits);
        switch ((a.M + 15) / 16) {
            case 1: hipLaunchKernelGGL((gemm_wstream_kernel<1>), grid, dim3(256), 0, st, p); break;
            case 2: hipLaunchKernelGGL((gemm_wstream_kernel<2>), grid, dim3(256), 0, st, p); break;
            case 3: hipLaunchKernelGGL((gemm_wstream_kernel<3>), grid, dim3(256), 0, st, p); break;
            default: hipLaunchKernelGGL((gemm_wstream_kernel<4>), grid, dim3(256), 0, st, p); break;
        }
    } else {
        const dim3 grid((a.N + 127) / 128, (a.M + 127) / 128, g.splits);
        hipLaunchKernelGGL((gemm_tiled_kernel<128, 128, 2, 2>), grid, dim3(256), 0, st, p);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// One-time weight repack: W [K][N] (math layout) -> tile-major Wp (see the header comment).
// interleave = 0: row(n) = n.  interleave = 1/2 (gate / up halves of the fused matrix):
// row(f) = (f/32)*64 + f%32 + (interleave == 2 ? 32 : 0), so that every aligned group of 64 rows
// holds gate rows f..f+31 followed by up rows f..f+31 and SwiGLU can run in the GEMM epilogue.
// grid (ceil(N/64), K/64), 256 threads; n_rows_out = rows of the packed matrix.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void repack_weight_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp, int K,
                                                            int N, int interleave) {
    __shared__ bf16_t tile[64][66];  // [k][n]
    const int n0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int k = k0 + r, n = n0 + tx;
        tile[r][tx] = (k < K && n < N) ? w[(size_t)k * N + n] : (bf16_t)0;
    }
    __syncthreads();
    const int KB = K >> 5;
    for (int c = threadIdx.x; c < 512; c += 256) {
        const int blk = c >> 6, l = c & 63;
        const int ntl = blk >> 1, kbl = blk & 1;
        const int nl = ntl * 16 + (l & 15);  // column inside the 64-wide source tile
        const int n = n0 + nl;
        if (n >= N) continue;
        int row = n;
        if (interleave) row = (n >> 5) * 64 + (n & 31) + (interleave == 2 ? 32 : 0);
        const int kl = kbl * 32 + (l >> 4) * 8;
        uint32_t v[4];
#pragma unroll
        for (int j = 0; j < 4; j++) v[j] = (uint32_t)tile[kl + 2 * j][nl] | ((uint32_t)tile[kl + 2 * j + 1][nl] << 16);
        const size_t dst = (((size_t)(row >> 4) * KB + (k0 >> 5) + kbl) * 64 + (l >> 4) * 16 + (row & 15)) * 8;
        *reinterpret_cast<uint4*>(wp + dst) = uint4{v[0], v[1], v[2], v[3]};
    }
}

hipError_t launch_repack_weight(const bf16_t* w, bf16_t* wp, int K, int N, int interleave, hipStream_t st) {
    hipLaunchKernelGGL(repack_weight_kernel, dim3((N + 63) / 64, K / 64), dim3(256), 0, st, w, wp, K, N, interleave);
    return hipGetLastError();
}

}  // namespace ps
