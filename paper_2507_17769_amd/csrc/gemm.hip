// Weight GEMMs of the layer (Sec. 2.1: query/key/value generation, O-projection, gate/up and
// down projections; Sec. 2.2: the operations with a batching effect -- at small token counts
// their cost is the weight bytes streamed, at large ones the MFMA work).
//
//   C[M][N] = A[M][K] * W[K][N],  A = activations (bf16, K contiguous), fp32 accumulate.
//
// Weights are repacked once at layer init into MFMA operand blocks (see repack_weight_kernel):
//   Wp[n/64][k_block = k/32][j = (n%64)/16][g = (k%32)/8][nn = n%16][8]     (1 KiB per [g][nn][8] block)
// so that one 16-byte load per lane fetches a contiguous KiB that already is the operand of a
// 16x16x32 MFMA (lane = 16 g + nn holds W^T[n][k0 + 8g .. +7]), and the four blocks of a 64-column
// group are adjacent: the four wavefronts of a block that owns 64 columns read one sequential stream
// of 4 KiB per k-block between them instead of four separate streams of 1 KiB, which is what keeps
// DRAM rows open when two thousand wavefronts stream at once.
//
// Two kernels:
//  * gemm_wstream_kernel (M <= 96, and up to 160 for all but the QKV-shaped projection): weight streaming.  The four computing wavefronts of a block own 16 of
//    its 64 output columns each and load their weight operands straight from HBM into registers
//    (no LDS hop), four stages of two k-blocks ahead; a fifth wavefront copies the activation k-blocks
//    that all four need into an LDS ring.
//  * gemm_dma_kernel (above that, or forced by the tile option above 64): 256x256 or 128x128 block tile, bf16 MFMA 32x32x16.  Activations and
//    weights are both stored as KiB blocks that already are MFMA operands, so a k-slice of the
//    tile is copied HBM/L2 -> LDS verbatim by global_load_lds (no register hop, no transform) into
//    a ring of four stages, three in flight; the wavefronts read operands back with one
//    ds_read_b128 per 32x16 operand, interleaved one-for-two with the MFMAs that consume the
//    previous half-stage.  Block ids are mapped so that the blocks of one XCD share weight tiles.
// Output is either fp32 partials [split][M][N] (the consumer kernel sums the splits, adds the
// residual, normalises, rotates ...) or, for the fused gate/up matrix, silu(gate) * up in bf16.
#include "ps_device.h"

#include <algorithm>
#include <mutex>

namespace ps {

struct GemmParams {
    const bf16_t* A;
    const bf16_t* Wp;
    int M, N, K;
    int kind;          // GemmOut::Kind
    void* out;         // fp32 [split][M][N] row-major, or bf16 [M][N/2] in operand order
    int kb_per_split;  // 32-wide k-blocks per block
};

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// ------------------------------------------------------------------------------------------
// Weight streaming kernel (M <= 160: up to ten row tiles of 16).  grid (N/64/NG, splits), 64 (4 NG + 1) threads, NG = 1 or 2 column groups per block.
//
// A block owns 64 output columns and a K range.  Its four computing wavefronts divide the columns
// (16 each: one 16-byte load per lane and k-block fetches a KiB that already is a 16x16x32
// operand, the four wavefronts' KiBs being adjacent), so that all four need the same activation
// k-blocks and a fifth wavefront can copy those into an LDS ring once per block
// (global_load_lds, verbatim KiB blocks) instead of each wavefront fetching them from L2 for
// itself: a quarter of the activation traffic (an eighth with two column groups, eight computing wavefronts, per
// block), and no reduction across wavefronts at the end.
// The copying is a wavefront of its own because vector loads return in order: a computing
// wavefront that also waited for activations (from L2, quickly) would wait for every weight load
// issued before them (from HBM, slowly).  Stages of two k-blocks, one barrier per stage.
// ------------------------------------------------------------------------------------------
// The consumers' plain LDS reads are ordered against the producer wavefront's global_load_lds copies by the
// hardware barrier alone.  The builtin is no memory fence for the compiler, which could move an LDS read across
// it: the empty asm statements with a memory clobber pin the reads to their side without emitting any wait.
__device__ __forceinline__ void ws_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int MT, int KIND, int NG>
__global__ __launch_bounds__(64 * (4 * NG + 1)) void gemm_wstream_kernel(GemmParams p) {
    constexpr int NCW = 4 * NG;        // computing wavefronts: four per group of 64 columns, NG groups share the activation ring
    constexpr int XS = MT * 2 * 1024;  // bytes of an activation stage: MT row tiles x 2 k-blocks
    constexpr int WSETS = 4;           // weight stages in registers: three requested ahead of the one in work (a
                                       // deeper ring costs registers, i.e. resident blocks, and measured slower)
    __shared__ __attribute__((aligned(1024))) uint8_t lds[3 * XS];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KB = p.K >> 5;
    const int kb0 = blockIdx.y * p.kb_per_split;
    const int n_st = (min(KB, kb0 + p.kb_per_split) - kb0) >> 1;  // kb_per_split is even
    if (n_st <= 0) return;

    if (wave == NCW) {
        // Producer.  KiB block b of a stage = (row tile b / 2, k-block parity b % 2).  Stages past the end repeat the
        // last one into a slot nobody reads, so that every phase is the same.
        const uint8_t* xa = reinterpret_cast<const uint8_t*>(p.A) + (size_t)kb0 * 1024 + lane * 16;
        auto copy_stage = [&](int st, int slot) {
            const uint8_t* g = xa + (size_t)min(st, n_st - 1) * 2048;
#pragma unroll
            for (int b = 0; b < 2 * MT; b++)
                PS_GLOBAL_TO_LDS(g + ((size_t)(b >> 1) * KB + (b & 1)) * 1024, lds + slot * XS + b * 1024);
        };
        copy_stage(0, 0);
        copy_stage(1, 1);
        vm_wait<0>();
        __builtin_amdgcn_s_barrier();
        int wslot = 2;
        for (int sg = 0; sg < n_st; sg++) {
            copy_stage(sg + 2, wslot);  // the slot stage sg - 1 has left
            wslot = wslot == 2 ? 0 : wslot + 1;
            vm_wait<2 * MT>();          // stage sg + 1 has landed; this phase's copies stay in flight
            __builtin_amdgcn_s_barrier();
        }
        vm_wait<0>();
        if constexpr (KIND == GemmOut::SWIGLU_BF16) {  // the epilogue's barriers: no copy is in flight any more / sums handed over
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_s_barrier();
        }
        return;
    }

    const int r = lane & 15, g = lane >> 4;
    // this wavefront's column tile: block [ng][kb][cw] of the packed matrix.  A group past the last one (odd group
    // count with NG = 2) streams the last group again and stores nothing: it still takes part in every barrier.
    const int n_groups = p.N >> 6;
    const int ng_own = blockIdx.x * NG + wave / 4, cw = wave & 3;
    const bool have_group = ng_own < n_groups;
    const int ng = have_group ? ng_own : n_groups - 1;
    const uint8_t* w_src = reinterpret_cast<const uint8_t*>(p.Wp) + (((size_t)ng * KB + kb0) * 4 + cw) * 1024 + lane * 16;
    auto load_w = [&](uint4 (&w)[2], int st) {
        const uint8_t* gp = w_src + (size_t)min(st, n_st - 1) * 8192;
        w[0] = ldg16(gp);
        w[1] = ldg16(gp + 4096);
    };
    f32x4_t acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) acc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    uint4 w[WSETS][2];
#pragma unroll
    for (int s = 0; s < WSETS - 1; s++) load_w(w[s], s);
    ws_barrier();  // activation stages 0 and 1 are in their slots

#define PS_WSHARE_PHASE(I, SG)                                                                                  \
    {                                                                                                           \
        load_w(w[((I) + WSETS - 1) % WSETS], (SG) + WSETS - 1);                                                 \
        const uint8_t* xs_ = lds + slot * XS + lane * 16;                                                       \
        uint4 x_[2][MT];                                                                                        \
        _Pragma("unroll") for (int q = 0; q < 2; q++)                                                           \
            _Pragma("unroll") for (int mt = 0; mt < MT; mt++) x_[q][mt] = *reinterpret_cast<const uint4*>(xs_ + (mt * 2 + q) * 1024); \
        _Pragma("unroll") for (int q = 0; q < 2; q++)                                                           \
            _Pragma("unroll") for (int mt = 0; mt < MT; mt++)                                                   \
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(w[(I)][q]), as_bf16x8(x_[q][mt]), acc[mt], 0, 0, 0); \
        slot = slot == 2 ? 0 : slot + 1;                                                                        \
        ws_barrier();                                                                                           \
    }
    int slot = 0, s = 0;
    for (; s + WSETS <= n_st; s += WSETS) {
        PS_WSHARE_PHASE(0, s)
        PS_WSHARE_PHASE(1, s + 1)
        PS_WSHARE_PHASE(2, s + 2)
        PS_WSHARE_PHASE(3, s + 3)
    }
    if (s < n_st) PS_WSHARE_PHASE(0, s)
    if (s + 1 < n_st) PS_WSHARE_PHASE(1, s + 1)
    if (s + 2 < n_st) PS_WSHARE_PHASE(2, s + 2)
#undef PS_WSHARE_PHASE

    // lane holds C[m = 16 mt + r][n = 64 ng + 16 cw + 4 g + 0..3]
    if constexpr (KIND == GemmOut::SWIGLU_BF16) {
        // column tiles 0, 1 = gate, tiles 2, 3 = up of the same 32 features: wavefronts 2 and 3 of a group hand their sums over
        float4* up4 = reinterpret_cast<float4*>(lds);  // [group in block][cw - 2][mt][lane]
        const int gi = wave / 4;
        ws_barrier();                                  // the ring is free: the producer's last copies have landed
        if (cw >= 2) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++) up4[((gi * 2 + cw - 2) * MT + mt) * 64 + lane] = float4{acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]};
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the LDS writes have been made before the barrier
        ws_barrier();
        if (cw >= 2 || !have_group) return;
        bf16_t* out = static_cast<bf16_t*>(p.out);
        const int F = p.N >> 1;
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const int m = mt * 16 + r;
            const float4 up = up4[((gi * 2 + cw) * MT + mt) * 64 + lane];
            if (m < p.M) {
                uint2 o;
                o.x = pack_bf16(silu_f(acc[mt][0]) * up.x, silu_f(acc[mt][1]) * up.y);
                o.y = pack_bf16(silu_f(acc[mt][2]) * up.z, silu_f(acc[mt][3]) * up.w);
                *reinterpret_cast<uint2*>(out + act_offset(m, ng * 32 + cw * 16 + 4 * g, F)) = o;
            }
        }
    } else {
        if (!have_group) return;
        float* out = static_cast<float*>(p.out) + (size_t)blockIdx.y * p.M * p.N;
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const int m = mt * 16 + r;
            if (m < p.M)
                *reinterpret_cast<float4*>(out + (size_t)m * p.N + ng * 64 + cw * 16 + 4 * g) = float4{acc[mt][0], acc[mt][1], acc[mt][2], acc[mt][3]};
        }
    }
}

// ------------------------------------------------------------------------------------------
// Tiled kernel.  One block per (row tile, column tile, K split) unit, WM x WN wavefronts.
//
// LDS holds NS stages; a stage is one 32-wide k-block of the tile: BM/16 activation blocks, then
// BN/16 weight blocks, each the KiB that a 16x16x32 operand occupies in memory (lane l's 16 bytes
// at l*16).  A 32x32x16 operand (rows r = l%32, k-half h = l/32 of k-sixteenth `sub`) is two such
// blocks side by side: lane l reads block r/16 at ((2 sub + h) * 16 + r%16) * 16.
//
// The LDS reads are inline assembly because the compiler, which cannot tell an LDS read from the
// LDS writes of global_load_lds in flight, would drain the load queue before each of them.  It
// therefore does not know that the read registers are written asynchronously: every wait below
// names the registers it makes valid, so that their consumers cannot move above it, and no read
// is left in flight where registers could be copied (the loop has a single straight-line body
// whose in-flight reads sit in loop-carried registers).
// ------------------------------------------------------------------------------------------
struct TiledParams {
    GemmParams g;
    int tiles_m, tiles_n, splits, units_per_xcd;
};

template <int BM, int BN, int WM, int WN, int NS, int KIND>
__global__ __launch_bounds__(64 * WM * WN) void gemm_dma_kernel(TiledParams tp) {
    const GemmParams& p = tp.g;
    constexpr int NW = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wavefront tile
    constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 MFMA tiles per wavefront
    constexpr int NBLK = (BM + BN) / 16;         // KiB blocks per stage
    constexpr int LPW = NBLK / NW;               // loads per wavefront per stage
    constexpr int STAGE = NBLK * 1024;           // bytes
    constexpr int NT = TM * TN, NR = TM + TN;
    static_assert(NBLK % NW == 0 && NS >= 3 && NS <= 4 && NT >= 2 && (TN == 4 || TN == 2) && TM <= 4, "shape");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // Consecutive block ids go to different XCDs (each with its own L2).  XCD x works through the units
    // [x * units_per_xcd, (x+1) * units_per_xcd) of the order (column tile, split, row tile), row tile
    // fastest: the blocks resident on one XCD at a time share a few weight tiles.
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int unit = xcd * tp.units_per_xcd + idx;
    if (idx >= tp.units_per_xcd || unit >= tp.tiles_m * tp.tiles_n * tp.splits) return;
    const int tm = unit % tp.tiles_m, rest = unit / tp.tiles_m;
    const int split = rest % tp.splits, tn = rest / tp.splits;
    const int m0 = tm * BM, n0 = tn * BN;
    const int KB = p.K >> 5;
    const int kb0 = split * p.kb_per_split;
    const int n_kb = min(KB, kb0 + p.kb_per_split) - kb0;
    if (n_kb <= 0) return;  // (the host plans no empty split)

    // this wavefront's LPW blocks of a stage (block b = wave + NW i): byte offsets from A / Wp, < 4 GiB
    const int m_tiles = (p.M + 15) >> 4, n_tiles = p.N >> 4;
    uint32_t off[LPW];
#pragma unroll
    for (int i = 0; i < LPW; i++) {
        const int b = wave + NW * i;
        // rows / columns past the edge re-read the last tile: its products land in accumulators that are not stored
        if (b < BM / 16) off[i] = (uint32_t)min(m0 / 16 + b, m_tiles - 1) * (uint32_t)KB * 1024u + lane * 16;
        else {
            const int nt = min(n0 / 16 + (b - BM / 16), n_tiles - 1);  // weight blocks: [nt/4][kb][nt%4]
            off[i] = ((uint32_t)(nt >> 2) * (uint32_t)KB * 4u + (uint32_t)(nt & 3)) * 1024u + lane * 16;
        }
    }
    const uint8_t* gA = reinterpret_cast<const uint8_t*>(p.A) + (size_t)kb0 * 1024;
    const uint8_t* gW = reinterpret_cast<const uint8_t*>(p.Wp) + (size_t)kb0 * 4096;
    auto issue_one = [&](int i, int s, int slot) {
        const int b = wave + NW * i;
        const uint8_t* g = b < BM / 16 ? gA + (size_t)s * 1024 : gW + (size_t)s * 4096;
        PS_GLOBAL_TO_LDS(g + off[i], lds + slot * STAGE + b * 1024);
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const int r = lane & 31, h = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const uint32_t a_lane = lds0 + (wm * (WTM / 16) + (r >> 4)) * 1024 + (h * 16 + (r & 15)) * 16;
    const uint32_t b_lane = lds0 + (BM / 16 + wn * (WTN / 16) + (r >> 4)) * 1024 + (h * 16 + (r & 15)) * 16;

    // Operand registers of a half-stage (one k-sixteenth): v[0..TM) = A tiles, v[TM..NR) = B tiles.  They are
    // read in the order q = 0: A0;  q = 1..TN: B0..B(TN-1);  q = TN+i: A_i (i >= 1), one read behind every
    // NT/NR-th MFMA of the half-stage before, and waited for row by row.
    struct Ops { u32x4_t v[NR]; } o0, o1;
#define PS_SLOT(q) ((q) == 0 ? 0 : (q) <= TN ? TM + (q) - 1 : (q) - TN)
#define PS_T_OF(q) (((q) + 1) * NT / NR - 1) /* MFMA behind which read q is issued */
#define PS_READQ(o, base_a, base_b, sub, q)                                                           \
    {                                                                                                  \
        if (PS_SLOT(q) < TM) o.v[PS_SLOT(q)] = lds_read16(base_a, PS_SLOT(q) * 2048 + (sub) * 512);    \
        else o.v[PS_SLOT(q)] = lds_read16(base_b, (PS_SLOT(q) - TM) * 2048 + (sub) * 512);             \
    }
    // Before MFMA t = i*TN (i >= 1) operand A_i must have landed.  Outstanding then: the reads of the same
    // half-stage behind A_i (TM - 1 - i of them) and the reads of the next half-stage issued so far.
    auto wait_row = [&](u32x4_t& a, int t) {
        int n_new = 0;
        for (int q = 0; q < NR; q++) n_new += (PS_T_OF(q) < t);
        switch ((TM - 1 - t / TN) + n_new) {  // t is a constant after unrolling: one case survives
            case 0: lgkm_tie<0>(a); break;
            case 1: lgkm_tie<1>(a); break;
            case 2: lgkm_tie<2>(a); break;
            case 3: lgkm_tie<3>(a); break;
            case 4: lgkm_tie<4>(a); break;
            case 5: lgkm_tie<5>(a); break;
            case 6: lgkm_tie<6>(a); break;
            case 7: lgkm_tie<7>(a); break;
            default: lgkm_tie<0>(a); break;
        }
    };
    // One half-stage: NT MFMAs on `o`, the reads of the next half-stage into `on`, and with WITH_LOADS the
    // LPW loads of stage s_next.  The scheduling barriers keep the written order.
#define PS_STEP(o, on, base_a, base_b, sub, WITH_LOADS, s_next, slot_next)                                             \
    {                                                                                                                  \
        _Pragma("unroll") for (int t = 0; t < NT; t++) {                                                               \
            if (t == 0) {                                                                                              \
                if constexpr (TN == 4) lgkm_tie<NR - 1 - TN>(o.v[0], o.v[TM], o.v[TM + 1], o.v[TM + 2], o.v[TM + 3]);  \
                else lgkm_tie<NR - 1 - TN>(o.v[0], o.v[TM], o.v[TM + 1]);                                              \
            } else if (t % TN == 0) {                                                                                  \
                wait_row(o.v[t / TN], t);                                                                              \
            }                                                                                                          \
            acc[t / TN][t % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, o.v[t / TN]),    \
                                                                          __builtin_bit_cast(bf16x8_t, o.v[TM + t % TN]), \
                                                                          acc[t / TN][t % TN], 0, 0, 0);               \
            _Pragma("unroll") for (int q_ = 0; q_ < NR; q_++)                                                          \
                if (PS_T_OF(q_) == t) PS_READQ(on, base_a, base_b, sub, q_)                                            \
            if (WITH_LOADS) {                                                                                          \
                _Pragma("unroll") for (int i_ = 0; i_ < LPW; i_++)                                                     \
                    if (i_ * NT / LPW == t) issue_one(i_, s_next, slot_next);                                          \
            }                                                                                                          \
            __builtin_amdgcn_sched_barrier(0);                                                                         \
        }                                                                                                              \
    }

    // NS slots, NS-1 stages in flight.  Loads past the last stage fetch the last stage again, into a slot
    // that nobody reads any more: the loop body is the same every time and the wait counts are constants.
#pragma unroll
    for (int s = 0; s < NS - 1; s++)
#pragma unroll
        for (int i = 0; i < LPW; i++) issue_one(i, min(s, n_kb - 1), s);
    vm_wait<(NS - 2) * LPW>();
    __builtin_amdgcn_s_barrier();
    uint32_t a_cur = a_lane, b_cur = b_lane;
#pragma unroll
    for (int q_ = 0; q_ < NR; q_++) PS_READQ(o0, a_cur, b_cur, 0, q_);
    int slot = 0;
    for (int s = 0; s < n_kb; s++) {
        __builtin_amdgcn_sched_barrier(0);
        PS_STEP(o0, o1, a_cur, b_cur, 1, false, 0, 0);
        // Past this barrier stage s+1 has landed for every wavefront, and every wavefront has consumed
        // stage s-1, whose slot the loads of stage s+NS-1 overwrite.  Reads of stage s may still be in
        // flight: its slot is not touched before the next barrier.
        vm_wait<(NS - 3) * LPW>();
        __builtin_amdgcn_s_barrier();
        const int next = slot + 1 == NS ? 0 : slot + 1;
        const int prev = slot == 0 ? NS - 1 : slot - 1;
        a_cur = a_lane + next * STAGE;
        b_cur = b_lane + next * STAGE;
        __builtin_amdgcn_sched_barrier(0);
        PS_STEP(o1, o0, a_cur, b_cur, 0, true, min(s + NS - 1, n_kb - 1), prev);
        slot = next;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the reads issued for the stage past the end
    vm_wait<0>();
#undef PS_SLOT
#undef PS_T_OF
#undef PS_READQ
#undef PS_STEP

    // lane holds column n = lane%32, rows 8*(e/4) + 4*(lane/32) + e%4 of each 32x32 tile.  The scheduling
    // barriers keep the tiles' stores apart: hoisting all accumulator reads to the top would need a
    // register for each of them, and the allocator would pay for that inside the main loop.
    const int col = lane & 31, rbase = (lane >> 5) * 4;
    if constexpr (KIND == GemmOut::SWIGLU_BF16) {
        // silu(gate) * up through LDS, one 32-row band of the wavefront tile at a time: the accumulators go
        // to a private [32][WTN] fp32 patch as they are, and come back as the 8 gate and 8 up values of one
        // row that make a 16-byte piece of the operand-order output, so that a wavefront stores whole KiB
        // blocks.  Rows past M are stored too: the buffer holds whole row tiles (gemm_out_bytes).
        constexpr int RS = WTN + 4;  // patch row stride in floats: the 16 rows of a read fall into different banks
        static_assert(32 * RS * 4 * NW <= NS * STAGE, "epilogue patch fits the stage ring");
        __syncthreads();  // every wavefront is done with the stages
        float* patch = reinterpret_cast<float*>(lds) + wave * 32 * RS;
        const int F = p.N >> 1;
        bf16_t* out = static_cast<bf16_t*>(p.out);
        const int g8 = lane >> 4, r16 = lane & 15;
#pragma unroll
        for (int i = 0; i < TM; i++) {
#pragma unroll
            for (int j = 0; j < TN; j++)
#pragma unroll
                for (int e = 0; e < 16; e++) patch[((e >> 2) * 8 + rbase + (e & 3)) * RS + j * 32 + col] = acc[i][j][e];
            const int mb = m0 + wm * WTM + i * 32;
#pragma unroll
            for (int band = 0; band < 2; band++)
#pragma unroll
                for (int j = 0; j < TN; j += 2) {
                    const int nb = n0 + wn * WTN + j * 32;  // multiple of 64: gate tile, then up tile of the same 32 features
                    const float* src = patch + (band * 16 + r16) * RS + j * 32 + g8 * 8;
                    const float4 ga = *reinterpret_cast<const float4*>(src), gb = *reinterpret_cast<const float4*>(src + 4);
                    const float4 ua = *reinterpret_cast<const float4*>(src + 32), ub = *reinterpret_cast<const float4*>(src + 36);
                    uint4 o;
                    o.x = pack_bf16(silu_f(ga.x) * ua.x, silu_f(ga.y) * ua.y);
                    o.y = pack_bf16(silu_f(ga.z) * ua.z, silu_f(ga.w) * ua.w);
                    o.z = pack_bf16(silu_f(gb.x) * ub.x, silu_f(gb.y) * ub.y);
                    o.w = pack_bf16(silu_f(gb.z) * ub.z, silu_f(gb.w) * ub.w);
                    // KiB block (row band, 32-feature block): lane = 16 g + row holds features 8 g .. 8 g + 7 of its row
                    if (nb < p.N)
                        *reinterpret_cast<uint4*>(out + ((size_t)((mb >> 4) + band) * (F >> 5) + (nb >> 6)) * 512 + lane * 8) = o;
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        const bool interior = m0 + BM <= p.M && n0 + BN <= p.N;
        float* out = static_cast<float*>(p.out) + (size_t)split * p.M * p.N;
#pragma unroll
        for (int i = 0; i < TM; i++)
#pragma unroll
            for (int j = 0; j < TN; j++) {
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const int m = m0 + wm * WTM + i * 32 + (e >> 2) * 8 + rbase + (e & 3);
                    const int n = n0 + wn * WTN + j * 32 + col;
                    if (interior || (m < p.M && n < p.N)) out[(size_t)m * p.N + n] = acc[i][j][e];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    }
}

// ------------------------------------------------------------------------------------------
// Planning and launch
// ------------------------------------------------------------------------------------------
struct GemmPlan {
    bool wstream;
    bool big_tile;     // tiled: 256x256 blocks (else 128x128)
    int splits;        // partial buffers written
    int kb_per_split;  // 32-wide k-blocks per block
};

// Tiled-kernel cost model, fitted to measured sweeps over the layer's GEMM shapes (M 144 .. 2304):
// a 256x256 block runs alone on a CU and takes ~1.0 us per 32-wide k-stage; two 128x128 blocks share a
// CU at ~0.62 us per stage each.  A unit costs its stages plus ~10 stages of prologue and epilogue,
// units run in rounds of one per slot, and every split beyond the first adds partial-sum traffic.
static double tiled_cost(int M, int N, int K, bool big, int splits, int* kb_per_split, int* eff_splits) {
    const int B = big ? 256 : 128, slots = big ? 256 : 512;
    const double t_stage = big ? 1.0 : 0.62;
    const int KB = K / 32, kps = (KB + splits - 1) / splits, s_eff = (KB + kps - 1) / kps;
    const long units = (long)((M + B - 1) / B) * ((N + B - 1) / B) * s_eff;
    const long rounds = (units + slots - 1) / slots;
    *kb_per_split = kps;
    *eff_splits = s_eff;
    return rounds * (kps + 10) * t_stage + (s_eff > 1 ? 2.0 * (s_eff - 1) * (double)M * N * 4 / 5e6 : 0.0);
}

static GemmPlan plan_gemm(int M, int N, int K, int kind, int split_opt, int tile_opt) {
    GemmPlan g;
    // measured: streaming wins up to 96 tokens for every projection, and up to 160 (ten row tiles) for all but the QKV-shaped
    // one (more columns than rows of weights: 48 blocks per split and six splits of partial sums; 129 tokens: 29 vs 24 us),
    // above all for the gate/up matrix (129 tokens: 61 vs 75 us) and the down projection (42 vs 46)
    g.wstream = M <= 64 || (tile_opt == 0 && (M <= 96 || (M <= 160 && (kind == GemmOut::SWIGLU_BF16 || N <= K))));
    g.big_tile = false;
    int s = 1;
    if (g.wstream) {
        const int groups = N / 64, KB = K / 32;
        if (kind != GemmOut::SWIGLU_BF16) {
            s = split_opt > 0 ? split_opt : (512 + groups - 1) / groups;  // aim at two blocks per CU
            s = std::min(s, 8);
            s = std::min(s, std::max(1, KB / 8));  // keep at least two k-blocks per wavefront slice
            s = std::max(s, 1);
        }
        int kps = (KB + s - 1) / s;
        kps += kps & 1;  // whole stages of two k-blocks
        g.kb_per_split = kps;
        g.splits = (KB + kps - 1) / kps;
    } else {
        const int s_lo = kind == GemmOut::SWIGLU_BF16 ? 1 : (split_opt > 0 ? std::min(split_opt, 8) : 1);
        const int s_hi = kind == GemmOut::SWIGLU_BF16 ? 1 : (split_opt > 0 ? s_lo : 8);
        double best = 0;
        bool first = true;
        for (int big = (tile_opt == 256 ? 1 : 0); big < (tile_opt == 128 ? 1 : 2); big++)
            for (int sp = s_lo; sp <= s_hi; sp++) {
                int kps, eff;
                const double c = tiled_cost(M, N, K, big != 0, sp, &kps, &eff);
                if (first || c < best) {
                    first = false; best = c;
                    g.big_tile = big != 0; g.splits = eff; g.kb_per_split = kps;
                }
            }
    }
    return g;
}

size_t gemm_out_bytes(int M, int N, int K, int kind, int split_opt, int tile_opt) {
    if (kind == GemmOut::SWIGLU_BF16) {
        // dense [rows][N/2] in operand order.  The tiled kernel stores whole row tiles without a row check
        // (rows past M are never read back), so the buffer holds M rounded up to its largest tile.
        const size_t rows = M <= 64 ? (size_t)((M + 15) / 16 * 16) : (size_t)((M + 255) / 256 * 256);
        return rows * (N / 2) * sizeof(bf16_t);
    }
    return (size_t)plan_gemm(M, N, K, kind, split_opt, tile_opt).splits * M * N * sizeof(float);
}

template <int BM, int BN, int WM, int WN, int NS, int KIND>
static hipError_t launch_tiled(const GemmParams& p, const GemmPlan& g, hipStream_t st) {
    constexpr int lds_bytes = (BM + BN) / 16 * 1024 * NS;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {   // more dynamic LDS than the default limit: raise it once per kernel
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_kernel<BM, BN, WM, WN, NS, KIND>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (attr_err != hipSuccess) return attr_err;
    TiledParams tp;
    tp.g = p;
    tp.tiles_m = (p.M + BM - 1) / BM;
    tp.tiles_n = (p.N + BN - 1) / BN;
    tp.splits = g.splits;
    const long units = (long)tp.tiles_m * tp.tiles_n * tp.splits;
    tp.units_per_xcd = (int)((units + 7) / 8);
    hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WM, WN, NS, KIND>), dim3(tp.units_per_xcd * 8), dim3(64 * WM * WN), lds_bytes, st, tp);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, int* n_splits, hipStream_t st) {
    if (n_splits) *n_splits = 1;
    if (a.M <= 0) return hipSuccess;
    if (a.N % 64 || a.K % 64) return hipErrorInvalidValue;
    // the tiled kernel addresses A and Wp with 32-bit byte offsets
    if (a.M > 64 && ((size_t)a.N * a.K * 2 >= (1ull << 32) || (size_t)((a.M + 15) / 16 * 16) * a.K * 2 >= (1ull << 32)))
        return hipErrorInvalidValue;
    const GemmPlan g = plan_gemm(a.M, a.N, a.K, a.kind, a.split_k, a.tile);
    if (gemm_out_bytes(a.M, a.N, a.K, a.kind, a.split_k, a.tile) > a.out_bytes) return hipErrorInvalidValue;
    GemmParams p;
    p.A = a.A; p.Wp = a.Wp; p.M = a.M; p.N = a.N; p.K = a.K; p.kind = a.kind; p.out = a.out;
    p.kb_per_split = g.kb_per_split;
    if (n_splits) *n_splits = g.splits;
    if (g.wstream) {
        const int mt = (a.M + 15) / 16;
        // Two column groups per block halve the activation copies (as many bytes as the weights at 64 tokens) at the
        // price of half as many blocks.  Measured: always a gain for the gate/up matrix (448 groups, no K split; 64
        // tokens: 54 -> 49 us), a gain for the split projections from four row tiles on, a loss below.
        const bool two = a.kind == GemmOut::SWIGLU_BF16 || mt >= 4;
        const dim3 grid(two ? (a.N / 64 + 1) / 2 : a.N / 64, g.splits);
#define PS_WS_LAUNCH(MT_)                                                                                                  \
    if (a.kind == GemmOut::SWIGLU_BF16) hipLaunchKernelGGL((gemm_wstream_kernel<MT_, GemmOut::SWIGLU_BF16, 2>), grid, dim3(576), 0, st, p); \
    else if (two) hipLaunchKernelGGL((gemm_wstream_kernel<MT_, GemmOut::PARTIAL_F32, 2>), grid, dim3(576), 0, st, p);             \
    else hipLaunchKernelGGL((gemm_wstream_kernel<MT_, GemmOut::PARTIAL_F32, 1>), grid, dim3(320), 0, st, p);
        switch (mt) {
            case 1: PS_WS_LAUNCH(1) break;
            case 2: PS_WS_LAUNCH(2) break;
            case 3: PS_WS_LAUNCH(3) break;
            case 4: PS_WS_LAUNCH(4) break;
            case 5: PS_WS_LAUNCH(5) break;
            case 6: PS_WS_LAUNCH(6) break;
            case 7: PS_WS_LAUNCH(7) break;
            case 8: PS_WS_LAUNCH(8) break;
            case 9: PS_WS_LAUNCH(9) break;
            default: PS_WS_LAUNCH(10) break;
        }
#undef PS_WS_LAUNCH
        return hipGetLastError();
    }
    if (a.kind == GemmOut::SWIGLU_BF16)
        return g.big_tile ? launch_tiled<256, 256, 2, 2, 4, GemmOut::SWIGLU_BF16>(p, g, st)
                          : launch_tiled<128, 128, 2, 2, 4, GemmOut::SWIGLU_BF16>(p, g, st);
    return g.big_tile ? launch_tiled<256, 256, 2, 2, 4, GemmOut::PARTIAL_F32>(p, g, st)
                      : launch_tiled<128, 128, 2, 2, 4, GemmOut::PARTIAL_F32>(p, g, st);
}

// ------------------------------------------------------------------------------------------
// One-time weight repack: W [K][N] (math layout) -> operand blocks Wp (see the header comment).
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
        const int rt = row >> 4;  // 16-row tile of the packed matrix: block [rt/4][kb][rt%4]
        const size_t dst = ((((size_t)(rt >> 2) * KB + (k0 >> 5) + kbl) * 4 + (rt & 3)) * 64 + (l >> 4) * 16 + (row & 15)) * 8;
        *reinterpret_cast<uint4*>(wp + dst) = uint4{v[0], v[1], v[2], v[3]};
    }
}

hipError_t launch_repack_weight(const bf16_t* w, bf16_t* wp, int K, int N, int interleave, hipStream_t st) {
    hipLaunchKernelGGL(repack_weight_kernel, dim3((N + 63) / 64, K / 64), dim3(256), 0, st, w, wp, K, N, interleave);
    return hipGetLastError();
}

}  // namespace ps
