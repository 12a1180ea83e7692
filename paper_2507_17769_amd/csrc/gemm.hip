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
//  * gemm_sk_kernel (above that, or forced by the tile option above 64): 256x256 or 128x128 block tile, bf16 MFMA 16x16x32.  Activations and
//    weights are both stored as KiB blocks that already are MFMA operands, so a k-slice of the
//    tile is copied HBM/L2 -> LDS verbatim by global_load_lds (no register hop, no transform) into
//    a ring of four stages, three in flight; the wavefronts read operands back with one
//    ds_read_b128 per 16x32 operand, interleaved with the MFMAs that consume the previous stage.
//    Blocks are resident once per compute unit and take whole tiles in waves; the K loops of the tiles
//    that do not fill a wave are cut evenly over the blocks ("stream-K"), see SkParams.
// Output is either fp32 partials [split][M][N] (one per K split of the streaming kernel; the consumer kernel sums the splits, adds the
// residual, normalises, rotates ...) or, for the fused gate/up matrix, silu(gate) * up in bf16.
#include "ps_device.h"
#include "sk_decomp.h"

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
        w[0] = ldg16_stream(gp);
        w[1] = ldg16_stream(gp + 4096);
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
// Tiled kernel.  LDS holds NS stages; a stage is one 32-wide k-block of the tile: BM/16 activation blocks, then
// BN/16 weight blocks, each the KiB that a 16x16x32 operand occupies in memory.
//
// The LDS reads are inline assembly because the compiler, which cannot tell an LDS read from the LDS writes of
// global_load_lds in flight, would drain the load queue before each of them.  It therefore does not know that
// the read registers are written asynchronously: every wait names the registers it makes valid, so that their
// consumers cannot move above it.
//
// Why the 16x16x32 MFMA: under the power limit it sustains more than the 32x32x16 form.  A loop of nothing
// but independent MFMAs on N(0,1) x N(0,0.02) operands (128x128 per wavefront, one wavefront per SIMD)
// runs at 2.06 PFLOP/s against 1.79-1.83 with the 32x32x16 form, while both reach the nominal 2.45 on
// all-zero operands: the small form reads and writes a quarter of the accumulator values per instruction
// for half the flops, and the clock the power management holds follows the energy per flop.
//
// A stage's KiB blocks ARE 16x16x32 operands (lane l's 16 bytes at l*16: row l%16, k 8*(l/16)..+7), so an
// operand is one ds_read_b128 at a constant offset.  The weight tile is the A operand and the activation
// tile the B operand: a lane then holds four consecutive output columns of one row (float4 stores of the
// partial sums), and for the gate/up matrix the gate and up values of the same four features sit in the same
// lane of two accumulators, so silu(gate) * up is formed in registers and stored as 8-byte pieces of the
// operand-order activation without a pass through LDS.
//
// Per stage and wavefront (256x256 block, 128x128 per wavefront): 64 MFMAs on the operand set read during the
// previous stage, the 16 reads of the next stage's operands (one behind every third MFMA, all waited for at
// the end of the stage, the last one having had more than 250 cycles), the wavefront's 8 copies of the stage
// three ahead, one barrier.  Two operand sets alternate, so the loop is unrolled by two stages and the
// registers of in-flight reads never cross a copy.
// ------------------------------------------------------------------------------------------
template <int N>
struct OpSet { u32x4_t v[N]; };

// acc += A . B, the accumulator pinned to the accumulation registers and the operands to the vector registers.
// Written as assembly because the register allocator, left to choose per instruction between the two register files
// for 256 accumulator registers plus 128 operand registers, shuffles them between the files inside the main loop.
// The compiler inserts no hazard waits around assembly: every accumulator is used again 64 (16) instructions later,
// far beyond the instruction's passes, and the epilogue waits before it reads the results.
__device__ __forceinline__ void mfma16_acc(f32x4_t& c, const u32x4_t& a, const u32x4_t& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

__device__ __forceinline__ void lgkm0_tie(OpSet<4>& o) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]));
}
__device__ __forceinline__ void vm0_tie(OpSet<4>& o) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]));
}
__device__ __forceinline__ void vm0_tie(OpSet<8>& o) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]), "+v"(o.v[4]), "+v"(o.v[5]), "+v"(o.v[6]), "+v"(o.v[7]));
}
__device__ __forceinline__ void lgkm0_tie(OpSet<8>& o) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]), "+v"(o.v[4]), "+v"(o.v[5]), "+v"(o.v[6]), "+v"(o.v[7]));
}
__device__ __forceinline__ void lgkm0_tie(OpSet<12>& o) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]), "+v"(o.v[4]), "+v"(o.v[5]), "+v"(o.v[6]), "+v"(o.v[7]),
                                          "+v"(o.v[8]), "+v"(o.v[9]), "+v"(o.v[10]), "+v"(o.v[11]));
}
__device__ __forceinline__ void lgkm0_tie(OpSet<16>& o) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]), "+v"(o.v[4]), "+v"(o.v[5]), "+v"(o.v[6]), "+v"(o.v[7]),
                                          "+v"(o.v[8]), "+v"(o.v[9]), "+v"(o.v[10]), "+v"(o.v[11]), "+v"(o.v[12]), "+v"(o.v[13]), "+v"(o.v[14]), "+v"(o.v[15]));
}

// Work decomposition ("stream-K" tail).  The tiles, in the order (column tile, row tile) with the row tile fastest,
// are dealt in contiguous ranges to the eight XCDs (one L2 each); block ids are handed out round-robin over the XCDs,
// so block id % 8 is the XCD and id / 8 = lb its index there, 0 .. B-1, B blocks per XCD being resident at once.
// An XCD with T tiles runs T / B waves of whole tiles (block lb takes tiles lb, lb + B, ...: the B tiles in flight
// are a few columns x all rows, so weight and activation panels are shared through the L2), and then the T % B
// tiles that are left, whose K loops it cuts into B equal runs, one per block: no partial last wave.  A run that
// covers part of a tile's K range parks its accumulators in a workspace slot and counts itself in on the tile;
// whichever block counts in last adds the parked pieces up, always in the order of their K ranges, and runs the
// epilogue.  Nobody waits for anybody: the blocks exchange nothing but the parked pieces and the counter, each
// side of which is fenced at device scope.
struct SkParams {
    GemmParams g;
    int tiles_m, tiles_n, splits, kp_per_split;   // K splits of every tile (1 for the gate/up matrix) and their length in pairs of k-blocks
    int tiles_per_xcd, blocks_per_xcd;            // units (tile, split) per XCD, resident blocks per XCD
    int cut_tail;       // 1: the tail's K loops are cut evenly over the blocks; 0: every tail tile is one block's
    int slots_per_xcd;  // parked pieces an XCD may hold (sk_decomp.h)
    float* frag;        // [xcd][slots_per_xcd][BM * BN] parked accumulators, in the lanes' own order
    int* counters;      // [tiles], zero on entry and again on exit
};

template <int BM, int BN, int NS, int KIND>
__global__ __launch_bounds__(256) void gemm_sk_kernel(SkParams sp) {
    const GemmParams& p = sp.g;
    constexpr int NW = 4;
    constexpr int WTM = BM / 2, WTN = BN / 2;    // wavefront tile: WTM token rows x WTN weight columns
    constexpr int TM = WTM / 16, TN = WTN / 16;  // activation tiles (B operands), weight tiles (A operands)
    constexpr int NBLK = (BM + BN) / 16;         // KiB blocks per stage
    constexpr int LPW = NBLK / NW;               // copies per wavefront per stage
    constexpr int STAGE = NBLK * 1024;
    constexpr int NT = TM * TN, NR = TM + TN;
    constexpr int RSTEP = (NT * 3 / 4) / NR > 0 ? (NT * 3 / 4) / NR : 1;   // MFMAs between two operand reads
    static_assert(NBLK % NW == 0 && NS >= 3 && NS <= 5 && (NR == 8 || NR == 12 || NR == 16) && NR * RSTEP <= NT, "shape");
    static_assert(KIND != GemmOut::SWIGLU_BF16 || TN % 4 == 0, "a wavefront owns whole gate/up groups of 64 columns");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];   // NS stages, then one word for the block's verdict
    int* const s_flag = reinterpret_cast<int*>(lds + NS * STAGE);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 15, g = lane >> 4;

    // A unit is a tile's share of K: (column tile, K split, row tile), the row tile fastest.  Where the text below says
    // tile it means unit; the tail's K loops are cut only when there is one split (sp.cut_tail implies sp.splits == 1).
    const int xcd = blockIdx.x & 7, lb = blockIdx.x >> 3, B = sp.blocks_per_xcd;
    const int n_units_all = sp.tiles_m * sp.tiles_n * sp.splits;
    const int t_first = xcd * sp.tiles_per_xcd, T = min(n_units_all, t_first + sp.tiles_per_xcd) - t_first;
    if (T <= 0) return;
    const int full = T / B, R = T - full * B;
    const int KB = p.K >> 5;
    const int KP = sp.splits == 1 ? KB >> 1 : sp.kp_per_split;   // pairs of 32-wide k-blocks in a unit (the last split may have fewer)
    const int m_tiles = (p.M + 15) >> 4, n_tiles = p.N >> 4;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const uint32_t x_lane = lds0 + (wm * TM) * 1024 + lane * 16;                // activation tiles of this wavefront
    const uint32_t w_lane = lds0 + (BM / 16 + wn * TN) * 1024 + lane * 16;      // weight tiles
    typedef OpSet<NR> Ops;   // v[0..TN) weight tiles (A operands), v[TN..NR) activation tiles (B operands)

    // the block's work: `full` whole tiles, then its run [it, it_end) of the XCD's tail, counted in pairs of k-blocks.
    // The tail is cut over Bt <= B blocks, fewer where the runs would get too short to be worth their parked pieces;
    // Bt <= R * KP, so no run is empty.
    // With cut_tail off the tail is not cut: Bt = R, every run is one whole tile and nothing is parked.
    const int Bt = R > 0 ? (sp.cut_tail ? sk_tail_blocks(B, R, KP) : R) : 0;
    int it = lb < Bt ? sk_run_begin(lb, Bt, R, KP) : 0;
    const int it_end = lb < Bt ? sk_run_begin(lb + 1, Bt, R, KP) : 0;
    // The tail comes first: its parked pieces are then added up while the other blocks are already at their whole
    // tiles, instead of at the very end with every block waiting.
    for (int w = 0;;) {
        int tile, kp0, kp1;
        if (it < it_end) {
            const int rt = it / KP;
            tile = t_first + full * B + rt;
            kp0 = it - rt * KP;
            kp1 = min(KP, it_end - rt * KP);
            it = rt * KP + kp1;
        } else {
            if (w >= full) break;
            tile = t_first + w * B + lb; kp0 = 0; kp1 = KP;
            w++;
        }
        const int tm = tile % sp.tiles_m, rest = tile / sp.tiles_m;
        const int split = rest % sp.splits, tn = rest / sp.splits;
        const int m0 = tm * BM, n0 = tn * BN;
        const int KPu = min(KB >> 1, (split + 1) * KP) - split * KP;   // this unit's pairs
        kp1 = min(kp1, KPu);
        const int kb0 = 2 * (split * KP + kp0), n_kb = 2 * (kp1 - kp0);

        // this wavefront's LPW blocks of a stage (block b = wave + NW i): byte offsets from A / Wp, < 4 GiB
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
            const uint8_t* gp = b < BM / 16 ? gA + (size_t)s * 1024 : gW + (size_t)s * 4096;
            PS_GLOBAL_TO_LDS(gp + off[i], lds + slot * STAGE + b * 1024);
        };

        f32x4_t acc[TN][TM];
#pragma unroll
        for (int i = 0; i < TN; i++)
#pragma unroll
            for (int j = 0; j < TM; j++) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        // the zeroing stays up here, a prologue away from the first matrix instruction that reads it (the compiler
        // sees no hazard between a register write and the assembly that follows)
        __builtin_amdgcn_sched_barrier(0);

        auto read_op = [&](Ops& o, int q, uint32_t xb, uint32_t wb) {
            if (q < TN) o.v[q] = lds_read16(wb, q * 1024);
            else o.v[q] = lds_read16(xb, (q - TN) * 1024);
        };
        // One stage: NT MFMAs on `cur`; the reads of the next stage (slot `rslot`) into `nxt`; the copies of stage
        // `s_load` into slot `lslot`.  The scheduling barriers keep the written order.
        auto stage = [&](Ops& cur, Ops& nxt, int rslot, int s_load, int lslot) {
            const uint32_t xb = x_lane + rslot * STAGE, wb = w_lane + rslot * STAGE;
#pragma unroll
            for (int t = 0; t < NT; t++) {
                const int i = t / TM, j = t % TM;
                mfma16_acc(acc[i][j], cur.v[i], cur.v[TN + j]);
                if (t % RSTEP == 0 && t / RSTEP < NR) read_op(nxt, t / RSTEP, xb, wb);
#pragma unroll
                for (int l = 0; l < LPW; l++)
                    if (t == (l + 1) * NT / (LPW + 1)) issue_one(l, s_load, lslot);
                __builtin_amdgcn_sched_barrier(0);
            }
            lgkm0_tie(nxt);
            __builtin_amdgcn_sched_barrier(0);
        };

        // Every wavefront is done with the previous tile's stages and with what its epilogue kept in the ring.
        __builtin_amdgcn_s_barrier();
        // NS slots, NS-1 stages in flight.  Copies past the last stage fetch the last stage again, into a slot
        // that nobody reads any more: the loop body is the same every time and the wait counts are constants.
#pragma unroll
        for (int s = 0; s < NS - 1; s++)
#pragma unroll
            for (int i = 0; i < LPW; i++) issue_one(i, min(s, n_kb - 1), s);
        vm_wait<(NS - 2) * LPW>();
        __builtin_amdgcn_s_barrier();
        Ops o0, o1;
#pragma unroll
        for (int q = 0; q < NR; q++) read_op(o0, q, x_lane, w_lane);
        lgkm0_tie(o0);
        __builtin_amdgcn_sched_barrier(0);
        int slot = 0;
        // Top of stage s: once every wavefront is past the barrier, stage s+1 has landed for all of them, and all of
        // them have read stage s (into registers, before the end of stage s-1) and stage s-1, whose slot the copies
        // of stage s+NS-1 overwrite.
#define PS_STAGE16(CUR, NXT, S)                                            \
        {                                                                  \
            vm_wait<(NS - 3) * LPW>();                                     \
            __builtin_amdgcn_s_barrier();                                  \
            const int next_ = slot + 1 == NS ? 0 : slot + 1;               \
            const int prev_ = slot == 0 ? NS - 1 : slot - 1;               \
            __builtin_amdgcn_sched_barrier(0);                             \
            stage(CUR, NXT, next_, min((S) + NS - 1, n_kb - 1), prev_);    \
            slot = next_;                                                  \
        }
        for (int s = 0; s < n_kb; s += 2) {   // n_kb is even: runs are counted in pairs of k-blocks
            PS_STAGE16(o0, o1, s)
            PS_STAGE16(o1, o0, s + 1)
        }
#undef PS_STAGE16
        vm_wait<0>();
        // the last matrix instructions have written their accumulators before anything reads them
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);

        // lane (r, g) holds, of tile (i, j): row m = 16 j + r, columns n = 16 i + 4 g + 0..3
        const bool whole = kp0 == 0 && kp1 == KPu;
        if (whole) {
            if constexpr (KIND == GemmOut::SWIGLU_BF16) {
                // weight tiles 4q, 4q+1 = gate and 4q+2, 4q+3 = up of the same 32 features: the pair sits in the same
                // lane.  The accumulators live in the accumulation registers, which the vector ALU cannot read; asking
                // the compiler for copies makes it spill inside the main loop.  So each lane parks one activation
                // tile's TN accumulators in its own 16 bytes of TN KiB blocks of the (now free) stage ring -- LDS
                // stores take accumulation registers as data -- and reads them back into vector registers: no other
                // lane is involved, no barrier is needed.
                const int F = p.N >> 1;
                bf16_t* out = static_cast<bf16_t*>(p.out);
                __builtin_amdgcn_s_barrier();   // every wavefront has read its last stage
                const uint32_t park = lds0 + wave * (TN * 1024) + lane * 16;
#pragma unroll
                for (int j = 0; j < TM; j++) {
                    const int m = m0 + wm * WTM + 16 * j + r;   // rows past M are stored too: the buffer holds whole row tiles
#pragma unroll
                    for (int i = 0; i < TN; i++) asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(park), "a"(acc[i][j]), "n"(i * 1024) : "memory");
                    OpSet<TN> v;
#pragma unroll
                    for (int i = 0; i < TN; i++) v.v[i] = lds_read16(park, i * 1024);
                    lgkm0_tie(v);
#pragma unroll
                    for (int q = 0; q < TN / 4; q++) {
                        const int nb = n0 + wn * WTN + 64 * q;
                        if (nb >= p.N) continue;
#pragma unroll
                        for (int h = 0; h < 2; h++) {
                            const f32x4_t ga = __builtin_bit_cast(f32x4_t, v.v[4 * q + h]), up = __builtin_bit_cast(f32x4_t, v.v[4 * q + 2 + h]);
                            uint2 o;
                            o.x = pack_bf16(silu_f(ga[0]) * up[0], silu_f(ga[1]) * up[1]);
                            o.y = pack_bf16(silu_f(ga[2]) * up[2], silu_f(ga[3]) * up[3]);
                            *reinterpret_cast<uint2*>(out + act_offset(m, (nb >> 1) + 16 * h + 4 * g, F)) = o;
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                float* out = static_cast<float*>(p.out) + (size_t)split * p.M * p.N;
#pragma unroll
                for (int j = 0; j < TM; j++) {
                    const int m = m0 + wm * WTM + 16 * j + r;
#pragma unroll
                    for (int i = 0; i < TN; i++) {
                        const int n = n0 + wn * WTN + 16 * i + 4 * g;
                        // straight from the accumulation registers (stores take them as data)
                        if (m < p.M && n < p.N) asm volatile("global_store_dwordx4 %0, %1, off" : : "v"(out + (size_t)m * p.N + n), "a"(acc[i][j]) : "memory");
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            continue;
        }

        // Part of the tile's K range.  Park the accumulators: piece (i, j) of wavefront `wave` at
        // [slot][wave][i * TM + j][lane] as a float4 (stores take accumulation registers as data).
        const size_t slot_floats = (size_t)BM * BN;
        const int rt = tile - (t_first + full * B);
        // piece (block lb, tail tile rt) -> slot lb + rt: a block's two pieces lie in consecutive tiles, and the next
        // block begins in its last tile or the one after, so the indices never collide
        float* const my_slot = sp.frag + ((size_t)xcd * sp.slots_per_xcd + sk_slot(lb, rt)) * slot_floats;
        {
            float* fp = my_slot + ((size_t)wave * NT * 64 + lane) * 4;
#pragma unroll
            for (int i = 0; i < TN; i++)
#pragma unroll
                for (int j = 0; j < TM; j++) {
                    float* q = fp + (size_t)(i * TM + j) * 256;
                    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(q), "a"(acc[i][j]) : "memory");
                }
        }
        // the runs that share this tile: blocks first_lb .. last_lb of this XCD, in the order of their K ranges
        const int first_lb = sk_first_block(rt, Bt, R, KP), last_lb = sk_last_block(rt, Bt, R, KP);
        // The pieces are exchanged with device-scope (sc1) stores and loads: written through to memory, read around
        // whatever an XCD's L2 may hold.  A device-scope fence would do as well, but it writes back and invalidates the
        // whole L2 of the XCD each time, and the 31 other blocks there lose their operand panels with it.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's pieces have been written through
        __syncthreads();                                    // ... and every thread's
        if (threadIdx.x == 0) {
            const int old = __hip_atomic_fetch_add(sp.counters + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *s_flag = old == last_lb - first_lb;
        }
        __syncthreads();
        const bool last = *s_flag != 0;
        if (!last) continue;
        if (threadIdx.x == 0) sp.counters[tile] = 0;   // clean for the next launch
        const int n_runs = last_lb - first_lb + 1;
        auto piece_of = [&](int c) -> const float* {
            return sp.frag + ((size_t)xcd * sp.slots_per_xcd + sk_slot(first_lb + c, rt)) * slot_floats + ((size_t)wave * NT * 64 + lane) * 4;
        };
#pragma unroll
        for (int j = 0; j < TM; j++) {
            const int m = m0 + wm * WTM + 16 * j + r;
            float4 sum[TN];
#pragma unroll
            for (int i = 0; i < TN; i++) sum[i] = float4{0.f, 0.f, 0.f, 0.f};
            for (int c = 0; c < n_runs; c += 2) {   // two runs' loads in flight at a time; always added in run order
                const bool two = c + 1 < n_runs;
                const float* q0 = piece_of(c);
                const float* q1 = piece_of(two ? c + 1 : c);
                OpSet<TN> v0, v1;
#pragma unroll
                for (int i = 0; i < TN; i++) asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v0.v[i]) : "v"(q0 + (size_t)(i * TM + j) * 256) : "memory");
#pragma unroll
                for (int i = 0; i < TN; i++) asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v1.v[i]) : "v"(q1 + (size_t)(i * TM + j) * 256) : "memory");
                vm0_tie(v0);
                vm0_tie(v1);
#pragma unroll
                for (int i = 0; i < TN; i++) {
                    const f32x4_t f = __builtin_bit_cast(f32x4_t, v0.v[i]);
                    sum[i].x += f[0]; sum[i].y += f[1]; sum[i].z += f[2]; sum[i].w += f[3];
                }
                if (two) {
#pragma unroll
                    for (int i = 0; i < TN; i++) {
                        const f32x4_t f = __builtin_bit_cast(f32x4_t, v1.v[i]);
                        sum[i].x += f[0]; sum[i].y += f[1]; sum[i].z += f[2]; sum[i].w += f[3];
                    }
                }
            }
            if constexpr (KIND == GemmOut::SWIGLU_BF16) {
                const int F = p.N >> 1;
                bf16_t* out = static_cast<bf16_t*>(p.out);
#pragma unroll
                for (int q = 0; q < TN / 4; q++) {
                    const int nb = n0 + wn * WTN + 64 * q;
                    if (nb >= p.N) continue;
#pragma unroll
                    for (int h = 0; h < 2; h++) {
                        const float4 ga = sum[4 * q + h], up = sum[4 * q + 2 + h];
                        uint2 o;
                        o.x = pack_bf16(silu_f(ga.x) * up.x, silu_f(ga.y) * up.y);
                        o.y = pack_bf16(silu_f(ga.z) * up.z, silu_f(ga.w) * up.w);
                        *reinterpret_cast<uint2*>(out + act_offset(m, (nb >> 1) + 16 * h + 4 * g, F)) = o;
                    }
                }
            } else {
                float* out = static_cast<float*>(p.out);
#pragma unroll
                for (int i = 0; i < TN; i++) {
                    const int n = n0 + wn * WTN + 16 * i + 4 * g;
                    if (m < p.M && n < p.N) *reinterpret_cast<float4*>(out + (size_t)m * p.N + n) = sum[i];
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Planning and launch
// ------------------------------------------------------------------------------------------
struct GemmPlan {
    bool wstream;
    bool big_tile;      // tiled: 256x256 blocks (else 128x128)
    int splits;         // partial buffers written
    int kb_per_split;   // 32-wide k-blocks per split
    bool cut_tail;      // tiled: cut the K loops of the last, partial wave of tiles over the blocks (one split only)
    int slots_per_xcd;  // tiled: parked pieces an XCD may hold
};

static int device_cus() {
    static int cus = 0;
    static std::once_flag once;
    std::call_once(once, [] {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        cus = (cus + 7) / 8 * 8;
    });
    return cus;
}

// Estimated time (us) of the tiled kernel for one choice of tile edge, K splits and tail cutting, from the rates measured
// on the layer shapes: a block takes about 1.4 us (0.9 us for a 128x128 tile, two of which share a compute unit) per pair
// of k-blocks plus a fixed prologue and epilogue per unit; blocks take units in waves; every split beyond the first is
// written and read back by the consumer; parked pieces of a cut tail cost about 1.4 us per MB all told (store, count,
// reload by the last block and the clock the extra traffic costs the rest of the step: measured on the gate/up and O
// matrices), less where whole tiles follow to hide them behind.
static double tiled_estimate(int M, int N, int K, int edge, int splits, bool cut, int* kp_per_split, int* eff_splits, int* slots_per_xcd) {
    const int B = device_cus() * (edge == 256 ? 1 : 2) / 8;
    const int KPt = K / 64;
    const int kps = (KPt + splits - 1) / splits, s_eff = (KPt + kps - 1) / kps;
    const int tiles = ((M + edge - 1) / edge) * ((N + edge - 1) / edge), units = tiles * s_eff;
    const int upx = (units + 7) / 8;
    const double t_pair = edge == 256 ? 1.4 : 0.9, t_fix = edge == 256 ? 8.0 : 4.0;
    const double unit_us = kps * t_pair + t_fix;
    double waves = 0, waves_uncut = 0;
    int slots = 0, pieces = 0;
    bool any_full = false;
    for (int x = 0; x < 8; x++) {
        const int T = std::min(units, (x + 1) * upx) - x * upx;
        if (T <= 0) break;
        const int full = T / B, R = T % B;
        any_full |= full > 0;
        waves_uncut = std::max(waves_uncut, (double)full + (R > 0));
        if (!cut || R == 0) { waves = std::max(waves, (double)full + (R > 0)); continue; }
        const int Bt = sk_tail_blocks(B, R, kps);
        waves = std::max(waves, full + (double)R / Bt);
        slots = std::max(slots, sk_slots(Bt, R));
        pieces += Bt > R ? sk_slots(Bt, R) : 0;
    }
    *kp_per_split = kps;
    *eff_splits = s_eff;
    *slots_per_xcd = slots;
    // With 256x256 tiles on every compute unit the device runs at its power limit, and compute units left idle by an
    // uncut tail give part of their share back as clock for the busy ones: measured on the 70B-shaped gate/up matrix,
    // cutting the tail of 4.4 waves bought nothing, where the arithmetic says 11 %.  Half the gain is what is counted.
    if (cut && edge == 256) waves = waves_uncut - 0.5 * (waves_uncut - waves);
    double us = waves * unit_us;
    if (s_eff > 1) us += 2.0 * (s_eff - 1) * (double)M * N * 4 / 3e6;
    if (cut) us += pieces * (double)edge * edge * 4 / 0.7e6 * (any_full ? 0.6 : 1.0) + 10.0;
    return us;
}

static GemmPlan plan_gemm(int M, int N, int K, int kind, int split_opt, int tile_opt, int sk_mode = 0) {
    GemmPlan g;
    // measured: streaming wins up to 96 tokens for every projection, and up to 160 (ten row tiles) for all but the QKV-shaped
    // one (more columns than rows of weights: 48 blocks per split and six splits of partial sums; 129 tokens: 29 vs 24 us),
    // above all for the gate/up matrix (129 tokens: 61 vs 75 us) and the down projection (42 vs 46)
    g.wstream = M <= 64 || (tile_opt == 0 && (M <= 96 || (M <= 160 && (kind == GemmOut::SWIGLU_BF16 || N <= K))));
    g.big_tile = false;
    g.splits = 1;
    g.kb_per_split = K / 32;
    g.cut_tail = false;
    g.slots_per_xcd = 0;
    if (g.wstream) {
        const int groups = N / 64, KB = K / 32;
        int s = 1;
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
        // every combination of tile edge, K splits (none for the gate/up matrix, whose epilogue is not linear) and, for
        // one split, tail cutting; the smallest estimate wins
        const int s_lo = kind == GemmOut::SWIGLU_BF16 ? 1 : (split_opt > 0 ? std::min(split_opt, 8) : 1);
        const int s_hi = kind == GemmOut::SWIGLU_BF16 ? 1 : (split_opt > 0 ? s_lo : 8);
        double best = 0;
        bool first = true;
        for (int edge : {128, 256}) {
            if ((tile_opt == 128 || tile_opt == 256) && edge != tile_opt) continue;
            for (int sp = s_lo; sp <= s_hi; sp++)
                for (int cut = 0; cut < (sp == 1 && sk_mode != 1 ? 2 : 1); cut++) {
                    int kps, eff, slots;
                    double us = tiled_estimate(M, N, K, edge, sp, cut != 0, &kps, &eff, &slots);
                    if (cut && slots == 0) continue;
                    if (cut && sk_mode == 2) us -= 1e9;   // test knob: a tail that can be cut is cut
                    if (first || us < best) {
                        first = false; best = us;
                        g.big_tile = edge == 256; g.splits = eff; g.kb_per_split = 2 * kps; g.cut_tail = cut != 0; g.slots_per_xcd = slots;
                    }
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

void gemm_workspace(int M, int N, int K, int kind, int split_opt, int tile_opt, int sk_mode, size_t* frag_bytes, int* n_counters) {
    *frag_bytes = 0;
    *n_counters = 0;
    if (M <= 0) return;
    const GemmPlan g = plan_gemm(M, N, K, kind, split_opt, tile_opt, sk_mode);
    if (g.wstream) return;
    const int b = g.big_tile ? 256 : 128;
    *frag_bytes = (size_t)8 * g.slots_per_xcd * b * b * sizeof(float);
    *n_counters = ((M + b - 1) / b) * ((N + b - 1) / b);
}

template <int BM, int BN, int NS, int KIND>
static hipError_t launch_sk(const GemmParams& p, const GemmArgs& a, const GemmPlan& g, hipStream_t st) {
    constexpr int lds_bytes = (BM + BN) / 16 * 1024 * NS + 16;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {   // more dynamic LDS than the default limit: raise it once per kernel
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_sk_kernel<BM, BN, NS, KIND>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    });
    if (attr_err != hipSuccess) return attr_err;
    SkParams sp;
    sp.g = p;
    sp.tiles_m = (p.M + BM - 1) / BM;
    sp.tiles_n = (p.N + BN - 1) / BN;
    sp.splits = g.splits;
    sp.kp_per_split = g.kb_per_split / 2;
    const int tiles = sp.tiles_m * sp.tiles_n;
    sp.tiles_per_xcd = (tiles * g.splits + 7) / 8;
    const int blocks = device_cus() * (BM == 256 ? 1 : 2);   // resident at once: one 256x256 block or two 128x128 blocks per CU
    sp.blocks_per_xcd = blocks / 8;
    sp.cut_tail = g.cut_tail ? 1 : 0;
    sp.slots_per_xcd = g.slots_per_xcd;
    sp.frag = a.sk_frag;
    sp.counters = a.sk_counters;
    if (g.cut_tail && ((size_t)8 * sp.slots_per_xcd * BM * BN * sizeof(float) > a.sk_frag_bytes || tiles > a.sk_n_counters || !a.sk_counters || !a.sk_frag || g.splits != 1))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_sk_kernel<BM, BN, NS, KIND>), dim3(blocks), dim3(256), lds_bytes, st, sp);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, int* n_splits, hipStream_t st) {
    if (n_splits) *n_splits = 1;
    if (a.M <= 0) return hipSuccess;
    if (a.N % 64 || a.K % 64) return hipErrorInvalidValue;
    // the tiled kernel addresses A and Wp with 32-bit byte offsets
    if (a.M > 64 && ((size_t)a.N * a.K * 2 >= (1ull << 32) || (size_t)((a.M + 15) / 16 * 16) * a.K * 2 >= (1ull << 32)))
        return hipErrorInvalidValue;
    const GemmPlan g = plan_gemm(a.M, a.N, a.K, a.kind, a.split_k, a.tile, a.sk_mode);
    if ((size_t)g.splits * (a.kind == GemmOut::SWIGLU_BF16 ? 0 : (size_t)a.M * a.N * sizeof(float)) > a.out_bytes ||
        gemm_out_bytes(a.M, a.N, a.K, a.kind, a.split_k, a.tile) > a.out_bytes)
        return hipErrorInvalidValue;
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
        return g.big_tile ? launch_sk<256, 256, 4, GemmOut::SWIGLU_BF16>(p, a, g, st) : launch_sk<128, 128, 4, GemmOut::SWIGLU_BF16>(p, a, g, st);
    return g.big_tile ? launch_sk<256, 256, 4, GemmOut::PARTIAL_F32>(p, a, g, st) : launch_sk<128, 128, 4, GemmOut::PARTIAL_F32>(p, a, g, st);
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
