// Integer side of the tiled GEMM's work decomposition (host and device): how the K loops of the tiles that do not
// fill a wave of blocks are cut into runs, which blocks share a tile, and where a run parks its accumulators.
// Units: B blocks of an XCD, R < B tail tiles, KP pairs of 32-wide k-blocks per tile; the tail is the interval
// [0, R * KP) of pairs, tile rt owning [rt * KP, (rt + 1) * KP).
#pragma once

namespace ps {

// A run shorter than this many pairs (1024 of K) is not worth a block of its own: its parked accumulators are as
// many bytes as the operands it reads.
constexpr int SK_MIN_RUN = 16;

// Blocks the tail is cut over: R <= Bt <= max(R, min(B, R * KP / SK_MIN_RUN)); never more than R * KP, so no run is empty.
__host__ __device__ inline int sk_tail_blocks(int B, int R, int KP) {
    const long by_len = (long)R * KP / SK_MIN_RUN;
    return (int)(by_len < R ? R : (by_len < B ? by_len : B));
}

// Run of block lb < Bt: pairs [sk_run_begin(lb), sk_run_begin(lb + 1)).
__host__ __device__ inline int sk_run_begin(int lb, int Bt, int R, int KP) { return (int)((long)lb * R * KP / Bt); }

// Blocks whose runs meet tail tile rt: first .. last, in the order of their K ranges.
__host__ __device__ inline int sk_first_block(int rt, int Bt, int R, int KP) {
    // smallest lb with run_begin(lb + 1) > rt * KP
    return (int)((((long)rt * KP + 1) * Bt + (long)R * KP - 1) / ((long)R * KP)) - 1;
}
__host__ __device__ inline int sk_last_block(int rt, int Bt, int R, int KP) {
    // largest lb with run_begin(lb) < (rt + 1) * KP
    (void)KP;
    return (int)(((long)(rt + 1) * Bt + R - 1) / R) - 1;
}

// Slot of the piece (block lb, tail tile rt) among the XCD's parked pieces.  A block's pieces lie in consecutive
// tiles and the next block begins in its last tile or the one after, so lb + rt never collides; the largest index is
// Bt + R - 2.
__host__ __device__ inline int sk_slot(int lb, int rt) { return lb + rt; }
__host__ __device__ inline int sk_slots(int Bt, int R) { return R > 0 ? Bt + R - 1 : 0; }

}  // namespace ps
