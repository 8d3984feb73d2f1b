// Helpers shared by the fused attention kernels: tile counting, LDS swizzle and
// the lane offsets of the global-to-LDS copy of K / V^T tiles.
#pragma once

#include "mfma_common.h"

namespace attnring {

constexpr int BC = 64;  // keys per staged tile

struct CountCfg {
    int b;        // rows per logical PE
    int b_shift;  // log2(b), or -1 when b is not a power of two
};

// ceil(x / b): the number of multiples of b in [0, x)
__device__ __forceinline__ unsigned cdiv_b(unsigned x, const CountCfg& cc)
{
    const unsigned y = x + (unsigned)cc.b - 1u;
    return cc.b_shift >= 0 ? (y >> cc.b_shift) : y / (unsigned)cc.b;
}
__device__ __forceinline__ bool is_multiple(int x, const CountCfg& cc)
{
    return cc.b_shift >= 0 ? (x & (cc.b - 1)) == 0 : (x % cc.b) == 0;
}

// Swizzled chunk position inside an LDS row of ROWB bytes (256 or 128).
template <int ROWB>
__device__ __forceinline__ int swz(int chunk, int row)
{
    return ROWB == 256 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
}

// One wavefront copies 1 KiB pieces of a [rows][ROWB] tile from global memory to
// LDS: piece m holds rows m*RPP .. ; lane L lands at byte 16*L of the piece and
// fetches the chunk that belongs there under the swizzle.  With the pieces of a
// wavefront 4 or 8 apart, the lane's byte offset inside its piece does not depend
// on the piece, so it is computed once (dma_lane_offset) and every copy is a
// uniform base (buffer descriptor and scalar offset) plus that offset.
template <int ROWB>
__device__ __forceinline__ unsigned dma_lane_offset(int first, int lane)
{
    constexpr int CPR = ROWB / 16;  // chunks per row
    constexpr int RPP = 64 / CPR;   // rows per piece
    const int rl = lane / CPR, p = lane % CPR;
    const int row = first * RPP + rl;
    return (unsigned)(rl * ROWB + swz<ROWB>(p, row) * 16);
}

}  // namespace attnring
