// Grouped GEMM: which expert an m-tile belongs to, found on the device from the row offsets.
#pragma once
#include "hif4_common.h"

namespace hif4 {

// Expert e owns rows [offs[e], offs[e+1]) of A and C and ceil(rows / BM) consecutive m-tiles of
// the tile list.  Finds the expert of m-tile `tile_m` and the tile's first row; every lane of
// the calling wave gets the same answer.  64 experts at a time: row counts from the offsets, an
// inclusive scan of their tile counts across the lanes, a ballot for the first lane whose
// running count passes tile_m.  Returns false when tile_m lies past the last tile (the grid of a
// grouped launch is an upper bound, the host does not know the counts).
// The offsets are the caller's: they are clamped to [0, total_rows] and an expert whose range runs
// backwards counts as empty, so that no row outside A and C is ever touched whatever they hold.
template <int BM>
__device__ __forceinline__ bool find_expert_tile(const int32_t *__restrict__ offs, int E, int total_rows, int tile_m, int lane,
                                                 int &e, int &row0, int &rows_end)
{
    for (int base = 0, acc = 0; base < E; base += 64) {
        const int ee = base + lane;
        int lo = 0, hi = 0;
        if (ee < E) {
            lo = offs[ee];
            hi = offs[ee + 1];
            lo = lo < 0 ? 0 : (lo > total_rows ? total_rows : lo);
            hi = hi < lo ? lo : (hi > total_rows ? total_rows : hi);
        }
        const int nt = (hi - lo + BM - 1) / BM;
        int incl = nt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int v = __shfl_up(incl, d, 64);
            if (lane >= d) incl += v;
        }
        const int total = __shfl(incl, 63, 64);
        if (tile_m < acc + total) {
            const int src = __ffsll((unsigned long long)__ballot(acc + incl > tile_m)) - 1;
            const int before = acc + __shfl(incl - nt, src, 64); // tiles of the experts ahead of this one
            e = __builtin_amdgcn_readfirstlane(base + src);
            row0 = __builtin_amdgcn_readfirstlane(__shfl(lo, src, 64) + (tile_m - before) * BM);
            rows_end = __builtin_amdgcn_readfirstlane(__shfl(hi, src, 64));
            return true;
        }
        acc += total;
    }
    return false;
}

} // namespace hif4
