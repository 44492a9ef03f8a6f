// Device-side map from a workgroup id to its (expert, n-tile, m-tile) for the grouped expert
// GEMMs.  m-tiles never straddle experts; the map is computed from expert_offsets on the
// device so that no host read-back sits between the permutation and the GEMM.
//
// XCD awareness: the hardware deals workgroup ids round-robin to the 8 accelerator dies
// (id % 8), each with its own L2.  Logical tiles are ordered expert-major, then n-tile, then
// m-tile, and die x takes the x-th contiguous eighth of that order: the m-tiles that share a
// weight tile, and the n-tiles that share an activation tile, run on one die at about the
// same time and meet in its L2.
#pragma once
#include "common.h"

namespace specmoe {

struct TileLoc {
    int expert;      // expert id
    int row0;        // first row of the tile in the permuted row space
    int tile_rows;   // valid rows in the tile (1 .. BM)
    int nt;          // n-tile index
    int blk0;        // 16-row blocks in front of the tile when every expert's rows are padded to
                     // a whole number of blocks (row numbering of the tile-packed matrices)
    int mt;          // m-tiles of the tile's expert (1: its weight tiles are read by one workgroup)
};

// Even split: an expert with M rows gets ceil(M / BM_MAX) m-tiles of equal height (rounded up
// to the row granule of the matrix instruction in use, 32 or 16), so no tile is a thin
// remainder that would stream a whole weight tile for a handful of rows.
struct EvenSplit {
    int mt;    // m-tiles of the expert
    int rpt;   // rows per tile (multiple of GRAN, <= BM_MAX); the last tile may hold fewer
};
template <int BM_MAX, int GRAN>
__device__ __forceinline__ EvenSplit even_split(int M) {
    EvenSplit s{0, 0};
    if (M <= 0) return s;
    const int mt0 = (M + BM_MAX - 1) / BM_MAX;
    s.rpt = ((M + mt0 - 1) / mt0 + GRAN - 1) / GRAN * GRAN;
    s.mt = (M + s.rpt - 1) / s.rpt;
    return s;
}

// GRAN = row granule of the matrix instruction in use (32 or 16).
// Wave-parallel: lane e works out expert e's split (64 experts per sweep), the running tile
// count comes from a wave scan, and the owning expert is the first lane whose range reaches the
// tile index.  Every wave of the workgroup calls this with all 64 lanes active and gets the same
// answer; a scalar walk over the experts costs several microseconds of integer divisions per
// workgroup, this one memory round trip and ~100 vector instructions.
template <int BM_MAX, int GRAN>
struct EvenPolicy {
    __device__ __forceinline__ static EvenSplit of(int M) { return even_split<BM_MAX, GRAN>(M); }
};
// fixed tile height BM: ceil(M / BM) tiles, the last one ragged
template <int BM>
struct FixedPolicy {
    __device__ __forceinline__ static EvenSplit of(int M) {
        EvenSplit s{0, BM};
        if (M > 0) s.mt = (M + BM - 1) / BM;
        return s;
    }
};

template <typename Split>
__device__ __forceinline__ bool locate_tile_impl(const int32_t* __restrict__ offsets, int E,
                                                 int NT, unsigned block_id, TileLoc& t) {
    const int lane = threadIdx.x % kWave;
    int total_mt = 0;
    for (int e0 = 0; e0 < E; e0 += kWave) {
        const int e = e0 + lane;
        const int M = e < E ? offsets[e + 1] - offsets[e] : 0;
        total_mt += wave_sum(Split::of(M).mt);
    }
    const long long G = (long long)total_mt * NT;
    const long long per_xcd = (G + kXcds - 1) / kXcds;
    const long long slot = block_id / kXcds;
    const long long L = (long long)(block_id % kXcds) * per_xcd + slot;
    if (slot >= per_xcd || L >= G) return false;
    int base_mt = 0;                              // m-tiles of the experts before this sweep
    int base_blk = 0;                             // 16-row blocks of the experts before this sweep
    int expert = -1, row0 = 0, rows = 0, nt = 0, blk0 = 0, mts = 0;
    for (int e0 = 0; e0 < E && expert < 0; e0 += kWave) {
        const int e = e0 + lane;
        const int lo = e < E ? offsets[e] : 0, hi = e < E ? offsets[e + 1] : 0;
        const EvenSplit sp = Split::of(hi - lo);
        const int nblk = (hi - lo + 15) / 16;
        int incl = sp.mt, incl_blk = nblk;        // inclusive scans over the lanes
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int v = __shfl_up(incl, off, kWave);
            const int vb = __shfl_up(incl_blk, off, kWave);
            if (lane >= off) { incl += v; incl_blk += vb; }
        }
        const long long end = (long long)(base_mt + incl) * NT;      // tiles up to and incl. e
        const unsigned long long hit = __ballot(sp.mt > 0 && L < end);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;              // first such expert
            const int mt = __shfl(sp.mt, src, kWave), rpt = __shfl(sp.rpt, src, kWave);
            const int excl = __shfl(incl, src, kWave) - mt;
            const int lo_s = __shfl(lo, src, kWave), hi_s = __shfl(hi, src, kWave);
            const long long rem = L - (long long)(base_mt + excl) * NT;
            nt = (int)(rem / mt);
            const int mi = (int)(rem - (long long)nt * mt);
            expert = e0 + src;
            mts = mt;
            row0 = lo_s + mi * rpt;
            rows = min(rpt, hi_s - row0);
            blk0 = base_blk + __shfl(incl_blk, src, kWave) - __shfl(nblk, src, kWave) +
                   mi * rpt / 16;                 // tile heights are multiples of 16
        }
        base_mt += __shfl(incl, kWave - 1, kWave);
        base_blk += __shfl(incl_blk, kWave - 1, kWave);
    }
    // the values are the same in every lane; say so to the compiler (scalar registers)
    t.expert = __builtin_amdgcn_readfirstlane(expert);
    t.row0 = __builtin_amdgcn_readfirstlane(row0);
    t.tile_rows = __builtin_amdgcn_readfirstlane(rows);
    t.nt = __builtin_amdgcn_readfirstlane(nt);
    t.blk0 = __builtin_amdgcn_readfirstlane(blk0);
    t.mt = __builtin_amdgcn_readfirstlane(mts);
    return t.expert >= 0;
}

template <int BM_MAX, int GRAN = 32>
__device__ __forceinline__ bool locate_tile_even(const int32_t* __restrict__ offsets, int E,
                                                 int NT, unsigned block_id, TileLoc& t) {
    return locate_tile_impl<EvenPolicy<BM_MAX, GRAN>>(offsets, E, NT, block_id, t);
}
template <int BM>
__device__ __forceinline__ bool locate_tile(const int32_t* __restrict__ offsets, int E, int NT,
                                            unsigned block_id, TileLoc& t) {
    return locate_tile_impl<FixedPolicy<BM>>(offsets, E, NT, block_id, t);
}

// Upper bound of the grid (host side): sum_e ceil(M_e/BM) <= floor(n_rows/BM) + E.
inline long long grid_upper_bound(int n_rows, int E, int BM, long long NT) {
    long long g = ((long long)(n_rows / BM) + E) * NT;
    return (g + kXcds - 1) / kXcds * kXcds;
}

}  // namespace specmoe
