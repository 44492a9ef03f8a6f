// Re-layout of a row-major bf16 matrix into the tile-packed form the large-batch expert GEMMs
// read with 1 KB wave-loads (layout: pipe_common.h).  One-time work per weight matrix
// (SpecMoE keeps the experts' parameters fixed during inference, Sec. 2.1), or per batch for
// an activation matrix.
#include "pipe_common.h"

namespace specmoe {
namespace {

// one thread per 16-byte piece of the output
__global__ __launch_bounds__(256) void pack_tiles_kernel(const U128* __restrict__ src,
                                                         U128* __restrict__ dst,
                                                         long long n_pieces, int K) {
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= n_pieces) return;
    const long long blk = g >> 6;
    const int piece = (int)(g & 63);
    const int r = piece >> 2, c = (piece & 3) ^ ((r >> 1) & 3);
    const int kblocks = K / pipe::kPackCols;
    const long long rb = blk / kblocks;
    const int kb = (int)(blk - rb * kblocks);
    // source: row rb*16 + r, columns kb*32 + c*8 .. +7  (16 bytes = 8 elements; K/8 pieces per row)
    dst[g] = src[(rb * 16 + r) * (long long)(K / 8) + kb * 4 + c];
}

// Gather + pack of the activation rows: row block b of the output (numbering: every expert's rows
// padded to whole 16-row blocks, experts in order) holds rows 16*lb .. 16*lb+15 of its expert,
// row r of the permuted order being x[row_src[r] / k]; rows beyond the expert's last row are zeros.
// Workgroup (b, s) writes k-blocks [s * kPackSeg, (s+1) * kPackSeg) of row block b; the block's
// expert is found with a wave scan over expert_offsets.  A thread keeps one piece position
// (row r, chunk c) of the 1 KB blocks for the whole segment, so it reads its source row index once.
constexpr int kPackSeg = 16;                      // k-blocks (1 KB each) per workgroup

__global__ __launch_bounds__(256) void gather_pack_rows_kernel(
    const U128* __restrict__ x, const int32_t* __restrict__ row_src, int topk,
    const int32_t* __restrict__ offsets, int E, int K, U128* __restrict__ dst) {
    // every wave works the block's expert out for itself (same answer): no LDS, no barrier
    const int lane = threadIdx.x % kWave;
    int base = 0, row0 = -1, rows = 0;
    for (int e0 = 0; e0 < E && row0 < 0; e0 += kWave) {
        const int e = e0 + lane;
        const int lo = e < E ? offsets[e] : 0, hi = e < E ? offsets[e + 1] : 0;
        const int nblk = (hi - lo + 15) / 16;
        int incl = nblk;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int v = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += v;
        }
        const unsigned long long hit = __ballot(nblk > 0 && (int)blockIdx.x < base + incl);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            const int lb =
                (int)blockIdx.x - (base + __shfl(incl, src, kWave) - __shfl(nblk, src, kWave));
            row0 = __shfl(lo, src, kWave) + lb * 16;
            rows = min(16, __shfl(hi, src, kWave) - row0);
        }
        base += __shfl(incl, kWave - 1, kWave);
    }
    if (row0 < 0) return;                         // beyond the last block in use
    const int kblocks = K / pipe::kPackCols;
    const int kb0 = blockIdx.y * kPackSeg, kb1 = min(kb0 + kPackSeg, kblocks);
    const int piece = lane, r = piece >> 2, c = (piece & 3) ^ ((r >> 1) & 3);
    const bool live = r < rows;
    size_t srow = 0;
    if (live) srow = row_src ? (size_t)(row_src[row0 + r] / topk) : (size_t)(row0 + r);
    const U128* in = x + srow * (size_t)(K / 8) + c;
    U128* out = dst + (size_t)blockIdx.x * kblocks * 64 + piece;
    const U128 zero = {0, 0, 0, 0};
#pragma unroll 4
    for (int kb = kb0 + (int)(threadIdx.x / kWave); kb < kb1; kb += 4)
        out[(size_t)kb * 64] = live ? in[kb * 4] : zero;
}

}  // namespace

hipError_t launch_gather_pack_rows(const bf16_t* x, const int32_t* row_src, int topk,
                                   const int32_t* offsets, int n_rows, int E, int K,
                                   bf16_t* dst, hipStream_t s) {
    const int max_blocks = n_rows / 16 + E;       // sum_e ceil(M_e / 16) <= n_rows / 16 + E
    const int segs = (K / pipe::kPackCols + kPackSeg - 1) / kPackSeg;
    hipLaunchKernelGGL(gather_pack_rows_kernel, dim3((unsigned)max_blocks, (unsigned)segs),
                       dim3(256), 0, s,
                       reinterpret_cast<const U128*>(x), row_src, topk, offsets, E, K,
                       reinterpret_cast<U128*>(dst));
    return hipGetLastError();
}

hipError_t launch_pack_tiles(const bf16_t* src, long long rows, int K, bf16_t* dst, hipStream_t s) {
    const long long n_pieces = rows * (long long)K / 8;
    if (n_pieces == 0) return hipSuccess;
    const long long grid = (n_pieces + 255) / 256;
    hipLaunchKernelGGL(pack_tiles_kernel, dim3((unsigned)grid), dim3(256), 0, s,
                       reinterpret_cast<const U128*>(src), reinterpret_cast<U128*>(dst), n_pieces, K);
    return hipGetLastError();
}

}  // namespace specmoe
