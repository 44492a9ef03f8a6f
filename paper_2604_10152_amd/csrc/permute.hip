// Stable grouping of the (token, slot) pairs by expert and the row gather that follows it.
// (SpecMoE Fig. 2: tokens that activate the same expert are served together; Sec. 3.2: the
// per-expert activation counts of the verification pass are the differences of expert_offsets.)
//
// Index phase: ONE workgroup of 16 wavefronts (8 beyond 64 experts).  Wave w owns the w-th contiguous slice of the
// flat pair array.  (A) per-wave, per-expert counts in LDS (integer atomics: order-free);
// (B) totals -> exclusive prefix sum over experts -> each wave's first destination row per
// expert; (C) every wave walks its slice in order, 64 pairs at a time, ranks equal experts
// inside the 64 with ballots, and bumps its private LDS cursors.  Contiguous slices walked in
// order make the sort stable with no ordered atomics.  Gather phase: a coalesced 16-byte copy
// of whole rows over the full grid.
#include "common.h"

namespace specmoe {
namespace {

constexpr int kPermWavesSmallE = 16;   // E <= 64: shorter slices per wave (the walk is serial)
constexpr int kPermWavesLargeE = 8;    // (waves + 1) * E counters have to fit the LDS default
constexpr int kBatch = 8;          // index rows fetched ahead per wavefront

// SMALL_E (E <= 64): in phase (C) lane e keeps expert e's cursor in a register and the loop
// over the distinct experts of a 64-pair row uses readlane instead of an LDS read-modify-write
// chain (the chain dominated the kernel: 19 -> ~9 us at 4096 pairs).
template <bool SMALL_E>
__global__ __launch_bounds__((SMALL_E ? kPermWavesSmallE : kPermWavesLargeE) * kWave)
void permute_index_kernel(
    const int32_t* __restrict__ idx, int P, int E, int32_t* __restrict__ offsets,
    int32_t* __restrict__ row_src, int32_t* __restrict__ row_of) {
    constexpr int kPermWaves = SMALL_E ? kPermWavesSmallE : kPermWavesLargeE;
    constexpr int kPermThreads = kPermWaves * kWave;
    extern __shared__ int lds[];             // wave_cnt[kPermWaves][E], excl[E]
    int* wave_cnt = lds;
    int* excl = lds + kPermWaves * E;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;

    for (int i = tid; i < kPermWaves * E; i += kPermThreads) wave_cnt[i] = 0;
    __syncthreads();

    // slice of this wave: multiple of 64 pairs so that (C) walks whole wavefronts
    int per_wave = (P + kPermWaves - 1) / kPermWaves;
    per_wave = (per_wave + kWave - 1) / kWave * kWave;
    const int lo = min(P, wave * per_wave), hi = min(P, lo + per_wave);
    int* mine = wave_cnt + wave * E;

    // (A) counts.  Indices are fetched kBatch wavefront-rows at a time so the loads overlap.
    // A slice of at most one such batch stays in registers for phase (C).
    const bool one_batch = per_wave <= kWave * kBatch;
    int ev[kBatch];
    for (int base = lo; base < hi; base += kWave * kBatch) {
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int p = base + b * kWave + lane;
            ev[b] = (p < hi) ? idx[p] : -1;
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b)
            if (base + b * kWave + lane < hi) atomicAdd(&mine[min(max(ev[b], 0), E - 1)], 1);
    }
    __syncthreads();

    for (int e = tid; e < E; e += kPermThreads) {                       // (B) totals
        int tot = 0;
#pragma unroll
        for (int w = 0; w < kPermWaves; ++w) tot += wave_cnt[w * E + e];
        excl[e] = tot;
    }
    __syncthreads();
    if (wave == 0) {                                                     // exclusive scan
        int carry = 0;
        for (int e0 = 0; e0 < E; e0 += kWave) {
            int e = e0 + lane;
            int v = (e < E) ? excl[e] : 0;
            int inc = v;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                int n = __shfl_up(inc, off, kWave);
                if (lane >= off) inc += n;
            }
            if (e < E) { excl[e] = carry + inc - v; offsets[e] = carry + inc - v; }
            carry += __shfl(inc, kWave - 1, kWave);
        }
        if (lane == 0) offsets[E] = carry;
    }
    __syncthreads();
    for (int e = tid; e < E; e += kPermThreads) {                       // first row per wave
        int run = excl[e];
#pragma unroll
        for (int w = 0; w < kPermWaves; ++w) {
            int c = wave_cnt[w * E + e];
            wave_cnt[w * E + e] = run;
            run += c;
        }
    }
    __syncthreads();

    const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    int cursor = (SMALL_E && lane < E) ? mine[lane] : 0;                // lane e: cursor of expert e
    for (int base0 = lo; base0 < hi; base0 += kWave * kBatch) {         // (C)
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int p = base0 + b * kWave + lane;
            const int raw = one_batch ? ev[b] : ((p < hi) ? idx[p] : -1);
            ev[b] = (p < hi) ? min(max(raw, 0), E - 1) : -1;
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int p = base0 + b * kWave + lane;
            const bool valid = p < hi;
            const int e = ev[b];
            unsigned long long todo = __ballot(valid);
            int dest = 0;
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const int cur = __builtin_amdgcn_readlane(e, leader);
                const unsigned long long grp = __ballot(e == cur);
                if (SMALL_E) {
                    const int first = __builtin_amdgcn_readlane(cursor, cur);
                    if (e == cur) dest = first + __popcll(grp & lt_mask);
                    if (lane == cur) cursor += __popcll(grp);
                } else {
                    if (e == cur) dest = mine[cur] + __popcll(grp & lt_mask);
                    __builtin_amdgcn_wave_barrier();
                    if (lane == leader) mine[cur] += __popcll(grp);
                    __builtin_amdgcn_wave_barrier();
                }
                todo &= ~grp;
            }
            if (valid) { row_src[dest] = p; row_of[p] = dest; }
        }
    }
}

template <typename Chunk>
__global__ __launch_bounds__(256) void gather_rows_kernel(
    const Chunk* __restrict__ x, const int32_t* __restrict__ row_src, int P, int k,
    int chunks_per_row, Chunk* __restrict__ x_perm) {
    const long long total = (long long)P * chunks_per_row;
    long long g = (long long)blockIdx.x * (256 * 4) + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i, g += 256) {
        if (g < total) {
            int r = (int)(g / chunks_per_row);
            int c = (int)(g - (long long)r * chunks_per_row);
            int t = row_src[r] / k;
            x_perm[g] = x[(long long)t * chunks_per_row + c];
        }
    }
}

}  // namespace

hipError_t launch_permute(const void* x, const int32_t* idx, int T, int d, int E, int k,
                          int dtype, void* x_perm, int32_t* offsets, int32_t* row_src,
                          int32_t* row_of, hipStream_t s) {
    const int P = T * k;
    if (E <= kWave)
        hipLaunchKernelGGL(permute_index_kernel<true>, dim3(1), dim3(kPermWavesSmallE * kWave),
                           (size_t)(kPermWavesSmallE + 1) * E * sizeof(int), s, idx, P, E, offsets,
                           row_src, row_of);
    else
        hipLaunchKernelGGL(permute_index_kernel<false>, dim3(1), dim3(kPermWavesLargeE * kWave),
                           (size_t)(kPermWavesLargeE + 1) * E * sizeof(int), s, idx, P, E, offsets,
                           row_src, row_of);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || x_perm == nullptr || P == 0) return err;
    const size_t row_bytes = (size_t)d * (dtype == 0 ? 4 : 2);
    const unsigned align = (unsigned)(((uintptr_t)x | (uintptr_t)x_perm) & 15u);
    if (row_bytes % 16 == 0 && align == 0) {
        int cpr = (int)(row_bytes / 16);
        long long total = (long long)P * cpr;
        hipLaunchKernelGGL(gather_rows_kernel<U128>, dim3((unsigned)((total + 1023) / 1024)),
                           dim3(256), 0, s, (const U128*)x, row_src, P, k, cpr, (U128*)x_perm);
    } else if (row_bytes % 4 == 0 && (align & 3u) == 0) {
        int cpr = (int)(row_bytes / 4);
        long long total = (long long)P * cpr;
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3((unsigned)((total + 1023) / 1024)),
                           dim3(256), 0, s, (const uint32_t*)x, row_src, P, k, cpr,
                           (uint32_t*)x_perm);
    } else {
        int cpr = (int)(row_bytes / 2);
        long long total = (long long)P * cpr;
        hipLaunchKernelGGL(gather_rows_kernel<uint16_t>, dim3((unsigned)((total + 1023) / 1024)),
                           dim3(256), 0, s, (const uint16_t*)x, row_src, P, k, cpr,
                           (uint16_t*)x_perm);
    }
    return hipGetLastError();
}

}  // namespace specmoe
