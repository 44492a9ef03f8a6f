// Temporally hot experts of one MoE block (SpecMoE Sec. 3.2 "Expert replacement policy", Fig. 7
// steps 3-4): during verification the activations of every expert are counted, and the N most
// activated experts become the draft experts of the next speculation phase.  The counts are the
// differences of expert_offsets, a by-product of moe_permute.  Ties go to the lower expert id.
// One wavefront: lane owns experts lane, lane+64, ...; N rounds of a wave-wide arg-max on the
// key (count descending, id ascending).  Integer work only.
#include "common.h"

namespace specmoe {
namespace {

__global__ __launch_bounds__(kWave) void hot_experts_kernel(const int32_t* __restrict__ offsets,
                                                            int E, int n,
                                                            int32_t* __restrict__ hot_ids,
                                                            int32_t* __restrict__ hot_counts) {
    const int lane = threadIdx.x;
    constexpr int kOwn = 1024 / kWave;                 // SPECMOE_MAX_EXPERTS / 64
    uint32_t taken = 0;
    for (int s = 0; s < n; ++s) {
        int bc = -1, bid = -1;
#pragma unroll 1
        for (int o = 0; o < kOwn; ++o) {
            const int e = lane + o * kWave;
            if (e >= E) break;
            if (taken & (1u << o)) continue;
            const int c = offsets[e + 1] - offsets[e];
            if (bid < 0 || c > bc || (c == bc && e < bid)) { bc = c; bid = e; }
        }
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
            const int oc = __shfl_xor(bc, off, kWave), oid = __shfl_xor(bid, off, kWave);
            if (oid >= 0 && (bid < 0 || oc > bc || (oc == bc && oid < bid))) { bc = oc; bid = oid; }
        }
        if ((bid % kWave) == lane) taken |= 1u << (bid / kWave);
        if (lane == 0) {
            hot_ids[s] = bid;
            if (hot_counts) hot_counts[s] = bc;
        }
    }
}

}  // namespace

hipError_t launch_hot_experts(const int32_t* offsets, int E, int n, int32_t* hot_ids,
                              int32_t* hot_counts, hipStream_t s) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(hot_experts_kernel, dim3(1), dim3(kWave), 0, s, offsets, E, n, hot_ids,
                       hot_counts);
    return hipGetLastError();
}

}  // namespace specmoe
