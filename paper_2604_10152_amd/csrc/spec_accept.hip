// Greedy acceptance of speculative draft tokens (SpecMoE Sec. 2.2, Fig. 4 and its caption;
// Sec. 4 "SpecMoE configuration": only drafts that exactly match the target's greedy tokens
// are accepted; the earliest mismatch and everything after it are dropped and the target's
// own token at that position is appended).  One lane per sequence; integer work only.
#include "common.h"

namespace specmoe {
namespace {

__global__ __launch_bounds__(256) void spec_accept_kernel(
    const int32_t* __restrict__ draft, const int32_t* __restrict__ target, int B, int gamma,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ out_tokens) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int32_t* dr = draft + (size_t)b * gamma;
    const int32_t* tg = target + (size_t)b * (gamma + 1);
    int32_t* ot = out_tokens + (size_t)b * (gamma + 1);
    int n = 0;
    while (n < gamma && dr[n] == tg[n]) ++n;
    accept_len[b] = n + 1;
    for (int i = 0; i <= gamma; ++i) ot[i] = (i <= n) ? tg[i] : -1;
}

}  // namespace

hipError_t launch_spec_accept(const int32_t* draft, const int32_t* target, int B, int gamma,
                              int32_t* accept_len, int32_t* out_tokens, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(spec_accept_kernel, dim3((B + 255) / 256), dim3(256), 0, s, draft,
                       target, B, gamma, accept_len, out_tokens);
    return hipGetLastError();
}

}  // namespace specmoe
