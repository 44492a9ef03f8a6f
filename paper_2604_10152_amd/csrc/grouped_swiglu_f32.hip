// Experts in fp32 mode: grouped SwiGLU FFN with plain fp32 FMA (no matrix cores, no reduced
// precision), LDS-tiled.  (SpecMoE Sec. 2.1: every expert is an FFN-sized block; only rows
// routed to an expert are multiplied with its weights.)
//
// This mode exists for the 1e-5 parity configuration; every load is bounds-checked so any
// d_model / d_ff works.  A workgroup owns a 64x64 output tile of one expert (64 contraction
// elements per step, the next step's operands prefetched into registers); the m-tile ->
// expert lookup walks expert_offsets on the device, so no host read-back is needed.
#include "common.h"

namespace specmoe {
namespace {

constexpr int kBM = 64, kBN = 64, kBK = 64, kThreads = 256;
constexpr int kLd = kBM * kBK / kThreads;     // elements of each operand tile per thread

// Finds the expert and the first row of global m-tile `mt` (tiles never straddle experts).
__device__ __forceinline__ bool locate_tile(const int32_t* offsets, int E, int mt, int bm,
                                            int& expert, int& row0, int& row_end) {
    int seen = 0;
    for (int e = 0; e < E; ++e) {
        const int lo = offsets[e], hi = offsets[e + 1];
        const int nt = (hi - lo + bm - 1) / bm;
        if (mt < seen + nt) {
            expert = e; row0 = lo + (mt - seen) * bm; row_end = hi;
            return true;
        }
        seen += nt;
    }
    return false;
}

template <bool kSwiglu>
__global__ __launch_bounds__(kThreads) void grouped_gemm_f32_kernel(
    const float* __restrict__ A, const int32_t* __restrict__ offsets,
    const float* __restrict__ W0, const float* __restrict__ W1, int E, int N, int K,
    float* __restrict__ C, const int32_t* __restrict__ row_src, int topk) {
    __shared__ float As[kBK][kBM + 4];
    __shared__ float B0s[kBK][kBN + 4];
    __shared__ float B1s[kSwiglu ? kBK : 1][kBN + 4];
    int expert, row0, row_end;
    if (!locate_tile(offsets, E, blockIdx.y, kBM, expert, row0, row_end)) return;
    const int n0 = blockIdx.x * kBN;
    const float* w0 = W0 + (size_t)expert * N * K;
    const float* w1 = kSwiglu ? W1 + (size_t)expert * N * K : nullptr;
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    float acc0[4][4] = {}, acc1[4][4] = {};

    // the k-tile after the current one travels from global memory into registers while the
    // current one is multiplied (one exposed memory round trip per tile instead of two)
    float ra[kLd], rb0[kLd], rb1[kSwiglu ? kLd : 1];
    size_t arow[kLd];
#pragma unroll
    for (int i = 0; i < kLd; ++i) {
        const int gr = row0 + (tid + i * kThreads) / kBK;
        arow[i] = (row_src && gr < row_end) ? (size_t)(row_src[gr] / topk) : (size_t)gr;
    }
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < kLd; ++i) {
            const int flat = tid + i * kThreads;       // 64 rows x kBK contraction elements
            const int r = flat / kBK, kk = flat % kBK;
            const int gr = row0 + r, gk = k0 + kk, gn = n0 + r;
            ra[i] = (gr < row_end && gk < K) ? A[arow[i] * K + gk] : 0.f;
            rb0[i] = (gn < N && gk < K) ? w0[(size_t)gn * K + gk] : 0.f;
            if (kSwiglu) rb1[i] = (gn < N && gk < K) ? w1[(size_t)gn * K + gk] : 0.f;
        }
    };
    gload(0);
    for (int k0 = 0; k0 < K; k0 += kBK) {
#pragma unroll
        for (int i = 0; i < kLd; ++i) {
            const int flat = tid + i * kThreads;
            const int r = flat / kBK, kk = flat % kBK;
            As[kk][r] = ra[i];
            B0s[kk][r] = rb0[i];
            if (kSwiglu) B1s[kk][r] = rb1[i];
        }
        __syncthreads();
        if (k0 + kBK < K) gload(k0 + kBK);
#pragma unroll
        for (int kk = 0; kk < kBK; ++kk) {
            float a[4], b0[4], b1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[kk][ty * 4 + i];
                b0[i] = B0s[kk][tx * 4 + i];
                b1[i] = kSwiglu ? B1s[kk][tx * 4 + i] : 0.f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(a[i], b0[j], acc0[i][j]);
                    if (kSwiglu) acc1[i][j] = fmaf(a[i], b1[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gr = row0 + ty * 4 + i;
        if (gr >= row_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc0[i][j];
            if (kSwiglu) {
                // silu in full fp32 precision (expf, true division)
                v = (v / (1.0f + expf(-v))) * acc1[i][j];
            }
            C[(size_t)gr * N + gn] = v;
        }
    }
}

}  // namespace

hipError_t launch_expert_up_f32(const float* x_perm, const int32_t* offsets, const float* wg,
                                const float* wu, int n_rows, int d, int f, int E, float* h,
                                hipStream_t s, const int32_t* row_src, int topk) {
    if (n_rows == 0) return hipSuccess;
    const int max_mt = n_rows / kBM + E;           // sum_e ceil(M_e/BM) <= floor(P/BM) + E
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<true>, dim3((f + kBN - 1) / kBN, max_mt),
                       dim3(kThreads), 0, s, x_perm, offsets, wg, wu, E, f, d, h, row_src, topk);
    return hipGetLastError();
}

hipError_t launch_expert_down_f32(const float* h, const int32_t* offsets, const float* wd,
                                  int n_rows, int d, int f, int E, float* y, hipStream_t s) {
    if (n_rows == 0) return hipSuccess;
    const int max_mt = n_rows / kBM + E;
    hipLaunchKernelGGL(grouped_gemm_f32_kernel<false>, dim3((d + kBN - 1) / kBN, max_mt),
                       dim3(kThreads), 0, s, h, offsets, wd, (const float*)nullptr, E, d, f, y,
                       (const int32_t*)nullptr, 1);
    return hipGetLastError();
}

}  // namespace specmoe
