// Gate-weighted mix of the selected experts' outputs (SpecMoE Sec. 2.1, Fig. 1b) and the
// RMSNorm helper of the multi-layer benchmark configuration.
//
// combine is a gather, not a scatter: one workgroup per token reads its k expert rows through
// row_of and accumulates them in fp32 in slot order, so the result is deterministic and needs
// no atomics.  Both kernels are single HBM passes with 16-byte accesses.
#include "common.h"

namespace specmoe {
namespace {

constexpr int kRowThreads = 256;

template <typename T> struct RowVec;
template <> struct RowVec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, float (&o)[4]) {
        float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    __device__ static void store(float* p, const float (&o)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
    }
};
template <> struct RowVec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, float (&o)[8]) {
        U128 v = *reinterpret_cast<const U128*>(p);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = bf16_bits_to_float(w[i] & 0xffffu);
            o[2 * i + 1] = bf16_bits_to_float(w[i] >> 16);
        }
    }
    __device__ static void store(bf16_t* p, const float (&o)[8]) {
        U128 v;
        v.x = pack_bf16x2(o[0], o[1]); v.y = pack_bf16x2(o[2], o[3]);
        v.z = pack_bf16x2(o[4], o[5]); v.w = pack_bf16x2(o[6], o[7]);
        *reinterpret_cast<U128*>(p) = v;
    }
};

template <typename T>
__global__ __launch_bounds__(kRowThreads) void combine_kernel(
    const T* __restrict__ y_perm, const int32_t* __restrict__ row_of,
    const float* __restrict__ w, const T* residual, int d, int k, int vec_ok, T* out) {
    const int t = blockIdx.x;
    constexpr int V = RowVec<T>::N;
    if (vec_ok) {                            // host checked: d % V == 0, 16-byte aligned bases
        for (int j = threadIdx.x * V; j < d; j += kRowThreads * V) {
            float acc[V];
            if (residual) RowVec<T>::load(residual + (size_t)t * d + j, acc);
            else {
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = 0.f;
            }
            for (int s = 0; s < k; ++s) {
                const int r = row_of[(size_t)t * k + s];
                const float ws = w[(size_t)t * k + s];
                float v[V];
                RowVec<T>::load(y_perm + (size_t)r * d + j, v);
#pragma unroll
                for (int i = 0; i < V; ++i) acc[i] = fmaf(ws, v[i], acc[i]);
            }
            RowVec<T>::store(out + (size_t)t * d + j, acc);
        }
    } else {
        for (int j = threadIdx.x; j < d; j += kRowThreads) {
            float acc = residual ? load_as_float(residual + (size_t)t * d + j) : 0.f;
            for (int s = 0; s < k; ++s) {
                const int r = row_of[(size_t)t * k + s];
                acc = fmaf(w[(size_t)t * k + s], load_as_float(y_perm + (size_t)r * d + j), acc);
            }
            store_from_float(out + (size_t)t * d + j, acc);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kRowThreads) void rmsnorm_kernel(
    const T* __restrict__ x, const T* __restrict__ gain, int d, float eps, T* __restrict__ out) {
    __shared__ float part[kRowThreads / kWave];
    const int t = blockIdx.x;
    const T* xt = x + (size_t)t * d;
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += kRowThreads) {
        float v = load_as_float(xt + j);
        ss = fmaf(v, v, ss);
    }
    ss = wave_sum(ss);
    if (threadIdx.x % kWave == 0) part[threadIdx.x / kWave] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < kRowThreads / kWave; ++i) tot += part[i];
    const float scale = 1.0f / sqrtf(tot / (float)d + eps);
    for (int j = threadIdx.x; j < d; j += kRowThreads)
        store_from_float(out + (size_t)t * d + j,
                         load_as_float(xt + j) * scale * load_as_float(gain + j));
}

}  // namespace

hipError_t launch_combine(const void* y_perm, const int32_t* row_of, const float* w,
                          const void* residual, int T, int d, int k, int dtype, void* out,
                          hipStream_t s) {
    if (T == 0 || d == 0) return hipSuccess;
    const bool aligned = (((uintptr_t)y_perm | (uintptr_t)residual | (uintptr_t)out) & 15u) == 0;
    if (dtype == 0)
        hipLaunchKernelGGL(combine_kernel<float>, dim3(T), dim3(kRowThreads), 0, s,
                           (const float*)y_perm, row_of, w, (const float*)residual, d, k,
                           (int)(aligned && d % 4 == 0), (float*)out);
    else
        hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(T), dim3(kRowThreads), 0, s,
                           (const bf16_t*)y_perm, row_of, w, (const bf16_t*)residual, d, k,
                           (int)(aligned && d % 8 == 0), (bf16_t*)out);
    return hipGetLastError();
}

hipError_t launch_rmsnorm(const void* x, const void* gain, int T, int d, float eps, int dtype,
                          void* out, hipStream_t s) {
    if (T == 0 || d == 0) return hipSuccess;
    if (dtype == 0)
        hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(T), dim3(kRowThreads), 0, s,
                           (const float*)x, (const float*)gain, d, eps, (float*)out);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(T), dim3(kRowThreads), 0, s,
                           (const bf16_t*)x, (const bf16_t*)gain, d, eps, (bf16_t*)out);
    return hipGetLastError();
}

}  // namespace specmoe
