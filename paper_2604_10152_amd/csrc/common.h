// Shared device helpers and launcher declarations of the gfx950 MoE verify-layer library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specmoe {

constexpr int kWave = 64;           // CDNA wavefront width
constexpr int kXcds = 8;            // MI355X: 8 accelerator dies, workgroups dealt round-robin

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

typedef uint32_t U128 __attribute__((ext_vector_type(4)));   // one 16-byte register quad

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}
__device__ __forceinline__ float load_as_float(const float* p) { return *p; }
__device__ __forceinline__ float load_as_float(const bf16_t* p) { return (float)(*p); }
__device__ __forceinline__ void store_from_float(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_from_float(bf16_t* p, float v) { *p = (bf16_t)v; }

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {(bf16_t)a, (bf16_t)b};
    return __builtin_bit_cast(uint32_t, v);
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float silu_f32(float z) { return z / (1.0f + __expf(-z)); }

// ---- launchers (host side, defined in the .hip files) -------------------------------
hipError_t launch_route_topk(const void* x, const void* wr, const float* bias, int T, int d,
                             int E, int k, int renorm, int dtype, int32_t* idx, float* w,
                             hipStream_t s, const int32_t* remap = nullptr);
// speculation phase (draft_route.hip)
size_t affinity_workspace_bytes(int E);
hipError_t launch_affinity_table(const void* wg, const void* wu, const void* wd, int E, int d,
                                 int f, int dtype, float* table, void* workspace, hipStream_t s);
hipError_t launch_nearest_draft(const float* affinity, int E, const int32_t* draft_ids,
                                int n_draft, int32_t* remap, hipStream_t s);
// sampling-based acceptance, greedy head, active-expert volume (spec_sample.hip)
hipError_t launch_spec_accept_sample(const int32_t* draft, const float* p_draft,
                                     const float* p_target, const float* u_accept,
                                     const float* u_sample, int B, int gamma, int V,
                                     int32_t* accept_len, int32_t* out_tokens, hipStream_t s);
hipError_t launch_greedy_tokens(const void* logits, int R, int V, int dtype, int32_t* tokens,
                                hipStream_t s);
hipError_t launch_active_expert_bytes(const int32_t* offsets, int E, long long bytes_per_expert,
                                      long long* out, hipStream_t s);
hipError_t launch_permute(const void* x, const int32_t* idx, int T, int d, int E, int k,
                          int dtype, void* x_perm, int32_t* offsets, int32_t* row_src,
                          int32_t* row_of, hipStream_t s);
hipError_t launch_expert_up_f32(const float* x_perm, const int32_t* offsets, const float* wg,
                                const float* wu, int n_rows, int d, int f, int E, float* h,
                                hipStream_t s, const int32_t* row_src = nullptr, int topk = 1);
hipError_t launch_expert_down_f32(const float* h, const int32_t* offsets, const float* wd,
                                  int n_rows, int d, int f, int E, float* y, hipStream_t s);
hipError_t launch_expert_up_bf16(const bf16_t* x_perm, const int32_t* offsets, const bf16_t* wg,
                                 const bf16_t* wu, int n_rows, int d, int f, int E, bf16_t* h,
                                 hipStream_t s, const int32_t* row_src = nullptr, int topk = 1);
hipError_t launch_expert_down_bf16(const bf16_t* h, const int32_t* offsets, const bf16_t* wd,
                                   int n_rows, int d, int f, int E, bf16_t* y, hipStream_t s);
hipError_t launch_expert_up_bf16_large16(const bf16_t* x_perm, const int32_t* offsets,
                                         const bf16_t* wg, const bf16_t* wu, int n_rows, int d,
                                         int f, int E, bf16_t* h, hipStream_t s,
    const int32_t* row_src, int topk);
hipError_t launch_expert_down_bf16_large16(const bf16_t* h, const int32_t* offsets,
                                           const bf16_t* wd, int n_rows, int d, int f, int E,
                                           bf16_t* y, hipStream_t s);
hipError_t launch_expert_up_bf16_packed(const bf16_t* x, const int32_t* offsets,
                                        const bf16_t* wg_packed, const bf16_t* wu_packed,
                                        int n_rows, int d, int f, int E, bf16_t* h_packed,
                                        hipStream_t s, const int32_t* row_src, int topk);
hipError_t launch_expert_down_bf16_packed(const bf16_t* h_packed, const int32_t* offsets,
                                          const bf16_t* wd_packed, int n_rows, int d, int f,
                                          int E, bf16_t* y, hipStream_t s);
hipError_t launch_expert_up_bf16_packed_x(const bf16_t* x_packed, const int32_t* offsets,
                                          const bf16_t* wg_packed, const bf16_t* wu_packed,
                                          int n_rows, int d, int f, int E, bf16_t* h,
                                          bool h_row_major, hipStream_t s);
hipError_t launch_gather_pack_rows(const bf16_t* x, const int32_t* row_src, int topk,
                                   const int32_t* offsets, int n_rows, int E, int K,
                                   bf16_t* dst, hipStream_t s);
hipError_t launch_pack_tiles(const bf16_t* src, long long rows, int K, bf16_t* dst, hipStream_t s);
hipError_t launch_expert_up_bf16_small(const bf16_t* x_perm, const int32_t* offsets,
                                       const bf16_t* wg, const bf16_t* wu, int n_rows, int d,
                                       int f, int E, bf16_t* h, hipStream_t s,
    const int32_t* row_src, int topk);
hipError_t launch_expert_down_bf16_small(const bf16_t* h, const int32_t* offsets,
                                         const bf16_t* wd, int n_rows, int d, int f, int E,
                                         bf16_t* y, hipStream_t s);
hipError_t launch_expert_up_bf16_mid(const bf16_t* x_perm, const int32_t* offsets,
                                     const bf16_t* wg, const bf16_t* wu, int n_rows, int d, int f,
                                     int E, bf16_t* h, hipStream_t s, const int32_t* row_src,
                                     int topk);
hipError_t launch_expert_down_bf16_mid(const bf16_t* h, const int32_t* offsets, const bf16_t* wd,
                                       int n_rows, int d, int f, int E, bf16_t* y, hipStream_t s);
hipError_t launch_combine(const void* y_perm, const int32_t* row_of, const float* w,
                          const void* residual, int T, int d, int k, int dtype, void* out,
                          hipStream_t s);
hipError_t launch_rmsnorm(const void* x, const void* gain, int T, int d, float eps, int dtype,
                          void* out, hipStream_t s);
hipError_t launch_hot_experts(const int32_t* offsets, int E, int n, int32_t* hot_ids,
                              int32_t* hot_counts, hipStream_t s);
hipError_t launch_spec_accept(const int32_t* draft, const int32_t* target, int B, int gamma,
                              int32_t* accept_len, int32_t* out_tokens, hipStream_t s);

}  // namespace specmoe
