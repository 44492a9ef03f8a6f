// Gate of one MoE block: router logits in fp64, top-k on logits, softmax gate weights.
// (SpecMoE Sec. 2.1: the gate selects the top-K experts per token.)
//
// One 64-lane wavefront owns one token.  Lanes stride the d_model axis with 16-byte loads,
// every expert column goes through the same lane partition and the same xor-butterfly, so two
// experts with identical router rows produce bit-identical logits and the tie is decided by
// expert id.  The E logits of the token live in LDS; top-k is k rounds of a wave-wide arg-max
// on the key (logit descending, expert id ascending).
#include "common.h"

namespace specmoe {
namespace {

constexpr int kRouteWaves = 4;      // tokens per workgroup
constexpr int kExpertChunk = 8;     // expert columns accumulated per pass over x[t,:]

template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, double (&o)[4]) {
        float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, double (&o)[8]) {
        U128 v = *reinterpret_cast<const U128*>(p);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = (double)bf16_bits_to_float(w[i] & 0xffffu);
            o[2 * i + 1] = (double)bf16_bits_to_float(w[i] >> 16);
        }
    }
};

__device__ __forceinline__ bool better(double av, int aid, double bv, int bid) {
    return (av > bv) || (av == bv && aid < bid);
}

template <typename T>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_topk_kernel(
    const T* __restrict__ x, const T* __restrict__ wr, const float* __restrict__ bias, int Tn,
    int d, int E, int k, int renorm, int vec_ok_i, int32_t* __restrict__ idx_out,
    float* __restrict__ w_out) {
    extern __shared__ double lds_logits[];   // [kRouteWaves][E]
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int t = blockIdx.x * kRouteWaves + wave;
    if (t >= Tn) return;                     // whole wave leaves; no block-wide barrier below
    double* logit = lds_logits + (size_t)wave * E;
    const T* xt = x + (size_t)t * d;
    constexpr int V = Vec<T>::N;
    const bool vec_ok = vec_ok_i != 0;     // host checked: d % V == 0 and 16-byte aligned bases

    for (int e0 = 0; e0 < E; e0 += kExpertChunk) {
        double acc[kExpertChunk];
#pragma unroll
        for (int c = 0; c < kExpertChunk; ++c) acc[c] = 0.0;
        if (vec_ok) {
            for (int j = lane * V; j < d; j += kWave * V) {
                double xv[V];
                Vec<T>::load(xt + j, xv);
#pragma unroll
                for (int c = 0; c < kExpertChunk; ++c) {
                    if (e0 + c < E) {
                        double wv[V];
                        Vec<T>::load(wr + (size_t)(e0 + c) * d + j, wv);
#pragma unroll
                        for (int i = 0; i < V; ++i) acc[c] = fma(xv[i], wv[i], acc[c]);
                    }
                }
            }
        } else {
            for (int j = lane; j < d; j += kWave) {
                double xv = (double)load_as_float(xt + j);
#pragma unroll
                for (int c = 0; c < kExpertChunk; ++c)
                    if (e0 + c < E)
                        acc[c] = fma(xv, (double)load_as_float(wr + (size_t)(e0 + c) * d + j), acc[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < kExpertChunk; ++c) {
            double s = wave_sum(acc[c]);
            if (lane == 0 && e0 + c < E)
                logit[e0 + c] = s + (bias ? (double)bias[e0 + c] : 0.0);
        }
    }
    __builtin_amdgcn_wave_barrier();
    __threadfence_block();

    // lane owns experts lane, lane+64, ...; `taken` marks the ones already selected.
    // Lane s keeps the result of round s (k <= 64), so the final stores are coalesced.
    constexpr int kOwn = 1024 / kWave;       // SPECMOE_MAX_EXPERTS / 64
    uint32_t taken = 0;
    double vmax = 0.0, denom = 1.0, wsum_sel = 0.0, my_p = 0.0;
    int my_id = 0;
    for (int s = 0; s < k; ++s) {
        double bv = 0.0; int bid = -1;
#pragma unroll 1
        for (int o = 0; o < kOwn; ++o) {
            int e = lane + o * kWave;
            if (e >= E) break;
            if (taken & (1u << o)) continue;
            double v = logit[e];
            if (bid < 0 || better(v, e, bv, bid)) { bv = v; bid = e; }
        }
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
            double ov = __shfl_xor(bv, off, kWave);
            int oid = __shfl_xor(bid, off, kWave);
            if (oid >= 0 && (bid < 0 || better(ov, oid, bv, bid))) { bv = ov; bid = oid; }
        }
        if ((bid % kWave) == lane) taken |= 1u << (bid / kWave);
        if (s == 0) {
            // softmax denominator over all E experts, relative to the largest logit
            vmax = bv;
            double part = 0.0;
            for (int e = lane; e < E; e += kWave) part += exp(logit[e] - vmax);
            denom = wave_sum(part);
        }
        double p = exp(bv - vmax) / denom;
        wsum_sel += p;                        // slot order, identical on every lane
        if (lane == s) { my_p = p; my_id = bid; }
    }
    if (lane < k) {
        idx_out[(size_t)t * k + lane] = my_id;
        w_out[(size_t)t * k + lane] = (float)(renorm ? my_p / wsum_sel : my_p);
    }
}

}  // namespace

hipError_t launch_route_topk(const void* x, const void* wr, const float* bias, int T, int d,
                             int E, int k, int renorm, int dtype, int32_t* idx, float* w,
                             hipStream_t s) {
    if (T == 0) return hipSuccess;
    dim3 grid((T + kRouteWaves - 1) / kRouteWaves), block(kRouteWaves * kWave);
    size_t lds = (size_t)kRouteWaves * E * sizeof(double);
    const bool aligned = (((uintptr_t)x | (uintptr_t)wr) & 15u) == 0;
    if (dtype == 0)
        hipLaunchKernelGGL(route_topk_kernel<float>, grid, block, lds, s, (const float*)x,
                           (const float*)wr, bias, T, d, E, k, renorm,
                           (int)(aligned && d % Vec<float>::N == 0), idx, w);
    else
        hipLaunchKernelGGL(route_topk_kernel<bf16_t>, grid, block, lds, s, (const bf16_t*)x,
                           (const bf16_t*)wr, bias, T, d, E, k, renorm,
                           (int)(aligned && d % Vec<bf16_t>::N == 0), idx, w);
    return hipGetLastError();
}

}  // namespace specmoe
