// Gate of one MoE block: router logits in fp64, top-k on logits, softmax gate weights.
// (SpecMoE Sec. 2.1: the gate selects the top-K experts per token.)
//
// A workgroup of 4 wavefronts owns TOK tokens.  The d_model axis is dealt to the 256 lanes in
// 16-byte chunks (chunk q -> wave (q/64)%4, lane q%64), every lane keeps fp64 partial sums
// for TOK tokens x EC experts (TOK*EC <= 64), so one router-weight load feeds TOK tokens.
// The TOK*EC partial sums of a wave are reduced over its 64 lanes by a transposing butterfly:
// at the step with lane distance h a lane hands the half of its values that its partner keeps
// to the partner and adds what it receives, so 63 exchange-and-add steps reduce all values at
// once (a plain butterfly needs 6 per value) and lane l ends up with the total of value l.
// Every value is summed over the same pairs of lanes in the same order, and fp addition is
// commutative, so two experts with identical router rows get bit-identical logits and the tie
// goes to the lower id.  The 4 wave totals are added in fixed order.  Wave t then ranks token
// t: the E logits sit in LDS, top-k is k rounds of a wave-wide arg-max on the key (logit
// descending, expert id ascending).
#include "common.h"

namespace specmoe {
namespace {

constexpr int kRouteWaves = 4;
constexpr int kRouteThreads = kRouteWaves * kWave;

// Transposing butterfly over the 64 lanes of a wave: v[0..CNT) in every lane -> v[0] = total of
// value (lane * CNT0 / 64) where CNT0 is the count at the first step.
template <int CNT, int BIT>
struct TransposeReduce {
    __device__ __forceinline__ static void run(double* v, int lane) {
        if constexpr (CNT > 1) {
            constexpr int H = CNT / 2;
            const bool up = (lane & BIT) != 0;
#pragma unroll
            for (int i = 0; i < H; ++i) {
                const double send = up ? v[i] : v[i + H];
                const double keep = up ? v[i + H] : v[i];
                v[i] = keep + __shfl_xor(send, BIT, kWave);
            }
            if constexpr (BIT > 1) TransposeReduce<H, BIT / 2>::run(v, lane);
        } else {
            v[0] += __shfl_xor(v[0], BIT, kWave);
            if constexpr (BIT > 1) TransposeReduce<1, BIT / 2>::run(v, lane);
        }
    }
};

template <typename T, bool VEC> struct Chunk;
template <> struct Chunk<float, true> {
    static constexpr int N = 4;
    typedef U128 Raw;
    __device__ static Raw load(const float* p) { return *reinterpret_cast<const U128*>(p); }
    __device__ static void widen(Raw v, double (&o)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (double)__uint_as_float(v[i]);
    }
};
template <> struct Chunk<bf16_t, true> {
    static constexpr int N = 8;
    typedef U128 Raw;
    __device__ static Raw load(const bf16_t* p) { return *reinterpret_cast<const U128*>(p); }
    __device__ static void widen(Raw v, double (&o)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = (double)bf16_bits_to_float(v[i] & 0xffffu);
            o[2 * i + 1] = (double)bf16_bits_to_float(v[i] >> 16);
        }
    }
};
template <typename T> struct Chunk<T, false> {          // any d_model, any alignment
    static constexpr int N = 1;
    typedef float Raw;
    __device__ static Raw load(const T* p) { return load_as_float(p); }
    __device__ static void widen(Raw v, double (&o)[1]) { o[0] = (double)v; }
};

__device__ __forceinline__ bool better(double av, int aid, double bv, int bid) {
    return (av > bv) || (av == bv && aid < bid);
}

template <typename T, bool VEC, int TOK, int EC>
__global__ __launch_bounds__(kRouteThreads) void route_topk_kernel(
    const T* __restrict__ x, const T* __restrict__ wr, const float* __restrict__ bias, int Tn,
    int d, int E, int k, int renorm, int32_t* __restrict__ idx_out, float* __restrict__ w_out,
    const int32_t* __restrict__ remap /* nullable: draft-mode expert substitution, [E] */) {
    static_assert(TOK * EC <= kWave && (TOK * EC & (TOK * EC - 1)) == 0, "values per wave");
    constexpr int NV = TOK * EC;                      // partial sums per lane and pass
    extern __shared__ double lds_d[];                 // logits[TOK][E], then part[4][NV]
    double* logits = lds_d;
    double* part = lds_d + (size_t)TOK * E;
    typedef Chunk<T, VEC> CH;
    constexpr int V = CH::N;
    constexpr int G = EC < 8 ? EC : 8;                // router rows loaded together
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int t0 = blockIdx.x * TOK;
    const int nq = d / V;                             // chunks per row (VEC: d % V == 0)

    for (int e0 = 0; e0 < E; e0 += EC) {
        double acc[NV];                               // index t * EC + c
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.0;
        for (int q = threadIdx.x; q < nq; q += kRouteThreads) {
            typename CH::Raw xr[TOK];
#pragma unroll
            for (int t = 0; t < TOK; ++t)
                xr[t] = CH::load(x + (size_t)min(t0 + t, Tn - 1) * d + (size_t)q * V);
            double xv[TOK][V];
#pragma unroll
            for (int t = 0; t < TOK; ++t) CH::widen(xr[t], xv[t]);
#pragma unroll
            for (int c0 = 0; c0 < EC; c0 += G) {
                typename CH::Raw wraw[G];
#pragma unroll
                for (int c = 0; c < G; ++c)
                    wraw[c] = CH::load(wr + (size_t)min(e0 + c0 + c, E - 1) * d + (size_t)q * V);
#pragma unroll
                for (int c = 0; c < G; ++c) {
                    double wv[V];
                    CH::widen(wraw[c], wv);
#pragma unroll
                    for (int t = 0; t < TOK; ++t)
#pragma unroll
                        for (int i = 0; i < V; ++i)
                            acc[t * EC + c0 + c] = fma(xv[t][i], wv[i], acc[t * EC + c0 + c]);
                }
            }
        }
        // lanes -> wave totals (transposing butterfly), waves -> workgroup total (order 0,1,2,3)
        TransposeReduce<NV, kWave / 2>::run(acc, lane);
        constexpr int REP = kWave / NV;               // lanes holding the same value
        if (lane % REP == 0) part[wave * NV + lane / REP] = acc[0];
        __syncthreads();
        if (threadIdx.x < NV) {
            const int t = threadIdx.x / EC, c = threadIdx.x % EC;
            if (e0 + c < E) {
                double s = part[threadIdx.x];
#pragma unroll
                for (int w = 1; w < kRouteWaves; ++w) s += part[w * NV + threadIdx.x];
                logits[(size_t)t * E + e0 + c] = s + (bias ? (double)bias[e0 + c] : 0.0);
            }
        }
        __syncthreads();
    }

    // wave t ranks token t0 + t (TOK <= 4 waves)
    if (wave >= TOK || t0 + wave >= Tn) return;
    const int t = t0 + wave;
    const double* logit = logits + (size_t)wave * E;
    // lane owns experts lane, lane+64, ...; `taken` marks the ones already selected.
    // Lane s keeps the result of round s (k <= 64), so the final stores are coalesced.
    constexpr int kOwn = 1024 / kWave;                // SPECMOE_MAX_EXPERTS / 64
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
            double p = 0.0;
            for (int e = lane; e < E; e += kWave) p += exp(logit[e] - vmax);
            denom = wave_sum(p);
        }
        double p = exp(bv - vmax) / denom;
        wsum_sel += p;                                // slot order, identical on every lane
        if (lane == s) { my_p = p; my_id = bid; }
    }
    if (lane < k) {
        idx_out[(size_t)t * k + lane] = remap ? remap[my_id] : my_id;
        w_out[(size_t)t * k + lane] = (float)(renorm ? my_p / wsum_sel : my_p);
    }
}

template <typename T, bool VEC, int TOK, int EC>
void launch_variant(const T* x, const T* wr, const float* bias, int Tn, int d, int E, int k,
                    int renorm, int32_t* idx, float* w, const int32_t* remap, hipStream_t s) {
    dim3 grid((Tn + TOK - 1) / TOK), block(kRouteThreads);
    size_t lds = ((size_t)TOK * E + (size_t)kRouteWaves * TOK * EC) * sizeof(double);
    hipLaunchKernelGGL((route_topk_kernel<T, VEC, TOK, EC>), grid, block, lds, s, x, wr, bias, Tn,
                       d, E, k, renorm, idx, w, remap);
}

// experts per pass: the smallest of 8/16/32/64 that covers E (64 for more), capped at 64/TOK
template <typename T, bool VEC, int TOK>
void launch_by_experts(const T* x, const T* wr, const float* bias, int Tn, int d, int E, int k,
                       int renorm, int32_t* idx, float* w, const int32_t* remap, hipStream_t s) {
    if (E <= 8 || TOK * 16 > kWave)
        launch_variant<T, VEC, TOK, (TOK * 8 <= kWave ? 8 : kWave / TOK)>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (E <= 16 || TOK * 32 > kWave)
        launch_variant<T, VEC, TOK, (TOK * 16 <= kWave ? 16 : kWave / TOK)>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (E <= 32 || TOK * 64 > kWave)
        launch_variant<T, VEC, TOK, (TOK * 32 <= kWave ? 32 : kWave / TOK)>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else
        launch_variant<T, VEC, TOK, kWave / TOK>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
}

template <typename T, int V>
void launch_typed(const void* x, const void* wr, const float* bias, int Tn, int d, int E, int k,
                  int renorm, int32_t* idx, float* w, const int32_t* remap, hipStream_t s) {
    const bool vec = (d % V == 0) && ((((uintptr_t)x | (uintptr_t)wr) & 15u) == 0);
    const bool many = Tn >= 1024;                     // enough tokens to fill the chip 4 at a time
    const T* xt = (const T*)x;
    const T* wt = (const T*)wr;
    if (vec && many) launch_by_experts<T, true, 4>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (vec) launch_by_experts<T, true, 1>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else launch_by_experts<T, false, 1>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
}

}  // namespace

hipError_t launch_route_topk(const void* x, const void* wr, const float* bias, int T, int d,
                             int E, int k, int renorm, int dtype, int32_t* idx, float* w,
                             hipStream_t s, const int32_t* remap) {
    if (T == 0) return hipSuccess;
    if (dtype == 0) launch_typed<float, 4>(x, wr, bias, T, d, E, k, renorm, idx, w, remap, s);
    else launch_typed<bf16_t, 8>(x, wr, bias, T, d, E, k, renorm, idx, w, remap, s);
    return hipGetLastError();
}

}  // namespace specmoe
