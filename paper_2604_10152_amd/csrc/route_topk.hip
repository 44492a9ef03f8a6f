// Gate of one MoE block: router logits in fp64, top-k on logits, softmax gate weights.
// (SpecMoE Sec. 2.1: the gate selects the top-K experts per token.)
//
// A workgroup owns TOK tokens and consists of 4 groups of 4 wavefronts; group g takes the
// expert chunks g, g+4, ... of EC experts each, so the widening of the router weights to fp64
// (the bulk of the work: every weight is converted once per workgroup) is spread over 1024
// lanes.  Inside a group the d_model axis is dealt to its 256 lanes in 16-byte chunks (chunk q
// -> wave (q/64)%4, lane q%64), every lane keeps fp64 partial sums for TOK tokens x EC experts
// (TOK*EC <= 16), so one router-weight load feeds TOK tokens.
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

constexpr int kRouteWaves = 4;                        // wavefronts per group
constexpr int kGroupThreads = kRouteWaves * kWave;
constexpr int kRouteGroups = 4;                       // groups per workgroup (split the experts)
constexpr int kRouteThreads = kRouteGroups * kGroupThreads;

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
    static_assert(TOK * EC <= 16 && (TOK * EC & (TOK * EC - 1)) == 0, "values per wave");
    constexpr int NV = TOK * EC;                      // partial sums per lane and pass
    extern __shared__ double lds_d[];                 // logits[TOK][E], then part[groups][4][NV]
    double* logits = lds_d;
    typedef Chunk<T, VEC> CH;
    constexpr int V = CH::N;
    constexpr int G = EC < 8 ? EC : 8;                // router rows loaded together
    const int lane = threadIdx.x % kWave;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int group = wave_all / kRouteWaves, wave = wave_all % kRouteWaves;
    const int gtid = threadIdx.x % kGroupThreads;     // thread index inside the group
    double* part = lds_d + (size_t)TOK * E + (size_t)group * kRouteWaves * NV;
    const int t0 = blockIdx.x * TOK;
    const int nq = d / V;                             // chunks per row (VEC: d % V == 0)

    // every group runs the same number of passes (the barriers inside are workgroup-wide); a
    // group whose chunk lies beyond E skips the arithmetic of that pass
    const int passes = (E + kRouteGroups * EC - 1) / (kRouteGroups * EC);
    for (int pass = 0; pass < passes; ++pass) {
        const int e0 = (pass * kRouteGroups + group) * EC;
        const bool live = e0 < E;
        double acc[NV];                               // index t * EC + c
#pragma unroll
        for (int i = 0; i < NV; ++i) acc[i] = 0.0;
        for (int q = gtid; live && q < nq; q += kGroupThreads) {
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
        if (gtid < NV) {
            const int t = gtid / EC, c = gtid % EC;
            if (e0 + c < E) {
                double s = part[gtid];
#pragma unroll
                for (int w = 1; w < kRouteWaves; ++w) s += part[w * NV + gtid];
                logits[(size_t)t * E + e0 + c] = s + (bias ? (double)bias[e0 + c] : 0.0);
            }
        }
        __syncthreads();
    }

    // wave t of the workgroup ranks token t0 + t (TOK <= 4)
    if (wave_all >= TOK || t0 + wave_all >= Tn) return;
    const int t = t0 + wave_all;
    const double* logit = logits + (size_t)wave_all * E;
    if (E <= kWave) {
        // One expert per lane: every lane counts the experts that beat its own on the key
        // (logit descending, id ascending) - its rank, i.e. the slot it would fill.  The other
        // lanes' logits arrive through v_readlane broadcasts (a few cycles each) instead of the
        // k x 6 dependent cross-lane exchanges of the arg-max rounds below.
        const bool valid = lane < E;
        const double v = valid ? logit[lane] : 0.0;
        const int vlo = (int)(uint32_t)__double_as_longlong(v);
        const int vhi = (int)(uint32_t)((uint64_t)__double_as_longlong(v) >> 32);
        auto lane_value = [&](double val, int src) __attribute__((always_inline)) -> double {
            const long long bits = __double_as_longlong(val);
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, src);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)bits >> 32), src);
            return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
        };
        int rank = 0;
        for (int j = 0; j < E; ++j) {
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(vlo, j);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane(vhi, j);
            const double vj = __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
            rank += better(vj, j, v, lane) ? 1 : 0;
        }
        const int first = __builtin_amdgcn_readfirstlane(
            __ffsll((long long)__ballot(valid && rank == 0)) - 1);
        const double vmax = lane_value(v, first);
        // softmax over all E experts, relative to the largest logit
        const double pe = valid ? exp(v - vmax) : 0.0;
        const double p = pe / wave_sum(pe);
        double wsum_sel = 0.0;                        // slot order, identical on every lane
        for (int sl = 0; sl < k; ++sl) {
            const int src = __builtin_amdgcn_readfirstlane(
                __ffsll((long long)__ballot(valid && rank == sl)) - 1);
            wsum_sel += lane_value(p, src);
        }
        if (valid && rank < k) {
            idx_out[(size_t)t * k + rank] = remap ? remap[lane] : lane;
            w_out[(size_t)t * k + rank] = (float)(renorm ? p / wsum_sel : p);
        }
        return;
    }
    // More than 64 experts: lane owns experts lane, lane+64, ...; `taken` marks the ones already
    // selected.  Lane s keeps the result of round s (k <= 64), so the final stores are coalesced.
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
    size_t lds = ((size_t)TOK * E + (size_t)kRouteGroups * kRouteWaves * TOK * EC) * sizeof(double);
    hipLaunchKernelGGL((route_topk_kernel<T, VEC, TOK, EC>), grid, block, lds, s, x, wr, bias, Tn,
                       d, E, k, renorm, idx, w, remap);
}

// experts per group and pass: a quarter of E rounded up to a power of two, at most 16 / TOK
template <typename T, bool VEC, int TOK>
void launch_by_experts(const T* x, const T* wr, const float* bias, int Tn, int d, int E, int k,
                       int renorm, int32_t* idx, float* w, const int32_t* remap, hipStream_t s) {
    constexpr int EC_MAX = 16 / TOK;
    const int quarter = (E + kRouteGroups - 1) / kRouteGroups;
    if (quarter <= 1)
        launch_variant<T, VEC, TOK, 1>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (quarter <= 2 || EC_MAX == 2)
        launch_variant<T, VEC, TOK, (EC_MAX < 2 ? EC_MAX : 2)>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (quarter <= 4 || EC_MAX == 4)
        launch_variant<T, VEC, TOK, (EC_MAX < 4 ? EC_MAX : 4)>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (quarter <= 8 || EC_MAX == 8)
        launch_variant<T, VEC, TOK, (EC_MAX < 8 ? EC_MAX : 8)>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else
        launch_variant<T, VEC, TOK, EC_MAX>(x, wr, bias, Tn, d, E, k, renorm, idx, w, remap, s);
}

template <typename T, int V>
void launch_typed(const void* x, const void* wr, const float* bias, int Tn, int d, int E, int k,
                  int renorm, int32_t* idx, float* w, const int32_t* remap, hipStream_t s) {
    const bool vec = (d % V == 0) && ((((uintptr_t)x | (uintptr_t)wr) & 15u) == 0);
    const T* xt = (const T*)x;
    const T* wt = (const T*)wr;
    if (!vec) {
        launch_by_experts<T, false, 1>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
        return;
    }
    // Tokens per workgroup.  The kernel is bound by the widening conversions to fp64 (about 8x
    // the cost of an fp64 FMA per instruction; its time does not depend on d_model below one
    // chunk per lane and does not depend on k).  Per SIMD of the busiest CU they number
    //   workgroups per CU x 4 waves x passes x 8 x (TOK + EC)
    // (every group of 4 waves widens its TOK token chunks and its EC router chunks per pass;
    // passes x EC covers a quarter of the experts).  More tokens per workgroup share the
    // widened router weights but leave CUs idle while the batch is small: take the minimum.
    int best_tok = 1;
    long long best = -1;
    for (int tok = 1; tok <= 4; tok *= 2) {
        const int ec_max = 16 / tok;
        int ec = 1;
        while (ec < ec_max && ec * kRouteGroups < E) ec *= 2;
        const long long passes = (E + kRouteGroups * ec - 1) / (kRouteGroups * ec);
        const long long wgs = (Tn + tok - 1) / tok;
        const long long per_cu = (wgs + 255) / 256;
        const long long load = per_cu * passes * (tok + ec);
        if (best < 0 || load < best) { best = load; best_tok = tok; }
    }
    if (best_tok == 4) launch_by_experts<T, true, 4>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else if (best_tok == 2) launch_by_experts<T, true, 2>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
    else launch_by_experts<T, true, 1>(xt, wt, bias, Tn, d, E, k, renorm, idx, w, remap, s);
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
