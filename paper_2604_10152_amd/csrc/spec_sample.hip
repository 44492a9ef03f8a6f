// Verification helpers beyond the greedy rule.
//
// spec_accept_sample_kernel — sampling-based verification (SpecMoE Sec. 6.3: Mixtral-8x7B and
//   Llama-4-Scout are verified with the sampling rule of the speculative-decoding method the
//   paper cites, temperature 1).  Draft token x at position i is kept when
//   u < min(1, pt(x)/pd(x)); at the first rejection the token is redrawn from the normalised
//   positive part of (pt - pd) and the rest is dropped; if every draft is kept one more token
//   is drawn from the target's distribution at position gamma.  The caller supplies the
//   uniforms, so the result is a deterministic function of the inputs.
//   Decisions are taken in fp64 on the fp32 inputs: u*pd and pt-pd are then exact, so the keep
//   test has no rounding at all; the inverse-CDF draw compares fp64 running sums with u*total.
// greedy_tokens_kernel — the greedy head (Sec. 4 "SpecMoE configuration"): id of the largest
//   logit per row, lower id on ties.
// active_expert_bytes_kernel — parameter bytes of the experts that received at least one row
//   (the per-block migration volume the paper's Fig. 3(b) plots; here: the HBM read volume).
#include "common.h"

namespace specmoe {
namespace {

constexpr int kSampleThreads = 1024;  // 16 waves: enough loads in flight for one CU per sequence
constexpr int kSampleWaves = kSampleThreads / kWave;
constexpr int kTileIds = kWave * 4;          // ids one wave covers per step: 4 per lane (16 bytes)
constexpr int kMaxLdsTiles = 2048;           // tile sums kept in LDS (V <= 524288); beyond that
                                             // the tiles are re-summed from memory

// inclusive wave scan (fp64)
__device__ __forceinline__ double wave_scan_incl(double v, int lane) {
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const double o = __shfl_up(v, off, kWave);
        if (lane >= off) v += o;
    }
    return v;
}

// One workgroup per sequence.  The draw needs the smallest id whose running weight exceeds
// u * total: wave w of the 16 sums the 256-id tiles w, w+16, ... (coalesced 16-byte loads, butterfly sum,
// fp64) into LDS, every thread walks the tile sums to find the tile where the threshold is
// crossed, and one wave scans that tile.  Only the order of the fp64 additions differs from a
// sequential running sum.
__global__ __launch_bounds__(kSampleThreads) void spec_accept_sample_kernel(
    const int32_t* __restrict__ draft, const float* __restrict__ p_draft,
    const float* __restrict__ p_target, const float* __restrict__ u_accept,
    const float* __restrict__ u_sample, int gamma, int V, int32_t* __restrict__ accept_len,
    int32_t* __restrict__ out_tokens) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const int lane = tid % kWave, wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    __shared__ int n_sh;
    __shared__ double tile_sum[kMaxLdsTiles];
    const int32_t* dr = draft + (size_t)b * gamma;
    const float* pd = p_draft + (size_t)b * gamma * V;
    const float* pt = p_target + (size_t)b * (gamma + 1) * V;

    // ---- first rejected position (gamma <= 64: one lane per draft token, first wave)
    if (wave == 0) {
        bool reject = false;
        if (lane < gamma) {
            const int x = dr[lane];
            if (x < 0 || x >= V) {
                reject = true;                      // an id outside the vocabulary is never kept
            } else {
                const double lhs = (double)u_accept[(size_t)b * gamma + lane] *
                                   (double)pd[(size_t)lane * V + x];
                reject = !(lhs < (double)pt[(size_t)lane * V + x]);
            }
        }
        const unsigned long long m = __ballot(reject);
        if (lane == 0) n_sh = m ? __ffsll((long long)m) - 1 : gamma;
    }
    __syncthreads();
    const int n = n_sh;
    const float* ptn = pt + (size_t)n * V;
    const float* pdn = n < gamma ? pd + (size_t)n * V : nullptr;
    const bool vec = (V % 4 == 0) && ((((uintptr_t)p_draft | (uintptr_t)p_target) & 15u) == 0);
    const int n_tiles = (V + kTileIds - 1) / kTileIds;

    // this lane's 4 weights of tile `tile` (0 beyond V)
    auto tile_weights = [&](int tile, bool resid, double (&w)[4]) {
        const int v0 = tile * kTileIds + lane * 4;
        float t[4] = {0.f, 0.f, 0.f, 0.f}, q[4] = {0.f, 0.f, 0.f, 0.f};
        if (vec && v0 + 3 < V) {
            const float4 a = *reinterpret_cast<const float4*>(ptn + v0);
            t[0] = a.x; t[1] = a.y; t[2] = a.z; t[3] = a.w;
            if (resid) {
                const float4 c = *reinterpret_cast<const float4*>(pdn + v0);
                q[0] = c.x; q[1] = c.y; q[2] = c.z; q[3] = c.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (v0 + i < V) {
                    t[i] = ptn[v0 + i];
                    if (resid) q[i] = pdn[v0 + i];
                }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double r = (double)t[i] - (double)q[i];      // q = 0 when drawing from pt
            w[i] = (v0 + i < V && r > 0.0) ? r : 0.0;
        }
    };
    auto tile_total = [&](int tile, bool resid) -> double {
        double w[4];
        tile_weights(tile, resid, w);
        return wave_sum((w[0] + w[1]) + (w[2] + w[3]));
    };
    // walk the tiles in id order; returns the total and the tile where `thr` is crossed
    auto sum_tiles = [&](bool resid) -> double {
        for (int tile = wave; tile < n_tiles; tile += kSampleWaves) {
            const double s = tile_total(tile, resid);
            if (lane == 0 && tile < kMaxLdsTiles) tile_sum[tile] = s;
        }
        __syncthreads();
        double tot = 0.0;
        for (int tile = 0; tile < n_tiles; ++tile)
            tot += tile < kMaxLdsTiles ? tile_sum[tile] : tile_total(tile, resid);
        return tot;
    };
    bool resid = pdn != nullptr;
    double total = sum_tiles(resid);
    if (resid && !(total > 0.0)) {                   // pt == pd everywhere: draw from pt
        __syncthreads();
        resid = false;
        total = sum_tiles(false);
    }
    if (wave != 0) return;
    const double thr = (double)u_sample[b] * total;
    int tok = V - 1;
    double before = 0.0;
    for (int tile = 0; tile < n_tiles; ++tile) {
        const double s = tile < kMaxLdsTiles ? tile_sum[tile] : tile_total(tile, resid);
        if (before + s > thr) {
            double w[4];
            tile_weights(tile, resid, w);
            const double c1 = w[0], c2 = c1 + w[1], c3 = c2 + w[2], c4 = c3 + w[3];
            const double excl = before + (wave_scan_incl(c4, lane) - c4);
            int first = 4;
            if (excl + c4 > thr) first = 3;
            if (excl + c3 > thr) first = 2;
            if (excl + c2 > thr) first = 1;
            if (excl + c1 > thr) first = 0;
            const unsigned long long hit = __ballot(first < 4);
            const unsigned long long pos = __ballot(c4 > 0.0);
            if (hit) {
                const int src = __ffsll((long long)hit) - 1;
                tok = tile * kTileIds + src * 4 + __shfl(first, src, kWave);
            } else if (pos) {
                // rounding: the tile's running sums stop a hair below the threshold;
                // take its last id with a positive weight
                const int src = 63 - __clzll((long long)pos);
                const int last = w[3] > 0.0 ? 3 : (w[2] > 0.0 ? 2 : (w[1] > 0.0 ? 1 : 0));
                tok = tile * kTileIds + src * 4 + __shfl(last, src, kWave);
            }
            break;
        }
        before += s;
    }
    if (lane == 0) {
        int32_t* ot = out_tokens + (size_t)b * (gamma + 1);
        for (int i = 0; i <= gamma; ++i) ot[i] = i < n ? dr[i] : (i == n ? tok : -1);
        accept_len[b] = n + 1;
    }
}

template <typename T> struct Row;
template <> struct Row<float> {
    static constexpr int N = 4;
    __device__ static float one(const float* p) { return *p; }
    __device__ static void vec(const float* p, float (&v)[4]) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
};
template <> struct Row<bf16_t> {
    static constexpr int N = 8;
    __device__ static float one(const bf16_t* p) {
        return __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t*>(p) << 16);
    }
    __device__ static void vec(const bf16_t* p, float (&v)[8]) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// One workgroup per row.  Thread t visits its ids in ascending order (16-byte chunks t, t+256,
// ... when the row allows it) and keeps the first maximum it sees; the reduction prefers the
// larger value, then the lower id.  Logits must not contain NaN.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void greedy_tokens_kernel(const T* __restrict__ logits, int V,
                                                            int32_t* __restrict__ tokens) {
    const T* row = logits + (size_t)blockIdx.x * V;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    float bv = 0.f;
    int bi = -1;
    if (VEC) {
        constexpr int N = Row<T>::N;
        for (int c = tid; c < V / N; c += 256) {
            float x[N];
            Row<T>::vec(row + (size_t)c * N, x);
#pragma unroll
            for (int q = 0; q < N; ++q)
                if (bi < 0 || x[q] > bv) { bv = x[q]; bi = c * N + q; }
        }
    } else {
        for (int v = tid; v < V; v += 256) {
            const float x = Row<T>::one(row + v);
            if (bi < 0 || x > bv) { bv = x; bi = v; }
        }
    }
    auto take = [&](float ov, int oi) {
        if (oi >= 0 && (bi < 0 || ov > bv || (ov == bv && oi < bi))) { bv = ov; bi = oi; }
    };
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1)
        take(__shfl_xor(bv, off, kWave), __shfl_xor(bi, off, kWave));
    __shared__ float sv[4];
    __shared__ int si[4];
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) take(sv[w], si[w]);
        tokens[blockIdx.x] = bi;
    }
}

__global__ __launch_bounds__(kWave) void active_expert_bytes_kernel(
    const int32_t* __restrict__ offsets, int E, long long bytes_per_expert,
    long long* __restrict__ out) {
    int n = 0;
    for (int e = threadIdx.x; e < E; e += kWave) n += (offsets[e + 1] - offsets[e]) > 0;
    n = wave_sum(n);
    if (threadIdx.x == 0) out[0] = (long long)n * bytes_per_expert;
}

}  // namespace

hipError_t launch_spec_accept_sample(const int32_t* draft, const float* p_draft,
                                     const float* p_target, const float* u_accept,
                                     const float* u_sample, int B, int gamma, int V,
                                     int32_t* accept_len, int32_t* out_tokens, hipStream_t s) {
    if (B == 0) return hipSuccess;
    hipLaunchKernelGGL(spec_accept_sample_kernel, dim3(B), dim3(kSampleThreads), 0, s, draft,
                       p_draft, p_target, u_accept, u_sample, gamma, V, accept_len, out_tokens);
    return hipGetLastError();
}

template <typename T>
static void launch_greedy_typed(const void* logits, int R, int V, int32_t* tokens, hipStream_t s) {
    const bool vec = V % Row<T>::N == 0 && ((uintptr_t)logits & 15u) == 0 &&
                     ((size_t)V * sizeof(T)) % 16 == 0;
    if (vec)
        hipLaunchKernelGGL((greedy_tokens_kernel<T, true>), dim3(R), dim3(256), 0, s,
                           (const T*)logits, V, tokens);
    else
        hipLaunchKernelGGL((greedy_tokens_kernel<T, false>), dim3(R), dim3(256), 0, s,
                           (const T*)logits, V, tokens);
}

hipError_t launch_greedy_tokens(const void* logits, int R, int V, int dtype, int32_t* tokens,
                                hipStream_t s) {
    if (R == 0) return hipSuccess;
    if (dtype == 0) launch_greedy_typed<float>(logits, R, V, tokens, s);
    else launch_greedy_typed<bf16_t>(logits, R, V, tokens, s);
    return hipGetLastError();
}

hipError_t launch_active_expert_bytes(const int32_t* offsets, int E, long long bytes_per_expert,
                                      long long* out, hipStream_t s) {
    hipLaunchKernelGGL(active_expert_bytes_kernel, dim3(1), dim3(kWave), 0, s, offsets, E,
                       bytes_per_expert, out);
    return hipGetLastError();
}

}  // namespace specmoe
