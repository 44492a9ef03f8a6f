// Speculation-phase expert substitution (SpecMoE Sec. 3.2 "Affinity-based expert selection
// mechanism", Fig. 8): the draft model keeps only N experts of a block resident and uses the
// target's gate unchanged; when the gate picks a non-resident expert, the resident expert that
// is closest to it in an offline table of pairwise L2 distances between the experts' parameters
// takes its place.
//
//   affinity_partial_kernel + affinity_finish_kernel : the E x E table (offline, one-time)
//   nearest_draft_kernel                             : remap[e] for one set of draft experts
//
// The routing kernel applies remap[] to the ids it writes (route_topk.hip).
//
// Table: an expert's parameters are its three matrices together, so
// D[i,j]^2 = sum over gate, up and down of (W_i - W_j)^2.  One pass streams the weights: a
// workgroup owns a block pair (8 experts x 8 experts) and a strided set of 16-byte column
// chunks, keeps the 64 running sums in fp64 registers, and leaves one partial per workgroup
// in the workspace; the finish kernel adds the partials in a fixed order (deterministic, no
// atomics).  HBM-bound for E = 8 (every weight byte is read once); for larger E the block pairs
// re-read the weights through L2 / Infinity Cache.
#include "common.h"

namespace specmoe {
namespace {

constexpr int kEB = 8;              // experts per block
constexpr int kAffGroups = 1024;    // workgroups (partials) per block pair
constexpr int kAffThreads = 256;

__host__ __device__ inline int n_blocks(int E) { return (E + kEB - 1) / kEB; }
__host__ __device__ inline int n_block_pairs(int E) { return n_blocks(E) * (n_blocks(E) + 1) / 2; }

// (I, J) with I <= J -> index in row-major order over the upper triangle
__device__ __forceinline__ int pair_index(int I, int J, int nb) {   // I <= J
    return I * nb - I * (I - 1) / 2 + (J - I);
}

template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, float (&v)[4]) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static void load(const bf16_t* p, float (&v)[8]) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// DIAG: block pairs (I, I) — only the 28 sums above the diagonal are kept (fewer registers, more
// waves in flight; for E <= 8 this is the whole table).  Otherwise blockIdx.y runs over the
// pairs I < J.
template <typename T, bool DIAG>
__global__ __launch_bounds__(kAffThreads) void affinity_partial_kernel(
    const T* __restrict__ wg, const T* __restrict__ wu, const T* __restrict__ wd, int E,
    size_t n1 /* elements of one matrix of one expert, multiple of Vec::N */,
    double* __restrict__ partial /* [pairs][kAffGroups][64] */) {
    constexpr int V = Vec<T>::N;
    const int nb = n_blocks(E);
    int I, J, bp;
    if (DIAG) {
        I = J = blockIdx.y;
        bp = pair_index(I, I, nb);
    } else {
        // blockIdx.y-th pair with I < J: skip the diagonal entries of the triangle order
        int rem = blockIdx.y, i = 0;
        while (rem >= nb - 1 - i) { rem -= nb - 1 - i; ++i; }
        I = i;
        J = i + 1 + rem;
        bp = pair_index(I, J, nb);
    }
    double acc[kEB][kEB];
#pragma unroll
    for (int i = 0; i < kEB; ++i)
#pragma unroll
        for (int j = 0; j < kEB; ++j) acc[i][j] = 0.0;

    const size_t nvec = n1 / V;
    const T* mats[3] = {wg, wu, wd};
    for (int m = 0; m < 3; ++m) {
        const T* W = mats[m];
        for (size_t q = (size_t)blockIdx.x * kAffThreads + threadIdx.x; q < nvec;
             q += (size_t)gridDim.x * kAffThreads) {
            float b[kEB][V];
#pragma unroll
            for (int j = 0; j < kEB; ++j)
                Vec<T>::load(W + (size_t)min(J * kEB + j, E - 1) * n1 + q * V, b[j]);
#pragma unroll
            for (int i = 0; i < kEB; ++i) {
                float a[V];
                if (DIAG) {
#pragma unroll
                    for (int v = 0; v < V; ++v) a[v] = b[i][v];
                } else {
                    Vec<T>::load(W + (size_t)min(I * kEB + i, E - 1) * n1 + q * V, a);
                }
#pragma unroll
                for (int j = 0; j < kEB; ++j) {
                    if (DIAG && j <= i) continue;
                    float s = 0.f;       // V squares in fp32, then one fp64 add
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float df = a[v] - b[j][v];
                        s = fmaf(df, df, s);
                    }
                    acc[i][j] += (double)s;
                }
            }
        }
    }
    // workgroup sum of the 64 values: xor butterfly per wave, then the 4 waves through LDS
    __shared__ double red[kAffThreads / kWave][kEB * kEB];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int i = 0; i < kEB; ++i)
#pragma unroll
        for (int j = 0; j < kEB; ++j) {
            if (DIAG && j <= i) {
                if (lane == 0) red[wave][i * kEB + j] = 0.0;
                continue;
            }
            const double v = wave_sum(acc[i][j]);
            if (lane == 0) red[wave][i * kEB + j] = v;
        }
    __syncthreads();
    if (threadIdx.x < kEB * kEB) {
        double v = 0.0;
        for (int w = 0; w < kAffThreads / kWave; ++w) v += red[w][threadIdx.x];
        partial[((size_t)bp * gridDim.x + blockIdx.x) * (kEB * kEB) + threadIdx.x] = v;
    }
}

// One wavefront per table entry: lane l adds partials l, l+64, ... in order, then a butterfly.
__global__ __launch_bounds__(kWave) void affinity_finish_kernel(const double* __restrict__ partial,
                                                                int E, int groups,
                                                                float* __restrict__ table) {
    const int idx = blockIdx.x;
    const int i = idx / E, j = idx % E;
    if (i == j) {
        if (threadIdx.x == 0) table[idx] = 0.f;
        return;
    }
    const int lo = min(i, j), hi = max(i, j);          // one sum serves both (i,j) and (j,i)
    const int nb = n_blocks(E);
    const int bp = pair_index(lo / kEB, hi / kEB, nb);
    const int slot = (lo % kEB) * kEB + (hi % kEB);
    double s = 0.0;
    for (int g = threadIdx.x; g < groups; g += kWave)
        s += partial[((size_t)bp * groups + g) * (kEB * kEB) + slot];
    s = wave_sum(s);
    if (threadIdx.x == 0) table[idx] = (float)sqrt(s);
}

// remap[e] = e for a draft expert, else the draft expert with the smallest D[e, .]; equal
// distances go to the lower id.  Ids outside [0, E) in draft_ids are ignored; with no valid id
// at all the map is the identity.
__global__ __launch_bounds__(256) void nearest_draft_kernel(const float* __restrict__ affinity,
                                                            int E,
                                                            const int32_t* __restrict__ draft_ids,
                                                            int n_draft,
                                                            int32_t* __restrict__ remap) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= E) return;
    int best = -1;
    float bd = 0.f;
    bool resident = false;
    for (int q = 0; q < n_draft; ++q) {
        const int dd = draft_ids[q];
        if (dd < 0 || dd >= E) continue;
        if (dd == e) resident = true;
        const float dist = affinity[(size_t)e * E + dd];
        if (best < 0 || dist < bd || (dist == bd && dd < best)) { best = dd; bd = dist; }
    }
    remap[e] = (resident || best < 0) ? e : best;
}

}  // namespace

size_t affinity_workspace_bytes(int E) {
    return (size_t)n_block_pairs(E) * kAffGroups * kEB * kEB * sizeof(double);
}

hipError_t launch_affinity_table(const void* wg, const void* wu, const void* wd, int E, int d,
                                 int f, int dtype, float* table, void* workspace, hipStream_t s) {
    const size_t n1 = (size_t)d * f;
    const int nb = n_blocks(E);
    dim3 grid_diag(kAffGroups, nb), grid_off(kAffGroups, nb * (nb - 1) / 2);
    double* partial = static_cast<double*>(workspace);
    if (dtype == 0) {
        const float *g = (const float*)wg, *u = (const float*)wu, *dn = (const float*)wd;
        hipLaunchKernelGGL((affinity_partial_kernel<float, true>), grid_diag, dim3(kAffThreads), 0,
                           s, g, u, dn, E, n1, partial);
        if (nb > 1)
            hipLaunchKernelGGL((affinity_partial_kernel<float, false>), grid_off,
                               dim3(kAffThreads), 0, s, g, u, dn, E, n1, partial);
    } else {
        const bf16_t *g = (const bf16_t*)wg, *u = (const bf16_t*)wu, *dn = (const bf16_t*)wd;
        hipLaunchKernelGGL((affinity_partial_kernel<bf16_t, true>), grid_diag, dim3(kAffThreads),
                           0, s, g, u, dn, E, n1, partial);
        if (nb > 1)
            hipLaunchKernelGGL((affinity_partial_kernel<bf16_t, false>), grid_off,
                               dim3(kAffThreads), 0, s, g, u, dn, E, n1, partial);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(affinity_finish_kernel, dim3(E * E), dim3(kWave), 0, s, partial, E,
                       kAffGroups, table);
    return hipGetLastError();
}

hipError_t launch_nearest_draft(const float* affinity, int E, const int32_t* draft_ids,
                                int n_draft, int32_t* remap, hipStream_t s) {
    hipLaunchKernelGGL(nearest_draft_kernel, dim3((E + 255) / 256), dim3(256), 0, s, affinity, E,
                       draft_ids, n_draft, remap);
    return hipGetLastError();
}

}  // namespace specmoe
