// Measured ceilings of the MI355X machine the benchmark runs on, to be quoted beside the published
// peaks: (1) the bf16 matrix instructions issued from registers with operands that change from
// one instruction to the next (the chip is power-limited, so the sustained rate depends on data
// toggling), (2) a read-only stream over a buffer far larger than every cache, (3) a
// global->LDS (LDS-DMA) stream over windows that stay resident in L2, in the two request shapes
// the expert GEMMs can produce (whole 128-byte lines, or 64-byte halves of lines).
// Measurement helpers only: a separate small library, not part of the verify-layer ABI.
#include "pipe_common.h"

namespace {

using namespace specmoe;
using namespace specmoe::pipe;

__device__ __forceinline__ bf16x8 pseudo_random_frag(unsigned s) {
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        s = s * 1664525u + 1013904223u;
        const unsigned h = s ^ (s >> 15);
        v[i] = (bf16_t)(((h & 0xffff) / 65536.0f - 0.5f) * 0.1f);
    }
    return v;
}

// clocks[0] = shader-clock cycles, clocks[1] = ticks of the constant 100 MHz counter, both over
// the loop of workgroup 0 / wave 0: their ratio is the shader clock under this load.
__device__ __forceinline__ void stamp(long long* clocks, long long c0, long long w0) {
    if (blockIdx.x == 0 && threadIdx.x == 0 && clocks) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

// 8 x 4 sub-tiles of 16x16 (the wave tile of the large-batch kernel), 32 instructions per pass
__global__ __launch_bounds__(512) void mfma16_loop(float* out, int iters, long long* clocks) {
    floatx4 acc[8][4];
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j)
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
    bf16x8 a[8], b[4];
    for (int i = 0; i < 8; ++i) a[i] = pseudo_random_frag(threadIdx.x * 131 + blockIdx.x * 7 + i);
    for (int j = 0; j < 4; ++j) b[j] = pseudo_random_frag(threadIdx.x * 17 + j * 5 + 99);
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
    stamp(clocks, c0, w0);
    float t = 0;
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j)
            for (int r = 0; r < 4; ++r) t += acc[i][j][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}

// 4 x 2 sub-tiles of 32x32, two operand sets: 16 instructions per pass
__global__ __launch_bounds__(512) void mfma32_loop(float* out, int iters, long long* clocks) {
    floatx16 acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    bf16x8 a[2][4], b[2][2];
    for (int s = 0; s < 2; ++s) {
        for (int i = 0; i < 4; ++i)
            a[s][i] = pseudo_random_frag(threadIdx.x * 131 + blockIdx.x * 7 + s * 1000 + i);
        for (int j = 0; j < 2; ++j) b[s][j] = pseudo_random_frag(threadIdx.x * 17 + s * 333 + j * 5 + 99);
    }
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[s][j], a[s][i], acc[i][j],
                                                                        0, 0, 0);
    }
    stamp(clocks, c0, w0);
    float t = 0;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int r = 0; r < 16; ++r) t += acc[i][j][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}

// read-only stream: 16 bytes per lane, 8 loads in flight per lane, grid-stride
__global__ __launch_bounds__(256) void hbm_read_loop(const U128* __restrict__ p, size_t n_vec,
                                                     U128* sink) {
    constexpr int UNROLL = 8;
    U128 acc = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 * UNROLL + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256 * UNROLL;
    for (; i + 256 * (UNROLL - 1) < n_vec; i += stride) {
        U128 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    if (acc[0] == 0x12345678u) sink[0] = acc;        // never true for the zero-filled buffer
}

// global -> LDS stream.  Every workgroup sweeps its own 256 KB window `iters` times; windows of
// workgroups on one XCD overlap inside a region small enough to stay in that XCD's L2.
// SEG = contiguous bytes per row piece: 1024 (a wave-load is 1 KB of consecutive memory), 128
// (8 rows x one whole line, rows 8 KB apart: what a BK = 64 stage asks for) or 64 (16 rows x half
// a line: a BK = 32 stage).
// NT: the loads carry the non-temporal hint (data read once).
template <int SEG, bool NT = false>
__global__ __launch_bounds__(512) void l2_lds_loop(const unsigned char* __restrict__ buf,
                                                   size_t region_bytes, int iters) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
    const uint32_t lds_base =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_raw;
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    constexpr uint32_t kWindow = 256u << 10, kPitch = 8192;       // window = 32 rows of 8 KB
    const unsigned char* base = uniform_ptr(buf + ((size_t)blockIdx.x * kWindow) % region_bytes);
    // lane -> byte offset inside the window for wave-load number q of a sweep
    constexpr int LPR = SEG / 16, RPL = kWave / LPR;               // lanes per row piece, rows per load
    const uint32_t lane_off = SEG == 1024 ? (uint32_t)lane * 16u
                                          : (uint32_t)(lane / LPR) * kPitch + (uint32_t)(lane % LPR) * 16u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll 1
        for (uint32_t q0 = 0; q0 < kWindow / 1024; q0 += 32) {     // 4 wave-loads per wave
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t q = q0 + u * 8 + wave;              // wave-load index in the window
                uint32_t off;
                if (SEG == 1024) {
                    off = q * 1024u;
                } else {
                    // RPL rows x SEG bytes: row block (q % (32 / RPL)), column piece q / (32 / RPL)
                    constexpr uint32_t RB = 32 / RPL;
                    off = (q % RB) * RPL * kPitch + (q / RB) * SEG;
                }
                if (NT) dma16_nt(base, off + lane_off, lds_base + ((u * 8 + wave) * 1024u));
                else dma16(base, off + lane_off, lds_base + ((u * 8 + wave) * 1024u));
            }
            wait_vmcnt<8>();
        }
    }
    wait_vmcnt<0>();
}

// ds_read_b128 throughput of one CU for a given lane -> byte-offset pattern: 8 wavefronts, each
// issues 8 reads (4 KB apart) per pass.  pattern 0: lane * 16 (consecutive, conflict-free by
// construction); 1: the fragment read of the large-batch expert GEMM (row lane%16 of a 64-byte-row
// tile, chunk (lane/16) ^ ((row/2)%4)); 2: lane * 256 (every lane in the same banks); 3: as 1 with
// the term (row/4)%4 (one sweep over the bank groups per 4 rows): a 2-way conflict on gfx950.
// clocks[0] = shader cycles of the timed loop of wave 0.
__global__ __launch_bounds__(512) void lds_read_loop(int pattern, int iters, long long* clocks,
                                                     U128* sink) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
    const int lane = threadIdx.x % kWave;
    for (int i = threadIdx.x; i < 65536 / 16; i += blockDim.x)
        reinterpret_cast<U128*>(lds_raw)[i] = U128{(uint32_t)i, 1, 2, 3};
    __syncthreads();
    int off;
    if (pattern == 0) off = lane * 16;
    else if (pattern == 1) off = (lane & 15) * 64 + (((lane >> 4) ^ (((lane & 15) / 2) % 4)) << 4);
    else if (pattern == 3) off = (lane & 15) * 64 + (((lane >> 4) ^ (((lane & 15) / 4) % 4)) << 4);
    else off = lane * 256;
    U128 acc = {0, 0, 0, 0};
    const uint32_t lds_off =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_raw + (uint32_t)off;
    const long long c0 = clock64();
    for (int it = 0; it < iters; ++it) {
        U128 r[8];
        asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:4096\n\t"
                     "ds_read_b128 %2, %8 offset:8192\n\tds_read_b128 %3, %8 offset:12288\n\t"
                     "ds_read_b128 %4, %8 offset:16384\n\tds_read_b128 %5, %8 offset:20480\n\t"
                     "ds_read_b128 %6, %8 offset:24576\n\tds_read_b128 %7, %8 offset:28672\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=v"(r[0]), "=v"(r[1]), "=v"(r[2]), "=v"(r[3]), "=v"(r[4]), "=v"(r[5]),
                       "=v"(r[6]), "=v"(r[7])
                     : "v"(lds_off)
                     : "memory");
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= r[u];
    }
    __syncthreads();
    if (threadIdx.x == 0 && clocks) clocks[0] = clock64() - c0;
    sink[threadIdx.x] = acc;
}

}  // namespace

extern "C" {

// One workgroup of 8 wavefronts; `sink` holds 512 x 16 bytes.  clocks[0] / (iters * 64) is the
// number of shader cycles the CU spends per ds_read_b128 wave-instruction.
int specmoe_peak_lds_read(int pattern, int iters, long long* clocks, void* sink, void* stream) {
    if (!sink || iters < 1 || pattern < 0 || pattern > 3) return 1;
    hipLaunchKernelGGL(lds_read_loop, dim3(1), dim3(512), 65536, (hipStream_t)stream, pattern,
                       iters, clocks, (U128*)sink);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

// kind 0: v_mfma_f32_16x16x32_bf16, kind 1: v_mfma_f32_32x32x16_bf16.  `out` holds
// blocks*512 floats, `clocks` two long longs (may be NULL).  Returns the flops of the launch
// through *flops.
int specmoe_peak_mfma(int kind, int blocks, int iters, float* out, long long* clocks,
                      double* flops, void* stream) {
    if (!out || blocks < 1 || iters < 1 || (kind != 0 && kind != 1)) return 1;
    hipStream_t s = (hipStream_t)stream;
    if (kind == 0) {
        hipLaunchKernelGGL(mfma16_loop, dim3(blocks), dim3(512), 0, s, out, iters, clocks);
        if (flops) *flops = (double)blocks * 8 * iters * 32 * 16384.0;
    } else {
        hipLaunchKernelGGL(mfma32_loop, dim3(blocks), dim3(512), 0, s, out, iters, clocks);
        if (flops) *flops = (double)blocks * 8 * iters * 16 * 32768.0;
    }
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

// Streams `bytes` (multiple of 16) from `buf` once; `sink` is 16 bytes of device memory.
int specmoe_peak_hbm_read(const void* buf, size_t bytes, int blocks, void* sink, void* stream) {
    if (!buf || !sink || blocks < 1 || bytes < 16) return 1;
    hipLaunchKernelGGL(hbm_read_loop, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const U128*)buf, bytes / 16, (U128*)sink);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

// `region_bytes` (multiple of 256 KB, at most the buffer size) is the part of `buf` the
// windows wrap around in; seg = 1024, 128 or 64.  Bytes moved = blocks * iters * 256 KB.
int specmoe_peak_l2_lds(const void* buf, size_t region_bytes, int blocks, int iters, int seg,
                        void* stream) {
    if (!buf || blocks < 1 || iters < 1 || region_bytes < (256u << 10) ||
        region_bytes % (256u << 10) != 0)
        return 1;
    hipStream_t s = (hipStream_t)stream;
    const unsigned char* b = (const unsigned char*)buf;
    if (seg == 1024) hipLaunchKernelGGL(l2_lds_loop<1024>, dim3(blocks), dim3(512), 32768, s, b, region_bytes, iters);
    else if (seg == 128) hipLaunchKernelGGL(l2_lds_loop<128>, dim3(blocks), dim3(512), 32768, s, b, region_bytes, iters);
    else if (seg == 64) hipLaunchKernelGGL(l2_lds_loop<64>, dim3(blocks), dim3(512), 32768, s, b, region_bytes, iters);
    else return 1;
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

// The 1024-byte-piece stream of specmoe_peak_l2_lds with the non-temporal hint on the loads.
int specmoe_peak_l2_lds_nt(const void* buf, size_t region_bytes, int blocks, int iters,
                           void* stream) {
    if (!buf || blocks < 1 || iters < 1 || region_bytes < (256u << 10) ||
        region_bytes % (256u << 10) != 0)
        return 1;
    hipLaunchKernelGGL((l2_lds_loop<1024, true>), dim3(blocks), dim3(512), 32768,
                       (hipStream_t)stream, (const unsigned char*)buf, region_bytes, iters);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

}  // extern "C"
