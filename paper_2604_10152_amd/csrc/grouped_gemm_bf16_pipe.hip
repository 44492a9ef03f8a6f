// Large-batch expert GEMMs on the gfx950 matrix cores: multi-stage LDS ring filled by
// direct global->LDS loads, MFMA fragments double-buffered in registers.
// (SpecMoE Sec. 2.1: only the rows routed to an expert meet its FFN-sized weights;
// Sec. 2.2: verification brings all B*(gamma+1) tokens at once, so each expert sees hundreds
// of rows and the contraction is MFMA-bound.)
//
// One workgroup = BM rows of one expert x BN weight rows.  Per step of BK contraction
// elements every wave issues its share of `global_load_lds_dwordx4` instructions: 64 lanes x
// 16 bytes go straight from L2/HBM into 1 KB of LDS, no staging registers, no ds_write.  The
// lane -> global chunk map carries the bank swizzle, so the LDS image is the swizzled tile.
// STAGES buffers form a ring; a stage is requested STAGES-1 steps before it is multiplied and
// must have landed one step before (vmcnt + one barrier per step), which leaves STAGES-2
// steps of MFMA work to cover the HBM latency.  Because readiness is established one step
// ahead, the first fragments of the next stage are read before the barrier and the matrix
// pipe does not drain at step boundaries.
//
// The loads are inline assembly on purpose: the compiler would otherwise put vmcnt(0) in
// front of every LDS read that follows an LDS-DMA load, which collapses the ring to depth 1.
// Hand-placed s_waitcnt vmcnt(n) is safe next to compiler-generated waits: extra outstanding
// loads can only make a compiler-chosen wait stricter, never weaker.
#include "common.h"
#include "tile_map.h"

#include <type_traits>

namespace specmoe {
namespace {

template <int BM_, int BN_, int BK_, int STAGES_, int WM_, int WN_, bool SWIGLU_, int KROT_ = 0>
struct PipeCfg {
    static constexpr int KROT = KROT_;               // k-loop rotation per n-tile, in steps
    static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_, WM = WM_, WN = WN_;
    static constexpr bool SWIGLU = SWIGLU_;
    static constexpr int NWAVES = WM * WN, THREADS = NWAVES * kWave;
    static constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);   // 32x32 sub-tiles per wave
    static constexpr int KK = BK / 16;                               // MFMA k-steps per stage
    static constexpr int ROW_BYTES = BK * 2, CHUNKS = BK / 8;        // 16-byte chunks per row
    static constexpr int RPG = 16 / CHUNKS;          // tile rows per sweep over the 16 bank groups
    static constexpr int ROWS_PER_DMA = 1024 / ROW_BYTES;            // rows one wave-load fills
    static constexpr int A_PW = BM / ROWS_PER_DMA / NWAVES;          // wave-loads per wave, A
    static constexpr int B_PW = BN / ROWS_PER_DMA / NWAVES;          // wave-loads per wave, B
    static constexpr int G = A_PW + B_PW;                            // loads per thread per stage
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE_BYTES;
    static constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(KK % 2 == 0, "fragment double buffer needs an even number of k-steps");
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "tile / wave grid mismatch");
    static_assert(BM % (ROWS_PER_DMA * NWAVES) == 0 && BN % (ROWS_PER_DMA * NWAVES) == 0,
                  "wave-loads must divide evenly");
    static_assert(!SWIGLU || ((BN / 2 / ROWS_PER_DMA) % NWAVES == 0 && TN % 2 == 0),
                  "gate/up halves must split on a wave-load round and pair up inside a wave");
    static_assert(STAGES >= 3 && (STAGES - 3) * G <= 63, "ring depth");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

// byte offset of 16-byte chunk c of tile row r: conflict-free for 128-bit accesses on the
// 64-bank LDS (16 consecutive lanes = 16 consecutive rows must hit 16 different bank groups)
template <typename C>
__device__ __forceinline__ int swz(int r, int c) {
    return r * C::ROW_BYTES + ((c ^ ((r / C::RPG) % C::CHUNKS)) << 4);
}

// 64 lanes x 16 bytes: global (uniform base + per-lane byte offset) -> LDS [lds_addr, +1024)
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(gbase), "s"(lds_addr) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// PROBE is 0 in the library.  The tuning harness instantiates 1 (matrix instructions
// removed) and 2 (global->LDS loads removed) to time the two halves of the pipeline alone.
template <typename C, int PROBE = 0>
__global__ __launch_bounds__(C::THREADS) void grouped_gemm_bf16_pipe_kernel(
    const bf16_t* __restrict__ A,        // [n_rows, K]
    const int32_t* __restrict__ offsets, // [E+1]
    const bf16_t* __restrict__ W0,       // [E, N, K]   (gate, or down)
    const bf16_t* __restrict__ W1,       // [E, N, K]   (up; SWIGLU only)
    int E, int N, int K, bf16_t* __restrict__ Cout /* [n_rows, N] */) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];

    const int NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    TileLoc t;
    if (!locate_tile<C::BM>(offsets, E, NT, blockIdx.x, t)) return;
    const int row0 = t.row0, tile_rows = t.tile_rows;
    const int n0 = t.nt * C::BN_OUT;
    const int nsub = (tile_rows + 31) / 32;

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave % C::WM, wn = wave / C::WM;
    const uint32_t lds_base =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_raw;

    // ---- global side of the wave-loads -------------------------------------------------
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(A + (size_t)row0 * K);
    const size_t wrow = (size_t)t.expert * N + min(n0, N - 1);
    const unsigned char* w0 = reinterpret_cast<const unsigned char*>(W0 + wrow * K);
    const unsigned char* w1 = C::SWIGLU ? reinterpret_cast<const unsigned char*>(W1 + wrow * K)
                                        : nullptr;
    const int n_left = N - n0;
    uint32_t a_off[C::A_PW], b_off[C::B_PW];
    {
        const int srow = lane / C::CHUNKS, pc = lane % C::CHUNKS;   // LDS slot of this lane
#pragma unroll
        for (int jj = 0; jj < C::A_PW; ++jj) {
            const int r = (wave + jj * C::NWAVES) * C::ROWS_PER_DMA + srow;
            const int c = pc ^ ((r / C::RPG) % C::CHUNKS);
            a_off[jj] = (uint32_t)((min(r, tile_rows - 1) * K + c * 8) * 2);
        }
#pragma unroll
        for (int jj = 0; jj < C::B_PW; ++jj) {
            const int r = (wave + jj * C::NWAVES) * C::ROWS_PER_DMA + srow;
            const int c = pc ^ ((r / C::RPG) % C::CHUNKS);
            const int rn = (C::SWIGLU && r >= C::BN / 2) ? r - C::BN / 2 : r;
            b_off[jj] = (uint32_t)((min(rn, n_left - 1) * K + c * 8) * 2);
        }
    }
    const int KT = K / C::BK;
    // Every tile row is K*2 bytes apart, a multiple of the 4 KB period of the L2 channel
    // interleave for the shapes of interest, so all rows of all tiles at one k offset sit in
    // the same channel.  Workgroups start together; without a stagger they would sweep the
    // channels in lockstep.  The k loop is therefore rotated by an amount that depends on the
    // n-tile only (m-tiles sharing a weight tile stay aligned and still meet in L2).
    const int kt0 = (int)(((long long)t.nt * C::KROT) % KT);
    auto issue_stage = [&](int kt, int buf) __attribute__((always_inline)) {
        int kq = min(kt, KT - 1) + kt0;                             // clamped: tail re-loads
        kq = kq >= KT ? kq - KT : kq;
        const size_t kb = (size_t)kq * C::ROW_BYTES;
        const uint32_t sbase = lds_base + (uint32_t)buf * C::STAGE_BYTES + wave * 1024u;
        if (PROBE == 2 && kt >= C::STAGES - 1) return;
#pragma unroll
        for (int jj = 0; jj < C::A_PW; ++jj)
            dma16(a_base + kb, a_off[jj], sbase + jj * C::NWAVES * 1024u);
#pragma unroll
        for (int jj = 0; jj < C::B_PW; ++jj) {
            const bool up = C::SWIGLU && (jj * C::NWAVES * C::ROWS_PER_DMA >= C::BN / 2);
            dma16((up ? w1 : w0) + kb, b_off[jj], sbase + C::A_BYTES + jj * C::NWAVES * 1024u);
        }
    };

    // ---- LDS side of the fragment reads ---------------------------------------------------
    // A sub-tile i: tile rows 32*(wm + WM*i) + lane%32 ; B sub-tile j: weight rows nb(j) + lane%32.
    // Sub-tile bases are multiples of 32 rows, which leaves the swizzle term unchanged, so one
    // per-lane offset per k-step serves all sub-tiles through immediate offsets.
    int a_rd[C::KK], b_rd[C::KK];
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk) {
        const int c = kk * 2 + (lane >> 5);
        a_rd[kk] = swz<C>(32 * wm + (lane & 31), c);
        b_rd[kk] = C::A_BYTES + swz<C>((lane & 31), c);
    }
    auto nb = [&](int j) __attribute__((always_inline)) -> int {     // B sub-tile base row
        if (C::SWIGLU) {
            constexpr int H = C::TN / 2;
            return (j < H) ? 32 * (wn * H + j) : C::BN / 2 + 32 * (wn * H + (j - H));
        }
        return 32 * (wn * C::TN + j);
    };

    const int ta = min(C::TM, max(0, (nsub - wm + C::WM - 1) / C::WM));   // active sub-tiles

    auto run = [&](auto ta_tag) __attribute__((always_inline)) {
        constexpr int TA = decltype(ta_tag)::value;
        constexpr int TAX = TA > 0 ? TA : 1;
        floatx16 acc[TAX][C::TN];
#pragma unroll
        for (int i = 0; i < TA; ++i)
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        bf16x8 af[2][TAX], bfr[2][C::TN];
        auto read_frags = [&](int set, int buf, int kk) __attribute__((always_inline)) {
            if (TA == 0) return;
            const unsigned char* sb = lds_raw + buf * C::STAGE_BYTES;
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
                bfr[set][j] = *reinterpret_cast<const bf16x8*>(sb + b_rd[kk] + nb(j) * C::ROW_BYTES);
#pragma unroll
            for (int i = 0; i < TA; ++i)
                af[set][i] = *reinterpret_cast<const bf16x8*>(sb + a_rd[kk] +
                                                               32 * C::WM * i * C::ROW_BYTES);
        };
        auto mfma_set = [&](int set) __attribute__((always_inline)) {
            if (PROBE == 1) {                      // keep the fragment reads alive, no MFMA
#pragma unroll
                for (int i = 0; i < TA; ++i)
                    asm volatile("" :: "v"(af[set][i]));
#pragma unroll
                for (int j = 0; j < C::TN; ++j)
                    asm volatile("" :: "v"(bfr[set][j]));
                return;
            }
#pragma unroll
            for (int i = 0; i < TA; ++i)
#pragma unroll
                for (int j = 0; j < C::TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bfr[set][j],
                                                                        acc[i][j], 0, 0, 0);
        };

        // prologue: request stages 0 .. STAGES-2, wait for 0 and 1
#pragma unroll
        for (int s = 0; s < C::STAGES - 1; ++s) issue_stage(s, s);
        wait_vmcnt<(C::STAGES - 3) * C::G>();
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);

        int buf = 0;                               // ring slot of stage kt
        for (int kt = 0; kt < KT; ++kt) {
            const int buf_next = (buf + 1 == C::STAGES) ? 0 : buf + 1;
            const int buf_free = (buf == 0) ? C::STAGES - 1 : buf - 1;   // held stage kt-1
            issue_stage(kt + C::STAGES - 1, buf_free);
#pragma unroll
            for (int kk = 0; kk < C::KK; ++kk) {
                if (kk + 1 < C::KK) read_frags((kk + 1) & 1, buf, kk + 1);
                else read_frags(0, buf_next, 0);   // stage kt+1 landed one step ago
                // the scheduler must not sink the next k-step's fragment reads below the
                // matrix instructions they are meant to overlap with
                __builtin_amdgcn_sched_barrier(0);
                mfma_set(kk & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            wait_vmcnt<(C::STAGES - 3) * C::G>();  // own share of stage kt+2 has landed
            __builtin_amdgcn_s_barrier();
            buf = buf_next;
        }
        wait_vmcnt<0>();                           // no load may outlive the workgroup's LDS

        // epilogue: accumulator element r of a lane is row 8*(r/4) + 4*(lane/32) + r%4,
        // column lane%32 of its 32x32 sub-tile
        const int col_in = lane & 31, khalf = lane >> 5;
#pragma unroll
        for (int i = 0; i < TA; ++i) {
            const int rbase = 32 * (wm + C::WM * i) + 4 * khalf;
            if (C::SWIGLU) {
                constexpr int H = C::TN / 2;
#pragma unroll
                for (int j = 0; j < H; ++j) {
                    const int col = n0 + 32 * (wn * H + j) + col_in;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = rbase + 8 * (r / 4) + (r % 4);
                        if (row < tile_rows && col < N) {
                            const float g = acc[i][j][r], u = acc[i][j + H][r];
                            Cout[(size_t)(row0 + row) * N + col] = (bf16_t)(silu_f32(g) * u);
                        }
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < C::TN; ++j) {
                    const int col = n0 + 32 * (wn * C::TN + j) + col_in;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = rbase + 8 * (r / 4) + (r % 4);
                        if (row < tile_rows && col < N)
                            Cout[(size_t)(row0 + row) * N + col] = (bf16_t)acc[i][j][r];
                    }
                }
            }
        }
    };

    static_assert(C::TM <= 4, "extend the dispatch below");
    switch (ta) {
        case 0: run(std::integral_constant<int, 0>{}); break;
        case 1: run(std::integral_constant<int, 1>{}); break;
        case 2: if constexpr (C::TM >= 2) run(std::integral_constant<int, 2>{}); break;
        case 3: if constexpr (C::TM >= 3) run(std::integral_constant<int, 3>{}); break;
        default: if constexpr (C::TM >= 4) run(std::integral_constant<int, 4>{}); break;
    }
}

template <typename C>
hipError_t launch_pipe(const bf16_t* A, const int32_t* offsets, const bf16_t* W0,
                       const bf16_t* W1, int n_rows, int E, int N, int K, bf16_t* Cout,
                       hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&grouped_gemm_bf16_pipe_kernel<C>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long long NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    const long long grid = grid_upper_bound(n_rows, E, C::BM, NT);
    hipLaunchKernelGGL(grouped_gemm_bf16_pipe_kernel<C>, dim3((unsigned)grid), dim3(C::THREADS),
                       C::LDS_BYTES, s, A, offsets, W0, W1, E, N, K, Cout);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_expert_up_bf16_large(const bf16_t* x_perm, const int32_t* offsets,
                                       const bf16_t* wg, const bf16_t* wu, int n_rows, int d,
                                       int f, int E, bf16_t* h, hipStream_t s) {
    return launch_pipe<PipeCfg<256, 256, 32, 4, 2, 4, true>>(x_perm, offsets, wg, wu, n_rows, E, f,
                                                             d, h, s);
}

hipError_t launch_expert_down_bf16_large(const bf16_t* h, const int32_t* offsets,
                                         const bf16_t* wd, int n_rows, int d, int f, int E,
                                         bf16_t* y, hipStream_t s) {
    return launch_pipe<PipeCfg<256, 256, 32, 4, 2, 4, false>>(h, offsets, wd, nullptr, n_rows, E,
                                                              d, f, y, s);
}

}  // namespace specmoe
