// Expert GEMMs for few to a few hundred rows per expert on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16): multi-stage LDS ring filled by direct global->LDS loads, MFMA
// fragments double-buffered in registers.
// (SpecMoE Sec. 2.1: only the rows routed to an expert meet its FFN-sized weights; with a
// small verification batch - Sec. 2.2 - an expert sees tens of rows and the kernel is bound
// by streaming its weights from HBM once.)
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
#include "pipe_common.h"

#include <type_traits>

namespace specmoe {
namespace {

using namespace pipe;

template <typename C>
__global__ __launch_bounds__(C::THREADS) void grouped_gemm_bf16_pipe_kernel(
    const bf16_t* __restrict__ A,        // [n_rows, K]
    const int32_t* __restrict__ offsets, // [E+1]
    const bf16_t* __restrict__ W0,       // [E, N, K]   (gate, or down)
    const bf16_t* __restrict__ W1,       // [E, N, K]   (up; SWIGLU only)
    int E, int N, int K, bf16_t* __restrict__ Cout /* [n_rows, N] */,
    const int32_t* __restrict__ row_src /* nullable: A row r is A[row_src[r] / topk] */, int topk) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];

    const int NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    TileLoc t;
    if (!locate_tile_even<C::BM>(offsets, E, NT, blockIdx.x, t)) return;
    const int row0 = t.row0, tile_rows = t.tile_rows;
    const int n0 = t.nt * C::BN_OUT;
    const int nsub = (tile_rows + 31) / 32;

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    // Waves w and w+4 share a SIMD.  Giving them different wm means a tile with an odd number
    // of 32-row sub-tiles loads every SIMD equally (5+4 instead of 5+5 and 4+4).
    const int wm = wave / C::WN, wn = wave % C::WN;
    const uint32_t lds_base =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_raw;

    // ---- global side of the wave-loads -------------------------------------------------
    // with row_src the activation rows are gathered on the fly (A is then the token matrix)
    const unsigned char* a_base = uniform_ptr(
        reinterpret_cast<const unsigned char*>(A + (row_src ? (size_t)0 : (size_t)row0 * K)));
    const size_t wrow = (size_t)t.expert * N + min(n0, N - 1);
    const unsigned char* w0 = uniform_ptr(reinterpret_cast<const unsigned char*>(W0 + wrow * K));
    const unsigned char* w1 =
        C::SWIGLU ? uniform_ptr(reinterpret_cast<const unsigned char*>(W1 + wrow * K)) : nullptr;
    const int n_left = N - n0;
    uint32_t a_off[C::A_PW], b_off[C::B_PW];
    int a_cnt = 0;                               // A wave-loads this wave issues per stage
    {
        const int srow = lane / C::CHUNKS, pc = lane % C::CHUNKS;   // LDS slot of this lane
#pragma unroll
        for (int jj = 0; jj < C::A_PW; ++jj) {
            const int r = (wave + jj * C::NWAVES) * C::ROWS_PER_DMA + srow;
            const int c = pc ^ ((r / C::RPG) % C::CHUNKS);
            const int rr = min(r, tile_rows - 1);
            const unsigned arow = row_src ? (unsigned)(row_src[row0 + rr] / topk) : (unsigned)rr;
            a_off[jj] = (arow * (unsigned)K + (unsigned)(c * 8)) * 2u;
            // this wave's A loads: wave-load j = wave + jj*NWAVES covers tile rows j*16.. ;
            // only loads that hold at least one real row are issued
            if ((wave + jj * C::NWAVES) * C::ROWS_PER_DMA < tile_rows) a_cnt = jj + 1;
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
    // One wave-load of stage kt into ring slot buf.  Loads 0 .. A_PW-1 are this wave's A rows
    // (issued only if they hold real rows), loads A_PW .. A_PW+B_PW-1 its weight rows.
    // nt_tag: the weight loads carry the non-temporal hint (tiles whose weights no other
    // workgroup reads)
    auto issue_one = [&](auto nt_tag, int which, int kt, int buf) __attribute__((always_inline)) {
        const size_t kb = (size_t)min(kt, KT - 1) * C::ROW_BYTES;   // clamped: tail re-loads
        const uint32_t sbase = lds_base + (uint32_t)buf * C::STAGE_BYTES + wave * 1024u;
#pragma unroll
        for (int jj = 0; jj < C::A_PW; ++jj)
            if (which == jj && jj < a_cnt)
                dma16(a_base + kb, a_off[jj], sbase + jj * C::NWAVES * 1024u);
#pragma unroll
        for (int jj = 0; jj < C::B_PW; ++jj) {
            const bool up = C::SWIGLU && (jj * C::NWAVES * C::ROWS_PER_DMA >= C::BN / 2);
            if (which == C::A_PW + jj) {
                if (decltype(nt_tag)::value)
                    dma16_nt((up ? w1 : w0) + kb, b_off[jj],
                             sbase + C::A_BYTES + jj * C::NWAVES * 1024u);
                else
                    dma16((up ? w1 : w0) + kb, b_off[jj],
                          sbase + C::A_BYTES + jj * C::NWAVES * 1024u);
            }
        }
    };
    auto issue_stage = [&](auto nt_tag, int kt, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < C::G_MAX; ++q) issue_one(nt_tag, q, kt, buf);
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
    // loads this wave has in flight per stage; stages STAGES-3 deep may still be outstanding
    // when the stage needed next must have landed
    const int vm_allow = (C::STAGES - 3) * (a_cnt + C::B_PW);

    auto run = [&](auto ta_tag, auto nt_tag) __attribute__((always_inline)) {
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
        auto mfma_row = [&](int set, int i) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[set][j], af[set][i],
                                                                    acc[i][j], 0, 0, 0);
        };

        // prologue: request stages 0 .. STAGES-2, wait for 0 and 1
#pragma unroll
        for (int s = 0; s < C::STAGES - 1; ++s) issue_stage(nt_tag, s, s);
        wait_vmcnt_dyn(vm_allow);
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);

        int buf = 0;                               // ring slot of stage kt
        for (int kt = 0; kt < KT; ++kt) {
            const int buf_next = (buf + 1 == C::STAGES) ? 0 : buf + 1;
            const int buf_free = (buf == 0) ? C::STAGES - 1 : buf - 1;   // held stage kt-1
            // The requests for stage kt+STAGES-1 go out one at a time between the matrix
            // instructions of the first k-step (all eight waves leave the barrier together; a
            // burst of wave-loads would back up the address unit and hold the MFMAs behind it).
            // sched_barrier(0) pins this order: the compiler's scheduler would otherwise sink
            // the fragment reads next to their use and bunch the loads.
#pragma unroll
            for (int kk = 0; kk < C::KK; ++kk) {
                if (kk + 1 < C::KK) read_frags((kk + 1) & 1, buf, kk + 1);
                else read_frags(0, buf_next, 0);         // stage kt+1 landed one step ago
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < TAX; ++i) {
                    if (i < TA) mfma_row(kk & 1, i);
                    __builtin_amdgcn_sched_barrier(0);
                    if (kk == 0) {
                        if (i < C::G_MAX) issue_one(nt_tag, i, kt + C::STAGES - 1, buf_free);
                        if (i == TAX - 1)
#pragma unroll
                            for (int q = TAX; q < C::G_MAX; ++q)
                                issue_one(nt_tag, q, kt + C::STAGES - 1, buf_free);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            wait_vmcnt_dyn(vm_allow);              // own share of stage kt+2 has landed
            __builtin_amdgcn_s_barrier();
            buf = buf_next;
        }
        wait_vmcnt<0>();                           // no load may outlive the workgroup's LDS

        // epilogue.  The matrix instruction is issued as (weights x activations^T), so a lane
        // holds ONE tile row (lane%32) and, for each g = r/4, four consecutive output columns
        // 8g + 4*(lane/32) + r%4, i.e. 8 bytes of bf16.
        //  - SwiGLU tile (BN/2 = 128 output columns, written once per n-tile of every row
        //    block: the h matrix is 117 MB at the large-batch shape): the 8-byte pieces go to an
        //    LDS image of the tile and the workgroup then writes whole 256-byte rows.
        //  - plain tile: 8-byte stores straight to global memory (y is small).
        const int row = lane & 31, chalf = (lane >> 5) * 4;
        if (C::SWIGLU) __builtin_amdgcn_s_barrier();   // every wave's loads have landed: LDS is free
#pragma unroll
        for (int i = 0; i < TA; ++i) {
            const int trow = 32 * (wm + C::WM * i) + row;
            if (!C::SWIGLU && trow >= tile_rows) continue;
            bf16_t* crow = Cout + (size_t)(row0 + trow) * N;
            constexpr int JN = C::SWIGLU ? C::TN / 2 : C::TN;
#pragma unroll
            for (int j = 0; j < JN; ++j) {
                const int ctile = 32 * (wn * JN + j) + chalf;     // column inside the tile
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (C::SWIGLU) {
                            const float gt = acc[i][j][4 * g + q], up = acc[i][j + JN][4 * g + q];
                            v[q] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * up;
                        } else {
                            v[q] = acc[i][j][4 * g + q];
                        }
                    }
                    const uint2 pk = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
                    if (C::SWIGLU) {
                        *reinterpret_cast<uint2*>(lds_raw + trow * kStageRowBytes +
                                                  (ctile + 8 * g) * 2) = pk;
                    } else {
                        const int col = n0 + ctile + 8 * g;
                        if (col + 3 < N) {
                            *reinterpret_cast<uint2*>(crow + col) = pk;
                        } else {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (col + q < N) crow[col + q] = (bf16_t)v[q];
                        }
                    }
                }
            }
        }
    };

    static_assert(C::TM <= 5, "extend the dispatch below");
    // An expert with a single m-tile: every weight tile of it is read by exactly one workgroup,
    // once - a pure stream out of HBM, which the non-temporal hint speeds up (6.3 vs 5.7 TB/s on a
    // plain LDS-DMA stream).  With several m-tiles the workgroups that share a weight tile meet
    // in the L2, and the hint would cost those hits.
    // (whole 128-byte lines per row and stage only: half-line loads rely on the L2 keeping the
    // other half for the next stage)
    const bool w_once = C::ROW_BYTES >= 128 && t.mt == 1 && (!C::SWIGLU || tile_rows <= 64);
    auto run_sel = [&](auto ta_tag) __attribute__((always_inline)) {
        if (w_once) run(ta_tag, std::true_type{});
        else run(ta_tag, std::false_type{});
    };
    switch (ta) {
        case 0: run_sel(std::integral_constant<int, 0>{}); break;
        case 1: run_sel(std::integral_constant<int, 1>{}); break;
        case 2: if constexpr (C::TM >= 2) run_sel(std::integral_constant<int, 2>{}); break;
        case 3: if constexpr (C::TM >= 3) run_sel(std::integral_constant<int, 3>{}); break;
        case 4: if constexpr (C::TM >= 4) run_sel(std::integral_constant<int, 4>{}); break;
        default: if constexpr (C::TM >= 5) run_sel(std::integral_constant<int, 5>{}); break;
    }

    if (C::SWIGLU) {
        // cooperative write-out of the staged tile: 16 bytes per lane, whole rows
        static_assert(!C::SWIGLU || (size_t)C::BM * kStageRowBytes <= C::LDS_BYTES, "stage tile");
        __builtin_amdgcn_s_barrier();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        constexpr int CPR = C::BN_OUT / 8;                  // 16-byte chunks per tile row
        constexpr int RPP = C::THREADS / CPR;               // rows per pass
        const int cr = tid / CPR, cc = tid % CPR;
        const int col = n0 + cc * 8;
        for (int r = cr; r < tile_rows; r += RPP) {
            const U128 v = *reinterpret_cast<const U128*>(lds_raw + r * kStageRowBytes + cc * 16);
            bf16_t* dst = Cout + (size_t)(row0 + r) * N + col;
            if (col + 7 < N) {
                *reinterpret_cast<U128*>(dst) = v;
            } else {
                for (int q = 0; q < 8; ++q)
                    if (col + q < N) dst[q] = reinterpret_cast<const bf16_t*>(&v)[q];
            }
        }
    }
}

template <typename C>
hipError_t launch_pipe(const bf16_t* A, const int32_t* offsets, const bf16_t* W0,
                       const bf16_t* W1, int n_rows, int E, int N, int K, bf16_t* Cout,
                       hipStream_t s, const int32_t* row_src = nullptr, int topk = 1) {
    // one-time, thread-safe (C++11 static initialisation): raise the dynamic LDS limit
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&grouped_gemm_bf16_pipe_kernel<C>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
    if (attr != hipSuccess) return attr;
    const long long NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    const long long grid = grid_upper_bound(n_rows, E, C::BM, NT);
    hipLaunchKernelGGL(grouped_gemm_bf16_pipe_kernel<C>, dim3((unsigned)grid), dim3(C::THREADS),
                       C::LDS_BYTES, s, A, offsets, W0, W1, E, N, K, Cout, row_src, topk);
    return hipGetLastError();
}

}  // namespace

// Few rows per expert: the weights stream from HBM once and nothing else matters.  64-row
// tiles, narrow N so that every CU owns a stream, 128-byte rows per step (BK = 64; 64-byte rows
// lose ~10 % of HBM throughput) and a 4 / 6 stage ring (~70-120 KB of requests in flight per CU).
hipError_t launch_expert_up_bf16_small(const bf16_t* x_perm, const int32_t* offsets,
                                       const bf16_t* wg, const bf16_t* wu, int n_rows, int d,
                                       int f, int E, bf16_t* h, hipStream_t s,
                                       const int32_t* row_src, int topk) {
    return launch_pipe<PipeCfg<64, 128, 64, 4, 1, 2, true>>(x_perm, offsets, wg, wu, n_rows, E, f,
                                                            d, h, s, row_src, topk);
}

hipError_t launch_expert_down_bf16_small(const bf16_t* h, const int32_t* offsets,
                                         const bf16_t* wd, int n_rows, int d, int f, int E,
                                         bf16_t* y, hipStream_t s) {
    return launch_pipe<PipeCfg<64, 128, 64, 6, 1, 4, false>>(h, offsets, wd, nullptr, n_rows, E,
                                                              d, f, y, s);
}

// In between (tens to a few hundred rows per expert, e.g. 16 experts with top-1 routing), down
// projection: still bound by streaming the weights, but 64-row tiles would re-read them several
// times through L2.  128-row tiles, 128-byte rows per step, 4-stage ring (128 KB).
hipError_t launch_expert_down_bf16_mid(const bf16_t* h, const int32_t* offsets, const bf16_t* wd,
                                       int n_rows, int d, int f, int E, bf16_t* y,
                                       hipStream_t s) {
    return launch_pipe<PipeCfg<128, 128, 64, 4, 2, 4, false>>(h, offsets, wd, nullptr, n_rows, E,
                                                              d, f, y, s);
}

}  // namespace specmoe
