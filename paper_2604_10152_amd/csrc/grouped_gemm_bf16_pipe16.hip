// Large- and mid-batch expert GEMMs (tiles of up to 320 or 192 rows), v_mfma_f32_16x16x32_bf16
// flavour of the pipelined kernel.
// (SpecMoE Sec. 2.1 / 2.2: the rows routed to an expert meet its FFN-sized weights; at
// verification time each expert sees hundreds of rows, so the contraction is MFMA-bound.)
//
// Same data movement as grouped_gemm_bf16_pipe.hip (global->LDS ring of BK = 32 stages),
// different matrix instruction: one 16x16x32 MFMA consumes a whole 64-byte tile row per lane,
// so a stage is ONE k-step.
// Why this shape: under the chip's power limit the 16x16x32 instruction sustains more bf16
// flops than 32x32x16 on the same operands (2.1 vs 1.8 PFLOP/s measured in a register-only
// loop with changing operands), and its 16-row granule wastes fewer matrix instructions on
// the ragged last rows of an expert.
//
// Loop schedule: ping-pong.  The two waves of a SIMD alternate between multiplying a k-step
// out of registers and loading / reading the next one.
//
// Operands may be tile-packed (pipe_common.h: 1 KB blocks of 16 rows x 32 columns that hold the
// LDS image of the piece).  A wave-load then reads 1 KB of consecutive memory, i.e. whole
// 128-byte lines, instead of sixteen 64-byte half lines of sixteen rows; the L2 serves requests,
// not bytes, and the kernel is bound by that request rate (row-major operands: 852 / 427 us
// for the gate/up / down projection of the 2048-token Mixtral-shaped layer, both operands packed:
// 788 / 380 us in the same harness).  PA: activations packed (the down projection's h, written
// packed by the gate/up kernel: PO); PB: weights packed (moe_pack_weights).
#include "pipe_common.h"

#include <type_traits>
#include <utility>

namespace specmoe {
namespace {

using namespace pipe;

template <typename F, int... Is>
__device__ __forceinline__ void dispatch_count(int n, F& f, std::integer_sequence<int, Is...>) {
    ((n == Is ? (f(std::integral_constant<int, Is>{}), 0) : 0), ...);
}

template <typename C, bool PA = false, bool PB = false, bool PO = false>
__global__ __launch_bounds__(C::THREADS) void grouped_gemm_bf16_pipe16_kernel(
    const bf16_t* __restrict__ A,        // [n_rows, K]
    const int32_t* __restrict__ offsets, // [E+1]
    const bf16_t* __restrict__ W0,       // [E, N, K]   (gate, or down)
    const bf16_t* __restrict__ W1,       // [E, N, K]   (up; SWIGLU only)
    int E, int N, int K, bf16_t* __restrict__ Cout /* [n_rows, N] */,
    const int32_t* __restrict__ row_src /* nullable: A row r is A[row_src[r] / topk] */, int topk) {
    static_assert(C::BK == 32, "a stage is exactly one 16x16x32 k-step");
    constexpr int TM16 = C::BM / (16 * C::WM);       // 16-row A sub-tiles per wave
    constexpr int TN16 = C::BN / (16 * C::WN);       // 16-col B sub-tiles per wave
    constexpr int A_SUB_BYTES = 16 * C::WM * C::ROW_BYTES;   // LDS distance of consecutive i
    static_assert(!C::SWIGLU || TN16 % 2 == 0, "gate and up sub-tiles pair up inside a wave");
    static_assert((16 * C::WM) % (C::RPG * C::CHUNKS) == 0, "sub-tile step must keep the swizzle");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];

    const int NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    TileLoc t;
    if (!locate_tile_even<C::BM, 16>(offsets, E, NT, blockIdx.x, t)) return;
    const int row0 = t.row0, tile_rows = t.tile_rows;
    const int n0 = t.nt * C::BN_OUT;
    const int nsub = (tile_rows + 15) / 16;

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    // waves w and w+4 share a SIMD: different wm keeps an odd sub-tile count balanced
    const int wm = wave / C::WN, wn = wave % C::WN;
    const uint32_t lds_base =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_raw;

    // ---- global side of the wave-loads (identical to the 32x32 kernel) --------------------
    // with row_src the activation rows are gathered on the fly (A is then the token matrix)
    // tile-packed operands: row block rb (16 rows) of a matrix with K columns starts at element
    // rb * 16 * K, its k-step kt at + kt * 512 (one 1 KB block)
    const unsigned char* a_base = uniform_ptr(reinterpret_cast<const unsigned char*>(
        A + (PA ? (size_t)t.blk0 * 16 * K : (row_src ? (size_t)0 : (size_t)row0 * K))));
    const size_t wrow = (size_t)t.expert * N + min(n0, N - 1);      // packed: a multiple of 16
    const unsigned char* w0 = uniform_ptr(reinterpret_cast<const unsigned char*>(W0 + wrow * K));
    const unsigned char* w1 =
        C::SWIGLU ? uniform_ptr(reinterpret_cast<const unsigned char*>(W1 + wrow * K)) : nullptr;
    const int n_left = N - n0;
    constexpr uint32_t A_KSTEP = PA ? 1024u : (uint32_t)C::ROW_BYTES;   // bytes per k-step
    constexpr uint32_t B_KSTEP = PB ? 1024u : (uint32_t)C::ROW_BYTES;
    uint32_t a_off[C::A_PW], b_off[C::B_PW];
    int a_cnt = 0;                               // A wave-loads this wave issues per stage
    {
        const int srow = lane / C::CHUNKS, pc = lane % C::CHUNKS;   // LDS slot of this lane
#pragma unroll
        for (int jj = 0; jj < C::A_PW; ++jj) {
            const int r = (wave + jj * C::NWAVES) * C::ROWS_PER_DMA + srow;
            const int c = pc ^ ((r / C::RPG) % C::CHUNKS);
            const int rr = min(r, tile_rows - 1);
            if (PA) {
                // wave-load j = row block j of the tile: 1 KB, lane l its l-th 16-byte piece
                const int jb = min(wave + jj * C::NWAVES, (tile_rows + 15) / 16 - 1);
                a_off[jj] = (unsigned)jb * 16u * (unsigned)K * 2u + (unsigned)lane * 16u;
            } else {
                const unsigned arow =
                    row_src ? (unsigned)(row_src[row0 + rr] / topk) : (unsigned)rr;
                a_off[jj] = (arow * (unsigned)K + (unsigned)(c * 8)) * 2u;
            }
            if ((wave + jj * C::NWAVES) * C::ROWS_PER_DMA < tile_rows) a_cnt = jj + 1;
        }
#pragma unroll
        for (int jj = 0; jj < C::B_PW; ++jj) {
            const int r = (wave + jj * C::NWAVES) * C::ROWS_PER_DMA + srow;
            const int c = pc ^ ((r / C::RPG) % C::CHUNKS);
            const int rn = (C::SWIGLU && r >= C::BN / 2) ? r - C::BN / 2 : r;
            if (PB) {
                const int jb = min(rn / 16, n_left / 16 - 1);        // row block of the weight tile
                b_off[jj] = (uint32_t)jb * 16u * (uint32_t)K * 2u + (uint32_t)lane * 16u;
            } else {
                b_off[jj] = (uint32_t)((min(rn, n_left - 1) * K + c * 8) * 2);
            }
        }
    }
    const int KT = K / C::BK;                    // even: the ABI requires K % 64 == 0
    // nt_tag: the weight loads carry the non-temporal hint (tiles whose weights no other
    // workgroup reads)
    auto issue_one = [&](auto nt_tag, int which, int kt, int buf) __attribute__((always_inline)) {
        // the k offset rides in the per-lane offset (one vector add per load); the base
        // pointers stay loop-invariant scalars.  Clamped: the last steps re-load stage KT-1.
        const uint32_t kq = (uint32_t)min(kt, KT - 1);
        const uint32_t ka = kq * A_KSTEP, kb = kq * B_KSTEP;
        const uint32_t sbase = lds_base + (uint32_t)buf * C::STAGE_BYTES + wave * 1024u;
#pragma unroll
        for (int jj = 0; jj < C::A_PW; ++jj)
            if (which == jj && jj < a_cnt)
                dma16(a_base, a_off[jj] + ka, sbase + jj * C::NWAVES * 1024u);
#pragma unroll
        for (int jj = 0; jj < C::B_PW; ++jj) {
            const bool up = C::SWIGLU && (jj * C::NWAVES * C::ROWS_PER_DMA >= C::BN / 2);
            if (which == C::A_PW + jj) {
                if (decltype(nt_tag)::value)
                    dma16_nt(up ? w1 : w0, b_off[jj] + kb,
                             sbase + C::A_BYTES + jj * C::NWAVES * 1024u);
                else
                    dma16(up ? w1 : w0, b_off[jj] + kb,
                          sbase + C::A_BYTES + jj * C::NWAVES * 1024u);
            }
        }
    };

    // ---- LDS side: lane l reads row (l%16) of a sub-tile, 16-byte chunk l/16 -----------------
    const int a_rd = swz<C>(16 * wm + (lane & 15), lane >> 4);
    const int b_rd = C::A_BYTES + swz<C>(lane & 15, lane >> 4);
    auto nb = [&](int j) __attribute__((always_inline)) -> int {     // B sub-tile base row
        if (C::SWIGLU) {
            constexpr int H = TN16 / 2;
            return (j < H) ? 16 * (wn * H + j) : C::BN / 2 + 16 * (wn * H + (j - H));
        }
        return 16 * (wn * TN16 + j);
    };

    const int ta = min(TM16, max(0, (nsub - wm + C::WM - 1) / C::WM));   // active A sub-tiles

    // epilogue: SwiGLU tiles are staged in LDS and written as whole rows by the workgroup,
    // plain tiles go straight to global memory, 8 bytes (4 columns) per lane.  acc[i] is the
    // wave's i-th A sub-tile (tile rows 16 * (wm + WM * i) ..).
    auto epilogue = [&](auto& acc, auto ta_tag) __attribute__((always_inline)) {
        constexpr int TA = decltype(ta_tag)::value;
        wait_vmcnt<0>();                           // no load may outlive the workgroup's LDS

        const int mrow = lane & 15, cq = (lane >> 4) * 4;
        if (C::SWIGLU && !PO) __builtin_amdgcn_s_barrier();   // every wave's loads have landed
#pragma unroll
        for (int i = 0; i < TA; ++i) {
            const int trow = 16 * (wm + C::WM * i) + mrow;
            if (!C::SWIGLU && trow >= tile_rows) continue;
            bf16_t* crow = Cout + (size_t)(row0 + trow) * N;
            constexpr int JN = C::SWIGLU ? TN16 / 2 : TN16;
#pragma unroll
            for (int j = 0; j < JN; ++j) {
                const int ctile = 16 * (wn * JN + j) + cq;            // column inside the tile
                float v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (C::SWIGLU) {
                        const float gt = acc[i][j][q], up = acc[i][j + JN][q];
                        v[q] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * up;
                    } else {
                        v[q] = acc[i][j][q];
                    }
                }
                const uint2 pk = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
                if (C::SWIGLU && PO) {
                    // tile-packed h straight from the registers: the wave's sub-tile j is the
                    // column half j of the 32-column block wn of row block (wm + WM*i); this
                    // lane holds half a 16-byte chunk.  Rows beyond the tile's last row (padding
                    // of the expert's last block) are written as zeros.
                    static_assert(!PO || (TN16 == 4 && C::BN_OUT == 128), "packed output tiling");
                    const int col0 = n0 + 32 * wn;
                    if (col0 < N) {
                        const int chunk = 2 * j + (cq >> 3);
                        const int piece = 4 * mrow + (chunk ^ ((mrow >> 1) & 3));
                        unsigned char* blk = reinterpret_cast<unsigned char*>(
                            Cout + ((size_t)(t.blk0 + wm + C::WM * i) * 16 * N +
                                    (size_t)(col0 / 32) * 512));
                        *reinterpret_cast<uint2*>(blk + piece * 16 + ((cq >> 2) & 1) * 8) =
                            trow < tile_rows ? pk : make_uint2(0u, 0u);
                    }
                } else if (C::SWIGLU) {
                    *reinterpret_cast<uint2*>(lds_raw + trow * kStageRowBytes + ctile * 2) = pk;
                } else {
                    const int col = n0 + ctile;
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
    };

    // ---- ping-pong schedule ----------------------------------------------------------------
    // The two waves that share a SIMD belong to different groups (wm = 0 / 1) and alternate:
    // while one multiplies a whole k-step out of registers (nothing but matrix instructions),
    // the other issues its wave-loads and reads its next fragments; a barrier, and they swap.
    // The matrix pipe of every SIMD always has exactly one wave feeding it, and fragment reads
    // and load issue never sit between two matrix instructions.  Group 1 runs one phase behind
    // group 0 (one extra barrier up front, group 0 pays it back at the end).
    //   phase 2kt  : group 0 reads stage kt            | group 1 multiplies stage kt-1
    //   phase 2kt+1: group 0 multiplies stage kt       | group 1 reads stage kt
    // Stage kt+3 is requested in the read phase of stage kt (its slot held stage kt-1, which
    // group 1 finished reading one phase earlier); before the barrier that ends phase 2kt+1
    // every wave waits for its share of stage kt+1, so a stage has 4 to 5 phases to land.
    auto run_pp = [&](auto ta_tag, auto nt_tag) __attribute__((always_inline)) {
        static_assert(C::WM == 2 && C::STAGES == 4, "two wave groups, ring of four");
        constexpr int TA = decltype(ta_tag)::value;
        constexpr int TAX = TA > 0 ? TA : 1;
        floatx4 acc[TAX][TN16];
#pragma unroll
        for (int i = 0; i < TA; ++i)
#pragma unroll
            for (int j = 0; j < TN16; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
        bf16x8 af[TAX], bfr[TN16];
        const int allow2 = 2 * (a_cnt + C::B_PW);          // two younger stages may be in flight

        // prologue: stages 0..2 requested, stage 0 landed and visible
#pragma unroll
        for (int s = 0; s < C::STAGES - 1; ++s)
#pragma unroll
            for (int q = 0; q < C::G_MAX; ++q) issue_one(nt_tag, q, s, s);
        wait_vmcnt_dyn(allow2);
        __builtin_amdgcn_s_barrier();
        if (wm == 1) __builtin_amdgcn_s_barrier();         // group 1 sits out phase 0

        int buf = 0;
        for (int kt = 0; kt < KT; ++kt) {
            // ---- read phase
#pragma unroll
            for (int q = 0; q < C::G_MAX; ++q)
                issue_one(nt_tag, q, kt + C::STAGES - 1, (buf + 3) & 3);
            if (TA > 0) {
                const unsigned char* sa = lds_raw + buf * C::STAGE_BYTES + a_rd;
                const unsigned char* sb = lds_raw + buf * C::STAGE_BYTES + b_rd;
#pragma unroll
                for (int j = 0; j < TN16; ++j)
                    bfr[j] = *reinterpret_cast<const bf16x8*>(sb + nb(j) * C::ROW_BYTES);
#pragma unroll
                for (int i = 0; i < TA; ++i)
                    af[i] = *reinterpret_cast<const bf16x8*>(sa + i * A_SUB_BYTES);
            }
            if (wm == 1) wait_vmcnt_dyn(allow2);           // phase 2kt+1 ends: stage kt+1 landed
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);             // nothing moves across the barriers
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // ---- multiply phase
#pragma unroll
            for (int i = 0; i < TA; ++i)
#pragma unroll
                for (int j = 0; j < TN16; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j], af[i], acc[i][j],
                                                                        0, 0, 0);
            if (wm == 0) wait_vmcnt_dyn(allow2);           // phase 2kt+1 ends: stage kt+1 landed
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            buf = (buf + 1) & 3;
        }
        if (wm == 0) __builtin_amdgcn_s_barrier();         // group 0 waits out group 1's last phase
        epilogue(acc, ta_tag);
    };

    // An expert with a single m-tile: every weight tile of it is read by exactly one workgroup,
    // once - a pure stream out of HBM, which the non-temporal hint speeds up (6.3 vs 5.7 TB/s on a
    // plain LDS-DMA stream).  With several m-tiles the workgroups that share a weight tile meet
    // in the L2, and the hint would cost those hits.
    // Only with tile-packed weights: a wave-load then covers whole 128-byte lines.  Row-major, a
    // BK = 32 stage takes half of every line and the next stage the other half; without
    // allocation in the L2 every line would come out of HBM twice (measured: 363 -> 469 us).
    const bool w_once = PB && t.mt == 1 && (!C::SWIGLU || tile_rows <= 64);
    auto run_sel = [&](auto ta_tag) __attribute__((always_inline)) {
        if (w_once) run_pp(ta_tag, std::true_type{});
        else run_pp(ta_tag, std::false_type{});
    };
    dispatch_count(ta, run_sel, std::make_integer_sequence<int, TM16 + 1>{});

    if (C::SWIGLU && !PO) {
        // cooperative write-out of the staged tile: 16 bytes per lane, whole rows
        static_assert(!C::SWIGLU || (size_t)C::BM * kStageRowBytes <= C::LDS_BYTES, "stage tile");
        static_assert(!C::SWIGLU || C::BN_OUT == 128, "stage row pitch assumes 128 columns");
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

template <typename C, bool PA = false, bool PB = false, bool PO = false>
hipError_t launch_pipe16(const bf16_t* A, const int32_t* offsets, const bf16_t* W0,
                         const bf16_t* W1, int n_rows, int E, int N, int K, bf16_t* Cout,
                         hipStream_t s, const int32_t* row_src = nullptr, int topk = 1) {
    // one-time, thread-safe (C++11 static initialisation): raise the dynamic LDS limit
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&grouped_gemm_bf16_pipe16_kernel<C, PA, PB, PO>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
    if (attr != hipSuccess) return attr;
    const long long NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    const long long grid = grid_upper_bound(n_rows, E, C::BM, NT);
    hipLaunchKernelGGL((grouped_gemm_bf16_pipe16_kernel<C, PA, PB, PO>), dim3((unsigned)grid),
                       dim3(C::THREADS), C::LDS_BYTES, s, A, offsets, W0, W1, E, N, K, Cout,
                       row_src, topk);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_expert_up_bf16_large16(const bf16_t* x_perm, const int32_t* offsets,
                                         const bf16_t* wg, const bf16_t* wu, int n_rows, int d,
                                         int f, int E, bf16_t* h, hipStream_t s,
                                         const int32_t* row_src, int topk) {
    return launch_pipe16<PipeCfg<320, 256, 32, 4, 2, 4, true>>(x_perm, offsets, wg, wu, n_rows, E,
                                                               f, d, h, s, row_src, topk);
}

hipError_t launch_expert_down_bf16_large16(const bf16_t* h, const int32_t* offsets,
                                           const bf16_t* wd, int n_rows, int d, int f, int E,
                                           bf16_t* y, hipStream_t s) {
    return launch_pipe16<PipeCfg<320, 256, 32, 4, 2, 4, false>>(h, offsets, wd, nullptr, n_rows, E,
                                                                d, f, y, s);
}

// Tile-packed variants: weights packed by moe_pack_weights, h tile-packed between the two
// projections.  This one gathers the token rows itself from the row-major token matrix (per-lane
// row addresses, 64-byte requests on the activation side) and always uses 320-row tiles.
hipError_t launch_expert_up_bf16_packed(const bf16_t* x, const int32_t* offsets,
                                        const bf16_t* wg_packed, const bf16_t* wu_packed,
                                        int n_rows, int d, int f, int E, bf16_t* h_packed,
                                        hipStream_t s, const int32_t* row_src, int topk) {
    return launch_pipe16<PipeCfg<320, 256, 32, 4, 2, 4, true>, false, true, true>(
        x, offsets, wg_packed, wu_packed, n_rows, E, f, d, h_packed, s, row_src, topk);
}

// Tile height by the average rows per expert, as for the row-major operands: 320-row tiles from
// 192 rows per expert, 192-row tiles below.  h_row_major: h is written [n_rows, f] row-major
// (for a down projection on row-major operands) instead of tile-packed.
hipError_t launch_expert_up_bf16_packed_x(const bf16_t* x_packed, const int32_t* offsets,
                                          const bf16_t* wg_packed, const bf16_t* wu_packed,
                                          int n_rows, int d, int f, int E, bf16_t* h,
                                          bool h_row_major, hipStream_t s) {
    typedef PipeCfg<320, 256, 32, 4, 2, 4, true> Large;
    typedef PipeCfg<192, 256, 32, 4, 2, 4, true> Mid;
    const bool large = (long long)n_rows >= 192ll * E;
    if (h_row_major)
        return large ? launch_pipe16<Large, true, true, false>(x_packed, offsets, wg_packed,
                                                               wu_packed, n_rows, E, f, d, h, s)
                     : launch_pipe16<Mid, true, true, false>(x_packed, offsets, wg_packed,
                                                             wu_packed, n_rows, E, f, d, h, s);
    return large ? launch_pipe16<Large, true, true, true>(x_packed, offsets, wg_packed, wu_packed,
                                                          n_rows, E, f, d, h, s)
                 : launch_pipe16<Mid, true, true, true>(x_packed, offsets, wg_packed, wu_packed,
                                                        n_rows, E, f, d, h, s);
}

hipError_t launch_expert_down_bf16_packed(const bf16_t* h_packed, const int32_t* offsets,
                                          const bf16_t* wd_packed, int n_rows, int d, int f,
                                          int E, bf16_t* y, hipStream_t s) {
    if ((long long)n_rows >= 192ll * E)
        return launch_pipe16<PipeCfg<320, 256, 32, 4, 2, 4, false>, true, true, false>(
            h_packed, offsets, wd_packed, nullptr, n_rows, E, d, f, y, s);
    return launch_pipe16<PipeCfg<192, 256, 32, 4, 2, 4, false>, true, true, false>(
        h_packed, offsets, wd_packed, nullptr, n_rows, E, d, f, y, s);
}

// In between (tens to a few hundred rows per expert, e.g. 16 experts with top-1 routing, 30 to
// 530 rows each), gate/up projection: the same kernel with tiles of at most 192 rows.  Hot experts
// are MFMA-bound, cold ones stream their weights; measured at that shape (gate/up alone): 192- and
// 256-row tiles 668 us, 128-row 796 us, 320-row 732 us, the 32x32x16 kernel with 128 x 128 tiles
// 750 us.  (For the down projection of that shape the 32x32x16 kernel stays ahead: 340 vs 388 us.)
hipError_t launch_expert_up_bf16_mid(const bf16_t* x_perm, const int32_t* offsets,
                                     const bf16_t* wg, const bf16_t* wu, int n_rows, int d, int f,
                                     int E, bf16_t* h, hipStream_t s, const int32_t* row_src,
                                     int topk) {
    return launch_pipe16<PipeCfg<192, 256, 32, 4, 2, 4, true>>(x_perm, offsets, wg, wu, n_rows, E,
                                                               f, d, h, s, row_src, topk);
}

}  // namespace specmoe
