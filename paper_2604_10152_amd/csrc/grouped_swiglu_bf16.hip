// Experts in bf16 mode: dispatch of the two expert contractions to a kernel family by shape,
// and the register-staged kernel used for short contractions.
// (SpecMoE Sec. 2.1: every expert is an FFN-sized block; only the rows routed to an expert
// are multiplied with its weights.  At verification time all B*(gamma+1) tokens arrive at
// once - Sec. 2.2 - which is what makes this a dense contraction worth the MFMA units.)
//
// Two launches: (1) h = silu(x Wg^T) * (x Wu^T) with gate and up columns of one f-range in
// the same tile so the SwiGLU epilogue happens on the accumulators; (2) y = h Wd^T.
// Both are "NT" GEMMs: A rows and W rows are contiguous along the contraction axis, which is
// the layout the bf16 matrix instructions want (each lane feeds 8 consecutive k of one row).
//
// Register-staged kernel (grouped_gemm_bf16_kernel, v_mfma_f32_32x32x16_bf16): a workgroup
// owns BM = 64 rows of ONE expert x BN weight rows, BK = 64 per step; the next step's tile is
// loaded into registers while the current one is multiplied, then stored to the other LDS
// buffer (16-byte chunks XOR-swizzled by row so that both the 128-byte-row stores and the
// MFMA fragment reads are bank-conflict free).  It serves short contraction axes (fine-grained
// experts), where a tile lives for a few dozen steps and several co-resident workgroups per CU
// hide each other's prologue and epilogue.  m-tiles never straddle experts; the tile ->
// (expert, n-tile, m-tile) map is computed on the device from expert_offsets (no host
// read-back), consecutive logical tiles go to the same XCD and its L2 (tile_map.h).
// 32-row MFMA sub-tiles beyond the expert's last row are skipped (wave-uniform), and waves
// take sub-tiles interleaved so that a partial tile stays balanced across the SIMDs.
#include "common.h"
#include "tile_map.h"

#include <type_traits>

namespace specmoe {
namespace {

constexpr int kBK = 64;                       // contraction elements per LDS stage
constexpr int kChunksPerRow = kBK / 8;        // 16-byte chunks per tile row (8)

template <int BM_, int BN_, int WM_, int WN_, bool SWIGLU_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr bool SWIGLU = SWIGLU_;
    static constexpr int THREADS = WM * WN * kWave;
    static constexpr int TM = BM / (32 * WM);             // 32-row sub-tiles per wave
    static constexpr int TN = BN / (32 * WN);             // 32-col sub-tiles per wave
    static constexpr int A_LD = BM * kChunksPerRow / THREADS;   // 16-byte loads per thread
    static constexpr int B_LD = BN * kChunksPerRow / THREADS;
    static constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;   // output columns per tile
    static constexpr size_t LDS_BYTES = 2ull * (BM + BN) * kBK * sizeof(bf16_t);
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "tile / wave grid mismatch");
    static_assert((BM * kChunksPerRow) % THREADS == 0 && (BN * kChunksPerRow) % THREADS == 0,
                  "loads must divide evenly");
    static_assert(!SWIGLU || (TN % 2 == 0), "gate and up sub-tiles must pair up in one wave");
};

// Element offset (bf16 units) of 16-byte chunk `c` of tile row `r` inside an LDS tile.
// gfx950's LDS has 64 four-byte banks and serves a 128-bit access 16 lanes at a time, so 16
// consecutive lanes must land in 16 different 16-byte bank groups.  A tile row is 128 bytes =
// 8 groups, odd rows start at group 8; XOR-ing the chunk with (r >> 1) & 7 makes the MFMA
// fragment reads (16 consecutive rows, one chunk) and the row-major stores (2 rows x 8 chunks)
// both conflict free (measured: 4.4 clk per ds_read_b128 against 8.0 with (r & 7)).
__device__ __forceinline__ int lds_off(int r, int c) {
    return r * kBK + ((c ^ ((r >> 1) & 7)) << 3);
}

template <typename C>
__global__ __launch_bounds__(C::THREADS) void grouped_gemm_bf16_kernel(
    const bf16_t* __restrict__ A,        // [n_rows, K]
    const int32_t* __restrict__ offsets, // [E+1]
    const bf16_t* __restrict__ W0,       // [E, N, K]   (gate, or down)
    const bf16_t* __restrict__ W1,       // [E, N, K]   (up; SWIGLU only)
    int E, int N, int K, bf16_t* __restrict__ Cout /* [n_rows, N] */,
    const int32_t* __restrict__ row_src /* nullable: A row r is A[row_src[r] / topk] */, int topk) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* lds_a = reinterpret_cast<bf16_t*>(lds_raw);                 // [2][BM*BK]
    bf16_t* lds_b = lds_a + 2 * C::BM * kBK;                            // [2][BN*BK]

    // ---- logical tile of this workgroup -------------------------------------------
    const int NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    TileLoc t;
    if (!locate_tile<C::BM>(offsets, E, NT, blockIdx.x, t)) return;
    const int expert = t.expert, row0 = t.row0, tile_rows = t.tile_rows, nt = t.nt;
    const int n0 = nt * C::BN_OUT;
    const int nsub = (tile_rows + 31) / 32;              // active 32-row sub-tiles

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // wave-uniform by construction
    const int wm = wave % C::WM, wn = wave / C::WM;

    // ---- per-thread global load offsets (elements, relative to uniform base pointers; rows
    //      clamped into the valid range so every load stays in bounds) ---------------------
    constexpr int kRowsPerPass = C::THREADS / kChunksPerRow;    // tile rows one load pass covers
    static_assert(!C::SWIGLU || (C::BN / 2) % kRowsPerPass == 0, "gate/up split must align");
    const bf16_t* a_base = A + (row_src ? (size_t)0 : (size_t)row0 * K);
    const bf16_t* w0 = W0 + ((size_t)expert * N + min(n0, N - 1)) * K;
    const bf16_t* w1 = C::SWIGLU ? W1 + ((size_t)expert * N + min(n0, N - 1)) * K : nullptr;
    const int n_left = N - n0;                             // weight rows left from n0 (>= 1)
    uint32_t a_off[C::A_LD], b_off[C::B_LD];
    int a_lds[C::A_LD], b_lds[C::B_LD];
    {
        const int r0 = tid / kChunksPerRow, c = tid % kChunksPerRow;
#pragma unroll
        for (int l = 0; l < C::A_LD; ++l) {
            const int r = r0 + l * kRowsPerPass;
            const int rr = min(r, tile_rows - 1);
            const unsigned arow = row_src ? (unsigned)(row_src[row0 + rr] / topk) : (unsigned)rr;
            a_off[l] = arow * (unsigned)K + (unsigned)(c * 8);
            a_lds[l] = lds_off(r, c);
        }
#pragma unroll
        for (int l = 0; l < C::B_LD; ++l) {
            const int r = r0 + l * kRowsPerPass;
            const int rn = (C::SWIGLU && r >= C::BN / 2) ? r - C::BN / 2 : r;
            b_off[l] = (uint32_t)(min(rn, n_left - 1) * K + c * 8);
            b_lds[l] = lds_off(r, c);
        }
    }

    // ---- fragment read offsets -------------------------------------------------------
    // A sub-tile i of this wave covers tile rows 32*(wm + WM*i) .. +31 (interleaved);
    // B sub-tile j covers weight rows nb(j) .. +31 of the LDS B tile.
    int a_row[C::TM], b_row[C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i) a_row[i] = 32 * (wm + C::WM * i) + (lane & 31);
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
        int nb;
        if (C::SWIGLU) {
            constexpr int H = C::TN / 2;
            nb = (j < H) ? 32 * (wn * H + j) : C::BN / 2 + 32 * (wn * H + (j - H));
        } else {
            nb = 32 * (wn * C::TN + j);
        }
        b_row[j] = nb + (lane & 31);
    }
    const int khalf = lane >> 5;                        // which 8-wide k group of a 16-k step

    U128 a_reg[C::A_LD], b_reg[C::B_LD];
    const int KT = K / kBK;

    auto load_global = [&](int kt) __attribute__((always_inline)) {
        const bf16_t* ak = a_base + (size_t)kt * kBK;
        const bf16_t* w0k = w0 + (size_t)kt * kBK;
        const bf16_t* w1k = C::SWIGLU ? w1 + (size_t)kt * kBK : nullptr;
#pragma unroll
        for (int l = 0; l < C::A_LD; ++l)
            a_reg[l] = *reinterpret_cast<const U128*>(ak + a_off[l]);
#pragma unroll
        for (int l = 0; l < C::B_LD; ++l) {
            const bool up = C::SWIGLU && (l * kRowsPerPass >= C::BN / 2);   // compile-time per l
            b_reg[l] = *reinterpret_cast<const U128*>((up ? w1k : w0k) + b_off[l]);
        }
    };
    auto store_lds = [&](int buf) __attribute__((always_inline)) {
        bf16_t* sa = lds_a + buf * C::BM * kBK;
        bf16_t* sb = lds_b + buf * C::BN * kBK;
#pragma unroll
        for (int l = 0; l < C::A_LD; ++l) *reinterpret_cast<U128*>(sa + a_lds[l]) = a_reg[l];
#pragma unroll
        for (int l = 0; l < C::B_LD; ++l) *reinterpret_cast<U128*>(sb + b_lds[l]) = b_reg[l];
    };

    // Number of this wave's sub-tiles that hold real rows.  Sub-tile i sits at tile row
    // 32*(wm + WM*i), so the active ones are exactly i = 0 .. ta-1.  The main loop and the
    // epilogue are instantiated once per value of ta: straight-line MFMA code in each, and a
    // partial tile issues only the matrix instructions it needs.
    const int ta = min(C::TM, max(0, (nsub - wm + C::WM - 1) / C::WM));

    auto run = [&](auto ta_tag) __attribute__((always_inline)) {
        constexpr int TA = decltype(ta_tag)::value;
        floatx16 acc[TA > 0 ? TA : 1][C::TN];
#pragma unroll
        for (int i = 0; i < TA; ++i)
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        load_global(0);
        store_lds(0);
        __syncthreads();

        for (int kt = 0; kt < KT; ++kt) {
            const int buf = kt & 1;
            // branch-free prefetch: the last step re-loads its own tile into the idle buffer
            load_global(min(kt + 1, KT - 1));
            // keep the prefetch at the top of the step: the instruction scheduler would
            // otherwise sink the loads next to their LDS stores and expose the HBM latency
            __builtin_amdgcn_sched_barrier(0);
            const bf16_t* sa = lds_a + buf * C::BM * kBK;
            const bf16_t* sb = lds_b + buf * C::BN * kBK;
            if (TA > 0) {
#pragma unroll
                for (int kk = 0; kk < kBK / 16; ++kk) {
                    const int c = kk * 2 + khalf;
                    bf16x8 bf[C::TN], af[TA > 0 ? TA : 1];
#pragma unroll
                    for (int j = 0; j < C::TN; ++j)
                        bf[j] = *reinterpret_cast<const bf16x8*>(sb + lds_off(b_row[j], c));
#pragma unroll
                    for (int i = 0; i < TA; ++i)
                        af[i] = *reinterpret_cast<const bf16x8*>(sa + lds_off(a_row[i], c));
#pragma unroll
                    for (int i = 0; i < TA; ++i)
#pragma unroll
                        for (int j = 0; j < C::TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                af[i], bf[j], acc[i][j], 0, 0, 0);
                }
            }
            store_lds(buf ^ 1);
            __syncthreads();
        }

        // epilogue: accumulator element r of a lane is row 8*(r/4) + 4*(lane/32) + r%4,
        // column lane%32 of its 32x32 sub-tile
        const int col_in = lane & 31;
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
hipError_t launch_one(const bf16_t* A, const int32_t* offsets, const bf16_t* W0,
                      const bf16_t* W1, int n_rows, int E, int N, int K, bf16_t* Cout,
                      hipStream_t s, const int32_t* row_src = nullptr, int topk = 1) {
    // one-time, thread-safe (C++11 static initialisation): raise the dynamic LDS limit
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&grouped_gemm_bf16_kernel<C>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
    if (attr != hipSuccess) return attr;
    const long long NT = (N + C::BN_OUT - 1) / C::BN_OUT;
    const long long max_mt = n_rows / C::BM + E;     // sum_e ceil(M_e/BM) <= floor(P/BM) + E
    long long grid = max_mt * NT;
    grid = (grid + kXcds - 1) / kXcds * kXcds;
    hipLaunchKernelGGL(grouped_gemm_bf16_kernel<C>, dim3((unsigned)grid), dim3(C::THREADS),
                       C::LDS_BYTES, s, A, offsets, W0, W1, E, N, K, Cout, row_src, topk);
    return hipGetLastError();
}

}  // namespace

// Rows per expert (average) from which a kernel family applies: >= 192 large (MFMA-bound,
// up to 320-row tiles), >= 48 with a long contraction mid (gate/up: up to 192-row tiles of the
// same kernel; down: 128-row tiles of the 32x32x16 pipeline), below that small (64-row tiles).
constexpr int g_large_rows = 192, g_mid_rows = 48;
static inline bool large_batch(int n_rows, int E) {
    return (long long)n_rows >= (long long)g_large_rows * E;
}
static inline bool mid_batch(int n_rows, int E, int K) {
    return K >= 4096 && (long long)n_rows >= (long long)g_mid_rows * E;
}
// Few rows per expert, two kernels: with a long contraction axis the deep global->LDS ring wins
// (5.8 vs 5.3 TB/s at the Mixtral shape); with a short one (fine-grained experts) a tile lives
// for a few dozen steps only and three co-resident register-staged workgroups per CU hide the
// prologue / epilogue of each other better (360 vs 490 us at the 64-expert shape).
constexpr int kLongK = 4096;

// Large batches: up to 320-row tiles, 8 wavefronts, MFMA-bound.  Fewer rows per expert: the
// weights stream once from HBM and narrow tiles give every CU its own stream (measured at 16
// experts x 128 rows on average: mid 1116 us, large 1231 us, small 1437 us per layer).
hipError_t launch_expert_up_bf16(const bf16_t* x_perm, const int32_t* offsets, const bf16_t* wg,
                                 const bf16_t* wu, int n_rows, int d, int f, int E, bf16_t* h,
                                 hipStream_t s, const int32_t* row_src, int topk) {
    if (n_rows == 0) return hipSuccess;
    if (large_batch(n_rows, E))
        return launch_expert_up_bf16_large16(x_perm, offsets, wg, wu, n_rows, d, f, E, h, s,
                                             row_src, topk);
    if (mid_batch(n_rows, E, d))
        return launch_expert_up_bf16_mid(x_perm, offsets, wg, wu, n_rows, d, f, E, h, s, row_src,
                                         topk);
    if (d >= kLongK)
        return launch_expert_up_bf16_small(x_perm, offsets, wg, wu, n_rows, d, f, E, h, s, row_src,
                                           topk);
    return launch_one<TileCfg<64, 256, 1, 4, true>>(x_perm, offsets, wg, wu, n_rows, E, f, d, h, s, row_src, topk);
}

hipError_t launch_expert_down_bf16(const bf16_t* h, const int32_t* offsets, const bf16_t* wd,
                                   int n_rows, int d, int f, int E, bf16_t* y, hipStream_t s) {
    if (n_rows == 0) return hipSuccess;
    if (large_batch(n_rows, E))
        return launch_expert_down_bf16_large16(h, offsets, wd, n_rows, d, f, E, y, s);
    if (mid_batch(n_rows, E, f))
        return launch_expert_down_bf16_mid(h, offsets, wd, n_rows, d, f, E, y, s);
    if (f >= kLongK) return launch_expert_down_bf16_small(h, offsets, wd, n_rows, d, f, E, y, s);
    return launch_one<TileCfg<64, 128, 1, 4, false>>(h, offsets, wd, nullptr, n_rows, E, d, f, y, s);
}

}  // namespace specmoe
