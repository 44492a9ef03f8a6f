// Configuration and inline-assembly helpers shared by the pipelined expert GEMM kernels
// (global->LDS ring, see grouped_gemm_bf16_pipe.hip for the scheme).
#pragma once
#include "common.h"
#include "tile_map.h"

namespace specmoe {
namespace pipe {

template <int BM_, int BN_, int BK_, int STAGES_, int WM_, int WN_, bool SWIGLU_>
struct PipeCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_, WM = WM_, WN = WN_;
    static constexpr bool SWIGLU = SWIGLU_;
    static constexpr int NWAVES = WM * WN, THREADS = NWAVES * kWave;
    static constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);   // 32x32 sub-tiles per wave
    static constexpr int KK = BK / 16;                               // MFMA k-steps per stage
    static constexpr int ROW_BYTES = BK * 2, CHUNKS = BK / 8;        // 16-byte chunks per row
    static constexpr int RPG = 2;                    // tile rows that share a swizzle term
    static constexpr int ROWS_PER_DMA = 1024 / ROW_BYTES;            // rows one wave-load fills
    static constexpr int A_LOADS = BM / ROWS_PER_DMA;                // wave-loads per stage, A
    static constexpr int A_PW = (A_LOADS + NWAVES - 1) / NWAVES;     // at most, per wave
    static constexpr int B_PW = BN / ROWS_PER_DMA / NWAVES;          // wave-loads per wave, B
    static constexpr int G_MAX = A_PW + B_PW;                        // loads per wave per stage
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE_BYTES;
    static constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    static_assert(BK == 32 || BK == 64 || BK == 128, "BK");
    static_assert(KK % 2 == 0, "fragment double buffer needs an even number of k-steps");
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0, "tile / wave grid mismatch");
    static_assert(BM % ROWS_PER_DMA == 0 && BN % (ROWS_PER_DMA * NWAVES) == 0,
                  "wave-loads must divide evenly");
    static_assert(!SWIGLU || ((BN / 2 / ROWS_PER_DMA) % NWAVES == 0 && TN % 2 == 0),
                  "gate/up halves must split on a wave-load round and pair up inside a wave");
    static_assert(STAGES >= 3 && (STAGES - 3) * G_MAX <= 63, "ring depth (vmcnt is 6 bits)");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

// Byte offset of 16-byte chunk c of tile row r: chunk c sits at position c ^ ((r / 2) % CHUNKS)
// of its row.  Measured on gfx950 (ds_read_b128, one CU, 8 wavefronts; 4.4 clk per instruction
// is the conflict-free rate): with 128-byte rows this term is conflict-free for the 32-row
// fragment reads of the 32x32x16 instruction; with 64-byte rows it is conflict-free for the
// 16-row reads of the 16x16x32 instruction, where the term (r / 4) % 4 - one sweep over the 16
// bank groups per 4 rows, the "obvious" choice - costs 8.0 clk per read (SQ_LDS_BANK_CONFLICT =
// half of SQ_LDS_IDX_ACTIVE) because the hardware pairs lanes 0-7 with lanes 16-23, not with
// lanes 8-15.
template <typename C>
__device__ __forceinline__ int swz(int r, int c) {
    return r * C::ROW_BYTES + ((c ^ ((r / C::RPG) % C::CHUNKS)) << 4);
}

// Tile-packed matrix [R rows, K columns] of bf16 (R % 16 == 0, K % 32 == 0), same size as the
// row-major one: 1 KB blocks of 16 rows x 32 columns; block (rb, kb) at byte offset
// (rb * (K / 32) + kb) * 1024, i.e. row block rb starts at element rb * 16 * K.  A block holds
// the LDS image of its piece under swz<> with 64-byte rows: the 16-byte chunk c (8 columns) of
// row r sits at piece index 4 * r + (c ^ ((r / 2) % 4)).  A wave-load of such a block is 1 KB
// of consecutive memory and lands in LDS ready for the fragment reads.
constexpr int kPackRows = 16, kPackCols = 32;

// Row pitch of the LDS image of a SwiGLU output tile (128 bf16 columns + 16 bytes of padding
// so that the 8-byte accumulator stores of 32 consecutive rows spread over the banks).
constexpr int kStageRowBytes = 128 * 2 + 16;

// 64 lanes x 16 bytes: global (uniform base + per-lane byte offset) -> LDS [lds_addr, +1024).
// The LDS destination travels in m0, which the statement overwrites (declared as a clobber).
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(gbase), "s"(lds_addr) : "memory", "m0");
}
// The same with the non-temporal hint: for data that is read once (expert weights streamed out
// of HBM).  Measured on a 4 GiB LDS-DMA stream: 5.7 TB/s without the hint, 6.3 TB/s with it.
__device__ __forceinline__ void dma16_nt(const void* gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :: "v"(voff), "s"(gbase), "s"(lds_addr) : "memory", "m0");
}
// tells the compiler that a pointer is the same in every lane (it then lives in scalar registers,
// which the "s" operand of dma16 requires)
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// s_waitcnt takes an immediate; n is wave-uniform and constant over the k loop
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
#define SPECMOE_W4(b) case b: wait_vmcnt<b>(); break; case b + 1: wait_vmcnt<b + 1>(); break; \
                      case b + 2: wait_vmcnt<b + 2>(); break; case b + 3: wait_vmcnt<b + 3>(); break;
    switch (n) {
        SPECMOE_W4(0) SPECMOE_W4(4) SPECMOE_W4(8) SPECMOE_W4(12) SPECMOE_W4(16) SPECMOE_W4(20)
        SPECMOE_W4(24) SPECMOE_W4(28) SPECMOE_W4(32) SPECMOE_W4(36) SPECMOE_W4(40) SPECMOE_W4(44)
        SPECMOE_W4(48) SPECMOE_W4(52) SPECMOE_W4(56)
        case 60: wait_vmcnt<60>(); break; case 61: wait_vmcnt<61>(); break;
        case 62: wait_vmcnt<62>(); break; default: wait_vmcnt<63>(); break;
    }
#undef SPECMOE_W4
}

}  // namespace pipe
}  // namespace specmoe
