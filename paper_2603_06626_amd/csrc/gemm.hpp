// Building blocks of the grouped bf16 MFMA GEMMs (gfx950): LDS tile layouts, direct global->LDS tile
// loads, MFMA fragment reads, the shared K-loop pipeline and the LDS-staged output writer.
//
// Shape.  A workgroup of 256 threads (4 waves) owns a 128 x 256 output tile (or 128 x 128 for each of two B
// operands that share one A tile) and walks K in steps of 32 through three LDS stages of 24 KB.  Two
// workgroups fit one CU (72 KB LDS, <= 256 registers per lane each), so while one sits at its barrier,
// waits for loads, or runs its prologue/epilogue, the other keeps the CU's matrix cores fed.
// Each wave owns all 128 rows and a 64-column slice: 4 x 2 accumulators of v_mfma_f32_32x32x16_bf16.
//
// Pipeline.  Global->LDS copies are direct (16 bytes per lane, no register staging) and run two K steps
// ahead: at step i the wave waits until only step i+1's copies are outstanding, the workgroup barrier
// publishes stage i and retires stage i-1, then step i+2's copies are issued into the retired stage.
//
// LDS layouts.  An operand tile is kept the way it lies in memory and read in the shape the MFMA wants:
//   KC ("K contiguous": activations as A, transposed weights as B): [rows][32] bf16, 64 B per row,
//       16-byte piece c of row r stored at piece c ^ ((r >> 2) & 3); a fragment is one 16-byte LDS read.
//   MC ("M/N contiguous": weights stored [K][N], and both operands of the weight-gradient GEMMs):
//       [32][W] bf16, 16-byte piece c of K-row r stored at piece c ^ ((r & 3) << 2); a fragment comes
//       from two transposing 8-byte LDS reads (ds_read_b64_tr_b16), each yielding 4 consecutive K of one
//       column.
//   Both swizzles make the fragment reads and the tile fills bank-conflict free; since a direct copy lands
//   at base + 16*lane, the swizzle is applied by choosing which global piece each lane copies.
//
// MFMA.  The weight-side fragment is passed as the first source and the activation-side fragment as the
// second, so a lane's 16 accumulators hold 4 groups of 4 consecutive output columns of one output row.
#pragma once
#include "common.hpp"

namespace grouter {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;            // K step
constexpr int kThreads = 256;      // 4 waves
constexpr int kStages = 3;
constexpr int kATileBytes = 8 * 1024;    // 128 x 32 bf16
constexpr int kBTileBytes = 16 * 1024;   // 32 x 256 bf16 (or two 32 x 128 halves, or 256 x 32 K-contiguous)
constexpr int kStageBytes = kATileBytes + kBTileBytes;
constexpr int kSmemBytes = kStages * kStageBytes;  // 72 KB
constexpr int kTileM = 128;

// 16 bytes per lane from global memory straight into LDS at lds_wave_addr + 16*lane (lds_wave_addr is the
// wave-uniform LDS byte address).  Issued as inline assembly on purpose: the compiler's own tracking of
// LDS-writing loads waits for all of them before any later LDS read, which would serialise the pipeline
// stages; here the only waits are the explicit ones in front of the stage barrier.  M0 is a register the
// compiler reserves and re-loads immediately before each of its own uses, so writing it here is safe.
__device__ __forceinline__ void async_copy16(const char* src, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_wave_addr), "v"(src)
                 : "memory");
}
template <int N>
__device__ __forceinline__ void wait_async_copies() {  // until at most N of this wave's copies are outstanding
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7fffu + ((ua >> 16) & 1u);
    ub += 0x7fffu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xffff0000u);
}
__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// ---------------------------------------------------------------------------------------------------
// KC tile: ROWS x 32.  Thread t fills, in pass p, the 16-byte slot (p*256 + t): row p*64 + (t>>2), stored
// piece t&3, which holds source piece (t&3) ^ ((t>>4)&3) of that row.
template <int ROWS>
struct KcTile {
    static constexpr int kPasses = ROWS / 64;
    static __device__ __forceinline__ int src_piece(int tid) { return (tid & 3) ^ ((tid >> 4) & 3); }
    static __device__ __forceinline__ int row_of(int tid, int pass) { return pass * 64 + (tid >> 2); }
    static __device__ __forceinline__ uint32_t wave_dst(uint32_t tile, int tid, int pass) {
        return __builtin_amdgcn_readfirstlane(tile + (uint32_t)(pass * 256 + (tid & ~63)) * 16u);
    }
    // 16-byte fragment of a 32-row block starting at r0 (multiple of 32), K sub-step kk (0..1)
    static __device__ __forceinline__ bf16x8 read_frag(const char* tile, int lane, int r0, int kk) {
        const int r = lane & 31;
        const int piece = (kk * 2 + (lane >> 5)) ^ ((r >> 2) & 3);
        return *(const bf16x8*)(tile + (r0 + r) * 64 + (piece << 4));
    }
};

// MC tile: 32 x W (W = 128 or 256).  Slot (p*256 + t) is K-row slot / (W/8), stored piece slot % (W/8).
template <int W>
struct McTile {
    static constexpr int kPieces = W / 8;               // 16-byte pieces per K-row
    static constexpr int kPasses = 32 * kPieces / 256;   // 2 or 4
    static constexpr int kRowsPerPass = 256 / kPieces;   // 16 or 8
    static __device__ __forceinline__ int krow_of(int tid, int pass) { return pass * kRowsPerPass + tid / kPieces; }
    static __device__ __forceinline__ int src_piece(int tid) {
        const int krow = tid / kPieces;
        return (tid % kPieces) ^ ((krow & 3) << 2);
    }
    static __device__ __forceinline__ uint32_t wave_dst(uint32_t tile, int tid, int pass) {
        return __builtin_amdgcn_readfirstlane(tile + (uint32_t)(pass * 256 + (tid & ~63)) * 16u);
    }
    // fragment of 32 columns starting at n0 (multiple of 32), K sub-step kk: two transposing 8-byte reads
    static __device__ __forceinline__ bf16x8 read_frag(const char* tile, int lane, int n0, int kk) {
        const int i = lane & 15;
        const int krow = kk * 16 + 8 * (lane >> 5) + (i >> 2);
        const int col = n0 + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
        const int piece = (col >> 3) ^ ((krow & 3) << 2);
        const int off = krow * (2 * W) + (piece << 4) + ((col >> 2) & 1) * 8;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(tile + off));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4*)(tile + off + 4 * (2 * W)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
};

__device__ __forceinline__ f32x16 mfma(bf16x8 w_side, bf16x8 x_side, f32x16 acc) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(w_side, x_side, acc, 0, 0, 0);
}

// Output coordinates of accumulator group q (0..3) of a 32x32 fragment: row = lane&31, 4 consecutive
// columns starting at 8*q + 4*(lane>>5).
__device__ __forceinline__ int frag_col4(int lane, int q) { return 8 * q + 4 * (lane >> 5); }

// XCD-aware placement: consecutive workgroup ids go round-robin to the 8 XCDs, so give every XCD one
// contiguous range of the `n_real` logical tiles (neighbouring tiles share operand panels in that
// XCD's L2).  Only ids below n_real may call this.
__device__ __forceinline__ int xcd_remap(int b, int n_real) {
    const int x = b & 7, q = b >> 3;
    const int base = n_real >> 3, rem = n_real & 7;
    return x * base + min(x, rem) + q;
}

// ---------------------------------------------------------------------------------------------------
// The K loop shared by every GEMM.  `issue_all(step, stage_lds_addr)` enqueues the kLoads direct copies
// per thread of K step `step`; `compute(stage_ptr, next_step, next_stage_lds_addr)` runs the MFMAs of one
// stage and, when next_step >= 0, drips that step's copies in between them so the memory pipeline sees a
// steady stream instead of a burst that would block the wave in front of its MFMAs.
template <int kLoads, class IssueAll, class Compute>
__device__ __forceinline__ void k_pipeline(int n_steps, char* smem, IssueAll issue_all, Compute compute) {
    const uint32_t smem_addr = lds_addr(smem);
    if (n_steps > 0) issue_all(0, smem_addr);
    if (n_steps > 1) issue_all(1, smem_addr + kStageBytes);
    int stage = 0;
#ifdef GROUTER_EXP_NO_LOADS
    wait_async_copies<0>();
    __syncthreads();
#endif
    for (int it = 0; it < n_steps; ++it) {
#ifndef GROUTER_EXP_NO_LOADS
        if (it + 1 < n_steps)
            wait_async_copies<kLoads>();
        else
            wait_async_copies<0>();
#endif
#ifndef GROUTER_EXP_NO_BARRIER
        __syncthreads();
#endif
        const int s2 = stage >= 1 ? stage - 1 : stage + 2;  // (it + 2) % 3
#ifdef GROUTER_EXP_NO_LOADS
        compute((const char*)smem + stage * kStageBytes, -1, smem_addr + s2 * kStageBytes);
#else
        compute((const char*)smem + stage * kStageBytes, it + 2 < n_steps ? it + 2 : -1, smem_addr + s2 * kStageBytes);
#endif
        stage = stage == kStages - 1 ? 0 : stage + 1;
    }
}

// Register-staged variant of the K loop (experiment): global -> VGPR loads issued at the top of a step,
// written to LDS at its end.
struct StagedRegs {
    u32x4 v[6];
};
template <class LoadAll, class StoreAll, class Compute>
__device__ __forceinline__ void k_pipeline_regs(int n_steps, char* smem, LoadAll load_all, StoreAll store_all,
                                                Compute compute) {
    StagedRegs r;
    if (n_steps > 0) { load_all(0, r); store_all(smem, r); }
    if (n_steps > 1) { load_all(1, r); store_all(smem + kStageBytes, r); }
    __syncthreads();
    int stage = 0;
    for (int it = 0; it < n_steps; ++it) {
        const int s2 = stage >= 1 ? stage - 1 : stage + 2;  // (it + 2) % 3
        if (it + 2 < n_steps) load_all(it + 2, r);
        compute((const char*)smem + stage * kStageBytes, -1, 0u);
        if (it + 2 < n_steps) store_all(smem + s2 * kStageBytes, r);
        __syncthreads();
        stage = stage == kStages - 1 ? 0 : stage + 1;
    }
}

template <int J>
struct IntC {
    static constexpr int value = J;
};

// ---------------------------------------------------------------------------------------------------
// Output staging: a 128 x COLS bf16 tile goes from accumulator layout through LDS and leaves as 16-byte
// pieces of whole rows, so every global store is a full contiguous row segment.
constexpr int kOutPitch256 = 256 * 2 + 16;  // bytes per staged row; the 16-byte pad spreads rows over banks
constexpr int kOutPitch128 = 128 * 2 + 16;

// Each lane deposits 4 consecutive columns (8 bytes) of its row.
template <int PITCH>
__device__ __forceinline__ void stage_put4(char* smem, int row, int col, float c0, float c1, float c2, float c3) {
    *(u32x2*)(smem + row * PITCH + col * 2) = u32x2{pack_bf16_rne(c0, c1), pack_bf16_rne(c2, c3)};
}

// Write the staged tile: rows [0, rows_valid), columns [0, cols_valid) (multiple of 8) to dst (row pitch ld).
template <int COLS, int PITCH>
__device__ __forceinline__ void stage_flush(const char* smem, int tid, bf16_t* dst, size_t ld, int rows_valid,
                                            int cols_valid) {
    constexpr int kPiecesPerRow = COLS / 8;
    constexpr int kRowsPerPass = kThreads / kPiecesPerRow;
    const int piece = tid % kPiecesPerRow;
    const int r0 = tid / kPiecesPerRow;
    if (piece * 8 >= cols_valid) return;
#pragma unroll 4
    for (int r = r0; r < rows_valid; r += kRowsPerPass) {
        const u32x4 v = *(const u32x4*)(smem + r * PITCH + piece * 16);
        *(u32x4*)(dst + (size_t)r * ld + piece * 8) = v;
    }
}

}  // namespace grouter
