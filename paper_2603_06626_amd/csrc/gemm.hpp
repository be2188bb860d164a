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
constexpr int kSmemBytes = kStages * kStageBytes;  // 72 KB: the three A tiles first, then the three B tiles, so that
                                                   // every fragment address is a 16-bit immediate off one of two bases
constexpr int kBRegion = kStages * kATileBytes;
constexpr int kTileM = 128;

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor (gfx9 layout) over [base, base + bytes): accesses at or past `bytes` return zero
// instead of touching memory, which is how every ragged edge (rows past an expert's end, K and N tails) is
// masked.  bytes must stay below 2^31 so that kOutOfRange plus any scalar offset still compares as outside.
constexpr uint32_t kOutOfRange = 0x80000000u;
__device__ __forceinline__ i32x4 make_buffer(const void* base, uint32_t bytes) {
    const uint64_t b = (uint64_t)base;
    i32x4 r;
    r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    r.y = __builtin_amdgcn_readfirstlane((int)((uint32_t)(b >> 32) & 0xffffu));
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);
    r.w = 0x00020000;  // 32-bit data format, no swizzle, stride 0
    return r;
}

// 16 bytes per lane from a buffer straight into LDS at lds_wave_addr + 16*lane (lds_wave_addr is the
// wave-uniform LDS byte address).  The lane reads buffer offset voff + soff: voff is fixed per lane over the
// whole K loop and soff is a scalar that advances with K, so a copy costs no vector ALU work at all.
// Issued as inline assembly on purpose: the compiler's own tracking of LDS-writing loads waits for all of
// them before any later LDS read, which would serialise the pipeline stages; here the only waits are the
// explicit ones in front of the stage barrier.  M0 is a register the compiler reserves and re-loads
// immediately before each of its own uses, so writing it here is safe.
__device__ __forceinline__ void async_copy16(i32x4 buf, uint32_t voff, uint32_t soff, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_wave_addr), "v"(voff), "s"(buf), "s"(soff)
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
    // LDS byte offset of pass `pass` inside the tile, to be added to the wave's own base (wave index * 1024)
    static constexpr uint32_t pass_offset(int pass) { return (uint32_t)pass * 256u * 16u; }
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
    // LDS byte offset of pass `pass` inside the tile, to be added to the wave's own base (wave index * 1024)
    static constexpr uint32_t pass_offset(int pass) { return (uint32_t)pass * 256u * 16u; }
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
template <int J>
struct IntC {
    static constexpr int value = J;
};

// The K loop shared by every GEMM.  `issue_all(step, IntC<stage>)` enqueues the kLoads direct copies
// per thread of K step `step`; `compute(IntC<stage>, IntC<drip>, next_step)` runs the MFMAs of LDS stage
// `stage` and, when drip is 1, drips the copies of step `next_step` (= current + 2, bound for stage
// (stage + 2) % 3) in between them.  The steady state is unrolled by the three stages so that every LDS
// address is a compile-time offset and the loop body carries no stage arithmetic and no conditionals;
// `compute_tail(stage, next_step_or_-1)` is the same work with a run-time stage, for the last few steps.
template <int kLoads, class IssueAll, class Compute, class ComputeTail>
__device__ __forceinline__ void k_pipeline(int n_steps, char* smem, IssueAll issue_all, Compute compute,
                                           ComputeTail compute_tail) {
    if (n_steps > 0) issue_all(0, IntC<0>{});
    if (n_steps > 1) issue_all(1, IntC<1>{});
    int it = 0;
    for (; it + 5 <= n_steps; it += 3) {  // steps it, it+1, it+2 each still have a step two ahead to fetch
        wait_async_copies<kLoads>();
        __syncthreads();
        compute(IntC<0>{}, IntC<1>{}, it + 2);
        wait_async_copies<kLoads>();
        __syncthreads();
        compute(IntC<1>{}, IntC<1>{}, it + 3);
        wait_async_copies<kLoads>();
        __syncthreads();
        compute(IntC<2>{}, IntC<1>{}, it + 4);
    }
    // at most four steps remain, starting in stage 0; they run through the run-time-indexed variant
    int stage = 0;
    for (; it < n_steps; ++it) {
        if (it + 1 < n_steps)
            wait_async_copies<kLoads>();
        else
            wait_async_copies<0>();
        __syncthreads();
        compute_tail(stage, it + 2 < n_steps ? it + 2 : -1);
        stage = stage == kStages - 1 ? 0 : stage + 1;
    }
}

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
