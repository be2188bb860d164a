// Building blocks of the grouped bf16 MFMA GEMMs (gfx950): LDS tile layouts, direct global->LDS tile
// loads, MFMA fragment reads, and the two kernel skeletons ("row" GEMMs whose ragged dimension is the
// expert's row count, and weight-gradient GEMMs whose ragged dimension is the reduction).
//
// Tiles.  A workgroup of 512 threads (8 waves, 2 x 4) owns a 256 x 256 output tile (or 256 x 128 for each
// of two B operands that share one A tile) and walks K in steps of 64 through two LDS stages of 64 KB.
// Global loads go straight to LDS (16 bytes per lane, no register staging); one barrier per K step.
//
// LDS layouts.  An operand tile is kept the way it lies in memory and read in the shape the MFMA wants:
//   KC ("K contiguous": activations as A, transposed weights as B): [rows][64] bf16, 128 B per row,
//       16-byte piece c of row r stored at piece c ^ ((r >> 1) & 7); fragments are one 16-byte LDS read.
//   MC ("M/N contiguous": weights stored [K][N], and both operands of the weight-gradient GEMMs):
//       [64][W] bf16, 16-byte piece c of K-row r stored at piece c ^ ((r & 3) << 2); fragments come
//       from two transposing 8-byte LDS reads (ds_read_b64_tr_b16), each yielding 4 consecutive K for
//       one column.
//   Both swizzles make the fragment reads and the tile fills bank-conflict free.
//
// MFMA.  v_mfma_f32_32x32x16_bf16; the weight-side fragment is passed as the first source and the
// activation-side fragment as the second, so a lane's 16 accumulators hold 4 groups of 4 consecutive
// output columns of one output row - stores and epilogue loads are 8-byte pieces of a row.
#pragma once
#include "common.hpp"

namespace grouter {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBK = 64;          // K step
constexpr int kThreads = 512;    // 8 waves
constexpr int kStageBytes = 64 * 1024;
constexpr int kATileBytes = 32 * 1024;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// 16 bytes per lane from global memory straight into LDS at lds_wave_addr + 16*lane (lds_wave_addr is the
// wave-uniform LDS byte address).  Issued as inline assembly on purpose: the compiler's own tracking of
// LDS-writing loads waits for all of them before any later LDS read, which would serialise the two
// pipeline stages; here the only wait is the explicit one in front of the stage barrier.
__device__ __forceinline__ void async_copy16(const char* src, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_wave_addr), "v"(src)
                 : "memory", "m0");
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
// KC tile: ROWS x 64.  Thread t fills, in pass `it`, the 16-byte slot (it*512 + t): row it*64 + (t>>3),
// stored piece t&7, which holds source piece (t&7) ^ ((t>>4)&7) of that row.
template <int ROWS>
struct KcTile {
    static constexpr int kPasses = ROWS / 64;
    // source piece (0..7) this thread copies, the same in every pass
    static __device__ __forceinline__ int src_piece(int tid) { return (tid & 7) ^ ((tid >> 4) & 7); }
    static __device__ __forceinline__ int row_of(int tid, int pass) { return pass * 64 + (tid >> 3); }
    static __device__ __forceinline__ uint32_t wave_dst(uint32_t tile, int tid, int pass) {
        return __builtin_amdgcn_readfirstlane(tile + (uint32_t)(pass * 512 + (tid & ~63)) * 16u);
    }
    // 16-byte fragment address of a 32-row block starting at r0 (multiple of 32), K sub-step kk (0..3)
    static __device__ __forceinline__ int frag_off(int lane, int r0, int kk) {
        const int piece = (kk * 2 + (lane >> 5)) ^ ((lane >> 1) & 7);
        return (r0 + (lane & 31)) * 128 + (piece << 4);
    }
    static __device__ __forceinline__ bf16x8 read_frag(const char* tile, int lane, int r0, int kk) {
        return *(const bf16x8*)(tile + frag_off(lane, r0, kk));
    }
};

// MC tile: 64 x W (W = 128 or 256).  Slot (it*512 + t) is K-row slot / (W/8), stored piece slot % (W/8).
template <int W>
struct McTile {
    static constexpr int kPieces = W / 8;              // 16-byte pieces per K-row
    static constexpr int kPasses = 64 * kPieces / 512;  // 2 or 4
    static constexpr int kRowsPerPass = 512 / kPieces;  // 32 or 16
    static __device__ __forceinline__ int krow_of(int tid, int pass) { return pass * kRowsPerPass + tid / kPieces; }
    static __device__ __forceinline__ int src_piece(int tid) {
        const int krow = tid / kPieces;
        return (tid % kPieces) ^ ((krow & 3) << 2);
    }
    static __device__ __forceinline__ uint32_t wave_dst(uint32_t tile, int tid, int pass) {
        return __builtin_amdgcn_readfirstlane(tile + (uint32_t)(pass * 512 + (tid & ~63)) * 16u);
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

}  // namespace grouter
