// Building blocks of the grouped bf16 MFMA GEMMs (gfx950): LDS tile layouts, direct global->LDS tile
// loads, MFMA fragment reads, the shared K-loop pipeline and the LDS-staged output writer.
//
// Shape.  A workgroup of 256 threads (4 waves) owns a 128 x 256 output tile (or 128 x 128 for each of two B
// operands that share one A tile).  Two workgroups fit one CU (80 KB LDS, <= 256 registers per lane each),
// so while one sits at its barrier, waits for loads, or runs its prologue/epilogue, the other keeps the
// CU's matrix cores fed.  Each wave owns all 128 rows and 64 columns: 4 x 2 accumulators of
// 32 x 32 blocks, each held in four v_mfma_f32_16x16x32_bf16 accumulators (this form sustains a higher rate
// under the chip's power limit than 32x32x16: fewer accumulator registers move per FLOP); one pipeline step
// is 32 MFMAs per wave.
//
// Loads.  Global->LDS copies are direct (buffer_load ... lds, 16 bytes per lane, no register staging) and
// run two steps ahead.  The vector L1 works on whole 128-byte lines - a copy instruction that touches 16
// half lines costs twice one that touches 8 full lines - so every copy instruction is laid out to cover
// full lines: K-contiguous operands are fetched 64 K-elements (128 B) per row at a time into "super tiles"
// that serve two consecutive steps, M/N-contiguous operands 32 K-rows at a time.
//
// LDS layouts (all bank-conflict free for both the copy and the fragment reads; since a direct copy lands at
// base + 16*lane, a swizzle is applied by choosing which global piece each lane copies):
//   KC super tile ("K contiguous": activations as A; transposed weights as B): [128 rows][64] bf16, 128 B
//       per row, 16-byte piece c of row r stored at piece c ^ ((r >> 1) & 7); a 16-row fragment over K = 32
//       is one 16-byte LDS read per lane.  Two buffers, refilled every second step.
//   MC tile ("M/N contiguous": weights stored [K][N], and both operands of the weight-gradient GEMMs):
//       [32][W] bf16, 16-byte piece c of K-row r stored at piece c ^ ((r & 3) << 2) ^ (((r >> 3) & 1) << 1); a
//       16-column fragment over K = 32 comes from two transposing 8-byte LDS reads (ds_read_b64_tr_b16), each
//       yielding 4 consecutive K of one column.  Three buffers, refilled every step.
//
// MFMA.  The weight-side fragment is passed as the first source and the activation-side fragment as the
// second, so each of a lane's accumulators holds 4 consecutive output columns of one output row.
#pragma once
#include "common.hpp"

namespace grouter {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

// A 32 x 32 block of the output lives in four 16 x 16 accumulators; an operand fragment of 32 rows (or columns)
// over K = 32 is two 16-wide halves of 8 bf16 per lane.
struct Acc32 {
    f32x4 s[4];
};
struct Frag32 {
    bf16x8 h[2];
};

constexpr int kThreads = 256;            // 4 waves
constexpr int kTileM = 128;
constexpr int kSuperBytes = 16 * 1024;   // KC super tile: 128 rows x 64 K
constexpr int kMcSmallBytes = 8 * 1024;  // MC tile 32 x 128
constexpr int kBTileBytes = 16 * 1024;   // per-step B buffer: MC 32 x 256, two MC 32 x 128 halves, or a KC super tile
constexpr int kBRegion = 2 * kSuperBytes;            // A buffers first (two super tiles or three small MC tiles)
constexpr int kSmemBytes = kBRegion + 3 * kBTileBytes;  // 80 KB

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
// them before any later LDS read, which would serialise the pipeline; here the only waits are the explicit
// ones in front of the step barrier.  M0 is named as clobbered, so the compiler re-loads it before any use of
// its own.
__device__ __forceinline__ void async_copy16(i32x4 buf, uint32_t voff, uint32_t soff, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_wave_addr), "v"(voff), "s"(buf), "s"(soff)
                 : "memory", "m0");
}
// The same for 4 bytes per lane: lands at lds_wave_addr + 4*lane.
__device__ __forceinline__ void async_copy4(i32x4 buf, uint32_t voff, uint32_t soff, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :
                 : "s"(lds_wave_addr), "v"(voff), "s"(buf), "s"(soff)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_async_copies() {  // until at most N of this wave's copies are outstanding
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// two fp32 -> two bf16 (round to nearest even) in one word, a in the low half: v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}
// 1 / (1 + e^-x) from the hardware exponential and reciprocal (about 1 ulp each; the results feed values that
// are rounded to bf16)
__device__ __forceinline__ float sigmoid_fast(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }
__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// ---------------------------------------------------------------------------------------------------
// KC super tile: 128 rows x 64 K.  Thread t fills, in pass p (0..3), the 16-byte slot (p*256 + t): row
// p*32 + (t>>3), stored piece t&7, which holds source piece (t&7) ^ ((t>>4)&7) of that row.  One copy
// instruction of a wave covers 8 rows x 128 B.
struct KcSuper {
    static constexpr int kPasses = 4;
    static __device__ __forceinline__ int src_piece(int tid) { return (tid & 7) ^ ((tid >> 4) & 7); }
    static __device__ __forceinline__ int row_of(int tid, int pass) { return pass * 32 + (tid >> 3); }
    static constexpr uint32_t pass_offset(int pass) { return (uint32_t)pass * 256u * 16u; }
    // fragment of the 32-row block starting at r0 (multiple of 32) over K half `half` (0..1) of the super tile:
    // lane l holds, for each 16-row half of the block, row l % 16 and the 8 K values from 8 * (l / 16)
    static __device__ __forceinline__ Frag32 read_frag(const char* tile, int lane, int r0, int half) {
        const int r = lane & 15;
        const int piece = (half * 4 + (lane >> 4)) ^ ((r >> 1) & 7);
        const char* at = tile + (r0 + r) * 128 + (piece << 4);
        Frag32 f;
        f.h[0] = *(const bf16x8*)at;
        f.h[1] = *(const bf16x8*)(at + 16 * 128);
        return f;
    }
};

// MC tile: 32 x W (W = 128 or 256).  Slot (p*256 + t) is K-row slot / (W/8), stored piece slot % (W/8).
template <int W>
struct McTile {
    static constexpr int kPieces = W / 8;               // 16-byte pieces per K-row
    static constexpr int kPasses = 32 * kPieces / 256;   // 2 or 4
    static constexpr int kRowsPerPass = 256 / kPieces;   // 16 or 8
    static __device__ __forceinline__ int krow_of(int tid, int pass) { return pass * kRowsPerPass + tid / kPieces; }
    static __device__ __forceinline__ int swizzle(int krow) { return ((krow & 3) << 2) ^ (((krow >> 3) & 1) << 1); }
    static __device__ __forceinline__ int src_piece(int tid, int pass) { return (tid % kPieces) ^ swizzle(krow_of(tid, pass)); }
    static constexpr uint32_t pass_offset(int pass) { return (uint32_t)pass * 256u * 16u; }
    // fragment of the 32 columns starting at n0 (multiple of 32) over the tile's 32 K-rows: per 16-column half two
    // transposing 8-byte reads; lane l ends up with column l % 16 and the 8 K values from 8 * (l / 16).  The 16
    // lanes of a group address a 4 (K) x 16 (columns) block; the swizzle keeps the four blocks that are read
    // together (K-rows 0-3 and 8-11, or 16-19 and 24-27, ...) on different banks.
    // What depends on the lane is computed once (lane_base: its K-row and its place inside column block 0); the
    // fragment's first column only flips address bits, so an address costs one XOR with a constant.
    static __device__ __forceinline__ uint32_t lane_base(int lane) {
        const int i = lane & 15;
        const int krow = 8 * (lane >> 4) + (i >> 2);
        const int c4 = (i & 3) * 4;
        return (uint32_t)(krow * (2 * W) + (((c4 >> 3) ^ swizzle(krow)) << 4) + ((c4 >> 2) & 1) * 8);
    }
    static __device__ __forceinline__ uint32_t column_bits(int n0) { return (uint32_t)(n0 >> 3) << 4; }   // n0 % 16 == 0
    static __device__ __forceinline__ Frag32 read_frag(const char* tile, uint32_t base, int n0) {
        Frag32 f;
#pragma unroll
        for (int cn = 0; cn < 2; ++cn) {
            const uint32_t off = base ^ column_bits(n0 + cn * 16);
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(tile + off));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                (__attribute__((address_space(3))) bf16x4*)(tile + off + 4 * (2 * W)));
            f.h[cn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
        return f;
    }
};

// acc += x_side (32 rows x K 32) * w_side (K 32 x 32 columns): sub-block q = 2 * (row half) + (column half).
__device__ __forceinline__ void mfma32(const Frag32& w_side, const Frag32& x_side, Acc32& acc) {
#pragma unroll
    for (int rm = 0; rm < 2; ++rm)
#pragma unroll
        for (int cn = 0; cn < 2; ++cn)
            acc.s[rm * 2 + cn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w_side.h[cn], x_side.h[rm], acc.s[rm * 2 + cn], 0, 0, 0);
}
__device__ __forceinline__ void clear(Acc32& acc) {
#pragma unroll
    for (int q = 0; q < 4; ++q) acc.s[q] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// Output coordinates of sub-block q (0..3) of a 32 x 32 block: row frag_row, 4 consecutive columns from frag_col4.
__device__ __forceinline__ int frag_row(int lane, int q) { return 16 * (q >> 1) + (lane & 15); }
__device__ __forceinline__ int frag_col4(int lane, int q) { return 16 * (q & 1) + 4 * (lane >> 4); }

// XCD-aware placement: consecutive workgroup ids go round-robin to the 8 XCDs, so give every XCD one
// contiguous range of the `n_real` logical tiles (neighbouring tiles share operand panels in that
// XCD's L2).  Only ids below n_real may call this.
__device__ __forceinline__ int xcd_remap(int b, int n_real) {
    const int x = b & 7, q = b >> 3;
    const int base = n_real >> 3, rem = n_real & 7;
    return x * base + min(x, rem) + q;
}

template <int J>
struct IntC {
    static constexpr int value = J;
};

// ---------------------------------------------------------------------------------------------------
// The step loop shared by every GEMM.  A step is 32 MFMAs per wave.  Per-step ("B") buffers rotate through
// three LDS slots and are fetched two steps ahead, four copies per thread and step; when kSuperA is set the
// A operand lives in two super-tile buffers that each serve two consecutive steps and are fetched (four
// copies) during the even step two ahead, otherwise A is part of the per-step buffers (two more copies).
//
//   prepare_a()                           called once, after the first per-step copies are on their way
//   issue_a(super_index, a_buffer)        kSuperA: enqueue the 4 copies of A super tile `super_index`
//   issue_b(step, IntC<slot>)             enqueue the per-step copies of `step` into slot `slot`
//   compute(IntC<slot>, IntC<half>, a_buffer, issue)   the 32 MFMAs of one step; `issue()` is called once
//                                         part-way through to enqueue the copies that belong to this step
//   compute_rt(slot, half, a_buffer, issue)   the same with run-time indices (loop tail)
// Copies complete in issue order, so "wait until at most N are outstanding" is all the synchronisation a wave
// needs before the step barrier: the N youngest are exactly the ones issued for later steps.
struct NoPrepare {
    __device__ __forceinline__ void operator()() const {}
};
template <bool kSuperA, int kStepCopies, class IssueA, class IssueB, class Compute, class ComputeRt, class PrepareA = NoPrepare>
__device__ __forceinline__ void step_pipeline(int n_steps, IssueA issue_a, IssueB issue_b, Compute compute,
                                              ComputeRt compute_rt, PrepareA prepare_a = PrepareA{}) {
    if (n_steps <= 0) return;
    constexpr int kACopies = kSuperA ? 4 : 0;
    // prologue: the per-step buffers of step 0 (their addresses are known first: a gathered A operand still
    // waits for its row map and finishes its offsets in prepare_a), A super tile 0, then the per-step buffers
    // of step 1
    issue_b(0, IntC<0>{});
    prepare_a();
    if (kSuperA) issue_a(0, 0);
    if (n_steps > 1) issue_b(1, IntC<1>{});
    int j = 0;
    int abuf = 0;  // A super buffer of the current step: (j / 2) % 2
    // Steady state, unrolled over the three slots and the two halves of a super tile.  Every copy named in
    // the body exists as long as step j + 7 does.
    for (; j + 8 <= n_steps; j += 6) {
#define GROUTER_STEP(u, SLOT, HALF)                                                                            \
    {                                                                                                          \
        if (kSuperA && (HALF) == 1) wait_async_copies<kStepCopies + kACopies>();                               \
        else wait_async_copies<kStepCopies>();                                                                 \
        __syncthreads();                                                                                       \
        const int cur = j + (u);                                                                               \
        compute(IntC<SLOT>{}, IntC<HALF>{}, abuf, [&]() {                                                      \
            if (kSuperA && (HALF) == 0) issue_a(cur / 2 + 1, abuf ^ 1);                                        \
            issue_b(cur + 2, IntC<((SLOT) + 2) % 3>{});                                                        \
        });                                                                                                    \
        if ((HALF) == 1) abuf ^= 1;                                                                            \
    }
        GROUTER_STEP(0, 0, 0)
        GROUTER_STEP(1, 1, 1)
        GROUTER_STEP(2, 2, 0)
        GROUTER_STEP(3, 0, 1)
        GROUTER_STEP(4, 1, 0)
        GROUTER_STEP(5, 2, 1)
#undef GROUTER_STEP
    }
    // Tail: the same schedule with run-time indices and existence checks; waits are exact.
    int slot = 0;
    for (; j < n_steps; ++j) {
        const int half = j & 1;
        // copies younger than the ones this step needs: those issued during step j-1
        const bool prev_issued_b = j + 1 < n_steps;                          // per-step copies of step j+1
        const bool prev_issued_a = kSuperA && half == 1 && (j + 1 < n_steps);  // super tile (j+1)/2, issued at even j-1
        if (prev_issued_b && prev_issued_a) wait_async_copies<kStepCopies + kACopies>();
        else if (prev_issued_b) wait_async_copies<kStepCopies>();
        else wait_async_copies<0>();
        __syncthreads();
        const int cur = j;
        compute_rt(slot, half, abuf, [&]() {
            if (kSuperA && half == 0 && cur + 2 < n_steps) issue_a(cur / 2 + 1, abuf ^ 1);
            if (cur + 2 < n_steps) {
                const int s2 = slot >= 1 ? slot - 1 : slot + 2;
                if (s2 == 0) issue_b(cur + 2, IntC<0>{});
                else if (s2 == 1) issue_b(cur + 2, IntC<1>{});
                else issue_b(cur + 2, IntC<2>{});
            }
        });
        if (half == 1) abuf ^= 1;
        slot = slot == 2 ? 0 : slot + 1;
    }
}

// ---------------------------------------------------------------------------------------------------
// Output staging: a 128 x COLS bf16 tile goes from accumulator layout through LDS and leaves as 16-byte
// pieces of whole rows, so every global store is a full contiguous row segment.
constexpr int kOutPitch256 = 256 * 2 + 16;  // bytes per staged row; the 16-byte pad spreads rows over banks
constexpr int kOutPitch128 = 128 * 2 + 16;

// Write the staged tile: rows [0, rows_valid), columns [0, cols_valid) (multiple of 8) to dst (row pitch ld).
// STREAM: the tile is not read again soon (weight gradients, saved activations), so it is stored with the
// streaming hint and does not displace operand panels in L2.  Otherwise (O and the per-row input gradient,
// which the k-way reduction reads right after this kernel) plain stores leave it in the memory-side cache.
template <int COLS, int PITCH, bool STREAM = true>
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
        u32x4* const to = (u32x4*)(dst + (size_t)r * ld + piece * 8);
        if constexpr (STREAM) __builtin_nontemporal_store(v, to);
        else *to = v;
    }
}

}  // namespace grouter
