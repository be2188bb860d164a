// The grouped-GEMM kernels.  See gemm.hpp for tile layouts and the step pipeline.
#pragma once
#include "gemm.hpp"

namespace grouter {

__device__ __forceinline__ u32x2 pack_acc(const Acc32& c, int q) {
    return u32x2{pack_bf16_rne(c.s[q][0], c.s[q][1]), pack_bf16_rne(c.s[q][2], c.s[q][3])};
}

// Accumulators -> LDS -> whole-row stores for one 128 x BN output tile.  A wave holds, for each of its 4 row
// blocks, FN column blocks of 32 x 32; `col_of(fn)` is the tile column where block fn starts and
// `packed(fm, fn, q)` returns the four bf16 (two packed words) of sub-block q of block (fm, fn).
template <int BN, int FN, bool STREAM = true, class ColOf, class Packed>
__device__ __forceinline__ void write_tile(char* smem, int tid, bf16_t* dst, size_t ld, int rows_valid, int cols_valid,
                                           ColOf col_of, Packed packed) {
    constexpr int PITCH = (BN == 256) ? kOutPitch256 : kOutPitch128;
    const int lane = tid & 63;
    __syncthreads();  // earlier LDS readers (step loop, previous output) are done
#pragma unroll
    for (int fm = 0; fm < 4; ++fm) {
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int m = fm * 32 + frag_row(lane, q);
                const int n = col_of(fn) + frag_col4(lane, q);
                *(u32x2*)(smem + m * PITCH + n * 2) = packed(fm, fn, q);
            }
        __builtin_amdgcn_sched_barrier(0);  // keep a fused epilogue's loads from piling up across fragments
    }
    __syncthreads();
    stage_flush<BN, PITCH, STREAM>(smem, tid, dst, ld, rows_valid, cols_valid);
}

struct RowsArgs {
    const int32_t* tiles;        // [max_tiles][8]: expert, the expert's first row, row count, first tile, tile count
    int max_tiles;
    PlanDims plan;               // header[1] = number of row tiles actually present
    const bf16_t* A0; const bf16_t* A1;   // [Nrows][K]
    const bf16_t* B0; const bf16_t* B1;   // [E] slabs of K*Ncols elements
    bf16_t* C0; bf16_t* C1; bf16_t* C2;   // [Nrows][Ncols]
    const bf16_t* E0; const bf16_t* E1;   // epilogue inputs [Nrows][Ncols]
    int K, Ncols, n_ntiles;
    int col_group;               // > 0: walk an expert's tiles in groups of this many column tiles, row tiles fastest
    // gathered A: row p of the tile list is row row_token[p] of the token-ordered matrix A0, whose size is
    // a_total_bytes
    const int32_t* row_token;
    uint32_t a_total_bytes;
    const float* row_gate;       // per expert-sorted row: Eq. 1's routing weight of the slot behind it
};

struct RowTile {
    int e, row0, rows, col0;
};
template <int BN>
__device__ __forceinline__ bool pick_row_tile(const RowsArgs& a, RowTile& t) {
    const int n_real = a.plan.row_tiles() * a.n_ntiles;   // negative for a plan of other dimensions
    if ((int)blockIdx.x >= n_real) return false;
    const int L = xcd_remap(blockIdx.x, n_real);
    const int mt = L / a.n_ntiles;
    int nt = L - mt * a.n_ntiles;
    // every tile of an expert carries the same record, so whichever of the expert's tiles this workgroup ends
    // up with, one load (which follows the header's) has told it everything
    typedef int32_t i32x8 __attribute__((ext_vector_type(8)));
    const i32x8 rec = *(const i32x8*)(a.tiles + 8 * (size_t)mt);
    const int e = rec[0], e_off = rec[1], e_rows = rec[2], first = rec[3], cnt = rec[4];
    int m_in = mt - first;
    if (a.col_group > 0) {
        // Inside one expert's block of (row tile, column tile) pairs, take the column tiles in groups of
        // col_group and let the row tiles run fastest: the workgroups resident on an XCD at one time then use few
        // weight panels, which stay in its L2 however far apart in time the workgroups started.
        const int q = m_in * a.n_ntiles + nt;
        const int per_group = cnt * a.col_group;
        const int grp = q / per_group, rem = q - grp * per_group;
        const int g_here = min(a.col_group, a.n_ntiles - grp * a.col_group);
        m_in = rem / g_here;
        nt = grp * a.col_group + (rem - m_in * g_here);
    }
    t.e = e;
    t.row0 = e_off + m_in * kTileM;
    t.rows = min(kTileM, e_rows - m_in * kTileM);
    t.col0 = nt * BN;
    return true;
}

// Gate weights of a 128-row tile.  A lane owns 8 rows (16 i + lane % 16), but the four lanes that share lane % 16
// own the same ones: each lane loads only the two rows of row block lane / 16 (unconditionally, so that the loads
// are issued back to back and nothing waits for them before the epilogue; rows past the tile's end give 0), and
// the epilogue fetches what it needs from the lane that holds it.
struct RowGates {
    float w[2];
};
__device__ __forceinline__ RowGates load_row_gates(const RowsArgs& a, const RowTile& t, int lane) {
    RowGates g;
    const int last = a.plan.N - 1;
#pragma unroll
    for (int rm = 0; rm < 2; ++rm) {
        const int m = (lane >> 4) * 32 + rm * 16 + (lane & 15);
        const float v = a.row_gate[min(t.row0 + m, last)];
        g.w[rm] = m < t.rows ? v : 0.f;
    }
    return g;
}
// gate weight of this lane's row in row block fm (32 rows), 16-row half rm
__device__ __forceinline__ float row_gate_of(const RowGates& g, int lane, int fm, int rm) {
    return __shfl(g.w[rm], fm * 16 + (lane & 15));
}

// Gathered A operand: row r of the tile is row row_token[t.row0 + r] of a token-ordered [.][K] matrix.  In pass p
// a wave copies the 8 consecutive tile rows from 32 p + 8 wave, so it fetches their 8 token ids with wave-uniform
// loads (which travel through the scalar cache and do not queue behind the vector-memory copies of the other
// workgroup on the CU).  The loads are issued first (TokenIds::load); the offsets are finished (offsets) only
// after the first weight copies are on their way, so those copies do not wait for the ids.
struct TokenIds {
    int id[4][8];
    __device__ __forceinline__ void load(const RowsArgs& a, const RowTile& t, int tid) {
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int32_t* const at = a.row_token + t.row0 + p * 32 + wave * 8;   // padded by a tile's height: no clamp
#pragma unroll
            for (int i = 0; i < 8; ++i) id[p][i] = at[i];
        }
    }
    // byte offsets of the 4 copies of a KC super tile
    __device__ __forceinline__ void offsets(const RowTile& t, int tid, int K, uint32_t voff[4]) {
        const int sel = (tid >> 3) & 7;
        const int piece = KcSuper::src_piece(tid);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            // the ids are taken as of here: everything derived from them stays behind the copies issued so far
            asm volatile("" : "+s"(id[p][0]), "+s"(id[p][1]), "+s"(id[p][2]), "+s"(id[p][3]), "+s"(id[p][4]),
                              "+s"(id[p][5]), "+s"(id[p][6]), "+s"(id[p][7]));
            int tok = id[p][0];
#pragma unroll
            for (int i = 1; i < 8; ++i) tok = sel == i ? id[p][i] : tok;
            const int r = p * 32 + (tid >> 3);
            voff[p] = r < t.rows ? ((uint32_t)tok * (uint32_t)K + piece * 8) * 2u : kOutOfRange;
        }
    }
};

// Per-lane offsets of the 4 copies of a KC super tile whose rows start at row `first_row` of a [.][K] matrix
// (rows >= n_rows_valid are masked): byte offset of (row, piece) relative to the buffer base.
__device__ __forceinline__ void super_offsets(int tid, int first_row, int n_rows_valid, int K, uint32_t voff[4]) {
    const int piece = KcSuper::src_piece(tid);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = first_row + KcSuper::row_of(tid, p);
        voff[p] = r < n_rows_valid ? ((uint32_t)r * (uint32_t)K + piece * 8) * 2u : kOutOfRange;
    }
}

// ===================================================================================================
// Forward row GEMMs: C[rows of expert e][Ncols] = A[rows][K] * B_e with B_e stored [K][Ncols] (MC).
//   kGateUp  B = W1_e, W3_e [d][f]; two accumulator sets G, U; epilogue H = r * silu(G)*U, r the row's gate
//            weight: folding Eq. 1's routing weight in here (everything downstream is linear in H) lets the
//            combine be a plain sum and the backward pass work on the unscaled upstream gradient; for backward
//            it keeps the two partial derivatives of silu(G)*U (C0: by G, C1: by U)
//   kDown    B = W2_e [f][d]; epilogue O
// A is fetched as KC super tiles (two steps each), B as MC tiles of 32 K-rows.
// GATHER_A: the rows of A are gathered from the token-ordered input - a lane's copy offsets are fixed over
// the K loop anyway, so pointing them at the source token's row costs nothing and the permuted copy of the
// input is never made.  FWD_ONLY (gate/up when no backward follows): only H is stored.
enum FwdMode { kGateUp = 0, kDown = 1 };

template <int MODE, bool GATHER_A = false, bool FWD_ONLY = false>
__global__ __launch_bounds__(kThreads, 2) void k_fwd_gemm(const RowsArgs a) {
    static_assert(!FWD_ONLY || MODE == kGateUp, "only the gate/up GEMM has a forward-only form");
    constexpr int NB = (MODE == kGateUp) ? 2 : 1;
    constexpr int BN = (NB == 2) ? 128 : 256;  // columns per B operand
    constexpr int FN = BN / 128;               // 32-column fragments per wave and B operand
    constexpr int kBHalf = kBTileBytes / 2;    // second B operand of the two-operand mode
    using BMc = McTile<BN>;
    static_assert(NB * BMc::kPasses == 4, "four B copies per thread and step");

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];
    RowTile t;
    if (!pick_row_tile<BN>(a, t)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wave_base = __builtin_amdgcn_readfirstlane((uint32_t)wave * 1024u);
    const uint32_t smem_addr = __builtin_amdgcn_readfirstlane(lds_addr(smem));
    const int K = a.K, Ncols = a.Ncols;
    const int n_steps = (K + 31) / 32;

    // The A buffer covers exactly this tile's valid rows and the B buffer exactly this expert's slab, so
    // everything outside them reads as zero.
    const i32x4 bufA = GATHER_A ? make_buffer(a.A0, a.a_total_bytes)
                                : make_buffer(a.A0 + (size_t)t.row0 * K, (uint32_t)t.rows * (uint32_t)K * 2u);
    const size_t slab = (size_t)t.e * K * Ncols;
    const uint32_t slab_bytes = (uint32_t)K * (uint32_t)Ncols * 2u;
    const i32x4 bufB0 = make_buffer(a.B0 + slab, slab_bytes);
    const i32x4 bufB1 = NB == 2 ? make_buffer(a.B1 + slab, slab_bytes) : bufB0;
    const int a_piece = KcSuper::src_piece(tid);
    RowGates row_gate{};
    if constexpr (MODE == kGateUp) row_gate = load_row_gates(a, t, lane);   // needed only by the epilogue
    uint32_t a_voff[4];
    TokenIds ids;
    if constexpr (GATHER_A) ids.load(a, t, tid);
    else super_offsets(tid, 0, 128, K, a_voff);   // rows past t.rows fall outside bufA on their own
    auto prepare_a = [&]() {
        if constexpr (GATHER_A) ids.offsets(t, tid, K, a_voff);
    };
    uint32_t b_voff[BMc::kPasses];
#pragma unroll
    for (int p = 0; p < BMc::kPasses; ++p) {
        const int b_col = t.col0 + BMc::src_piece(tid, p) * 8;
        b_voff[p] = b_col < Ncols ? ((uint32_t)BMc::krow_of(tid, p) * (uint32_t)Ncols + b_col) * 2u : kOutOfRange;
    }

    auto issue_a = [&](int super, int abuf) {
        const int k0 = super * 64;
        const bool partial = k0 + 64 > K;  // the last super tile may stop mid-row
        const uint32_t dst = smem_addr + abuf * kSuperBytes + wave_base;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint32_t v = a_voff[p];
            if (partial) v = (k0 + a_piece * 8 < K) ? v : kOutOfRange;
            async_copy16(bufA, v, (uint32_t)k0 * 2u, dst + KcSuper::pass_offset(p));
        }
    };
    auto issue_b = [&](int step, auto slot_c) {
        const uint32_t dst = smem_addr + kBRegion + decltype(slot_c)::value * kBTileBytes + wave_base;
        const uint32_t soff = (uint32_t)step * 32u * (uint32_t)Ncols * 2u;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int p = 0; p < BMc::kPasses; ++p)
                async_copy16(nb ? bufB1 : bufB0, b_voff[p], soff, dst + nb * kBHalf + BMc::pass_offset(p));
    };

    Acc32 acc[NB][4][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < 4; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) clear(acc[nb][fm][fn]);

    // One step: all fragments are requested up front (LDS returns them in order, so the first MFMAs start once
    // the first ones have landed), the step's copies are enqueued after the first eight MFMAs.
    const uint32_t b_lane = BMc::lane_base(lane) ^ BMc::column_bits(wave * (BN / 4));   // this wave's columns
    auto step_body = [&](const char* At, const char* Bt, int half, auto issue) {
        Frag32 af[4], bf[2];
#pragma unroll
        for (int g = 0; g < 2; ++g) bf[g] = BMc::read_frag(Bt + (g / FN) * kBHalf, b_lane, (g % FN) * 32);
#pragma unroll
        for (int fm = 0; fm < 4; ++fm) af[fm] = KcSuper::read_frag(At, lane, fm * 32, half);
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) {
                mfma32(bf[g], af[fm], acc[g / FN][fm][g % FN]);
                if (g == 0 && fm == 1) issue();
            }
    };
    auto compute = [&](auto slot_c, auto half_c, int abuf, auto issue) {
        step_body(smem + abuf * kSuperBytes, smem + kBRegion + decltype(slot_c)::value * kBTileBytes,
                  decltype(half_c)::value, issue);
    };
    auto compute_rt = [&](int slot, int half, int abuf, auto issue) {
        step_body(smem + abuf * kSuperBytes, smem + kBRegion + slot * kBTileBytes, half, issue);
    };
    step_pipeline<true, 4>(n_steps, issue_a, issue_b, compute, compute_rt, prepare_a);

    // ---- epilogue: accumulators -> (fused elementwise) -> LDS -> whole-row 16-byte stores
    const int cols_valid = min(BN, Ncols - t.col0);
    const size_t tile_at = (size_t)t.row0 * Ncols + t.col0;
    auto col_of = [&](int fn) { return wave * (BN / 4) + fn * 32; };
    if constexpr (MODE == kGateUp) {
        float gate[4][2];
#pragma unroll
        for (int fm = 0; fm < 4; ++fm)
#pragma unroll
            for (int rm = 0; rm < 2; ++rm) gate[fm][rm] = row_gate_of(row_gate, lane, fm, rm);
        if constexpr (FWD_ONLY) {
            write_tile<BN, FN>(smem, tid, a.C2 + tile_at, (size_t)Ncols, t.rows, cols_valid, col_of, [&](int fm, int fn, int q) {
                float h[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float g = acc[0][fm][fn].s[q][r];
                    h[r] = gate[fm][q >> 1] * (g * sigmoid_fast(g) * acc[1][fm][fn].s[q][r]);
                }
                return u32x2{pack_bf16_rne(h[0], h[1]), pack_bf16_rne(h[2], h[3])};
            });
        } else {
            // What backward needs of G and U are the two partial derivatives of silu(G) * U, so those are what is
            // kept: with s = sigmoid(G), Q = silu(G) = G s (the derivative by U) and P = U (s + Q (1 - s)) (the
            // derivative by G).  Evaluated once, here, from the fp32 accumulators, which they replace in place; H
            // is packed on the side.  The dH epilogue is then two multiplications per element.
            u32x2 hp[4][FN][4];
#pragma unroll
            for (int fm = 0; fm < 4; ++fm)
#pragma unroll
                for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float h[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float g = acc[0][fm][fn].s[q][r], u = acc[1][fm][fn].s[q][r];
                            const float s = sigmoid_fast(g);
                            const float qv = g * s;
                            acc[0][fm][fn].s[q][r] = u * (s + qv * (1.f - s));
                            acc[1][fm][fn].s[q][r] = qv;
                            h[r] = gate[fm][q >> 1] * (qv * u);
                        }
                        hp[fm][fn][q] = u32x2{pack_bf16_rne(h[0], h[1]), pack_bf16_rne(h[2], h[3])};
                    }
            write_tile<BN, FN>(smem, tid, a.C0 + tile_at, (size_t)Ncols, t.rows, cols_valid, col_of,
                               [&](int fm, int fn, int q) { return pack_acc(acc[0][fm][fn], q); });
            write_tile<BN, FN>(smem, tid, a.C1 + tile_at, (size_t)Ncols, t.rows, cols_valid, col_of,
                               [&](int fm, int fn, int q) { return pack_acc(acc[1][fm][fn], q); });
            write_tile<BN, FN>(smem, tid, a.C2 + tile_at, (size_t)Ncols, t.rows, cols_valid, col_of,
                               [&](int fm, int fn, int q) { return hp[fm][fn][q]; });
        }
    } else {
        // O is read by the combine that follows: plain stores
        write_tile<BN, FN, false>(smem, tid, a.C0 + tile_at, (size_t)Ncols, t.rows, cols_valid, col_of,
                                              [&](int fm, int fn, int q) { return pack_acc(acc[0][fm][fn], q); });
    }
}

// ===================================================================================================
// Backward row GEMMs against transposed weights: C[rows][Ncols] = A[rows][K] * B_e^T with B_e stored
// [Ncols][K], so both operands are K-contiguous and both are fetched as KC super tiles of 64 K.
//   kDh   dH = r * (dY_rows W2_e^T) (K = d, Ncols = f; the rows of dY are gathered through the plan's row map
//         and the row's gate weight r is applied in fp32 afterwards); epilogue dG, dU = dH times the saved
//         derivatives of silu(G)*U by G and by U (E0, E1)
//   kDxp  dXp = dG W1_e^T + dU W3_e^T (two K phases of f each, Ncols = d)
// A step is one half of the 128 x 256 tile's columns over one 64-wide K block: step j uses A super tile j/2
// and the B super tile of half j%2; wave w owns 32 columns of each half, normally [64w + 32h, 64w + 32h + 32).
enum BwdMode { kDh = 0, kDxp = 1 };

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_bwd_gemm(const RowsArgs a) {
    constexpr int BN = 256;
    constexpr int NPH = (MODE == kDxp) ? 2 : 1;
    constexpr bool GATHER_A = MODE == kDh;  // dH reads the upstream gradient's rows straight from dY [T][d]

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];
    RowTile t;
    if (!pick_row_tile<BN>(a, t)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wave_base = __builtin_amdgcn_readfirstlane((uint32_t)wave * 1024u);
    const uint32_t smem_addr = __builtin_amdgcn_readfirstlane(lds_addr(smem));
    const int K = a.K, Ncols = a.Ncols;
    const int n_super = (K + 63) / 64;          // per phase
    const int n_steps = 2 * n_super * NPH;

    const i32x4 bufA0 = GATHER_A ? make_buffer(a.A0, a.a_total_bytes)
                                 : make_buffer(a.A0 + (size_t)t.row0 * K, (uint32_t)t.rows * (uint32_t)K * 2u);
    const i32x4 bufA1 = NPH == 2 ? make_buffer(a.A1 + (size_t)t.row0 * K, (uint32_t)t.rows * (uint32_t)K * 2u) : bufA0;
    const size_t slab = (size_t)t.e * K * Ncols;
    const uint32_t slab_bytes = (uint32_t)K * (uint32_t)Ncols * 2u;
    const i32x4 bufB0 = make_buffer(a.B0 + slab, slab_bytes);
    const i32x4 bufB1 = NPH == 2 ? make_buffer(a.B1 + slab, slab_bytes) : bufB0;
    const int piece = KcSuper::src_piece(tid);
    uint32_t a_voff[4], b_voff[2][4];
    TokenIds ids;
    if constexpr (GATHER_A) ids.load(a, t, tid);
    else super_offsets(tid, 0, 128, K, a_voff);
    auto prepare_a = [&]() {
        if constexpr (GATHER_A) ids.offsets(t, tid, K, a_voff);
    };
    RowGates row_gate{};
    if constexpr (MODE == kDh) row_gate = load_row_gates(a, t, lane);   // needed only by the epilogue
    // Which tile column row 32 p + i of step half h's B super tile (the rows wave p multiplies) stands for.  A wave's
    // two 32-column blocks lie side by side, so that it owns whole 128-byte lines of every output row; only a tile
    // whose columns 128.. lie past the matrix (Ncols % 256 <= 128 in the last column tile) puts all of its existing
    // columns into half 0, and half 1 is then skipped altogether.
    const bool right_half = t.col0 + 128 < Ncols;
    auto tile_col = [&](int h, int p) { return right_half ? 64 * p + 32 * h : 128 * h + 32 * p; };
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = t.col0 + tile_col(h, p) + (tid >> 3);   // a row of the [Ncols][K] weight slab
            b_voff[h][p] = r < Ncols ? ((uint32_t)r * (uint32_t)K + piece * 8) * 2u : kOutOfRange;
        }

    auto issue_super = [&](i32x4 buf, const uint32_t voff[4], int k0, uint32_t dst) {
        const bool partial = k0 + 64 > K;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            uint32_t v = voff[p];
            if (partial) v = (k0 + piece * 8 < K) ? v : kOutOfRange;
            async_copy16(buf, v, (uint32_t)k0 * 2u, dst + KcSuper::pass_offset(p));
        }
    };
    auto issue_a = [&](int super, int abuf) {
        const int ph = (NPH == 2 && super >= n_super) ? 1 : 0;
        issue_super(ph ? bufA1 : bufA0, a_voff, (super - ph * n_super) * 64, smem_addr + abuf * kSuperBytes + wave_base);
    };
    auto issue_b = [&](int step, auto slot_c) {
        const int super = step >> 1;
        const int ph = (NPH == 2 && super >= n_super) ? 1 : 0;
        const uint32_t dst = smem_addr + kBRegion + decltype(slot_c)::value * kBTileBytes + wave_base;
        if (step & 1) issue_super(ph ? bufB1 : bufB0, b_voff[1], (super - ph * n_super) * 64, dst);
        else issue_super(ph ? bufB1 : bufB0, b_voff[0], (super - ph * n_super) * 64, dst);
    };

    Acc32 acc[4][2];  // [row block][column half]
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) clear(acc[fm][hf]);

    // One step: 2 K halves of the super tiles x (4 A fragments, 1 B fragment) = 32 MFMAs into the wave's column
    // block `half`.  A tile without a right half skips half 1's fragment reads and MFMAs; its copies are still issued
    // (they are masked and fetch nothing), so the pipeline's copy counts stay as they are.
    auto step_body = [&](const char* At, const char* Bt, auto half_c, auto issue) {
        constexpr int hf = decltype(half_c)::value;
        if (hf == 1 && !right_half) {
            issue();
            return;
        }
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {  // one K half at a time keeps the fragment registers at 40
            Frag32 af[4];
            const Frag32 bf = KcSuper::read_frag(Bt, lane, wave * 32, kh);
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) af[fm] = KcSuper::read_frag(At, lane, fm * 32, kh);
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) {
                mfma32(bf, af[fm], acc[fm][hf]);
                if (kh == 0 && fm == 1) issue();
            }
        }
    };
    auto compute = [&](auto slot_c, auto half_c, int abuf, auto issue) {
        step_body(smem + abuf * kSuperBytes, smem + kBRegion + decltype(slot_c)::value * kBTileBytes, half_c, issue);
    };
    auto compute_rt = [&](int slot, int half, int abuf, auto issue) {
        if (half) step_body(smem + abuf * kSuperBytes, smem + kBRegion + slot * kBTileBytes, IntC<1>{}, issue);
        else step_body(smem + abuf * kSuperBytes, smem + kBRegion + slot * kBTileBytes, IntC<0>{}, issue);
    };
    step_pipeline<true, 4>(n_steps, issue_a, issue_b, compute, compute_rt, prepare_a);

    const int cols_valid = min(BN, Ncols - t.col0);
    const size_t tile_at = (size_t)t.row0 * Ncols + t.col0;
    auto col_of = [&](int hf) { return tile_col(hf, wave); };
    if constexpr (MODE == kDh) {
        // dG = dH * P,  dU = dH * Q with the forward pass's P = U s (1 + G (1 - s)) and Q = G s, s = sigmoid(G);
        // dH = gate weight * accumulator.
        // After one barrier (the step loop's LDS readers are done) every wave finishes its own 128 rows x 64
        // columns by itself, 32 rows at a time, in its own quarter of the LDS, so the waves neither wait for each
        // other nor for stores: the saved P and Q pieces of a chunk come in through the same direct copies as
        // the operands (two chunks ahead, two buffers), every lane picks its 8-byte pieces out of LDS and puts
        // dG / dU back in their place, and the lane that fetched a 16-byte piece stores the finished one at the
        // same offset of the output (P, Q, dG and dU share one layout).
        // A chunk buffer holds P then Q, each 32 rows x 128 B (the wave's two 32-column blocks); the 32-byte
        // piece p of row r sits at piece p ^ ((r >> 1) & 3) and its two 16-byte halves swap when r & 8, which
        // spreads the fragment-shaped picks (16 rows x 32 B per access) over all banks.
        constexpr uint32_t kWaveLds = kSmemBytes / 4;
        constexpr uint32_t kHalfChunk = 32 * 128;         // P or Q of one chunk
        constexpr uint32_t kChunkBytes = 2 * kHalfChunk;
        static_assert(2 * kChunkBytes <= kWaveLds, "two chunk buffers per wave");
        const uint32_t my_lds = __builtin_amdgcn_readfirstlane((uint32_t)wave * kWaveLds);
        const uint32_t rows_bytes = (uint32_t)t.rows * (uint32_t)Ncols * 2u;
        const size_t rows_at = (size_t)t.row0 * Ncols;
        const i32x4 bufP = make_buffer(a.E0 + rows_at, rows_bytes);
        const i32x4 bufQ = make_buffer(a.E1 + rows_at, rows_bytes);
        const __amdgpu_buffer_rsrc_t out_dg = __builtin_amdgcn_make_buffer_rsrc((void*)(a.C0 + rows_at), 0, (int)rows_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t out_du = __builtin_amdgcn_make_buffer_rsrc((void*)(a.C1 + rows_at), 0, (int)rows_bytes, 0x00020000);
        uint32_t pq_voff[4];   // of the piece this lane moves in pass p: rows past the tile's end fall outside the buffers
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = p * 8 + (lane >> 3);
            const int p32 = ((lane >> 1) & 3) ^ ((r >> 1) & 3);
            const int h16 = (lane & 1) ^ ((r >> 3) & 1);
            const int col = t.col0 + col_of(p32 >> 1) + (p32 & 1) * 16 + h16 * 8;
            pq_voff[p] = col < Ncols ? ((uint32_t)r * (uint32_t)Ncols + col) * 2u : kOutOfRange;
        }
        const uint32_t chunk_stride = 32u * (uint32_t)Ncols * 2u;
        auto issue_rows = [&](int c) {   // the saved pieces of chunk c: 8 copies
            const uint32_t dst = smem_addr + my_lds + (uint32_t)(c & 1) * kChunkBytes;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                async_copy16(bufP, pq_voff[p], (uint32_t)c * chunk_stride, dst + p * 1024u);
                async_copy16(bufQ, pq_voff[p], (uint32_t)c * chunk_stride, dst + kHalfChunk + p * 1024u);
            }
        };
        const int n_chunks = (t.rows + 31) >> 5;
        // the compiler's own wait for the row gates (loaded before the step loop) is taken here, while nothing is
        // in flight: placed at their first use it would also wait for the copies issued below
        asm volatile("" : : "v"(row_gate.w[0]), "v"(row_gate.w[1]));
        __syncthreads();  // the step loop's readers are done with this LDS
        issue_rows(0);
        if (n_chunks > 1) issue_rows(1);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (c >= n_chunks) break;
            // Chunk c's copies: what this wave issued after them are chunk c-1's 8 stores and chunk c+1's 8 copies.
            if (c + 1 < 4 && c + 1 < n_chunks) {
                if (c == 0) wait_async_copies<8>(); else wait_async_copies<16>();
            } else {
                if (c == 0) wait_async_copies<0>(); else wait_async_copies<8>();
            }
            char* const ldsP = smem + my_lds + (c & 1) * kChunkBytes;
            char* const ldsQ = ldsP + kHalfChunk;
            const float gate[2] = {row_gate_of(row_gate, lane, c, 0), row_gate_of(row_gate, lane, c, 1)};
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                if (hf == 1 && !right_half) break;   // those columns do not exist
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int rr = frag_row(lane, q);
                    const int p32 = (hf * 2 + (q & 1)) ^ ((rr >> 1) & 3);
                    const int sub = (lane >> 4) ^ (((rr >> 3) & 1) << 1);
                    const int at = rr * 128 + p32 * 32 + sub * 8;
                    const u32x2 pp = *(const u32x2*)(ldsP + at);
                    const u32x2 qp = *(const u32x2*)(ldsQ + at);
                    const float pv[4] = {bf16_lo(pp.x), bf16_hi(pp.x), bf16_lo(pp.y), bf16_hi(pp.y)};
                    const float qv[4] = {bf16_lo(qp.x), bf16_hi(qp.x), bf16_lo(qp.y), bf16_hi(qp.y)};
                    float dg[4], du[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float dh = gate[q >> 1] * acc[c][hf].s[q][r];
                        dg[r] = dh * pv[r];
                        du[r] = dh * qv[r];
                    }
                    *(u32x2*)(ldsP + at) = u32x2{pack_bf16_rne(dg[0], dg[1]), pack_bf16_rne(dg[2], dg[3])};
                    *(u32x2*)(ldsQ + at) = u32x2{pack_bf16_rne(du[0], du[1]), pack_bf16_rne(du[2], du[3])};
                }
            }
            // the wave's own LDS accesses stay in order, so the finished pieces can be picked up right away
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const u32x4 vg = *(const u32x4*)(ldsP + p * 1024 + lane * 16);
                const u32x4 vu = *(const u32x4*)(ldsQ + p * 1024 + lane * 16);
                __builtin_amdgcn_raw_buffer_store_b128(vg, out_dg, (int)pq_voff[p], (int)((uint32_t)c * chunk_stride), 0);
                __builtin_amdgcn_raw_buffer_store_b128(vu, out_du, (int)pq_voff[p], (int)((uint32_t)c * chunk_stride), 0);
            }
            // this buffer is free again (the stores hold its contents in registers): chunk c+2 may land in it
            if (c + 2 < 4 && c + 2 < n_chunks) issue_rows(c + 2);
        }
    } else {
        // the per-row input gradient is read by the reduction over each token's k rows that follows: plain stores
        write_tile<BN, 2, false>(smem, tid, a.C0 + tile_at, (size_t)Ncols, t.rows, cols_valid, col_of,
                                             [&](int fm, int hf, int q) { return pack_acc(acc[fm][hf], q); });
    }
}

// ===================================================================================================
// Weight-gradient GEMMs: C_e[Mdim][Ndim] = A_e^T * B_e, reduction over the expert's rows.
//   A [Nrows][Mdim], B0/B1 [Nrows][Ndim] in expert-sorted row order; C0/C1 [E][Mdim][Ndim].
//   NB = 1: one B (dW2 = H^T dY_rows).  NB = 2: two B sharing A (dW1 = x_rows^T dG, dW3 = x_rows^T dU).
// Both operands are M/N-contiguous MC tiles of 32 rows.  Experts are walked heaviest first so the long
// reductions start early; an expert without rows gets zeros.
//
// DwShare: which part of an expert's n_mt x n_nt tile grid XCD x works on.  Consecutive workgroup ids go round-robin to
// the 8 XCDs, each with its own L2; the grid is cut into 2 x 4 rectangles, one per XCD, so an A panel is
// fetched by 4 XCDs and a B panel by 2 instead of by all 8.  Which half / quarter gets the odd tiles rotates
// with the expert's load rank, so uneven cuts even out over experts; the pattern repeats every 4 ranks.
struct DwShare {
    int m_begin, msz, n_begin, nsz;
    __host__ __device__ DwShare(int x, int rank, int n_mt, int n_nt) {
        const int i = ((x >> 2) + rank) & 1, g = ((x & 3) + rank) & 3;
        const int m_lo = n_mt >> 1, m_extra = n_mt & 1;
        msz = m_lo + (i == 0 ? m_extra : 0);
        m_begin = i == 0 ? 0 : m_lo + m_extra;
        const int n_lo = n_nt >> 2, n_extra = n_nt & 3;
        nsz = n_lo + (g < n_extra ? 1 : 0);
        n_begin = g * n_lo + (g < n_extra ? g : n_extra);
    }
    __host__ __device__ int tiles() const { return msz * nsz; }
};

struct DwArgs {
    PlanDims plan;
    const int32_t* by_load;
    const int32_t* offsets;
    const int32_t* counts;
    const bf16_t* A;
    const bf16_t* B0; const bf16_t* B1;
    bf16_t* C0; bf16_t* C1;
    int Mdim, Ndim, n_mt, n_nt, n_experts;
    const int32_t* row_token;    // gathered operand: the token behind each expert-sorted row
    uint32_t gathered_bytes;     // size of the token-ordered matrix the gathered operand is read from
};

// GATHER: 0 = both operands lie in expert-sorted row order; 1 = A, 2 = B (NB == 1) is instead read from a
// token-ordered matrix [T][.] through row_token, so the expert-sorted copy of that matrix need not exist.
// Rows are the reduction dimension here, so a lane's copy offsets change every step: each wave keeps the
// token ids of the next steps' 32 rows in a small LDS ring, filled by one more direct copy per step four
// steps ahead (by then certainly landed: the step's wait leaves only the previous step's copies outstanding).
// Past the expert's last row the ids read as token 0; the other operand is zero there, so nothing is added.
enum DwGather { kGatherNone = 0, kGatherA = 1, kGatherB = 2 };
constexpr int kIdRingAt = 24 * 1024;  // between the A slots (3 x 8 KB) and the B slots (from 32 KB)

template <int NB, int GATHER = kGatherNone>
__global__ __launch_bounds__(kThreads, 2) void k_dw_gemm(const DwArgs a) {
    static_assert(GATHER != kGatherB || NB == 1, "a gathered B operand is only provided for one B");
    constexpr int kStepCopies = GATHER == kGatherNone ? 6 : 7;
    constexpr int BN = (NB == 2) ? 128 : 256;
    constexpr int FN = BN / 128;
    constexpr int kBHalf = kBTileBytes / 2;
    using ATile = McTile<128>;
    using BTile = McTile<BN>;
    static_assert(ATile::kPasses == 2 && NB * BTile::kPasses == 4, "six copies per thread and step");

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wave_base = __builtin_amdgcn_readfirstlane((uint32_t)wave * 1024u);
    const uint32_t smem_addr = __builtin_amdgcn_readfirstlane(lds_addr(smem));
    // Tile -> workgroup mapping (see DwShare): XCD x = blockIdx % 8 walks its rectangles heaviest expert first.
    if (!a.plan.match()) return;
    int rank, mt, nt;
    {
        const int x = blockIdx.x & 7, q = blockIdx.x >> 3;
        int per_quad = 0;
#pragma unroll
        for (int tq = 0; tq < 4; ++tq) per_quad += DwShare(x, tq, a.n_mt, a.n_nt).tiles();
        if (per_quad == 0) return;
        const int quad = q / per_quad;
        int r = q - quad * per_quad;
        rank = quad * 4;
        DwShare sh(x, rank, a.n_mt, a.n_nt);
#pragma unroll 1
        for (int tq = 0; tq < 3 && r >= sh.tiles(); ++tq) {
            r -= sh.tiles();
            ++rank;
            sh = DwShare(x, rank, a.n_mt, a.n_nt);
        }
        if (rank >= a.n_experts || r >= sh.tiles()) return;
        mt = sh.m_begin + r / sh.nsz;
        nt = sh.n_begin + r % sh.nsz;
    }
    const int e = a.by_load[rank];
    const int off = a.offsets[e], cnt = a.counts[e];
    const int m0 = mt * kTileM, n0 = nt * BN;
    const int Mdim = a.Mdim, Ndim = a.Ndim;

    // The buffers cover exactly the expert's rows, so the last step reads zeros past the expert's end.
    const i32x4 bufA = GATHER == kGatherA ? make_buffer(a.A, a.gathered_bytes)
                                          : make_buffer(a.A + (size_t)off * Mdim, (uint32_t)cnt * (uint32_t)Mdim * 2u);
    const i32x4 bufB0 = GATHER == kGatherB ? make_buffer(a.B0, a.gathered_bytes)
                                           : make_buffer(a.B0 + (size_t)off * Ndim, (uint32_t)cnt * (uint32_t)Ndim * 2u);
    const i32x4 bufB1 = NB == 2 ? make_buffer(a.B1 + (size_t)off * Ndim, (uint32_t)cnt * (uint32_t)Ndim * 2u) : bufB0;
    int a_col[2], b_col[BTile::kPasses];   // the piece a lane copies depends on the K-row, hence on the pass
    uint32_t a_voff[2], b_voff[BTile::kPasses];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        a_col[p] = m0 + ATile::src_piece(tid, p) * 8;
        a_voff[p] = a_col[p] < Mdim ? ((uint32_t)ATile::krow_of(tid, p) * (uint32_t)Mdim + a_col[p]) * 2u : kOutOfRange;
    }
#pragma unroll
    for (int p = 0; p < BTile::kPasses; ++p) {
        b_col[p] = n0 + BTile::src_piece(tid, p) * 8;
        b_voff[p] = b_col[p] < Ndim ? ((uint32_t)BTile::krow_of(tid, p) * (uint32_t)Ndim + b_col[p]) * 2u : kOutOfRange;
    }

    // token ids of the expert's rows, for the gathered operand
    const i32x4 bufTok = make_buffer(GATHER != kGatherNone ? a.row_token + off : nullptr, (uint32_t)cnt * 4u);
    const uint32_t id_ring = smem_addr + kIdRingAt + __builtin_amdgcn_readfirstlane((uint32_t)wave * 128u);
    auto issue_ids = [&](int step) {  // rows 32*step .. 32*step+31 -> this wave's ring slot step % 8
        if (lane < 32) async_copy4(bufTok, (uint32_t)lane * 4u, (uint32_t)step * 128u, id_ring + (uint32_t)(step & 7) * 512u);
    };
    auto token_of = [&](int step, int krow) {
        return *(const int32_t*)(smem + kIdRingAt + wave * 128 + (step & 7) * 512 + krow * 4);
    };

    // The ids a thread needs for the copies of one step (one per pass of the gathered operand) are read from the
    // ring at the start of the step that issues those copies, together with the step's fragment reads, so the
    // copies in the middle of the MFMA stream find them in registers.
    constexpr int kGatherPasses = GATHER == kGatherA ? 2 : (GATHER == kGatherB ? BTile::kPasses : 1);
    int32_t tok[kGatherPasses] = {};
    int next_issue = 2;   // the step whose copies the next compute() issues (0 and 1 belong to the prologue)
    auto load_ids = [&](int step) {
#pragma unroll
        for (int p = 0; p < kGatherPasses; ++p)
            tok[p] = token_of(step, GATHER == kGatherA ? ATile::krow_of(tid, p) : BTile::krow_of(tid, p));
    };
    auto issue_a = [&](int, int) {};
    auto issue_b = [&](int step, auto slot_c) {  // per-step copies: the A tile (2), the B tile(s) (4), and the ids
        constexpr int slot = decltype(slot_c)::value;
        if constexpr (GATHER != kGatherNone) {
            if (step < 2) load_ids(step);   // prologue; later steps were read ahead by compute()
        }
        const uint32_t k0 = (uint32_t)step * 32u;
        const uint32_t a_dst = smem_addr + slot * kMcSmallBytes + wave_base;
        const uint32_t b_dst = smem_addr + kBRegion + slot * kBTileBytes + wave_base;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            if constexpr (GATHER == kGatherA) {
                const uint32_t row = (uint32_t)tok[p] * (uint32_t)Mdim;
                async_copy16(bufA, a_col[p] < Mdim ? (row + a_col[p]) * 2u : kOutOfRange, 0u, a_dst + ATile::pass_offset(p));
            } else {
                async_copy16(bufA, a_voff[p], k0 * (uint32_t)Mdim * 2u, a_dst + ATile::pass_offset(p));
            }
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int p = 0; p < BTile::kPasses; ++p) {
                if constexpr (GATHER == kGatherB) {
                    const uint32_t row = (uint32_t)tok[p] * (uint32_t)Ndim;
                    async_copy16(bufB0, b_col[p] < Ndim ? (row + b_col[p]) * 2u : kOutOfRange, 0u, b_dst + BTile::pass_offset(p));
                } else {
                    async_copy16(nb ? bufB1 : bufB0, b_voff[p], k0 * (uint32_t)Ndim * 2u,
                                 b_dst + nb * kBHalf + BTile::pass_offset(p));
                }
            }
        if constexpr (GATHER != kGatherNone) issue_ids(step + 4);
    };
    if constexpr (GATHER != kGatherNone) {
#pragma unroll
        for (int s0 = 0; s0 < 4; ++s0) issue_ids(s0);
        wait_async_copies<0>();
    }

    Acc32 acc[NB][4][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < 4; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn) clear(acc[nb][fm][fn]);

    const uint32_t a_lane = ATile::lane_base(lane);
    const uint32_t b_lane = BTile::lane_base(lane) ^ BTile::column_bits(wave * (BN / 4));   // this wave's columns
    auto step_body = [&](const char* At, const char* Bt, auto issue) {
        Frag32 af[4], bf[2];
        // the 12 fragment addresses are derived from these two in every step (an XOR each) instead of being
        // held in registers over the whole loop
        uint32_t ab = a_lane, bb = b_lane;
        asm volatile("" : "+v"(ab), "+v"(bb));
#pragma unroll
        for (int g = 0; g < 2; ++g) bf[g] = BTile::read_frag(Bt + (g / FN) * kBHalf, bb, (g % FN) * 32);
#pragma unroll
        for (int fm = 0; fm < 4; ++fm) af[fm] = ATile::read_frag(At, ab, fm * 32);
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) {
                mfma32(bf[g], af[fm], acc[g / FN][fm][g % FN]);
                if (g == 0 && fm == 1) issue();
            }
    };
    auto compute = [&](auto slot_c, auto, int, auto issue) {
        constexpr int slot = decltype(slot_c)::value;
        if constexpr (GATHER != kGatherNone) load_ids(next_issue++);
        step_body(smem + slot * kMcSmallBytes, smem + kBRegion + slot * kBTileBytes, issue);
    };
    auto compute_rt = [&](int slot, int, int, auto issue) {
        if constexpr (GATHER != kGatherNone) load_ids(next_issue++);
        step_body(smem + slot * kMcSmallBytes, smem + kBRegion + slot * kBTileBytes, issue);
    };
    step_pipeline<false, kStepCopies>((cnt + 31) / 32, issue_a, issue_b, compute, compute_rt);
    if constexpr (GATHER != kGatherNone) wait_async_copies<0>();  // id copies of steps that do not exist

    const int rows_valid = min(kTileM, Mdim - m0);
    const int cols_valid = min(BN, Ndim - n0);
    const size_t tile_at = (size_t)e * Mdim * Ndim + (size_t)m0 * Ndim + n0;
    auto col_of = [&](int fn) { return wave * (BN / 4) + fn * 32; };
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        write_tile<BN, FN>(smem, tid, (nb ? a.C1 : a.C0) + tile_at, (size_t)Ndim, rows_valid, cols_valid, col_of,
                           [&](int fm, int fn, int q) { return pack_acc(acc[nb][fm][fn], q); });
}

}  // namespace grouter
