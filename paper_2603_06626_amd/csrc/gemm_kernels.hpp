// The two grouped-GEMM kernels.  See gemm.hpp for tile layouts and the K-loop pipeline.
#pragma once
#include "gemm.hpp"

namespace grouter {

// One stage of MFMA work for a wave that owns 128 rows x (2 fragments of 32 columns): every fragment of both
// K halves is requested up front (LDS returns them in order, so the first MFMAs start as soon as the first
// half has landed and the second half arrives underneath them); the next-but-one step's six copies are
// dripped in between the four MFMA groups.  read_a(kk, fm) / read_b(kk, g) fetch fragments, acc_of(g, fm)
// names the accumulator, issue(IntC<j>) enqueues copy j.
template <class ReadA, class ReadB, class AccOf, class Issue>
__device__ __forceinline__ void compute_stage(bool drip, ReadA read_a, ReadB read_b, AccOf acc_of, Issue issue) {
    bf16x8 af[2][4], bf[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int fm = 0; fm < 4; ++fm) af[kk][fm] = read_a(kk, fm);
#pragma unroll
        for (int g = 0; g < 2; ++g) bf[kk][g] = read_b(kk, g);
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int g = 0; g < 2; ++g) {
#pragma unroll
            for (int fm = 0; fm < 4; ++fm) acc_of(g, fm) = mfma(bf[kk][g], af[kk][fm], acc_of(g, fm));
            if (drip) {
                if (kk == 0 && g == 0) { issue(IntC<0>{}); issue(IntC<1>{}); }
                if (kk == 0 && g == 1) { issue(IntC<2>{}); issue(IntC<3>{}); }
                if (kk == 1 && g == 0) issue(IntC<4>{});
                if (kk == 1 && g == 1) issue(IntC<5>{});
            }
        }
}

// Accumulators -> LDS -> whole-row stores for one 128 x BN output tile.  `packed(fm, fn, q)` returns the four
// bf16 (two packed words) of accumulator group (fm, fn, q).
template <int BN, class Packed>
__device__ __forceinline__ void write_tile(char* smem, int tid, bf16_t* dst, size_t ld, int rows_valid, int cols_valid,
                                           Packed packed) {
    constexpr int FN = BN / 128;
    constexpr int PITCH = (BN == 256) ? kOutPitch256 : kOutPitch128;
    const int lane = tid & 63, wave = tid >> 6;
    __syncthreads();  // earlier LDS readers (K loop, previous output) are done
#pragma unroll
    for (int fm = 0; fm < 4; ++fm) {
        const int m = fm * 32 + (lane & 31);
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = wave * (BN / 4) + fn * 32 + frag_col4(lane, q);
                *(u32x2*)(smem + m * PITCH + n * 2) = packed(fm, fn, q);
            }
        __builtin_amdgcn_sched_barrier(0);  // keep a fused epilogue's loads from piling up across fragments
    }
    __syncthreads();
    stage_flush<BN, PITCH>(smem, tid, dst, ld, rows_valid, cols_valid);
}

__device__ __forceinline__ u32x2 pack_acc(const f32x16& c, int q) {
    return u32x2{pack_bf16_rne(c[q * 4], c[q * 4 + 1]), pack_bf16_rne(c[q * 4 + 2], c[q * 4 + 3])};
}

// ===================================================================================================
// Row GEMMs: C[rows of expert e][Ncols] = A[rows][K] * B_e, rows taken from the plan's 128-row tile list.
//   kGateUp  B = W1_e, W3_e stored [K=d][Ncols=f] (MC); two accumulator sets; epilogue G, U, H = silu(G)*U
//   kDown    B = W2_e stored [K=f][Ncols=d] (MC); epilogue O
//   kDh      B = W2_e read as [Ncols=f][K=d] (KC, i.e. dO * W2^T); epilogue dG, dU from saved G, U
//   kDxp     two K phases: dG * W1_e^T then dU * W3_e^T, W read as [Ncols=d][K=f] (KC); epilogue dXp
enum RowsMode { kGateUp = 0, kDown = 1, kDh = 2, kDxp = 3 };

struct RowsArgs {
    const int32_t* tiles;        // [3][max_tiles]: expert, first row, valid rows (tile height 128)
    int max_tiles;
    const int32_t* n_tiles_ptr;  // number of row tiles actually present
    const bf16_t* A0; const bf16_t* A1;   // [Nrows][K]
    const bf16_t* B0; const bf16_t* B1;   // [E] slabs of K*Ncols elements
    bf16_t* C0; bf16_t* C1; bf16_t* C2;   // [Nrows][Ncols]
    const bf16_t* E0; const bf16_t* E1;   // epilogue inputs [Nrows][Ncols]
    int K, Ncols, n_ntiles;
};

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_rows_gemm(const RowsArgs a) {
    constexpr bool kBKc = (MODE == kDh || MODE == kDxp);
    constexpr int NB = (MODE == kGateUp) ? 2 : 1;
    constexpr int BN = (NB == 2) ? 128 : 256;  // columns per B operand
    constexpr int FN = BN / 128;               // 32-column fragments per wave and B operand
    constexpr int NPH = (MODE == kDxp) ? 2 : 1;
    constexpr int kBHalf = kBTileBytes / 2;    // second B operand of the two-operand mode
    using ATile = KcTile<128>;
    using BKc = KcTile<256>;
    using BMc = McTile<BN>;
    constexpr int kBPasses = kBKc ? BKc::kPasses : BMc::kPasses;
    static_assert(ATile::kPasses == 2 && (kBKc ? kBPasses : NB * kBPasses) == 4, "six copies per thread and step");

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wave_base = __builtin_amdgcn_readfirstlane((uint32_t)wave * 1024u);
    const int n_real = (*a.n_tiles_ptr) * a.n_ntiles;
    if ((int)blockIdx.x >= n_real) return;
    const int L = xcd_remap(blockIdx.x, n_real);
    const int mt = L / a.n_ntiles, nt = L - mt * a.n_ntiles;
    const int e = a.tiles[mt];
    const int row0 = a.tiles[a.max_tiles + mt];
    const int rows = a.tiles[2 * a.max_tiles + mt];
    const int col0 = nt * BN;
    const int K = a.K, Ncols = a.Ncols;
    const int nk = (K + kBK - 1) / kBK;
    const bool k_tail = (K % kBK) != 0;  // only K-contiguous tiles need care: their last step stops mid-row

    // ---- buffers and per-lane offsets, fixed over the K loop.  The A buffer covers exactly this tile's valid
    // rows and the B buffer exactly this expert's slab, so everything outside them reads as zero.
    const size_t a_tile_off = (size_t)row0 * K;
    const i32x4 bufA0 = make_buffer(a.A0 + a_tile_off, (uint32_t)rows * (uint32_t)K * 2u);
    const i32x4 bufA1 = NPH == 2 ? make_buffer(a.A1 + a_tile_off, (uint32_t)rows * (uint32_t)K * 2u) : bufA0;
    const size_t slab = (size_t)e * K * Ncols;
    const uint32_t slab_bytes = (uint32_t)K * (uint32_t)Ncols * 2u;
    const i32x4 bufB0 = make_buffer(a.B0 + slab, slab_bytes);
    const i32x4 bufB1 = (NB == 2 || NPH == 2) ? make_buffer(a.B1 + slab, slab_bytes) : bufB0;

    const int a_piece = ATile::src_piece(tid);
    uint32_t a_voff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) a_voff[p] = ((uint32_t)ATile::row_of(tid, p) * (uint32_t)K + a_piece * 8) * 2u;
    const int b_piece = kBKc ? BKc::src_piece(tid) : BMc::src_piece(tid);
    uint32_t b_voff[kBPasses];
    if (kBKc) {
#pragma unroll
        for (int p = 0; p < kBPasses; ++p) {
            const int n = col0 + BKc::row_of(tid, p);
            b_voff[p] = n < Ncols ? ((uint32_t)n * (uint32_t)K + b_piece * 8) * 2u : kOutOfRange;
        }
    } else {
        const int col = col0 + b_piece * 8;
#pragma unroll
        for (int p = 0; p < kBPasses; ++p)
            b_voff[p] = col < Ncols ? ((uint32_t)BMc::krow_of(tid, p) * (uint32_t)Ncols + col) * 2u : kOutOfRange;
    }

    // copy j (0..5) of K step `it`: j = 0,1 the A passes; j = 2..5 the B passes (of both operands when NB = 2)
    const uint32_t smem_addr = __builtin_amdgcn_readfirstlane(lds_addr(smem));
    auto issue_one = [&](int it, auto stage_c, auto jc) {
        constexpr int j = decltype(jc)::value;
        const uint32_t a_dst = smem_addr + decltype(stage_c)::value * kATileBytes + wave_base;
        const uint32_t b_dst = smem_addr + kBRegion + decltype(stage_c)::value * kBTileBytes + wave_base;
        const int ph = (NPH == 2 && it >= nk) ? 1 : 0;
        const int k0 = (it - ph * nk) * kBK;
        const bool last = k_tail && (k0 + kBK > K);
        if constexpr (j < 2) {
            uint32_t v = a_voff[j];
            if (last) v = (k0 + a_piece * 8 < K) ? v : kOutOfRange;
            async_copy16(ph ? bufA1 : bufA0, v, (uint32_t)k0 * 2u, a_dst + ATile::pass_offset(j));
        } else if constexpr (kBKc) {
            constexpr int p = j - 2;
            uint32_t v = b_voff[p];
            if (last) v = (k0 + b_piece * 8 < K) ? v : kOutOfRange;
            async_copy16(ph ? bufB1 : bufB0, v, (uint32_t)k0 * 2u, b_dst + BKc::pass_offset(p));
        } else {
            constexpr int nb = (j - 2) / kBPasses;
            constexpr int p = (j - 2) % kBPasses;
            async_copy16(nb ? bufB1 : bufB0, b_voff[p], (uint32_t)k0 * (uint32_t)Ncols * 2u,
                         b_dst + nb * kBHalf + BMc::pass_offset(p));
        }
    };
    auto issue_all = [&](int it, auto stage) {
        issue_one(it, stage, IntC<0>{}); issue_one(it, stage, IntC<1>{}); issue_one(it, stage, IntC<2>{});
        issue_one(it, stage, IntC<3>{}); issue_one(it, stage, IntC<4>{}); issue_one(it, stage, IntC<5>{});
    };

    f32x16 acc[NB][4][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < 4; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][fm][fn][v] = 0.f;

    auto compute = [&](auto stage_c, auto drip_c, int next_it) {
        constexpr int stage = decltype(stage_c)::value;
        const char* At = smem + stage * kATileBytes;
        const char* Bt = smem + kBRegion + stage * kBTileBytes;
        constexpr IntC<(stage + 2) % kStages> next_stage{};
        compute_stage(decltype(drip_c)::value != 0,
            [&](int kk, int fm) { return ATile::read_frag(At, lane, fm * 32, kk); },
            [&](int kk, int g) {
                const int nb = g / FN, fn = g % FN;
                if (kBKc) return BKc::read_frag(Bt, lane, wave * 64 + fn * 32, kk);
                return BMc::read_frag(Bt + nb * kBHalf, lane, wave * (BN / 4) + fn * 32, kk);
            },
            [&](int g, int fm) -> f32x16& { return acc[g / FN][fm][g % FN]; },
            [&](auto jc) { issue_one(next_it, next_stage, jc); });
    };

    // the same stage with run-time addresses (used for the last steps of the K loop only)
    auto issue_rt = [&](int it, int stage, auto jc) {
        if (stage == 0) issue_one(it, IntC<0>{}, jc);
        else if (stage == 1) issue_one(it, IntC<1>{}, jc);
        else issue_one(it, IntC<2>{}, jc);
    };
    auto compute_tail = [&](int stage, int next_it) {
        const char* At = smem + stage * kATileBytes;
        const char* Bt = smem + kBRegion + stage * kBTileBytes;
        const int next_stage = stage >= 1 ? stage - 1 : stage + 2;
        compute_stage(next_it >= 0,
            [&](int kk, int fm) { return ATile::read_frag(At, lane, fm * 32, kk); },
            [&](int kk, int g) {
                const int nb = g / FN, fn = g % FN;
                if (kBKc) return BKc::read_frag(Bt, lane, wave * 64 + fn * 32, kk);
                return BMc::read_frag(Bt + nb * kBHalf, lane, wave * (BN / 4) + fn * 32, kk);
            },
            [&](int g, int fm) -> f32x16& { return acc[g / FN][fm][g % FN]; },
            [&](auto jc) { issue_rt(next_it, next_stage, jc); });
    };

    k_pipeline<6>(nk * NPH, smem, issue_all, compute, compute_tail);

    // ---- epilogue: accumulators -> (fused elementwise) -> LDS -> whole-row 16-byte stores
    const int cols_valid = min(BN, Ncols - col0);
    const size_t tile_at = (size_t)row0 * Ncols + col0;
    if constexpr (MODE == kGateUp) {
        write_tile<BN>(smem, tid, a.C0 + tile_at, (size_t)Ncols, rows, cols_valid,
                       [&](int fm, int fn, int q) { return pack_acc(acc[0][fm][fn], q); });
        write_tile<BN>(smem, tid, a.C1 + tile_at, (size_t)Ncols, rows, cols_valid,
                       [&](int fm, int fn, int q) { return pack_acc(acc[1][fm][fn], q); });
        write_tile<BN>(smem, tid, a.C2 + tile_at, (size_t)Ncols, rows, cols_valid, [&](int fm, int fn, int q) {
            float h[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float g = acc[0][fm][fn][q * 4 + r];
                h[r] = g / (1.f + __expf(-g)) * acc[1][fm][fn][q * 4 + r];
            }
            return u32x2{pack_bf16_rne(h[0], h[1]), pack_bf16_rne(h[2], h[3])};
        });
    } else if constexpr (MODE == kDh) {
        // dG = dH * U * s * (1 + G (1 - s)),  dU = dH * G * s,  s = sigmoid(G).  G and U are read as 8-byte row
        // pieces, once per output (the second read hits in cache), which keeps the accumulators untouched.
#pragma unroll
        for (int out = 0; out < 2; ++out)
            write_tile<BN>(smem, tid, (out ? a.C1 : a.C0) + tile_at, (size_t)Ncols, rows, cols_valid,
                           [&](int fm, int fn, int q) {
                               const int m = fm * 32 + (lane & 31);
                               const int n = wave * (BN / 4) + fn * 32 + frag_col4(lane, q);
                               u32x2 gp = u32x2{0u, 0u}, up = u32x2{0u, 0u};
                               if (m < rows && n < cols_valid) {
                                   const size_t at = tile_at + (size_t)m * Ncols + n;
                                   gp = *(const u32x2*)(a.E0 + at);
                                   up = *(const u32x2*)(a.E1 + at);
                               }
                               const float g[4] = {bf16_lo(gp.x), bf16_hi(gp.x), bf16_lo(gp.y), bf16_hi(gp.y)};
                               const float u[4] = {bf16_lo(up.x), bf16_hi(up.x), bf16_lo(up.y), bf16_hi(up.y)};
                               float c[4];
#pragma unroll
                               for (int r = 0; r < 4; ++r) {
                                   const float sg = 1.f / (1.f + __expf(-g[r]));
                                   const float dh = acc[0][fm][fn][q * 4 + r];
                                   c[r] = out == 0 ? dh * u[r] * sg * (1.f + g[r] * (1.f - sg)) : dh * g[r] * sg;
                               }
                               return u32x2{pack_bf16_rne(c[0], c[1]), pack_bf16_rne(c[2], c[3])};
                           });
    } else {
        write_tile<BN>(smem, tid, a.C0 + tile_at, (size_t)Ncols, rows, cols_valid,
                       [&](int fm, int fn, int q) { return pack_acc(acc[0][fm][fn], q); });
    }
}

// ===================================================================================================
// Weight-gradient GEMMs: C_e[Mdim][Ndim] = A_e^T * B_e, reduction over the expert's rows.
//   A [Nrows][Mdim], B0/B1 [Nrows][Ndim] in expert-sorted row order; C0/C1 [E][Mdim][Ndim].
//   NB = 1: one B (dW2 = H^T dO).  NB = 2: two B sharing A (dW1 = Xp^T dG, dW3 = Xp^T dU).
// Experts are walked heaviest first so the long reductions start early; an expert without rows gets zeros.
struct DwArgs {
    const int32_t* by_load;
    const int32_t* offsets;
    const int32_t* counts;
    const bf16_t* A;
    const bf16_t* B0; const bf16_t* B1;
    bf16_t* C0; bf16_t* C1;
    int Mdim, Ndim, n_mt, n_nt;
};

template <int NB>
__global__ __launch_bounds__(kThreads, 2) void k_dw_gemm(const DwArgs a) {
    constexpr int BN = (NB == 2) ? 128 : 256;
    constexpr int FN = BN / 128;
    constexpr int kBHalf = kBTileBytes / 2;
    using ATile = McTile<128>;
    using BTile = McTile<BN>;
    static_assert(ATile::kPasses == 2 && NB * BTile::kPasses == 4, "six copies per thread and step");

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wave_base = __builtin_amdgcn_readfirstlane((uint32_t)wave * 1024u);
    const int per_e = a.n_mt * a.n_nt;
    const int rank = blockIdx.x / per_e;
    const int rem = blockIdx.x - rank * per_e;
    const int mt = rem / a.n_nt, nt = rem - mt * a.n_nt;
    const int e = a.by_load[rank];
    const int off = a.offsets[e], cnt = a.counts[e];
    const int m0 = mt * kTileM, n0 = nt * BN;
    const int Mdim = a.Mdim, Ndim = a.Ndim;

    // The buffers cover exactly the expert's rows, so the last K step reads zeros past the expert's end.
    const i32x4 bufA = make_buffer(a.A + (size_t)off * Mdim, (uint32_t)cnt * (uint32_t)Mdim * 2u);
    const i32x4 bufB0 = make_buffer(a.B0 + (size_t)off * Ndim, (uint32_t)cnt * (uint32_t)Ndim * 2u);
    const i32x4 bufB1 = NB == 2 ? make_buffer(a.B1 + (size_t)off * Ndim, (uint32_t)cnt * (uint32_t)Ndim * 2u) : bufB0;
    const int a_col = m0 + ATile::src_piece(tid) * 8;
    const int b_col = n0 + BTile::src_piece(tid) * 8;
    uint32_t a_voff[2], b_voff[BTile::kPasses];
#pragma unroll
    for (int p = 0; p < 2; ++p)
        a_voff[p] = a_col < Mdim ? ((uint32_t)ATile::krow_of(tid, p) * (uint32_t)Mdim + a_col) * 2u : kOutOfRange;
#pragma unroll
    for (int p = 0; p < BTile::kPasses; ++p)
        b_voff[p] = b_col < Ndim ? ((uint32_t)BTile::krow_of(tid, p) * (uint32_t)Ndim + b_col) * 2u : kOutOfRange;

    const uint32_t smem_addr = __builtin_amdgcn_readfirstlane(lds_addr(smem));
    auto issue_one = [&](int it, auto stage_c, auto jc) {
        constexpr int j = decltype(jc)::value;
        const uint32_t a_dst = smem_addr + decltype(stage_c)::value * kATileBytes + wave_base;
        const uint32_t b_dst = smem_addr + kBRegion + decltype(stage_c)::value * kBTileBytes + wave_base;
        const uint32_t k0 = (uint32_t)it * kBK;
        if constexpr (j < 2) {
            async_copy16(bufA, a_voff[j], k0 * (uint32_t)Mdim * 2u, a_dst + ATile::pass_offset(j));
        } else {
            constexpr int nb = (j - 2) / BTile::kPasses;
            constexpr int p = (j - 2) % BTile::kPasses;
            async_copy16(nb ? bufB1 : bufB0, b_voff[p], k0 * (uint32_t)Ndim * 2u,
                         b_dst + nb * kBHalf + BTile::pass_offset(p));
        }
    };
    auto issue_all = [&](int it, auto stage) {
        issue_one(it, stage, IntC<0>{}); issue_one(it, stage, IntC<1>{}); issue_one(it, stage, IntC<2>{});
        issue_one(it, stage, IntC<3>{}); issue_one(it, stage, IntC<4>{}); issue_one(it, stage, IntC<5>{});
    };

    f32x16 acc[NB][4][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < 4; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][fm][fn][v] = 0.f;

    auto compute = [&](auto stage_c, auto drip_c, int next_it) {
        constexpr int stage = decltype(stage_c)::value;
        const char* At = smem + stage * kATileBytes;
        const char* Bt = smem + kBRegion + stage * kBTileBytes;
        constexpr IntC<(stage + 2) % kStages> next_stage{};
        compute_stage(decltype(drip_c)::value != 0,
            [&](int kk, int fm) { return ATile::read_frag(At, lane, fm * 32, kk); },
            [&](int kk, int g) {
                const int nb = g / FN, fn = g % FN;
                return BTile::read_frag(Bt + nb * kBHalf, lane, wave * (BN / 4) + fn * 32, kk);
            },
            [&](int g, int fm) -> f32x16& { return acc[g / FN][fm][g % FN]; },
            [&](auto jc) { issue_one(next_it, next_stage, jc); });
    };

    // the same stage with run-time addresses (used for the last steps of the K loop only)
    auto issue_rt = [&](int it, int stage, auto jc) {
        if (stage == 0) issue_one(it, IntC<0>{}, jc);
        else if (stage == 1) issue_one(it, IntC<1>{}, jc);
        else issue_one(it, IntC<2>{}, jc);
    };
    auto compute_tail = [&](int stage, int next_it) {
        const char* At = smem + stage * kATileBytes;
        const char* Bt = smem + kBRegion + stage * kBTileBytes;
        const int next_stage = stage >= 1 ? stage - 1 : stage + 2;
        compute_stage(next_it >= 0,
            [&](int kk, int fm) { return ATile::read_frag(At, lane, fm * 32, kk); },
            [&](int kk, int g) {
                const int nb = g / FN, fn = g % FN;
                return BTile::read_frag(Bt + nb * kBHalf, lane, wave * (BN / 4) + fn * 32, kk);
            },
            [&](int g, int fm) -> f32x16& { return acc[g / FN][fm][g % FN]; },
            [&](auto jc) { issue_rt(next_it, next_stage, jc); });
    };

    k_pipeline<6>((cnt + kBK - 1) / kBK, smem, issue_all, compute, compute_tail);

    const int rows_valid = min(kTileM, Mdim - m0);
    const int cols_valid = min(BN, Ndim - n0);
    const size_t tile_at = (size_t)e * Mdim * Ndim + (size_t)m0 * Ndim + n0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
        write_tile<BN>(smem, tid, (nb ? a.C1 : a.C0) + tile_at, (size_t)Ndim, rows_valid, cols_valid,
                       [&](int fm, int fn, int q) { return pack_acc(acc[nb][fm][fn], q); });
}

}  // namespace grouter
