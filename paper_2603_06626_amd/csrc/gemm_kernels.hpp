// The two grouped-GEMM kernels.  See gemm.hpp for tile layouts and the K-loop pipeline.
#pragma once
#include "gemm.hpp"

namespace grouter {

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
    const char* zero;            // >= 16 zero bytes
    const bf16_t* A0; const bf16_t* A1;   // [Nrows][K]
    const bf16_t* B0; const bf16_t* B1;   // [E] slabs of K*Ncols elements
    bf16_t* C0; bf16_t* C1; bf16_t* C2;   // [Nrows][Ncols]
    const bf16_t* E0; const bf16_t* E1;   // epilogue inputs [Nrows][Ncols]
    int K, Ncols, n_ntiles;
    int64_t Nrows;
};

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_rows_gemm(const RowsArgs a) {
    constexpr bool kBKc = (MODE == kDh || MODE == kDxp);
    constexpr int NB = (MODE == kGateUp) ? 2 : 1;
    constexpr int BN = (NB == 2) ? 128 : 256;  // columns per B operand
    constexpr int FN = BN / 128;               // 32-column fragments per wave and B operand
    constexpr int FM = 4;
    constexpr int NPH = (MODE == kDxp) ? 2 : 1;
    constexpr int kBHalf = kBTileBytes / 2;    // second B operand of the two-operand mode
    using ATile = KcTile<128>;
    using BKc = KcTile<256>;
    using BMc = McTile<BN>;
    constexpr int kBPasses = kBKc ? BKc::kPasses : BMc::kPasses;
    constexpr int kLoads = ATile::kPasses + (kBKc ? kBPasses : NB * kBPasses);
    constexpr int PITCH = (BN == 256) ? kOutPitch256 : kOutPitch128;

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    // ---- per-thread source offsets (bytes), fixed over the K loop
    const int a_piece = ATile::src_piece(tid);
    size_t a_off[ATile::kPasses];
#pragma unroll
    for (int p = 0; p < ATile::kPasses; ++p) {
        const int64_t grow = min((int64_t)row0 + ATile::row_of(tid, p), a.Nrows - 1);
        a_off[p] = ((size_t)grow * K + a_piece * 8) * 2;
    }
    const size_t slab = (size_t)e * K * Ncols * 2;
    const int b_piece = kBKc ? BKc::src_piece(tid) : BMc::src_piece(tid);
    size_t b_off[kBPasses];
    bool b_colvalid = true;
    if (kBKc) {
#pragma unroll
        for (int p = 0; p < kBPasses; ++p) {
            const int n = min(col0 + BKc::row_of(tid, p), Ncols - 1);
            b_off[p] = slab + ((size_t)n * K + b_piece * 8) * 2;
        }
    } else {
        const int col = col0 + b_piece * 8;
        b_colvalid = col < Ncols;
#pragma unroll
        for (int p = 0; p < kBPasses; ++p) b_off[p] = slab + ((size_t)BMc::krow_of(tid, p) * Ncols + col) * 2;
    }

    // copy number j (0 <= j < kLoads) of K step `it`: first the A passes, then the B passes
    auto issue_one = [&](int it, uint32_t stage, auto jc) {
        constexpr int j = decltype(jc)::value;
        const int ph = (NPH == 2 && it >= nk) ? 1 : 0;
        const int k0 = (it - ph * nk) * kBK;
        if constexpr (j < ATile::kPasses) {
            const char* Ab = (const char*)(ph ? a.A1 : a.A0);
            const bool a_kvalid = k0 + a_piece * 8 < K;
            const char* src = a_kvalid ? Ab + a_off[j] + (size_t)k0 * 2 : a.zero;
            async_copy16(src, ATile::wave_dst(stage, tid, j));
        } else if constexpr (kBKc) {
            constexpr int p = j - ATile::kPasses;
            const char* Bb = (const char*)(ph ? a.B1 : a.B0);
            const bool b_kvalid = k0 + b_piece * 8 < K;
            const char* src = b_kvalid ? Bb + b_off[p] + (size_t)k0 * 2 : a.zero;
            async_copy16(src, BKc::wave_dst(stage + kATileBytes, tid, p));
        } else {
            constexpr int nb = (j - ATile::kPasses) / kBPasses;
            constexpr int p = (j - ATile::kPasses) % kBPasses;
            const char* Bb = (const char*)(nb ? a.B1 : a.B0);
            const bool v = b_colvalid && (k0 + BMc::krow_of(tid, p) < K);
            const char* src = v ? Bb + b_off[p] + (size_t)k0 * Ncols * 2 : a.zero;
            async_copy16(src, BMc::wave_dst(stage + kATileBytes + nb * kBHalf, tid, p));
        }
    };
    auto issue_all = [&](int it, uint32_t stage) {
        issue_one(it, stage, IntC<0>{});
        issue_one(it, stage, IntC<1>{});
        issue_one(it, stage, IntC<2>{});
        issue_one(it, stage, IntC<3>{});
        issue_one(it, stage, IntC<4>{});
        issue_one(it, stage, IntC<5>{});
    };
    static_assert(kLoads == 6, "the drip schedule below places exactly 6 copies");
#ifdef GROUTER_REG_STAGE
    auto copy_src = [&](int it, auto jc) -> const char* {
        constexpr int j = decltype(jc)::value;
        const int ph = (NPH == 2 && it >= nk) ? 1 : 0;
        const int k0 = (it - ph * nk) * kBK;
        if constexpr (j < ATile::kPasses) {
            const char* Ab = (const char*)(ph ? a.A1 : a.A0);
            return (k0 + a_piece * 8 < K) ? Ab + a_off[j] + (size_t)k0 * 2 : a.zero;
        } else if constexpr (kBKc) {
            constexpr int p = j - ATile::kPasses;
            const char* Bb = (const char*)(ph ? a.B1 : a.B0);
            return (k0 + b_piece * 8 < K) ? Bb + b_off[p] + (size_t)k0 * 2 : a.zero;
        } else {
            constexpr int nb = (j - ATile::kPasses) / kBPasses;
            constexpr int p = (j - ATile::kPasses) % kBPasses;
            const char* Bb = (const char*)(nb ? a.B1 : a.B0);
            const bool v = b_colvalid && (k0 + BMc::krow_of(tid, p) < K);
            return v ? Bb + b_off[p] + (size_t)k0 * Ncols * 2 : a.zero;
        }
    };
    auto copy_dst = [&](char* stage, auto jc) -> char* {   // this lane's 16-byte LDS slot of copy j
        constexpr int j = decltype(jc)::value;
        if constexpr (j < ATile::kPasses) return stage + (size_t)(j * 256 + tid) * 16;
        else if constexpr (kBKc) return stage + kATileBytes + (size_t)((j - ATile::kPasses) * 256 + tid) * 16;
        else {
            constexpr int nb = (j - ATile::kPasses) / kBPasses;
            constexpr int p = (j - ATile::kPasses) % kBPasses;
            return stage + kATileBytes + nb * kBHalf + (size_t)(p * 256 + tid) * 16;
        }
    };
    auto load_all = [&](int it, StagedRegs& r) {
        r.v[0] = *(const u32x4*)copy_src(it, IntC<0>{}); r.v[1] = *(const u32x4*)copy_src(it, IntC<1>{});
        r.v[2] = *(const u32x4*)copy_src(it, IntC<2>{}); r.v[3] = *(const u32x4*)copy_src(it, IntC<3>{});
        r.v[4] = *(const u32x4*)copy_src(it, IntC<4>{}); r.v[5] = *(const u32x4*)copy_src(it, IntC<5>{});
    };
    auto store_all = [&](char* stage, const StagedRegs& r) {
        *(u32x4*)copy_dst(stage, IntC<0>{}) = r.v[0]; *(u32x4*)copy_dst(stage, IntC<1>{}) = r.v[1];
        *(u32x4*)copy_dst(stage, IntC<2>{}) = r.v[2]; *(u32x4*)copy_dst(stage, IntC<3>{}) = r.v[3];
        *(u32x4*)copy_dst(stage, IntC<4>{}) = r.v[4]; *(u32x4*)copy_dst(stage, IntC<5>{}) = r.v[5];
    };
#endif

    f32x16 acc[NB][FM][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][fm][fn][v] = 0.f;

    // One stage: 2 K sub-steps x 2 B fragments x 4 A fragments = 16 MFMAs, with the next-but-one step's six
    // copies dripped in after MFMA 2, 4, 6, 8, 12 and 16.
    // One stage: every fragment of both K halves is requested up front (LDS returns them in order, so the
    // first MFMAs start as soon as the first half has landed and the second half arrives underneath them);
    // the next-but-one step's six copies are dripped in between the four MFMA groups.
    auto compute = [&](const char* At, int next_it, uint32_t next_stage) {
        const char* Bt = At + kATileBytes;
        const bool drip = next_it >= 0;
        bf16x8 af[2][FM], bf[2][2];
#ifdef GROUTER_EXP_NO_LDSREAD
        At = smem; Bt = smem + kATileBytes;   // loop-invariant addresses: the reads are hoisted out of the K loop
#endif
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) af[kk][fm] = ATile::read_frag(At, lane, fm * 32, kk);
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int nb = g / FN, fn = g % FN;
                if (kBKc)
                    bf[kk][g] = BKc::read_frag(Bt, lane, wave * 64 + fn * 32, kk);
                else
                    bf[kk][g] = BMc::read_frag(Bt + nb * kBHalf, lane, wave * (BN / 4) + fn * 32, kk);
            }
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int nb = g / FN, fn = g % FN;
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) acc[nb][fm][fn] = mfma(bf[kk][g], af[kk][fm], acc[nb][fm][fn]);
                if (drip) {
                    if (kk == 0 && g == 0) { issue_one(next_it, next_stage, IntC<0>{}); issue_one(next_it, next_stage, IntC<1>{}); }
                    if (kk == 0 && g == 1) { issue_one(next_it, next_stage, IntC<2>{}); issue_one(next_it, next_stage, IntC<3>{}); }
                    if (kk == 1 && g == 0) issue_one(next_it, next_stage, IntC<4>{});
                    if (kk == 1 && g == 1) issue_one(next_it, next_stage, IntC<5>{});
                }
            }
    };

#ifdef GROUTER_REG_STAGE
    k_pipeline_regs(nk * NPH, smem, load_all, store_all, compute);
#else
    k_pipeline<kLoads>(nk * NPH, smem, issue_all, compute);
#endif

    // ---- epilogue: accumulators -> (fused elementwise) -> LDS -> whole-row 16-byte stores
    const int cols_valid = min(BN, Ncols - col0);
    const size_t tile_at = (size_t)row0 * Ncols + col0;
    constexpr int kOutputs = (MODE == kGateUp) ? 3 : (MODE == kDh ? 2 : 1);
#pragma unroll
    for (int out = 0; out < kOutputs; ++out) {
        __syncthreads();  // the K loop's (or the previous output's) LDS reads are done
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            const int m = fm * 32 + (lane & 31);
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = wave * (BN / 4) + fn * 32 + frag_col4(lane, q);
                    float c[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) c[r] = acc[0][fm][fn][q * 4 + r];
                    if (MODE == kGateUp) {
                        if (out == 1) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) c[r] = acc[NB - 1][fm][fn][q * 4 + r];
                        } else if (out == 2) {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                c[r] = c[r] / (1.f + __expf(-c[r])) * acc[NB - 1][fm][fn][q * 4 + r];
                        }
                    } else if (MODE == kDh) {
                        // dG = dH * U * s * (1 + G (1 - s)),  dU = dH * G * s,  s = sigmoid(G)
                        float g[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f};
                        if (m < rows && n < cols_valid) {
                            const size_t at = tile_at + (size_t)m * Ncols + n;
                            const u32x2 gp = *(const u32x2*)(a.E0 + at);
                            const u32x2 up = *(const u32x2*)(a.E1 + at);
                            g[0] = bf16_lo(gp.x); g[1] = bf16_hi(gp.x); g[2] = bf16_lo(gp.y); g[3] = bf16_hi(gp.y);
                            u[0] = bf16_lo(up.x); u[1] = bf16_hi(up.x); u[2] = bf16_lo(up.y); u[3] = bf16_hi(up.y);
                        }
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float s = 1.f / (1.f + __expf(-g[r]));
                            c[r] = out == 0 ? c[r] * u[r] * s * (1.f + g[r] * (1.f - s)) : c[r] * g[r] * s;
                        }
                    }
                    stage_put4<PITCH>(smem, m, n, c[0], c[1], c[2], c[3]);
                }
        }
        __syncthreads();
        bf16_t* dst = (out == 0 ? a.C0 : (out == 1 ? a.C1 : a.C2)) + tile_at;
        stage_flush<BN, PITCH>(smem, tid, dst, (size_t)Ncols, rows, cols_valid);
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
    const char* zero;
    const bf16_t* A;
    const bf16_t* B0; const bf16_t* B1;
    bf16_t* C0; bf16_t* C1;
    int Mdim, Ndim, n_mt, n_nt;
};

template <int NB>
__global__ __launch_bounds__(kThreads, 2) void k_dw_gemm(const DwArgs a) {
    constexpr int BN = (NB == 2) ? 128 : 256;
    constexpr int FN = BN / 128;
    constexpr int FM = 4;
    constexpr int kBHalf = kBTileBytes / 2;
    using ATile = McTile<128>;
    using BTile = McTile<BN>;
    constexpr int kLoads = ATile::kPasses + NB * BTile::kPasses;
    constexpr int PITCH = (BN == 256) ? kOutPitch256 : kOutPitch128;

    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per_e = a.n_mt * a.n_nt;
    const int rank = blockIdx.x / per_e;
    const int rem = blockIdx.x - rank * per_e;
    const int mt = rem / a.n_nt, nt = rem - mt * a.n_nt;
    const int e = a.by_load[rank];
    const int off = a.offsets[e], cnt = a.counts[e];
    const int m0 = mt * kTileM, n0 = nt * BN;
    const int Mdim = a.Mdim, Ndim = a.Ndim;

    const int a_col = m0 + ATile::src_piece(tid) * 8;
    const bool a_valid = a_col < Mdim;
    const int b_col = n0 + BTile::src_piece(tid) * 8;
    const bool b_valid = b_col < Ndim;
    const size_t a_base = ((size_t)off * Mdim + a_col) * 2;
    const size_t b_base = ((size_t)off * Ndim + b_col) * 2;

    // copy number j (0 <= j < kLoads) of K step `it`: first the A passes, then the B passes
    auto issue_one = [&](int it, uint32_t stage, auto jc) {
        constexpr int j = decltype(jc)::value;
        const int k0 = it * kBK;
        if constexpr (j < ATile::kPasses) {
            const int kr = k0 + ATile::krow_of(tid, j);
            const char* src = (a_valid && kr < cnt) ? (const char*)a.A + a_base + (size_t)kr * Mdim * 2 : a.zero;
            async_copy16(src, ATile::wave_dst(stage, tid, j));
        } else {
            constexpr int nb = (j - ATile::kPasses) / BTile::kPasses;
            constexpr int p = (j - ATile::kPasses) % BTile::kPasses;
            const char* Bb = (const char*)(nb ? a.B1 : a.B0);
            const int kr = k0 + BTile::krow_of(tid, p);
            const char* src = (b_valid && kr < cnt) ? Bb + b_base + (size_t)kr * Ndim * 2 : a.zero;
            async_copy16(src, BTile::wave_dst(stage + kATileBytes + nb * kBHalf, tid, p));
        }
    };
    auto issue_all = [&](int it, uint32_t stage) {
        issue_one(it, stage, IntC<0>{});
        issue_one(it, stage, IntC<1>{});
        issue_one(it, stage, IntC<2>{});
        issue_one(it, stage, IntC<3>{});
        issue_one(it, stage, IntC<4>{});
        issue_one(it, stage, IntC<5>{});
    };
    static_assert(kLoads == 6, "the drip schedule below places exactly 6 copies");
#ifdef GROUTER_REG_STAGE
    auto copy_src = [&](int it, auto jc) -> const char* {
        constexpr int j = decltype(jc)::value;
        const int k0 = it * kBK;
        if constexpr (j < ATile::kPasses) {
            const int kr = k0 + ATile::krow_of(tid, j);
            return (a_valid && kr < cnt) ? (const char*)a.A + a_base + (size_t)kr * Mdim * 2 : a.zero;
        } else {
            constexpr int nb = (j - ATile::kPasses) / BTile::kPasses;
            constexpr int p = (j - ATile::kPasses) % BTile::kPasses;
            const char* Bb = (const char*)(nb ? a.B1 : a.B0);
            const int kr = k0 + BTile::krow_of(tid, p);
            return (b_valid && kr < cnt) ? Bb + b_base + (size_t)kr * Ndim * 2 : a.zero;
        }
    };
    auto copy_dst = [&](char* stage, auto jc) -> char* {
        constexpr int j = decltype(jc)::value;
        if constexpr (j < ATile::kPasses) return stage + (size_t)(j * 256 + tid) * 16;
        else {
            constexpr int nb = (j - ATile::kPasses) / BTile::kPasses;
            constexpr int p = (j - ATile::kPasses) % BTile::kPasses;
            return stage + kATileBytes + nb * kBHalf + (size_t)(p * 256 + tid) * 16;
        }
    };
    auto load_all = [&](int it, StagedRegs& r) {
        r.v[0] = *(const u32x4*)copy_src(it, IntC<0>{}); r.v[1] = *(const u32x4*)copy_src(it, IntC<1>{});
        r.v[2] = *(const u32x4*)copy_src(it, IntC<2>{}); r.v[3] = *(const u32x4*)copy_src(it, IntC<3>{});
        r.v[4] = *(const u32x4*)copy_src(it, IntC<4>{}); r.v[5] = *(const u32x4*)copy_src(it, IntC<5>{});
    };
    auto store_all = [&](char* stage, const StagedRegs& r) {
        *(u32x4*)copy_dst(stage, IntC<0>{}) = r.v[0]; *(u32x4*)copy_dst(stage, IntC<1>{}) = r.v[1];
        *(u32x4*)copy_dst(stage, IntC<2>{}) = r.v[2]; *(u32x4*)copy_dst(stage, IntC<3>{}) = r.v[3];
        *(u32x4*)copy_dst(stage, IntC<4>{}) = r.v[4]; *(u32x4*)copy_dst(stage, IntC<5>{}) = r.v[5];
    };
#endif

    f32x16 acc[NB][FM][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][fm][fn][v] = 0.f;

    auto compute = [&](const char* At, int next_it, uint32_t next_stage) {
        const char* Bt = At + kATileBytes;
        const bool drip = next_it >= 0;
        bf16x8 af[2][FM], bf[2][2];
#ifdef GROUTER_EXP_NO_LDSREAD
        At = smem; Bt = smem + kATileBytes;   // loop-invariant addresses: the reads are hoisted out of the K loop
#endif
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) af[kk][fm] = ATile::read_frag(At, lane, fm * 32, kk);
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int nb = g / FN, fn = g % FN;
                bf[kk][g] = BTile::read_frag(Bt + nb * kBHalf, lane, wave * (BN / 4) + fn * 32, kk);
            }
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int nb = g / FN, fn = g % FN;
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) acc[nb][fm][fn] = mfma(bf[kk][g], af[kk][fm], acc[nb][fm][fn]);
                if (drip) {
                    if (kk == 0 && g == 0) { issue_one(next_it, next_stage, IntC<0>{}); issue_one(next_it, next_stage, IntC<1>{}); }
                    if (kk == 0 && g == 1) { issue_one(next_it, next_stage, IntC<2>{}); issue_one(next_it, next_stage, IntC<3>{}); }
                    if (kk == 1 && g == 0) issue_one(next_it, next_stage, IntC<4>{});
                    if (kk == 1 && g == 1) issue_one(next_it, next_stage, IntC<5>{});
                }
            }
    };

#ifdef GROUTER_REG_STAGE
    k_pipeline_regs((cnt + kBK - 1) / kBK, smem, load_all, store_all, compute);
#else
    k_pipeline<kLoads>((cnt + kBK - 1) / kBK, smem, issue_all, compute);
#endif

    const int rows_valid = min(kTileM, Mdim - m0);
    const int cols_valid = min(BN, Ndim - n0);
    const size_t tile_at = (size_t)e * Mdim * Ndim + (size_t)m0 * Ndim + n0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        __syncthreads();
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& c = acc[nb][fm][fn];
                    stage_put4<PITCH>(smem, fm * 32 + (lane & 31), wave * (BN / 4) + fn * 32 + frag_col4(lane, q),
                                      c[q * 4], c[q * 4 + 1], c[q * 4 + 2], c[q * 4 + 3]);
                }
        __syncthreads();
        stage_flush<BN, PITCH>(smem, tid, (nb ? a.C1 : a.C0) + tile_at, (size_t)Ndim, rows_valid, cols_valid);
    }
}

}  // namespace grouter
