// The two grouped-GEMM kernel skeletons.  See gemm.hpp for tile layouts.
#pragma once
#include "gemm.hpp"

namespace grouter {

// ===================================================================================================
// Row GEMMs: C[rows of expert e][Ncols] = A[rows][K] * B_e, rows taken from the plan's row-tile list.
//   kGateUp  B = W1_e, W3_e stored [K=d][Ncols=f] (MC); two accumulator sets; epilogue G, U, H = silu(G)*U
//   kDown    B = W2_e stored [K=f][Ncols=d] (MC); epilogue O
//   kDh      B = W2_e read as [Ncols=f][K=d] (KC, i.e. dO * W2^T); epilogue dG, dU from saved G, U
//   kDxp     two K phases: dG * W1_e^T then dU * W3_e^T, W read as [Ncols=d][K=f] (KC); epilogue dXp
enum RowsMode { kGateUp = 0, kDown = 1, kDh = 2, kDxp = 3 };

struct RowsArgs {
    const int32_t* tiles;        // [3][max_tiles]: expert, first row, valid rows (tile height 256)
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
__global__ __launch_bounds__(kThreads) void k_rows_gemm(const RowsArgs a) {
    constexpr bool kBKc = (MODE == kDh || MODE == kDxp);
    constexpr int NB = (MODE == kGateUp) ? 2 : 1;
    constexpr int BN = (NB == 2) ? 128 : 256;  // columns per B operand
    constexpr int FN = BN / 128;               // 32-column fragments per wave and B operand
    constexpr int FM = 4;
    constexpr int NPH = (MODE == kDxp) ? 2 : 1;
    constexpr int kBTileBytes = 64 * BN * 2;
    using ATile = KcTile<256>;
    using BKc = KcTile<256>;
    using BMc = McTile<BN>;
    constexpr int kBPasses = kBKc ? BKc::kPasses : BMc::kPasses;

    __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];

    const uint32_t smem_addr = lds_addr(smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int n_real = (*a.n_tiles_ptr) * a.n_ntiles;
    if ((int)blockIdx.x >= n_real) return;
    const int L = xcd_remap(blockIdx.x, n_real);
    const int mt = L / a.n_ntiles, nt = L - mt * a.n_ntiles;
    const int e = a.tiles[mt];
    const int row0 = a.tiles[a.max_tiles + mt];
    const int rows = a.tiles[2 * a.max_tiles + mt];
    const int col0 = nt * BN;
    const int K = a.K, Ncols = a.Ncols;

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

    auto issue = [&](int it, uint32_t stage) {
        const int ph = (NPH == 2 && it >= (K + kBK - 1) / kBK) ? 1 : 0;
        const int k0 = (it - ph * ((K + kBK - 1) / kBK)) * kBK;
        const char* Ab = (const char*)(ph ? a.A1 : a.A0);
        const bool a_kvalid = k0 + a_piece * 8 < K;
#pragma unroll
        for (int p = 0; p < ATile::kPasses; ++p) {
            const char* src = a_kvalid ? Ab + a_off[p] + (size_t)k0 * 2 : a.zero;
            async_copy16(src, ATile::wave_dst(stage, tid, p));
        }
        if (kBKc) {
            const char* Bb = (const char*)(ph ? a.B1 : a.B0);
            const bool b_kvalid = k0 + b_piece * 8 < K;
#pragma unroll
            for (int p = 0; p < kBPasses; ++p) {
                const char* src = b_kvalid ? Bb + b_off[p] + (size_t)k0 * 2 : a.zero;
                async_copy16(src, BKc::wave_dst(stage + kATileBytes, tid, p));
            }
        } else {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const char* Bb = (const char*)(nb ? a.B1 : a.B0);
#pragma unroll
                for (int p = 0; p < kBPasses; ++p) {
                    const bool v = b_colvalid && (k0 + BMc::krow_of(tid, p) < K);
                    const char* src = v ? Bb + b_off[p] + (size_t)k0 * Ncols * 2 : a.zero;
                    async_copy16(src, BMc::wave_dst(stage + kATileBytes + nb * kBTileBytes, tid, p));
                }
            }
        }
    };

    f32x16 acc[NB][FM][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][fm][fn][v] = 0.f;

    const int total_it = ((K + kBK - 1) / kBK) * NPH;
    issue(0, smem_addr);
    for (int it = 0; it < total_it; ++it) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (it + 1 < total_it) issue(it + 1, smem_addr + ((it + 1) & 1) * kStageBytes);
        const char* At = smem + (it & 1) * kStageBytes;
        const char* Bt = At + kATileBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[FM];
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) af[fm] = ATile::read_frag(At, lane, wm * 128 + fm * 32, kk);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    bf16x8 bfr;
                    if (kBKc)
                        bfr = BKc::read_frag(Bt, lane, wn * 64 + fn * 32, kk);
                    else
                        bfr = BMc::read_frag(Bt + nb * kBTileBytes, lane, wn * (BN / 4) + fn * 32, kk);
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm) acc[nb][fm][fn] = mfma(bfr, af[fm], acc[nb][fm][fn]);
                }
        }
    }

    // ---- epilogue: 8-byte pieces of output rows
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        const int m = wm * 128 + fm * 32 + (lane & 31);
        if (m >= rows) continue;
        const size_t rowbase = (size_t)(row0 + m) * Ncols;
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = col0 + wn * (BN / 4) + fn * 32 + frag_col4(lane, q);
                if (col >= Ncols) continue;
                const size_t at = rowbase + col;
                float c0[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) c0[r] = acc[0][fm][fn][q * 4 + r];
                if (MODE == kGateUp) {
                    float h[4], u[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        u[r] = acc[NB - 1][fm][fn][q * 4 + r];
                        h[r] = c0[r] / (1.f + __expf(-c0[r])) * u[r];
                    }
                    *(u32x2*)(a.C0 + at) = u32x2{pack_bf16_rne(c0[0], c0[1]), pack_bf16_rne(c0[2], c0[3])};
                    *(u32x2*)(a.C1 + at) = u32x2{pack_bf16_rne(u[0], u[1]), pack_bf16_rne(u[2], u[3])};
                    *(u32x2*)(a.C2 + at) = u32x2{pack_bf16_rne(h[0], h[1]), pack_bf16_rne(h[2], h[3])};
                } else if (MODE == kDh) {
                    const u32x2 gp = *(const u32x2*)(a.E0 + at);
                    const u32x2 up = *(const u32x2*)(a.E1 + at);
                    const float g[4] = {bf16_lo(gp.x), bf16_hi(gp.x), bf16_lo(gp.y), bf16_hi(gp.y)};
                    const float u[4] = {bf16_lo(up.x), bf16_hi(up.x), bf16_lo(up.y), bf16_hi(up.y)};
                    float dg[4], du[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float s = 1.f / (1.f + __expf(-g[r]));
                        dg[r] = c0[r] * u[r] * s * (1.f + g[r] * (1.f - s));
                        du[r] = c0[r] * g[r] * s;
                    }
                    *(u32x2*)(a.C0 + at) = u32x2{pack_bf16_rne(dg[0], dg[1]), pack_bf16_rne(dg[2], dg[3])};
                    *(u32x2*)(a.C1 + at) = u32x2{pack_bf16_rne(du[0], du[1]), pack_bf16_rne(du[2], du[3])};
                } else {
                    *(u32x2*)(a.C0 + at) = u32x2{pack_bf16_rne(c0[0], c0[1]), pack_bf16_rne(c0[2], c0[3])};
                }
            }
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
__global__ __launch_bounds__(kThreads) void k_dw_gemm(const DwArgs a) {
    constexpr int BN = (NB == 2) ? 128 : 256;
    constexpr int FN = BN / 128;
    constexpr int FM = 4;
    constexpr int kBTileBytes = 64 * BN * 2;
    using ATile = McTile<256>;
    using BTile = McTile<BN>;

    __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];

    const uint32_t smem_addr = lds_addr(smem);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int per_e = a.n_mt * a.n_nt;
    const int rank = blockIdx.x / per_e;
    const int rem = blockIdx.x - rank * per_e;
    const int mt = rem / a.n_nt, nt = rem - mt * a.n_nt;
    const int e = a.by_load[rank];
    const int off = a.offsets[e], cnt = a.counts[e];
    const int m0 = mt * 256, n0 = nt * BN;
    const int Mdim = a.Mdim, Ndim = a.Ndim;

    const int a_col = m0 + ATile::src_piece(tid) * 8;
    const bool a_valid = a_col < Mdim;
    const int b_col = n0 + BTile::src_piece(tid) * 8;
    const bool b_valid = b_col < Ndim;
    const size_t a_base = ((size_t)off * Mdim + a_col) * 2;
    const size_t b_base = ((size_t)off * Ndim + b_col) * 2;

    auto issue = [&](int it, uint32_t stage) {
        const int k0 = it * kBK;
#pragma unroll
        for (int p = 0; p < ATile::kPasses; ++p) {
            const int kr = k0 + ATile::krow_of(tid, p);
            const char* src = (a_valid && kr < cnt) ? (const char*)a.A + a_base + (size_t)kr * Mdim * 2 : a.zero;
            async_copy16(src, ATile::wave_dst(stage, tid, p));
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const char* Bb = (const char*)(nb ? a.B1 : a.B0);
#pragma unroll
            for (int p = 0; p < BTile::kPasses; ++p) {
                const int kr = k0 + BTile::krow_of(tid, p);
                const char* src = (b_valid && kr < cnt) ? Bb + b_base + (size_t)kr * Ndim * 2 : a.zero;
                async_copy16(src, BTile::wave_dst(stage + kATileBytes + nb * kBTileBytes, tid, p));
            }
        }
    };

    f32x16 acc[NB][FM][FN];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < FN; ++fn)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][fm][fn][v] = 0.f;

    const int total_it = (cnt + kBK - 1) / kBK;
    if (total_it > 0) issue(0, smem_addr);
    for (int it = 0; it < total_it; ++it) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (it + 1 < total_it) issue(it + 1, smem_addr + ((it + 1) & 1) * kStageBytes);
        const char* At = smem + (it & 1) * kStageBytes;
        const char* Bt = At + kATileBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[FM];
#pragma unroll
            for (int fm = 0; fm < FM; ++fm) af[fm] = ATile::read_frag(At, lane, wm * 128 + fm * 32, kk);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) {
                    const bf16x8 bfr = BTile::read_frag(Bt + nb * kBTileBytes, lane, wn * (BN / 4) + fn * 32, kk);
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm) acc[nb][fm][fn] = mfma(bfr, af[fm], acc[nb][fm][fn]);
                }
        }
    }

    const size_t slab = (size_t)e * Mdim * Ndim;
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
        const int m = m0 + wm * 128 + fm * 32 + (lane & 31);
        if (m >= Mdim) continue;
#pragma unroll
        for (int fn = 0; fn < FN; ++fn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + wn * (BN / 4) + fn * 32 + frag_col4(lane, q);
                if (col >= Ndim) continue;
                const size_t at = slab + (size_t)m * Ndim + col;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    bf16_t* C = nb ? a.C1 : a.C0;
                    const f32x16& c = acc[nb][fm][fn];
                    *(u32x2*)(C + at) =
                        u32x2{pack_bf16_rne(c[q * 4], c[q * 4 + 1]), pack_bf16_rne(c[q * 4 + 2], c[q * 4 + 3])};
                }
            }
    }
}

}  // namespace grouter
