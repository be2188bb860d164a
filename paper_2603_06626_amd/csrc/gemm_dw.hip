// Weight-gradient grouped GEMMs: dW2_e = (gate * H)_e^T dY_e, and dW1_e = x_e^T dG_e, dW3_e = x_e^T dU_e, where
// x_e and dY_e are the expert's rows of the token-ordered x and dY, read through the plan's row map.
#include "gemm_kernels.hpp"

namespace grouter {

static DwArgs base_args(const PlanView& P) {
    DwArgs a{};
    a.plan = P.dims();
    a.by_load = P.by_load;
    a.offsets = P.offsets;
    a.counts = P.counts;
    return a;
}

// 8 XCDs x (largest per-XCD share): the share pattern repeats every 4 experts
static unsigned dw_grid(int E, int n_mt, int n_nt) {
    int worst = 0;
    for (int x = 0; x < 8; ++x) {
        int per_quad = 0;
        for (int tq = 0; tq < 4; ++tq) per_quad += DwShare(x, tq, n_mt, n_nt).tiles();
        worst = per_quad > worst ? per_quad : worst;
    }
    return 8u * (unsigned)(((E + 3) / 4) * worst);
}

// H here is the saved gate-weighted H, so the upstream gradient enters unscaled, straight from dY [T][d].
hipError_t launch_dw2(const PlanView& P, int d, int f, const bf16_t* H, const bf16_t* dY, bf16_t* dW2, hipStream_t s) {
    DwArgs a = base_args(P);
    a.A = H; a.B0 = dY; a.C0 = dW2;
    a.Mdim = f; a.Ndim = d; a.n_mt = (f + kTileM - 1) / kTileM; a.n_nt = (d + 255) / 256;
    a.n_experts = P.E;
    a.row_token = P.row_token; a.gathered_bytes = (uint32_t)((uint64_t)P.T * (uint64_t)d * 2u);
    hipLaunchKernelGGL((k_dw_gemm<1, kGatherB>), dim3(dw_grid(P.E, a.n_mt, a.n_nt)), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_dw13(const PlanView& P, int d, int f, const bf16_t* x, const bf16_t* dG, const bf16_t* dU,
                       bf16_t* dW1, bf16_t* dW3, hipStream_t s) {
    DwArgs a = base_args(P);
    a.A = x; a.B0 = dG; a.B1 = dU; a.C0 = dW1; a.C1 = dW3;
    a.Mdim = d; a.Ndim = f; a.n_mt = (d + kTileM - 1) / kTileM; a.n_nt = (f + 127) / 128;
    a.n_experts = P.E;
    a.row_token = P.row_token; a.gathered_bytes = (uint32_t)((uint64_t)P.T * (uint64_t)d * 2u);
    hipLaunchKernelGGL((k_dw_gemm<2, kGatherA>), dim3(dw_grid(P.E, a.n_mt, a.n_nt)), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace grouter
