// Forward grouped GEMMs: G,U = x_rows W1_e, x_rows W3_e with the fused gate-weighted SiLU*up epilogue (the rows of
// x read through the plan's row map), and O = H W2_e.
#include "gemm_kernels.hpp"

namespace grouter {

static RowsArgs base_args(const PlanView& P) {
    RowsArgs a{};
    a.tiles = P.tiles_small;
    a.max_tiles = P.max_tiles_small;
    a.plan = P.dims();
    a.col_group = 3;  // measured best of 0 (plain order), 1, 2, 3 on the forward GEMMs
    return a;
}

static unsigned rows_grid(const PlanView& P, int n_ntiles) { return (unsigned)P.max_tiles_small * (unsigned)n_ntiles; }

hipError_t launch_gateup(const PlanView& P, int d, int f, const bf16_t* x, const float* row_gate, const bf16_t* W1,
                         const bf16_t* W3, bf16_t* dSdG, bf16_t* dSdU, bf16_t* H, hipStream_t s) {
    RowsArgs a = base_args(P);
    a.A0 = x; a.B0 = W1; a.B1 = W3; a.C0 = dSdG; a.C1 = dSdU; a.C2 = H;
    a.K = d; a.Ncols = f; a.n_ntiles = (f + 127) / 128;
    a.row_token = P.row_token; a.a_total_bytes = (uint32_t)((uint64_t)P.T * (uint64_t)d * 2u);
    a.row_gate = row_gate;
    if (dSdG && dSdU)
        hipLaunchKernelGGL((k_fwd_gemm<kGateUp, true, false>), dim3(rows_grid(P, a.n_ntiles)), dim3(kThreads), 0, s, a);
    else  // forward only: nothing is kept for backward
        hipLaunchKernelGGL((k_fwd_gemm<kGateUp, true, true>), dim3(rows_grid(P, a.n_ntiles)), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_down(const PlanView& P, int d, int f, const bf16_t* H, const bf16_t* W2, bf16_t* O, hipStream_t s) {
    RowsArgs a = base_args(P);
    a.A0 = H; a.B0 = W2; a.C0 = O;
    a.K = f; a.Ncols = d; a.n_ntiles = (d + 255) / 256;
    hipLaunchKernelGGL(k_fwd_gemm<kDown>, dim3(rows_grid(P, a.n_ntiles)), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace grouter
