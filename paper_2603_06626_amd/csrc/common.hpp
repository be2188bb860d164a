// Shared host/device definitions of the grouter library: plan workspace layout, launch prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace grouter {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

constexpr int kMaxExperts = 1024;
constexpr int kPlanChunk = 512;   // routed slots handled by one wave in the plan kernels
constexpr int kTileRowsSmall = 128;  // row-tile heights for which the plan keeps a tile list

static inline __host__ __device__ size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Device layout of a routing plan.  Offsets are in bytes from plan_ws; every section is 256-byte aligned.
struct PlanLayout {
    int64_t T;
    int k, E;
    int64_t N;
    int n_chunks;
    int max_tiles_small;    // upper bound on row tiles: N/rows + E
    size_t off_header;      // int32[64]: [0]=status flags, [1]=#row tiles, [2]=N, [3]=k, [4]=E the plan was built for
    size_t off_chunk_bad;   // int32[n_chunks]: chunk holds an id outside [0,E)
    size_t off_counts;      // int32[E]
    size_t off_offsets;     // int32[E+1]
    size_t off_by_load;     // int32[E] expert ids, heaviest first (ties: lower id first)
    size_t off_row_to_src;  // int32[N]
    size_t off_src_to_row;  // int32[N]
    size_t off_row_token;   // int32[N + 128] = row_to_src / k: the token whose row sits at each expert-sorted position
                            // (the last 128 are padding: a row tile's ids are fetched without a bounds check)
    size_t off_row_gate;    // fp32[N]: gate weight of the slot behind each row, once grouter_plan_set_gates has run
    size_t off_chunk_hist;  // int32[E][n_chunks]; after the scan: exclusive base of each chunk inside its expert
    size_t off_tiles_small; // int32[max_tiles_small][8]: expert, the expert's first row, row count, first tile, tile count, 3 unused
    size_t total;
};

static inline __host__ PlanLayout make_plan_layout(int64_t T, int k, int E) {
    PlanLayout L{};
    L.T = T; L.k = k; L.E = E; L.N = T * (int64_t)k;
    L.n_chunks = (int)((L.N + kPlanChunk - 1) / kPlanChunk);
    L.max_tiles_small = (int)(L.N / kTileRowsSmall) + E;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.off_header = take(256);
    L.off_chunk_bad = take(sizeof(int32_t) * (size_t)L.n_chunks);
    L.off_counts = take(sizeof(int32_t) * (size_t)E);
    L.off_offsets = take(sizeof(int32_t) * (size_t)(E + 1));
    L.off_by_load = take(sizeof(int32_t) * (size_t)E);
    L.off_row_to_src = take(sizeof(int32_t) * (size_t)L.N);
    L.off_src_to_row = take(sizeof(int32_t) * (size_t)L.N);
    L.off_row_token = take(sizeof(int32_t) * (size_t)(L.N + kTileRowsSmall));
    L.off_row_gate = take(sizeof(float) * (size_t)L.N);
    L.off_chunk_hist = take(sizeof(int32_t) * (size_t)L.n_chunks * (size_t)E);
    L.off_tiles_small = take(sizeof(int32_t) * 8 * (size_t)L.max_tiles_small);
    L.total = o;
    return L;
}

// What a kernel compares against the plan header before it trusts anything else in the workspace: a plan
// built for other dimensions has differently placed sections, and the kernels then leave at once.
struct PlanDims {
    const int32_t* header;
    int N, k, E;
    __device__ __forceinline__ bool match() const { return row_tiles() >= 0; }
    // the plan's number of row tiles, or -1 if the plan was built for other dimensions; one 32-byte load
    __device__ __forceinline__ int row_tiles() const {
        typedef int32_t i32x8 __attribute__((ext_vector_type(8)));
        const i32x8 h = *(const i32x8*)header;
        return ((h[2] == N) & (h[3] == k) & (h[4] == E)) ? h[1] : -1;
    }
};

// Device-side view of a plan handed to kernels.
struct PlanView {
    const int32_t* header;
    const int32_t* counts;
    const int32_t* offsets;
    const int32_t* by_load;
    const int32_t* row_to_src;
    const int32_t* src_to_row;
    const int32_t* row_token;
    const float* row_gate;
    const int32_t* tiles_small;  int max_tiles_small;
    int64_t T; int k, E; int64_t N;
    __host__ PlanDims dims() const { return PlanDims{header, (int)N, k, E}; }
};

static inline __host__ PlanView make_plan_view(const void* ws, const PlanLayout& L) {
    const char* b = (const char*)ws;
    PlanView v{};
    v.header = (const int32_t*)(b + L.off_header);
    v.counts = (const int32_t*)(b + L.off_counts);
    v.offsets = (const int32_t*)(b + L.off_offsets);
    v.by_load = (const int32_t*)(b + L.off_by_load);
    v.row_to_src = (const int32_t*)(b + L.off_row_to_src);
    v.src_to_row = (const int32_t*)(b + L.off_src_to_row);
    v.row_token = (const int32_t*)(b + L.off_row_token);
    v.row_gate = (const float*)(b + L.off_row_gate);
    v.tiles_small = (const int32_t*)(b + L.off_tiles_small); v.max_tiles_small = L.max_tiles_small;
    v.T = L.T; v.k = L.k; v.E = L.E; v.N = L.N;
    return v;
}

// ---- launchers (each defined in the .hip file that holds its kernels) -------------------------------
hipError_t launch_plan_build(const void* idx, int idx_dtype, const PlanLayout& L, void* plan_ws, hipStream_t s);
// routing statistics (stats.hip)
hipError_t launch_sample_stats(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                               double* entropy, int64_t* loads, double* maxvio, const uint64_t* expert_nodes, int n_nodes,
                               int32_t* comm, int32_t* best_node, hipStream_t s);
hipError_t launch_affinity(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                           double* entropy, int64_t* loads, double* maxvio, hipStream_t s);
hipError_t launch_placement(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, const uint64_t* expert_nodes,
                            int n_nodes, int32_t* comm, int32_t* best_node, hipStream_t s);
hipError_t launch_coactivation(const void* idx, int idx_dtype, int64_t T, int k, int E, int64_t* P, hipStream_t s);
hipError_t launch_fold_groups(const int64_t* P, int E_S, int E_T, int32_t* group_of, hipStream_t s);
hipError_t launch_fold_weights(const float* W, const int32_t* group_of, int d, int E_S, int E_T, float* out, hipStream_t s);
hipError_t launch_mfma_probe(int mode, int iters, int workgroups, float* out, hipStream_t s);
hipError_t launch_row_gates(const PlanView& P, const bf16_t* gate_w, float* row_gate, hipStream_t s);
hipError_t launch_permute(const PlanView& P, int d, const bf16_t* in, const bf16_t* gate_w, bf16_t* out, hipStream_t s);
hipError_t launch_combine(const PlanView& P, int d, const bf16_t* in, const bf16_t* gate_w, bf16_t* out, hipStream_t s);

// Grouped GEMM phases.  Activation matrices are [N][d] or [N][f] in expert-sorted row order.  dSdG and dSdU are
// the partial derivatives of S = silu(G) * U by G and by U, which the forward pass keeps for backward instead of G, U.
hipError_t launch_gateup(const PlanView& P, int d, int f, const bf16_t* x, const float* row_gate, const bf16_t* W1,
                         const bf16_t* W3, bf16_t* dSdG, bf16_t* dSdU, bf16_t* H, hipStream_t s);
hipError_t launch_down(const PlanView& P, int d, int f, const bf16_t* H, const bf16_t* W2, bf16_t* O, hipStream_t s);
hipError_t launch_dh(const PlanView& P, int d, int f, const bf16_t* dY, const float* row_gate, const bf16_t* W2,
                     const bf16_t* dSdG, const bf16_t* dSdU, bf16_t* dG, bf16_t* dU, hipStream_t s);
hipError_t launch_dxp(const PlanView& P, int d, int f, const bf16_t* dG, const bf16_t* dU, const bf16_t* W1,
                      const bf16_t* W3, bf16_t* dXp, hipStream_t s);
hipError_t launch_dw2(const PlanView& P, int d, int f, const bf16_t* H, const bf16_t* dY, bf16_t* dW2, hipStream_t s);
hipError_t launch_dw13(const PlanView& P, int d, int f, const bf16_t* x, const bf16_t* dG, const bf16_t* dU,
                       bf16_t* dW1, bf16_t* dW3, hipStream_t s);

}  // namespace grouter
