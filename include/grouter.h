/*
 * grouter.h - C ABI of the MI355X (gfx950) fixed-routing MoE expert layer.
 *
 * The layer is Sec. 2.1, Eq. 1 of the Grouter paper, y = sum_i r(x)_i f_i(x), evaluated under a routing
 * that was computed ahead of time and handed in (Sec. 3.3.1, "Decoupling Preemptive Routing": per token
 * the k active expert ids and their gate weights are cached - uint8 ids and bfloat16 scores in the
 * paper's storage format, App. "Efficiency Experiment Detail" - and passed to the MoE layers).
 * Because the router is frozen (App. A, the "ideal expert gradient"), backward produces gradients for
 * the expert weights and for the layer input only; the gate weights receive none.
 *
 * The paper leaves the expert f_i abstract.  Here it is a bias-free SwiGLU FFN
 *      f_e(x) = ( silu(x W1_e) * (x W3_e) ) W2_e ,   silu(g) = g / (1 + exp(-g)),
 * with W1 = gate projection, W3 = up projection, W2 = down projection.
 *
 * Conventions
 *   T tokens, d = model width, f = expert hidden width, E experts, k experts per token, N = T*k routed
 *   slots.  Flat slot index i = t*k + j.  "Row" p is a position in expert-sorted order.
 *   All float tensors are bfloat16 (IEEE bit patterns, 2 bytes), row-major, dense; accumulation is
 *   fp32; fp32 -> bf16 is round-to-nearest-even.  Weights are stored input-major: W1,W3 [E][d][f],
 *   W2 [E][f][d], so x W needs no transpose.
 *   Every pointer is a DEVICE pointer owned by the caller unless stated otherwise; the library never
 *   allocates or frees device memory.  `stream` is a hipStream_t passed as void* (NULL = default
 *   stream).  Calls only enqueue work and return; the single exception is grouter_plan_status.
 *   Outputs are overwritten in full, never accumulated into.
 *   Limits: 1 <= k <= E <= 1024 (E <= 256 for uint8 ids), T*k < 2^31, d % 8 == 0, f % 8 == 0,
 *   d*f*2 < 2^31 (one expert's weight slab) and T*k*max(d,f)*2 < 2^31 (an activation matrix in
 *   expert-sorted order): the kernels use 32-bit byte offsets inside those.  The size queries return
 *   0 and the compute calls GROUTER_ERR_INVALID_ARG beyond these limits.
 *
 *   Every call that takes plan_ws also takes the (T,k,E) the plan was built for.  The build records them
 *   in the plan; a kernel that finds other values there leaves at once, so a mismatched call writes nothing
 *   (and reads nothing outside the plan header) - its outputs are then simply not produced.
 *
 * Errors: every function returning int yields GROUTER_OK (0) or a negative code.  Argument checks run
 * on the host before anything is launched.
 */
#ifndef GROUTER_H
#define GROUTER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    GROUTER_OK = 0,
    GROUTER_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size, k > E, unsupported d/f/E */
    GROUTER_ERR_WORKSPACE_TOO_SMALL = -2,
    GROUTER_ERR_INDEX_OUT_OF_RANGE = -3, /* an expert id outside [0,E) was seen while building a plan */
    GROUTER_ERR_HIP = -4                 /* a HIP runtime call failed; see grouter_last_hip_error */
};

enum { GROUTER_IDX_INT32 = 0, GROUTER_IDX_UINT8 = 1 };

/* Human-readable name of an error code (static storage, host pointer). */
const char* grouter_strerror(int code);
/* hipError_t of the most recent failing HIP call made by this library on the calling thread. */
int grouter_last_hip_error(void);

/* ---- workspace sizes (host-only arithmetic; 0 is returned for invalid arguments) ------------------ */
/* bytes of device memory a routing plan for (T,k,E) occupies */
size_t grouter_plan_bytes(int64_t T, int k, int E);
/* bytes of the forward context: P,Q,H [N][f] (P, Q: the partial derivatives of silu(G)*U by G and by U), O[N][d]
 * and the per-row gate weights [N] fp32; it is what backward reads, so keep it alive and untouched between
 * grouter_moe_fwd and grouter_moe_bwd */
size_t grouter_ctx_bytes(int64_t T, int k, int d, int f);
/* bytes of scratch backward needs (dG,dU[N][f] and the per-row input gradient [N][d]); contents are dead
 * after the call */
size_t grouter_bwd_scratch_bytes(int64_t T, int k, int d, int f);

/* ---- routing plan: per-expert histogram, exclusive scan, stable scatter ---------------------------
 * Built once per routing and reused by every layer and by both passes (Sec. 3.1, "Shared Grouter":
 * one routing result guides all MoE layers).
 *   topk_idx   [T][k] expert ids, int32 or uint8 according to idx_dtype
 *   plan_ws    caller-allocated, 256-byte aligned, >= grouter_plan_bytes(T,k,E); the plan lives here
 * The plan is the stable counting sort of the N slots by expert id: rows of one expert are contiguous
 * and keep ascending slot order, which makes every index array unique.
 * An id outside [0,E) is recorded in the plan (see grouter_plan_status) and treated as expert 0 so
 * that no access leaves the workspace.
 */
int grouter_plan_build(const void* topk_idx, int idx_dtype, int64_t T, int k, int E, void* plan_ws,
                       size_t plan_ws_bytes, void* stream);

/* Attaches gate weights to a built plan (the paper caches ids and scores together, so they usually belong to
 * the routing as much as the ids do): the weight of the slot behind every expert-sorted row is laid out in the
 * plan once, and grouter_moe_fwd / _fwd_only / _bwd called with gate_w == NULL use it instead of laying the
 * weights of their own gate_w argument out on every call.  gate_w [T][k] bf16.  Call it after grouter_plan_build
 * on the same stream (or ordered after it); a rebuilt plan needs its gates set again.  Calling the layer with
 * gate_w == NULL on a plan whose gates were never set reads undefined weights.
 */
int grouter_plan_set_gates(void* plan_ws, int64_t T, int k, int E, const void* gate_w, void* stream);

/* Borrowed device views into plan_ws (host-only pointer arithmetic, no launch):
 *   counts[E], offsets[E+1] (exclusive scan, offsets[E] = N), row_to_src[N] (slot held by row p),
 *   src_to_row[N] (inverse permutation).  Any out-pointer may be NULL. */
int grouter_plan_views(const void* plan_ws, int64_t T, int k, int E, const int32_t** counts,
                       const int32_t** offsets, const int32_t** row_to_src, const int32_t** src_to_row);

/* Waits for `stream`, then returns GROUTER_ERR_INDEX_OUT_OF_RANGE if the build met a bad id. */
int grouter_plan_status(const void* plan_ws, void* stream);

/* ---- permute / dispatch and combine / un-permute, exposed on their own ----------------------------
 * grouter_permute:  out[p][:] = s_p * in[row_to_src[p] / k][:]   (the "token dispatch" gather)
 *   in [T][d], out [N][d]; gate_w NULL -> s_p = 1, else s_p = gate_w[row_to_src[p]] (Eq. 1's r_i), the
 *   product rounded once to bf16.  grouter_moe_fwd / _bwd do not call it: their GEMMs read the rows of x
 *   and dY in place; it is the pack step an expert-parallel dispatch would send from.
 * grouter_combine:  out[t][:] = sum_{j<k} s_{t,j} * in[src_to_row[t*k+j]][:]  in fp32, j ascending
 *   in [N][d], out [T][d]; gate_w [T][k] or NULL for weight 1 (what the layer itself uses for y and dX,
 *   because it folds the gate weights into H).
 */
int grouter_permute(const void* plan_ws, int64_t T, int k, int E, int d, const void* in, const void* gate_w,
                    void* out, void* stream);
int grouter_combine(const void* plan_ws, int64_t T, int k, int E, int d, const void* in, const void* gate_w,
                    void* out, void* stream);

/* ---- forward: y = sum_j gate_w[t][j] * f_{idx[t][j]}(x[t])   (Eq. 1) ------------------------------
 *   x [T][d], gate_w [T][k] (or NULL: the gates set with grouter_plan_set_gates), W1,W3 [E][d][f], W2 [E][f][d],
 *   y [T][d]
 *   ctx_ws     >= grouter_ctx_bytes(T,k,d,f), 256-byte aligned; receives, in expert-sorted row order, with
 *              G = x W1, U = x W3, s = sigmoid(G): Q = G s (= silu(G), the derivative of silu(G)*U by U),
 *              P = U s (1 + G (1 - s)) (its derivative by G) - all backward needs of G and U -,
 *              H = r * silu(G)*U (r = the row's gate weight: Eq. 1 is linear in each expert's output, so
 *              the weight is folded in here) and O = H W2, each rounded to bf16, plus the per-row gate
 *              weights as fp32 when the call brings gate_w.  The gate/up GEMM reads its rows
 *              straight from x through the plan's row map; y is then the plain sum of a token's k rows of O.
 */
int grouter_moe_fwd(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                    const void* gate_w, const void* W1, const void* W3, const void* W2, void* y, void* ctx_ws,
                    size_t ctx_ws_bytes, void* stream);

/* ---- forward when no backward follows (evaluation, inference): the same y as grouter_moe_fwd, bit for
 *      bit (Eq. 1 with the cached routing of Sec. 3.3.1), without the saved context: the gate/up GEMM reads
 *      its rows straight from x through the plan's row map and stores only H = r * silu(x W1) * (x W3), r the
 *      row's gate weight.
 *   ws >= grouter_fwd_only_bytes(T,k,d,f), 256-byte aligned; receives H [N][f], O [N][d] and the per-row gate
 *      weights [N] as fp32.
 */
size_t grouter_fwd_only_bytes(int64_t T, int k, int d, int f);
int grouter_moe_fwd_only(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                         const void* gate_w, const void* W1, const void* W3, const void* W2, void* y, void* ws,
                         size_t ws_bytes, void* stream);

/* ---- forward for callers that cannot allocate device memory and have no workspace at hand (code under
 *      HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): grouter_moe_fwd_only with
 *      its workspace (H, O, per-row gate weights) in a static device array of GROUTER_STATIC_WS_BYTES that the
 *      library holds on every GPU it runs on until the process ends.  Same arguments, same y bit for bit.
 *      Problems with grouter_fwd_only_bytes(T,k,d,f) > GROUTER_STATIC_WS_BYTES get
 *      GROUTER_ERR_WORKSPACE_TOO_SMALL.  The call allocates nothing (the first call on a device looks the
 *      array's address up once).  All calls on one GPU share that GPU's array: calls that may overlap in time
 *      on one GPU (different streams, different host threads) race and must be ordered by the caller.
 */
#define GROUTER_STATIC_WS_BYTES (64u << 20)
size_t grouter_static_ws_bytes(void);
int grouter_moe_fwd_only_static(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                                const void* gate_w, const void* W1, const void* W3, const void* W2, void* y,
                                void* stream);

/* ---- backward of L = <y, dY> with the routing fixed (App. A) --------------------------------------
 *   dY [T][d]; ctx_ws as left by grouter_moe_fwd for the same inputs (gate_w NULL or not, as it was there);
 *   dX [T][d], dW1,dW3 [E][d][f], dW2 [E][f][d] - all overwritten; an expert with no token gets zeros.
 *   scratch_ws >= grouter_bwd_scratch_bytes(T,k,d,f), 256-byte aligned; receives dG, dU [N][f] and the
 *              per-row input gradient [N][d].  dY and x are read in place through the plan's row map.
 */
int grouter_moe_bwd(const void* plan_ws, int64_t T, int k, int E, int d, int f, const void* x,
                    const void* gate_w, const void* W1, const void* W3, const void* W2, const void* dY,
                    const void* ctx_ws, size_t ctx_ws_bytes, void* dX, void* dW1, void* dW3, void* dW2,
                    void* scratch_ws, size_t scratch_bytes, void* stream);

/* ==== routing statistics from cached top-k ids (inputs of the offline optimisers) ==================
 * Common to the calls below: topk_idx holds k ids per token in the given dtype (GROUTER_IDX_*), 1 <= k <= 64,
 * 1 <= E <= 1024 (E <= 256 for uint8 ids and for grouter_coactivation).  Membership is an indicator per
 * token: an id repeated inside one token counts once; ids outside [0,E) are ignored.  All outputs are
 * overwritten.  Integer results do not depend on scheduling (integer atomics only).
 */

/* ---- routing affinity of S samples of L tokens each (Sec. 3.3.2, first equation) --------------------
 *   topk_idx [S][L][k]
 *   counts  [S][E] int32   tokens of sample s whose top-k set contains expert e (affinity = counts / L)
 *   entropy_bits [S] f64   Shannon entropy, base 2, of counts[s][:] normalised to sum 1 (the quantity the
 *                          expert-grouping filter of App. "Efficiency Experiment Detail" thresholds); 0 for
 *                          a sample without valid ids
 *   loads   [E] int64      column sums of counts (tokens given to each expert)
 *   maxvio  [1] f64        (max_e loads - mean loads) / mean loads   (App. "Maximal Violation")
 */
int grouter_affinity(const void* topk_idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                     double* entropy_bits, int64_t* loads, double* maxvio, void* stream);

/* ---- sample placement (App. "Efficiency Experiment Detail", algorithm "Optimize Sample-to-Node
 *      Assignment") ----------------------------------------------------------------------------------
 *   expert_nodes [E] uint64  bit n set <=> expert e is placed on node n (sets may overlap), n_nodes <= 64
 *   comm      [S][n_nodes] int32   tokens of sample s with at least one of their experts on node n
 *   best_node [S] int32            the first node attaining the maximum of comm[s][:]
 */
int grouter_sample_placement(const void* topk_idx, int idx_dtype, int64_t S, int L, int k, int E,
                             const uint64_t* expert_nodes, int n_nodes, int32_t* comm, int32_t* best_node,
                             void* stream);

/* ---- both of the above in one pass over the ids (every id is read once): the same outputs, bit for bit, as
 *      grouter_affinity followed by grouter_sample_placement on the same ids.
 */
int grouter_sample_stats(const void* topk_idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                         double* entropy_bits, int64_t* loads, double* maxvio, const uint64_t* expert_nodes, int n_nodes,
                         int32_t* comm, int32_t* best_node, void* stream);

/* ---- expert folding (Sec. 3.2.1) --------------------------------------------------------------------
 * grouter_coactivation: topk_idx [T][k]; P [E][E] int64, P[i][j] = tokens whose top-k set contains both
 *   i and j (the diagonal holds each expert's token count).  E <= 256.
 * grouter_fold_groups: greedy affinity grouping of E_S source experts into E_T <= E_S groups, filled one
 *   after the other; the first E_S mod E_T groups get floor(E_S/E_T)+1 members, the rest floor(E_S/E_T); a
 *   group starts with the lowest unassigned expert and then repeatedly takes the unassigned expert with the
 *   largest sum of P over the group's members (lowest number on ties).  group_of [E_S] int32.  E_S <= 1024.
 * grouter_fold_weights: out = W_s M with W_s [d][E_S] fp32, M[i][group_of[i]] = 1, out [d][E_T] fp32; each
 *   output sums its members in ascending expert order in fp32.  group_of entries outside [0,E_T) drop out.
 */
int grouter_coactivation(const void* topk_idx, int idx_dtype, int64_t T, int k, int E, int64_t* P, void* stream);
int grouter_fold_groups(const int64_t* P, int E_S, int E_T, int32_t* group_of, void* stream);
int grouter_fold_weights(const float* W_s, const int32_t* group_of, int d, int E_S, int E_T, float* out,
                         void* stream);

/* ---- per-kernel timing (HIP events on the caller's stream) ----------------------------------------
 * While enabled, every phase (one kernel, or the few kernels of the plan build) is bracketed by events on
 * the stream it is launched on; consecutive phases inside one call share the event between them.  grouter_timing_read waits for those events and accumulates elapsed milliseconds and
 * launch counts per phase; phases are indexed by the GROUTER_PH_* constants.  Host-side state shared by
 * all threads (guarded by a mutex).  Launches made while their stream is being captured into a graph are
 * not timed.  At most 4096 launches are kept between reads.
 */
enum {
    GROUTER_PH_PLAN = 0,      /* histogram + scan + scatter */
    GROUTER_PH_PERMUTE = 1,   /* grouter_permute without gate weights */
    GROUTER_PH_GATEUP = 2,    /* G,U GEMMs + SiLU*up */
    GROUTER_PH_DOWN = 3,      /* O = H W2 */
    GROUTER_PH_COMBINE = 4,   /* y */
    GROUTER_PH_DO = 5,        /* grouter_permute with gate weights */
    GROUTER_PH_DH = 6,        /* dH GEMM + dSwiGLU */
    GROUTER_PH_DW2 = 7,
    GROUTER_PH_DW13 = 8,
    GROUTER_PH_DXP = 9,
    GROUTER_PH_DXREDUCE = 10,
    GROUTER_PH_AFFINITY = 11,  /* affinity counts, entropy, loads, MaxVio */
    GROUTER_PH_PLACEMENT = 12,
    GROUTER_PH_COACT = 13,
    GROUTER_PH_FOLD = 14,      /* greedy grouping, folded weights */
    GROUTER_PH_SAMPLE_STATS = 15, /* grouter_sample_stats: affinity and placement in one pass */
    GROUTER_PH_COUNT = 16
};
int grouter_timing_enable(int on);
int grouter_timing_read(double* ms /*[GROUTER_PH_COUNT]*/, int64_t* launches /*[GROUTER_PH_COUNT]*/);
const char* grouter_phase_name(int phase);

/* ---- matrix-core ceiling probe (a measurement aid, not part of the layer) ----------------------------
 * Launches `workgroups` workgroups of 4 waves on pseudo-random operands; no global memory is read.  Per step
 * every wave does the matrix-core work of a 128 x 64 wave tile over 16 of K (8 * 32768 FLOP, the instruction mix
 * of the GEMM main loops).  iters (the number of steps) must be a multiple of 4.
 *   mode 0  8 independent v_mfma_f32_32x32x16_bf16 per step, operand fragments kept in registers
 *   mode 1  as mode 0, the 6 fragments of every step read again from LDS with 16-byte reads
 *   mode 2  16 independent v_mfma_f32_16x16x32_bf16 per step (what the kernels issue), fragments in registers
 *   mode 3  as mode 2, fragments read again from LDS
 *   mode 4  only the LDS fragment reads, as 16-byte reads, no MFMAs
 *   mode 5  only the LDS fragment reads, as pairs of transposing 8-byte reads in the address pattern of the
 *           kernels' N-contiguous tiles, no MFMAs
 *   mode 6  mode 2 with a 128 x 128 wave tile: 256 accumulator registers, hence one workgroup per CU and one
 *           wave per SIMD (launch one workgroup per CU)
 *   mode 7  mode 3 with that wave tile
 * FLOP per launch (modes 0-3, 6, 7) = workgroups * 4 * iters * 8 * 32768; bytes read from LDS per launch
 * (modes 4, 5) = workgroups * 4 * iters * 6 KiB.
 * `out` (device, fp32, at least workgroups * 256 elements; out_elems says how many it holds) only receives a
 * checksum per lane that keeps the results alive.  Timed by the caller (events on `stream`).
 * Errors: GROUTER_ERR_INVALID_ARG for a mode outside 0..7, iters <= 0 or not a multiple of 4, workgroups <= 0 or
 * above 2^20; GROUTER_ERR_WORKSPACE_TOO_SMALL when out_elems < workgroups * 256.
 */
int grouter_mfma_probe(int mode, int iters, int workgroups, float* out, size_t out_elems, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GROUTER_H */
