/*
 * CPU oracle for the fixed-routing MoE expert layer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker that the HIP library is compared against.  Only the test-suite, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it; the product path never does, and
 * it shares no code, header, table or helper with the HIP kernels.
 *
 * What it computes is the plain definition, token by token, with no permutation, no blocking and no
 * intermediate rounding:
 *
 *   forward  (Sec. 2.1, Eq. 1-2):  y_t = sum_j w[t][j] * f_{idx[t][j]}(x_t),
 *            where idx / w are the cached top-k expert ids and gate weights handed in from outside
 *            (Sec. 3.3.1: routing is precomputed and passed to the MoE layers), and each expert is a
 *            bias-free SwiGLU FFN  f_e(x) = (silu(x W1_e) * (x W3_e)) W2_e,  silu(g) = g / (1 + e^-g).
 *            The paper leaves f_e abstract; SwiGLU with W1 = gate, W3 = up, W2 = down is the reading
 *            used throughout this repository.
 *   backward (App. A, the expert-gradient expression with the router held fixed):  for L = <y, dY>,
 *            dW_e = dL/dy * sum_i r_i * grad f_i  restricted to expert e, and dX = dL/dx through the
 *            experts only.  No gradient is produced for the gate weights: the router is frozen and
 *            does not read x.
 *   plan:    per-expert counts, exclusive offsets and the stable counting-sort permutation of the
 *            T*k routed slots by expert id (ties kept in ascending slot order i = t*k + j).
 *
 * The float routines exist in two precisions generated from one body: *_f64 (used to verify the
 * oracle itself, and as the reference on small shapes) and *_f32 (the plain fp32 loop).
 * Work is spread over OpenMP threads by token (y, dX) and by disjoint output rows (dW); every
 * accumulation runs in one fixed order, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Stable counting sort of the N = T*k routed slots by expert id.
 *   idx[N]          expert id of flat slot i = t*k + j
 *   counts[E]       number of slots routed to each expert
 *   offsets[E+1]    exclusive prefix sum of counts; offsets[E] = N
 *   row_to_src[N]   slot index held by permuted row p (rows of one expert are contiguous, and inside
 *                   an expert they keep ascending slot order)
 *   src_to_row[N]   inverse permutation
 * Returns 0, or -1 when an id lies outside [0, E) (outputs are then unspecified).
 */
int oracle_plan(const int32_t* idx, int64_t N, int E, int32_t* counts, int32_t* offsets, int32_t* row_to_src,
                int32_t* src_to_row) {
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int64_t i = 0; i < N; ++i) {
        if (idx[i] < 0 || idx[i] >= E) return -1;
        counts[idx[i]] += 1;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
    for (int e = 0; e < E; ++e) cursor[e] = offsets[e];
    for (int64_t i = 0; i < N; ++i) {
        int32_t p = cursor[idx[i]]++;
        row_to_src[p] = (int32_t)i;
        src_to_row[i] = p;
    }
    free(cursor);
    return 0;
}

#define REAL double
#define EXP exp
#define NAME(base) base##_f64
#include "moe_body.inc"
#undef REAL
#undef EXP
#undef NAME

#define REAL float
#define EXP expf
#define NAME(base) base##_f32
#include "moe_body.inc"
#undef REAL
#undef EXP
#undef NAME
