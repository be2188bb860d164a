// Routing statistics computed from cached top-k expert ids (integer work, one pass over the ids each):
//   * per-sample routing affinity counts, their entropy, expert loads and the maximal violation
//     (Sec. 3.3.2 first equation; App. "Efficiency Experiment Detail", expert grouping; App. "Maximal Violation")
//   * sample placement: per (sample, node) the number of tokens that find an expert on the node, and the
//     best node (App. "Efficiency Experiment Detail", algorithm "Optimize Sample-to-Node Assignment")
//   * expert folding: co-activation matrix, greedy affinity grouping, folded score weights (Sec. 3.2.1)
//
// All three id-reading kernels share one scheme: a workgroup copies a run of tokens' ids into LDS with
// 16-byte coalesced loads (ids are 1 or 4 bytes, k per token, so a lane reading "its" token straight from
// global memory would touch k-byte fragments), then one lane handles one token out of LDS and counts with
// LDS atomics.  Membership is an indicator per token: an id repeated inside a token counts once, ids outside
// [0,E) are ignored.  Integer atomics commute, so every result is bit-reproducible.
#include "common.hpp"

namespace grouter {

namespace {

constexpr int kStatThreads = 256;
constexpr int kStageBytes = 16 * 1024;  // ids staged per pass
constexpr int kMaxStatK = 64;           // a token's validity mask is one 64-bit word

// Copy `bytes` bytes from src (any alignment) to the 16-byte aligned LDS buffer.  When the source run is
// 16-byte aligned the bulk goes as 16-byte pieces; the rest (and unaligned runs) element-wise.
template <int THREADS = 256>
__device__ __forceinline__ void stage_ids(const unsigned char* __restrict__ src, unsigned char* lds, int bytes, int tid) {
    int done = 0;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        const int pieces = bytes >> 4;
        for (int i = tid; i < pieces; i += THREADS)
            reinterpret_cast<uint4*>(lds)[i] = reinterpret_cast<const uint4*>(src)[i];
        done = pieces << 4;
    }
    for (int i = done + tid; i < bytes; i += THREADS) lds[i] = src[i];
}

// Bit j of the result is set when slot j of the token holds an id in [0,E) that no earlier slot holds.
template <class IdxT>
__device__ __forceinline__ uint64_t unique_slots(const IdxT* ids, int k, int E) {
    uint64_t m = 0;
    for (int j = 0; j < k; ++j) {
        const int64_t e = (int64_t)ids[j];
        bool ok = e >= 0 && e < E;
        for (int i = 0; i < j; ++i) ok = ok && ((int64_t)ids[i] != e);
        if (ok) m |= 1ull << j;
    }
    return m;
}

// Fast path for k <= 8 (the paper's models route to 8 or fewer experts): the token's ids live in registers,
// e[j] = id of slot j, or -1 when the slot does not exist, is out of range, or repeats an earlier slot.
template <class IdxT>
__device__ __forceinline__ void load_unique8(const IdxT* ids, int k, int E, int (&e)[8]) {
    if (sizeof(IdxT) == 1 && k == 8) {
        const uint2 w = *reinterpret_cast<const uint2*>(ids);  // token t sits at byte 8*t of the staged run
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            e[j] = (int)((w.x >> (8 * j)) & 0xffu);
            e[4 + j] = (int)((w.y >> (8 * j)) & 0xffu);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = j < k ? (int)ids[j] : -1;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (e[j] < 0 || e[j] >= E) e[j] = -1;
#pragma unroll
    for (int j = 1; j < 8; ++j) {
        bool dup = false;
#pragma unroll
        for (int i = 0; i < j; ++i) dup = dup || (e[i] == e[j]);
        if (dup) e[j] = -1;
    }
}

// ---------------------------------------------------------------------------------------------------
// One workgroup per sample: histogram of token membership, entropy of the normalised histogram (fp64, fixed
// summation order), and the sample's contribution to the global loads.
template <class IdxT>
__global__ __launch_bounds__(kStatThreads) void k_affinity(const IdxT* __restrict__ idx, int L, int k, int E,
                                                           int chunk_tokens, int32_t* __restrict__ counts,
                                                           double* __restrict__ entropy,
                                                           unsigned long long* __restrict__ loads) {
    __shared__ __attribute__((aligned(16))) unsigned char s_ids[kStageBytes];
    __shared__ int32_t s_hist[kMaxExperts];
    __shared__ double s_red[kStatThreads];
    __shared__ long long s_tot[kStatThreads];
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    for (int e = tid; e < E; e += kStatThreads) s_hist[e] = 0;
    const IdxT* base = idx + (size_t)s * L * k;
    for (int t0 = 0; t0 < L; t0 += chunk_tokens) {
        const int toks = min(chunk_tokens, L - t0);
        __syncthreads();  // previous pass done with s_ids (and s_hist cleared on the first)
        stage_ids(reinterpret_cast<const unsigned char*>(base + (size_t)t0 * k), s_ids, toks * k * (int)sizeof(IdxT), tid);
        __syncthreads();
        for (int t = tid; t < toks; t += kStatThreads) {
            const IdxT* ids = reinterpret_cast<const IdxT*>(s_ids) + t * k;
            if (k <= 8) {
                int e[8];
                load_unique8(ids, k, E, e);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (e[j] >= 0) atomicAdd(&s_hist[e[j]], 1);
            } else {
                const uint64_t m = unique_slots(ids, k, E);
                for (int j = 0; j < k; ++j)
                    if ((m >> j) & 1) atomicAdd(&s_hist[(int)ids[j]], 1);
            }
        }
    }
    __syncthreads();
    long long tot = 0;
    double clogc = 0.0;
    for (int e = tid; e < E; e += kStatThreads) {
        const int c = s_hist[e];
        counts[s * E + e] = c;
        if (c > 0) {
            atomicAdd(&loads[e], (unsigned long long)c);
            tot += c;
            clogc += (double)c * log2((double)c);
        }
    }
    s_red[tid] = clogc;
    s_tot[tid] = tot;
    __syncthreads();
    for (int w = kStatThreads / 2; w > 0; w >>= 1) {
        if (tid < w) {
            s_red[tid] += s_red[tid + w];
            s_tot[tid] += s_tot[tid + w];
        }
        __syncthreads();
    }
    if (tid == 0) {
        // H = -sum p log2 p with p = c / tot  =  log2(tot) - (sum c log2 c) / tot
        const double n = (double)s_tot[0];
        entropy[s] = s_tot[0] > 0 ? log2(n) - s_red[0] / n : 0.0;
    }
}

__global__ void k_fill_u64(unsigned long long* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

// (max L - mean L) / mean L over the E loads; one workgroup.
__global__ __launch_bounds__(kStatThreads) void k_maxvio(const unsigned long long* __restrict__ loads, int E,
                                                         double* __restrict__ out) {
    __shared__ unsigned long long s_max[kStatThreads], s_sum[kStatThreads];
    const int tid = threadIdx.x;
    unsigned long long mx = 0, sum = 0;
    for (int e = tid; e < E; e += kStatThreads) {
        const unsigned long long v = loads[e];
        mx = v > mx ? v : mx;
        sum += v;
    }
    s_max[tid] = mx;
    s_sum[tid] = sum;
    __syncthreads();
    for (int w = kStatThreads / 2; w > 0; w >>= 1) {
        if (tid < w) {
            s_max[tid] = s_max[tid + w] > s_max[tid] ? s_max[tid + w] : s_max[tid];
            s_sum[tid] += s_sum[tid + w];
        }
        __syncthreads();
    }
    if (tid == 0) {
        const double mean = (double)s_sum[0] / (double)E;
        out[0] = s_sum[0] > 0 ? ((double)s_max[0] - mean) / mean : 0.0;
    }
}

// ---------------------------------------------------------------------------------------------------
// One workgroup per sample.  expert_nodes[e] has bit n set when expert e lives on node n, so the nodes a
// token reaches are the OR over its experts; per node the wave counts its lanes with one ballot.
template <class IdxT>
__global__ __launch_bounds__(kStatThreads) void k_placement(const IdxT* __restrict__ idx, int L, int k, int E,
                                                            int chunk_tokens, const uint64_t* __restrict__ expert_nodes,
                                                            int n_nodes, int32_t* __restrict__ comm,
                                                            int32_t* __restrict__ best_node) {
    __shared__ __attribute__((aligned(16))) unsigned char s_ids[kStageBytes];
    __shared__ uint64_t s_nodes[kMaxExperts];
    __shared__ int32_t s_comm[64];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t s = blockIdx.x;
    for (int e = tid; e < E; e += kStatThreads) s_nodes[e] = expert_nodes[e];
    if (tid < 64) s_comm[tid] = 0;
    const IdxT* base = idx + (size_t)s * L * k;
    int acc = 0;  // lane n of every wave counts node n
    for (int t0 = 0; t0 < L; t0 += chunk_tokens) {
        const int toks = min(chunk_tokens, L - t0);
        __syncthreads();
        stage_ids(reinterpret_cast<const unsigned char*>(base + (size_t)t0 * k), s_ids, toks * k * (int)sizeof(IdxT), tid);
        __syncthreads();
        // whole waves take part in every ballot: the loop bound is rounded up to the workgroup size
        for (int tb = 0; tb < toks; tb += kStatThreads) {
            const int t = tb + tid;
            uint64_t reach = 0;
            if (t < toks) {
                const IdxT* ids = reinterpret_cast<const IdxT*>(s_ids) + t * k;
                if (k <= 8) {
                    int e[8];
                    load_unique8(ids, k, E, e);
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (e[j] >= 0) reach |= s_nodes[e[j]];
                } else {
                    for (int j = 0; j < k; ++j) {
                        const int64_t e = (int64_t)ids[j];
                        if (e >= 0 && e < E) reach |= s_nodes[e];
                    }
                }
            }
            for (int n = 0; n < n_nodes; ++n) {
                const uint64_t b = __ballot((reach >> n) & 1);
                if (lane == n) acc += __popcll(b);
            }
        }
    }
    if (lane < n_nodes && acc) atomicAdd(&s_comm[lane], acc);
    __syncthreads();
    if (tid < n_nodes) comm[s * n_nodes + tid] = s_comm[tid];
    if (tid == 0) {
        int best = 0, mx = -1;
        for (int n = 0; n < n_nodes; ++n)
            if (s_comm[n] > mx) {
                mx = s_comm[n];
                best = n;
            }
        best_node[s] = best;
    }
}

// ---------------------------------------------------------------------------------------------------
// Co-activation counts.  A workgroup owns a contiguous run of tokens and counts pairs (i <= j) in an LDS
// matrix of 16-bit counters (two per 32-bit word, EP x EP with EP >= E); before any counter could reach 2^16
// (every token adds at most 1 to a counter) the matrix is flushed into the 64-bit global matrix with
// atomics, mirrored across the diagonal, and cleared.
constexpr int kFlushTokens = 32768;
constexpr int kCoactThreads = 1024;  // many waves per CU hide the latency of the LDS atomics

template <int EP>
__device__ __forceinline__ void coact_flush(uint32_t* s_cnt, int E, unsigned long long* __restrict__ P, int tid) {
    for (int w = tid; w < EP * EP / 2; w += kCoactThreads) {
        const uint32_t v = s_cnt[w];
        if (!v) continue;
        s_cnt[w] = 0;
        const int i = (2 * w) / EP, j = (2 * w) % EP;
        const uint32_t lo = v & 0xffffu, hi = v >> 16;
        if (lo) {
            atomicAdd(&P[(size_t)i * E + j], (unsigned long long)lo);
            if (i != j) atomicAdd(&P[(size_t)j * E + i], (unsigned long long)lo);
        }
        if (hi) {
            atomicAdd(&P[(size_t)i * E + j + 1], (unsigned long long)hi);
            if (i != j + 1) atomicAdd(&P[(size_t)(j + 1) * E + i], (unsigned long long)hi);
        }
    }
}

template <int EP>
__device__ __forceinline__ void coact_count(uint32_t* s_cnt, int ea, int eb) {
    const int i = min(ea, eb), j = max(ea, eb);
    const int cell = i * EP + j;
    atomicAdd(&s_cnt[cell >> 1], 1u << ((cell & 1) * 16));
}

template <class IdxT, int EP>
__global__ __launch_bounds__(kCoactThreads) void k_coactivation(const IdxT* __restrict__ idx, int64_t T, int k, int E,
                                                                int chunk_tokens, int64_t tokens_per_group,
                                                                unsigned long long* __restrict__ P) {
    __shared__ __attribute__((aligned(16))) unsigned char s_ids[kStageBytes];
    __shared__ uint32_t s_cnt[EP * EP / 2];
    const int tid = threadIdx.x;
    for (int w = tid; w < EP * EP / 2; w += kCoactThreads) s_cnt[w] = 0;
    const int64_t begin = (int64_t)blockIdx.x * tokens_per_group;
    const int64_t end = min(T, begin + tokens_per_group);
    int since_flush = 0;
    for (int64_t t0 = begin; t0 < end; t0 += chunk_tokens) {
        const int toks = (int)min((int64_t)chunk_tokens, end - t0);
        __syncthreads();
        if (since_flush + toks > kFlushTokens) {
            coact_flush<EP>(s_cnt, E, P, tid);
            since_flush = 0;
            __syncthreads();
        }
        stage_ids<kCoactThreads>(reinterpret_cast<const unsigned char*>(idx + (size_t)t0 * k), s_ids,
                                 toks * k * (int)sizeof(IdxT), tid);
        __syncthreads();
        for (int t = tid; t < toks; t += kCoactThreads) {
            const IdxT* ids = reinterpret_cast<const IdxT*>(s_ids) + t * k;
            if (k <= 8) {
                int e[8];
                load_unique8(ids, k, E, e);
#pragma unroll
                for (int a = 0; a < 8; ++a) {
                    if (e[a] < 0) continue;
#pragma unroll
                    for (int b = a; b < 8; ++b)
                        if (e[b] >= 0) coact_count<EP>(s_cnt, e[a], e[b]);
                }
            } else {
                const uint64_t m = unique_slots(ids, k, E);
                for (int a = 0; a < k; ++a) {
                    if (!((m >> a) & 1)) continue;
                    for (int b = a; b < k; ++b)
                        if ((m >> b) & 1) coact_count<EP>(s_cnt, (int)ids[a], (int)ids[b]);
                }
            }
        }
        since_flush += toks;
    }
    __syncthreads();
    coact_flush<EP>(s_cnt, E, P, tid);
}

// ---------------------------------------------------------------------------------------------------
// Greedy affinity grouping, one workgroup, thread j <-> source expert j.  Groups are filled one after the
// other; a group starts with the lowest unassigned expert, then takes the unassigned expert with the
// largest summed co-activation with its members (lowest number on ties).
constexpr long long kNoCandidate = -0x7fffffffffffffffLL - 1;  // below every real score

// THREADS >= E_S.  STAGED (E_S <= 128): the whole matrix is first copied into LDS, so a round's row read is an
// LDS access instead of a global round trip on the critical path of E_S dependent rounds.
template <int THREADS, bool STAGED>
__global__ __launch_bounds__(THREADS) void k_fold_groups(const long long* __restrict__ P, int E_S, int E_T,
                                                         int32_t* __restrict__ group_of) {
    constexpr int kWaves = THREADS / 64;
    __shared__ long long s_key[kWaves];
    __shared__ int s_idx[kWaves];
    __shared__ int s_pick;
    __shared__ long long s_P[STAGED ? 128 * 128 : 1];
    const int j = threadIdx.x;
    const int lane = j & 63, wave = j >> 6;
    if (STAGED) {
        for (int i = j; i < E_S * E_S; i += THREADS) s_P[i] = P[i];
        __syncthreads();
    }
    const bool real = j < E_S;
    bool assigned = !real;
    long long score = 0;
    const int g_avg = E_S / E_T, n_extra = E_S % E_T;
    for (int g = 0; g < E_T; ++g) {
        const int size = g_avg + (g < n_extra ? 1 : 0);
        for (int m = 0; m < size; ++m) {
            // key: for the first member every unassigned expert ties (lowest number wins); later the score
            long long key = assigned ? kNoCandidate : (m == 0 ? 0 : score);
            int who = j;
            for (int off = 32; off > 0; off >>= 1) {
                const long long ok = __shfl_down(key, off);
                const int ow = __shfl_down(who, off);
                if (ok > key || (ok == key && ow < who)) {
                    key = ok;
                    who = ow;
                }
            }
            if (lane == 0) {
                s_key[wave] = key;
                s_idx[wave] = who;
            }
            __syncthreads();
            if (j == 0) {
                long long bk = s_key[0];
                int bw = s_idx[0];
                for (int w = 1; w < kWaves; ++w)
                    if (s_key[w] > bk || (s_key[w] == bk && s_idx[w] < bw)) {
                        bk = s_key[w];
                        bw = s_idx[w];
                    }
                s_pick = bw;
            }
            __syncthreads();
            const int pick = s_pick;
            if (j == pick) {
                assigned = true;
                group_of[j] = g;
            }
            if (real) score = (m == 0 ? 0 : score) + (STAGED ? s_P[pick * E_S + j] : P[(size_t)pick * E_S + j]);
            __syncthreads();  // s_pick, s_key are rewritten by the next round
        }
    }
}

// out[r][g] = sum over source experts e with group_of[e] == g of W[r][e], e ascending, fp32.
__global__ __launch_bounds__(kStatThreads) void k_fold_weights(const float* __restrict__ W, const int32_t* __restrict__ group_of,
                                                               int E_S, int E_T, float* __restrict__ out) {
    __shared__ float s_w[kMaxExperts];
    __shared__ int32_t s_g[kMaxExperts];
    const int r = blockIdx.x;
    for (int e = threadIdx.x; e < E_S; e += kStatThreads) {
        s_w[e] = W[(size_t)r * E_S + e];
        s_g[e] = group_of[e];
    }
    __syncthreads();
    for (int g = threadIdx.x; g < E_T; g += kStatThreads) {
        float acc = 0.f;
        for (int e = 0; e < E_S; ++e)
            if (s_g[e] == g) acc += s_w[e];
        out[(size_t)r * E_T + g] = acc;
    }
}

int chunk_tokens_for(int k, int idx_dtype) {
    const int per_token = k * (idx_dtype == 1 ? 1 : 4);
    return kStageBytes / per_token;  // >= 64 for k <= 64
}

}  // namespace

hipError_t launch_affinity(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                           double* entropy, int64_t* loads, double* maxvio, hipStream_t s) {
    auto* l = reinterpret_cast<unsigned long long*>(loads);
    hipLaunchKernelGGL(k_fill_u64, dim3((E + 255) / 256), dim3(256), 0, s, l, (int64_t)E);
    const int ct = chunk_tokens_for(k, idx_dtype);
    if (idx_dtype == 1)
        hipLaunchKernelGGL(k_affinity<uint8_t>, dim3((unsigned)S), dim3(kStatThreads), 0, s, (const uint8_t*)idx, L, k, E,
                           ct, counts, entropy, l);
    else
        hipLaunchKernelGGL(k_affinity<int32_t>, dim3((unsigned)S), dim3(kStatThreads), 0, s, (const int32_t*)idx, L, k, E,
                           ct, counts, entropy, l);
    hipLaunchKernelGGL(k_maxvio, dim3(1), dim3(kStatThreads), 0, s, l, E, maxvio);
    return hipGetLastError();
}

hipError_t launch_placement(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, const uint64_t* expert_nodes,
                            int n_nodes, int32_t* comm, int32_t* best_node, hipStream_t s) {
    const int ct = chunk_tokens_for(k, idx_dtype);
    if (idx_dtype == 1)
        hipLaunchKernelGGL(k_placement<uint8_t>, dim3((unsigned)S), dim3(kStatThreads), 0, s, (const uint8_t*)idx, L, k, E,
                           ct, expert_nodes, n_nodes, comm, best_node);
    else
        hipLaunchKernelGGL(k_placement<int32_t>, dim3((unsigned)S), dim3(kStatThreads), 0, s, (const int32_t*)idx, L, k, E,
                           ct, expert_nodes, n_nodes, comm, best_node);
    return hipGetLastError();
}

template <class IdxT>
static void launch_coact_t(const IdxT* idx, int64_t T, int k, int E, int ct, unsigned long long* P, hipStream_t s) {
    // One resident workgroup per CU at most: every group ends with a flush of its whole matrix through global
    // atomics, so more groups than CUs only adds flush traffic.
    int64_t groups = (T + 8191) / 8192;
    if (groups > 256) groups = 256;
    if (groups < 1) groups = 1;
    const int64_t per = (T + groups - 1) / groups;
    const dim3 grid((unsigned)((T + per - 1) / per)), block(kCoactThreads);
    if (E <= 64)
        hipLaunchKernelGGL((k_coactivation<IdxT, 64>), grid, block, 0, s, idx, T, k, E, ct, per, P);
    else if (E <= 128)
        hipLaunchKernelGGL((k_coactivation<IdxT, 128>), grid, block, 0, s, idx, T, k, E, ct, per, P);
    else
        hipLaunchKernelGGL((k_coactivation<IdxT, 256>), grid, block, 0, s, idx, T, k, E, ct, per, P);
}

hipError_t launch_coactivation(const void* idx, int idx_dtype, int64_t T, int k, int E, int64_t* P, hipStream_t s) {
    auto* p = reinterpret_cast<unsigned long long*>(P);
    const int64_t n = (int64_t)E * E;
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    const int ct = chunk_tokens_for(k, idx_dtype);
    if (idx_dtype == 1) launch_coact_t((const uint8_t*)idx, T, k, E, ct, p, s);
    else launch_coact_t((const int32_t*)idx, T, k, E, ct, p, s);
    return hipGetLastError();
}

hipError_t launch_fold_groups(const int64_t* P, int E_S, int E_T, int32_t* group_of, hipStream_t s) {
    const long long* p = (const long long*)P;
    if (E_S <= 128) hipLaunchKernelGGL((k_fold_groups<128, true>), dim3(1), dim3(128), 0, s, p, E_S, E_T, group_of);
    else if (E_S <= 256) hipLaunchKernelGGL((k_fold_groups<256, false>), dim3(1), dim3(256), 0, s, p, E_S, E_T, group_of);
    else hipLaunchKernelGGL((k_fold_groups<1024, false>), dim3(1), dim3(1024), 0, s, p, E_S, E_T, group_of);
    return hipGetLastError();
}

hipError_t launch_fold_weights(const float* W, const int32_t* group_of, int d, int E_S, int E_T, float* out, hipStream_t s) {
    hipLaunchKernelGGL(k_fold_weights, dim3((unsigned)d), dim3(kStatThreads), 0, s, W, group_of, E_S, E_T, out);
    return hipGetLastError();
}

}  // namespace grouter
