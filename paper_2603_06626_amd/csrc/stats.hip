// Routing statistics computed from cached top-k expert ids (integer work, one pass over the ids each):
//   * per-sample routing affinity counts, their entropy, expert loads and the maximal violation
//     (Sec. 3.3.2 first equation; App. "Efficiency Experiment Detail", expert grouping; App. "Maximal Violation")
//   * sample placement: per (sample, node) the number of tokens that find an expert on the node, and the
//     best node (App. "Efficiency Experiment Detail", algorithm "Optimize Sample-to-Node Assignment")
//   * expert folding: co-activation matrix, greedy affinity grouping, folded score weights (Sec. 3.2.1)
//
// The per-sample statistics (affinity counts, entropy, loads, placement) come from one kernel that reads every id
// once: a lane takes one token, loads its k ids with one coalesced access (8 bytes for the cached format of
// k = 8 one-byte ids), counts membership with LDS atomics and votes per node with wave ballots.  The
// co-activation matrix is a Gram matrix, P = sum over tokens of ind_t ind_t^T with ind_t the 0/1 membership vector of
// a token: a workgroup writes the indicator bytes of 256 tokens into LDS (expert-major, so that 16 consecutive
// tokens of one expert are one 16-byte read) and accumulates P on the matrix cores with 8-bit integer MFMAs,
// exact in int32.  Membership is an indicator per token: an id repeated inside a token counts once, ids outside
// [0,E) are ignored.  Integer arithmetic throughout, so every result is bit-reproducible.
#include "common.hpp"

namespace grouter {

namespace {

constexpr int kStatThreads = 256;
constexpr int kMaxStatK = 64;           // a token's validity mask is one 64-bit word

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

// ---------------------------------------------------------------------------------------------------
// Fast path for k <= 8 (the paper's models route to 8 or fewer experts): the ids of token t live in registers,
// e[j] = id of slot j, or -1 when the slot does not exist, is out of range, or repeats an earlier slot.
// One 8-byte access for the cached format (uint8, k = 8), two 16-byte ones for int32 ids with k = 8.
struct RawIds8 {   // the k <= 8 ids of one token as fetched, before range check and de-duplication
    int e[8];
};
template <class IdxT>
__device__ __forceinline__ RawIds8 fetch_token8(const IdxT* __restrict__ base, int64_t t, int k) {
    RawIds8 r;
    const IdxT* ids = base + t * k;
    if (sizeof(IdxT) == 1 && k == 8 && (reinterpret_cast<uintptr_t>(base) & 7u) == 0) {
        const uint2 w = *reinterpret_cast<const uint2*>(ids);
        r.e[0] = (int)w.x;      // unpacked by decode_token8
        r.e[1] = (int)w.y;
    } else if (sizeof(IdxT) == 4 && k == 8 && (reinterpret_cast<uintptr_t>(base) & 15u) == 0) {
        const int4 a = reinterpret_cast<const int4*>(ids)[0], b = reinterpret_cast<const int4*>(ids)[1];
        r.e[0] = a.x; r.e[1] = a.y; r.e[2] = a.z; r.e[3] = a.w;
        r.e[4] = b.x; r.e[5] = b.y; r.e[6] = b.z; r.e[7] = b.w;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) r.e[j] = j < k ? (int)ids[j] : -1;
    }
    return r;
}
// the 8 ids as fetched (slots past k hold -1), without any filtering
template <class IdxT>
__device__ __forceinline__ void unpack_token8(const IdxT* __restrict__ base, const RawIds8& r, int k, int (&e)[8]) {
    if (sizeof(IdxT) == 1 && k == 8 && (reinterpret_cast<uintptr_t>(base) & 7u) == 0) {
        const uint32_t x = (uint32_t)r.e[0], y = (uint32_t)r.e[1];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            e[j] = (int)((x >> (8 * j)) & 0xffu);
            e[4 + j] = (int)((y >> (8 * j)) & 0xffu);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = r.e[j];
    }
}
template <class IdxT>
__device__ __forceinline__ void decode_token8(const IdxT* __restrict__ base, const RawIds8& r, int k, int E, int (&e)[8]) {
    if (sizeof(IdxT) == 1 && k == 8 && (reinterpret_cast<uintptr_t>(base) & 7u) == 0) {
        const uint32_t x = (uint32_t)r.e[0], y = (uint32_t)r.e[1];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            e[j] = (int)((x >> (8 * j)) & 0xffu);
            e[4 + j] = (int)((y >> (8 * j)) & 0xffu);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = r.e[j];
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
template <class IdxT>
__device__ __forceinline__ void load_token8(const IdxT* __restrict__ base, int64_t t, int k, int E, int (&e)[8]) {
    decode_token8(base, fetch_token8(base, t, k), k, E, e);
}

// One workgroup per sample, one pass over its ids for both statistics:
//   AFF    histogram of token membership, entropy of the normalised histogram (fp64, fixed summation order) and the
//          sample's contribution to the global loads
//   PLACE  expert_nodes[e] has bit n set when expert e lives on node n, so the nodes a token reaches are the OR
//          over its experts; per node the wave counts its lanes with one ballot
template <class IdxT, bool AFF, bool PLACE>
__global__ __launch_bounds__(kStatThreads) void k_sample_stats(const IdxT* __restrict__ idx, int L, int k, int E,
                                                               int32_t* __restrict__ counts, double* __restrict__ entropy,
                                                               unsigned long long* __restrict__ loads,
                                                               const uint64_t* __restrict__ expert_nodes, int n_nodes,
                                                               int32_t* __restrict__ comm, int32_t* __restrict__ best_node) {
    __shared__ int32_t s_hist[AFF ? kMaxExperts : 1];
    __shared__ uint64_t s_nodes[PLACE ? kMaxExperts : 1];
    __shared__ int32_t s_comm[64];
    __shared__ double s_red[kStatThreads];
    __shared__ long long s_tot[kStatThreads];
    const int tid = threadIdx.x, lane = tid & 63;
    const int64_t s = blockIdx.x;
    if (AFF)
        for (int e = tid; e < E; e += kStatThreads) s_hist[e] = 0;
    if (PLACE) {
        for (int e = tid; e < E; e += kStatThreads) s_nodes[e] = expert_nodes[e];
        if (tid < 64) s_comm[tid] = 0;
    }
    __syncthreads();
    const IdxT* base = idx + (size_t)s * L * k;
    int acc = 0;  // PLACE: lane n of every wave counts node n
    // whole waves take part in every ballot: the loop bound is rounded up to the workgroup size
    for (int tb = 0; tb < L; tb += kStatThreads) {
        const int t = tb + tid;
        uint64_t reach = 0;
        if (t < L) {
            if (k <= 8) {
                int e[8];
                load_token8(base, t, k, E, e);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (e[j] >= 0) {
                        if (AFF) atomicAdd(&s_hist[e[j]], 1);
                        if (PLACE) reach |= s_nodes[e[j]];
                    }
            } else {
                const IdxT* ids = base + (size_t)t * k;
                const uint64_t m = unique_slots(ids, k, E);
                for (int j = 0; j < k; ++j)
                    if ((m >> j) & 1) {
                        if (AFF) atomicAdd(&s_hist[(int)ids[j]], 1);
                        if (PLACE) reach |= s_nodes[(int)ids[j]];
                    }
            }
        }
        if (PLACE)
            for (int n = 0; n < n_nodes; ++n) {
                const uint64_t b = __ballot((reach >> n) & 1);
                if (lane == n) acc += __popcll(b);
            }
    }
    if (PLACE && lane < n_nodes && acc) atomicAdd(&s_comm[lane], acc);
    __syncthreads();
    if (PLACE) {
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
    if (!AFF) return;
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
// Co-activation counts P[i][j] = number of tokens whose top-k set holds both i and j: the Gram matrix of the
// token x expert indicator matrix.  A workgroup owns a contiguous run of tokens and walks it TOK tokens at a
// time: every lane sets the (at most k) bytes of its token in an expert-major byte matrix ind[e][t] in LDS (and
// clears them again after use), and the workgroup multiplies ind by its transpose with v_mfma_i32_32x32x32_i8.
// Both MFMA operands are 16 consecutive token bytes of one expert, i.e. one 16-byte LDS read, and the same read
// serves as row operand and as column operand.  P is symmetric, so only the 32 x 32 blocks on and above the
// diagonal are computed: wave pair p owns block rows p and NBLK-1-p, together NBLK+1 blocks whatever p is.
// The waves of part q of a pair take the 32-token slabs q, q + SPLIT, ... of a pass, so several MFMA chains and
// LDS reads are in flight per SIMD.  Counts stay exact: a workgroup adds at most 1 per token and cell, far
// below 2^31.  At the end the parts are summed through LDS and part 0 adds the blocks into the 64-bit global
// matrix with integer atomics; k_coact_mirror then fills the blocks below the diagonal.
typedef int i32x16_t __attribute__((ext_vector_type(16)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

template <int EP, int SPLIT, int TOK, int PAIR>
struct CoactPair {
    static constexpr int NBLK = EP / 32;
    static constexpr int NSLOT = NBLK + 1;           // blocks this pair owns
    static constexpr int NF = NBLK - PAIR;           // operand fragments it reads per slab: blocks PAIR .. NBLK-1
    static constexpr int ROW_B = NBLK - 1 - PAIR;
    static constexpr int PITCH = TOK + 16;
    // block (row, col) of slot s
    static constexpr int row_of(int s) { return s < NF ? PAIR : ROW_B; }
    static constexpr int col_of(int s) { return s < NF ? PAIR + s : ROW_B + (s - NF); }

    static __device__ __forceinline__ void slabs(const unsigned char* s_ind, int frag_at, int part, i32x16_t (&acc)[NSLOT]) {
#pragma unroll
        for (int i = 0; i < TOK / (32 * SPLIT); ++i) {
            const int s32 = part + i * SPLIT;
            i32x4_t f[NF];
#pragma unroll
            for (int c = 0; c < NF; ++c)
                f[c] = *reinterpret_cast<const i32x4_t*>(s_ind + (PAIR + c) * 32 * PITCH + frag_at + s32 * 32);
#pragma unroll
            for (int s = 0; s < NSLOT; ++s)
                acc[s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f[row_of(s) - PAIR], f[col_of(s) - PAIR], acc[s], 0, 0, 0);
        }
    }
};

template <class IdxT, int EP, int SPLIT, int TOK>
__global__ __launch_bounds__(EP / 64 * SPLIT * 64) void k_coactivation(const IdxT* __restrict__ idx, int64_t T, int k, int E,
                                                                    int64_t tokens_per_group, unsigned long long* __restrict__ P) {
    constexpr int NBLK = EP / 32;        // 32-expert blocks per side
    constexpr int NPAIR = NBLK / 2;      // wave pairs: block rows p and NBLK-1-p
    constexpr int NSLOT = NBLK + 1;
    constexpr int THREADS = NPAIR * 64 * SPLIT;
    constexpr int PITCH = TOK + 16;      // bytes per expert row: 16-byte reads of neighbouring experts miss each other's banks
    static_assert(NBLK % 2 == 0 && NPAIR <= 4, "block rows are owned in pairs");
    static_assert(TOK % (32 * SPLIT) == 0 && TOK <= THREADS, "one token per lane, whole slabs per part");
    static_assert(EP * PITCH >= NPAIR * 16 * 64 * 4, "the indicator buffer can hold one accumulator per pair");
    // one more row than experts: ids that do not count (out of range, slots past k, lanes without a token) are
    // pointed at it, so the set and clear passes are eight unconditional byte stores each.  (Two indicator
    // buffers, with the clear of pass i-1 and the set of pass i+1 issued under the MFMAs of pass i and one
    // barrier per pass, measured slower: 0.128 vs 0.118 ms on the 8.4 M-token corpus.)
    __shared__ __attribute__((aligned(16))) unsigned char s_ind[(EP + 1) * PITCH];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rp = wave % NPAIR, part = wave / NPAIR;
    const int64_t begin = (int64_t)blockIdx.x * tokens_per_group;
    const int64_t end = min(T, begin + tokens_per_group);
    i32x16_t acc[NSLOT];
#pragma unroll
    for (int s = 0; s < NSLOT; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = 0;
    const int frag_at = (lane & 31) * PITCH + 16 * (lane >> 5);   // this lane's 16 tokens of expert (block * 32 + lane % 32)
    static_assert((TOK & (TOK - 1)) == 0, "TOK is a power of two");
    const int kDummy = EP * PITCH + (tid & (TOK - 1));   // this lane's byte of the spare row (never read)
    // k <= 8: the ids of the next pass are fetched before the MFMAs of this one, so their latency is hidden
    RawIds8 ahead{};
    if (k <= 8 && tid < TOK && begin + tid < end) ahead = fetch_token8(idx, begin + tid, k);
    for (int i = tid; i < (EP + 1) * PITCH / 16; i += THREADS) reinterpret_cast<uint4*>(s_ind)[i] = uint4{0u, 0u, 0u, 0u};
    __syncthreads();
    for (int64_t t0 = begin; t0 < end; t0 += TOK) {
        const int toks = (int)min((int64_t)TOK, end - t0);
        // set this pass's bytes; after the MFMAs every lane clears the bytes it set, so the matrix is never swept
        int mine[8];
        if (k <= 8) {
            unpack_token8(idx, ahead, k, mine);
#pragma unroll
            for (int j = 0; j < 8; ++j) {   // a repeated id sets the same byte again
                mine[j] = (tid < toks && (unsigned)mine[j] < (unsigned)E) ? mine[j] * PITCH + tid : kDummy;
                s_ind[mine[j]] = 1;
            }
            if (tid < TOK && t0 + TOK + tid < end) ahead = fetch_token8(idx, t0 + TOK + tid, k);
        } else if (tid < toks) {
            const IdxT* ids = idx + (size_t)(t0 + tid) * k;
            for (int j = 0; j < k; ++j) {
                const int64_t e = (int64_t)ids[j];
                if (e >= 0 && e < E) s_ind[e * PITCH + tid] = 1;   // a repeated id sets the same byte again
            }
        }
        __syncthreads();
        // (columns past the last token of a short pass are zero, so the slabs need no bound of their own)
        if (rp == 0) CoactPair<EP, SPLIT, TOK, 0>::slabs(s_ind, frag_at, part, acc);
        if constexpr (NPAIR > 1) { if (rp == 1) CoactPair<EP, SPLIT, TOK, 1>::slabs(s_ind, frag_at, part, acc); }
        if constexpr (NPAIR > 2) { if (rp == 2) CoactPair<EP, SPLIT, TOK, 2>::slabs(s_ind, frag_at, part, acc); }
        if constexpr (NPAIR > 3) { if (rp == 3) CoactPair<EP, SPLIT, TOK, 3>::slabs(s_ind, frag_at, part, acc); }
        __syncthreads();   // every wave has read the indicator
        if (k <= 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) s_ind[mine[j]] = 0;
        } else if (tid < toks) {
            const IdxT* ids = idx + (size_t)(t0 + tid) * k;
            for (int j = 0; j < k; ++j) {
                const int64_t e = (int64_t)ids[j];
                if (e >= 0 && e < E) s_ind[e * PITCH + tid] = 0;
            }
        }
        // no barrier needed here: a lane clears and then sets only bytes of its own token column
    }
    // sum the parts: part q hands its accumulators to part 0 through LDS, one slot of every pair at a time
    int* const xchg = reinterpret_cast<int*>(s_ind);
#pragma unroll 1
    for (int q = 1; q < SPLIT; ++q) {
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            __syncthreads();
            if (part == q) {
#pragma unroll
                for (int v = 0; v < 16; ++v) xchg[(rp * 16 + v) * 64 + lane] = acc[s][v];
            }
            __syncthreads();
            if (part == 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[s][v] += xchg[(rp * 16 + v) * 64 + lane];
            }
        }
    }
    if (part != 0) return;
    // accumulator element v of a lane is row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32 of the block
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
        // slot -> block (uniform per wave; same mapping as CoactPair)
        const int nf = NBLK - rp;
        const int brow = s < nf ? rp : NBLK - 1 - rp;
        const int bcol = s < nf ? rp + s : (NBLK - 1 - rp) + (s - nf);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = brow * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            const int col = bcol * 32 + (lane & 31);
            const int c = acc[s][v];
            if (row < E && col < E && c) atomicAdd(&P[(size_t)row * E + col], (unsigned long long)c);
        }
    }
}

// The blocks below the diagonal are the transposes of the ones above it (a mirrored atomic per cell would touch
// one cache line per lane): filled in afterwards, one workgroup per row.
__global__ __launch_bounds__(256) void k_coact_mirror(int E, unsigned long long* __restrict__ P) {
    const int row = blockIdx.x;
    for (int col = threadIdx.x; col < (row & ~31); col += 256) P[(size_t)row * E + col] = P[(size_t)col * E + row];
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

}  // namespace

// counts == nullptr skips the affinity half, comm == nullptr the placement half.
hipError_t launch_sample_stats(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                               double* entropy, int64_t* loads, double* maxvio, const uint64_t* expert_nodes, int n_nodes,
                               int32_t* comm, int32_t* best_node, hipStream_t s) {
    auto* l = reinterpret_cast<unsigned long long*>(loads);
    const dim3 grid((unsigned)S), block(kStatThreads);
    if (counts) hipLaunchKernelGGL(k_fill_u64, dim3((E + 255) / 256), dim3(256), 0, s, l, (int64_t)E);
#define GROUTER_STATS(T_, A_, P_)                                                                                  \
    hipLaunchKernelGGL((k_sample_stats<T_, A_, P_>), grid, block, 0, s, (const T_*)idx, L, k, E, counts, entropy, l, \
                       expert_nodes, n_nodes, comm, best_node)
    if (idx_dtype == 1) {
        if (counts && comm) GROUTER_STATS(uint8_t, true, true);
        else if (counts) GROUTER_STATS(uint8_t, true, false);
        else GROUTER_STATS(uint8_t, false, true);
    } else {
        if (counts && comm) GROUTER_STATS(int32_t, true, true);
        else if (counts) GROUTER_STATS(int32_t, true, false);
        else GROUTER_STATS(int32_t, false, true);
    }
#undef GROUTER_STATS
    if (counts) hipLaunchKernelGGL(k_maxvio, dim3(1), dim3(kStatThreads), 0, s, l, E, maxvio);
    return hipGetLastError();
}

hipError_t launch_affinity(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, int32_t* counts,
                           double* entropy, int64_t* loads, double* maxvio, hipStream_t s) {
    return launch_sample_stats(idx, idx_dtype, S, L, k, E, counts, entropy, loads, maxvio, nullptr, 0, nullptr, nullptr, s);
}

hipError_t launch_placement(const void* idx, int idx_dtype, int64_t S, int L, int k, int E, const uint64_t* expert_nodes,
                            int n_nodes, int32_t* comm, int32_t* best_node, hipStream_t s) {
    return launch_sample_stats(idx, idx_dtype, S, L, k, E, nullptr, nullptr, nullptr, nullptr, expert_nodes, n_nodes, comm,
                               best_node, s);
}

template <class IdxT>
static void launch_coact_t(const IdxT* idx, int64_t T, int k, int E, unsigned long long* P, hipStream_t s) {
    // Every workgroup ends by adding its whole matrix into the global one, so no more groups than there are CUs.
    constexpr int kTok = 512;
    constexpr int max_groups = 256;   // measured on 8.4 M tokens: 128 groups 0.31 ms, 256 groups 0.18 ms, 512 groups 0.20 ms
    int64_t groups = (T + 2 * kTok - 1) / (2 * kTok);
    if (groups > max_groups) groups = max_groups;
    if (groups < 1) groups = 1;
    const int64_t per = ((T + groups - 1) / groups + kTok - 1) / kTok * kTok;
    const dim3 grid((unsigned)((T + per - 1) / per));
    if (E <= 64)
        hipLaunchKernelGGL((k_coactivation<IdxT, 64, 8, kTok>), grid, dim3(512), 0, s, idx, T, k, E, per, P);
    else if (E <= 128)
        hipLaunchKernelGGL((k_coactivation<IdxT, 128, 4, kTok>), grid, dim3(512), 0, s, idx, T, k, E, per, P);
    else
        hipLaunchKernelGGL((k_coactivation<IdxT, 256, 2, kTok>), grid, dim3(512), 0, s, idx, T, k, E, per, P);
}

hipError_t launch_coactivation(const void* idx, int idx_dtype, int64_t T, int k, int E, int64_t* P, hipStream_t s) {
    auto* p = reinterpret_cast<unsigned long long*>(P);
    const int64_t n = (int64_t)E * E;
    hipLaunchKernelGGL(k_fill_u64, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    if (idx_dtype == 1) launch_coact_t((const uint8_t*)idx, T, k, E, p, s);
    else launch_coact_t((const int32_t*)idx, T, k, E, p, s);
    if (E > 32) hipLaunchKernelGGL(k_coact_mirror, dim3((unsigned)E), dim3(256), 0, s, E, p);
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
