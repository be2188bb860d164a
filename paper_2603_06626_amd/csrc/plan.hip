// Routing-plan kernels: per-expert histogram, exclusive scan and stable scatter of the N = T*k routed
// slots (the cached top-k expert ids of Sec. 3.3.1), plus the row-tile list the grouped GEMMs walk.
//
// The scatter must reproduce the stable counting sort exactly (ties in ascending slot order), so ranks
// come from prefix counts, never from the arrival order of atomics.  Three launches:
//   1. hist     one wave per chunk of 512 consecutive slots -> chunk_hist[e][chunk], chunk_bad[chunk]
//   2. finish   one workgroup: per expert an exclusive scan over its chunks (chunk_hist becomes the chunk's
//               base inside the expert) and its count; then offsets, experts by descending load, the
//               row-tile list and the header (status flag, tile count)
//   3. scatter  one wave per chunk walks its slots 64 at a time in order; a lane's rank among the lanes
//               of the same expert comes from wave ballots, the running per-expert cursor from LDS
// Nothing is accumulated into memory that an earlier launch must have cleared, so a plan can be rebuilt in
// place and the build can be captured into a HIP graph as it is.
#include "common.hpp"

namespace grouter {

// An id outside [0,E) is reported through *bad and handled as expert 0, so no access leaves the workspace.
template <typename IdxT>
__device__ __forceinline__ int load_expert(const IdxT* idx, int64_t i, int E, bool* bad) {
    int e = (int)idx[i];
    if (e < 0 || e >= E) {
        *bad = true;
        e = 0;
    }
    return e;
}

// chunk_hist is laid out [E][n_chunks] so that the scan over chunks of one expert reads contiguously.
template <typename IdxT>
__global__ __launch_bounds__(64) void k_plan_hist(const IdxT* __restrict__ idx, int64_t N, int E, int n_chunks,
                                                  int32_t* __restrict__ chunk_hist, int32_t* __restrict__ chunk_bad) {
    __shared__ int32_t cnt[kMaxExperts];
    const int lane = threadIdx.x;
    const int chunk = blockIdx.x;
    for (int e = lane; e < E; e += 64) cnt[e] = 0;
    __syncthreads();
    const int64_t base = (int64_t)chunk * kPlanChunk;
    bool bad = false;
    for (int it = 0; it < kPlanChunk / 64; ++it) {
        const int64_t i = base + it * 64 + lane;
        if (i < N) atomicAdd(&cnt[load_expert(idx, i, E, &bad)], 1);
    }
    __syncthreads();
    for (int e = lane; e < E; e += 64) chunk_hist[(size_t)e * n_chunks + chunk] = cnt[e];
    const bool any_bad = __any(bad);
    if (lane == 0) chunk_bad[chunk] = any_bad ? 1 : 0;
}

constexpr int kFinishThreads = 1024;  // thread e <-> expert e (E <= 1024)
constexpr int kFinishWaves = kFinishThreads / 64;

// Exclusive prefix sum over the workgroup's threads; *total receives the sum.  s_w: kFinishWaves + 1 words.
__device__ __forceinline__ int block_exclusive_scan(int v, int32_t* s_w, int tid, int* total) {
    const int lane = tid & 63, wave = tid >> 6;
    int incl = v;
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const int w = lane < kFinishWaves ? s_w[lane] : 0;
        int wi = w;
        for (int o = 1; o < kFinishWaves; o <<= 1) {
            const int up = __shfl_up(wi, o, 64);
            if (lane >= o) wi += up;
        }
        if (lane < kFinishWaves) s_w[lane] = wi - w;
        if (lane == kFinishWaves - 1) s_w[kFinishWaves] = wi;
    }
    __syncthreads();
    const int res = s_w[wave] + incl - v;
    *total = s_w[kFinishWaves];
    __syncthreads();  // s_w may be reused right away
    return res;
}

// One workgroup finishes the counting: chunk scans, counts, offsets, load ranking, tile list, header.
__global__ __launch_bounds__(kFinishThreads) void k_plan_finish(int E, int k, int N, int n_chunks, int32_t* __restrict__ chunk_hist,
                                                                const int32_t* __restrict__ chunk_bad,
                                                                int32_t* __restrict__ counts, int32_t* __restrict__ header,
                                                                int32_t* __restrict__ offsets, int32_t* __restrict__ by_load,
                                                                int32_t* __restrict__ tiles, int max_tiles) {
    __shared__ int32_t s_cnt[kMaxExperts];
    __shared__ int32_t s_off[kMaxExperts];
    __shared__ int32_t s_order[kMaxExperts];  // expert id at each load rank
    __shared__ int32_t s_first[kMaxExperts + 1];  // first tile of each load rank
    __shared__ int32_t s_w[kFinishWaves + 1];
    __shared__ int32_t s_bad;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_bad = 0;
    // per expert: exclusive scan of its per-chunk counts (in place) and its total.  A wave takes four experts at
    // a time and requests the first two 64-chunk blocks of all four before it scans any of them, so the global
    // loads overlap instead of forming a chain of dependent round trips.
    for (int e0 = wave; e0 < E; e0 += 4 * kFinishWaves) {
        int v[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = e0 + i * kFinishWaves;
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int c = b * 64 + lane;
                v[i][b] = (e < E && c < n_chunks) ? chunk_hist[(size_t)e * n_chunks + c] : 0;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = e0 + i * kFinishWaves;
            if (e >= E) break;
            int32_t* row = chunk_hist + (size_t)e * n_chunks;
            int carry = 0;
            for (int c0 = 0; c0 < n_chunks; c0 += 64) {
                const int c = c0 + lane;
                int val;
                if (c0 == 0) val = v[i][0];
                else if (c0 == 64) val = v[i][1];
                else val = c < n_chunks ? row[c] : 0;
                int incl = val;
                for (int o = 1; o < 64; o <<= 1) {
                    const int up = __shfl_up(incl, o, 64);
                    if (lane >= o) incl += up;
                }
                if (c < n_chunks) row[c] = carry + incl - val;
                carry += __shfl(incl, 63, 64);
            }
            if (lane == 0) {
                s_cnt[e] = carry;
                counts[e] = carry;
            }
        }
    }
    __syncthreads();
    int bad = 0;
    for (int c = tid; c < n_chunks; c += kFinishThreads) bad |= chunk_bad[c];
    if (bad) atomicOr(&s_bad, 1);
    // offsets
    const int cnt = tid < E ? s_cnt[tid] : 0;
    int total;
    const int off = block_exclusive_scan(cnt, s_w, tid, &total);
    if (tid < E) {
        s_off[tid] = off;
        offsets[tid] = off;
    }
    if (tid == 0) offsets[E] = total;
    // rank experts by load, heaviest first, ties by lower id
    if (tid < E) {
        int rank = 0;
        for (int o = 0; o < E; ++o) {
            const int co = s_cnt[o];
            rank += (co > cnt) || (co == cnt && o < tid);
        }
        s_order[rank] = tid;
        by_load[rank] = tid;
    }
    __syncthreads();
    // row tiles in load-rank order: thread r owns the expert of rank r
    const int e = tid < E ? s_order[tid] : 0;
    const int rows = tid < E ? s_cnt[e] : 0;
    const int n_tiles = (rows + kTileRowsSmall - 1) / kTileRowsSmall;
    int total_tiles;
    const int t = block_exclusive_scan(n_tiles, s_w, tid, &total_tiles);
    if (tid == 0) {
        header[0] = s_bad;  // every atomicOr above happened before the barriers inside the scans
        header[1] = total_tiles;
        header[2] = N;
        header[3] = k;
        header[4] = E;
    }
    if (tid < E) s_first[tid] = t;
    if (tid == 0) s_first[E] = total_tiles;
    __syncthreads();
    // every tile is written by its own thread: find the load rank whose tile range holds tile ti
    for (int ti = tid; ti < min(total_tiles, max_tiles); ti += kFinishThreads) {
        int lo = 0, hi = E - 1;  // largest rank r with s_first[r] <= ti (ranks without tiles share their successor's start)
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_first[mid] <= ti) lo = mid;
            else hi = mid - 1;
        }
        // one 32-byte record per tile, the same for every tile of an expert: a kernel that is handed tile ti learns
        // from it where any other tile of that expert lies, with one load
        const int ex = s_order[lo];
        int32_t* const rec = tiles + 8 * (size_t)ti;
        rec[0] = ex;
        rec[1] = s_off[ex];
        rec[2] = s_cnt[ex];
        rec[3] = s_first[lo];
        rec[4] = s_first[lo + 1] - s_first[lo];
        rec[5] = rec[6] = rec[7] = 0;
    }
}

template <typename IdxT>
__global__ __launch_bounds__(64) void k_plan_scatter(const IdxT* __restrict__ idx, int64_t N, int E, int k, int bits,
                                                     int n_chunks, const int32_t* __restrict__ chunk_base,
                                                     const int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ row_to_src, int32_t* __restrict__ src_to_row,
                                                     int32_t* __restrict__ row_token) {
    __shared__ int32_t cursor[kMaxExperts];
    const int lane = threadIdx.x;
    const int chunk = blockIdx.x;
    for (int e = lane; e < E; e += 64) cursor[e] = offsets[e] + chunk_base[(size_t)e * n_chunks + chunk];
    __syncthreads();
    const int64_t base = (int64_t)chunk * kPlanChunk;
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    for (int it = 0; it < kPlanChunk / 64; ++it) {
        const int64_t i = base + it * 64 + lane;
        const bool valid = i < N;
        bool bad_unused = false;  // already reported by the histogram pass
        const int e = valid ? load_expert(idx, i, E, &bad_unused) : 0;
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (e >> b) & 1;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        int p = 0;
        if (valid) {
            const int rank = __popcll(peers & below);
            p = cursor[e] + rank;
            row_to_src[p] = (int32_t)i;
            src_to_row[i] = p;
            row_token[p] = (int32_t)(i / k);
        }
        __syncthreads();
        if (valid && (peers >> lane) == 1ull) cursor[e] = p + 1;  // highest lane of the group advances the cursor
        __syncthreads();
    }
}

hipError_t launch_plan_build(const void* idx, int idx_dtype, const PlanLayout& L, void* plan_ws, hipStream_t s) {
    char* b = (char*)plan_ws;
    int32_t* header = (int32_t*)(b + L.off_header);
    int32_t* hist = (int32_t*)(b + L.off_chunk_hist);
    int32_t* bad = (int32_t*)(b + L.off_chunk_bad);
    int32_t* counts = (int32_t*)(b + L.off_counts);
    int32_t* offsets = (int32_t*)(b + L.off_offsets);
    int bits = 0;
    while ((1 << bits) < L.E) ++bits;
    const dim3 grid((unsigned)L.n_chunks), wave(64);
    if (idx_dtype == 0)
        hipLaunchKernelGGL(k_plan_hist<int32_t>, grid, wave, 0, s, (const int32_t*)idx, L.N, L.E, L.n_chunks, hist, bad);
    else
        hipLaunchKernelGGL(k_plan_hist<uint8_t>, grid, wave, 0, s, (const uint8_t*)idx, L.N, L.E, L.n_chunks, hist, bad);
    hipLaunchKernelGGL(k_plan_finish, dim3(1), dim3(kFinishThreads), 0, s, L.E, L.k, (int)L.N, L.n_chunks, hist, (const int32_t*)bad, counts,
                       header, offsets, (int32_t*)(b + L.off_by_load), (int32_t*)(b + L.off_tiles_small), L.max_tiles_small);
    if (idx_dtype == 0)
        hipLaunchKernelGGL(k_plan_scatter<int32_t>, grid, wave, 0, s, (const int32_t*)idx, L.N, L.E, L.k, bits,
                           L.n_chunks, (const int32_t*)hist, (const int32_t*)offsets, (int32_t*)(b + L.off_row_to_src),
                           (int32_t*)(b + L.off_src_to_row), (int32_t*)(b + L.off_row_token));
    else
        hipLaunchKernelGGL(k_plan_scatter<uint8_t>, grid, wave, 0, s, (const uint8_t*)idx, L.N, L.E, L.k, bits,
                           L.n_chunks, (const int32_t*)hist, (const int32_t*)offsets, (int32_t*)(b + L.off_row_to_src),
                           (int32_t*)(b + L.off_src_to_row), (int32_t*)(b + L.off_row_token));
    return hipGetLastError();
}

}  // namespace grouter
