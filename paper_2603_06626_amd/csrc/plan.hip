// Routing-plan kernels: per-expert histogram, exclusive scan and stable scatter of the N = T*k routed
// slots (the cached top-k expert ids of Sec. 3.3.1), plus the row-tile lists the grouped GEMMs walk.
//
// The scatter must reproduce the stable counting sort exactly (ties in ascending slot order), so ranks
// come from prefix counts, never from the arrival order of atomics:
//   1. hist      one wave per chunk of 512 consecutive slots -> chunk_hist[e][chunk]
//   2. chunkscan one wave per expert: exclusive scan over chunks (chunk_hist becomes the chunk's base
//                inside the expert) and the expert's count
//   3. finish    one workgroup: offsets, experts by descending load, row-tile lists
//   4. scatter  one wave per chunk walks its slots 64 at a time in order; a lane's rank among the
//               lanes of the same expert comes from wave ballots, the running per-expert cursor from LDS
#include "common.hpp"

namespace grouter {

template <typename IdxT>
__device__ __forceinline__ int load_expert(const IdxT* idx, int64_t i, int E, int32_t* status) {
    int e = (int)idx[i];
    if (e < 0 || e >= E) {
        atomicOr(status, 1);
        e = 0;
    }
    return e;
}

__global__ __launch_bounds__(64) void k_plan_clear(int32_t* __restrict__ header, int32_t* __restrict__ zero_page) {
    header[threadIdx.x] = 0;
    zero_page[threadIdx.x] = 0;
}

// chunk_hist is laid out [E][n_chunks] so that the scan over chunks of one expert reads contiguously.
template <typename IdxT>
__global__ __launch_bounds__(64) void k_plan_hist(const IdxT* __restrict__ idx, int64_t N, int E, int n_chunks,
                                                  int32_t* __restrict__ chunk_hist, int32_t* status) {
    __shared__ int32_t cnt[kMaxExperts];
    const int lane = threadIdx.x;
    const int chunk = blockIdx.x;
    for (int e = lane; e < E; e += 64) cnt[e] = 0;
    __syncthreads();
    const int64_t base = (int64_t)chunk * kPlanChunk;
    for (int it = 0; it < kPlanChunk / 64; ++it) {
        const int64_t i = base + it * 64 + lane;
        if (i < N) atomicAdd(&cnt[load_expert(idx, i, E, status)], 1);
    }
    __syncthreads();
    for (int e = lane; e < E; e += 64) chunk_hist[(size_t)e * n_chunks + chunk] = cnt[e];
}

// One wave per expert: exclusive scan of that expert's per-chunk counts (in place) and its total.
__global__ __launch_bounds__(64) void k_plan_chunkscan(int n_chunks, int32_t* __restrict__ chunk_hist,
                                                       int32_t* __restrict__ counts) {
    const int lane = threadIdx.x;
    int32_t* row = chunk_hist + (size_t)blockIdx.x * n_chunks;
    int carry = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += 64) {
        const int c = c0 + lane;
        const int v = c < n_chunks ? row[c] : 0;
        int incl = v;
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (c < n_chunks) row[c] = carry + incl - v;
        carry += __shfl(incl, 63, 64);
    }
    if (lane == 0) counts[blockIdx.x] = carry;
}

__device__ __forceinline__ void write_tiles(int32_t* tiles, int max_tiles, int first_tile, int e, int row0, int cnt,
                                            int tile_rows) {
    int t = first_tile;
    for (int r = 0; r < cnt; r += tile_rows, ++t) {
        if (t < max_tiles) {
            tiles[t] = e;
            tiles[max_tiles + t] = row0 + r;
            tiles[2 * max_tiles + t] = min(tile_rows, cnt - r);
        }
    }
}

// One workgroup: offsets, experts by descending load, row-tile lists for both tile heights.
__global__ __launch_bounds__(256) void k_plan_finish(int E, const int32_t* __restrict__ counts,
                                                     int32_t* __restrict__ header, int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ by_load, int32_t* __restrict__ tiles_small,
                                                     int max_small, int32_t* __restrict__ tiles_large, int max_large) {
    __shared__ int32_t s_cnt[kMaxExperts];
    __shared__ int32_t s_off[kMaxExperts + 1];
    __shared__ int32_t s_order[kMaxExperts];         // expert id at each load rank
    __shared__ int32_t s_tile0[2][kMaxExperts + 1];  // first tile of each load rank, per tile height
    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += 256) s_cnt[e] = counts[e];
    __syncthreads();
    if (tid == 0) {  // E <= 1024: a serial scan out of LDS is a few microseconds and trivially right
        int run = 0;
        for (int e = 0; e < E; ++e) {
            s_off[e] = run;
            run += s_cnt[e];
        }
        s_off[E] = run;
    }
    __syncthreads();
    for (int e = tid; e <= E; e += 256) offsets[e] = s_off[e];
    // rank experts by load, heaviest first, ties by lower id
    for (int e = tid; e < E; e += 256) {
        const int c = s_cnt[e];
        int rank = 0;
        for (int o = 0; o < E; ++o) {
            const int co = s_cnt[o];
            rank += (co > c) || (co == c && o < e);
        }
        s_order[rank] = e;
        by_load[rank] = e;
    }
    __syncthreads();
    if (tid < 2) {
        const int rows = tid == 0 ? kTileRowsSmall : kTileRowsLarge;
        int run = 0;
        for (int r = 0; r < E; ++r) {
            s_tile0[tid][r] = run;
            run += (s_cnt[s_order[r]] + rows - 1) / rows;
        }
        s_tile0[tid][E] = run;
        header[1 + tid] = run;
    }
    __syncthreads();
    for (int r = tid; r < E; r += 256) {
        const int e = s_order[r];
        write_tiles(tiles_small, max_small, s_tile0[0][r], e, s_off[e], s_cnt[e], kTileRowsSmall);
        write_tiles(tiles_large, max_large, s_tile0[1][r], e, s_off[e], s_cnt[e], kTileRowsLarge);
    }
}

template <typename IdxT>
__global__ __launch_bounds__(64) void k_plan_scatter(const IdxT* __restrict__ idx, int64_t N, int E, int k, int bits,
                                                     int n_chunks, const int32_t* __restrict__ chunk_base,
                                                     const int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ row_to_src, int32_t* __restrict__ src_to_row,
                                                     int32_t* __restrict__ row_token, int32_t* status) {
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
        const int e = valid ? load_expert(idx, i, E, status) : 0;
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
    int32_t* counts = (int32_t*)(b + L.off_counts);
    int32_t* offsets = (int32_t*)(b + L.off_offsets);
    int bits = 0;
    while ((1 << bits) < L.E) ++bits;
    const dim3 grid((unsigned)L.n_chunks), wave(64);
    // the header is cleared by a kernel, not a memset node, so the build can be captured into a HIP graph
    hipLaunchKernelGGL(k_plan_clear, dim3(1), wave, 0, s, header, (int32_t*)(b + L.off_zero));
    if (idx_dtype == 0)
        hipLaunchKernelGGL(k_plan_hist<int32_t>, grid, wave, 0, s, (const int32_t*)idx, L.N, L.E, L.n_chunks, hist, header);
    else
        hipLaunchKernelGGL(k_plan_hist<uint8_t>, grid, wave, 0, s, (const uint8_t*)idx, L.N, L.E, L.n_chunks, hist, header);
    hipLaunchKernelGGL(k_plan_chunkscan, dim3((unsigned)L.E), wave, 0, s, L.n_chunks, hist, counts);
    hipLaunchKernelGGL(k_plan_finish, dim3(1), dim3(256), 0, s, L.E, (const int32_t*)counts, header, offsets,
                       (int32_t*)(b + L.off_by_load), (int32_t*)(b + L.off_tiles_small), L.max_tiles_small,
                       (int32_t*)(b + L.off_tiles_large), L.max_tiles_large);
    if (idx_dtype == 0)
        hipLaunchKernelGGL(k_plan_scatter<int32_t>, grid, wave, 0, s, (const int32_t*)idx, L.N, L.E, L.k, bits,
                           L.n_chunks, (const int32_t*)hist, (const int32_t*)offsets, (int32_t*)(b + L.off_row_to_src),
                           (int32_t*)(b + L.off_src_to_row), (int32_t*)(b + L.off_row_token), header);
    else
        hipLaunchKernelGGL(k_plan_scatter<uint8_t>, grid, wave, 0, s, (const uint8_t*)idx, L.N, L.E, L.k, bits,
                           L.n_chunks, (const int32_t*)hist, (const int32_t*)offsets, (int32_t*)(b + L.off_row_to_src),
                           (int32_t*)(b + L.off_src_to_row), (int32_t*)(b + L.off_row_token), header);
    return hipGetLastError();
}

}  // namespace grouter
