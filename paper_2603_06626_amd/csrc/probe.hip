// Matrix-core ceiling probe: the MFMA instruction stream of the GEMM main loops with nothing else around it.
//
// Every wave runs `iters` steps of 8 independent v_mfma_f32_32x32x16_bf16 (2 x 4 fragments: the shape of one
// K=16 half step of the grouped GEMMs) on pseudo-random operands, so the measured rate is what the chip's
// power limit and clocks allow for this instruction mix, not a data-sheet number.
//   mode 0: operand fragments stay in registers (matrix cores alone);
//   mode 1: the 6 operand fragments of every step are read again from LDS with 16-byte reads, as the GEMM
//           main loops do (matrix cores + LDS reads, still no global-memory traffic);
//   modes 2, 3: as 0 and 1 with v_mfma_f32_16x16x32_bf16 on the same wave tile (iters must be even);
//   modes 4, 5: no MFMAs at all, only LDS fragment reads (16-byte reads / transposing 8-byte pairs with the
//               N-contiguous tiles' own address pattern), 6 KB per wave and step;
//   modes 6, 7: as 2 and 3 with a 128 x 128 wave tile: 256 accumulator registers, one wave per SIMD (iters % 4 == 0).
// The result written to `out` only keeps the accumulators alive.
#include "gemm.hpp"

namespace grouter {
namespace {

constexpr int kProbeLdsWords = 12288;   // 48 KB per workgroup: two workgroups per CU, as in the GEMMs

__device__ __forceinline__ uint32_t probe_hash(uint32_t v) {
    v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
    return v;
}
// two bf16 values with random sign and mantissa and magnitude in [0.5, 1)
__device__ __forceinline__ uint32_t probe_bf16_pair(uint32_t v) { return (probe_hash(v) & 0x807f807fu) | 0x3f003f00u; }

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_mfma_probe(int iters, float* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kProbeLdsWords];
    const int tid = threadIdx.x;
    for (int i = tid; i < kProbeLdsWords; i += kThreads) lds[i] = probe_bf16_pair(i * 2654435761u + blockIdx.x);
    __syncthreads();
    const char* base = (const char*)lds;
    const uint32_t lane_off = (uint32_t)(tid & 63) * 16u + (uint32_t)(tid >> 6) * 12288u;
    auto frag = [&](uint32_t piece) {
        const uint32_t off = (lane_off + piece * 1024u) % (uint32_t)(kProbeLdsWords * 4);
        return *(const bf16x8*)(base + off);
    };
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bf16x8 a[2], b[4];
    a[0] = frag(0); a[1] = frag(1);
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = frag(2 + j);
    uint32_t piece = 6;
#pragma unroll 2
    for (int it = 0; it < iters; ++it) {
        bf16x8 na[2], nb[4];
        if (MODE == 1) {   // next step's fragments are requested before this step's MFMAs, as in the GEMM pipeline
            na[0] = frag(piece); na[1] = frag(piece + 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) nb[j] = frag(piece + 2 + j);
            piece = (piece + 6) % 48u;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        if (MODE == 1) {
            a[0] = na[0]; a[1] = na[1];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = nb[j];
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
    out[(size_t)blockIdx.x * kThreads + tid] = sum;
}

// The same work per step from v_mfma_f32_16x16x32_bf16: a 64 x 128 wave tile is 4 x 8 fragments of 16 x 16, one
// K=32 step is 32 MFMAs fed by 12 fragments (two steps of the 32x32x16 form: 16 MFMAs, 12 fragments).
template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_mfma_probe16(int iters, float* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kProbeLdsWords];
    const int tid = threadIdx.x;
    for (int i = tid; i < kProbeLdsWords; i += kThreads) lds[i] = probe_bf16_pair(i * 2654435761u + blockIdx.x);
    __syncthreads();
    const char* base = (const char*)lds;
    const uint32_t lane_off = (uint32_t)(tid & 63) * 16u + (uint32_t)(tid >> 6) * 12288u;
    auto frag = [&](uint32_t piece) {
        const uint32_t off = (lane_off + piece * 1024u) % (uint32_t)(kProbeLdsWords * 4);
        return *(const bf16x8*)(base + off);
    };
    f32x4 acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    bf16x8 a[4], b[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = frag(i);
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = frag(4 + j);
    uint32_t piece = 12;
    for (int it = 0; it < iters; it += 2) {   // one pass = two steps of the 32x32x16 probe
        bf16x8 na[4], nb[8];
        if (MODE == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i) na[i] = frag(piece + i);
#pragma unroll
            for (int j = 0; j < 8; ++j) nb[j] = frag(piece + 4 + j);
            piece = (piece + 12) % 48u;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        if (MODE == 1) {
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = na[i];
#pragma unroll
            for (int j = 0; j < 8; ++j) b[j] = nb[j];
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum += acc[i][j][v];
    out[(size_t)blockIdx.x * kThreads + tid] = sum;
}

// One wave per SIMD with a 128 x 128 wave tile (256 accumulator registers): 64 MFMAs of 16x16x32 per K = 32 step
// fed by 16 fragments of 16 bytes per lane.  MODE 0: operands in registers; MODE 1: re-read from LDS every step.
template <int MODE>
__global__ __launch_bounds__(kThreads, 1) void k_mfma_probe_big(int iters, float* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kProbeLdsWords];
    const int tid = threadIdx.x;
    for (int i = tid; i < kProbeLdsWords; i += kThreads) lds[i] = probe_bf16_pair(i * 2654435761u + blockIdx.x);
    __syncthreads();
    const char* base = (const char*)lds;
    const uint32_t lane_off = (uint32_t)(tid & 63) * 16u + (uint32_t)(tid >> 6) * 12288u;
    auto frag = [&](uint32_t piece) {
        const uint32_t off = (lane_off + piece * 1024u) % (uint32_t)(kProbeLdsWords * 4);
        return *(const bf16x8*)(base + off);
    };
    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = frag(i); b[i] = frag(8 + i); }
    uint32_t piece = 16;
    for (int it = 0; it < iters; it += 4) {   // one pass = four steps of the small probes (64 MFMAs of 16x16x32)
        bf16x8 na[8], nb[8];
        if (MODE == 1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { na[i] = frag(piece + i); nb[i] = frag(piece + 8 + i); }
            piece = (piece + 16) % 48u;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        if (MODE == 1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { a[i] = na[i]; b[i] = nb[i]; }
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) sum += acc[i][j][v];
    out[(size_t)blockIdx.x * kThreads + tid] = sum;
}

// LDS read rate alone: every wave reads `iters` x 6 KB of operand fragments and folds them into one register.
//   TR = false: 16-byte reads, 1 KB per wave and read, linear addresses (the K-contiguous tiles' fragment reads);
//   TR = true:  pairs of transposing 8-byte reads with the address pattern and swizzle of the [32][256]
//               N-contiguous tile (McTile<256>): 6 half fragments of 16 columns per iteration over three tiles.
template <bool TR>
__global__ __launch_bounds__(kThreads, 2) void k_lds_read_probe(int iters, float* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint32_t lds[kProbeLdsWords];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < kProbeLdsWords; i += kThreads) lds[i] = probe_bf16_pair(i * 2654435761u + blockIdx.x);
    __syncthreads();
    const char* base = (const char*)lds;
    const uint32_t lane_off = (uint32_t)lane * 16u + (uint32_t)wave * 12288u;
    const uint32_t mc_lane = McTile<256>::lane_base(lane) ^ McTile<256>::column_bits(wave * 64);
    u32x4 fold = {0u, 0u, 0u, 0u};
    uint32_t piece = 0;
#pragma unroll 2
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 6; ++j) {
            if constexpr (TR) {
                // tile (piece / 6 + j / 4) % 3, column block j % 4 of this wave's 64 columns
                const uint32_t off = (mc_lane ^ McTile<256>::column_bits((j & 3) * 16)) + ((piece / 6 + (j >> 2)) % 3u) * 16384u;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(base + off));
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)(base + off + 4 * 512));
                const u32x2 a = __builtin_bit_cast(u32x2, lo), b = __builtin_bit_cast(u32x2, hi);
                fold.x ^= a.x; fold.y ^= a.y; fold.z ^= b.x; fold.w ^= b.y;
            } else {
                const uint32_t off = (lane_off + (piece + j) * 1024u) % (uint32_t)(kProbeLdsWords * 4);
                const u32x4 v = *(const u32x4*)(base + off);
                fold.x ^= v.x; fold.y ^= v.y; fold.z ^= v.z; fold.w ^= v.w;
            }
        }
        piece = (piece + 6) % 48u;
    }
    out[(size_t)blockIdx.x * kThreads + tid] = __uint_as_float((fold.x ^ fold.y ^ fold.z ^ fold.w) & 0x3f7fffffu);
}

}  // namespace

hipError_t launch_mfma_probe(int mode, int iters, int workgroups, float* out, hipStream_t s) {
    switch (mode) {
        case 0: hipLaunchKernelGGL(k_mfma_probe<0>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        case 1: hipLaunchKernelGGL(k_mfma_probe<1>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        case 2: hipLaunchKernelGGL(k_mfma_probe16<0>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        case 3: hipLaunchKernelGGL(k_mfma_probe16<1>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        case 4: hipLaunchKernelGGL(k_lds_read_probe<false>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        case 5: hipLaunchKernelGGL(k_lds_read_probe<true>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        case 6: hipLaunchKernelGGL(k_mfma_probe_big<0>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
        default: hipLaunchKernelGGL(k_mfma_probe_big<1>, dim3(workgroups), dim3(kThreads), 0, s, iters, out); break;
    }
    return hipGetLastError();
}

}  // namespace grouter
