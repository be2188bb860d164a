// Permute / dispatch (gather token rows into expert-sorted order) and combine / un-permute (gate-weighted
// k-way sum back into token order): the two memory-bound ends of Eq. 1's sparse evaluation.
//
// Both move whole rows of d bf16 values and both walk the token side (the [T][d] tensor) in order, so the
// small tensor is streamed once and the k-fold fan-out / fan-in goes to whole rows of the big one.  A
// workgroup first stages the indices and gate weights of its group of tokens in LDS (one coalesced read
// instead of one dependent scalar read per lane), then streams the payload as 16-byte lanes: consecutive
// lanes cover consecutive 16-byte pieces of one row, so every global access is a full contiguous row
// segment.  The payload itself does not pass through LDS - rows are at least 16 bytes wide and already
// contiguous, so staging them would only add latency.
#include "common.hpp"

namespace grouter {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }
// fp32 pair -> packed bf16 pair, round-to-nearest-even (inputs are finite)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7fffu + ((ua >> 16) & 1u);
    ub += 0x7fffu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xffff0000u);
}

constexpr int kDispatchTokens = 8;   // tokens per workgroup
constexpr int kMaxStagedSlots = 512;  // tokens-per-workgroup * k staged per workgroup; larger k reads indices from global

// out[src_to_row[t*k+j]][:] = s_{t,j} * in[t][:],  s = 1 or gate_w[t*k+j].
// Token-major: every source row is read once and written to its k destinations, so the source is fetched
// from HBM once instead of once per XCD that happens to own one of its destinations.
template <bool SCALE>
__global__ __launch_bounds__(256) void k_permute(const PlanDims plan, const int32_t* __restrict__ src_to_row,
                                                 const bf16_t* __restrict__ gate_w, int64_t T, int k, int chunks_per_row,
                                                 const u32x4* __restrict__ in, u32x4* __restrict__ out) {
    __shared__ int32_t s_row[kMaxStagedSlots];
    __shared__ float s_w[kMaxStagedSlots];
    if (!plan.match()) return;
    const int64_t t0 = (int64_t)blockIdx.x * kDispatchTokens;
    const int toks = (int)min((int64_t)kDispatchTokens, T - t0);
    const bool staged = kDispatchTokens * k <= kMaxStagedSlots;
    if (staged) {
        for (int i = threadIdx.x; i < toks * k; i += 256) {
            s_row[i] = src_to_row[t0 * k + i];
            if (SCALE) s_w[i] = __uint_as_float((uint32_t)gate_w[t0 * k + i] << 16);
        }
    }
    __syncthreads();
    const int total = toks * chunks_per_row;
    for (int c = threadIdx.x; c < total; c += 256) {
        const int r = c / chunks_per_row;
        const int q = c - r * chunks_per_row;
        const u32x4 v = in[(size_t)(t0 + r) * chunks_per_row + q];
        for (int j = 0; j < k; ++j) {
            int row;
            float w = 1.f;
            if (staged) {
                row = s_row[r * k + j];
                if (SCALE) w = s_w[r * k + j];
            } else {
                row = src_to_row[(t0 + r) * k + j];
                if (SCALE) w = __uint_as_float((uint32_t)gate_w[(t0 + r) * k + j] << 16);
            }
            u32x4 o = v;
            if (SCALE) {
                o.x = pack_bf16(w * bf16_lo(v.x), w * bf16_hi(v.x));
                o.y = pack_bf16(w * bf16_lo(v.y), w * bf16_hi(v.y));
                o.z = pack_bf16(w * bf16_lo(v.z), w * bf16_hi(v.z));
                o.w = pack_bf16(w * bf16_lo(v.w), w * bf16_hi(v.w));
            }
            out[(size_t)row * chunks_per_row + q] = o;
        }
    }
}

// Tokens per workgroup of the combine: as few as give every thread one 16-byte piece (one token for rows of
// 4 KB and more) - many small workgroups keep more independent row reads in flight than few large ones
// (measured on 8192 x 2048, k = 6, input fresh from the GEMM before: 8 tokens 4.9 TB/s, 1 token 5.7 TB/s).
static inline int combine_tokens_per_block(int chunks_per_row) {
    const int t = 256 / (chunks_per_row > 0 ? chunks_per_row : 1);
    return t < 1 ? 1 : (t > 16 ? 16 : t);
}

// out[t][:] = sum_j s_{t,j} * in[src_to_row[t*k+j]][:]   (fp32, j ascending)
template <bool SCALE>
__global__ __launch_bounds__(256) void k_combine(const PlanDims plan, const int32_t* __restrict__ src_to_row,
                                                 const bf16_t* __restrict__ gate_w, int64_t T, int k, int chunks_per_row,
                                                 int tokens_per_block, const u32x4* __restrict__ in,
                                                 u32x4* __restrict__ out) {
    __shared__ int32_t s_row[kMaxStagedSlots];
    __shared__ float s_w[kMaxStagedSlots];
    if (!plan.match()) return;
    const int64_t t0 = (int64_t)blockIdx.x * tokens_per_block;
    const int toks = (int)min((int64_t)tokens_per_block, T - t0);
    const bool staged = tokens_per_block * k <= kMaxStagedSlots;
    if (staged) {
        for (int i = threadIdx.x; i < toks * k; i += 256) {
            s_row[i] = src_to_row[t0 * k + i];
            if (SCALE) s_w[i] = __uint_as_float((uint32_t)gate_w[t0 * k + i] << 16);
        }
    }
    __syncthreads();
    const int total = toks * chunks_per_row;
    for (int c = threadIdx.x; c < total; c += 256) {
        const int r = c / chunks_per_row;
        const int q = c - r * chunks_per_row;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < k; ++j) {
            int row;
            float w = 1.f;
            if (staged) {
                row = s_row[r * k + j];
                if (SCALE) w = s_w[r * k + j];
            } else {
                row = src_to_row[(t0 + r) * k + j];
                if (SCALE) w = __uint_as_float((uint32_t)gate_w[(t0 + r) * k + j] << 16);
            }
            const u32x4 v = __builtin_nontemporal_load(in + (size_t)row * chunks_per_row + q);   // each row is read once
            acc[0] += w * bf16_lo(v.x); acc[1] += w * bf16_hi(v.x);
            acc[2] += w * bf16_lo(v.y); acc[3] += w * bf16_hi(v.y);
            acc[4] += w * bf16_lo(v.z); acc[5] += w * bf16_hi(v.z);
            acc[6] += w * bf16_lo(v.w); acc[7] += w * bf16_hi(v.w);
        }
        u32x4 o;
        o.x = pack_bf16(acc[0], acc[1]);
        o.y = pack_bf16(acc[2], acc[3]);
        o.z = pack_bf16(acc[4], acc[5]);
        o.w = pack_bf16(acc[6], acc[7]);
        out[(size_t)(t0 + r) * chunks_per_row + q] = o;
    }
}

// row_gate[p] = gate_w[row_to_src[p]] widened to fp32: the routing weight of the slot behind each
// expert-sorted row, laid out the way the GEMM epilogues read it.
__global__ __launch_bounds__(256) void k_row_gates(const PlanDims plan, const int32_t* __restrict__ row_to_src,
                                                   const bf16_t* __restrict__ gate_w, int64_t N, float* __restrict__ row_gate) {
    if (!plan.match()) return;
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p < N) row_gate[p] = __uint_as_float((uint32_t)gate_w[row_to_src[p]] << 16);
}

hipError_t launch_row_gates(const PlanView& P, const bf16_t* gate_w, float* row_gate, hipStream_t s) {
    hipLaunchKernelGGL(k_row_gates, dim3((unsigned)((P.N + 255) / 256)), dim3(256), 0, s, P.dims(), P.row_to_src, gate_w, P.N, row_gate);
    return hipGetLastError();
}

hipError_t launch_permute(const PlanView& P, int d, const bf16_t* in, const bf16_t* gate_w, bf16_t* out, hipStream_t s) {
    const unsigned blocks = (unsigned)((P.T + kDispatchTokens - 1) / kDispatchTokens);
    if (gate_w)
        hipLaunchKernelGGL(k_permute<true>, dim3(blocks), dim3(256), 0, s, P.dims(), P.src_to_row, gate_w, P.T, P.k, d / 8,
                           (const u32x4*)in, (u32x4*)out);
    else
        hipLaunchKernelGGL(k_permute<false>, dim3(blocks), dim3(256), 0, s, P.dims(), P.src_to_row, gate_w, P.T, P.k, d / 8,
                           (const u32x4*)in, (u32x4*)out);
    return hipGetLastError();
}

hipError_t launch_combine(const PlanView& P, int d, const bf16_t* in, const bf16_t* gate_w, bf16_t* out, hipStream_t s) {
    const int tpb = combine_tokens_per_block(d / 8);
    const unsigned blocks = (unsigned)((P.T + tpb - 1) / tpb);
    if (gate_w)
        hipLaunchKernelGGL(k_combine<true>, dim3(blocks), dim3(256), 0, s, P.dims(), P.src_to_row, gate_w, P.T, P.k, d / 8,
                           tpb, (const u32x4*)in, (u32x4*)out);
    else
        hipLaunchKernelGGL(k_combine<false>, dim3(blocks), dim3(256), 0, s, P.dims(), P.src_to_row, gate_w, P.T, P.k, d / 8,
                           tpb, (const u32x4*)in, (u32x4*)out);
    return hipGetLastError();
}

}  // namespace grouter
