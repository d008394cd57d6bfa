// Gating and routing: logits = x . w_gate^T (+ bias), softmax over experts, top-k with
// lowest-index tie-break, gate weights, per-expert token histogram, prefix sums and the
// top-H hot mask (paper Section 2.1 for the gating network, Section 3.3 for the token
// counts and the hot set).
#include "common.hpp"

namespace moe {

// ---------------------------------------------------------------------------
// logits, bf16 storage: MFMA 16x16x32 with the gate rows as the A operand and the token
// rows as the B operand, so a lane ends up with 4 consecutive experts of one token.
// Block = 4 wavefronts on the same 16*TF tokens; wave w takes experts [64w, 64w+64) of
// every 256-expert chunk.  Operands come straight from global memory (the gate matrix is
// L2-resident, x is read once).
// ---------------------------------------------------------------------------
template <int TF>
__global__ __launch_bounds__(256) void gate_logits_bf16_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
    const float* __restrict__ bias, float* __restrict__ logits, int32_t* __restrict__ counts,
    int T, int d, int E) {
    if (blockIdx.x == 0)
        for (int e = threadIdx.x; e < E; e += blockDim.x) counts[e] = 0;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * (16 * TF);
    const uint16_t* xrow[TF];
#pragma unroll
    for (int tf = 0; tf < TF; ++tf) {
        int t = min(t0 + tf * 16 + r, T - 1);
        xrow[tf] = x + static_cast<size_t>(t) * d + g * 8;
    }
    for (int ec = 0; ec < E; ec += 256) {
        const int eb = ec + wave * 64;
        if (eb >= E) continue;
        const uint16_t* wrow[4];
#pragma unroll
        for (int nf = 0; nf < 4; ++nf) {
            int e = min(eb + nf * 16 + r, E - 1);
            wrow[nf] = wg + static_cast<size_t>(e) * d + g * 8;
        }
        f32x4 acc[4][TF];
#pragma unroll
        for (int nf = 0; nf < 4; ++nf)
#pragma unroll
            for (int tf = 0; tf < TF; ++tf) acc[nf][tf] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
        for (int k0 = 0; k0 < d; k0 += 32) {
            bf16x8 a[4], b[TF];
#pragma unroll
            for (int nf = 0; nf < 4; ++nf) a[nf] = *reinterpret_cast<const bf16x8*>(wrow[nf] + k0);
#pragma unroll
            for (int tf = 0; tf < TF; ++tf) b[tf] = *reinterpret_cast<const bf16x8*>(xrow[tf] + k0);
#pragma unroll
            for (int nf = 0; nf < 4; ++nf)
#pragma unroll
                for (int tf = 0; tf < TF; ++tf)
                    acc[nf][tf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[nf], b[tf], acc[nf][tf], 0, 0, 0);
        }
#pragma unroll
        for (int tf = 0; tf < TF; ++tf) {
            const int t = t0 + tf * 16 + r;
            if (t >= T) continue;
#pragma unroll
            for (int nf = 0; nf < 4; ++nf)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = eb + nf * 16 + g * 4 + i;
                    if (e < E) logits[static_cast<size_t>(t) * E + e] = acc[nf][tf][i] + (bias ? bias[e] : 0.f);
                }
        }
    }
}

// logits, fp32 storage: one thread per (token, expert), sequential fp32 FMA over d.
__global__ void gate_logits_f32_kernel(const float* __restrict__ x, const float* __restrict__ wg,
                                       const float* __restrict__ bias, float* __restrict__ logits,
                                       int32_t* __restrict__ counts, int T, int d, int E) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (blockIdx.x == 0)
        for (int e = threadIdx.x; e < E; e += blockDim.x) counts[e] = 0;
    if (i >= static_cast<size_t>(T) * E) return;
    const int t = static_cast<int>(i / E), e = static_cast<int>(i % E);
    const float* xr = x + static_cast<size_t>(t) * d;
    const float* wr = wg + static_cast<size_t>(e) * d;
    float s = 0.f;
    for (int c = 0; c < d; ++c) s = fmaf(xr[c], wr[c], s);
    logits[i] = s + (bias ? bias[e] : 0.f);
}

// ---------------------------------------------------------------------------
// softmax + top-k: one wavefront per token, lanes strided over the experts.  k+1 rounds
// of a (value, index) arg-max across the wave; on equal values the lower index wins, in
// the lane-local scan and in every exchange, so the order is exactly "descending logit,
// ties by lowest expert index".  Token counts go through an LDS histogram per block and
// one integer atomic per non-empty bin.
// ---------------------------------------------------------------------------
constexpr int kRouteTokensPerBlock = 64;

__global__ __launch_bounds__(256) void softmax_topk_kernel(
    const float* __restrict__ logits, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ margin, int32_t* __restrict__ counts, int T, int E, int k, int renorm) {
    __shared__ int32_t hist[MOE_MAX_E];
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist[e] = 0;
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tbeg = blockIdx.x * kRouteTokensPerBlock;
    const int tend = min(T, tbeg + kRouteTokensPerBlock);
    constexpr int C = MOE_MAX_E / 64;
    const float NEG = -__builtin_huge_valf();
    for (int t = tbeg + wave; t < tend; t += 4) {
        float v[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int e = lane + 64 * c;
            v[c] = (e < E) ? logits[static_cast<size_t>(t) * E + e] : NEG;
        }
        float sel_v[MOE_MAX_K + 1];
        int sel_i[MOE_MAX_K + 1];
        const int rounds = min(k + 1, E);
        float vmax = 0.f, denom = 0.f;
        for (int j = 0; j < rounds; ++j) {
            float bv = NEG;
            int bi = 0x7fffffff;
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const int e = lane + 64 * c;
                if (e < E && (v[c] > bv || bi == 0x7fffffff)) { bv = v[c]; bi = e; }
            }
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1) {
                const float ov = __shfl_xor(bv, s);
                const int oi = __shfl_xor(bi, s);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            sel_v[j] = bv;
            sel_i[j] = min(bi, E - 1);   // NaN logits must not produce an out-of-range expert
            if (j == 0) {
                vmax = bv;
                float part = 0.f;
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if (lane + 64 * c < E) part += expf(v[c] - vmax);
#pragma unroll
                for (int s = 32; s >= 1; s >>= 1) part += __shfl_xor(part, s);
                denom = part;
            }
            // retire the winner: its owner lane drops it from later rounds
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (lane + 64 * c == bi) v[c] = NEG;
        }
        if (lane == 0) {
            float p[MOE_MAX_K];
            float psum = 0.f;
            for (int j = 0; j < k; ++j) {
                p[j] = expf(sel_v[j] - vmax) / denom;
                psum += p[j];
            }
            for (int j = 0; j < k; ++j) {
                topk_idx[static_cast<size_t>(t) * k + j] = sel_i[j];
                topk_w[static_cast<size_t>(t) * k + j] = renorm ? p[j] / psum : p[j];
                atomicAdd(&hist[sel_i[j]], 1);
            }
            if (margin) {
                float m = __builtin_huge_valf();
                for (int j = 0; j + 1 < rounds; ++j) m = fminf(m, sel_v[j] - sel_v[j + 1]);
                margin[t] = m;
            }
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x)
        if (hist[e] != 0) atomicAdd(&counts[e], hist[e]);
}

// ---------------------------------------------------------------------------
// prefix sums of the counts and the top-H hot mask (rank by count, ties by lowest index).
// One block of 1024 threads, one thread per expert.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void route_finalize_kernel(const int32_t* __restrict__ counts,
                                                              int32_t* __restrict__ offsets,
                                                              uint8_t* __restrict__ hot_mask, int E,
                                                              int H) {
    __shared__ int32_t c[MOE_MAX_E];
    __shared__ int32_t scan[MOE_MAX_E];
    const int e = threadIdx.x;
    const int mine = (e < E) ? counts[e] : 0;
    c[e] = mine;
    scan[e] = mine;
    __syncthreads();
    for (int s = 1; s < MOE_MAX_E; s <<= 1) {
        const int add = (e >= s) ? scan[e - s] : 0;
        __syncthreads();
        scan[e] += add;
        __syncthreads();
    }
    if (e < E) offsets[e] = scan[e] - mine;
    if (e == E - 1) offsets[E] = scan[e];
    if (hot_mask != nullptr && H >= 0 && e < E) {
        int rank = 0;
        for (int o = 0; o < E; ++o) rank += (c[o] > mine || (c[o] == mine && o < e)) ? 1 : 0;
        hot_mask[e] = rank < H ? 1 : 0;
    }
}

__global__ void mask_out_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int E) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) dst[e] = src ? (src[e] ? 1 : 0) : 1;
}

hipError_t launch_mask_out(const uint8_t* mask_or_null, uint8_t* dst, int E, hipStream_t st) {
    hipLaunchKernelGGL(mask_out_kernel, dim3((E + 255) / 256), dim3(256), 0, st, mask_or_null, dst, E);
    return hipGetLastError();
}

__global__ void zero_i32_kernel(int32_t* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_route(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                        int32_t* idx, float* gate, float* margin, int32_t* counts,
                        int32_t* offsets, int32_t H, uint8_t* hot_mask, float* logits_ws,
                        hipStream_t st) {
    const int T = s.T, d = s.d_model, E = s.E;
    if (T == 0) {   // no tokens: all counts and offsets are zero
        hipLaunchKernelGGL(zero_i32_kernel, dim3((E + 255) / 256), dim3(256), 0, st, counts, E);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
        hipLaunchKernelGGL(route_finalize_kernel, dim3(1), dim3(1024), 0, st, counts, offsets, hot_mask, E, H);
        return hipGetLastError();
    }
    if (s.dtype == MOE_BF16) {
        if (T >= 1024) {
            hipLaunchKernelGGL(gate_logits_bf16_kernel<4>, dim3((T + 63) / 64), dim3(256), 0, st,
                               static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_gate),
                               bias, logits_ws, counts, T, d, E);
        } else {
            hipLaunchKernelGGL(gate_logits_bf16_kernel<1>, dim3((T + 15) / 16), dim3(256), 0, st,
                               static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_gate),
                               bias, logits_ws, counts, T, d, E);
        }
    } else {
        const size_t n = static_cast<size_t>(T) * E;
        hipLaunchKernelGGL(gate_logits_f32_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256),
                           0, st, static_cast<const float*>(x), static_cast<const float*>(w_gate), bias,
                           logits_ws, counts, T, d, E);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(softmax_topk_kernel,
                       dim3((T + kRouteTokensPerBlock - 1) / kRouteTokensPerBlock), dim3(256), 0, st,
                       logits_ws, idx, gate, margin, counts, T, E, s.k, s.renormalize);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(route_finalize_kernel, dim3(1), dim3(1024), 0, st, counts, offsets, hot_mask, E, H);
    return hipGetLastError();
}

}  // namespace moe
