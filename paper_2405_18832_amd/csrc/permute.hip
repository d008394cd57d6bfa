// Dispatch: a deterministic, stable counting sort of the T*k assignments by expert, and the
// gather of token rows into expert-contiguous order (paper Section 2.1: tokens are routed to
// their experts; Section 4.1: drop-less and padding-less, so every assignment gets exactly
// one slot and segments have no padding).
//
// The sort never orders anything through atomics on global memory: assignments are cut into
// chunks of 256 consecutive flat ids, each chunk is counted (kernel 1), the per-expert counts
// are prefix-summed over the chunks (kernel 2), and each chunk then places its assignments
// in flat-id order (kernel 3).  The result is the same on every run.
#include "common.hpp"

namespace moe {

// kernel 1: hist[chunk][e] = number of assignments of expert e inside the chunk
__global__ __launch_bounds__(64) void perm_hist_kernel(const int32_t* __restrict__ idx,
                                                       int32_t* __restrict__ hist, int A, int E) {
    __shared__ int32_t h[MOE_MAX_E];
    for (int e = threadIdx.x; e < E; e += 64) h[e] = 0;
    __syncthreads();
    const int base = blockIdx.x * kPermChunk;
    for (int i = threadIdx.x; i < kPermChunk; i += 64) {
        const int a = base + i;
        if (a < A) atomicAdd(&h[min(max(idx[a], 0), E - 1)], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 64) hist[static_cast<size_t>(blockIdx.x) * E + e] = h[e];
}

// kernel 2: in place, hist[chunk][e] <- sum of hist[c'][e] over chunks c' < chunk.
// One wavefront per expert, lanes strided over the chunks, wave-level inclusive scan.
__global__ __launch_bounds__(64) void perm_scan_kernel(int32_t* __restrict__ hist, int nchunks, int E) {
    const int e = blockIdx.x, lane = threadIdx.x;
    int carry = 0;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
        const int c = c0 + lane;
        const int v = (c < nchunks) ? hist[static_cast<size_t>(c) * E + e] : 0;
        int incl = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const int o = __shfl_up(incl, s);
            if (lane >= s) incl += o;
        }
        if (c < nchunks) hist[static_cast<size_t>(c) * E + e] = carry + incl - v;
        carry += __shfl(incl, 63);
    }
}

// kernel 3: place the chunk's assignments.  The wavefront walks the chunk 64 flat ids at a
// time; lanes that hold the same expert find each other with one ballot per bit of the expert
// id, take consecutive slots in lane order, and the last of them advances the running slot.
__global__ __launch_bounds__(64) void perm_place_kernel(const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ offsets,
                                                        const int32_t* __restrict__ chunk_base,
                                                        int32_t* __restrict__ perm,
                                                        int32_t* __restrict__ inv_perm, int A, int E,
                                                        int ebits) {
    __shared__ int32_t next[MOE_MAX_E];
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64)
        next[e] = offsets[e] + chunk_base[static_cast<size_t>(blockIdx.x) * E + e];
    __syncthreads();
    const int base = blockIdx.x * kPermChunk;
    for (int i0 = 0; i0 < kPermChunk; i0 += 64) {
        const int a = base + i0 + lane;
        const bool live = a < A;
        const int e = live ? min(max(idx[a], 0), E - 1) : 0;   // clamped: a bad index must not fault
        uint64_t same = __ballot(live);
        for (int b = 0; b < ebits; ++b) {
            const uint64_t has = __ballot(live && ((e >> b) & 1));
            same &= ((e >> b) & 1) ? has : ~has;
        }
        const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        const int rank = __popcll(same & below);
        int pos = 0;
        if (live) pos = next[e] + rank;
        __syncthreads();
        const bool last = live && ((same >> lane) >> 1) == 0;   // no higher lane with this expert
        if (last) next[e] = pos + 1;
        __syncthreads();
        if (live && pos >= 0 && pos < A) {   // offsets that do not belong to idx must not fault
            perm[pos] = a;
            inv_perm[a] = pos;
        }
    }
}

// gather: x_perm[p] = x[perm[p] / k]; one wavefront per row, 16 bytes (or 4) per lane and step
template <typename V>
__global__ __launch_bounds__(256) void gather_rows_kernel(const V* __restrict__ x,
                                                          const int32_t* __restrict__ perm,
                                                          V* __restrict__ x_perm, int A, int T, int k,
                                                          int row_vecs) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + wave;
    if (p >= A) return;
    const int t = min(max(perm[p] / k, 0), T - 1);
    const V* src = x + static_cast<size_t>(t) * row_vecs;
    V* dst = x_perm + static_cast<size_t>(p) * row_vecs;
    for (int c = lane; c < row_vecs; c += 64) dst[c] = src[c];
}

hipError_t launch_permute(const moe_shape& s, const void* x, const int32_t* idx,
                          const int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                          int32_t* hist_ws, hipStream_t st) {
    const int A = s.T * s.k, E = s.E;
    const int nchunks = (A + kPermChunk - 1) / kPermChunk;
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    hipLaunchKernelGGL(perm_hist_kernel, dim3(nchunks), dim3(64), 0, st, idx, hist_ws, A, E);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(perm_scan_kernel, dim3(E), dim3(64), 0, st, hist_ws, nchunks, E);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(perm_place_kernel, dim3(nchunks), dim3(64), 0, st, idx, offsets, hist_ws, perm,
                       inv_perm, A, E, ebits);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (x_perm != nullptr) {
        const size_t row_bytes = static_cast<size_t>(s.d_model) * elem_size(s.dtype);
        const unsigned grid = static_cast<unsigned>((A + 3) / 4);
        if (row_bytes % 16 == 0) {
            hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3(grid), dim3(256), 0, st,
                               static_cast<const uint4*>(x), perm, static_cast<uint4*>(x_perm), A, s.T, s.k,
                               static_cast<int>(row_bytes / 16));
        } else if (row_bytes % 4 == 0) {
            hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3(grid), dim3(256), 0, st,
                               static_cast<const uint32_t*>(x), perm, static_cast<uint32_t*>(x_perm), A,
                               s.T, s.k, static_cast<int>(row_bytes / 4));
        } else {
            hipLaunchKernelGGL(gather_rows_kernel<uint16_t>, dim3(grid), dim3(256), 0, st,
                               static_cast<const uint16_t*>(x), perm, static_cast<uint16_t*>(x_perm), A,
                               s.T, s.k, static_cast<int>(row_bytes / 2));
        }
        err = hipGetLastError();
    }
    return err;
}

}  // namespace moe
