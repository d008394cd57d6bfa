// Dispatch: a deterministic, stable counting sort of the T*k assignments by expert, and the
// gather of token rows into expert-contiguous order (paper Section 2.1: tokens are routed to
// their experts; Section 4.1: drop-less and padding-less, so every assignment gets exactly
// one slot and segments have no padding).
//
// The sort never orders anything through atomics on global memory: assignments are cut into
// chunks of consecutive flat ids, each chunk is counted (kernel 1, or the routing kernel when
// the whole layer runs), the per-expert counts are prefix-summed over the chunks (kernel 2),
// and each chunk then places its assignments in flat-id order (kernel 3).  The result is the
// same on every run.
#include "common.hpp"

namespace moe {

// kernel 1: hist[chunk][e] = number of assignments of expert e inside the chunk.
// One wavefront per chunk, 4 chunks per block.
__global__ __launch_bounds__(256) void perm_hist_kernel(const int32_t* __restrict__ idx,
                                                        int32_t* __restrict__ hist, int A, int E,
                                                        int chunk, int nchunks) {
    __shared__ int32_t h[4][MOE_MAX_E];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + wave;
    for (int e = lane; e < E; e += 64) h[wave][e] = 0;
    __syncthreads();
    if (c < nchunks) {
        const int base = c * chunk;
        for (int i = lane; i < chunk; i += 64) {
            const int a = base + i;
            if (a < A) atomicAdd(&h[wave][min(max(idx[a], 0), E - 1)], 1);
        }
    }
    __syncthreads();
    if (c < nchunks)
        for (int e = lane; e < E; e += 64) hist[static_cast<size_t>(c) * E + e] = h[wave][e];
}

// kernel 3: place the chunk's assignments (kernel 2, the prefix sum over chunks, is
// scan_finalize_kernel).  The wavefront walks its chunk 64 flat ids at a time; lanes that hold
// the same expert find each other with one ballot per bit of the expert id, take consecutive
// slots in lane order, and the last of them advances the expert's running slot.
// Writes (each may be NULL) perm[pos] = a, inv_perm[a] = pos, tokmap[pos] = a / k.
__global__ __launch_bounds__(256) void perm_place_kernel(const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ offsets,
                                                         const int32_t* __restrict__ chunk_base,
                                                         int32_t* __restrict__ perm,
                                                         int32_t* __restrict__ inv_perm,
                                                         int32_t* __restrict__ tokmap, int A, int E, int k,
                                                         int ebits, int chunk, int nchunks) {
    __shared__ int32_t next_all[4][MOE_MAX_E];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + wave;
    if (c >= nchunks) return;                   // no block-wide barrier below: waves are independent
    int32_t* next = next_all[wave];
    for (int e = lane; e < E; e += 64) next[e] = offsets[e] + chunk_base[static_cast<size_t>(c) * E + e];
    __builtin_amdgcn_wave_barrier();
    place_chunk(idx, next, perm, inv_perm, tokmap, A, E, k, ebits, chunk, c);
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

// gather into the blocked layout of the products' row operand (h_index): element (p, c) of xk is
// x[tokmap[p]][c] (tokmap may be NULL: identity).  One thread per 16 bytes.  Eight consecutive threads take the
// 128 bytes of one row that make up two k-steps, so every line of a token row is fetched whole and once (with
// one k-step per group of four threads the two halves of a line were read by blocks on different XCDs, and the
// kernel fetched twice its input); a wavefront then writes two runs of 512 contiguous bytes, the same eight rows
// of both k-steps.  The rows past A of the last row block stay unwritten.
__global__ __launch_bounds__(256) void gather_kmajor_kernel(const uint4* __restrict__ x,
                                                            const int32_t* __restrict__ tokmap,
                                                            uint4* __restrict__ xk, int A, int T, int row_vecs,
                                                            size_t total) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= total) return;
    // thread order: [row block][pair of k-steps][row in block][8 pieces of 16 bytes: 4 of each k-step]
    const int piece = static_cast<int>(i & 7);
    const int r = static_cast<int>((i >> 3) & (kRowBlock - 1));
    const size_t bk = i >> 11;                          // row block * kpairs + pair
    const int ksteps = row_vecs >> 2, kpairs = (ksteps + 1) >> 1;
    const int kb = static_cast<int>(bk % kpairs) * 2 + (piece >> 2), c = piece & 3;
    const size_t rb = bk / kpairs;
    const size_t p = rb * kRowBlock + r;
    if (p >= static_cast<size_t>(A) || kb >= ksteps) return;
    const int t = tokmap ? min(max(tokmap[p], 0), T - 1) : static_cast<int>(p);   // no map: x already has the A rows in order
    xk[((rb * ksteps + kb) * kRowBlock + r) * 4 + c] = x[static_cast<size_t>(t) * row_vecs + kb * 4 + c];
}

hipError_t launch_gather_kmajor(const moe_shape& s, const void* x, const int32_t* tokmap, void* xk, hipStream_t st) {
    const int A = s.T * s.k;
    const size_t Ab = (static_cast<size_t>(A) + kRowBlock - 1) / kRowBlock * kRowBlock;
    const size_t ksteps = static_cast<size_t>(s.d_model) / 32;
    const size_t total = Ab * ((ksteps + 1) / 2) * 8;                 // one thread per 16 bytes, k-steps in pairs
    hipLaunchKernelGGL(gather_kmajor_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint4*>(x), tokmap, static_cast<uint4*>(xk), A, s.T, s.d_model / 8, total);
    return hipGetLastError();
}

hipError_t launch_place(const moe_shape& s, const int32_t* idx, const int32_t* offsets, const int32_t* chunk_base,
                        int32_t* perm, int32_t* inv_perm, int32_t* tokmap, int chunk, hipStream_t st) {
    const int A = s.T * s.k, E = s.E;
    const int nchunks = (A + chunk - 1) / chunk;
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    hipLaunchKernelGGL(perm_place_kernel, dim3((nchunks + 3) / 4), dim3(256), 0, st, idx, offsets, chunk_base, perm,
                       inv_perm, tokmap, A, E, s.k, ebits, chunk, nchunks);
    return hipGetLastError();
}

hipError_t launch_gather(const moe_shape& s, const void* x, const int32_t* perm, void* x_perm, hipStream_t st) {
    const int A = s.T * s.k;
    const size_t row_bytes = static_cast<size_t>(s.d_model) * elem_size(s.dtype);
    const unsigned grid = static_cast<unsigned>((A + 3) / 4);
    if (row_bytes % 16 == 0) {
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3(grid), dim3(256), 0, st, static_cast<const uint4*>(x), perm,
                           static_cast<uint4*>(x_perm), A, s.T, s.k, static_cast<int>(row_bytes / 16));
    } else {
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3(grid), dim3(256), 0, st,
                           static_cast<const uint32_t*>(x), perm, static_cast<uint32_t*>(x_perm), A, s.T, s.k,
                           static_cast<int>(row_bytes / 4));
    }
    return hipGetLastError();
}

hipError_t launch_permute(const moe_shape& s, const void* x, const int32_t* idx,
                          const int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                          int32_t* hist_ws, hipStream_t st) {
    const int A = s.T * s.k, E = s.E;
    const int nchunks = (A + kPermChunk - 1) / kPermChunk;
    hipLaunchKernelGGL(perm_hist_kernel, dim3((nchunks + 3) / 4), dim3(256), 0, st, idx, hist_ws, A, E, kPermChunk,
                       nchunks);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    err = launch_scan_finalize(hist_ws, nchunks, E, nullptr, nullptr, -1, nullptr, nullptr, nullptr, nullptr, st);
    if (err != hipSuccess) return err;
    err = launch_place(s, idx, offsets, hist_ws, perm, inv_perm, nullptr, kPermChunk, st);
    if (err != hipSuccess) return err;
    if (x_perm != nullptr) err = launch_gather(s, x, perm, x_perm, st);
    return err;
}

}  // namespace moe
