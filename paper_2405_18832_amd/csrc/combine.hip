// Combine: weight each token's expert outputs by its gate weights, sum them and store the
// result at the token's original position (paper Section 2.1: outputs are combined and
// re-organised into the original order of the input tokens).  With an expert mask only the
// masked-in experts contribute (Section 3.3: the share of one side of the hot/cold split).
#include "common.hpp"

namespace moe {

// One wavefront per token and run of `cols` columns (blockIdx.y; the whole row when there are many tokens,
// 64 * VEC columns each when there are few: a decoder step's handful of tokens would otherwise walk their rows
// step after step in one wavefront each, 5.4 us for one token of 2048 columns); a lane owns 4 consecutive
// columns per 256-column step, reads them as one 16-byte piece from each of the token's k rows of y_perm and
// keeps the sum in fp32.
template <typename ST, int VEC>
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ y_perm,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const int32_t* __restrict__ idx,
                                                      const float* __restrict__ gate,
                                                      const uint8_t* __restrict__ mask,
                                                      ST* __restrict__ out, int T, int d, int k, int E,
                                                      int A, int cols) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + wave;
    if (t >= T) return;
    // The token's k rows, by slot; a slot whose expert is masked out (or invalid) is skipped.  Everything is
    // indexed by compile-time slot numbers (a compacted list would be indexed dynamically and its loads would
    // be issued and waited for one by one), and the slots that count are added in ascending order.
    const float* rows[MOE_MAX_K];
    float w[MOE_MAX_K];
    bool on[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
        rows[j] = y_perm;
        w[j] = 0.f;
        on[j] = false;
        if (j < k) {
            const int a = t * k + j;
            const int e = idx[a];
            const int p = inv_perm[a];
            on[j] = (e >= 0 && e < E && p >= 0 && p < A) && (mask == nullptr || mask[e] != 0);
            if (on[j]) {
                rows[j] = y_perm + static_cast<size_t>(p) * d;
                w[j] = gate[a];
            }
        }
    }
    ST* o = out + static_cast<size_t>(t) * d;
    const int c_begin = static_cast<int>(blockIdx.y) * cols, c_end = min(d, c_begin + cols);
    for (int c = c_begin + lane * VEC; c < c_end; c += 64 * VEC) {
        float v[MOE_MAX_K][VEC];
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j) {              // all the loads of the step first
            if (!on[j]) continue;                          // wave-uniform: one token per wavefront
            if (VEC == 4) {
                const float4 q = *reinterpret_cast<const float4*>(rows[j] + c);
                v[j][0] = q.x;
                v[j][1 % VEC] = q.y;
                v[j][2 % VEC] = q.z;
                v[j][3 % VEC] = q.w;
            } else {
                v[j][0] = rows[j][c];
            }
        }
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j) {
            if (!on[j]) continue;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w[j], v[j][i], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) Storage<ST>::store(o + c + i, acc[i]);
    }
}

hipError_t launch_combine(const moe_shape& s, const float* y_perm, const int32_t* inv_perm,
                          const int32_t* idx, const float* gate, const uint8_t* mask, void* out,
                          hipStream_t st) {
    const int T = s.T, d = s.d_model, k = s.k, E = s.E, A = s.T * s.k;
    // about 2048 wavefronts when the tokens alone do not give as many: runs of whole 64 * VEC-column steps
    const int vec = d % 4 == 0 ? 4 : 1, steps = (d + 64 * vec - 1) / (64 * vec);
    int ny = 2048 / (T > 0 ? T : 1);
    ny = ny < 1 ? 1 : (ny > steps ? steps : ny);
    const int cols = (steps + ny - 1) / ny * 64 * vec;
    const dim3 grid((T + 3) / 4, (d + cols - 1) / cols), block(256);
    if (s.dtype == MOE_BF16) {
        if (d % 4 == 0)
            hipLaunchKernelGGL((combine_kernel<uint16_t, 4>), grid, block, 0, st, y_perm, inv_perm, idx, gate,
                               mask, static_cast<uint16_t*>(out), T, d, k, E, A, cols);
        else
            hipLaunchKernelGGL((combine_kernel<uint16_t, 1>), grid, block, 0, st, y_perm, inv_perm, idx, gate,
                               mask, static_cast<uint16_t*>(out), T, d, k, E, A, cols);
    } else {
        if (d % 4 == 0)
            hipLaunchKernelGGL((combine_kernel<float, 4>), grid, block, 0, st, y_perm, inv_perm, idx, gate, mask,
                               static_cast<float*>(out), T, d, k, E, A, cols);
        else
            hipLaunchKernelGGL((combine_kernel<float, 1>), grid, block, 0, st, y_perm, inv_perm, idx, gate, mask,
                               static_cast<float*>(out), T, d, k, E, A, cols);
    }
    return hipGetLastError();
}

}  // namespace moe
