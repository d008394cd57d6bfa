// LDS-tiled MFMA product for experts with many rows (the compute-bound "hot" experts of the
// paper's Section 3.3: enough tokens per expert that the product is bound by matrix throughput,
// not by reading the expert's parameters):
//
//   out[row, n] = sum_k act[row, k] * W_e[n, k]          (FIRST: relu, rounded to bf16)
//
// Block = 8 wavefronts on a 256 (rows) x 256 (columns) output tile, K in steps of 64 through
// double-buffered LDS.  Both operands sit in LDS in MFMA-fragment order (16 x 32 fragments of
// 1 KiB, one 16-byte piece per lane), so every LDS read of the inner loop is a conflict-free
// 1 KiB wavefront read.  Global memory is copied straight into LDS (16 bytes per lane, no
// registers in between): the packed weights are already in fragment order in HBM, and for the
// activation rows (optionally gathered through `rowmap`) each lane fetches the piece that
// belongs at its own slot.  Wavefront (wm, wn) of the 2 x 4 grid owns 128 rows x 64 columns:
// 4 weight fragments (MFMA A operand) x 8 row fragments (B operand) of 16x16x32 per 32-k step,
// 128 accumulator registers.  Blocks are persistent over (row tile, column tile) pairs taken
// from the device-built list of large-expert row tiles.
#include "common.hpp"

namespace moe {

constexpr int kTM = kBigTileRows;   // 256 rows
constexpr int kTN = 256;            // columns
constexpr int kTK = 64;             // k per LDS stage
constexpr int kStageBytes = kTM * kTK * 2;          // 32 KiB per operand per stage

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

// 16 bytes per lane from global memory straight into LDS at `lds_base + 16 * lane` (no registers)
__device__ __forceinline__ void copy16_to_lds(const void* src, unsigned char* lds_base) {
    __builtin_amdgcn_global_load_lds((gptr_t)(src), (lptr_t)(lds_base), 16, 0, 0);
}

template <bool FIRST>
__global__ __launch_bounds__(512) void ffn_tile_kernel(const uint16_t* __restrict__ act,
                                                       const int32_t* __restrict__ rowmap,
                                                       const uint16_t* __restrict__ wpk,
                                                       void* __restrict__ outp, const Tile* __restrict__ tiles,
                                                       const int32_t* __restrict__ ntiles_p, int N, int K) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // stage st: 32 activation fragments at smem + st * 2 * kStageBytes, 32 weight fragments behind them;
    // fragment (block b of 16 rows/columns, kb) of a stage sits at ((b * 2 + kb) * 1024) bytes
    auto As = [&](int st) { return smem + st * 2 * kStageBytes; };
    auto Bs = [&](int st) { return smem + st * 2 * kStageBytes + kStageBytes; };

    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int wm = wave >> 2, wn = wave & 3;
    const int r = lane & 15, g = lane >> 4;
    const int nblk = N >> 4, kblk = K >> 5;
    const int ntn = (N + kTN - 1) / kTN;
    const int nkt = (kblk + 1) >> 1;                    // k stages of 64
    const int total = ntiles_p[0] * ntn;

    for (int u = blockIdx.x; u < total; u += gridDim.x) {
        const Tile tl = tiles[u / ntn];
        const int nt = u % ntn;
        // This wavefront stages fragments 4*wave .. 4*wave+3 of each operand: blocks 2*wave and 2*wave+1,
        // both 32-k halves.  A lane fetches the 16 bytes that belong at its own slot of the fragment:
        // row (lane % 16) of the block, k-group (lane / 16).
        const uint16_t* arow[2];
        const uint16_t* brow[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int row = tl.row0 + min((2 * wave + i) * 16 + r, tl.rows - 1);
            if (rowmap != nullptr) row = rowmap[row];
            arow[i] = act + static_cast<size_t>(row) * K + g * 8;
            const int nb = min(nt * 16 + 2 * wave + i, nblk - 1);
            brow[i] = wpk + (static_cast<size_t>(tl.expert) * nblk + nb) * kblk * 512 + lane * 8;
        }

        f32x4 acc[4][8];
#pragma unroll
        for (int nf = 0; nf < 4; ++nf)
#pragma unroll
            for (int tf = 0; tf < 8; ++tf) acc[nf][tf] = f32x4{0.f, 0.f, 0.f, 0.f};

        auto stage_in = [&](int st, int kt) {
            const int nk32 = min(2, kblk - 2 * kt);          // the last stage may hold one 32-k half only
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    if (kb < nk32) {
                        copy16_to_lds(arow[i] + kt * 64 + kb * 32, As(st) + ((2 * wave + i) * 2 + kb) * 1024);
                        copy16_to_lds(brow[i] + (static_cast<size_t>(2 * kt + kb)) * 512,
                                      Bs(st) + ((2 * wave + i) * 2 + kb) * 1024);
                    }
        };
        auto compute = [&](int st, int nk32) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                if (kb < nk32) {
                    bf16x8 w[4];
#pragma unroll
                    for (int nf = 0; nf < 4; ++nf)
                        w[nf] = *reinterpret_cast<const bf16x8*>(Bs(st) + (((wn * 4 + nf) * 2 + kb) * 64 + lane) * 16);
#pragma unroll
                    for (int tf = 0; tf < 8; ++tf) {
                        const bf16x8 x =
                            *reinterpret_cast<const bf16x8*>(As(st) + (((wm * 8 + tf) * 2 + kb) * 64 + lane) * 16);
#pragma unroll
                        for (int nf = 0; nf < 4; ++nf)
                            acc[nf][tf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nf], x, acc[nf][tf], 0, 0, 0);
                    }
                }
            }
        };

        __syncthreads();                 // every wavefront is done reading the previous unit's stages
        stage_in(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's copies have landed in LDS
        __syncthreads();
        for (int kt = 0; kt < nkt; ++kt) {
            if (kt + 1 < nkt) stage_in((kt + 1) & 1, kt + 1);     // in flight while this stage is consumed
            compute(kt & 1, min(2, kblk - 2 * kt));
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
        }

        // epilogue: lane holds 4 consecutive columns of one row per accumulator
#pragma unroll
        for (int tf = 0; tf < 8; ++tf) {
            const int lr = wm * 128 + tf * 16 + r;
            if (lr >= tl.rows) continue;
            const size_t rowoff = static_cast<size_t>(tl.row0 + lr) * N;
#pragma unroll
            for (int nf = 0; nf < 4; ++nf) {
                const int nb = nt * 16 + wn * 4 + nf;
                if (nb >= nblk) continue;
                const int n = nb * 16 + g * 4;
                const f32x4 v = acc[nf][tf];
                if (FIRST) {
                    uint2 pk;
                    pk.x = f32_to_bf16(fmaxf(v[0], 0.f)) | (static_cast<uint32_t>(f32_to_bf16(fmaxf(v[1], 0.f))) << 16);
                    pk.y = f32_to_bf16(fmaxf(v[2], 0.f)) | (static_cast<uint32_t>(f32_to_bf16(fmaxf(v[3], 0.f))) << 16);
                    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(outp) + rowoff + n) = pk;
                } else {
                    *reinterpret_cast<f32x4*>(static_cast<float*>(outp) + rowoff + n) = v;
                }
            }
        }
    }
}

template <bool FIRST>
static hipError_t launch_tile(const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk, void* outp,
                              const Tile* tiles, const int32_t* ntiles, int N, int K, long max_tiles,
                              hipStream_t st) {
    auto kern = ffn_tile_kernel<FIRST>;
    constexpr int lds = 4 * kStageBytes;        // 128 KiB: above the default per-block limit
    static int per_cu = 0;
    if (per_cu == 0) {
        hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (ea != hipSuccess) return ea;
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, 512, lds) != hipSuccess || n <= 0) n = 1;
        per_cu = n;
    }
    const long ntn = (N + kTN - 1) / kTN;
    long grid = static_cast<long>(device_cu_count()) * per_cu;
    if (grid > max_tiles * ntn) grid = max_tiles * ntn;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(512), lds, st, act, rowmap, wpk, outp, tiles,
                       ntiles, N, K);
    return hipGetLastError();
}

hipError_t launch_tile_product(bool first, const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk,
                               void* outp, const Tile* tiles, const int32_t* ntiles, int N, int K, long max_tiles,
                               hipStream_t st) {
    return first ? launch_tile<true>(act, rowmap, wpk, outp, tiles, ntiles, N, K, max_tiles, st)
                 : launch_tile<false>(act, rowmap, wpk, outp, tiles, ntiles, N, K, max_tiles, st);
}

}  // namespace moe
