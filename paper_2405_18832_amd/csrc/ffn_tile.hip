// LDS-tiled MFMA product for experts with many rows (the compute-bound "hot" experts of the
// paper's Section 3.3: enough tokens per expert that the product is bound by matrix throughput,
// not by reading the expert's parameters):
//
//   out[row, n] = sum_k act[row, k] * W_e[n, k]          (FIRST: relu, rounded to bf16)
//
// Block = 8 wavefronts on a 256 (rows) x 256 (columns) output tile, K in steps of 32 through a
// ring of four LDS stages (the copies of three stages are in flight while one is consumed).  Both operands sit in LDS in MFMA-fragment order (16 x 32 fragments of
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
constexpr int kTK = 32;             // k per LDS stage
constexpr int kStages = 4;          // ring of LDS stages: one being consumed, up to three in flight
constexpr int kOperandBytes = kTM * kTK * 2;        // 16 KiB per operand per stage
constexpr int kStageBytes = 2 * kOperandBytes;      // 32 KiB per stage

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

// 16 bytes per lane from global memory straight into LDS at `lds_base + 16 * lane` (no registers)
__device__ __forceinline__ void copy16_to_lds(const void* src, unsigned char* lds_base) {
    __builtin_amdgcn_global_load_lds((gptr_t)(src), (lptr_t)(lds_base), 16, 0, 0);
}

// One 32-k LDS stage of the inner product for one wavefront: 4 weight fragments x 8 row fragments.
// `wbase` / `xbase` point at this lane's 16 bytes of the wavefront's first weight / row fragment;
// the next fragment lies 1 KiB further.  LDS reads run one pair of row fragments ahead of the MFMAs
// that consume them.
__device__ __forceinline__ void tile_stage(const unsigned char* __restrict__ wbase,
                                           const unsigned char* __restrict__ xbase, f32x4 (&acc)[4][8]) {
    bf16x8 w[4], x0, x1, y0, y1;
#pragma unroll
    for (int nf = 0; nf < 4; ++nf) w[nf] = *reinterpret_cast<const bf16x8*>(wbase + nf * 1024);
    x0 = *reinterpret_cast<const bf16x8*>(xbase);
    x1 = *reinterpret_cast<const bf16x8*>(xbase + 1024);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        if (p + 1 < 4) {                                   // reads for the next pair go out first
            y0 = *reinterpret_cast<const bf16x8*>(xbase + (2 * p + 2) * 1024);
            y1 = *reinterpret_cast<const bf16x8*>(xbase + (2 * p + 3) * 1024);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int nf = 0; nf < 4; ++nf) {
            acc[nf][2 * p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nf], x0, acc[nf][2 * p], 0, 0, 0);
            acc[nf][2 * p + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nf], x1, acc[nf][2 * p + 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (p + 1 < 4) {
            x0 = y0;
            x1 = y1;
        }
    }
}

template <bool FIRST>
__global__ __launch_bounds__(512) void ffn_tile_kernel(const uint16_t* __restrict__ act,
                                                       const int32_t* __restrict__ rowmap,
                                                       const uint16_t* __restrict__ wpk,
                                                       void* __restrict__ outp, const Tile* __restrict__ tiles,
                                                       const int32_t* __restrict__ ntiles_p, int N, int K) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // stage st: 16 row fragments at smem + st * kStageBytes, 16 weight fragments behind them
    auto As = [&](int st) { return smem + st * kStageBytes; };
    auto Bs = [&](int st) { return smem + st * kStageBytes + kOperandBytes; };

    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int wm = wave >> 2, wn = wave & 3;
    const int r = lane & 15, g = lane >> 4;
    const int nblk = N >> 4, kblk = K >> 5;
    const int ntn = (N + kTN - 1) / kTN;
    const int ntiles = ntiles_p[0];

    // Unit order.  Blocks are handed to the 8 XCDs round-robin, and each XCD has its own L2.  The blocks
    // of one XCD therefore work, at any time, on a compact GM x GN patch of (row tile, column tile) space,
    // so that its L2 serves every activation panel GN times and every weight panel GM times; the 8 XCDs
    // take 8 patches of the same column group (same weight panels, served to the others by the
    // last-level cache).  Falls back to row-major order when the grid does not split that way.
    const int G = gridDim.x;
    const int GN = min(ntn, 8);
    const bool patches = (G % 8 == 0) && ((G / 8) % GN == 0);
    const int S = patches ? G / 8 : 1;
    const int GM = patches ? S / GN : 1;
    const int nrg = (ntiles + GM - 1) / GM, ncg = (ntn + GN - 1) / GN;
    const int ngroups = nrg * ncg;
    const int total = patches ? ((ngroups + 7) / 8) * G : ntiles * ntn;

    for (int L = blockIdx.x; L < total; L += G) {
        int mt, nt;
        if (patches) {
            const int grp = (L / G) * 8 + (blockIdx.x & 7), slot = blockIdx.x >> 3;
            if (grp >= ngroups) continue;
            mt = (grp % nrg) * GM + slot / GN;
            nt = (grp / nrg) * GN + slot % GN;
            if (mt >= ntiles || nt >= ntn) continue;
        } else {
            mt = L / ntn;
            nt = L % ntn;
        }
        const Tile tl = tiles[mt];
        // This wavefront stages fragments 2*wave and 2*wave+1 of each operand.  A lane fetches the 16
        // bytes that belong at its own slot of the fragment: row (lane % 16), k-group (lane / 16).
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

        auto stage_in = [&](int st, int kb) {              // 4 copies per wavefront and stage
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                copy16_to_lds(arow[i] + kb * 32, As(st) + (2 * wave + i) * 1024);
                copy16_to_lds(brow[i] + static_cast<size_t>(kb) * 512, Bs(st) + (2 * wave + i) * 1024);
            }
        };

        const int wave_w = (wn * 4 * 64 + lane) * 16, wave_x = (wm * 8 * 64 + lane) * 16;
        __syncthreads();                 // every wavefront is done reading the previous unit's stages
#pragma unroll
        for (int sidx = 0; sidx < kStages - 1; ++sidx)
            if (sidx < kblk) stage_in(sidx, sidx);
        for (int kb = 0; kb < kblk; ++kb) {
            // stage kb must have landed; the copies of up to two later stages (4 each) may stay in flight
            const int later = min(kStages - 2, kblk - 1 - kb);
            if (later >= 2) __builtin_amdgcn_s_waitcnt(0x0F78);          // vmcnt(8)
            else if (later == 1) __builtin_amdgcn_s_waitcnt(0x0F74);     // vmcnt(4)
            else __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0)
            // ... for every wavefront, and nobody still reads stage kb-1.  A bare barrier: __syncthreads()
            // would first drain every outstanding copy (its fence waits for vmcnt(0)) and empty the ring.
            asm volatile("s_barrier" ::: "memory");
            if (kb + kStages - 1 < kblk) stage_in((kb + kStages - 1) % kStages, kb + kStages - 1);
            tile_stage(Bs(kb % kStages) + wave_w, As(kb % kStages) + wave_x, acc);
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
    constexpr int lds = kStages * kStageBytes;  // 128 KiB: above the default per-block limit
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
