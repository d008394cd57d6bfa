// Expert FFNs as a grouped product over variable token counts:
//   y_perm[rows of e] = relu(x_perm[rows of e] . W1_e^T) . W2_e^T        for every active expert e
// (paper Section 2.1: an expert is two linear layers with an activation between; Sections 3.1
// and 3.4: each is C = A x B, the first with a trailing ReLU).  The paper's observation that
// most experts receive very few tokens, so that their cost is reading their parameters
// (Section 2.2), is what shapes the kernel below: it streams every active expert's weights
// exactly once at full memory bandwidth while the few token rows ride along as the other MFMA
// operand.
#include <algorithm>

#include "tile_schedule.hpp"

namespace moe {

// ---------------------------------------------------------------------------
// weight packing: [E][N][K] row-major  ->  [E][N/16][K/32] fragments of 64 lanes x 8 elements.
// One thread per 16-byte piece of the destination.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint4* __restrict__ src,
                                                        uint4* __restrict__ dst, int N, int K,
                                                        size_t total) {
    const size_t c = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (c >= total) return;
    const size_t per_expert = static_cast<size_t>(N) * K / 8;
    const size_t e = c / per_expert, ce = c % per_expert;
    const int kblk = K / 32;
    const size_t frag = ce / 64;
    const int l = static_cast<int>(ce % 64);
    const int nb = static_cast<int>(frag / kblk), kb = static_cast<int>(frag % kblk);
    const int n = nb * 16 + (l & 15), kk = kb * 32 + (l >> 4) * 8;
    dst[c] = src[(e * N + n) * (K / 8) + kk / 8];
}

__global__ __launch_bounds__(256) void copy_u32_kernel(const uint32_t* __restrict__ src,
                                                       uint32_t* __restrict__ dst, size_t total) {
    const size_t c = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (c < total) dst[c] = src[c];
}

hipError_t launch_pack(const moe_shape& s, int which, const void* src, void* dst, hipStream_t st) {
    const int N = which == 1 ? s.d_ff : s.d_model, K = which == 1 ? s.d_model : s.d_ff;
    if (s.dtype == MOE_BF16) {
        const size_t total = static_cast<size_t>(s.E) * N * K / 8;
        hipLaunchKernelGGL(pack_bf16_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0,
                           st, static_cast<const uint4*>(src), static_cast<uint4*>(dst), N, K, total);
    } else {
        const size_t total = static_cast<size_t>(s.E) * N * K;
        hipLaunchKernelGGL(copy_u32_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0,
                           st, static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst), total);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// tile lists from caller-supplied offsets (the stand-alone expert-FFN call): every active,
// masked-in expert's row segment cut into row tiles.  One block, one thread per expert.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void build_tiles_kernel(const int32_t* __restrict__ offsets,
                                                           const uint8_t* __restrict__ mask, int E, int A,
                                                           const TileLists lists) {
    __shared__ int32_t scan[MOE_MAX_E];
    const int e = threadIdx.x;
    int row0 = 0, m = 0;
    bool bad = false;
    if (e < E) {
        row0 = offsets[e];
        m = offsets[e + 1] - row0;
        bad = row0 < 0 || m < 0 || row0 + m > A;
        if (mask != nullptr && mask[e] == 0) m = 0;
    }
    // Offsets that are not prefix sums (a negative count anywhere, a segment outside [0, A]): run nothing at all.
    // With every count >= 0 the segments are disjoint and their sum is at most A, which is what the capacity of
    // the tile lists assumes.
    if (__syncthreads_or(bad ? 1 : 0)) m = 0;
    emit_tiles(e, row0, m, lists, scan);
}

// ---------------------------------------------------------------------------
// bf16 weight-streaming product.
//
//   out[row, n] = sum_k act[row, k] * W_e[n, k]          (FIRST: relu, rounded to bf16)
//
// MFMA 16x16x32: the A operand is a packed 16(n) x 32(k) weight fragment -- one contiguous
// 1 KiB load per wavefront, 16 bytes per lane, straight from HBM into registers -- and the B
// operand is 16 token rows x 32 k of the activations (L2/L1 hits; every wave of a block reads
// the same rows).  A wavefront owns 4 n-blocks (64 output columns) x up to TFMAX*16 token rows
// over one k-slice; the KSPLIT wavefronts that share an output tile add their partial sums in
// LDS in a fixed order.  Blocks are persistent and stride over (tile, n-group) units, whose
// number is only known on the device.
//
// The inner loop is specialised on the exact number of token fragments of the tile (TFC), so
// every k-step issues a fixed number of loads: the compiler can then count outstanding loads
// exactly and keeps PF k-steps in flight across loop iterations (with a data-dependent number
// of loads it drains the queue on every iteration).
// With `rowmap`, row p of the activations is read from act[rowmap[p]] (the token gather of the
// dispatch step folded into the first product); output rows are always in permuted order.
// ---------------------------------------------------------------------------
// tuning constants (overridable at build time)
#ifndef MOE_PF_TF1
#define MOE_PF_TF1 6      // k-steps of loads in flight per wavefront, tiles of <= 16 rows
#endif
#ifndef MOE_PF_TF2
#define MOE_PF_TF2 4      // ... tiles of <= 32 rows
#endif
#ifndef MOE_PF_TF3
#define MOE_PF_TF3 3      // ... tiles of <= 48 rows
#endif
#ifndef MOE_PF_TF4
#define MOE_PF_TF4 3      // ... tiles of <= 64 rows
#endif
#ifndef MOE_PF_NARROW
#define MOE_PF_NARROW 16  // ... when a wavefront owns one column block only (one KiB of weights per step)
#endif
#ifndef MOE_PF_LDS
#define MOE_PF_LDS 6      // k-steps of weight loads in flight when the rows come from LDS
#endif

// s_waitcnt immediate that waits for vmcnt <= n only (n < 64: low four bits in [3:0], the rest in [15:14])
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

constexpr size_t kStreamRowLdsMax = 128 * 1024;   // largest row tile kept in LDS by the streaming kernel

template <int TFC> struct StreamPF;
template <> struct StreamPF<1> { static constexpr int value = MOE_PF_TF1; };
template <> struct StreamPF<2> { static constexpr int value = MOE_PF_TF2; };
template <> struct StreamPF<3> { static constexpr int value = MOE_PF_TF3; };
template <> struct StreamPF<4> { static constexpr int value = MOE_PF_TF4; };

// Token row and gate weight of the lane's rows (row fragment tf, row lane % 16) for a folded second product;
// fetched when a unit starts so that the two dependent loads are long done when the unit's output is stored.
template <int TFC, bool FOLD>
__device__ __forceinline__ void fold_rows(const FoldOut& fold, const Tile tl, int (&ftok)[TFC], float (&fw)[TFC]) {
    const int r = threadIdx.x & 15;
#pragma unroll
    for (int tf = 0; tf < TFC; ++tf) {
        ftok[tf] = 0;
        fw[tf] = 0.f;
        if (FOLD) {
            ftok[tf] = fold.tokmap[tl.row0 + min(tf * 16 + r, tl.rows - 1)];
            fw[tf] = fold.gate[ftok[tf]];
        }
    }
}

// Output of one column group (4 n-blocks) x TFC row fragments of a tile, by one whole wavefront.
template <int TFC, int FIRST, bool FOLD, int GW = 4>
__device__ __forceinline__ void store_group(void* __restrict__ outp, const Tile tl, const int ng, const int nblk,
                                            const int N, const float* __restrict__ be,
                                            const f32x4 (&acc)[GW][TFC], const FoldOut& fold,
                                            const int (&ftok)[TFC], const float (&fw)[TFC]) {
    static_assert(GW == 4 || (FIRST == 0 && !FOLD), "paired stores need groups of 4 column blocks");
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
#pragma unroll
    for (int tf = 0; tf < TFC; ++tf) {
        const int lr = tf * 16 + r;
        const bool ok = lr < tl.rows;
        if constexpr (FIRST != 0 && GW == 4) {
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const int nb = ng * 4 + 2 * m;             // N / 16 is even: the pair exists or not as a whole
                if (nb >= nblk) continue;                  // wave-uniform
                store_h_pair<FIRST, true>(outp, tl.row0 + lr, ok, nb * 16, N, be, acc[2 * m][tf], acc[2 * m + 1][tf]);
            }
        } else if constexpr (FOLD && GW == 4) {            // the layer output itself
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const int nb = ng * 4 + 2 * m;
                if (nb >= nblk) continue;                  // wave-uniform
                store_folded_pair(fold.out, ftok[tf], fw[tf], ok, nb * 16, N, be, acc[2 * m][tf], acc[2 * m + 1][tf]);
            }
        } else {
#pragma unroll
            for (int nf = 0; nf < GW; ++nf) {
                const int nb = ng * GW + nf;
                if (ok && nb < nblk)
                    store_out<0, true>(outp, tl.row0 + lr, nb * 16 + g * 4, N, be, acc[nf][tf]);
            }
        }
    }
}

// One wavefront's share of one unit: 4 n-blocks x TFC token fragments over k-steps [kb0, kb1).
template <int TFC, int TFMAX, int KSPLIT, int FIRST, bool FOLD, int GW = 4>
__device__ __forceinline__ void stream_unit(const uint16_t* __restrict__ act,
                                            const int32_t* __restrict__ rowmap,
                                            const uint16_t* __restrict__ wpk, void* __restrict__ outp,
                                            const Tile tl, const int ng, const bool active, const int N,
                                            const int K, const int kb0, const int kb1, f32x4* red,
                                            const bool act_kmajor,
                                            const float* __restrict__ bias, const FoldOut& fold) {
    constexpr int PF = GW == 4 ? StreamPF<TFC>::value : MOE_PF_NARROW;
    constexpr int NGB = 4 / KSPLIT;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int ks = wave % KSPLIT, ngs = wave / KSPLIT;
    const int nblk = N >> 4, kblk = K >> 5;
    f32x4 acc[GW][TFC];
#pragma unroll
    for (int nf = 0; nf < GW; ++nf)
#pragma unroll
        for (int tf = 0; tf < TFC; ++tf) acc[nf][tf] = f32x4{0.f, 0.f, 0.f, 0.f};

    int ftok[TFC];
    float fw[TFC];
    fold_rows<TFC, FOLD>(fold, tl, ftok, fw);
    if (active && kb0 < kb1) {
        const uint16_t* wp[GW];
#pragma unroll
        for (int nf = 0; nf < GW; ++nf) {
            const int nb = min(ng * GW + nf, nblk - 1);
            wp[nf] = wpk + (static_cast<size_t>(tl.expert) * nblk + nb) * kblk * 512 + lane * 8;
        }
        const bool km = FIRST == 0 ? true : act_kmajor;     // the second product always reads h
        const uint16_t* ap[TFC];
#pragma unroll
        for (int tf = 0; tf < TFC; ++tf) {
            int row = tl.row0 + min(tf * 16 + r, tl.rows - 1);
            if (rowmap != nullptr) row = rowmap[row];       // gather: permuted position -> token row
            // operand rows are row-major (the caller's x or x_perm) or k-step-major (h, gathered x)
            ap[tf] = km ? act + h_index(row, g * 8, kblk) : act + static_cast<size_t>(row) * K + g * 8;
        }
        const size_t kstride = km ? kStepStride : 32;   // elements per k-step
        bf16x8 a[PF][GW], b[PF][TFC];
        auto issue = [&](int slot, int kb) {
#pragma unroll
            for (int nf = 0; nf < GW; ++nf)
                a[slot][nf] = *reinterpret_cast<const bf16x8*>(wp[nf] + static_cast<size_t>(kb) * 512);
#pragma unroll
            for (int tf = 0; tf < TFC; ++tf) b[slot][tf] = *reinterpret_cast<const bf16x8*>(ap[tf] + kb * kstride);
        };
        auto fma = [&](int slot) {
#pragma unroll
            for (int tf = 0; tf < TFC; ++tf)
#pragma unroll
                for (int nf = 0; nf < GW; ++nf)
                    acc[nf][tf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[slot][nf], b[slot][tf], acc[nf][tf], 0, 0, 0);
        };
        // prologue: always PF steps of loads (past the end the last step is re-read, never used)
#pragma unroll
        for (int p = 0; p < PF; ++p) issue(p, min(kb0 + p, kb1 - 1));
        int kb = kb0;
        for (; kb + 2 * PF <= kb1; kb += PF) {            // steady state: fixed number of loads per step
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                fma(p);
                issue(p, kb + p + PF);
            }
        }
        if (kb + PF < kb1) {                               // one partial round of refills
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                fma(p);
                issue(p, min(kb + p + PF, kb1 - 1));
            }
            kb += PF;
        }
#pragma unroll
        for (int p = 0; p < PF; ++p)                       // drain: no more loads
            if (kb + p < kb1) fma(p);
    }

    if (KSPLIT > 1) {
        if (active && ks > 0) {
            f32x4* dst = red + (static_cast<size_t>((ks - 1) * NGB + ngs) * GW * TFMAX) * 64 + lane;
#pragma unroll
            for (int nf = 0; nf < GW; ++nf)
#pragma unroll
                for (int tf = 0; tf < TFC; ++tf) dst[(nf * TFMAX + tf) * 64] = acc[nf][tf];
        }
        // LDS only: a bare barrier after the LDS writes have completed.  (__syncthreads() also waits for
        // every outstanding global store, i.e. for the previous unit's output rows: a store latency per unit.)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (active && ks == 0) {
#pragma unroll
            for (int s = 1; s < KSPLIT; ++s) {
                const f32x4* src = red + (static_cast<size_t>((s - 1) * NGB + ngs) * GW * TFMAX) * 64 + lane;
#pragma unroll
                for (int nf = 0; nf < GW; ++nf)
#pragma unroll
                    for (int tf = 0; tf < TFC; ++tf) acc[nf][tf] += src[(nf * TFMAX + tf) * 64];
            }
        }
    }
    if (active && ks == 0) {
        const float* be = bias ? bias + static_cast<size_t>(tl.expert) * N : nullptr;
        store_group<TFC, FIRST, FOLD, GW>(outp, tl, ng, nblk, N, be, acc, fold, ftok, fw);
    }
    if (KSPLIT > 1) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // `red` may be reused
}

// The same unit when all four wavefronts of the block share the tile's rows over the same k range
// (KSPLIT = 1: the block covers four column groups): the rows are copied once per block into LDS, in
// MFMA-fragment order, instead of being fetched by every wavefront at every k-step.  That takes the
// row operand out of the vector-memory queue that the weights stream through (one quarter of the
// requests, issued once, asynchronously) and out of the registers that hold loads in flight.
// `tok_lds` holds TFC * K / 32 fragments of 1 KiB: fragment (tf, kb) at (tf * K / 32 + kb) * 1024.
template <int TFC, int FIRST, bool FOLD>
__device__ __forceinline__ void stream_unit_lds(const uint16_t* __restrict__ act,
                                                const int32_t* __restrict__ rowmap,
                                                const uint16_t* __restrict__ wpk, void* __restrict__ outp,
                                                const Tile tl, const int ng, const bool active, const int N,
                                                const int K, const bool act_kmajor,
                                                const float* __restrict__ bias, unsigned char* tok_lds,
                                                const FoldOut& fold) {
    constexpr int PF = MOE_PF_LDS;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 15, g = lane >> 4;
    const int nblk = N >> 4, kblk = K >> 5;
    f32x4 acc[4][TFC];
#pragma unroll
    for (int nf = 0; nf < 4; ++nf)
#pragma unroll
        for (int tf = 0; tf < TFC; ++tf) acc[nf][tf] = f32x4{0.f, 0.f, 0.f, 0.f};

    int ftok[TFC];
    float fw[TFC];
    fold_rows<TFC, FOLD>(fold, tl, ftok, fw);
    // the token rows behind the lane's permuted positions: fetched before the barrier, whose wait hides them
    int rows_of[TFC];
#pragma unroll
    for (int tf = 0; tf < TFC; ++tf) {
        rows_of[tf] = tl.row0 + min(tf * 16 + r, tl.rows - 1);
        if (rowmap != nullptr) rows_of[tf] = rowmap[rows_of[tf]];
    }
    // every wavefront has finished reading the previous unit's rows
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    // rows -> LDS: wavefront w copies the fragments (tf, kb) with kb = w, w + 4, ...; a lane fetches the
    // 16 bytes of its own slot: row (lane % 16), k-group (lane / 16)
    const size_t kstride = act_kmajor ? kStepStride : 32;   // elements per k-step
    const uint32_t lds0 = lds_address(tok_lds);
#pragma unroll
    for (int tf = 0; tf < TFC; ++tf) {
        const int row = rows_of[tf];
        const uint16_t* ap =
            act_kmajor ? act + h_index(row, g * 8, kblk) : act + static_cast<size_t>(row) * K + g * 8;
        for (int kb = wave; kb < kblk; kb += 4) copy16_to_lds(ap + kb * kstride, lds0 + (tf * kblk + kb) * 1024);
    }

    const uint16_t* wp[4];
#pragma unroll
    for (int nf = 0; nf < 4; ++nf) {
        const int nb = min(ng * 4 + nf, nblk - 1);
        wp[nf] = wpk + (static_cast<size_t>(tl.expert) * nblk + nb) * kblk * 512 + lane * 8;
    }
    bf16x8 a[PF][4];
    auto issue = [&](int slot, int kb) {
#pragma unroll
        for (int nf = 0; nf < 4; ++nf)
            a[slot][nf] = *reinterpret_cast<const bf16x8*>(wp[nf] + static_cast<size_t>(kb) * 512);
    };
    if (active) {
#pragma unroll
        for (int p = 0; p < PF; ++p) issue(p, min(p, kblk - 1));   // past the end: re-read, never used
    }
    // The row copies were issued before the weight loads, and loads complete in order: they have landed
    // once at most the weight loads are outstanding ... for every wavefront.
    if (active) __builtin_amdgcn_s_waitcnt(vmcnt_imm(PF * 4));
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("s_barrier" ::: "memory");

    if (active) {
        const unsigned char* bl = tok_lds + lane * 16;
        auto fma = [&](int slot, int kb) {
            bf16x8 b[TFC];
#pragma unroll
            for (int tf = 0; tf < TFC; ++tf) b[tf] = *reinterpret_cast<const bf16x8*>(bl + (tf * kblk + kb) * 1024);
#pragma unroll
            for (int tf = 0; tf < TFC; ++tf)
#pragma unroll
                for (int nf = 0; nf < 4; ++nf)
                    acc[nf][tf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[slot][nf], b[tf], acc[nf][tf], 0, 0, 0);
        };
        int kb = 0;
        for (; kb + 2 * PF <= kblk; kb += PF) {
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                fma(p, kb + p);
                issue(p, kb + p + PF);
            }
        }
        if (kb + PF < kblk) {
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                fma(p, kb + p);
                issue(p, min(kb + p + PF, kblk - 1));
            }
            kb += PF;
        }
#pragma unroll
        for (int p = 0; p < PF; ++p)
            if (kb + p < kblk) fma(p, kb + p);

        const float* be = bias ? bias + static_cast<size_t>(tl.expert) * N : nullptr;
        store_group<TFC, FIRST, FOLD>(outp, tl, ng, nblk, N, be, acc, fold, ftok, fw);
    }
}

template <int TFMAX, int KSPLIT, int FIRST, bool FOLD>
__global__ __launch_bounds__(256) void ffn_stream_kernel(const uint16_t* __restrict__ act,
                                                         const int32_t* __restrict__ rowmap,
                                                         const uint16_t* __restrict__ wpk,
                                                         void* __restrict__ outp,
                                                         const Tile* __restrict__ tiles,
                                                         const int32_t* __restrict__ ntiles_p, int N,
                                                         int K, int balance,
                                                         const Tile* __restrict__ big_tiles,
                                                         const float* __restrict__ partials, int tile_grid,
                                                         int act_kmajor, int rows_in_lds,
                                                         const float* __restrict__ bias, const FoldOut fold) {
    extern __shared__ __attribute__((aligned(16))) unsigned char tok_lds[];
    constexpr int NGB = 4 / KSPLIT;   // n-groups (of 64 columns) per block
    __shared__ f32x4 red[KSPLIT > 1 ? (KSPLIT - 1) * NGB * 4 * TFMAX * 64 : 1];
    const int wave = threadIdx.x >> 6;
    const int ks = wave % KSPLIT, ngs = wave / KSPLIT;
    const int nblk = N >> 4, kblk = K >> 5;
    const int ngroups = (nblk + 3) >> 2;
    const int ngchunks = (ngroups + NGB - 1) / NGB;
    const int kb_per = (kblk + KSPLIT - 1) / KSPLIT;
    const int kb0 = min(kblk, ks * kb_per), kb1 = min(kblk, kb0 + kb_per);
    const int nbu = ntiles_p[0] * ngchunks;
    int stride = gridDim.x;
    if (balance) {
        // Units are equal-sized, so a grid that does not divide them ends with a round of few blocks and
        // little data in flight.  Use only as many blocks as make every block run the same number of
        // units (the others exit): the memory system sees a constant number of streams to the end.
        const int rounds = (nbu + stride - 1) / stride;
        if (rounds > 0) stride = (nbu + rounds - 1) / rounds;
        if (static_cast<int>(blockIdx.x) >= stride) return;
    }
    // Blocks go to the 8 XCDs round-robin and each XCD has its own L2: give the blocks of one XCD
    // consecutive units, i.e. the column groups of the same tile, so that the tile's activation rows are
    // fetched into that L2 once instead of into all eight.
    const int pb = (stride % 8 == 0) ? static_cast<int>(blockIdx.x & 7) * (stride >> 3) + static_cast<int>(blockIdx.x >> 3)
                                     : static_cast<int>(blockIdx.x);
    // First the rows that the tiled kernel before this one left as partial tiles (large experts; no overlap
    // with the rows of the small experts below).  When at least a quarter of the blocks have no streaming unit
    // they do it, side by side with the others' streaming; else everybody does, before streaming.
    if (partials != nullptr) {
        const int idle = stride - nbu;                    // blocks with pb >= nbu have no unit (balance is off here)
        if (idle * 4 >= stride) {
            if (pb >= nbu)
                finish_split_units<FIRST, FOLD>(big_tiles, ntiles_p[1], partials, outp, N, K >> 5, tile_grid, bias, fold,
                                                pb - nbu, idle);
        } else {
            finish_split_units<FIRST, FOLD>(big_tiles, ntiles_p[1], partials, outp, N, K >> 5, tile_grid, bias, fold,
                                            static_cast<int>(blockIdx.x), static_cast<int>(gridDim.x));
        }
    }
    for (int base = 0; base < nbu; base += stride) {
        const int bu = base + pb;
        if (bu >= nbu) break;                             // block-uniform
        const Tile tl = tiles[bu / ngchunks];
        const int ng = (bu % ngchunks) * NGB + ngs;
        const bool active = ng < ngroups;                 // wave-uniform
        const int tfc = (tl.rows + 15) >> 4;              // token fragments in use: block-uniform
        if (KSPLIT == 1 && rows_in_lds) {
            const bool km = act_kmajor != 0;
            if (TFMAX >= 4 && tfc == 4)
                stream_unit_lds<4, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, km, bias, tok_lds, fold);
            else if (TFMAX >= 4 && tfc == 3)
                stream_unit_lds<3, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, km, bias, tok_lds, fold);
            else if (TFMAX >= 2 && tfc == 2)
                stream_unit_lds<2, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, km, bias, tok_lds, fold);
            else
                stream_unit_lds<1, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, km, bias, tok_lds, fold);
            continue;
        }
        if (TFMAX >= 4 && tfc == 4)
            stream_unit<4, TFMAX, KSPLIT, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, kb0, kb1, red, act_kmajor != 0, bias, fold);
        else if (TFMAX >= 4 && tfc == 3)
            stream_unit<3, TFMAX, KSPLIT, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, kb0, kb1, red, act_kmajor != 0, bias, fold);
        else if (TFMAX >= 2 && tfc == 2)
            stream_unit<2, TFMAX, KSPLIT, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, kb0, kb1, red, act_kmajor != 0, bias, fold);
        else
            stream_unit<1, TFMAX, KSPLIT, FIRST, FOLD>(act, rowmap, wpk, outp, tl, ng, active, N, K, kb0, kb1, red, act_kmajor != 0, bias, fold);
    }
}

// ---------------------------------------------------------------------------
// fp32 storage: plain FMA kernel (small layers only).  Tiles of 16 rows; a thread owns one
// output column of a tile and walks the rows.
// ---------------------------------------------------------------------------
template <bool FIRST>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ act,
                                                      const int32_t* __restrict__ rowmap,
                                                      const float* __restrict__ w,
                                                      float* __restrict__ outp,
                                                      const Tile* __restrict__ tiles,
                                                      const int32_t* __restrict__ ntiles_p, int N, int K,
                                                      int activation, const float* __restrict__ bias) {
    const int nchunks = (N + 255) / 256;
    const int nbu = ntiles_p[0] * nchunks;
    for (int bu = blockIdx.x; bu < nbu; bu += gridDim.x) {
        const Tile tl = tiles[bu / nchunks];
        const int n = (bu % nchunks) * 256 + threadIdx.x;
        if (n >= N) continue;
        const float* wr = w + (static_cast<size_t>(tl.expert) * N + n) * K;
        for (int i = 0; i < tl.rows; ++i) {
            const int src = rowmap ? rowmap[tl.row0 + i] : tl.row0 + i;
            const float* ar = act + static_cast<size_t>(src) * K;
            // four running sums over c mod 4 (16-byte loads, four independent chains), added pairwise at the end
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            int c = 0;
            if ((K & 3) == 0) {                            // rows of x, h and the weights are then 16-byte aligned
                for (; c < K; c += 4) {
                    const float4 a = *reinterpret_cast<const float4*>(ar + c);
                    const float4 b = *reinterpret_cast<const float4*>(wr + c);
                    s0 = fmaf(a.x, b.x, s0);
                    s1 = fmaf(a.y, b.y, s1);
                    s2 = fmaf(a.z, b.z, s2);
                    s3 = fmaf(a.w, b.w, s3);
                }
            }
            for (; c < K; ++c) s0 = fmaf(ar[c], wr[c], s0);
            float s = (s0 + s1) + (s2 + s3);
            if (bias) s += bias[static_cast<size_t>(tl.expert) * N + n];
            outp[static_cast<size_t>(tl.row0 + i) * N + n] = FIRST ? activate(s, activation) : s;
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// per device, written once by configure_ffn_kernels (under the set-up lock) before any launch reads them
static int g_cus[kMaxDevices] = {0};

int device_cu_count() {
    const int n = g_cus[current_device_index()];
    return n > 0 ? n : 256;
}

// resident blocks per CU of a weight-streaming kernel without dynamic LDS, per device
template <int TFMAX, int KSPLIT, int FIRST, bool FOLD>
struct StreamKernelInfo {
    static int per_cu[kMaxDevices];
};
template <int TFMAX, int KSPLIT, int FIRST, bool FOLD>
int StreamKernelInfo<TFMAX, KSPLIT, FIRST, FOLD>::per_cu[kMaxDevices] = {0};

// Second product of a layer of at most 16 tokens when its experts are so few that groups of 64 columns leave
// most CUs without a unit (one decoder token with two experts: 64 units): a unit is one 16-column block, the
// four wavefronts of a block split the contraction as usual and keep 16 KiB-steps of weights in flight each.
__global__ __launch_bounds__(256) void ffn_stream_narrow_kernel(const uint16_t* __restrict__ act,
                                                                const uint16_t* __restrict__ wpk,
                                                                void* __restrict__ outp,
                                                                const Tile* __restrict__ tiles,
                                                                const int32_t* __restrict__ ntiles_p, int N, int K,
                                                                const float* __restrict__ bias) {
    __shared__ f32x4 red[3 * 64];
    const int ks = threadIdx.x >> 6;
    const int nblk = N >> 4, kblk = K >> 5;
    const int kb_per = (kblk + 3) / 4;
    const int kb0 = min(kblk, ks * kb_per), kb1 = min(kblk, kb0 + kb_per);
    const int nbu = ntiles_p[0] * nblk;
    // as in ffn_stream_kernel: every block that runs gets the same number of units, and the blocks of an XCD
    // take consecutive units
    int stride = gridDim.x;
    const int rounds = (nbu + stride - 1) / stride;
    if (rounds > 0) stride = (nbu + rounds - 1) / rounds;
    if (static_cast<int>(blockIdx.x) >= stride) return;
    const int pb = (stride % 8 == 0) ? static_cast<int>(blockIdx.x & 7) * (stride >> 3) + static_cast<int>(blockIdx.x >> 3)
                                     : static_cast<int>(blockIdx.x);
    const FoldOut none{nullptr, nullptr, nullptr};
    for (int base = 0; base < nbu; base += stride) {
        const int bu = base + pb;
        if (bu >= nbu) break;                             // block-uniform
        stream_unit<1, 1, 4, 0, false, 1>(act, nullptr, wpk, outp, tiles[bu / nblk], bu % nblk, true, N, K, kb0, kb1, red,
                                          true, bias, none);
    }
}

template <int TFMAX, int KSPLIT, int FIRST, bool FOLD>
static hipError_t launch_stream(const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk, void* outp,
                                const Tile* tiles, const int32_t* ntiles, int N, int K, long max_units,
                                const Tile* big_tiles, const float* partials, bool act_kmajor,
                                const float* bias, const FoldOut& fold, hipStream_t st) {
    auto kern = ffn_stream_kernel<TFMAX, KSPLIT, FIRST, FOLD>;
    const int per_cu = std::max(1, StreamKernelInfo<TFMAX, KSPLIT, FIRST, FOLD>::per_cu[current_device_index()]);
    // KSPLIT = 1: the tile's rows (16 * TFMAX x K, bf16) go through LDS when they fit (the kernel's dynamic-LDS
    // limit was raised by configure_ffn_kernels)
    const size_t row_bytes = static_cast<size_t>(16) * TFMAX * K * 2;
    const bool rows_in_lds = KSPLIT == 1 && row_bytes <= kStreamRowLdsMax;
    const size_t lds = rows_in_lds ? row_bytes : 0;
    // resident blocks per CU: what registers allow, and what the row tiles in LDS leave room for
    int blocks_per_cu = per_cu;
    if (lds > 0) blocks_per_cu = std::max(1, std::min(per_cu, static_cast<int>(kLdsPerCu / lds)));
    long grid = static_cast<long>(device_cu_count()) * blocks_per_cu;
    if (grid > max_units && partials == nullptr) grid = max_units;   // with partial tiles to add: all blocks
    if (grid < 1) grid = 1;
    // decode-sized tiles (many units per block): balanced grid; larger tiles: every block stays busy
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(256), lds, st, act, rowmap, wpk, outp, tiles,
                       ntiles, N, K, TFMAX <= 2 ? 1 : 0, big_tiles, partials, tile_product_grid(),
                       act_kmajor ? 1 : 0, rows_in_lds ? 1 : 0, bias, fold);
    return hipGetLastError();
}

template <int TFMAX, int FIRST, bool FOLD>
static hipError_t launch_stream_kf(int ksplit, const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk,
                                   void* outp, const Tile* tiles, const int32_t* ntiles, int N, int K,
                                   long max_tiles, const Tile* big_tiles, const float* partials,
                                   bool act_kmajor, const float* bias, const FoldOut& fold, hipStream_t st) {
    const long ngroups = (N / 16 + 3) / 4;
    if (ksplit == 4)
        return launch_stream<TFMAX, 4, FIRST, FOLD>(act, rowmap, wpk, outp, tiles, ntiles, N, K, max_tiles * ngroups,
                                                    big_tiles, partials, act_kmajor, bias, fold, st);
    if (ksplit == 2)
        return launch_stream<TFMAX, 2, FIRST, FOLD>(act, rowmap, wpk, outp, tiles, ntiles, N, K,
                                                    max_tiles * ((ngroups + 1) / 2), big_tiles, partials,
                                                    act_kmajor, bias, fold, st);
    return launch_stream<TFMAX, 1, FIRST, FOLD>(act, rowmap, wpk, outp, tiles, ntiles, N, K,
                                                max_tiles * ((ngroups + 3) / 4), big_tiles, partials,
                                                act_kmajor, bias, fold, st);
}

// the folded form exists for the second product only
template <int TFMAX, int FIRST>
static hipError_t launch_stream_k(int ksplit, const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk,
                                  void* outp, const Tile* tiles, const int32_t* ntiles, int N, int K,
                                  long max_tiles, const Tile* big_tiles, const float* partials,
                                  bool act_kmajor, const float* bias, const FoldOut& fold, hipStream_t st) {
    if constexpr (FIRST == 0) {
        if (fold.out != nullptr)
            return launch_stream_kf<TFMAX, 0, true>(ksplit, act, rowmap, wpk, outp, tiles, ntiles, N, K, max_tiles,
                                                    big_tiles, partials, act_kmajor, bias, fold, st);
    }
    return launch_stream_kf<TFMAX, FIRST, false>(ksplit, act, rowmap, wpk, outp, tiles, ntiles, N, K, max_tiles,
                                                 big_tiles, partials, act_kmajor, bias, fold, st);
}

template <int TFMAX, int KSPLIT, int FIRST, bool FOLD>
static hipError_t configure_stream(int dev) {
    auto kern = ffn_stream_kernel<TFMAX, KSPLIT, FIRST, FOLD>;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, 256, 0) != hipSuccess || n <= 0) n = 1;
    StreamKernelInfo<TFMAX, KSPLIT, FIRST, FOLD>::per_cu[dev] = n;
    if (KSPLIT == 1)
        return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   static_cast<int>(kStreamRowLdsMax));
    return hipSuccess;
}

template <int TFMAX, int KSPLIT>
static hipError_t configure_stream_products(int dev) {
    hipError_t e;
    if ((e = configure_stream<TFMAX, KSPLIT, kFirstRelu, false>(dev)) != hipSuccess) return e;
    if ((e = configure_stream<TFMAX, KSPLIT, kFirstGelu, false>(dev)) != hipSuccess) return e;
    if ((e = configure_stream<TFMAX, KSPLIT, 0, false>(dev)) != hipSuccess) return e;
    return configure_stream<TFMAX, KSPLIT, 0, true>(dev);
}

template <int TFMAX>
static hipError_t configure_stream_splits(int dev) {
    hipError_t e;
    if ((e = configure_stream_products<TFMAX, 1>(dev)) != hipSuccess) return e;
    if ((e = configure_stream_products<TFMAX, 2>(dev)) != hipSuccess) return e;
    return configure_stream_products<TFMAX, 4>(dev);
}

hipError_t configure_ffn_kernels(int dev) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    g_cus[dev] = n;
    hipError_t e;
    if ((e = configure_stream_splits<1>(dev)) != hipSuccess) return e;
    if ((e = configure_stream_splits<2>(dev)) != hipSuccess) return e;
    return configure_stream_splits<4>(dev);
}

// Split K (k-steps of 32) over up to 4 wavefronts.  Decode-sized tiles want many short units
// (>= 16 steps each) for an even spread over the chip; tiles with several row fragments carry more
// per-unit work and keep >= 24 steps per wavefront.  Decode-sized tiles whose rows fit into LDS do not
// split at all when that still leaves two units for every CU (`tiles_expected`: about how many tiles there
// will be): a wavefront then streams its whole contraction in one go, with the rows read from LDS
// (measured on the decode preset, first product: 285 -> 257 us).
#ifndef MOE_KS4_MIN_STEPS
#define MOE_KS4_MIN_STEPS 96
#endif
#ifndef MOE_KS2_MIN_STEPS
#define MOE_KS2_MIN_STEPS 32     // (48 before: with 32 the first product of a d_model = 1024 layer with few small
#endif                           // experts spreads over twice the blocks: 21.7 -> 16.0 us on the Switch-large preset)
static int pick_ksplit(int K, int N, int tfmax, long tiles_expected) {
    const int steps = K / 32;
    if (tfmax <= 2) {
        const bool rows_fit = static_cast<size_t>(16) * tfmax * K * 2 <= kStreamRowLdsMax;
        const long units_unsplit = tiles_expected * ((N / 64 + 3) / 4);
        if (rows_fit && units_unsplit >= 2L * device_cu_count()) return 1;
    }
    const int s4 = tfmax <= 2 ? 64 : MOE_KS4_MIN_STEPS, s2 = tfmax <= 2 ? 32 : MOE_KS2_MIN_STEPS;
    if (steps >= s4) return 4;
    if (steps >= s2) return 2;
    return 1;
}

// events recorded around the two products when a caller asked for them (profiling aid)
static hipEvent_t g_profile_events[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};

void set_profile_events(const hipEvent_t* ev) {
    for (int i = 0; i < 5; ++i) g_profile_events[i] = ev ? ev[i] : nullptr;
}

static hipError_t mark(int i, hipStream_t st) {
    return g_profile_events[i] ? hipEventRecord(g_profile_events[i], st) : hipSuccess;
}

// token fragments per tile: an expert holds at most T rows (a token picks an expert at most once)
static int ffn_tfmax(const moe_shape& s) { return s.T <= 16 ? 1 : (s.T <= 32 ? 2 : 4); }

int ffn_tile_rows(const moe_shape& s) { return s.dtype == MOE_BF16 ? 16 * ffn_tfmax(s) : 16; }

TileLists ffn_tile_lists(const moe_shape& s, Tile* small_ws, Tile* big_ws, int32_t* ntiles_ws, float* partials_ws) {
    TileLists l;
    l.small_tiles = small_ws;
    l.big_tiles = big_ws;
    l.ntiles = ntiles_ws;
    l.small_rows = ffn_tile_rows(s);
    // a large expert needs kBigMinRows rows, and an expert holds at most T rows
    l.big_min = (s.dtype == MOE_BF16 && s.T >= kBigMinRows) ? kBigMinRows : 0;
    l.partials = l.big_min > 0 ? partials_ws : nullptr;
    l.join_tiles = l.big_min > 0 ? tiled_join_tiles(s) : 0;
    return l;
}

// one full round of the tiled kernel's units in the product with the fewer column tiles
int tiled_join_tiles(const moe_shape& s) {
    const int narrow = s.d_model < s.d_ff ? s.d_model : s.d_ff;
    const int col_tiles = (narrow + 255) / 256;
    return (tile_product_grid() + col_tiles - 1) / col_tiles;
}

// the two grouped products over existing tile lists
// The extra pass over the token rows pays once the layer is large (measured: a gain from 4 M elements of
// gathered rows on, a small loss at 1.5 M, where the launch costs more than the better-shaped loads save).
#ifndef MOE_GATHER_MIN_MELEMS
#define MOE_GATHER_MIN_MELEMS 4      // gathered elements (T * k * d_model), in units of 2^20, from which the pass pays
#endif
bool layer_gathers_kmajor(const moe_shape& s) {
    return s.dtype == MOE_BF16 && s.T >= kBigMinRows &&
           static_cast<long>(s.T) * s.k * s.d_model >= (static_cast<long>(MOE_GATHER_MIN_MELEMS) << 20);
}

hipError_t launch_expert_products(const moe_shape& s, const void* act, const int32_t* rowmap, bool act_kmajor,
                                  const void* w1, const void* w2, const float* b1, const float* b2, float* y_perm,
                                  void* h_ws, const TileLists& lists, const FoldOut& fold, hipStream_t st) {
    const int A = s.T * s.k, E = s.E, d = s.d_model, f = s.d_ff;
    const int tile_rows = lists.small_rows;
    const Tile* tiles = lists.small_tiles;
    const int32_t* ntiles = lists.ntiles;
    const long max_tiles = A / tile_rows + (E < A ? E : A);
    const bool big = lists.big_min > 0;
    int32_t* part1 = lists.ntiles + kSplitCounter;
    int32_t* part2 = part1 + 1;
    hipError_t err;
    if ((err = mark(0, st)) != hipSuccess) return err;

    if (s.dtype == MOE_F32) {
        const long g1 = max_tiles * ((f + 255) / 256), g2 = max_tiles * ((d + 255) / 256);
        const long cap = static_cast<long>(device_cu_count()) * 8;
        if ((err = mark(1, st)) != hipSuccess) return err;
        hipLaunchKernelGGL(ffn_f32_kernel<true>, dim3(static_cast<unsigned>(g1 < cap ? g1 : cap)), dim3(256), 0, st,
                           static_cast<const float*>(act), rowmap, static_cast<const float*>(w1),
                           static_cast<float*>(h_ws), tiles, ntiles, f, d, s.activation, b1);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
        if ((err = mark(2, st)) != hipSuccess || (err = mark(3, st)) != hipSuccess) return err;
        hipLaunchKernelGGL(ffn_f32_kernel<false>, dim3(static_cast<unsigned>(g2 < cap ? g2 : cap)), dim3(256), 0, st,
                           static_cast<const float*>(h_ws), static_cast<const int32_t*>(nullptr),
                           static_cast<const float*>(w2), y_perm, tiles, ntiles, d, f, s.activation, b2);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
        return mark(4, st);
    }

    const uint16_t* xp = static_cast<const uint16_t*>(act);
    const uint16_t* p1 = static_cast<const uint16_t*>(w1);
    const uint16_t* p2 = static_cast<const uint16_t*>(w2);
    uint16_t* h = static_cast<uint16_t*>(h_ws);
    const long tiles_expected = A < E ? A : E;      // every assignment on its own expert, at most E of them
    const int ks1 = pick_ksplit(d, f, ffn_tfmax(s), tiles_expected), ks2 = pick_ksplit(f, d, ffn_tfmax(s), tiles_expected);
    const Tile* bt = lists.big_tiles;
    const float* pt = big ? lists.partials : nullptr;
    // Per product: the tiled kernel (large experts) first, then the streaming kernel (small experts), which
    // also adds up the partial tiles that the tiled kernel left for the units it cut along K.
    if (big) {
        err = launch_tile_product(true, xp, rowmap, p1, h, bt, ntiles + 1, part1, lists.partials, f, d, act_kmajor, s.activation, b1,
                                  FoldOut{nullptr, nullptr, nullptr}, st);
        if (err != hipSuccess) return err;
    }
    if ((err = mark(1, st)) != hipSuccess) return err;
    const bool gelu = s.activation == MOE_ACT_GELU;
    switch (ffn_tfmax(s) * 2 + (gelu ? 1 : 0)) {
        case 2: err = launch_stream_k<1, kFirstRelu>(ks1, xp, rowmap, p1, h, tiles, ntiles, f, d, max_tiles, bt, pt, act_kmajor, b1, FoldOut{nullptr, nullptr, nullptr}, st); break;
        case 3: err = launch_stream_k<1, kFirstGelu>(ks1, xp, rowmap, p1, h, tiles, ntiles, f, d, max_tiles, bt, pt, act_kmajor, b1, FoldOut{nullptr, nullptr, nullptr}, st); break;
        case 4: err = launch_stream_k<2, kFirstRelu>(ks1, xp, rowmap, p1, h, tiles, ntiles, f, d, max_tiles, bt, pt, act_kmajor, b1, FoldOut{nullptr, nullptr, nullptr}, st); break;
        case 5: err = launch_stream_k<2, kFirstGelu>(ks1, xp, rowmap, p1, h, tiles, ntiles, f, d, max_tiles, bt, pt, act_kmajor, b1, FoldOut{nullptr, nullptr, nullptr}, st); break;
        case 8: err = launch_stream_k<4, kFirstRelu>(ks1, xp, rowmap, p1, h, tiles, ntiles, f, d, max_tiles, bt, pt, act_kmajor, b1, FoldOut{nullptr, nullptr, nullptr}, st); break;
        default: err = launch_stream_k<4, kFirstGelu>(ks1, xp, rowmap, p1, h, tiles, ntiles, f, d, max_tiles, bt, pt, act_kmajor, b1, FoldOut{nullptr, nullptr, nullptr}, st); break;
    }
    if (err != hipSuccess) return err;
    if ((err = mark(2, st)) != hipSuccess) return err;
    if (big) {
        err = launch_tile_product(false, h, nullptr, p2, y_perm, bt, ntiles + 1, part2, lists.partials, d, f, true, s.activation, b2, fold, st);
        if (err != hipSuccess) return err;
    }
    if ((err = mark(3, st)) != hipSuccess) return err;
    // few tokens and few experts: units of one column block, so that every CU has one
    const bool narrow = ffn_tfmax(s) == 1 && ks2 == 4 && fold.out == nullptr && pt == nullptr &&
                        tiles_expected * ((d / 16 + 3) / 4) < device_cu_count();
    if (narrow) {
        long grid = max_tiles * (d / 16);
        if (grid > device_cu_count()) grid = device_cu_count();
        hipLaunchKernelGGL(ffn_stream_narrow_kernel, dim3(static_cast<unsigned>(grid < 1 ? 1 : grid)), dim3(256), 0, st, h, p2,
                           static_cast<void*>(y_perm), tiles, ntiles, d, f, b2);
        if ((err = hipGetLastError()) != hipSuccess) return err;
        return mark(4, st);
    }
    switch (ffn_tfmax(s)) {
        case 1: err = launch_stream_k<1, 0>(ks2, h, nullptr, p2, y_perm, tiles, ntiles, d, f, max_tiles, bt, pt, true, b2, fold, st); break;
        case 2: err = launch_stream_k<2, 0>(ks2, h, nullptr, p2, y_perm, tiles, ntiles, d, f, max_tiles, bt, pt, true, b2, fold, st); break;
        default: err = launch_stream_k<4, 0>(ks2, h, nullptr, p2, y_perm, tiles, ntiles, d, f, max_tiles, bt, pt, true, b2, fold, st); break;
    }
    if (err != hipSuccess) return err;
    return mark(4, st);
}

hipError_t launch_expert_ffn(const moe_shape& s, const void* x_perm, const void* w1, const void* w2,
                             const float* b1, const float* b2,
                             const int32_t* offsets, const uint8_t* mask, float* y_perm, void* h_ws,
                             Tile* tiles_ws, Tile* tiles_big_ws, int32_t* ntiles_ws, float* partials_ws,
                             void* x_kmajor_ws, hipStream_t st) {
    const TileLists lists = ffn_tile_lists(s, tiles_ws, tiles_big_ws, ntiles_ws, partials_ws);
    hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(1024), 0, st, offsets, mask, s.E, s.T * s.k, lists);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (layer_gathers_kmajor(s)) {      // large layer: re-lay the permuted rows k-step-major first
        err = launch_gather_kmajor(s, x_perm, nullptr, x_kmajor_ws, st);
        if (err != hipSuccess) return err;
        return launch_expert_products(s, x_kmajor_ws, nullptr, true, w1, w2, b1, b2, y_perm, h_ws, lists,
                                      FoldOut{nullptr, nullptr, nullptr}, st);
    }
    return launch_expert_products(s, x_perm, nullptr, false, w1, w2, b1, b2, y_perm, h_ws, lists,
                                  FoldOut{nullptr, nullptr, nullptr}, st);
}

}  // namespace moe
