// Schedule of the LDS-tiled product over the (row tile, column tile) units of the large experts, shared
// by the kernel that runs it (ffn_tile.hip) and the kernel that finishes it (ffn.hip).
//
// All units cost the same.  G blocks run U / G full rounds of whole units in a fixed, XCD-aware order.
// The R = U mod G units left over would keep R blocks busy for a whole round and the rest of the chip
// idle, so each of them is cut along K into `split` parts; blocks take parts from a counter as they
// become free, and every part leaves an fp32 partial tile in the workspace.  The partial tiles are added
// up in part order -- whichever block computed them -- by the next kernel on the stream: the kernel
// boundary makes them visible across the XCDs' L2s without any fence.
#pragma once
#include "common.hpp"

namespace moe {

constexpr int kTileCols = 256;      // columns per unit (rows: kBigTileRows)
constexpr int kMaxSplit = 8;        // parts per left-over unit, at most ...
#ifndef MOE_MIN_SPLIT_STEPS
#define MOE_MIN_SPLIT_STEPS 32
#endif
constexpr int kMinSplitSteps = MOE_MIN_SPLIT_STEPS;  // ... and 32-k steps per part, at least

struct TileSchedule {
    int ntiles, ntn;    // row tiles, column tiles
    int rounds, R;      // full rounds of G units; units left over
    int split;          // parts per left-over unit (1: not cut, written directly)
    int GM, GN;         // patch of consecutive units: GM row tiles x GN column tiles
};

#ifdef __HIPCC__
__device__ __forceinline__ TileSchedule tile_schedule(int ntiles, int N, int kblk, int G, bool have_partials) {
    TileSchedule s;
    s.ntiles = ntiles;
    s.ntn = (N + kTileCols - 1) / kTileCols;
    const int U = ntiles * s.ntn;
    s.rounds = U / G;
    s.R = U - s.rounds * G;
    s.split = 1;
    if (s.R > 0 && have_partials) {
        const int by_blocks = G / s.R, by_steps = kblk / kMinSplitSteps, by_slots = kSplitSlots / s.R;
        s.split = min(min(by_blocks, kMaxSplit), min(by_steps, by_slots));
        if (s.split < 2) s.split = 1;
    }
    s.GN = min(s.ntn, 8);
    s.GM = (G % 8 == 0 && (G / 8) % s.GN == 0) ? (G / 8) / s.GN : 1;
    return s;
}

// Unit u of the ntiles x ntn grid.  Units are numbered so that a run of consecutive units is a compact
// patch: column tiles in groups of GN, and inside a group GM row tiles at a time.  Every u in
// [0, ntiles * ntn) maps to exactly one (row tile, column tile).
__device__ __forceinline__ void unit_of(const TileSchedule& s, int u, int& mt, int& nt) {
    const int per_group = s.ntiles * s.GN;
    const int cg = u / per_group;                       // the last group may hold fewer than GN columns
    const int wn = min(s.GN, s.ntn - cg * s.GN);
    const int v = u - cg * per_group;                   // < ntiles * wn
    const int chunk = v / (s.GM * wn), slot = v - chunk * (s.GM * wn);
    mt = chunk * s.GM + slot / wn;                      // < ntiles, also in a last, shorter chunk
    nt = cg * s.GN + slot % wn;
}

// 4 values of one output row, columns n ... n + 3 (n a multiple of 4).  FIRST != 0 (first product; the value
// names the activation, kFirstRelu or kFirstGelu): activation, bf16, into the blocked h of N columns; FIRST == 0 (second product): fp32 into row-major y of N columns.  `bias`: the expert's N bias values
// (fp32) or NULL, added before the activation / the store.  STREAMED: the store carries the non-temporal
// hint, so the rows go to memory while the kernel runs instead of staying behind as dirty L2 lines that the
// next kernel's weight stream has to push out (the streaming kernel's stores; measured on the Switch-base
// preset: following product 65 -> 62 us; no effect on the fp32 rows of the second product, which are stored
// plainly).  The tiled kernel's rows are re-read from L2 and are stored plainly.
template <int FIRST, bool STREAMED = false>
__device__ __forceinline__ void store_out(void* outp, int row, int n, int N, const float* bias,
                                          f32x4 v) {
    if (bias != nullptr) v += *reinterpret_cast<const f32x4*>(bias + n);
    if (FIRST) {
        const f32x4 z = activate4<FIRST == kFirstGelu ? MOE_ACT_GELU : MOE_ACT_RELU>(v);
        uint2 pk;
        pk.x = pack_bf16x2(z[0], z[1]);
        pk.y = pack_bf16x2(z[2], z[3]);
        uint32_t* q = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(outp) + h_index(row, n, N >> 5));
        if (STREAMED) {
            __builtin_nontemporal_store(pk.x, q);      // merged into one 8-byte store
            __builtin_nontemporal_store(pk.y, q + 1);
        } else {
            *reinterpret_cast<uint2*>(q) = pk;
        }
    } else {
        *reinterpret_cast<f32x4*>(static_cast<float*>(outp) + static_cast<size_t>(row) * N + n) = v;
    }
}

// Second-product output of a row whose layer output is written directly (FoldOut): 4 columns n ... n + 3 of
// out[t], t and the row's gate weight w looked up by the caller.  fmaf(w, y, 0) and one rounding to bf16: what
// the combine step does for a token with a single expert.
__device__ __forceinline__ void store_folded(uint16_t* out, int t, float w, int n, int N, const float* bias, f32x4 v) {
    if (bias != nullptr) v += *reinterpret_cast<const f32x4*>(bias + n);
    uint2 pk;
    pk.x = pack_bf16x2(fmaf(w, v[0], 0.f), fmaf(w, v[1], 0.f));
    pk.y = pack_bf16x2(fmaf(w, v[2], 0.f), fmaf(w, v[3], 0.f));
    *reinterpret_cast<uint2*>(out + static_cast<size_t>(t) * N + n) = pk;
}

// First-product output of two adjacent 16-column blocks (columns n0 ... n0 + 31: one k-step block of h) for
// the 16 rows of an accumulator pair.  Called by a whole wavefront (no divergence around it): lane (r, g),
// r = lane % 16 the row, g = lane / 16, holds columns n0 + 4g ... + 3 in v0 and n0 + 16 + 4g ... + 3 in v1.
// After activation and rounding, one v_permlane16_swap per packed register trades the odd 16-lane rows of the
// first block with the even rows of the second, which leaves every lane with 8 consecutive columns of its
// row: the wavefront's store is one contiguous KiB of h (16 rows x 64 bytes) instead of two stores of
// 32-byte pieces.  `row_ok`: the lane's row exists (the others take part in the exchange only).
template <int FIRST, bool STREAMED>
__device__ __forceinline__ void store_h_pair(void* outp, int row, bool row_ok, int n0, int N,
                                             const float* bias, f32x4 v0, f32x4 v1) {
    static_assert(FIRST != 0, "first product only");
    const int g = (threadIdx.x & 63) >> 4;
    if (bias != nullptr) {
        v0 += *reinterpret_cast<const f32x4*>(bias + n0 + g * 4);
        v1 += *reinterpret_cast<const f32x4*>(bias + n0 + 16 + g * 4);
    }
    constexpr int ACT = FIRST == kFirstGelu ? MOE_ACT_GELU : MOE_ACT_RELU;
    const f32x4 z0 = activate4<ACT>(v0), z1 = activate4<ACT>(v1);
    const auto lo = __builtin_amdgcn_permlane16_swap(pack_bf16x2(z0[0], z0[1]), pack_bf16x2(z1[0], z1[1]), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(pack_bf16x2(z0[2], z0[3]), pack_bf16x2(z1[2], z1[3]), false, false);
    // even g: columns 4g ... 4g + 7 of the first block; odd g: columns 4(g-1) ... + 7 of the second
    const int n = n0 + (g & 1) * 16 + (g & 2) * 4;
    if (!row_ok) return;
    uint32_t* q = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(outp) + h_index(row, n, N >> 5));
    if (STREAMED) {
        __builtin_nontemporal_store(lo[0], q);             // merged into one 16-byte store
        __builtin_nontemporal_store(hi[0], q + 1);
        __builtin_nontemporal_store(lo[1], q + 2);
        __builtin_nontemporal_store(hi[1], q + 3);
    } else {
        *reinterpret_cast<uint4*>(q) = uint4{lo[0], hi[0], lo[1], hi[1]};
    }
}

// store_folded for two adjacent 16-column blocks (columns n0 ... n0 + 31) of the 16 rows of an accumulator
// pair, by a whole wavefront, with the lane exchange of store_h_pair: every lane ends up with 8 consecutive
// columns of its row, one 16-byte store (64 contiguous bytes per token row and instruction).  The output is
// not read again by the layer: non-temporal.
__device__ __forceinline__ void store_folded_pair(uint16_t* out, int t, float w, bool row_ok, int n0, int N,
                                                  const float* bias, f32x4 v0, f32x4 v1) {
    const int g = (threadIdx.x & 63) >> 4;
    if (bias != nullptr) {
        v0 += *reinterpret_cast<const f32x4*>(bias + n0 + g * 4);
        v1 += *reinterpret_cast<const f32x4*>(bias + n0 + 16 + g * 4);
    }
    const auto lo = __builtin_amdgcn_permlane16_swap(pack_bf16x2(fmaf(w, v0[0], 0.f), fmaf(w, v0[1], 0.f)),
                                                     pack_bf16x2(fmaf(w, v1[0], 0.f), fmaf(w, v1[1], 0.f)), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(pack_bf16x2(fmaf(w, v0[2], 0.f), fmaf(w, v0[3], 0.f)),
                                                     pack_bf16x2(fmaf(w, v1[2], 0.f), fmaf(w, v1[3], 0.f)), false, false);
    const int n = n0 + (g & 1) * 16 + (g & 2) * 4;
    if (!row_ok) return;
    uint32_t* q = reinterpret_cast<uint32_t*>(out + static_cast<size_t>(t) * N + n);
    __builtin_nontemporal_store(lo[0], q);                 // merged into one 16-byte store
    __builtin_nontemporal_store(hi[0], q + 1);
    __builtin_nontemporal_store(lo[1], q + 2);
    __builtin_nontemporal_store(hi[1], q + 3);
}

// ---- outputs of the tiled product's 32 x 32 accumulators (v_mfma_f32_32x32x16_bf16) --------------------
// Lane l of a wavefront holds, for token row l % 32 of the block, the output columns n0 + 8 q + 4 (l / 32) + i
// in accumulator register 4 q + i (q, i = 0 ... 3): four groups of four consecutive columns.

// First product: activation, bf16, into the blocked h.  The 32 columns of the block are one k-step group of h
// (64 bytes per row).  After rounding, lanes l and l + 32 (same row) trade two of their four column groups with
// v_permlane32_swap, which leaves the lower lane with columns 0 ... 15 and the upper lane with 16 ... 31: 32
// contiguous bytes per lane, and the wavefront's two stores cover 2 KiB of consecutive rows.  Called by a whole
// wavefront (no divergence around it); `row_ok`: the lane's row exists.
template <int FIRST>
__device__ __forceinline__ void store_h_block32(void* outp, int row, bool row_ok, int n0, int N, const float* bias,
                                                const f32x16& acc) {
    static_assert(FIRST != 0, "first product only");
    constexpr int ACT = FIRST == kFirstGelu ? MOE_ACT_GELU : MOE_ACT_RELU;
    const int L = (threadIdx.x & 63) >> 5;
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f32x4 v = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        if (bias != nullptr) v += *reinterpret_cast<const f32x4*>(bias + n0 + 8 * q + 4 * L);
        const f32x4 z = activate4<ACT>(v);
        lo[q] = pack_bf16x2(z[0], z[1]);
        hi[q] = pack_bf16x2(z[2], z[3]);
    }
    const auto s0 = __builtin_amdgcn_permlane32_swap(lo[0], lo[2], false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(hi[0], hi[2], false, false);
    const auto s2 = __builtin_amdgcn_permlane32_swap(lo[1], lo[3], false, false);
    const auto s3 = __builtin_amdgcn_permlane32_swap(hi[1], hi[3], false, false);
    if (!row_ok) return;
    uint4* q = reinterpret_cast<uint4*>(static_cast<uint16_t*>(outp) + h_index(row, n0 + 16 * L, N >> 5));
    q[0] = uint4{s0[0], s1[0], s0[1], s1[1]};
    q[1] = uint4{s2[0], s3[0], s2[1], s3[1]};
}

// Second product whose rows are the layer output (FoldOut): gate weight times the row, one rounding to bf16
// (what the combine step does for a token with a single expert), the same lane exchange, 32 contiguous bytes
// of out[t] per lane; not read again by the layer: non-temporal.
__device__ __forceinline__ void store_folded_block32(uint16_t* out, int t, float w, bool row_ok, int n0, int N,
                                                     const float* bias, const f32x16& acc) {
    const int L = (threadIdx.x & 63) >> 5;
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f32x4 v = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        if (bias != nullptr) v += *reinterpret_cast<const f32x4*>(bias + n0 + 8 * q + 4 * L);
        lo[q] = pack_bf16x2(fmaf(w, v[0], 0.f), fmaf(w, v[1], 0.f));
        hi[q] = pack_bf16x2(fmaf(w, v[2], 0.f), fmaf(w, v[3], 0.f));
    }
    const auto s0 = __builtin_amdgcn_permlane32_swap(lo[0], lo[2], false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(hi[0], hi[2], false, false);
    const auto s2 = __builtin_amdgcn_permlane32_swap(lo[1], lo[3], false, false);
    const auto s3 = __builtin_amdgcn_permlane32_swap(hi[1], hi[3], false, false);
    if (!row_ok) return;
    uint32_t* q = reinterpret_cast<uint32_t*>(out + static_cast<size_t>(t) * N + n0 + 16 * L);
    const uint32_t v8[8] = {s0[0], s1[0], s0[1], s1[1], s2[0], s3[0], s2[1], s3[1]};
#pragma unroll
    for (int i = 0; i < 8; ++i) __builtin_nontemporal_store(v8[i], q + i);     // merged into two 16-byte stores
}

// Adds up the partial tiles that a tiled product of grid G left behind and writes the output rows.
// Called by every thread of `nblocks` blocks of the following kernel, `block` being the caller's rank among
// them.  A wavefront takes four consecutive rows of a
// cut unit at a time (a row of a unit is 256 columns: 4 per lane): what is the same for the whole row -- the unit,
// its row tile, for a folded output the row's token and gate weight -- is looked up once per wavefront, and the
// 4 x split loads of partial sums go out together (one row at a time, with a lookup per element, the pass was a
// chain of dependent trips to memory: 35 of the 50 us of the kernel that did it on the Switch-large preset).
template <int FIRST, bool FOLD>
__device__ __forceinline__ void finish_split_units(const Tile* __restrict__ big_tiles, int ntiles_big,
                                                   const float* __restrict__ partials, void* __restrict__ outp,
                                                   int N, int kblk, int G,
                                                   const float* __restrict__ bias, const FoldOut fold, int block,
                                                   int nblocks) {
    if (ntiles_big <= 0 || partials == nullptr) return;
    const TileSchedule s = tile_schedule(ntiles_big, N, kblk, G, true);
    if (s.split < 2) return;
    constexpr int kRowsAtOnce = 4;
    constexpr int kGroups = kBigTileRows / kRowsAtOnce;         // row groups per unit
    constexpr size_t kTileFloats = static_cast<size_t>(kBigTileRows) * kTileCols;
    const int lane = threadIdx.x & 63;
    const int waves_per_block = blockDim.x >> 6;
    const int first = __builtin_amdgcn_readfirstlane(block * waves_per_block + static_cast<int>(threadIdx.x >> 6));
    const int nwaves = nblocks * waves_per_block;
    const int total = s.R * kGroups;
    for (int i = first; i < total; i += nwaves) {              // wave-uniform
        const int ru = i / kGroups, lr0 = (i % kGroups) * kRowsAtOnce;
        int mt, nt;
        unit_of(s, s.rounds * G + ru, mt, nt);
        const Tile tl = big_tiles[mt];
        if (lr0 >= tl.rows) continue;
        const int c = nt * kTileCols + lane * 4;
        const float* base = partials + static_cast<size_t>(ru) * s.split * kTileFloats + static_cast<size_t>(lr0) * kTileCols + lane * 4;
        f32x4 sum[kRowsAtOnce];
        int tok[kRowsAtOnce];
#pragma unroll
        for (int q = 0; q < kRowsAtOnce; ++q) {
            sum[q] = *reinterpret_cast<const f32x4*>(base + q * kTileCols);
            tok[q] = (FOLD && lr0 + q < tl.rows) ? fold.tokmap[tl.row0 + lr0 + q] : 0;
        }
        for (int p = 1; p < s.split; ++p) {                    // in part order, whichever block computed the parts
#pragma unroll
            for (int q = 0; q < kRowsAtOnce; ++q)
                sum[q] += *reinterpret_cast<const f32x4*>(base + static_cast<size_t>(p) * kTileFloats + q * kTileCols);
        }
        const float* be = bias ? bias + static_cast<size_t>(tl.expert) * N : nullptr;
#pragma unroll
        for (int q = 0; q < kRowsAtOnce; ++q) {
            if (lr0 + q >= tl.rows || c >= N) continue;
            if constexpr (FOLD) {
                store_folded(fold.out, tok[q], fold.gate[tok[q]], c, N, be, sum[q]);
            } else {
                store_out<FIRST>(outp, tl.row0 + lr0 + q, c, N, be, sum[q]);
            }
        }
    }
}
#endif

}  // namespace moe
