// Shared declarations of the MoE FFN library for gfx950: storage helpers, the
// workspace layout and the internal launch functions that the C ABI composes.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

// ---- bf16 storage <-> fp32 ------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round to nearest, ties to even; NaN stays NaN: the hardware conversion (v_cvt_pk_bf16_f32), two values
// per instruction
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return static_cast<uint16_t>(pack_bf16x2(f, 0.f) & 0xffffu); }

template <typename ST> struct Storage;
template <> struct Storage<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Storage<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16(v); }
};

// ---- expert tiles: the unit the FFN kernels schedule ------------------------
// A tile is up to `tile_rows` consecutive rows of one expert's segment of x_perm.
struct Tile {
    int32_t expert;
    int32_t row0;    // first row in x_perm / h / y_perm
    int32_t rows;    // 1 .. tile_rows
    int32_t pad;
};

// Tiles of experts with at least kBigMinRows rows go to the LDS-tiled MFMA kernel (tiles of
// kBigTileRows rows); smaller experts are weight-streaming work.
constexpr int kBigTileRows = 256;
constexpr int kBigMinRows = 128;
// Experts between one streaming tile and kBigMinRows rows would have their weights streamed once per
// streaming tile; as one mostly empty tile of the tiled kernel they cost about what a single pass over their
// weights costs -- as long as the tiled kernel has whole rounds of units to run anyway, which hide the one
// more unit per column tile.  They join the large experts when the tiles of the experts with kBigMinRows rows
// already number `join_tiles` (the host's figure: one full round of units in the narrower product); with
// fewer, an under-filled tiled kernel would only get longer.
inline __host__ __device__ int tiled_min_rows(int big_tiles_at_min, int small_rows, int join_tiles) {
    return (join_tiles > 0 && big_tiles_at_min >= join_tiles) ? small_rows + 1 : kBigMinRows;
}
// The LDS-tiled kernel cuts the units of its last, partly filled round along K; the parts leave fp32
// partial tiles (kBigTileRows x 256) in the workspace and are handed out through a counter.
constexpr int kSplitSlots = 256;        // partial tiles in the workspace
constexpr int kSplitCounter = 2;        // ints [2] and [3] of the `ntiles` array: the part counters of the
                                        // first and of the second product

// trailing activation of the first linear layer (Section 3.4): 0 = ReLU, 1 = GeLU in its defining form
// z * Phi(z) = 0.5 z (1 + erf(z / sqrt 2))
#ifdef __HIPCC__
__device__ __forceinline__ float gelu_erf(float z) { return 0.5f * z * (1.f + erff(z * 0.70710678118654752f)); }

__device__ __forceinline__ float activate(float z, int act) { return act == MOE_ACT_GELU ? gelu_erf(z) : fmaxf(z, 0.f); }

// Four values at once, the activation a compile-time constant: the MFMA kernels are instantiated per
// activation (as a run-time choice in their epilogues it cost the ReLU layers 5-10 % of the kernel).
template <int ACT>
__device__ __forceinline__ f32x4 activate4(f32x4 v) {
    if (ACT == MOE_ACT_GELU) return f32x4{gelu_erf(v[0]), gelu_erf(v[1]), gelu_erf(v[2]), gelu_erf(v[3])};
    return f32x4{fmaxf(v[0], 0.f), fmaxf(v[1], 0.f), fmaxf(v[2], 0.f), fmaxf(v[3], 0.f)};
}

// template argument FIRST of the product kernels: 0 = second product, else first product with ...
constexpr int kFirstRelu = 1;
constexpr int kFirstGelu = 2;
#endif

// Layout of the bf16 row operands that the products read 32 k at a time (the intermediate
// h = act(x . W1^T) and the gathered token rows): blocks of kRowBlock rows, and inside a block k-step-major,
// [rows / 256][K / 32][256][32].  The 32 values of consecutive rows are 64 bytes apart, so a 16-row MFMA
// operand fragment is one contiguous KiB (row-major, each row would contribute half a cache line), a row
// tile of one k-step is at most two contiguous runs, and consecutive k-steps of a row are 16 KiB apart: a
// block that walks along K reads one linear stream.  (With the k-step outermost over all A rows, [K / 32][A][32],
// consecutive steps of a 32 k-row layer were 2 MiB apart and the global-to-LDS copies of the tiled kernel ran
// at two thirds of the rate they reach on a linear stream.)  Element (row, n) of a tensor with `ksteps` = K / 32:
constexpr int kRowBlock = 256;
#ifdef __HIPCC__
__device__ __forceinline__ size_t h_index(int row, int n, int ksteps) {
    return ((static_cast<size_t>(row >> 8) * ksteps + (n >> 5)) * kRowBlock + (row & (kRowBlock - 1))) * 32 + (n & 31);
}
constexpr int kStepStride = kRowBlock * 32;     // elements between consecutive k-steps of a row
#endif

#ifdef __HIPCC__
typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

// byte address inside LDS of a pointer to __shared__ memory
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return static_cast<uint32_t>(reinterpret_cast<size_t>((lptr_t)(p)));
}

// 16 bytes per lane from global memory straight into LDS at `lds_base + 16 * lane` (no registers);
// `lds_base` (an LDS byte address) is the same for the whole wavefront and goes into M0.  Written as inline assembly: after the
// compiler's own builtin for this instruction it makes every later wait for an LDS read a wait for all
// outstanding LDS reads (as long as a copy is in flight, which here is always), and the loops that
// use it depend on waiting only for the oldest ones.  The copies are counted by vmcnt; the code waits for
// them explicitly, and orders them against LDS reads with barriers.  M0 is not live across statements
// in compiled code for this target (the compiler sets it right before each use of its own); it cannot be named
// in the clobber list, the compiler rejects reserved registers there ("may not be preserved across the asm
// statement"), so that property is what the statement relies on.
__device__ __forceinline__ void copy16_to_lds(const void* src, uint32_t lds_base) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(dst) : "memory");
}

#endif

struct TileLists {
    Tile* small_tiles;     // capacity A / small_rows + E
    Tile* big_tiles;       // capacity A / kBigTileRows + E (unused when big_min == 0)
    int32_t* ntiles;       // [0] small count, [1] big count, [2], [3] part counters of the tiled products
    float* partials;       // kSplitSlots partial tiles (nullptr when big_min == 0)
    int small_rows;        // rows per small tile
    int big_min;           // experts with >= big_min rows are "big"; 0 = none
    int join_tiles;        // tiles of big experts from which the mid-sized experts join them (tiled_min_rows); 0 = never
};

#ifdef __HIPCC__
// Places one chunk of consecutive flat assignment ids (counting sort, last step): called by one whole
// wavefront.  `next` (LDS, E ints, private to the wavefront) holds each expert's first free slot for this
// chunk and is advanced.  The wavefront walks its chunk 64 flat ids at a time; lanes that hold the same
// expert find each other with one ballot per bit of the expert id, take consecutive slots in lane order,
// and the last of them advances the expert's slot.  Writes (each may be NULL) perm[pos] = a,
// inv_perm[a] = pos, tokmap[pos] = a / k.
__device__ __forceinline__ void place_chunk(const int32_t* __restrict__ idx, int32_t* next,
                                            int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                            int32_t* __restrict__ tokmap, int A, int E, int k, int ebits, int chunk,
                                            int c) {
    const int lane = threadIdx.x & 63;
    const int base = c * chunk;
    for (int i0 = 0; i0 < chunk; i0 += 64) {
        const int a = base + i0 + lane;
        const bool live = (i0 + lane < chunk) && a < A;
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
        __builtin_amdgcn_wave_barrier();
        const bool last = live && ((same >> lane) >> 1) == 0;   // no higher lane with this expert
        if (last) next[e] = pos + 1;
        __builtin_amdgcn_wave_barrier();
        if (live && pos >= 0 && pos < A) {   // offsets that do not belong to idx must not fault
            if (perm) perm[pos] = a;
            if (inv_perm) inv_perm[a] = pos;
            if (tokmap) tokmap[pos] = a / k;
        }
    }
}

// Inclusive prefix sum over the 1024 threads of a block (thread e contributes v): shuffles inside each
// wavefront, one LDS round for the 16 wavefront totals.  `tmp` is an LDS array of >= 16 ints; two barriers.
__device__ __forceinline__ int block_scan_1024(int v, int32_t* tmp) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const int o = __shfl_up(incl, s);
        if (lane >= s) incl += o;
    }
    __syncthreads();                       // tmp may still be read from a previous call
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += tmp[w];
    return base + incl;
}

// Called by all 1024 threads of a block, thread e owning expert e (row0, m rows; m = 0 when the
// expert is empty or masked out).  `scan` is an LDS array of MOE_MAX_E ints.
__device__ __forceinline__ void emit_tiles(int e, int row0, int m, const TileLists tl, int32_t* scan) {
    int min_rows = tl.big_min;
    if (tl.big_min > 0 && tl.join_tiles > 0) {
        // tiles of the experts that are large in any case, summed over the block
        const int incl = block_scan_1024(m >= tl.big_min ? (m + kBigTileRows - 1) / kBigTileRows : 0, scan);
        __syncthreads();
        if (threadIdx.x == 1023) scan[16] = incl;
        __syncthreads();
        min_rows = tiled_min_rows(scan[16], tl.small_rows, tl.join_tiles);
    }
    const bool big = tl.big_min > 0 && m >= min_rows;
    for (int pass = 0; pass < 2; ++pass) {
        const int rows = pass == 0 ? tl.small_rows : kBigTileRows;
        const bool mine = (pass == 1) == big;
        const int nt = mine ? (m + rows - 1) / rows : 0;
        const int incl = block_scan_1024(nt, scan);
        Tile* out = pass == 0 ? tl.small_tiles : tl.big_tiles;
        const int base = incl - nt;
        for (int i = 0; i < nt; ++i) {
            Tile t;
            t.expert = e;
            t.row0 = row0 + i * rows;
            t.rows = min(rows, m - i * rows);
            t.pad = 0;
            out[base + i] = t;
        }
        if (e == MOE_MAX_E - 1) tl.ntiles[pass] = incl;
        if (pass == 0 && e < 2) tl.ntiles[kSplitCounter + e] = 0;
        if (tl.big_min <= 0 && pass == 0) {      // no large experts possible
            if (e == 0) tl.ntiles[1] = 0;
            break;
        }
    }
}
#endif

// ---- workspace ----------------------------------------------------------------
struct WsLayout {
    size_t hist;       // int32 [ceil(T/16), E]  chunk histograms / slot bases of the counting sort
    size_t ntiles;     // int32 [64]  ([0] = tiles of small experts, [1] = of large experts, [2], [3] counters)
    size_t tiles;      // Tile [A/16 + E + 1]   row tiles of the weight-streaming kernel
    size_t tiles_big;  // Tile [A/256 + E + 1]  row tiles of the LDS-tiled kernel
    size_t h;          // dtype [A rounded up to kRowBlock, f]
    size_t idx;        // int32 [A]         -- the rest is used by moe_layer_forward only
    size_t gate;       // float [A]
    size_t counts;     // int32 [E]
    size_t offsets;    // int32 [E + 1]
    size_t perm;       // int32 [A]
    size_t inv_perm;   // int32 [A]
    size_t mask;       // uint8 [E]
    size_t tokmap;     // int32 [A]  token row of each permuted position
    size_t y_perm;     // float [A, d]
    size_t partials;   // float [kSplitSlots, 256, 256]  (only when an expert can reach kBigMinRows rows)
    size_t x_kmajor;   // bf16 [A rounded up to kRowBlock, d]  gathered token rows in the blocked layout (same condition)
    size_t gate_part;  // float [kGateSplit, T rounded up to 16, E]  partial gate logits (layers with route_is_split)
    size_t total;
};

// Layers with few tokens (decode steps) cut the gate product over many one-wavefront blocks and along the
// contraction into kGateSplit slices (partial logits in the workspace).  Measured: a gain up to 64 tokens
// (one block per 16 tokens leaves reading the gate weights to a few CUs), none at 2048 tokens.
constexpr int kGateSplit = 8;
#ifndef MOE_SPLIT_ROUTE_TOKENS
#define MOE_SPLIT_ROUTE_TOKENS 64
#endif
constexpr int kSplitRouteTokens = MOE_SPLIT_ROUTE_TOKENS;
inline bool route_is_split(const moe_shape& s) { return s.dtype == MOE_BF16 && s.T <= kSplitRouteTokens; }
constexpr int kPermChunk = 256;   // assignments per counting-sort chunk (one wavefront)

inline size_t elem_size(int32_t dtype) { return dtype == MOE_BF16 ? 2 : 4; }

inline WsLayout ws_layout(const moe_shape& s) {
    WsLayout L{};
    const size_t A = static_cast<size_t>(s.T) * s.k, E = s.E, es = elem_size(s.dtype);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off += (bytes + 255) & ~static_cast<size_t>(255);
        return at;
    };
    L.hist = take(((static_cast<size_t>(s.T) + 15) / 16 + 1) * E * 4);
    L.ntiles = take(64 * 4);
    L.tiles = take((A / 16 + E + 1) * sizeof(Tile));
    L.tiles_big = take((A / 256 + E + 1) * sizeof(Tile));
    const size_t Ab = (A + kRowBlock - 1) / kRowBlock * kRowBlock;     // the blocked layouts hold whole row blocks
    L.h = take(Ab * s.d_ff * es);
    L.idx = take(A * 4);
    L.gate = take(A * 4);
    L.counts = take(E * 4);
    L.offsets = take((E + 1) * 4);
    L.perm = take(A * 4);
    L.inv_perm = take(A * 4);
    L.mask = take(E);
    L.tokmap = take(A * 4);
    L.y_perm = take(A * s.d_model * 4);
    const bool big = s.dtype == MOE_BF16 && s.T >= kBigMinRows;
    L.partials = take(big ? static_cast<size_t>(kSplitSlots) * kBigTileRows * 256 * 4 : 0);
    L.x_kmajor = take(big ? Ab * s.d_model * es : 0);
    L.gate_part = take(route_is_split(s) ? static_cast<size_t>(kGateSplit) * ((s.T + 15) / 16 * 16) * E * 4 : 0);
    L.total = off;
    return L;
}

// ---- internal launchers (all asynchronous on `st`; return hipSuccess or the launch error)
hipError_t launch_route(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                        int32_t* idx, float* gate, float* margin, int32_t* counts,
                        int32_t* offsets, int32_t H, uint8_t* hot_mask, int32_t* hist_ws, float* gate_part_ws,
                        hipStream_t st);
int route_chunk_tokens(const moe_shape& s);
hipError_t launch_select_hot(int E, const int32_t* counts, double alpha, double bw_a, double bw_b, int32_t* H_out,
                             uint8_t* hot_mask, hipStream_t st);
hipError_t launch_route_fused(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                              int32_t* idx, float* gate, float* margin, int32_t* chunk_hist, float* gate_part_ws,
                              hipStream_t st);
// Top-1 layers without an expert mask: the second product writes the layer output itself.  Row p of the
// permuted order belongs to token tokmap[p] and to nobody else, so out[tokmap[p]] = gate[tokmap[p]] * y[p],
// rounded to bf16, is the combine step's result for that token (same operations, same rounding) and the
// fp32 rows of y never go to memory.  out == nullptr: the product writes y as usual.
struct FoldOut {
    uint16_t* out;           // [T, N] bf16
    const int32_t* tokmap;   // [A]
    const float* gate;       // [T] (k = 1)
};

// what the finalize kernel needs to place the assignments itself (small layers: one launch less)
struct PlaceArgs {
    const int32_t* idx;    // nullptr: do not place
    int32_t* perm;
    int32_t* inv_perm;
    int32_t* tokmap;
    int A, k, chunk;
};
bool scan_can_place(const moe_shape& s);
hipError_t launch_route_finalize(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                                 int32_t* idx, float* gate, float* margin, int32_t* hist_ws, float* gate_part_ws,
                                 int32_t* counts, int32_t* offsets, int H, uint8_t* hot_mask, const uint8_t* mask_in,
                                 const TileLists* lists, const PlaceArgs* place, hipStream_t st);
hipError_t launch_scan_finalize(int32_t* chunk_hist, int nchunks, int E, int32_t* counts, int32_t* offsets, int H,
                                uint8_t* hot_mask, const uint8_t* mask_in, const TileLists* lists,
                                const PlaceArgs* place, hipStream_t st);
TileLists ffn_tile_lists(const moe_shape& s, Tile* small_ws, Tile* big_ws, int32_t* ntiles_ws, float* partials_ws);
hipError_t launch_place(const moe_shape& s, const int32_t* idx, const int32_t* offsets, const int32_t* chunk_base,
                        int32_t* perm, int32_t* inv_perm, int32_t* tokmap, int chunk, hipStream_t st);
int ffn_tile_rows(const moe_shape& s);
int tiled_join_tiles(const moe_shape& s);
hipError_t launch_expert_products(const moe_shape& s, const void* act, const int32_t* rowmap, bool act_kmajor,
                                  const void* w1, const void* w2, const float* b1, const float* b2, float* y_perm,
                                  void* h_ws, const TileLists& lists, const FoldOut& fold, hipStream_t st);
bool layer_gathers_kmajor(const moe_shape& s);
hipError_t launch_gather_kmajor(const moe_shape& s, const void* x, const int32_t* tokmap, void* xk, hipStream_t st);
hipError_t launch_tile_product(bool first, const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk,
                               void* outp, const Tile* tiles, const int32_t* ntiles, int32_t* part_counter,
                               float* partials, int N, int K, bool act_kmajor, int activation,
                               const float* bias, const FoldOut& fold, hipStream_t st);
int tile_product_grid();
hipError_t launch_permute(const moe_shape& s, const void* x, const int32_t* idx,
                          const int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                          int32_t* hist_ws, hipStream_t st);
hipError_t launch_expert_ffn(const moe_shape& s, const void* x_perm, const void* w1, const void* w2,
                             const float* b1, const float* b2,
                             const int32_t* offsets, const uint8_t* mask, float* y_perm,
                             void* h_ws, Tile* tiles_ws, Tile* tiles_big_ws, int32_t* ntiles_ws, float* partials_ws,
                             void* x_kmajor_ws, hipStream_t st);
hipError_t launch_combine(const moe_shape& s, const float* y_perm, const int32_t* inv_perm,
                          const int32_t* idx, const float* gate, const uint8_t* mask, void* out,
                          hipStream_t st);
hipError_t launch_pack(const moe_shape& s, int which, const void* src, void* dst, hipStream_t st);
hipError_t launch_mask_out(const uint8_t* mask_or_null, uint8_t* dst, int E, hipStream_t st);

void set_profile_events(const hipEvent_t* five_events_or_null);

// number of compute units of the current device (cached)
int device_cu_count();

// ---- one-time set-up per device ---------------------------------------------------------------
// Raising a kernel's dynamic-LDS limit and asking for its occupancy are calls into the runtime that do not
// belong on a launch path (they cost time, and a first call made while a stream is being captured would
// land inside the capture).  ensure_ready() makes them all, for every kernel of the library, once per
// device and under a lock; every entry point that launches kernels calls it first.
constexpr int kMaxDevices = 64;
constexpr size_t kLdsPerCu = 160 * 1024;
hipError_t ensure_ready();                       // api.hip
int current_device_index();                      // api.hip: hipGetDevice clamped to [0, kMaxDevices)
hipError_t configure_ffn_kernels(int dev);       // ffn.hip
hipError_t configure_tile_kernels(int dev);      // ffn_tile.hip
hipError_t configure_route_kernels(int dev);     // route.hip

}  // namespace moe
