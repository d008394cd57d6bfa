// LDS-tiled MFMA product for experts with many rows (the compute-bound "hot" experts of the
// paper's Section 3.3: enough tokens per expert that the product is bound by matrix throughput,
// not by reading the expert's parameters):
//
//   out[row, n] = sum_k act[row, k] * W_e[n, k]          (FIRST: relu, rounded to bf16)
//
// Block = 8 wavefronts on a 256 (rows) x 256 (columns) output tile, K in steps of 32 through a
// ring of four LDS stages of 32 KiB: the copies of two stages are in flight while two are being
// read (the current one, and the next one into registers ahead of its MFMAs).  Both operands sit in LDS in MFMA-fragment order (16 x 32 fragments of
// 1 KiB, one 16-byte piece per lane), so every LDS read of the inner loop is a conflict-free
// 1 KiB wavefront read.  Global memory is copied straight into LDS (16 bytes per lane, no
// registers in between): the packed weights are already in fragment order in HBM, and for the
// activation rows (optionally gathered through `rowmap`) each lane fetches the piece that
// belongs at its own slot.  Wavefront (wm, wn) of the 2 x 4 grid owns 128 rows x 64 columns:
// 4 weight fragments (MFMA A operand) x 8 row fragments (B operand) of 16x16x32 per 32-k step,
// 128 accumulator registers.  Blocks are persistent over (row tile, column tile) pairs taken
// from the device-built list of large-expert row tiles.
#include <type_traits>

#include "tile_schedule.hpp"

namespace moe {

constexpr int kTM = kBigTileRows;   // 256 rows
constexpr int kTN = kTileCols;      // 256 columns
constexpr int kTK = 32;             // k per LDS stage
constexpr int kStages = 4;          // ring of LDS stages: two being read, two in flight (a fifth, which
                                    // fits, bought nothing: the copies are not limited by ring depth)
constexpr int kAhead = kStages - 1; // the iteration for stage j issues the copies of stage j + kAhead
constexpr int kOperandBytes = kTM * kTK * 2;        // 16 KiB per operand per stage
constexpr int kStageBytes = 2 * kOperandBytes;      // 32 KiB per stage

// Wait until at most `stages` stages' worth of this wavefront's copies (4 each) are still in flight.
__device__ __forceinline__ void wait_copies(int stages) {
    if (stages >= 3) __builtin_amdgcn_s_waitcnt(0x0F7C);         // vmcnt(12)
    else if (stages == 2) __builtin_amdgcn_s_waitcnt(0x0F78);    // vmcnt(8)
    else if (stages == 1) __builtin_amdgcn_s_waitcnt(0x0F74);    // vmcnt(4)
    else __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0)
}

// Register fragments of one wavefront: the 4 weight fragments of a stage, double-buffered over stages,
// and the 8 row fragments as 4 pairs.
struct StageFrags {
    bf16x8 w[2][4];
    bf16x8 x[4][2];
};

__device__ __forceinline__ void lds_read_w(bf16x8 (&w)[4], const unsigned char* base) {
#pragma unroll
    for (int nf = 0; nf < 4; ++nf) w[nf] = *reinterpret_cast<const bf16x8*>(base + nf * 1024);
}

__device__ __forceinline__ void lds_read_x(bf16x8 (&x)[2], const unsigned char* base, int pair) {
    x[0] = *reinterpret_cast<const bf16x8*>(base + (2 * pair) * 1024);
    x[1] = *reinterpret_cast<const bf16x8*>(base + (2 * pair + 1) * 1024);
}

// 4 weight fragments x row-fragment pair P: 8 MFMAs
template <int P>
__device__ __forceinline__ void mfma_pair(const bf16x8 (&w)[4], const bf16x8 (&x)[2], f32x4 (&acc)[4][8]) {
#pragma unroll
    for (int nf = 0; nf < 4; ++nf) {
        acc[nf][2 * P] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nf], x[0], acc[nf][2 * P], 0, 0, 0);
        acc[nf][2 * P + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[nf], x[1], acc[nf][2 * P + 1], 0, 0, 0);
    }
}

template <int FIRST>
__global__ __launch_bounds__(512) void ffn_tile_kernel(const uint16_t* __restrict__ act,
                                                       const int32_t* __restrict__ rowmap,
                                                       const uint16_t* __restrict__ wpk,
                                                       void* __restrict__ outp, const Tile* __restrict__ tiles,
                                                       const int32_t* __restrict__ ntiles_p,
                                                       int32_t* __restrict__ part_counter,
                                                       float* __restrict__ partials, int N, int K,
                                                       int act_kmajor,
                                                       const float* __restrict__ bias, const FoldOut fold) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // between units, when no stage is in use, the first word of the ring passes the next part's number on
    int* next_part = reinterpret_cast<int*>(smem);
    // stage st: 16 row fragments at smem + st * kStageBytes, 16 weight fragments behind them

    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int wm = wave >> 2, wn = wave & 3;
    const int r = lane & 15, g = lane >> 4;
    const int nblk = N >> 4, kblk = K >> 5;
    const int ntn = (N + kTN - 1) / kTN;
    const int ntiles = ntiles_p[0];
    if (ntiles <= 0) return;                            // no large expert in this call (block-uniform)
    // LDS byte address of the first of the two fragments that this wavefront copies in, stage 0
    const uint32_t copy_base = lds_address(smem) + 2 * wave * 1024;

    // Blocks are handed to the 8 XCDs round-robin, and each XCD has its own L2: block b takes position pb
    // of a round, so that the blocks of one XCD hold G / 8 consecutive units, a GM x GN patch whose
    // activation panels that L2 serves GN times and whose weight panels GM times.
    const int G = gridDim.x;
    const TileSchedule sch = tile_schedule(ntiles, N, kblk, G, partials != nullptr);
    const int pb = (G % 8 == 0) ? static_cast<int>(blockIdx.x & 7) * (G >> 3) + static_cast<int>(blockIdx.x >> 3)
                                : static_cast<int>(blockIdx.x);
    const int nleft = sch.R * sch.split;                // parts of the left-over units

    // A unit of work: (row tile mt, column tile nt) over k-steps [kb0, kb0 + nk), whole (nparts == 1) or
    // one of nparts parts of a left-over unit.
    struct Unit {
        int u, part, nparts, nt, kb0, nk;
        Tile tl;
        bool valid;
    };
    auto unit_at = [&](int it) {
        Unit w;
        w.valid = true;
        w.part = 0;
        if (it < sch.rounds) {
            w.u = it * G + pb;
            w.nparts = 1;
        } else {
            // The parts of the left-over units; there are no more of them than blocks.
            int id;
            if (sch.rounds > 0) {
                // After full rounds the blocks arrive at different times (a few per cent of the rounds' time):
                // a counter hands the parts out in order of arrival (which block computes a part has no
                // influence on the result).  The first word of the ring is free now: every wavefront that
                // gets past the first barrier has read its last stage.
                __syncthreads();
                if (t == 0) *next_part = (nleft > 0) ? atomicAdd(part_counter, 1) : 0;
                __syncthreads();
                id = *next_part;
                w.valid = id < nleft;                      // block-uniform; every block ends up here
            } else {
                // No full round: all blocks start together, one part each.  Part-major numbering and an
                // equal run of consecutive numbers per XCD, so that the blocks of an XCD hold the same
                // K-slice of neighbouring units, which share their row and weight panels in that XCD's L2
                // (handed out in order of arrival, the parts of a Switch-large-sized second product hit in
                // L2 0.46 of the time and ran at the rate their CUs could pull from memory).
                const int n8 = (nleft + 7) >> 3;
                const bool xcds = G % 8 == 0;
                id = xcds ? static_cast<int>(blockIdx.x & 7) * n8 + static_cast<int>(blockIdx.x >> 3)
                          : static_cast<int>(blockIdx.x);
                w.valid = it == 0 && id < nleft && (!xcds || static_cast<int>(blockIdx.x >> 3) < n8);
                id = id % max(sch.R, 1) * sch.split + id / max(sch.R, 1);     // (unit, part) from part-major
            }
            w.u = sch.rounds * G + (w.valid ? id / sch.split : 0);
            w.part = w.valid ? id % sch.split : 0;
            w.nparts = sch.split;
        }
        int mt = 0;
        w.nt = 0;
        if (w.valid) unit_of(sch, w.u, mt, w.nt);
        w.kb0 = kblk * w.part / w.nparts;                  // kblk * kMaxSplit fits easily
        w.nk = kblk * (w.part + 1) / w.nparts - w.kb0;
        w.tl = tiles[w.valid ? mt : 0];
        return w;
    };

    // 4 copies per wavefront and stage; stages are copied in order, so the pointers just advance.
    // This wavefront stages fragments 2*wave and 2*wave+1 of each operand.  A lane fetches the 16
    // bytes that belong at its own slot of the fragment: row (lane % 16), k-group (lane / 16).
    const uint16_t* arow[2];
    const uint16_t* brow[2];
    const size_t kstride = act_kmajor ? kStepStride : 32;   // elements per k-step
    auto copy_piece = [&](int st, int q) {             // q = 0 ... 3: row fragment 0, weight 0, row 1, weight 1
        const int i = q >> 1;
        if ((q & 1) == 0) {
            copy16_to_lds(arow[i], copy_base + st * kStageBytes + i * 1024);
            arow[i] += kstride;
        } else {
            copy16_to_lds(brow[i], copy_base + st * kStageBytes + kOperandBytes + i * 1024);
            brow[i] += 512;
        }
    };
    auto stage_in = [&](int st) {
#pragma unroll
        for (int q = 0; q < 4; ++q) copy_piece(st, q);
    };
    // Point the copies at a unit's first k-step.
    auto point_copies_at = [&](const Unit& w) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int row = w.tl.row0 + min((2 * wave + i) * 16 + r, w.tl.rows - 1);
            if (rowmap != nullptr) row = rowmap[row];
            // operand rows are row-major (the caller's x or x_perm) or k-step-major (h, gathered x)
            arow[i] = act_kmajor ? act + h_index(row, w.kb0 * 32 + g * 8, kblk)
                                 : act + static_cast<size_t>(row) * K + static_cast<size_t>(w.kb0) * 32 + g * 8;
            const int nb = min(w.nt * 16 + 2 * wave + i, nblk - 1);
            brow[i] = wpk + ((static_cast<size_t>(w.tl.expert) * nblk + nb) * kblk + w.kb0) * 512 + lane * 8;
        }
    };
    // The ring runs on across units: `slot` is the slot of the current unit's current stage, and the first
    // stage of the next unit follows the last stage of this one.
    int slot = 0;
    // Start a unit from a standstill: its first stages into the slots from `slot` on.  Every wavefront must be
    // done reading the ring (its MFMAs have consumed the last stage): a bare barrier, so that output stores
    // still in flight need not complete first.
    auto start_unit = [&](const Unit& w) {
        point_copies_at(w);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int sidx = 0; sidx < kAhead; ++sidx)
            if (sidx < w.nk) stage_in((slot + sidx) % kStages);
    };

    const int wave_w = kOperandBytes + (wn * 4 * 64 + lane) * 16, wave_x = (wm * 8 * 64 + lane) * 16;
    Unit cur = unit_at(0);
    if (cur.valid) start_unit(cur);
    for (int it = 0; cur.valid; ++it) {
        const int nk = cur.nk;
        // Inside the full rounds the next unit is known in advance: its tile descriptor is fetched now, not
        // between the units, where the load's latency would be exposed (1.5 us per unit).
        const bool next_known = it + 1 < sch.rounds;
        Unit nxt;
        if (next_known) nxt = unit_at(it + 1);
        // The next unit's first stages go out during this unit's last iterations, in the slots that fall free
        // there, when the unit is known by then, needs no row lookups (a vector load here would make the
        // compiler wait for every copy in flight) and both units are at least as long as the ring is deep.
        const bool ahead = next_known && nxt.valid && rowmap == nullptr && nk >= kAhead && nxt.nk >= kAhead;
        f32x4 acc[4][8];
#pragma unroll
        for (int nf = 0; nf < 4; ++nf)
#pragma unroll
            for (int tf = 0; tf < 8; ++tf) acc[nf][tf] = f32x4{0.f, 0.f, 0.f, 0.f};
        StageFrags fr;
        // One stage of 32 k, software-pipelined across stages so that the MFMA pipe never waits for LDS.
        // The iteration for stage j starts by making sure that stage j + 1 has landed for every wavefront
        // (own copies by vmcnt, the others' by the barrier; __syncthreads() would drain every outstanding
        // copy and empty the ring) and by refilling the slot of stage j - 1, which nobody reads any more,
        // with stage j + kAhead.  The fragments of stage j are in registers by then, except row pair 3: every
        // group of 8 MFMAs is followed by the LDS reads that refill the registers it has just freed with
        // stage j + 1, so each read has at least 8 MFMAs to complete.  (At its first use of an LDS result
        // after a global-to-LDS copy was issued the compiler waits for all outstanding LDS reads, not
        // only the needed ones: here that is at the first MFMA, when only old reads are outstanding.)
        // `steady`: stage j + kAhead exists, so nothing in the iteration is conditional.
        auto iterate = [&](auto cbuf, auto steady, int j) {
            constexpr int C = decltype(cbuf)::value;
            constexpr bool STEADY = decltype(steady)::value;
            const int slot_next = slot + 1 == kStages ? 0 : slot + 1;
            const int slot_free = slot == 0 ? kStages - 1 : slot - 1;          // held stage j - 1
            const unsigned char* st_cur = smem + slot * kStageBytes;
            const unsigned char* st_nxt = smem + slot_next * kStageBytes;
            const bool more = STEADY || j + 1 < nk;        // block-uniform
            if (more) {
                // stages j + 2 ... j + kAhead - 1 (as far as they exist) may stay in flight; with the next unit's
                // stages behind them that is always kAhead - 2 stages' worth
                wait_copies((STEADY || ahead) ? kAhead - 2 : min(j + kAhead - 1, nk - 1) - (j + 1));
                asm volatile("s_barrier" ::: "memory");
            } else if (ahead) {
                asm volatile("s_barrier" ::: "memory");   // the slot of stage j - 1 is about to be refilled
            }
            // from here on the stages that go out are the next unit's
            if (!STEADY && ahead && j + kAhead == nk) point_copies_at(nxt);
            // the four copies of stage j + kAhead are issued between the first MFMAs, whose execution
            // covers the scalar and address arithmetic of the copies
            const bool refill = (more && (STEADY || j + kAhead < nk)) || (!STEADY && ahead && j + kAhead >= nk);
#pragma unroll
            for (int nf = 0; nf < 4; ++nf) {
                __builtin_amdgcn_sched_barrier(0);
                acc[nf][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr.w[C][nf], fr.x[0][0], acc[nf][0], 0, 0, 0);
                acc[nf][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr.w[C][nf], fr.x[0][1], acc[nf][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (refill) copy_piece(slot_free, nf);
            }
            __builtin_amdgcn_sched_barrier(0);
            lds_read_x(fr.x[3], st_cur + wave_x, 3);
            if (more) {
                lds_read_w(fr.w[C ^ 1], st_nxt + wave_w);
                lds_read_x(fr.x[0], st_nxt + wave_x, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_pair<1>(fr.w[C], fr.x[1], acc);
            __builtin_amdgcn_sched_barrier(0);
            if (more) lds_read_x(fr.x[1], st_nxt + wave_x, 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_pair<2>(fr.w[C], fr.x[2], acc);
            __builtin_amdgcn_sched_barrier(0);
            if (more) lds_read_x(fr.x[2], st_nxt + wave_x, 2);
            __builtin_amdgcn_sched_barrier(0);
            mfma_pair<3>(fr.w[C], fr.x[3], acc);
            __builtin_amdgcn_sched_barrier(0);
            slot = slot_next;
        };

        // The first waits may also wait for the previous unit's output stores, which were issued after this
        // unit's first copies and count in vmcnt like them: never too short, since no more than the given
        // number of operations stays outstanding and the copies complete in order.
        wait_copies(min(kAhead, nk) - 1);                  // stage 0 has landed ...
        asm volatile("s_barrier" ::: "memory");           // ... for every wavefront
        lds_read_w(fr.w[0], smem + slot * kStageBytes + wave_w);
        lds_read_x(fr.x[0], smem + slot * kStageBytes + wave_x, 0);
        lds_read_x(fr.x[1], smem + slot * kStageBytes + wave_x, 1);
        lds_read_x(fr.x[2], smem + slot * kStageBytes + wave_x, 2);
        int j = 0;
        for (; j + 1 + kAhead < nk; j += 2) {
            iterate(std::integral_constant<int, 0>{}, std::true_type{}, j);
            iterate(std::integral_constant<int, 1>{}, std::true_type{}, j + 1);
        }
        // at most kAhead + 1 stages are left, and j is even: the buffers keep alternating
        if (j < nk) iterate(std::integral_constant<int, 0>{}, std::false_type{}, j);
        if (j + 1 < nk) iterate(std::integral_constant<int, 1>{}, std::false_type{}, j + 1);
        if (j + 2 < nk) iterate(std::integral_constant<int, 0>{}, std::false_type{}, j + 2);
        if (j + 3 < nk) iterate(std::integral_constant<int, 1>{}, std::false_type{}, j + 3);
        if (j + 4 < nk) iterate(std::integral_constant<int, 0>{}, std::false_type{}, j + 4);

        // The next unit's first copies go out before this unit's output is stored: the copies' latency and
        // the stores overlap, and the load of the next tile's descriptor does not wait behind the stores.
        if (!next_known) nxt = unit_at(it + 1);
        if (nxt.valid && !ahead) start_unit(nxt);

        // Lane holds 4 consecutive columns of one row per accumulator.
        if (cur.nparts > 1) {
            // part of a unit: the partial tile goes to the workspace; the next kernel adds the parts up
            float* mine = partials + (static_cast<size_t>(cur.u - sch.rounds * G) * cur.nparts + cur.part) * (kTM * kTN);
#pragma unroll
            for (int tf = 0; tf < 8; ++tf)
#pragma unroll
                for (int nf = 0; nf < 4; ++nf)
                    *reinterpret_cast<f32x4*>(mine + (wm * 128 + tf * 16 + r) * kTN + (wn * 4 + nf) * 16 + g * 4) =
                        acc[nf][tf];
        } else {
            const float* be = bias ? bias + static_cast<size_t>(cur.tl.expert) * N : nullptr;
#pragma unroll
            for (int tf = 0; tf < 8; ++tf) {
                const int lr = wm * 128 + tf * 16 + r;
                const bool ok = lr < cur.tl.rows;
                if constexpr (FIRST != 0) {
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        const int nb = cur.nt * 16 + wn * 4 + 2 * m;   // N / 16 is even: a pair exists as a whole
                        if (nb >= nblk) continue;                       // wave-uniform
                        store_h_pair<FIRST, false>(outp, cur.tl.row0 + lr, ok, nb * 16, N, be, acc[2 * m][tf],
                                                   acc[2 * m + 1][tf]);
                    }
                } else {
                    int ftok = 0;
                    float fw = 0.f;
                    if (fold.out != nullptr && ok) {                    // folded layer output (top-1, no mask)
                        ftok = fold.tokmap[cur.tl.row0 + lr];
                        fw = fold.gate[ftok];
                    }
                    if (fold.out != nullptr) {                          // block-uniform
#pragma unroll
                        for (int m = 0; m < 2; ++m) {
                            const int nb = cur.nt * 16 + wn * 4 + 2 * m;
                            if (nb >= nblk) continue;                   // wave-uniform
                            store_folded_pair(fold.out, ftok, fw, ok, nb * 16, N, be, acc[2 * m][tf], acc[2 * m + 1][tf]);
                        }
                    } else {
#pragma unroll
                        for (int nf = 0; nf < 4; ++nf) {
                            const int nb = cur.nt * 16 + wn * 4 + nf;
                            if (ok && nb < nblk)
                                store_out<0>(outp, cur.tl.row0 + lr, nb * 16 + g * 4, N, be, acc[nf][tf]);
                        }
                    }
                }
            }
        }
        cur = nxt;
    }
}

template <int FIRST>
static hipError_t launch_tile(const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk, void* outp,
                              const Tile* tiles, const int32_t* ntiles, int32_t* part_counter, float* partials, int N,
                              int K, bool act_kmajor, const float* bias, const FoldOut& fold, hipStream_t st) {
    auto kern = ffn_tile_kernel<FIRST>;
    constexpr int lds = kStages * kStageBytes;  // 128 KiB: above the default per-block limit (raised by configure_tile_kernels)
    // Always the whole chip, one block per CU (the LDS ring allows no more): how many units there are is
    // only known on the device, and few units are cut along K over blocks that would otherwise idle.
    const int grid = tile_product_grid();
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(512), lds, st, act, rowmap, wpk, outp, tiles,
                       ntiles, part_counter, partials, N, K, act_kmajor ? 1 : 0, bias, fold);
    return hipGetLastError();
}

int tile_product_grid() { return device_cu_count(); }

template <int FIRST>
static hipError_t configure_tile() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_tile_kernel<FIRST>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kStages * kStageBytes);
}

hipError_t configure_tile_kernels(int) {
    hipError_t e;
    if ((e = configure_tile<0>()) != hipSuccess) return e;
    if ((e = configure_tile<kFirstRelu>()) != hipSuccess) return e;
    return configure_tile<kFirstGelu>();
}

hipError_t launch_tile_product(bool first, const uint16_t* act, const int32_t* rowmap, const uint16_t* wpk,
                               void* outp, const Tile* tiles, const int32_t* ntiles, int32_t* part_counter,
                               float* partials, int N, int K, bool act_kmajor, int activation,
                               const float* bias, const FoldOut& fold, hipStream_t st) {
    if (!first)
        return launch_tile<0>(act, rowmap, wpk, outp, tiles, ntiles, part_counter, partials, N, K,
                              act_kmajor, bias, fold, st);
    if (activation == MOE_ACT_GELU)
        return launch_tile<kFirstGelu>(act, rowmap, wpk, outp, tiles, ntiles, part_counter, partials, N, K,
                                       act_kmajor, bias, fold, st);
    return launch_tile<kFirstRelu>(act, rowmap, wpk, outp, tiles, ntiles, part_counter, partials, N, K,
                                   act_kmajor, bias, fold, st);
}

}  // namespace moe
