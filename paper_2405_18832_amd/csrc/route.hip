// Gating and routing: logits = x . w_gate^T (+ bias), softmax over experts, top-k with
// lowest-index tie-break, gate weights, per-expert token histogram, prefix sums and the
// top-H hot mask (paper Section 2.1 for the gating network, Section 3.3 for the token
// counts and the hot set).
//
// Two kernels.  route_fused_kernel: one block per chunk of 16*TF tokens computes the chunk's
// logits into LDS, picks each token's experts there and leaves the chunk's per-expert
// histogram in the workspace.  scan_finalize_kernel: one block turns the chunk histograms
// into counts, prefix sums (per expert over chunks, and over experts), the hot mask and the
// expert tile list.  Nothing is ordered through atomics on global memory, so every output
// is the same on every run.
#include "common.hpp"

namespace moe {

constexpr int kMaxRounds = MOE_MAX_K + 1;

// Value of the lane n places away inside the lane's row of 16 (a DPP row rotation, no LDS traffic).  Four
// steps with n = 8, 4, 2, 1 leave every lane of the row with the reduction over the row; for sums the
// operand pairs are those of the xor butterfly (after a step with n the values have period n in the row).
template <int N>
__device__ __forceinline__ float row_rot(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xF, 0xF, false));
}
template <int N>
__device__ __forceinline__ int row_rot(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x120 + N, 0xF, 0xF, false);
}

// ---------------------------------------------------------------------------
// top-k of one token from its logits row in LDS, by a group of 16 lanes (4 tokens per wave).
// k rounds (k + 1 when the margin is wanted) of a (value, index) arg-max; on equal values the
// lower index wins, in the lane-local scan and in every exchange, so the order is "descending
// logit, ties by lowest expert index".  A winner is retired by setting its logit to -inf.
// ---------------------------------------------------------------------------
// V > 0: the row has at most 16 * V experts and the lane keeps its V logits (experts sub, sub + 16, ...) in
// registers for all rounds; V == 0: any E, the row is read from LDS in every round and a winner is retired by
// overwriting its logit there.  (Every LDS read in the per-round loops is a round trip the next compare waits
// for: with the row in registers the top-k of a 64-token chunk of 128 experts takes a third of the time.)
template <int V>
__device__ __forceinline__ void topk_row(float* __restrict__ row, int E, int k, int renorm, int sub, bool live,
                                         int32_t* __restrict__ idx_out, float* __restrict__ w_out,
                                         float* __restrict__ margin_out, int32_t* __restrict__ hist) {
    const float NEG = -__builtin_huge_valf();
    float sel_v[kMaxRounds];
    int sel_i[kMaxRounds];
    const int rounds = min(k + (margin_out != nullptr ? 1 : 0), E);   // the margin needs one more winner
    float vmax = 0.f, denom = 1.f;
    float v[V > 0 ? V : 1];
    if constexpr (V > 0) {
#pragma unroll
        for (int q = 0; q < V; ++q) v[q] = (sub + 16 * q < E) ? row[sub + 16 * q] : NEG;
    }
#pragma unroll 1
    for (int j = 0; j < rounds; ++j) {
        float bv = NEG;
        int bi = 0x7fffffff;
        if constexpr (V > 0) {
#pragma unroll
            for (int q = 0; q < V; ++q) {
                const int e = sub + 16 * q;
                if (e < E && (v[q] > bv || bi == 0x7fffffff)) { bv = v[q]; bi = e; }
            }
        } else {
            for (int e = sub; e < E; e += 16) {
                const float x = row[e];
                if (x > bv || bi == 0x7fffffff) { bv = x; bi = e; }
            }
        }
        auto better = [&](float ov, int oi) {
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        };
        better(row_rot<8>(bv), row_rot<8>(bi));
        better(row_rot<4>(bv), row_rot<4>(bi));
        better(row_rot<2>(bv), row_rot<2>(bi));
        better(row_rot<1>(bv), row_rot<1>(bi));
        bi = min(bi, E - 1);          // NaN logits must not produce an out-of-range expert
        if (j == 0) {
            vmax = bv;
            float part = 0.f;
            if constexpr (V > 0) {
#pragma unroll
                for (int q = 0; q < V; ++q)
                    if (sub + 16 * q < E) part += expf(v[q] - vmax);
            } else {
                for (int e = sub; e < E; e += 16) part += expf(row[e] - vmax);
            }
            part += row_rot<8>(part);
            part += row_rot<4>(part);
            part += row_rot<2>(part);
            part += row_rot<1>(part);
            denom = part;
        }
#pragma unroll
        for (int q = 0; q < kMaxRounds; ++q)
            if (q == j) { sel_v[q] = bv; sel_i[q] = bi; }
        if constexpr (V > 0) {
#pragma unroll
            for (int q = 0; q < V; ++q)
                if (sub + 16 * q == bi) v[q] = NEG;
        } else {
            if (sub == 0) row[bi] = NEG;
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (live && sub == 0) {
        float p[MOE_MAX_K];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j)
            if (j < k) {
                p[j] = expf(sel_v[j] - vmax) / denom;
                psum += p[j];
            }
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j)
            if (j < k) {
                idx_out[j] = sel_i[j];
                w_out[j] = renorm ? p[j] / psum : p[j];
                atomicAdd(&hist[sel_i[j]], 1);      // LDS, integer: order does not matter
            }
        if (margin_out) {
            float m = __builtin_huge_valf();
#pragma unroll
            for (int j = 0; j + 1 < kMaxRounds; ++j)
                if (j + 1 < rounds) m = fminf(m, sel_v[j] - sel_v[j + 1]);
            *margin_out = m;
        }
    }
}

// called by whole wavefronts; E is uniform
__device__ __forceinline__ void topk_from_lds(float* __restrict__ row, int E, int k, int renorm, int sub,
                                              bool live, int32_t* __restrict__ idx_out,
                                              float* __restrict__ w_out, float* __restrict__ margin_out,
                                              int32_t* __restrict__ hist) {
    if (E <= 64) topk_row<4>(row, E, k, renorm, sub, live, idx_out, w_out, margin_out, hist);
    else if (E <= 128) topk_row<8>(row, E, k, renorm, sub, live, idx_out, w_out, margin_out, hist);
    else if (E <= 256) topk_row<16>(row, E, k, renorm, sub, live, idx_out, w_out, margin_out, hist);
    else topk_row<0>(row, E, k, renorm, sub, live, idx_out, w_out, margin_out, hist);
}

// Floats per token row of the logits in LDS: whole groups of 16 * NF experts (the accumulate step writes
// full fragments) plus 4, which keeps the rows 16-byte aligned and moves consecutive rows to different banks.
__host__ __device__ inline int route_row_stride(int E, int NF) { return (E + 16 * NF - 1) / (16 * NF) * (16 * NF) + 4; }

// ---------------------------------------------------------------------------
// route_fused_kernel<ST, TF, NW, NF>: block = NW wavefronts, chunk = 16*TF tokens.
//  bf16: MFMA 16x16x32 with gate rows as the A operand and token rows as the B operand (a lane
//  ends up with 4 consecutive experts of one token).  Experts are taken NF fragments (16*NF
//  experts) at a time; the NW wavefronts split the contraction (each reads its own slice of
//  every row, so x and the gate matrix cross L1 once per block) and add their partial logits
//  into LDS one after the other, in wave order (deterministic).  Every k-step issues exactly
//  NF + TF loads (rows past the end are clamped, their results dropped), two steps ahead.
//  fp32: plain FMA dot products, one (token, expert) pair per thread and pass.
// The chunk's histogram goes to chunk_hist[chunk * E + e].
// Dynamic LDS: logits [16*TF][route_row_stride(E, NF)] floats, then the histogram [E] ints.
// ---------------------------------------------------------------------------
template <typename ST, int TF, int NW, int NF>
__global__ __launch_bounds__(NW * 64) void route_fused_kernel(const ST* __restrict__ x, const ST* __restrict__ wg,
                                                              const float* __restrict__ bias,
                                                              int32_t* __restrict__ topk_idx,
                                                              float* __restrict__ topk_w,
                                                              float* __restrict__ margin,
                                                              int32_t* __restrict__ chunk_hist, int T, int d,
                                                              int E, int k, int renorm) {
    constexpr int TOK = 16 * TF;
    constexpr int NT = NW * 64;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int Ep = route_row_stride(E, NF);
    float* L = lds;
    int32_t* hist = reinterpret_cast<int32_t*>(lds + TOK * Ep);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t0 = blockIdx.x * TOK;
    for (int e = threadIdx.x; e < E; e += NT) hist[e] = 0;

    if constexpr (sizeof(ST) == 2) {
        const int r = lane & 15, g = lane >> 4;
        const int ksteps = d >> 5;
        const int per = (ksteps + NW - 1) / NW;
        const int kb0 = min(ksteps, wave * per), kb1 = min(ksteps, kb0 + per);
        const uint16_t* xrow[TF];
#pragma unroll
        for (int tf = 0; tf < TF; ++tf)
            xrow[tf] = reinterpret_cast<const uint16_t*>(x) + static_cast<size_t>(min(t0 + tf * 16 + r, T - 1)) * d + g * 8;
        for (int ec = 0; ec < E; ec += 16 * NF) {
            const uint16_t* wrow[NF];
#pragma unroll
            for (int nf = 0; nf < NF; ++nf)
                wrow[nf] = reinterpret_cast<const uint16_t*>(wg) + static_cast<size_t>(min(ec + nf * 16 + r, E - 1)) * d + g * 8;
            f32x4 acc[NF][TF];
#pragma unroll
            for (int nf = 0; nf < NF; ++nf)
#pragma unroll
                for (int tf = 0; tf < TF; ++tf) acc[nf][tf] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (kb0 < kb1) {
                constexpr int PF = 2;
                bf16x8 a[PF][NF], b[PF][TF];
                auto issue = [&](int slot, int kb) {
#pragma unroll
                    for (int tf = 0; tf < TF; ++tf) b[slot][tf] = *reinterpret_cast<const bf16x8*>(xrow[tf] + kb * 32);
#pragma unroll
                    for (int nf = 0; nf < NF; ++nf) a[slot][nf] = *reinterpret_cast<const bf16x8*>(wrow[nf] + kb * 32);
                };
                auto fma = [&](int slot) {
#pragma unroll
                    for (int nf = 0; nf < NF; ++nf)
#pragma unroll
                        for (int tf = 0; tf < TF; ++tf)
                            acc[nf][tf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[slot][nf], b[slot][tf], acc[nf][tf], 0, 0, 0);
                };
#pragma unroll
                for (int p = 0; p < PF; ++p) issue(p, min(kb0 + p, kb1 - 1));
                int kb = kb0;
                for (; kb + 2 * PF <= kb1; kb += PF) {
#pragma unroll
                    for (int p = 0; p < PF; ++p) {
                        fma(p);
                        issue(p, kb + p + PF);
                    }
                }
                if (kb + PF < kb1) {
#pragma unroll
                    for (int p = 0; p < PF; ++p) {
                        fma(p);
                        issue(p, min(kb + p + PF, kb1 - 1));
                    }
                    kb += PF;
                }
#pragma unroll
                for (int p = 0; p < PF; ++p)
                    if (kb + p < kb1) fma(p);
            }
            // Partial sums are added in wave order (deterministic).  The wavefront whose turn it is reads all
            // the sums so far as 16-byte pieces (a lane's 4 experts of a token are adjacent), then writes them
            // back: one LDS latency per turn.  Rows are padded to whole fragments, so nothing here depends on E.
            f32x4 first[NF];                               // what the first wavefront starts from: the bias
#pragma unroll
            for (int nf = 0; nf < NF; ++nf) {
                first[nf] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (bias != nullptr && wave == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) first[nf][i] = bias[min(ec + nf * 16 + g * 4 + i, E - 1)];
                }
            }
            for (int w = 0; w < NW; ++w) {
                if (wave == w) {
                    f32x4 sofar[NF][TF];
#pragma unroll
                    for (int nf = 0; nf < NF; ++nf)
#pragma unroll
                        for (int tf = 0; tf < TF; ++tf) {
                            const f32x4* p = reinterpret_cast<const f32x4*>(L + (tf * 16 + r) * Ep + ec + nf * 16 + g * 4);
                            sofar[nf][tf] = (w == 0) ? first[nf] : *p;
                        }
#pragma unroll
                    for (int nf = 0; nf < NF; ++nf)
#pragma unroll
                        for (int tf = 0; tf < TF; ++tf) {
                            f32x4* p = reinterpret_cast<f32x4*>(L + (tf * 16 + r) * Ep + ec + nf * 16 + g * 4);
                            *p = acc[nf][tf] + sofar[nf][tf];
                        }
                }
                __syncthreads();
            }
        }
    } else {
        for (int i = threadIdx.x; i < TOK * E; i += NT) {
            const int tl = i / E, e = i % E;
            const float* xr = reinterpret_cast<const float*>(x) + static_cast<size_t>(min(t0 + tl, T - 1)) * d;
            const float* wr = reinterpret_cast<const float*>(wg) + static_cast<size_t>(e) * d;
            float s = 0.f;
            for (int c = 0; c < d; ++c) s = fmaf(xr[c], wr[c], s);
            L[tl * Ep + e] = s + (bias ? bias[e] : 0.f);
        }
        __syncthreads();
    }

    // top-k: 4 tokens per wavefront and pass
    const int grp = lane >> 4, sub = lane & 15;
#pragma unroll 1
    for (int tl = wave * 4 + grp; tl < TOK; tl += NW * 4) {
        const int t = t0 + tl;
        const bool live = t < T;
        const size_t o = static_cast<size_t>(live ? t : 0) * k;
        topk_from_lds(L + tl * Ep, E, k, renorm, sub, live, topk_idx + o, topk_w + o,
                      margin ? margin + (live ? t : 0) : nullptr, hist);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += NT) chunk_hist[static_cast<size_t>(blockIdx.x) * E + e] = hist[e];
}

// ---------------------------------------------------------------------------
// scan_finalize_kernel: one block of 1024 threads (16 wavefronts).
//  phase 1: for every expert, exclusive prefix sum of its chunk histogram over the chunks, in
//           place (the slot bases of the counting sort); the total is the expert's token count.
//  phase 2: prefix sums over experts -> offsets; top-H hot mask (rank by count, ties by lowest
//           index); the tile list of the expert FFN (every active, masked-in expert's segment
//           cut into row tiles: one list for small experts, one for large ones).
// Any output pointer may be NULL.
// ---------------------------------------------------------------------------
constexpr int kScanPlaceMaxE = 256;     // largest E and ...
constexpr long kScanPlaceMaxA = 512;    // ... most assignments for which the finalize block also places

// the work of scan_finalize_kernel, by a block of 1024 threads
__device__ __forceinline__ void scan_finalize_body(int32_t* __restrict__ chunk_hist, int nchunks, int E,
                                                   int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                   int H, uint8_t* __restrict__ hot_mask,
                                                   const uint8_t* __restrict__ mask_in, const TileLists lists,
                                                   const int want_tiles, const PlaceArgs place) {
    __shared__ int32_t cnt[MOE_MAX_E];
    __shared__ int32_t scan[MOE_MAX_E];
    __shared__ int32_t place_next[16][kScanPlaceMaxE];   // per wavefront: next free slot of every expert
    __shared__ int32_t group_total[1024];                // phase 1: [group][expert] sums over a group's chunks
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // phase 1: chunk_hist is [nchunks][E], so threads that take consecutive experts of one chunk read and
    // write contiguously.  The block is cut into ngrp = 1024 / Ew groups of Ew threads (Ew = E rounded up to
    // whole wavefronts); group q owns the chunks [q * seg, (q + 1) * seg), adds them up per expert 8 loads at
    // a time, the group totals meet in LDS, and the segment is rewritten with its exclusive prefix sums (kept
    // in registers between the two sweeps when it has at most 8 chunks, else read again from L2).  (One
    // shuffle scan of 6 steps per 64 chunks and expert, as before, cost 5.5 us on 64 experts x 128 chunks:
    // the shuffles are LDS round trips that wait for one another.)
    {
        const int Ew = min(1024, (E + 63) & ~63), ngrp = 1024 / Ew;
        const int q = threadIdx.x / Ew, ex = threadIdx.x - q * Ew;
        const bool have = q < ngrp && ex < E;              // threads past ngrp * Ew (none when Ew divides 1024)
        const int seg = (nchunks + ngrp - 1) / ngrp;
        const int c_begin = min(q * seg, nchunks), c_end = min(c_begin + seg, nchunks);
        int32_t* col = chunk_hist + (have ? ex : 0);
        int first[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        int total = 0;
        for (int c0 = c_begin; c0 < c_end; c0 += 8) {
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (have && c0 + i < c_end) ? col[static_cast<size_t>(c0 + i) * E] : 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (c0 == c_begin) first[i] = v[i];
                total += v[i];
            }
        }
        if (have) group_total[q * Ew + ex] = total;
        __syncthreads();
        int carry = 0;                                     // chunks of the groups before this one
        if (have) {
            for (int o = 0; o < q; ++o) carry += group_total[o * Ew + ex];
            if (q == ngrp - 1) cnt[ex] = carry + total;
        }
        if (seg <= 8) {                                    // block-uniform
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (have && c_begin + i < c_end) col[static_cast<size_t>(c_begin + i) * E] = carry;
                carry += first[i];
            }
        } else {
            for (int c0 = c_begin; c0 < c_end; c0 += 8) {
                int v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = (have && c0 + i < c_end) ? col[static_cast<size_t>(c0 + i) * E] : 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (have && c0 + i < c_end) col[static_cast<size_t>(c0 + i) * E] = carry;
                    carry += v[i];
                }
            }
        }
    }
    __syncthreads();
    const int e = threadIdx.x;
    const int mine = (e < E) ? cnt[e] : 0;
    const int incl = block_scan_1024(mine, scan);
    const int row0 = incl - mine;
    if (e < E) {
        if (counts) counts[e] = mine;
        if (offsets) offsets[e] = row0;
    }
    if (e == E - 1 && offsets) offsets[E] = incl;
    bool on = e < E;
    if (H >= 0 && e < E) {
        int rank = 0;
        for (int o = 0; o < E; ++o) rank += (cnt[o] > mine || (cnt[o] == mine && o < e)) ? 1 : 0;
        on = rank < H;
        if (hot_mask) hot_mask[e] = on ? 1 : 0;
    } else if (mask_in != nullptr && e < E) {
        on = mask_in[e] != 0;
    }
    if (want_tiles) emit_tiles(e, row0, on ? mine : 0, lists, scan);     // uniform: a kernel argument
    if (place.idx == nullptr) return;                                    // uniform
    // Small layers: this block also places the assignments (the last step of the counting sort), wavefront
    // w taking chunks w, w + 16, ...: one launch less on a path that is a chain of short kernels.  The slot
    // bases written to chunk_hist in phase 1 are read back by the same block after a barrier.
    __syncthreads();
    if (e < E) cnt[e] = row0;                                            // cnt now holds the offsets
    __threadfence_block();
    __syncthreads();
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    int32_t* next = place_next[wave];
    for (int c = wave; c < nchunks; c += 16) {
        for (int x = lane; x < E; x += 64) next[x] = cnt[x] + chunk_hist[static_cast<size_t>(c) * E + x];
        __builtin_amdgcn_wave_barrier();
        place_chunk(place.idx, next, place.perm, place.inv_perm, place.tokmap, place.A, E, place.k, ebits,
                    place.chunk, c);
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ __launch_bounds__(1024) void scan_finalize_kernel(int32_t* __restrict__ chunk_hist, int nchunks,
                                                             int E, int32_t* __restrict__ counts,
                                                             int32_t* __restrict__ offsets, int H,
                                                             uint8_t* __restrict__ hot_mask,
                                                             const uint8_t* __restrict__ mask_in,
                                                             const TileLists lists, const int want_tiles,
                                                             const PlaceArgs place) {
    scan_finalize_body(chunk_hist, nchunks, E, counts, offsets, H, hot_mask, mask_in, lists, want_tiles, place);
}

// Hot-set size from the counts (Section 3.3, Eq. 6) and the top-H mask.  One block, thread e owns
// expert e.  The real-valued H is formed in double precision with individually rounded operations
// (no fused multiply-add), so that it is the same number a plain double evaluation gives.
__global__ __launch_bounds__(1024) void select_hot_kernel(const int32_t* __restrict__ counts, int E, double alpha,
                                                          double bw_a, double bw_b, int32_t* __restrict__ H_out,
                                                          uint8_t* __restrict__ hot_mask) {
    __shared__ int32_t cnt[MOE_MAX_E];
    __shared__ int32_t active;
    const int e = threadIdx.x;
    if (e == 0) active = 0;
    const int mine = e < E ? counts[e] : 0;
    cnt[e] = mine;
    __syncthreads();
    if (e < E && mine > 0) atomicAdd(&active, 1);
    __syncthreads();
    const double share = __ddiv_rn(__dmul_rn(alpha, bw_a), __dadd_rn(bw_a, bw_b));
    const double h = floor(__dadd_rn(__dmul_rn(share, static_cast<double>(active)), 0.5));
    const int H = h >= static_cast<double>(E) ? E : (h <= 0.0 ? 0 : static_cast<int>(h));
    if (e == 0 && H_out != nullptr) *H_out = H;
    if (e < E && hot_mask != nullptr) {
        int rank = 0;
        for (int o = 0; o < E; ++o) rank += (cnt[o] > mine || (cnt[o] == mine && o < e)) ? 1 : 0;
        hot_mask[e] = rank < H ? 1 : 0;
    }
}

hipError_t launch_select_hot(int E, const int32_t* counts, double alpha, double bw_a, double bw_b, int32_t* H_out,
                             uint8_t* hot_mask, hipStream_t st) {
    hipLaunchKernelGGL(select_hot_kernel, dim3(1), dim3(1024), 0, st, counts, E, alpha, bw_a, bw_b, H_out, hot_mask);
    return hipGetLastError();
}

__global__ void mask_out_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int E) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) dst[e] = src ? (src[e] ? 1 : 0) : 1;
}

hipError_t launch_mask_out(const uint8_t* mask_or_null, uint8_t* dst, int E, hipStream_t st) {
    hipLaunchKernelGGL(mask_out_kernel, dim3((E + 255) / 256), dim3(256), 0, st, mask_or_null, dst, E);
    return hipGetLastError();
}

// chunk size (tokens per routing block) and wavefronts per block, from the shape alone
#ifndef ROUTE_MID_NW
#define ROUTE_MID_NW 4     // wavefronts per block of the 16-token variant (measured: 4 < 2 < 8 < 1 < 16 in time)
#endif
#ifndef ROUTE_T4K_NW
#define ROUTE_T4K_NW 4      // wavefronts per block of the 32-token variant
#endif
#ifndef ROUTE_BIG_NW
#define ROUTE_BIG_NW 4     // wavefronts per block (contraction slices) of the 64-token variant
#endif
struct RouteCfg { int tok, nw, nf; };
static RouteCfg route_cfg(const moe_shape& s) {
    RouteCfg c{16, 4, 1};
    if (s.dtype != MOE_BF16) return c;
    c.nf = s.E >= 113 ? 8 : (s.E >= 49 ? 4 : (s.E >= 17 ? 2 : 1));
    if (route_is_split(s)) { c.tok = 16; c.nw = 8; return c; }   // the split path works in chunks of 16 tokens
    if (s.T <= 64) { c.tok = 16; c.nw = 16; c.nf = c.nf > 4 ? 4 : c.nf; }   // few blocks: split the contraction 16 ways
                                                                            // (128 registers per lane: 4 fragments at a time)
    // More tokens per block reuse every gate-weight fragment for more token fragments, but only as long as
    // there is still a block for every CU (measured, 128 experts: 4096 tokens take 13.9 us in 256 blocks of 16
    // and 17.4 us in 128 blocks of 32; 16384 tokens 39 us in 256 blocks of 64 and 47 us in 512 blocks of 32).
    else if (s.T >= 64 * device_cu_count() && s.E <= 256) { c.tok = 64; c.nw = ROUTE_BIG_NW; }
    else if (s.T >= 32 * device_cu_count() && s.E <= 256) { c.tok = 32; c.nw = ROUTE_T4K_NW; }
    else { c.tok = 16; c.nw = ROUTE_MID_NW; }
    return c;
}

int route_chunk_tokens(const moe_shape& s) { return route_cfg(s).tok; }

// Most dynamic LDS a routing kernel asks for: 16 tokens x (1024 experts padded to whole groups of fragments)
// logits plus the histogram is 78 KiB; 64 tokens x 256 experts is 67 KiB.  configure_route_kernels raises every
// routing kernel's limit to this once.
constexpr size_t kRouteLdsMax = 96 * 1024;

template <typename ST, int TF, int NW, int NF>
static hipError_t configure_route() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(route_fused_kernel<ST, TF, NW, NF>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kRouteLdsMax));
}

template <typename ST, int TF, int NW, int NF>
static hipError_t launch_route_inst(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                                    int32_t* idx, float* gate, float* margin, int32_t* chunk_hist, hipStream_t st) {
    constexpr int tok = 16 * TF;
    const unsigned grid = static_cast<unsigned>((s.T + tok - 1) / tok);
    const size_t lds = static_cast<size_t>(tok) * route_row_stride(s.E, NF) * 4 + static_cast<size_t>(s.E) * 4;
    auto kern = route_fused_kernel<ST, TF, NW, NF>;
    if (lds > kRouteLdsMax) return hipErrorInvalidValue;     // cannot happen for E <= MOE_MAX_E (see kRouteLdsMax)
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), lds, st, static_cast<const ST*>(x),
                       static_cast<const ST*>(w_gate), bias, idx, gate, margin, chunk_hist, s.T, s.d_model, s.E, s.k,
                       s.renormalize);
    return hipGetLastError();
}

template <int TF, int NW>
static hipError_t launch_route_nf(int nf, const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                                  int32_t* idx, float* gate, float* margin, int32_t* chunk_hist, hipStream_t st) {
    switch (nf) {
        case 8:
            if constexpr (NW <= 8)
                return launch_route_inst<uint16_t, TF, NW, 8>(s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
            [[fallthrough]];
        case 4: return launch_route_inst<uint16_t, TF, NW, 4>(s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
        case 2: return launch_route_inst<uint16_t, TF, NW, 2>(s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
        default: return launch_route_inst<uint16_t, TF, NW, 1>(s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
    }
}

// Few tokens (a decode step): the gate product is one skinny GEMM whose cost is reading the gate weights, and
// one block per 16 tokens would leave that to one or two CUs.  gate_partial_kernel cuts it into
// (16 experts) x (1 / kGateSplit of the contraction) x (16 tokens) pieces, one wavefront each, which leave fp32
// partial logits in the workspace; route_topk_kernel adds the slices in order (plus the bias) and does the
// softmax / top-k / chunk histogram per 16 tokens as route_fused_kernel does.
__global__ __launch_bounds__(64) void gate_partial_kernel(const uint16_t* __restrict__ x,
                                                          const uint16_t* __restrict__ wg,
                                                          float* __restrict__ part, int T, int d, int E, int Tpad) {
    const int lane = threadIdx.x, r = lane & 15, g = lane >> 4;
    const int nb = blockIdx.x, ks = blockIdx.y, tf = blockIdx.z;
    const int ksteps = d >> 5;
    const int per = (ksteps + kGateSplit - 1) / kGateSplit;
    const int kb0 = min(ksteps, ks * per), kb1 = min(ksteps, kb0 + per);
    const uint16_t* xr = x + static_cast<size_t>(min(tf * 16 + r, T - 1)) * d + g * 8;
    const uint16_t* wr = wg + static_cast<size_t>(min(nb * 16 + r, E - 1)) * d + g * 8;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int PF = 8;
    for (int kb = kb0; kb < kb1; kb += PF) {
        bf16x8 a[PF], b[PF];
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int kk = min(kb + p, kb1 - 1);            // past the end: re-read, not used
            a[p] = *reinterpret_cast<const bf16x8*>(wr + kk * 32);
            b[p] = *reinterpret_cast<const bf16x8*>(xr + kk * 32);
        }
#pragma unroll
        for (int p = 0; p < PF; ++p)
            if (kb + p < kb1) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[p], b[p], acc, 0, 0, 0);
    }
    // lane (r, g): token tf * 16 + r, experts nb * 16 + 4 g + 0..3
    const int t = tf * 16 + r;
    float* dst = part + (static_cast<size_t>(ks) * Tpad + t) * E;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = nb * 16 + g * 4 + i;
        if (t < Tpad && e < E) dst[e] = acc[i];
    }
}

__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ part,
                                                         const float* __restrict__ bias,
                                                         int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                         float* __restrict__ margin,
                                                         int32_t* __restrict__ chunk_hist, int T, int E, int k,
                                                         int renorm, int Tpad) {
    extern __shared__ float lds[];
    const int Ep = E + 1;
    float* L = lds;
    int32_t* hist = reinterpret_cast<int32_t*>(lds + 16 * Ep);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t0 = blockIdx.x * 16;
    for (int e = threadIdx.x; e < E; e += 256) hist[e] = 0;
    // 4 logits per thread and pass: their 4 * kGateSplit partial sums are loaded before any is added (a wait
    // per logit otherwise: this kernel is two blocks of pure latency on the decode path)
    for (int i0 = threadIdx.x; i0 < 16 * E; i0 += 4 * 256) {
        float p[4][kGateSplit];
        float b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + u * 256, 16 * E - 1);   // past the end: re-read, not stored
            const int tl = i / E, e = i - tl * E;
            const int t = min(t0 + tl, Tpad - 1);
            b[u] = bias ? bias[e] : 0.f;
#pragma unroll
            for (int ks = 0; ks < kGateSplit; ++ks) p[u][ks] = part[(static_cast<size_t>(ks) * Tpad + t) * E + e];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * 256;
            if (i >= 16 * E) break;
            const int tl = i / E, e = i - tl * E;
            float s = b[u];
#pragma unroll
            for (int ks = 0; ks < kGateSplit; ++ks) s += p[u][ks];      // fixed order
            L[tl * Ep + e] = s;
        }
    }
    __syncthreads();
    const int grp = lane >> 4, sub = lane & 15;
    const int tl = wave * 4 + grp;                     // 4 wavefronts x 4 tokens
    const int t = t0 + tl;
    const bool live = t < T;
    const size_t o = static_cast<size_t>(live ? t : 0) * k;
    topk_from_lds(L + tl * Ep, E, k, renorm, sub, live, topk_idx + o, topk_w + o,
                  margin ? margin + (live ? t : 0) : nullptr, hist);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) chunk_hist[static_cast<size_t>(blockIdx.x) * E + e] = hist[e];
}

// route_topk_kernel and scan_finalize_kernel in one block of 1024 threads, for layers of at most 64 tokens and
// 256 experts (decoder steps): the 16 wavefronts take 4 tokens each, the four 16-token chunks keep their
// histograms in LDS, and the block goes straight on to the prefix sums, tile lists and (small layers) the
// placement.  One launch and one trip through memory less on a path that is a chain of short kernels.
// Dynamic LDS: logits [64][E + 1] floats, then histograms [4][E] ints.
constexpr int kTopkFinalizeMaxE = 256;
__global__ __launch_bounds__(1024) void route_topk_finalize_kernel(const float* __restrict__ part,
                                                                   const float* __restrict__ bias,
                                                                   int32_t* __restrict__ topk_idx,
                                                                   float* __restrict__ topk_w,
                                                                   float* __restrict__ margin,
                                                                   int32_t* __restrict__ chunk_hist, int T, int E, int k,
                                                                   int renorm, int Tpad, int32_t* __restrict__ counts,
                                                                   int32_t* __restrict__ offsets, int H,
                                                                   uint8_t* __restrict__ hot_mask,
                                                                   const uint8_t* __restrict__ mask_in,
                                                                   const TileLists lists, const int want_tiles,
                                                                   const PlaceArgs place) {
    extern __shared__ float lds[];
    const int Ep = E + 1;
    float* L = lds;
    int32_t* hist = reinterpret_cast<int32_t*>(lds + 64 * Ep);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nchunks = Tpad >> 4;                         // <= 4
    for (int i = threadIdx.x; i < 4 * E; i += 1024) hist[i] = 0;
    // 4 logits per thread and pass, their 4 * kGateSplit partial sums loaded before any is added
    for (int i0 = threadIdx.x; i0 < Tpad * E; i0 += 4 * 1024) {
        float p[4][kGateSplit];
        float b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + u * 1024, Tpad * E - 1);   // past the end: re-read, not stored
            const int tl = i / E, e = i - tl * E;
            b[u] = bias ? bias[e] : 0.f;
#pragma unroll
            for (int ks = 0; ks < kGateSplit; ++ks) p[u][ks] = part[(static_cast<size_t>(ks) * Tpad + tl) * E + e];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * 1024;
            if (i >= Tpad * E) break;
            const int tl = i / E, e = i - tl * E;
            float sum = b[u];
#pragma unroll
            for (int ks = 0; ks < kGateSplit; ++ks) sum += p[u][ks];      // fixed order
            L[tl * Ep + e] = sum;
        }
    }
    __syncthreads();
    const int grp = lane >> 4, sub = lane & 15;
    const int tl = wave * 4 + grp;                         // 16 wavefronts x 4 tokens
    if (wave * 4 < Tpad) {                                 // wave-uniform: Tpad is a multiple of 16
        const bool live = tl < T;
        const size_t o = static_cast<size_t>(live ? tl : 0) * k;
        topk_from_lds(L + tl * Ep, E, k, renorm, sub, live, topk_idx + o, topk_w + o,
                      margin ? margin + (live ? tl : 0) : nullptr, hist + (tl >> 4) * E);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nchunks * E; i += 1024) chunk_hist[i] = hist[i];     // [chunk][E], as the other kernels
    __threadfence_block();
    __syncthreads();
    scan_finalize_body(chunk_hist, nchunks, E, counts, offsets, H, hot_mask, mask_in, lists, want_tiles, place);
}

constexpr size_t kTopkFinalizeLdsMax = static_cast<size_t>(64) * (kTopkFinalizeMaxE + 1) * 4 + 4 * kTopkFinalizeMaxE * 4;

template <int TF, int NW>
static hipError_t configure_route_nf() {
    hipError_t e;
    if constexpr (NW <= 8) {
        if ((e = configure_route<uint16_t, TF, NW, 8>()) != hipSuccess) return e;
    }
    if ((e = configure_route<uint16_t, TF, NW, 4>()) != hipSuccess) return e;
    if ((e = configure_route<uint16_t, TF, NW, 2>()) != hipSuccess) return e;
    return configure_route<uint16_t, TF, NW, 1>();
}

hipError_t configure_route_kernels(int) {
    hipError_t e;
    if ((e = configure_route<float, 1, 4, 1>()) != hipSuccess) return e;
    if ((e = configure_route_nf<1, 16>()) != hipSuccess) return e;
    if ((e = configure_route_nf<4, ROUTE_BIG_NW>()) != hipSuccess) return e;
    if ((e = configure_route_nf<2, ROUTE_T4K_NW>()) != hipSuccess) return e;
    if ((e = configure_route_nf<1, ROUTE_MID_NW>()) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(route_topk_kernel),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kRouteLdsMax))) != hipSuccess)
        return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(route_topk_finalize_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kTopkFinalizeLdsMax));
}

static hipError_t launch_route_small(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                                     int32_t* idx, float* gate, float* margin, int32_t* chunk_hist, float* part,
                                     hipStream_t st) {
    const int tfs = (s.T + 15) / 16, Tpad = tfs * 16, nbs = (s.E + 15) / 16;
    hipLaunchKernelGGL(gate_partial_kernel, dim3(nbs, kGateSplit, tfs), dim3(64), 0, st,
                       static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_gate), part, s.T, s.d_model, s.E,
                       Tpad);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const size_t lds = static_cast<size_t>(16) * (s.E + 1) * 4 + static_cast<size_t>(s.E) * 4;   // <= 70 KiB
    hipLaunchKernelGGL(route_topk_kernel, dim3(tfs), dim3(256), lds, st, part, bias, idx, gate, margin, chunk_hist, s.T,
                       s.E, s.k, s.renormalize, Tpad);
    return hipGetLastError();
}

hipError_t launch_route_fused(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                              int32_t* idx, float* gate, float* margin, int32_t* chunk_hist, float* gate_part_ws,
                              hipStream_t st) {
    if (s.dtype != MOE_BF16)
        return launch_route_inst<float, 1, 4, 1>(s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
    if (route_is_split(s) && gate_part_ws != nullptr)
        return launch_route_small(s, x, w_gate, bias, idx, gate, margin, chunk_hist, gate_part_ws, st);
    const RouteCfg c = route_cfg(s);
    if (c.nw == 16) return launch_route_nf<1, 16>(c.nf, s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
    if (c.tok == 64) return launch_route_nf<4, ROUTE_BIG_NW>(c.nf, s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
    if (c.tok == 32) return launch_route_nf<2, ROUTE_T4K_NW>(c.nf, s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
    return launch_route_nf<1, ROUTE_MID_NW>(c.nf, s, x, w_gate, bias, idx, gate, margin, chunk_hist, st);
}

// the finalize block places the assignments itself when there are few of them and the per-wavefront slot
// tables fit into LDS
bool scan_can_place(const moe_shape& s) {
    return s.E <= kScanPlaceMaxE && static_cast<long>(s.T) * s.k <= kScanPlaceMaxA;
}

hipError_t launch_scan_finalize(int32_t* chunk_hist, int nchunks, int E, int32_t* counts, int32_t* offsets, int H,
                                uint8_t* hot_mask, const uint8_t* mask_in, const TileLists* lists,
                                const PlaceArgs* place, hipStream_t st) {
    const TileLists none{nullptr, nullptr, nullptr, nullptr, 16, 0};
    const PlaceArgs no_place{nullptr, nullptr, nullptr, nullptr, 0, 1, 1};
    hipLaunchKernelGGL(scan_finalize_kernel, dim3(1), dim3(1024), 0, st, chunk_hist, nchunks, E, counts, offsets, H,
                       hot_mask, mask_in, lists ? *lists : none, lists ? 1 : 0, place ? *place : no_place);
    return hipGetLastError();
}

// routing followed by the finalize step; one kernel does both for decoder-sized layers
hipError_t launch_route_finalize(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                                 int32_t* idx, float* gate, float* margin, int32_t* hist_ws, float* gate_part_ws,
                                 int32_t* counts, int32_t* offsets, int H, uint8_t* hot_mask, const uint8_t* mask_in,
                                 const TileLists* lists, const PlaceArgs* place, hipStream_t st) {
    int nchunks = 0;
    if (s.T > 0) {
        const int tok = route_chunk_tokens(s);
        nchunks = (s.T + tok - 1) / tok;
        if (route_is_split(s) && gate_part_ws != nullptr && s.E <= kTopkFinalizeMaxE) {
            const int tfs = (s.T + 15) / 16, Tpad = tfs * 16, nbs = (s.E + 15) / 16;
            hipLaunchKernelGGL(gate_partial_kernel, dim3(nbs, kGateSplit, tfs), dim3(64), 0, st,
                               static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w_gate), gate_part_ws, s.T,
                               s.d_model, s.E, Tpad);
            hipError_t err = hipGetLastError();
            if (err != hipSuccess) return err;
            // at most kTopkFinalizeLdsMax: the limit configure_route_kernels has raised this kernel to
            const size_t lds = static_cast<size_t>(64) * (s.E + 1) * 4 + static_cast<size_t>(4) * s.E * 4;
            const TileLists none{nullptr, nullptr, nullptr, nullptr, 16, 0};
            const PlaceArgs no_place{nullptr, nullptr, nullptr, nullptr, 0, 1, 1};
            hipLaunchKernelGGL(route_topk_finalize_kernel, dim3(1), dim3(1024), lds, st, gate_part_ws, bias, idx, gate,
                               margin, hist_ws, s.T, s.E, s.k, s.renormalize, Tpad, counts, offsets, H, hot_mask, mask_in,
                               lists ? *lists : none, lists ? 1 : 0, place ? *place : no_place);
            return hipGetLastError();
        }
        hipError_t err = launch_route_fused(s, x, w_gate, bias, idx, gate, margin, hist_ws, gate_part_ws, st);
        if (err != hipSuccess) return err;
    }
    return launch_scan_finalize(hist_ws, nchunks, s.E, counts, offsets, H, hot_mask, mask_in, lists, place, st);
}

hipError_t launch_route(const moe_shape& s, const void* x, const void* w_gate, const float* bias,
                        int32_t* idx, float* gate, float* margin, int32_t* counts,
                        int32_t* offsets, int32_t H, uint8_t* hot_mask, int32_t* hist_ws, float* gate_part_ws,
                        hipStream_t st) {
    return launch_route_finalize(s, x, w_gate, bias, idx, gate, margin, hist_ws, gate_part_ws, counts, offsets, H, hot_mask,
                                 nullptr, nullptr, nullptr, st);
}

}  // namespace moe
