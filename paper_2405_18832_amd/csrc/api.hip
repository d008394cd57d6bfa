// C ABI of the MoE FFN library: argument validation on the host, then asynchronous kernel
// launches on the caller's stream.  No entry point allocates, synchronises or copies to the host.
#include <atomic>
#include <cmath>
#include <mutex>

#include "common.hpp"

using namespace moe;

// Scratch memory of the entry point that allocates nothing (moe_layer_forward_noalloc): one array per GPU that
// loads this library, held until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress; the device address it yields (per device) is what kernels and host calls are given.
constexpr size_t kScratchBytes = static_cast<size_t>(MOE_NOALLOC_MAX_WORKSPACE);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

std::mutex g_setup_mutex;
std::atomic<bool> g_device_ready[kMaxDevices];
void* g_scratch_ptr[kMaxDevices] = {nullptr};     // device address of `scratch` on each device (set under the lock)

moe_status check_shape(const moe_shape* s) {
    if (s == nullptr) return MOE_ERR_INVALID_ARG;
    if (s->T < 0 || s->d_model <= 0 || s->d_ff <= 0 || s->E <= 0 || s->k <= 0) return MOE_ERR_INVALID_ARG;
    if (s->k > s->E) return MOE_ERR_INVALID_ARG;
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_INVALID_ARG;
    if (s->renormalize != 0 && s->renormalize != 1) return MOE_ERR_INVALID_ARG;
    if (s->activation != MOE_ACT_RELU && s->activation != MOE_ACT_GELU) return MOE_ERR_UNSUPPORTED;
    if (s->k > MOE_MAX_K || s->E > MOE_MAX_E) return MOE_ERR_UNSUPPORTED;
    if (s->dtype == MOE_BF16 && (s->d_model % 32 != 0 || s->d_ff % 32 != 0)) return MOE_ERR_UNSUPPORTED;
    // int32 indexing of assignments and of rows
    const long long A = static_cast<long long>(s->T) * s->k;
    if (A > 0x3fffffffLL) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

moe_status check_ws(const moe_shape* s, const void* ws, size_t ws_bytes) {
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return MOE_ERR_WORKSPACE;
    if (ws_bytes < ws_layout(*s).total) return MOE_ERR_WORKSPACE;
    return MOE_OK;
}

inline moe_status from_hip(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_HIP; }

template <typename T> inline T* at(void* ws, size_t off) {
    return reinterpret_cast<T*>(static_cast<char*>(ws) + off);
}

}  // namespace

namespace moe {

int current_device_index() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    return dev;
}

hipError_t ensure_ready() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (g_device_ready[dev].load(std::memory_order_acquire)) return hipSuccess;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (g_device_ready[dev].load(std::memory_order_acquire)) return hipSuccess;
    if ((e = configure_ffn_kernels(dev)) != hipSuccess) return e;
    if ((e = configure_tile_kernels(dev)) != hipSuccess) return e;
    if ((e = configure_route_kernels(dev)) != hipSuccess) return e;
    // this device's copy of the scratch array (each GPU has its own, at its own address)
    void* p = nullptr;
    if ((e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
    g_device_ready[dev].store(true, std::memory_order_release);
    return hipSuccess;
}

}  // namespace moe

extern "C" {

moe_status moe_init(void) { return from_hip(ensure_ready()); }

const char* moe_status_string(moe_status s) {
    switch (s) {
        case MOE_OK: return "MOE_OK";
        case MOE_ERR_INVALID_ARG: return "MOE_ERR_INVALID_ARG";
        case MOE_ERR_UNSUPPORTED: return "MOE_ERR_UNSUPPORTED";
        case MOE_ERR_WORKSPACE: return "MOE_ERR_WORKSPACE";
        case MOE_ERR_HIP: return "MOE_ERR_HIP";
    }
    return "MOE_ERR_UNKNOWN";
}

size_t moe_workspace_bytes(const moe_shape* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    return ws_layout(*shape).total;
}

size_t moe_packed_weight_bytes(const moe_shape* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    return static_cast<size_t>(shape->E) * shape->d_model * shape->d_ff * elem_size(shape->dtype);
}

int32_t moe_tiled_kernel_min_rows(const moe_shape* shape, const int32_t* rows_host) {
    if (check_shape(shape) != MOE_OK || rows_host == nullptr) return 0;
    (void)ensure_ready();                                   // the device's CU count; a default stands in without one
    const TileLists l = ffn_tile_lists(*shape, nullptr, nullptr, nullptr, nullptr);
    if (l.big_min <= 0) return 0;
    int big_tiles = 0;
    for (int e = 0; e < shape->E; ++e)
        if (rows_host[e] >= l.big_min) big_tiles += (rows_host[e] + kBigTileRows - 1) / kBigTileRows;
    return tiled_min_rows(big_tiles, l.small_rows, l.join_tiles);
}

void moe_set_profile_events(void* const* events) {
    set_profile_events(reinterpret_cast<const hipEvent_t*>(events));
}

moe_status moe_pack_weights(const moe_shape* shape, int32_t which, const void* src, void* dst, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((which != 1 && which != 2) || src == nullptr || dst == nullptr || src == dst) return MOE_ERR_INVALID_ARG;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    return from_hip(launch_pack(*shape, which, src, dst, static_cast<hipStream_t>(stream)));
}

moe_status moe_route(const moe_shape* shape, const void* x, const void* w_gate, const float* gate_bias,
                     int32_t* topk_idx, float* topk_w, float* margin, int32_t* counts, int32_t* offsets,
                     int32_t H, uint8_t* hot_mask, void* ws, size_t ws_bytes, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (counts == nullptr || offsets == nullptr) return MOE_ERR_INVALID_ARG;
    if (H >= 0 && hot_mask == nullptr) return MOE_ERR_INVALID_ARG;
    // with no tokens the per-token buffers are empty and may be NULL
    if (shape->T > 0 && (x == nullptr || w_gate == nullptr || topk_idx == nullptr || topk_w == nullptr))
        return MOE_ERR_INVALID_ARG;
    st = check_ws(shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    const WsLayout L = ws_layout(*shape);
    return from_hip(launch_route(*shape, x, w_gate, gate_bias, topk_idx, topk_w, margin, counts, offsets, H,
                                 hot_mask, at<int32_t>(ws, L.hist), at<float>(ws, L.gate_part),
                                 static_cast<hipStream_t>(stream)));
}

size_t moe_parameter_movement_bytes(const moe_shape* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    return static_cast<size_t>(2) * shape->E * shape->d_model * shape->d_ff * elem_size(shape->dtype);
}

size_t moe_activation_movement_bytes(const moe_shape* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    return static_cast<size_t>(2) * shape->T * shape->d_model * elem_size(shape->dtype);
}

moe_status moe_plan_devices(int32_t E, const int32_t* counts, const uint8_t* skip, int32_t n_devices,
                            int32_t* device_of) {
    if (counts == nullptr || device_of == nullptr || n_devices < 1 || E < 1 || E > MOE_MAX_E) return MOE_ERR_INVALID_ARG;
    for (int e = 0; e < E; ++e)
        if (counts[e] < 0) return MOE_ERR_INVALID_ARG;
    int order[MOE_MAX_E];
    int n = 0;
    for (int e = 0; e < E; ++e) {
        device_of[e] = -1;
        if (counts[e] > 0 && (skip == nullptr || skip[e] == 0)) order[n++] = e;
    }
    // insertion sort, stable: count descending, equal counts stay in index order
    for (int i = 1; i < n; ++i) {
        const int e = order[i];
        int j = i;
        while (j > 0 && counts[order[j - 1]] < counts[e]) {
            order[j] = order[j - 1];
            --j;
        }
        order[j] = e;
    }
    for (int i = 0; i < n; ++i) device_of[order[i]] = i % n_devices;
    return MOE_OK;
}

moe_status moe_fetch_experts(const moe_shape* shape, int32_t which, const void* src_host,
                             const uint8_t* fetch_mask_host, void* dst_device, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if ((which != 1 && which != 2) || src_host == nullptr || fetch_mask_host == nullptr || dst_device == nullptr)
        return MOE_ERR_INVALID_ARG;
    const size_t per_expert = static_cast<size_t>(shape->d_model) * shape->d_ff * elem_size(shape->dtype);
    for (int e = 0; e < shape->E; ++e) {
        if (fetch_mask_host[e] == 0) continue;
        const hipError_t err = hipMemcpyAsync(static_cast<char*>(dst_device) + e * per_expert,
                                              static_cast<const char*>(src_host) + e * per_expert, per_expert,
                                              hipMemcpyHostToDevice, static_cast<hipStream_t>(stream));
        if (err != hipSuccess) return MOE_ERR_HIP;
    }
    return MOE_OK;
}

moe_status moe_select_hot(const moe_shape* shape, const int32_t* counts, double alpha, double bw_a, double bw_b,
                          int32_t* H_out, uint8_t* hot_mask, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (counts == nullptr) return MOE_ERR_INVALID_ARG;
    if (!(alpha >= 0.0) || !(bw_a > 0.0) || !(bw_b >= 0.0) || std::isinf(alpha) || std::isinf(bw_a) || std::isinf(bw_b))
        return MOE_ERR_INVALID_ARG;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    return from_hip(launch_select_hot(shape->E, counts, alpha, bw_a, bw_b, H_out, hot_mask,
                                      static_cast<hipStream_t>(stream)));
}

moe_status moe_tune_alpha(double alpha, double bw_a, double bw_b, int32_t n_batches, const int32_t* activated,
                          int32_t n_candidates, const double* times, double* alpha_out, int32_t* best_offset_out) {
    if (activated == nullptr || times == nullptr || n_batches < 1 || n_candidates < 1) return MOE_ERR_INVALID_ARG;
    if (!(alpha >= 0.0) || !(bw_a > 0.0) || !(bw_b >= 0.0) || std::isinf(alpha) || std::isinf(bw_a) || std::isinf(bw_b))
        return MOE_ERR_INVALID_ARG;
    long long total_activ = 0;
    for (int b = 0; b < n_batches; ++b) {
        if (activated[b] < 0) return MOE_ERR_INVALID_ARG;
        total_activ += activated[b];
        for (int c = 0; c < n_candidates; ++c) {
            const double t = times[static_cast<size_t>(b) * n_candidates + c];
            if (!(t > 0.0) || std::isinf(t)) return MOE_ERR_INVALID_ARG;
        }
    }
    // totals per candidate, summed in batch order; the smallest total wins, the smaller offset on equal totals
    int best = 0;
    double best_total = 0.0;
    for (int c = 0; c < n_candidates; ++c) {
        double total = 0.0;
        for (int b = 0; b < n_batches; ++b) total = total + times[static_cast<size_t>(b) * n_candidates + c];
        if (c == 0 || total < best_total) {
            best = c;
            best_total = total;
        }
    }
    double tuned = alpha;
    if (best != 0 && total_activ != 0) {
        const double rho = bw_a / (bw_a + bw_b);
        const double mean = static_cast<double>(total_activ) / static_cast<double>(n_batches);
        const double step = static_cast<double>(best) / (rho * mean);
        tuned = alpha + step;
    }
    if (alpha_out != nullptr) *alpha_out = tuned;
    if (best_offset_out != nullptr) *best_offset_out = best;
    return MOE_OK;
}

moe_status moe_permute(const moe_shape* shape, const void* x, const int32_t* topk_idx, const int32_t* offsets,
                       int32_t* perm, int32_t* inv_perm, void* x_perm, void* ws, size_t ws_bytes, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    if (topk_idx == nullptr || offsets == nullptr || perm == nullptr || inv_perm == nullptr)
        return MOE_ERR_INVALID_ARG;
    if (x_perm != nullptr && x == nullptr) return MOE_ERR_INVALID_ARG;
    st = check_ws(shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    const WsLayout L = ws_layout(*shape);
    return from_hip(launch_permute(*shape, x, topk_idx, offsets, perm, inv_perm, x_perm, at<int32_t>(ws, L.hist),
                                   static_cast<hipStream_t>(stream)));
}

moe_status moe_expert_ffn(const moe_shape* shape, const void* x_perm, const void* w1, const void* w2,
                          const int32_t* offsets, const uint8_t* mask, float* y_perm, void* ws, size_t ws_bytes,
                          void* stream) {
    return moe_expert_ffn_biased(shape, x_perm, w1, nullptr, w2, nullptr, offsets, mask, y_perm, ws, ws_bytes, stream);
}

moe_status moe_expert_ffn_biased(const moe_shape* shape, const void* x_perm, const void* w1, const float* b1,
                                 const void* w2, const float* b2, const int32_t* offsets, const uint8_t* mask,
                                 float* y_perm, void* ws, size_t ws_bytes, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    if (x_perm == nullptr || w1 == nullptr || w2 == nullptr || offsets == nullptr || y_perm == nullptr)
        return MOE_ERR_INVALID_ARG;
    st = check_ws(shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    const WsLayout L = ws_layout(*shape);
    return from_hip(launch_expert_ffn(*shape, x_perm, w1, w2, b1, b2, offsets, mask, y_perm, at<void>(ws, L.h),
                                      at<Tile>(ws, L.tiles), at<Tile>(ws, L.tiles_big), at<int32_t>(ws, L.ntiles),
                                      at<float>(ws, L.partials), at<void>(ws, L.x_kmajor), static_cast<hipStream_t>(stream)));
}

moe_status moe_combine(const moe_shape* shape, const float* y_perm, const int32_t* inv_perm,
                       const int32_t* topk_idx, const float* topk_w, const uint8_t* mask, void* out, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (shape->T == 0) return MOE_OK;
    if (y_perm == nullptr || inv_perm == nullptr || topk_idx == nullptr || topk_w == nullptr || out == nullptr)
        return MOE_ERR_INVALID_ARG;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    return from_hip(launch_combine(*shape, y_perm, inv_perm, topk_idx, topk_w, mask, out,
                                   static_cast<hipStream_t>(stream)));
}

moe_status moe_layer_forward(const moe_shape* shape, const void* x, const void* w_gate, const float* gate_bias,
                             const void* w1, const void* w2, const uint8_t* mask, int32_t H, void* out,
                             int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* perm,
                             uint8_t* hot_mask_out, void* ws, size_t ws_bytes, void* stream) {
    return moe_layer_forward_biased(shape, x, w_gate, gate_bias, w1, nullptr, w2, nullptr, mask, H, out, topk_idx,
                                    topk_w, counts, perm, hot_mask_out, ws, ws_bytes, stream);
}

moe_status moe_layer_forward_biased(const moe_shape* shape, const void* x, const void* w_gate,
                                    const float* gate_bias, const void* w1, const float* b1, const void* w2,
                                    const float* b2, const uint8_t* mask, int32_t H, void* out, int32_t* topk_idx,
                                    float* topk_w, int32_t* counts, int32_t* perm, uint8_t* hot_mask_out, void* ws,
                                    size_t ws_bytes, void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    if (shape->T > 0 && (x == nullptr || w_gate == nullptr || w1 == nullptr || w2 == nullptr || out == nullptr))
        return MOE_ERR_INVALID_ARG;
    st = check_ws(shape, ws, ws_bytes);
    if (st != MOE_OK) return st;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const WsLayout L = ws_layout(*shape);
    int32_t* idx = topk_idx ? topk_idx : at<int32_t>(ws, L.idx);
    float* gate = topk_w ? topk_w : at<float>(ws, L.gate);
    int32_t* cnt = counts ? counts : at<int32_t>(ws, L.counts);
    int32_t* offsets = at<int32_t>(ws, L.offsets);
    int32_t* inv = at<int32_t>(ws, L.inv_perm);
    uint8_t* own_mask = at<uint8_t>(ws, L.mask);
    const bool derive = (mask == nullptr && H >= 0);
    const uint8_t* used = mask ? mask : (derive ? own_mask : nullptr);

    // route -> chunk histograms; one block turns them into counts, offsets, slot bases, the hot mask and the
    // tile list; the chunks place their assignments; the first product gathers token rows through tokmap.
    int32_t* hist = at<int32_t>(ws, L.hist);
    int32_t* tokmap = at<int32_t>(ws, L.tokmap);
    const TileLists lists = ffn_tile_lists(*shape, at<Tile>(ws, L.tiles), at<Tile>(ws, L.tiles_big),
                                           at<int32_t>(ws, L.ntiles), at<float>(ws, L.partials));
    hipError_t e;
    const int tok = route_chunk_tokens(*shape);
    // few assignments: the finalize block also places them (one launch less)
    const bool fused_place = shape->T > 0 && scan_can_place(*shape);
    const PlaceArgs place{idx, perm, inv, tokmap, shape->T * shape->k, shape->k, tok * shape->k};
    e = launch_route_finalize(*shape, x, w_gate, gate_bias, idx, gate, nullptr, hist, at<float>(ws, L.gate_part), cnt,
                              offsets, derive ? H : -1, derive ? own_mask : nullptr, mask, &lists,
                              fused_place ? &place : nullptr, hs);
    if (e != hipSuccess) return MOE_ERR_HIP;
    if (hot_mask_out != nullptr) {
        e = launch_mask_out(used, hot_mask_out, shape->E, hs);
        if (e != hipSuccess) return MOE_ERR_HIP;
    }
    if (shape->T == 0) return MOE_OK;
    if (!fused_place) {
        e = launch_place(*shape, idx, offsets, hist, perm, inv, tokmap, tok * shape->k, hs);
        if (e != hipSuccess) return MOE_ERR_HIP;
    }
    // One expert per token and every expert running: each row of the permuted order is the whole output of
    // its token, so the second product scales it by the gate weight and writes `out` directly (Section 2.1's
    // combine step without the fp32 round trip through memory); otherwise a combine pass follows.
    const bool folded = shape->k == 1 && used == nullptr && shape->dtype == MOE_BF16;
    const FoldOut fold{folded ? static_cast<uint16_t*>(out) : nullptr, tokmap, gate};
    if (layer_gathers_kmajor(*shape)) {
        // layers large enough for the tiled kernel: one pass gathers the token rows into the k-step-major
        // layout that lets both kernels fetch operand rows as full cache lines
        void* xk = at<void>(ws, L.x_kmajor);
        e = launch_gather_kmajor(*shape, x, tokmap, xk, hs);
        if (e != hipSuccess) return MOE_ERR_HIP;
        e = launch_expert_products(*shape, xk, nullptr, true, w1, w2, b1, b2, at<float>(ws, L.y_perm), at<void>(ws, L.h), lists,
                                   fold, hs);
    } else {
        e = launch_expert_products(*shape, x, tokmap, false, w1, w2, b1, b2, at<float>(ws, L.y_perm), at<void>(ws, L.h), lists,
                                   fold, hs);
    }
    if (e != hipSuccess) return MOE_ERR_HIP;
    if (folded) return MOE_OK;                 // the second product has written `out`
    e = launch_combine(*shape, at<float>(ws, L.y_perm), inv, idx, gate, used, out, hs);
    return from_hip(e);
}

size_t moe_noalloc_max_workspace(void) { return kScratchBytes; }

moe_status moe_layer_forward_noalloc(const moe_shape* shape, const void* x, const void* w_gate, const float* gate_bias,
                                     const void* w1, const void* w2, const uint8_t* mask, int32_t H, void* out,
                                     void* stream) {
    moe_status st = check_shape(shape);
    if (st != MOE_OK) return st;
    // the layer's whole workspace must fit into the static array
    if (ws_layout(*shape).total > kScratchBytes) return MOE_ERR_WORKSPACE;
    if (ensure_ready() != hipSuccess) return MOE_ERR_HIP;
    void* ws = g_scratch_ptr[current_device_index()];      // the device address, never the array's name
    if (ws == nullptr) return MOE_ERR_HIP;
    // Everything the layer reads from its workspace it has written earlier in the same call (counters and
    // histograms are cleared by its kernels), so the contents a previous call left behind do not matter.
    return moe_layer_forward_biased(shape, x, w_gate, gate_bias, w1, nullptr, w2, nullptr, mask, H, out, nullptr,
                                    nullptr, nullptr, nullptr, nullptr, ws, kScratchBytes, stream);
}

}  // extern "C"
