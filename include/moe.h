/*
 * moe.h -- C ABI of the MoE FFN layer forward for AMD MI355X (gfx950).
 *
 * The layer is the one the MoNDE paper (arXiv 2405.18832) describes in Section 2.1
 * and Fig. 1: a gating network scores every (token, expert) pair, each token is
 * routed to its top-k experts, each expert is linear -> ReLU -> linear, and the
 * expert outputs are weighted, summed and put back in the original token order.
 * Section 3.3 splits the experts into a "hot" set (the H experts with the most
 * tokens) and the rest; every call that runs experts takes an expert mask so the
 * same library computes the whole layer or only one side's share.
 *
 * Notation: T tokens, d = d_model, f = d_ff, E experts, k experts per token,
 * A = T*k assignments; the flat assignment id is a = t*k + j, slot j = 0 being the
 * token's best expert.
 *
 * General rules for every entry point
 *  - Every pointer is a DEVICE pointer owned by the caller unless it says "host".
 *    The library never allocates, frees or keeps a pointer.  Scratch memory comes
 *    from the caller's workspace `ws` (device, 256-byte aligned, at least
 *    moe_workspace_bytes(shape) bytes).
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls are
 *    asynchronous on it; they never synchronise and never copy to the host.  Token
 *    counts stay on the device: kernels read them there.
 *  - Arguments are validated on the host before anything is launched; on an error
 *    nothing is written (one exception, stated there: moe_fetch_experts).  Errors are
 *    return codes only.
 *  - Every entry point works on the calling thread's current HIP device.  The first call on a
 *    device (or moe_init) sets the kernels up for it once, under a lock; after that, calls from
 *    several host threads and on several devices are independent, except where a call says
 *    otherwise (moe_set_profile_events, moe_layer_forward_noalloc).
 *  - Row-major everywhere, last index contiguous.  dtype selects the storage type
 *    of x, w_gate, W1, W2, x_perm and out; products are accumulated in fp32.
 *    Gate weights, logits margins and y_perm are always fp32; indices are int32.
 *  - MOE_BF16 requires d_model % 32 == 0 and d_ff % 32 == 0.  1 <= k <= 8, k <= E,
 *    E <= 1024, T >= 0.  With T == 0 the per-token buffers are empty and may be NULL:
 *    moe_route still writes zero counts/offsets (and the hot mask), the other calls are
 *    no-ops that return MOE_OK.
 */
#ifndef MOE_FFN_MI355X_H
#define MOE_FFN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1,   /* null pointer, bad size, bad enum value            */
    MOE_ERR_UNSUPPORTED = 2,   /* legal request outside what the kernels cover      */
    MOE_ERR_WORKSPACE = 3,     /* ws is NULL, misaligned or smaller than required   */
    MOE_ERR_HIP = 4            /* a HIP call or kernel launch failed                */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

/* trailing activation of an expert's first linear layer (Section 3.4: "ReLU or GeLU") */
typedef enum { MOE_ACT_RELU = 0, MOE_ACT_GELU = 1 } moe_activation;

typedef struct {
    int32_t T, d_model, d_ff, E, k;
    int32_t dtype;         /* moe_dtype                                              */
    int32_t renormalize;   /* 0: gate = p_e ; 1: gate = p_e / sum of the chosen k p   */
    int32_t activation;    /* moe_activation: 0 = ReLU, 1 = GeLU (z * Phi(z), erf form) */
} moe_shape;

#define MOE_MAX_K 8
#define MOE_MAX_E 1024

/*
 * One-time set-up for the current device: raises the kernels' dynamic-LDS limits and asks the runtime for
 * their occupancy.  Optional -- every entry point that launches kernels does the same on its first call on a
 * device -- but a caller that records its first call into a HIP graph should call it before the capture
 * starts, so that none of these runtime calls happens while the stream is capturing.  Thread-safe; repeated
 * calls return at once.  MOE_ERR_HIP if the runtime refuses.
 */
moe_status moe_init(void);

/* Human-readable name of a status code (host pointer to a static string). */
const char* moe_status_string(moe_status s);

/* Bytes of workspace that any entry point may need for this shape (0 on a bad shape). */
size_t moe_workspace_bytes(const moe_shape* shape);

/* Bytes of one packed expert-weight tensor (W1 and W2 have the same size). */
size_t moe_packed_weight_bytes(const moe_shape* shape);

/*
 * One-time weight preparation (inference weights are static; Section 4.1 runs
 * pre-trained models).  `which` = 1: src is W1 [E, f, d]; `which` = 2: src is
 * W2 [E, d, f]; both "out-features x in-features".  dst receives the layout that
 * moe_expert_ffn / moe_layer_forward read:
 *   MOE_F32 : a plain copy.
 *   MOE_BF16: for each expert, 16-row x 32-column fragments, fragment (nb, kb) at
 *             element offset ((nb * (K/32)) + kb) * 512; inside a fragment the 8
 *             elements src[16*nb + (l % 16)][32*kb + 8*(l / 16) + 0..7] sit at
 *             offset 8*l, l = 0..63 -- one 16-byte piece per wavefront lane, in the
 *             order the MFMA 16x16x32 operand wants them, so a whole fragment is one
 *             contiguous 1 KiB load.
 * src and dst must not overlap.
 */
moe_status moe_pack_weights(const moe_shape* shape, int32_t which, const void* src,
                            void* dst, void* stream);

/*
 * Gating and routing (Section 2.1; Section 3.3 for the histogram and the hot set).
 *   x [T, d], w_gate [E, d] (row e = gate weights of expert e), gate_bias [E] fp32 or NULL.
 *   logits = x . w_gate^T + bias (fp32); p = softmax over experts;
 *   topk_idx [T, k]: experts of the k largest logits, descending, equal logits ordered
 *                    by lowest expert index;
 *   topk_w  [T, k]: p of the chosen experts, renormalised over the k if shape->renormalize;
 *   margin  [T] or NULL: smallest gap between consecutive entries of the k+1 largest logits;
 *   counts  [E]: assignments per expert; offsets [E+1]: exclusive prefix sum, offsets[E] = A;
 *   H >= 0 and hot_mask != NULL: hot_mask[e] = 1 for the min(H, E) experts with the largest
 *                    counts (equal counts ordered by lowest index), else 0.  H < 0: untouched.
 */
moe_status moe_route(const moe_shape* shape, const void* x, const void* w_gate,
                     const float* gate_bias, int32_t* topk_idx, float* topk_w, float* margin,
                     int32_t* counts, int32_t* offsets, int32_t H, uint8_t* hot_mask,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * Data-movement model of Section 3.2, in bytes of the shape's storage dtype (host arithmetic, no GPU):
 *   parameter movement  (Eq. 1) = 2 * E * d_model * d_ff  values: all experts' weights to the compute device;
 *   activation movement (Eq. 2) = 2 * T * d_model        values: the tokens to the experts and back.
 * 0 on a bad shape.
 */
size_t moe_parameter_movement_bytes(const moe_shape* shape);
size_t moe_activation_movement_bytes(const moe_shape* shape);

/*
 * Load balancing over several expert-holding devices (Section 3.3, last paragraph: the expert workloads,
 * sorted by compute intensity, are dealt out round-robin).  Host arithmetic, no GPU, HOST pointers.
 *   counts [E]   tokens per expert (all experts have the same shape, so compute intensity orders like the
 *                token count); skip [E] or NULL: experts with skip[e] != 0 take no part (e.g. the hot set that
 *                stays on the main device).
 *   device_of [E] out: experts with counts[e] > 0 that are not skipped, ordered by count descending (equal
 *                counts by lowest index), get devices 0, 1, ..., n_devices-1, 0, 1, ... in that order; every
 *                other expert gets -1.
 * MOE_ERR_INVALID_ARG on a NULL counts / device_of, n_devices < 1 or a negative count; nothing is written then.
 */
moe_status moe_plan_devices(int32_t E, const int32_t* counts, const uint8_t* skip, int32_t n_devices,
                            int32_t* device_of);

/*
 * Parameter movement on demand (Section 3.2, Section 4.1: only activated experts are brought in): copies the
 * packed weights (`which` = 1: W1, 2: W2) of the experts with fetch_mask[e] != 0 from a HOST buffer holding all
 * E experts' packed weights (layout of moe_pack_weights; pinned memory for an asynchronous copy) to the same
 * offsets of a DEVICE buffer of the same size, one copy per expert on `stream`; other experts' device memory
 * is left as it is.  fetch_mask is a HOST array [E] -- the caller has brought counts or a hot mask over, that
 * being the one host round trip the scheme needs.  Returns after enqueueing.  Arguments are validated before
 * the first copy; if the runtime then refuses a copy the call returns MOE_ERR_HIP at once, and the copies of
 * the experts before that one stay enqueued (the only case in this library where an error leaves a partial
 * effect: treat the destination's contents as undefined).
 */
moe_status moe_fetch_experts(const moe_shape* shape, int32_t which, const void* src_host,
                             const uint8_t* fetch_mask_host, void* dst_device, void* stream);

/*
 * Hot-set size of the load-balancing rule (Section 3.3, Eq. 3-6) and the hot mask it implies.
 * The hot workflow is fed at bandwidth bw_a, the cold one at bw_b (any common unit); both are
 * bound by moving expert parameters, so equal runtimes put bw_a / (bw_a + bw_b) of the activated
 * experts (those with at least one token) on the hot side; alpha is the paper's tuning factor:
 *   H = alpha * bw_a / (bw_a + bw_b) * #{e : counts[e] > 0},
 * evaluated in double precision in this order, rounded to the nearest integer with halves up and
 * clipped to [0, E] (the paper leaves the rounding open).
 *   counts [E] device, as written by moe_route; H_out: device int32 (may be NULL);
 *   hot_mask [E] device (may be NULL): 1 for the H experts with the largest counts, equal counts
 *   ordered by lowest index -- the mask moe_expert_ffn / moe_combine / moe_layer_forward take.
 * alpha >= 0, bw_a > 0, bw_b >= 0, all finite, else MOE_ERR_INVALID_ARG.  One small kernel on `stream`.
 */
moe_status moe_select_hot(const moe_shape* shape, const int32_t* counts, double alpha, double bw_a,
                          double bw_b, int32_t* H_out, uint8_t* hot_mask, void* stream);

/*
 * Auto-tuning of alpha (Section 3.3, the paragraph after Eq. 6: the factor is tuned by running profiled inference
 * on a small set of past input batches and finding the local optimum among the candidates H, H + 1, H + 2).
 * Host arithmetic, no GPU, HOST pointers.  The caller runs its past batches with H_b + c hot experts, c = 0 ...
 * n_candidates - 1 (H_b = moe_select_hot at the current alpha; moe_layer_forward takes H directly) and measures:
 *   activated [n_batches]                activated experts of each batch (experts with at least one token);
 *   times     [n_batches, n_candidates]  measured time of batch b with H_b + c hot experts (any unit, > 0).
 * best_offset_out: the c with the smallest total time over the batches (the smallest such c on equal totals).
 * alpha_out: the paper leaves open how the chosen candidate becomes a new alpha; here it is the alpha at which
 * Eq. 6's real-valued H of a batch with the mean number of activated experts is best_offset larger:
 *   alpha + best_offset / (bw_a / (bw_a + bw_b) * mean(activated)),
 * evaluated in double precision in this order; alpha itself when best_offset is 0 or no expert was activated.
 * Either output may be NULL.  MOE_ERR_INVALID_ARG on NULL inputs, n_batches < 1, n_candidates < 1, a negative
 * count, a time that is not finite and positive, or bandwidths / alpha outside moe_select_hot's domain; nothing
 * is written then.
 */
moe_status moe_tune_alpha(double alpha, double bw_a, double bw_b, int32_t n_batches, const int32_t* activated,
                          int32_t n_candidates, const double* times, double* alpha_out, int32_t* best_offset_out);

/*
 * Dispatch (Section 2.1 "route each token to the top-k experts"; Section 4.1: drop-less,
 * padding-less).  Stable counting sort of the A assignments by expert:
 *   perm [A]: perm[p] = flat assignment id at sorted position p (experts ascending, inside
 *             an expert ascending flat id);  inv_perm [A]: inv_perm[perm[p]] = p;
 *   x_perm [A, d] (dtype) or NULL: x_perm[p] = x[perm[p] / k].
 * `offsets` must be the prefix sums that belong to `topk_idx` (as moe_route writes them).
 */
moe_status moe_permute(const moe_shape* shape, const void* x, const int32_t* topk_idx,
                       const int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * Expert FFNs as one grouped product (Section 2.1: two linear layers with an activation
 * between; Section 3.1/3.4: C = A x B with a trailing ReLU, then C = A x B).
 * For every expert e with mask[e] != 0 (mask == NULL: all) and offsets[e+1] > offsets[e]:
 *   y_perm[offsets[e] .. offsets[e+1]) = relu(X_e . W1_e^T) . W2_e^T        (fp32 rows)
 * x_perm [A, d] (dtype); w1, w2: packed by moe_pack_weights; y_perm [A, d] fp32.
 * Rows of masked-out or empty experts are left unwritten.  The hidden activation is
 * rounded to dtype once between the two products.
 */
moe_status moe_expert_ffn(const moe_shape* shape, const void* x_perm, const void* w1,
                          const void* w2, const int32_t* offsets, const uint8_t* mask,
                          float* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_expert_ffn with expert biases, as the linear layers of some released MoE checkpoints carry them (the
 * paper's experts are the two weight matrices, Section 2.1; this is the optional variant):
 *   y_perm[rows of e] = act(x_perm[rows] . W1_e^T + b1_e) . W2_e^T + b2_e
 * b1 [E, d_ff] and b2 [E, d_model]: fp32, device, row e = expert e; either may be NULL (no bias).  Everything
 * else as moe_expert_ffn, which is this call with both NULL.
 */
moe_status moe_expert_ffn_biased(const moe_shape* shape, const void* x_perm, const void* w1, const float* b1,
                                 const void* w2, const float* b2, const int32_t* offsets, const uint8_t* mask,
                                 float* y_perm, void* ws, size_t ws_bytes, void* stream);

/*
 * Combine (Section 2.1: outputs are combined and re-organised into the original token order):
 *   out[t] = sum over j < k with mask[topk_idx[t,j]] != 0 of topk_w[t,j] * y_perm[inv_perm[t*k+j]]
 * accumulated in fp32, rounded once to dtype.  Masked-out rows of y_perm are not read.
 * out [T, d] (dtype).
 */
moe_status moe_combine(const moe_shape* shape, const float* y_perm, const int32_t* inv_perm,
                       const int32_t* topk_idx, const float* topk_w, const uint8_t* mask,
                       void* out, void* stream);

/*
 * For tools that attribute time or bytes to the two kernels of the expert FFN (the paper's compute-bound and
 * memory-bound experts, Section 3.1): the smallest number of rows with which an expert's rows are run by the
 * LDS-tiled kernel rather than the weight-streaming one in a call where the experts have `rows_host[e]` rows
 * (HOST array [E]; 0 for experts that are empty or masked out).  It is 128, or one more than a streaming tile
 * holds when the experts of 128 rows and more already fill the tiled kernel for a round; 0 when the shape
 * never uses the tiled kernel (fp32, or fewer than 128 tokens) or on invalid arguments.  The current device's
 * size enters (as in the calls themselves).
 */
int32_t moe_tiled_kernel_min_rows(const moe_shape* shape, const int32_t* rows_host);

/*
 * Profiling aid for callers that time the kernels of the expert FFN separately (the paper reasons
 * about an expert's cost product by product, Section 2.2 and Eq. 3-4).  `events` is a HOST array of
 * five hipEvent_t created by the caller (entries may be NULL), or NULL to stop.  Until the next call,
 * every expert-FFN launch (from moe_expert_ffn or moe_layer_forward) records, on the launch's stream:
 *   [0] before the first product (x.W1^T, ReLU) of the large experts' tiled kernel (if launched),
 *   [1] after it, [2] after the first product of the small experts' weight-streaming kernel,
 *   [3] after the second product (h.W2^T) of the tiled kernel, [4] after that of the streaming kernel.
 * The handles are copied; the array need not outlive the call.  Process-global (all devices, all threads) and
 * not thread-safe: set it only while no other thread is inside an expert-FFN call.
 */
void moe_set_profile_events(void* const* events);

/*
 * The whole layer on one stream with no host synchronisation: route -> permute ->
 * expert FFN -> combine.  mask != NULL: only those experts run and are summed (the
 * hot share or the cold share of Section 3.3).  mask == NULL and H >= 0: the hot mask
 * is computed on the device from the token counts (top-H) and used.  mask == NULL and
 * H < 0: the whole layer.  Gate weights never depend on the mask.
 * Optional outputs (each may be NULL): topk_idx [T,k], topk_w [T,k], counts [E],
 * perm [A], hot_mask_out [E] (the mask that was used; all ones for the whole layer).
 */
moe_status moe_layer_forward(const moe_shape* shape, const void* x, const void* w_gate,
                             const float* gate_bias, const void* w1, const void* w2,
                             const uint8_t* mask, int32_t H, void* out,
                             int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* perm,
                             uint8_t* hot_mask_out, void* ws, size_t ws_bytes, void* stream);

/* moe_layer_forward with expert biases (see moe_expert_ffn_biased); moe_layer_forward is this call with b1 = b2 = NULL. */
moe_status moe_layer_forward_biased(const moe_shape* shape, const void* x, const void* w_gate,
                                    const float* gate_bias, const void* w1, const float* b1, const void* w2,
                                    const float* b2, const uint8_t* mask, int32_t H, void* out, int32_t* topk_idx,
                                    float* topk_w, int32_t* counts, int32_t* perm, uint8_t* hot_mask_out, void* ws,
                                    size_t ws_bytes, void* stream);

/*
 * moe_layer_forward for callers that must not allocate device memory and have no workspace to pass: code
 * running under HIP graph capture, tight serving loops (a decoder step per call), harnesses that forbid
 * hipMalloc.  The layer's workspace is a static device array inside the library, MOE_NOALLOC_MAX_WORKSPACE
 * bytes on every GPU the library runs on, held until the process ends; the call makes no hipMalloc / hipFree
 * and calls no allocating routine.  Shapes whose moe_workspace_bytes() exceeds that size are refused with
 * MOE_ERR_WORKSPACE before anything is launched (decoder steps of the paper's models, up to 127 tokens of an
 * NLLB-MoE-shaped layer, need 4 to 7 MiB; layers of 128 tokens or more ask for 64 MiB of partial-tile space
 * and do not fit).  Arguments as moe_layer_forward, without the optional outputs;
 * the result is bit-identical to moe_layer_forward on the same inputs.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different
 * streams or threads) race and give undefined results; calls on one stream, or ordered by events, are fine.
 * Nothing from an earlier call is reused: the layer clears the counters it needs in its own kernels.
 */
#define MOE_NOALLOC_MAX_WORKSPACE (16u << 20)
size_t moe_noalloc_max_workspace(void);     /* = MOE_NOALLOC_MAX_WORKSPACE */
moe_status moe_layer_forward_noalloc(const moe_shape* shape, const void* x, const void* w_gate,
                                     const float* gate_bias, const void* w1, const void* w2,
                                     const uint8_t* mask, int32_t H, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_FFN_MI355X_H */
