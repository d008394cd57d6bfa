"""CPU oracle for the MoE FFN layer forward -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

A plain, slow, fp64 numpy implementation of what the layer computes, written
from the paper's description of an MoE FFN layer (Section 2.1 and Fig. 1: a
gating network scores every (token, expert) pair, each token goes to its
top-k experts, each expert is linear -> activation -> linear, and the expert
outputs are combined and put back in the original token order) and of the
hot/cold expert split (Section 3.3: the H experts with the highest load form
the hot set; "activated" experts are those with at least one token).

Only tests, the smoke check and the bench's CPU-baseline leg may import this
module.  It shares no code with the HIP path and imports nothing from it.

Because the sparse layer equals its dense definition exactly (up to rounding
order), the oracle is that definition written out; `layer_bruteforce` is the
"every expert on every token, select afterwards" form used to cross-check it.

Parity status: no numeric layer output is printed anywhere in the paper, so
absolute values are pinned through brute force, closed-form special cases,
a hand-derived worked example, invariants and metamorphic relations (see
tests).  The gate-weighting rule (probability of the chosen expert, optionally
renormalised over the chosen k) is a reading of "outputs are combined"
(Section 2.1), which the paper leaves open: in that sense `gate_weights` is
"parity unpinned" with respect to the paper's text.  `activation_movement`
(Eq. 2) is a one-line formula for which the paper prints no value: its test
can only restate it and check its ratio to Eq. 1 (whose Table 2 sizes are
pinned), so it is "parity unpinned" as well.  `tune_alpha` is a reading of
the paragraph after Eq. 6 (the paper does not say how the best candidate
becomes a new alpha): "parity unpinned" with respect to the paper, its
arithmetic pinned by hand-worked examples.

Conventions: T tokens, d = d_model, f = d_ff, E experts, k experts per token,
A = T*k assignments, flat assignment id a = t*k + j (slot j = 0 is the best
expert).  Weight matrices are [out_features, in_features].
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def gate_logits(x, w_gate, b_gate=None):
    """L[t,e] = sum_i x[t,i] * w_gate[e,i] (+ b[e]).  Section 2.1: the gating
    function scores each token against every expert."""
    L = np.asarray(x, F64) @ np.asarray(w_gate, F64).T
    if b_gate is not None:
        L = L + np.asarray(b_gate, F64)[None, :]
    return L


def softmax_rows(L):
    """Probability distribution over the experts for each token (Section 2.1)."""
    L = np.asarray(L, F64)
    z = np.exp(L - L.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


def topk_experts(L, k):
    """idx[t, j] = expert with the (j+1)-th largest logit of token t; equal
    logits are ordered by lowest expert index.  Selection is made on logits
    (softmax is monotone, so the order is the same as on probabilities)."""
    L = np.array(L, F64, copy=True)
    T, E = L.shape
    assert 1 <= k <= E
    idx = np.empty((T, k), np.int32)
    rows = np.arange(T)
    for j in range(k):
        best = np.argmax(L, axis=1)          # first maximum = lowest index
        idx[:, j] = best
        L[rows, best] = -np.inf
    return idx


def topk_margin(L, k):
    """Smallest gap between consecutive entries of the k+1 largest logits of each
    token (k largest if k == E).  A token whose margin is tiny can legitimately be
    routed differently by a lower-precision implementation."""
    L = np.asarray(L, F64)
    E = L.shape[1]
    n = min(k + 1, E)
    top = -np.sort(-L, axis=1)[:, :n]
    if n == 1:
        return np.full(L.shape[0], np.inf)
    return np.min(top[:, :-1] - top[:, 1:], axis=1)


def gate_weights(p, idx, renormalize):
    """g[t,j] = p[t, idx[t,j]], divided by the sum over the chosen k when
    `renormalize` (top-2 NLLB-style); raw probability otherwise (Switch-style
    top-1: the output is scaled by the router probability)."""
    p = np.asarray(p, F64)
    g = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renormalize:
        g = g / g.sum(axis=1, keepdims=True)
    return g


def expert_histogram(idx, E):
    """counts[e] = number of assignments routed to e; offsets = exclusive prefix
    sum with offsets[E] = A.  Drop-less, padding-less routing (Section 4.1):
    every assignment is kept, nothing is padded."""
    counts = np.zeros(E, np.int32)
    for e in np.asarray(idx).reshape(-1):
        counts[e] += 1
    offsets = np.zeros(E + 1, np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    return counts, offsets


def activated_experts(counts):
    """Number of experts with at least one token (Section 3.3, Expert_Activ)."""
    return int(np.count_nonzero(np.asarray(counts) > 0))


def stable_permutation(idx, E):
    """perm[p] = flat assignment id sitting at sorted position p when assignments
    are grouped by expert (experts ascending; inside an expert, ascending flat id);
    inv_perm[a] = position of assignment a."""
    flat = np.asarray(idx).reshape(-1)
    A = flat.shape[0]
    perm = np.empty(A, np.int32)
    pos = 0
    for e in range(E):
        for a in range(A):
            if flat[a] == e:
                perm[pos] = a
                pos += 1
    assert pos == A
    inv = np.empty(A, np.int32)
    for p in range(A):
        inv[perm[p]] = p
    return perm, inv


def stable_permutation_fast(idx, E):
    """Same result as `stable_permutation` through numpy's stable sort; used where
    A is too large for the double loop (checked against it in the tests)."""
    flat = np.asarray(idx).reshape(-1)
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(flat.shape[0], dtype=np.int32)
    return perm, inv


def hot_mask_top_h(counts, H):
    """mask[e] = 1 for the H experts with the largest token counts (Section 3.3:
    the top-H most loaded experts are the hot set); equal counts are ordered by
    lowest expert index.  H is clipped to [0, E]."""
    counts = np.asarray(counts)
    E = counts.shape[0]
    H = max(0, min(int(H), E))
    c = counts.astype(np.int64).copy()
    mask = np.zeros(E, np.uint8)
    for _ in range(H):
        e = int(np.argmax(c))
        mask[e] = 1
        c[e] = -1
    return mask


def hot_expert_count(counts, alpha, bw_a, bw_b):
    """H of the load-balancing rule (Section 3.3, Eq. 3-6): the two workflows are bound by the
    bandwidth that feeds them, t_a = Expert_a / BW_a and t_b = Expert_b / BW_b with
    Expert_a + Expert_b = Expert_Activ (the experts with at least one token); equal runtimes give
    Expert_a = BW_a / (BW_a + BW_b) * Expert_Activ, and H = alpha * Expert_a with the tuning
    factor alpha.  The paper does not say how the real number becomes a count: it is rounded to the
    nearest integer, halves up, and clipped to [0, E]."""
    E = int(np.asarray(counts).shape[0])
    activ = activated_experts(counts)
    h = float(alpha) * float(bw_a) / (float(bw_a) + float(bw_b)) * float(activ)
    return max(0, min(int(np.floor(h + 0.5)), E))


def tune_alpha(alpha, bw_a, bw_b, activated, times):
    """Auto-tuning of the scaling factor alpha (Section 3.3, the paragraph after Eq. 6: profiled inference on a
    small set of past input batches finds the local optimum among the candidates H, H + 1, H + 2).

    activated[b]: number of activated experts of past batch b; times[b][c]: measured time of the layer on batch
    b with H_b + c hot experts, c = 0 ... C-1, where H_b is Eq. 6 at the current alpha.  The offset c* with the
    smallest total time over the batches is taken (the smallest such offset when totals are equal).  The paper
    does not say how the chosen candidate turns into a new alpha; the reading here: the alpha at which Eq. 6's
    real-valued H, for a batch with the mean number of activated experts, is c* larger than at the current one:
        alpha_new = alpha + c* / (rho * mean(activated)),   rho = BW_a / (BW_a + BW_b),
    and alpha stays as it is when c* = 0 or no batch activated any expert.  Returns (alpha_new, c*)."""
    times = np.asarray(times, F64)
    activated = np.asarray(activated)
    B, C = times.shape
    assert activated.shape == (B,) and B >= 1 and C >= 1
    totals = np.zeros(C, F64)
    for b in range(B):              # summed in batch order
        for c in range(C):
            totals[c] = totals[c] + times[b, c]
    best = 0
    for c in range(1, C):
        if totals[c] < totals[best]:
            best = c
    total_activ = 0
    for b in range(B):
        total_activ += int(activated[b])
    if best == 0 or total_activ == 0:
        return float(alpha), best
    rho = float(bw_a) / (float(bw_a) + float(bw_b))
    mean = float(total_activ) / float(B)
    return float(alpha) + float(best) / (rho * mean), best


def plan_devices(counts, n_devices, skip=None):
    """Load balancing over several expert-holding devices (Section 3.3, last paragraph): the experts
    that have tokens (and are not in `skip`, e.g. the hot set kept on the main device), sorted by
    compute intensity -- the token count, all experts having the same shape -- are dealt out
    round-robin.  Equal counts keep their index order.  Returns device_of[E], -1 for experts that take
    no part."""
    counts = np.asarray(counts)
    device_of = np.full(counts.shape[0], -1, dtype=np.int64)
    taking_part = [e for e in range(counts.shape[0]) if counts[e] > 0 and (skip is None or not skip[e])]
    by_load = sorted(taking_part, key=lambda e: (-int(counts[e]), e))
    for position, e in enumerate(by_load):
        device_of[e] = position % n_devices
    return device_of


def parameter_movement(E, d_model, d_ff):
    """Number of expert parameters of one MoE layer, i.e. what moving every expert to the compute
    device moves (Section 3.2, Eq. 1): two matrices of d_model x d_ff per expert."""
    return 2 * int(E) * int(d_model) * int(d_ff)


def activation_movement(tokens, d_model):
    """Number of activation values that cross the link when the tokens go to the experts instead
    (Section 3.2, Eq. 2): every token's d_model values out and back; tokens = B * S."""
    return 2 * int(tokens) * int(d_model)


def round_bf16(a):
    """Round fp64 values to the nearest bfloat16 (8 significant bits, ties to even),
    returned as fp64.  Written from the format's definition (sign, 8 exponent bits,
    7 stored mantissa bits); overflow and subnormals are not handled because the
    oracle only applies it to hidden activations of moderate size."""
    a = np.asarray(a, F64)
    m, e = np.frexp(a)                 # a = m * 2**e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0     # keep 8 significant bits; rint = ties to even
    return np.ldexp(q, e)


def gelu(z):
    """GeLU in its defining form z * Phi(z), Phi the standard normal distribution function:
    0.5 * z * (1 + erf(z / sqrt(2))).  Section 3.4 names "ReLU or GeLU" as the trailing
    activation without saying which GeLU; the definition is taken, not the tanh approximation."""
    from scipy.special import erf
    z = np.asarray(z, F64)
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def expert_ffn(X_e, W1_e, W2_e, h_dtype=None, activation="relu", b1_e=None, b2_e=None):
    """Y = act(X W1^T + b1) W2^T + b2 for one expert (Section 2.1: two linear layers with an
    activation in between; Section 3.4: a gemm with a trailing ReLU or GeLU, then a gemm).
    W1_e [f, d], W2_e [d, f]; activation = "relu" (default) or "gelu".  The paper's experts are the
    two weight matrices; b1_e [f] and b2_e [d] (default: none) are the biases that linear layers of
    released checkpoints of the NLLB family carry, added the way a linear layer adds them.

    h_dtype = None keeps the hidden activation in fp64 (the exact definition).
    h_dtype = "bf16" rounds it once to bfloat16 before the second product, which is
    what a bfloat16 inference run (Section 4.1) stores between the two linear layers;
    all sums stay in fp64."""
    h = np.asarray(X_e, F64) @ np.asarray(W1_e, F64).T
    if b1_e is not None:
        h = h + np.asarray(b1_e, F64)[None, :]
    if activation == "relu":
        h = np.maximum(h, 0.0)
    elif activation == "gelu":
        h = gelu(h)
    else:
        raise ValueError(activation)
    if h_dtype == "bf16":
        h = round_bf16(h)
    elif h_dtype not in (None, "f32", "f64"):
        raise ValueError(h_dtype)
    y = h @ np.asarray(W2_e, F64).T
    if b2_e is not None:
        y = y + np.asarray(b2_e, F64)[None, :]
    return y


def permute_tokens(x, perm, k):
    """x_perm[p] = x[perm[p] // k]: token rows in expert-contiguous order."""
    return np.asarray(x)[np.asarray(perm) // k]


def combine(y_perm, inv_perm, idx, g, mask=None):
    """out[t] = sum_j [mask[idx[t,j]]] * g[t,j] * y_perm[inv_perm[t*k+j]]
    (Section 2.1: outputs are combined and restored to the original token order).
    Rows of y_perm that belong to masked-out experts are never read."""
    T, k = idx.shape
    d = y_perm.shape[1]
    out = np.zeros((T, d), F64)
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            if mask is not None and not mask[e]:
                continue
            out[t] += g[t, j] * np.asarray(y_perm[inv_perm[t * k + j]], F64)
    return out


def route(x, w_gate, b_gate, k, renormalize):
    """Steps 1-2 of the layer: logits, softmax, top-k, gate weights, histogram."""
    L = gate_logits(x, w_gate, b_gate)
    p = softmax_rows(L)
    idx = topk_experts(L, k)
    g = gate_weights(p, idx, renormalize)
    counts, offsets = expert_histogram(idx, w_gate.shape[0])
    return dict(logits=L, probs=p, idx=idx, g=g, counts=counts, offsets=offsets,
                margin=topk_margin(L, k))


def layer_forward(x, w_gate, b_gate, expert, k, renormalize, mask=None,
                  return_intermediates=False, h_dtype=None, activation="relu"):
    """Whole MoE FFN layer.  `expert(e)` returns (W1_e, W2_e) or, for experts with biases,
    (W1_e, W2_e, b1_e, b2_e); it is called only for experts that received tokens and are not
    masked out.  With a mask, only the
    masked-in experts' share of the output is produced (Section 3.3: hot experts
    on one device, the rest elsewhere; gates are fixed before the split)."""
    x = np.asarray(x, F64)
    E = w_gate.shape[0]
    r = route(x, w_gate, b_gate, k, renormalize)
    idx, g, offsets = r["idx"], r["g"], r["offsets"]
    perm, inv = stable_permutation_fast(idx, E)
    x_perm = permute_tokens(x, perm, k)
    y_perm = np.zeros((perm.shape[0], x.shape[1]), F64)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo or (mask is not None and not mask[e]):
            continue
        we = expert(e)
        y_perm[lo:hi] = expert_ffn(x_perm[lo:hi], we[0], we[1], h_dtype, activation, *we[2:4])
    out = combine(y_perm, inv, idx, g, mask)
    if return_intermediates:
        r.update(perm=perm, inv_perm=inv, x_perm=x_perm, y_perm=y_perm, out=out)
        return r
    return out


def layer_bruteforce(x, w_gate, b_gate, W1, W2, k, renormalize, mask=None, activation="relu",
                     b1=None, b2=None):
    """Dense definition: run every expert on every token, then keep each token's
    top-k experts, weight and sum.  Tiny inputs only."""
    x = np.asarray(x, F64)
    T, d = x.shape
    E = w_gate.shape[0]
    Yall = np.empty((T, E, d), F64)
    for e in range(E):
        Yall[:, e, :] = expert_ffn(x, W1[e], W2[e], activation=activation,
                                   b1_e=None if b1 is None else b1[e], b2_e=None if b2 is None else b2[e])
    L = gate_logits(x, w_gate, b_gate)
    p = softmax_rows(L)
    idx = topk_experts(L, k)
    g = gate_weights(p, idx, renormalize)
    out = np.zeros((T, d), F64)
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            if mask is None or mask[e]:
                out[t] += g[t, j] * Yall[t, e]
    return out


def rel_error(got, ref):
    """Element-wise |got-ref| / max(|ref|, rms(ref)); the value-parity statistic."""
    ref = np.asarray(ref, F64)
    got = np.asarray(got, F64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return np.abs(got - ref) / den


def rel_error_rows(got, ref):
    """Element-wise |got-ref| / max(|ref|, rms of the element's own row of ref), for 2-D arrays
    [rows, d].  Token rows of an MoE layer differ in scale (the gate weight multiplies the whole
    row), so the floor that keeps the relative error meaningful near zero is taken per row; a row
    of zeros (a token none of whose experts ran) gets the floor 1, i.e. its absolute error."""
    ref = np.asarray(ref, F64)
    got = np.asarray(got, F64)
    out = np.empty(ref.shape, F64)
    for i in range(ref.shape[0]):
        rms = float(np.sqrt(np.mean(ref[i] * ref[i]))) if ref.shape[1] else 0.0
        floor = rms if rms > 0 else 1.0
        out[i] = np.abs(got[i] - ref[i]) / np.maximum(np.abs(ref[i]), floor)
    return out


def row_error_norms(got, ref):
    """Per row ||got-ref||_2 / ||ref||_2 (the relative error of the row as a vector); a row of
    zeros in ref reports ||got||_2, its absolute error."""
    ref = np.asarray(ref, F64)
    got = np.asarray(got, F64)
    out = np.empty(ref.shape[0], F64)
    for i in range(ref.shape[0]):
        num = float(np.sqrt(np.sum((got[i] - ref[i]) ** 2)))
        den = float(np.sqrt(np.sum(ref[i] ** 2)))
        out[i] = num / den if den > 0 else num
    return out
