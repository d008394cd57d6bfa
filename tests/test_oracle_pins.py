"""Pins for the CPU oracle: what the paper's definition and plain mathematics fix.

None of these compares the oracle with itself through the same code path: they use
brute force over all experts, a hand-derived rational example, closed-form special
cases that reduce to a plain matmul, invariants and metamorphic relations.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny(T=5, d=6, f=10, E=3, k=2, seed=7, bias=False):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    wg = rng.standard_normal((E, d))
    b = rng.standard_normal(E) if bias else None
    W1 = rng.standard_normal((E, f, d)) / np.sqrt(d)
    W2 = rng.standard_normal((E, d, f)) / np.sqrt(f)
    return x, wg, b, W1, W2


def run(x, wg, b, W1, W2, k, renorm, mask=None, **kw):
    return orc.layer_forward(x, wg, b, lambda e: (W1[e], W2[e]), k, renorm, mask, **kw)


# ---------------------------------------------------------------- worked example
def _frac(a):
    return np.array([[float(Fraction(n, d)) for n, d in row] for row in a])


def test_worked_example_fig1_shape():
    g = json.load(open(os.path.join(GOLD, "worked_example.json")))
    x = np.array(g["x"], float)
    wg = np.log(np.array(g["w_gate_log_of"], float))
    W1 = np.array(g["W1"], float)
    W2 = np.array(g["W2"], float)
    r = run(x, wg, None, W1, W2, 2, True, return_intermediates=True)
    assert np.allclose(r["probs"], _frac(g["probs_num_den"]), atol=1e-15)
    assert r["idx"].tolist() == g["topk_idx"]
    assert np.allclose(r["g"], _frac(g["gates_renorm_num_den"]), atol=1e-15)
    assert r["counts"].tolist() == g["counts"]
    assert r["offsets"].tolist() == g["offsets"]
    assert r["perm"].tolist() == g["perm"]
    assert r["inv_perm"].tolist() == g["inv_perm"]
    assert np.allclose(r["out"], _frac(g["out_top2_renorm_num_den"]), atol=1e-14)
    assert np.allclose(run(x, wg, None, W1, W2, 2, False),
                       _frac(g["out_top2_raw_num_den"]), atol=1e-14)
    assert np.allclose(run(x, wg, None, W1, W2, 1, False),
                       _frac(g["out_top1_raw_num_den"]), atol=1e-14)
    mask = orc.hot_mask_top_h(r["counts"], 1)
    assert mask.tolist() == g["hot_mask_H1"]
    assert np.allclose(run(x, wg, None, W1, W2, 2, True, mask),
                       _frac(g["out_top2_renorm_hot_only_num_den"]), atol=1e-14)
    m = np.log([a / b for a, b in g["margin_log_of_ratio"]])
    assert np.allclose(r["margin"], m, atol=1e-14)
    # the permutation and the slow definition agree on this case too
    p2, i2 = orc.stable_permutation(r["idx"], 3)
    assert p2.tolist() == g["perm"] and i2.tolist() == g["inv_perm"]
    assert orc.activated_experts(r["counts"]) == 3


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("T,d,f,E,k,renorm,bias", [
    (5, 6, 10, 3, 2, True, False),      # Fig. 1's shape
    (5, 6, 10, 3, 2, False, True),
    (9, 4, 7, 5, 1, False, False),
    (9, 4, 7, 5, 3, True, True),
    (1, 3, 2, 2, 2, True, False),
])
def test_sparse_equals_dense_bruteforce(T, d, f, E, k, renorm, bias):
    x, wg, b, W1, W2 = tiny(T, d, f, E, k, seed=T * 31 + E, bias=bias)
    a = run(x, wg, b, W1, W2, k, renorm)
    bf = orc.layer_bruteforce(x, wg, b, W1, W2, k, renorm)
    assert np.allclose(a, bf, rtol=0, atol=1e-12)
    mask = (np.arange(E) % 2).astype(np.uint8)
    assert np.allclose(run(x, wg, b, W1, W2, k, renorm, mask),
                       orc.layer_bruteforce(x, wg, b, W1, W2, k, renorm, mask), atol=1e-12)


def test_bruteforce_on_tiny_preset():
    cfg = wl.CONFIGS["tiny_f32"]
    L = wl.make_layer(cfg)
    W1, W2 = L.all_experts()
    a = orc.layer_forward(L.x, L.w_gate, L.b_gate, L.expert, cfg.k, cfg.renormalize)
    bf = orc.layer_bruteforce(L.x, L.w_gate, L.b_gate, W1, W2, cfg.k, cfg.renormalize)
    assert np.allclose(a, bf, atol=1e-12)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("name", ["tiny_f32", "switch_base", "nllb_decode"])
def test_routing_invariants(name):
    cfg = wl.CONFIGS[name]
    x = wl.make_activations(cfg)
    wg, b = wl.make_gate(cfg)
    r = orc.route(x, wg, b, cfg.k, cfg.renormalize)
    idx, g, counts, offsets = r["idx"], r["g"], r["counts"], r["offsets"]
    A = cfg.T * cfg.k
    assert counts.sum() == A and offsets[0] == 0 and offsets[-1] == A
    assert np.all(np.diff(offsets) == counts)
    assert np.array_equal(counts, np.bincount(idx.reshape(-1), minlength=cfg.E))
    perm, inv = orc.stable_permutation_fast(idx, cfg.E)
    assert np.array_equal(np.sort(perm), np.arange(A))           # bijection
    assert np.array_equal(perm[inv], np.arange(A))
    keys = idx.reshape(-1)[perm]
    assert np.all(np.diff(keys) >= 0)                            # expert-contiguous
    same = np.diff(keys) == 0
    assert np.all(np.diff(perm)[same] > 0)                       # stable inside an expert
    # gates are the softmax probabilities of the chosen experts
    p = r["probs"]
    assert np.allclose(p.sum(1), 1, atol=1e-12)
    chosen = np.take_along_axis(p, idx.astype(np.int64), 1)
    if cfg.renormalize:
        assert np.allclose(g.sum(1), 1, atol=1e-12)
        assert np.allclose(g * chosen.sum(1, keepdims=True), chosen, atol=1e-15)
    else:
        assert np.array_equal(g, chosen)
    assert np.all(g > 0) and np.all(g <= 1)
    # slot order: descending logits; each token's experts are distinct
    Lc = np.take_along_axis(r["logits"], idx.astype(np.int64), 1)
    assert np.all(np.diff(Lc, axis=1) <= 0)
    if cfg.k == 2:
        assert np.all(idx[:, 0] != idx[:, 1])
    # the chosen set is a top-k set: nothing outside beats the worst chosen logit
    rest = r["logits"].copy()
    np.put_along_axis(rest, idx.astype(np.int64), -np.inf, 1)
    assert np.all(rest.max(1) <= Lc[:, -1])


def test_small_permutation_matches_definition():
    rng = np.random.default_rng(3)
    idx = rng.integers(0, 7, size=(40, 2)).astype(np.int32)
    a = orc.stable_permutation(idx, 7)
    b = orc.stable_permutation_fast(idx, 7)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_topk_ties_go_to_lowest_index():
    L = np.array([[1.0, 3.0, 3.0, 3.0, 0.0], [2.0, 2.0, 2.0, 2.0, 2.0]])
    assert orc.topk_experts(L, 2).tolist() == [[1, 2], [0, 1]]
    assert orc.topk_experts(L, 1).tolist() == [[1], [0]]
    assert orc.topk_margin(L, 2).tolist() == [0.0, 0.0]
    assert orc.topk_margin(np.array([[5.0, 1.0, 3.0]]), 1).tolist() == [2.0]
    assert orc.topk_margin(np.array([[5.0, 1.0, 3.0]]), 2).tolist() == [2.0]


def test_hot_mask_top_h():
    c = np.array([3, 9, 0, 9, 1, 3], np.int32)
    assert orc.hot_mask_top_h(c, 0).tolist() == [0, 0, 0, 0, 0, 0]
    assert orc.hot_mask_top_h(c, 1).tolist() == [0, 1, 0, 0, 0, 0]
    assert orc.hot_mask_top_h(c, 3).tolist() == [1, 1, 0, 1, 0, 0]
    assert orc.hot_mask_top_h(c, 6).tolist() == [1] * 6
    assert orc.hot_mask_top_h(c, 99).tolist() == [1] * 6
    assert orc.activated_experts(c) == 5


# ---------------------------------------------------------------- special cases
def test_data_movement_model_eq1_eq2():
    # Table 2 prints the total expert size of the two models: 51.5 GB for Switch-Large-128 (24 MoE layers,
    # d_model 1024, 128 experts) and 103.1 GB for NLLB-MoE (12 MoE layers, d_model 2048, 128 experts), in
    # bf16; per layer that is Eq. 1 with d_ff = 4 d_model.
    assert abs(24 * orc.parameter_movement(128, 1024, 4096) * 2 / 1e9 - 51.5) < 0.1
    assert abs(12 * orc.parameter_movement(128, 2048, 8192) * 2 / 1e9 - 103.1) < 0.1
    # Eq. 2 against its reading: B sequences of S tokens, d_model values each way
    assert orc.activation_movement(4 * 512, 1024) == 2 * 4 * 512 * 1024
    # the paper's point (Section 3.2): for inference-sized batches the activations are orders of magnitude
    # smaller than the parameters, and the ratio is E * d_ff / tokens
    for E, d, f, tok in [(128, 1024, 4096, 512), (128, 2048, 8192, 1), (64, 768, 3072, 2048)]:
        ratio = orc.parameter_movement(E, d, f) / orc.activation_movement(tok, d)
        assert abs(ratio - E * f / tok) < 1e-9
    assert orc.parameter_movement(128, 2048, 8192) / orc.activation_movement(512, 2048) == 2048.0


def test_hot_expert_count_eq6():
    # values worked out by hand from Eq. 6 (tests/golden/hot_count_examples.json)
    with open(os.path.join(GOLD, "hot_count_examples.json")) as fh:
        cases = json.load(fh)["cases"]
    for c in cases:
        assert orc.activated_experts(c["counts"]) == c["activ"]
        assert orc.hot_expert_count(c["counts"], c["alpha"], c["bw_a"], c["bw_b"]) == c["H"]
    # the rule's purpose (Eq. 3-5): with alpha = 1 the two bandwidth-bound runtimes H / BW_a and
    # (Expert_Activ - H) / BW_b are equal up to the rounding of H, i.e. H is within 1/2 of the real solution
    rng = np.random.default_rng(11)
    for _ in range(200):
        E = int(rng.integers(1, 200))
        counts = rng.integers(0, 4, E)
        a, b = float(rng.uniform(1, 100)), float(rng.uniform(1, 1000))
        H = orc.hot_expert_count(counts, 1.0, a, b)
        activ = int((counts > 0).sum())
        assert abs(H * (a + b) - a * activ) <= 0.5 * (a + b) * (1 + 1e-12)
        assert 0 <= H <= activ
    # alpha scales the real-valued solution before rounding
    assert orc.hot_expert_count([1] * 90, 2.0, 1.0, 8.0) == 20


def test_single_expert_is_a_plain_ffn():
    x, wg, b, W1, W2 = tiny(T=7, E=1, k=1, bias=True)
    ref = torch.relu(torch.from_numpy(x) @ torch.from_numpy(W1[0]).T) @ torch.from_numpy(W2[0]).T
    assert np.allclose(run(x, wg, b, W1, W2, 1, False), ref.numpy(), atol=1e-12)
    assert np.allclose(run(x, wg, b, W1, W2, 1, True), ref.numpy(), atol=1e-12)


def test_k_equals_E_is_the_dense_mixture():
    x, wg, b, W1, W2 = tiny(T=6, E=4, k=4, bias=True)
    xt = torch.from_numpy(x)
    p = torch.softmax(xt @ torch.from_numpy(wg).T + torch.from_numpy(b), dim=1)
    ys = torch.stack([torch.relu(xt @ torch.from_numpy(W1[e]).T) @ torch.from_numpy(W2[e]).T
                      for e in range(4)], 1)                       # [T,E,d]
    ref = (p[:, :, None] * ys).sum(1).numpy()
    assert np.allclose(run(x, wg, b, W1, W2, 4, True), ref, atol=1e-12)
    assert np.allclose(run(x, wg, b, W1, W2, 4, False), ref, atol=1e-12)


def test_identical_experts_and_zero_w2():
    x, wg, b, W1, W2 = tiny(T=8, E=5, k=2)
    W1s = np.repeat(W1[:1], 5, 0)
    W2s = np.repeat(W2[:1], 5, 0)
    ffn = np.maximum(x @ W1[0].T, 0) @ W2[0].T
    assert np.allclose(run(x, wg, b, W1s, W2s, 2, True), ffn, atol=1e-12)
    r = orc.route(x, wg, b, 2, False)
    assert np.allclose(run(x, wg, b, W1s, W2s, 2, False), r["g"].sum(1, keepdims=True) * ffn,
                       atol=1e-12)
    assert np.all(run(x, wg, b, W1, np.zeros_like(W2), 2, True) == 0)


def test_relu_is_applied_between_the_layers():
    # one expert, W1 = -I: every hidden unit is negative for positive inputs -> output 0
    x = np.abs(np.random.default_rng(0).standard_normal((4, 3))) + 0.1
    W1 = -np.eye(3)[None]
    W2 = np.ones((1, 3, 3))
    assert np.all(run(x, np.zeros((1, 3)), None, W1, W2, 1, False) == 0)
    assert np.allclose(run(-x, np.zeros((1, 3)), None, W1, W2, 1, False),
                       np.repeat(x.sum(1, keepdims=True), 3, 1))


# ---------------------------------------------------------------- metamorphic
def test_gelu_variant():
    # the activation itself against a library routine that shares nothing with the oracle ...
    z = np.linspace(-8, 8, 4001)
    ref = torch.nn.functional.gelu(torch.from_numpy(z), approximate="none").numpy()
    assert np.allclose(orc.gelu(z), ref, rtol=1e-13, atol=1e-15)
    # ... and against what the definition z * Phi(z) fixes: gelu(z) - gelu(-z) = z, gelu(0) = 0, the value at 1
    # from Phi(1) = 0.8413447460685429 (standard normal table), identity for large z, zero for very negative z
    assert np.allclose(orc.gelu(z) - orc.gelu(-z), z, atol=1e-14)
    assert orc.gelu(0.0) == 0.0
    assert abs(float(orc.gelu(1.0)) - 0.8413447460685429) < 1e-15
    assert abs(float(orc.gelu(40.0)) - 40.0) < 1e-12 and abs(float(orc.gelu(-40.0))) < 1e-12
    # the tanh approximation is a different function: a plausible mix-up must not pass
    approx = torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    assert np.abs(orc.gelu(z) - approx).max() > 1e-4
    # in the layer: brute force over all experts agrees, and the expert is act(x W1^T) W2^T with torch's matmuls
    x, wg, b, W1, W2 = tiny(T=9, E=4, k=2, bias=True)
    out = run(x, wg, b, W1, W2, 2, True, activation="gelu")
    bf = orc.layer_bruteforce(x, wg, b, W1, W2, 2, True, activation="gelu")
    assert np.allclose(out, bf, rtol=1e-12, atol=1e-12)
    xt, w1t, w2t = (torch.from_numpy(a) for a in (x, W1[1], W2[1]))
    ref = (torch.nn.functional.gelu(xt @ w1t.T, approximate="none") @ w2t.T).numpy()
    assert np.allclose(orc.expert_ffn(x, W1[1], W2[1], activation="gelu"), ref, rtol=1e-12, atol=1e-12)
    assert not np.allclose(out, run(x, wg, b, W1, W2, 2, True), atol=1e-3)       # and differs from ReLU
    with pytest.raises(ValueError):
        orc.expert_ffn(x, W1[0], W2[0], activation="silu")


def test_expert_biases():
    x, wg, b, W1, W2 = tiny(T=9, E=4, k=2, bias=True)
    rng = np.random.default_rng(5)
    b1, b2 = rng.standard_normal((4, W1.shape[1])), rng.standard_normal((4, W2.shape[1]))
    # one expert against a library's linear layers
    xt = torch.from_numpy(x)
    lin = torch.nn.functional.linear
    ref = lin(torch.relu(lin(xt, torch.from_numpy(W1[2]), torch.from_numpy(b1[2]))), torch.from_numpy(W2[2]),
              torch.from_numpy(b2[2])).numpy()
    assert np.allclose(orc.expert_ffn(x, W1[2], W2[2], b1_e=b1[2], b2_e=b2[2]), ref, rtol=1e-12, atol=1e-12)
    # zero biases change nothing; the output bias is a plain shift; the hidden bias is not (ReLU in between)
    y0 = orc.expert_ffn(x, W1[2], W2[2])
    assert np.array_equal(orc.expert_ffn(x, W1[2], W2[2], b1_e=np.zeros_like(b1[2]), b2_e=np.zeros_like(b2[2])), y0)
    assert np.allclose(orc.expert_ffn(x, W1[2], W2[2], b2_e=b2[2]) - y0, b2[2][None, :], atol=1e-12)
    assert not np.allclose(orc.expert_ffn(x, W1[2], W2[2], b1_e=b1[2]) - y0, (b1[2] @ W2[2].T)[None, :], atol=1e-6)
    # in the layer: brute force over all experts, and with renormalised gates the output biases of the chosen
    # experts enter with weights that sum to one
    out = orc.layer_forward(x, wg, b, lambda e: (W1[e], W2[e], b1[e], b2[e]), 2, True)
    bf = orc.layer_bruteforce(x, wg, b, W1, W2, 2, True, b1=b1, b2=b2)
    assert np.allclose(out, bf, rtol=1e-12, atol=1e-12)
    same = np.tile(b2[:1], (4, 1))
    out_s = orc.layer_forward(x, wg, b, lambda e: (W1[e], W2[e], None, same[e]), 2, True)
    out_0 = orc.layer_forward(x, wg, b, lambda e: (W1[e], W2[e]), 2, True)
    assert np.allclose(out_s - out_0, same[:1], atol=1e-12)


def test_expert_relabelling_and_token_permutation():
    x, wg, b, W1, W2 = tiny(T=11, E=6, k=2, bias=True, seed=5)
    base = run(x, wg, b, W1, W2, 2, True)
    q = np.random.default_rng(1).permutation(6)
    assert np.allclose(run(x, wg[q], b[q], W1[q], W2[q], 2, True), base, atol=1e-12)
    tp = np.random.default_rng(2).permutation(11)
    assert np.allclose(run(x[tp], wg, b, W1, W2, 2, True), base[tp], atol=1e-12)


def test_scaling_and_logit_shift():
    x, wg, b, W1, W2 = tiny(T=11, E=6, k=2, bias=True, seed=6)
    base = run(x, wg, b, W1, W2, 2, False)
    assert np.allclose(run(x, wg, b, W1, 3.5 * W2, 2, False), 3.5 * base, atol=1e-12)
    assert np.allclose(run(x, wg, b + 2.25, W1, W2, 2, False), base, atol=1e-12)
    # positive homogeneity of relu: scaling W1 by c > 0 scales the output by c
    assert np.allclose(run(x, wg, b, 0.5 * W1, W2, 2, False), 0.5 * base, atol=1e-12)


def test_mask_algebra():
    x, wg, b, W1, W2 = tiny(T=13, E=6, k=2, bias=True, seed=8)
    full = run(x, wg, b, W1, W2, 2, True)
    m = np.array([1, 0, 1, 1, 0, 0], np.uint8)
    hot = run(x, wg, b, W1, W2, 2, True, m)
    cold = run(x, wg, b, W1, W2, 2, True, 1 - m)
    assert np.allclose(hot + cold, full, atol=1e-12)
    assert np.all(run(x, wg, b, W1, W2, 2, True, np.zeros(6, np.uint8)) == 0)
    assert np.array_equal(run(x, wg, b, W1, W2, 2, True, np.ones(6, np.uint8)), full)


def test_transposed_operand_would_be_caught():
    # d != f and non-symmetric weights: using W1 or W2 transposed cannot even multiply,
    # and a gate indexed [d,E] instead of [E,d] gives another routing -- check the layout
    x, wg, b, W1, W2 = tiny(T=4, d=3, f=5, E=3, k=1)
    L = orc.gate_logits(x, wg, None)
    assert np.allclose(L, np.einsum("td,ed->te", x, wg), atol=1e-14)
    y = orc.expert_ffn(x, W1[0], W2[0])
    h = np.maximum(np.einsum("td,fd->tf", x, W1[0]), 0)
    assert np.allclose(y, np.einsum("tf,df->td", h, W2[0]), atol=1e-14)


# ---------------------------------------------------------------- storage rounding
def test_bf16_rounding_matches_torch_and_oracle():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(200000) * np.exp(rng.uniform(-8, 8, 200000))).astype(np.float32)
    a[:5] = [0.0, 1.0, 1.00390625, 1.01171875, -3.0]       # includes exact ties
    ref = torch.from_numpy(a).to(torch.bfloat16)
    bits = wl.f32_to_bf16_bits(a)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(bits), ref.float().numpy())
    assert np.array_equal(orc.round_bf16(a.astype(np.float64)), ref.double().numpy())
    # ties go to even
    assert orc.round_bf16(np.array([1.00390625, 1.01171875])).tolist() == [1.0, 1.015625]


def test_h_rounding_mode_is_close_to_exact():
    cfg = wl.CONFIGS["switch_base"]
    W1, W2 = wl.make_expert(cfg, 0)
    x = wl.make_activations(cfg)[:16]
    y = orc.expert_ffn(x, W1, W2)
    yb = orc.expert_ffn(x, W1, W2, "bf16")
    err = orc.rel_error(yb, y)
    assert 1e-4 < err.max() < 1e-2
    assert np.sqrt(np.mean((yb - y) ** 2)) / np.sqrt(np.mean(y ** 2)) < 3e-3


def test_plan_devices_round_robin_by_load():
    """Section 3.3, last paragraph: expert workloads sorted by compute intensity are dealt out round-robin.
    A hand-worked case, and what the rule guarantees: device sizes differ by at most one expert, the device
    loads are ordered like the device numbers, and no device carries more than the lightest one plus the
    largest single expert."""
    #            e:  0   1   2   3   4   5   6   7
    counts = np.array([5, 0, 9, 5, 1, 7, 0, 3])
    # by load: e2(9) e5(7) e0(5) e3(5) e7(3) e4(1); ties (e0, e3) by index; on 3 devices: 0 1 2 0 1 2
    assert orc.plan_devices(counts, 3).tolist() == [2, -1, 0, 0, 2, 1, -1, 1]
    # the hot set stays where it is: skip e2 and e5 -> e0 e3 e7 e4 on 2 devices: 0 1 0 1
    skip = np.array([0, 0, 1, 0, 0, 1, 0, 0])
    assert orc.plan_devices(counts, 2, skip).tolist() == [0, -1, -1, 1, 1, -1, -1, 0]
    rng = np.random.default_rng(7)
    for E, G in [(16, 2), (128, 4), (128, 5), (64, 64), (10, 16)]:
        c = (rng.zipf(1.3, size=E) % 500) * (rng.random(E) < 0.8)
        dev = orc.plan_devices(c, G)
        active = c > 0
        assert np.all(dev[~active] == -1) and np.all((dev[active] >= 0) & (dev[active] < G))
        sizes = np.array([(dev == g).sum() for g in range(G)])
        loads = np.array([c[dev == g].sum() for g in range(G)])
        assert sizes.max() - sizes.min() <= 1 and np.all(np.diff(sizes) <= 0)
        assert np.all(np.diff(loads) <= 0)                       # device 0 gets the heaviest of every round
        assert loads.max() - loads.min() <= c.max()
        # every round hands out non-increasing counts
        order = sorted(np.flatnonzero(active), key=lambda e: (-c[e], e))
        assert [dev[e] for e in order] == [i % G for i in range(len(order))]


# ---------------------------------------------------------------- the parity statistics themselves
def test_error_statistics_on_a_hand_worked_example():
    # ref = [[3, 4], [0, 0.5]], got = [[3.3, 3.8], [0.05, 0.5]]  (worked by hand)
    # global rms(ref) = sqrt((9 + 16 + 0 + 0.25) / 4) = sqrt(6.3125) = 2.5124689...
    #   rel_error: |d| = [[0.3, 0.2], [0.05, 0]], floors max(|ref|, rms) = [[3, 4], [rms, rms]]
    #            -> [[0.1, 0.05], [0.05 / 2.5124689, 0]]
    # per-row rms: row 0 sqrt(12.5) = 3.5355339, row 1 sqrt(0.125) = 0.35355339
    #   rel_error_rows: floors [[3.5355339, 4], [0.35355339, 0.5]] -> [[0.3 / 3.5355339, 0.05], [0.05 / 0.35355339, 0]]
    # row norms: row 0 sqrt(0.09 + 0.04) / 5 = 0.0721110, row 1 0.05 / 0.5 = 0.1
    ref = np.array([[3.0, 4.0], [0.0, 0.5]])
    got = np.array([[3.3, 3.8], [0.05, 0.5]])
    e = orc.rel_error(got, ref)
    assert np.allclose(e, [[0.1, 0.05], [0.05 / 2.5124689052802225, 0.0]], rtol=1e-12, atol=1e-15)
    er = orc.rel_error_rows(got, ref)
    assert np.allclose(er, [[0.3 / 3.5355339059327378, 0.05], [0.05 / 0.35355339059327379, 0.0]], rtol=1e-12, atol=1e-15)
    assert np.allclose(orc.row_error_norms(got, ref), [0.07211102550927978, 0.1], rtol=1e-12)
    # numbers, not only formulas: 0.3 / 3.5355339 = 0.0848528..., 0.05 / 0.35355339 = 0.1414213...
    assert abs(er[0, 0] - 0.0848528137) < 1e-9 and abs(er[1, 0] - 0.1414213562) < 1e-9
    assert abs(e[1, 0] - 0.0199007438) < 1e-9


def test_error_statistics_properties():
    rng = np.random.default_rng(5)
    ref = rng.standard_normal((7, 33))
    # exact agreement -> zero everywhere; a scaled copy -> the scale's relative error on large elements
    assert orc.rel_error(ref, ref).max() == 0 and orc.rel_error_rows(ref, ref).max() == 0
    assert orc.row_error_norms(ref, ref).max() == 0
    got = ref * 1.01
    assert np.allclose(orc.row_error_norms(got, ref), 0.01, rtol=1e-9)
    assert orc.rel_error_rows(got, ref).max() <= 0.01 * (1 + 1e-9)       # never above the true relative error
    big = np.abs(ref) >= np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    assert np.allclose(orc.rel_error_rows(got, ref)[big], 0.01, rtol=1e-9)
    # a larger denominator would loosen every value check: the floor is never above max(|ref|, row rms)
    tiny = np.abs(ref) < 1e-3
    if tiny.any():
        rms = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True)) * np.ones_like(ref)
        assert np.allclose(orc.rel_error_rows(ref + 1e-3, ref)[tiny], (1e-3 / rms)[tiny], rtol=1e-9)
    # rows differ in scale: the per-row statistic is invariant under scaling a row of both arrays
    s = np.array([1e-3, 1, 10, 1e3, 1, 1, 1e-6])[:, None]
    g2 = ref + 0.01 * rng.standard_normal(ref.shape)
    assert np.allclose(orc.rel_error_rows(g2 * s, ref * s), orc.rel_error_rows(g2, ref), rtol=1e-9)
    assert np.allclose(orc.row_error_norms(g2 * s, ref * s), orc.row_error_norms(g2, ref), rtol=1e-9)
    # a row of zeros in ref: absolute error
    z = np.zeros((1, 4))
    assert np.allclose(orc.rel_error_rows(z + 0.25, z), 0.25) and np.allclose(orc.row_error_norms(z + 0.25, z), 0.5)
    assert np.allclose(orc.rel_error(z + 0.25, z), 0.25)


# ---------------------------------------------------------------- alpha auto-tuning (Section 3.3, after Eq. 6)
def test_tune_alpha_hand_worked_and_properties():
    with open(os.path.join(GOLD, "alpha_tuning_examples.json")) as fh:
        cases = json.load(fh)["cases"]
    for c in cases:
        a, best = orc.tune_alpha(c["alpha"], c["bw_a"], c["bw_b"], c["activated"], c["times"])
        assert best == c["best"], c
        assert abs(a - c["alpha_new"]) <= 1e-15 * max(1.0, abs(c["alpha_new"])), c
    rng = np.random.default_rng(17)
    for _ in range(100):
        B, C = int(rng.integers(1, 6)), int(rng.integers(1, 4))
        t = rng.uniform(1.0, 2.0, (B, C))
        act = rng.integers(1, 120, B)
        alpha, a, b = float(rng.uniform(0.2, 3)), float(rng.uniform(1, 100)), float(rng.uniform(1, 1000))
        an, best = orc.tune_alpha(alpha, a, b, act, t)
        # the chosen offset has the smallest total; among equal totals the smallest offset
        tot = t.sum(axis=0)
        assert tot[best] <= tot.min() * (1 + 1e-12) and best == int(np.argmin(tot))
        # the meaning of the new alpha: Eq. 6's real-valued H of the mean batch rises by exactly the offset
        rho, mean = a / (a + b), act.mean()
        assert abs(an * rho * mean - (alpha * rho * mean + best)) <= 1e-9 * (1 + alpha * rho * mean + best)
        # neither the unit of the times nor the order of the batches matters
        p = rng.permutation(B)
        an2, best2 = orc.tune_alpha(alpha, a, b, act[p], 1000.0 * t[p])
        assert best2 == best and abs(an2 - an) <= 1e-12 * an
        # candidate 0 best -> unchanged
        t0 = t.copy()
        t0[:, 0] = 0.5
        assert orc.tune_alpha(alpha, a, b, act, t0) == (alpha, 0)
    # a larger offset moves the integer H of Eq. 6 up by about that much on a batch of the mean size
    an, best = orc.tune_alpha(1.0, 64.0, 512.0, [45, 45], [[3.0, 2.0, 1.0], [3.0, 2.0, 1.0]])
    assert best == 2
    assert orc.hot_expert_count([1] * 45, an, 64.0, 512.0) == orc.hot_expert_count([1] * 45, 1.0, 64.0, 512.0) + 2
