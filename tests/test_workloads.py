"""Sanity of the seeded synthetic inputs (shapes, determinism, skew like the paper's Fig. 3)."""
import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc


def counts_of(cfg):
    x = wl.make_activations(cfg)
    wg, b = wl.make_gate(cfg)
    return orc.route(x, wg, b, cfg.k, cfg.renormalize)


def test_presets_match_the_configs():
    c = wl.CONFIGS
    assert [(c[n].T, c[n].d_model, c[n].d_ff, c[n].E, c[n].k) for n in wl.CONFIG_ORDER] == [
        (64, 64, 256, 8, 2), (2048, 768, 3072, 64, 1), (4096, 1024, 4096, 128, 1),
        (32, 2048, 8192, 128, 2), (16384, 2048, 8192, 128, 2)]
    # Table 2: expert parameter sizes 51.5 GB (24 sparse layers... of Switch-Large-128) and
    # 103.1 GB (NLLB-MoE) equal layers * E * 2*d_model*d_ff * 2 bytes with d_ff = 4*d_model
    sl, nl = c["switch_large_skew"], c["nllb_prefill_skew"]
    assert abs(24 * sl.E * 2 * sl.d_model * sl.d_ff * 2 / 1e9 - 51.5) < 0.1
    assert abs(12 * nl.E * 2 * nl.d_model * nl.d_ff * 2 / 1e9 - 103.1) < 0.1


def test_determinism_and_storage():
    cfg = wl.CONFIGS["switch_base"]
    a, b = wl.make_expert(cfg, 3), wl.make_expert(cfg, 3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert not np.array_equal(a[0], wl.make_expert(cfg, 4)[0])
    assert a[0].shape == (cfg.d_ff, cfg.d_model) and a[1].shape == (cfg.d_model, cfg.d_ff)
    # values are exactly representable in bf16
    assert np.array_equal(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(a[0])), a[0])
    assert abs(a[0].std() * np.sqrt(cfg.d_model) - 1) < 0.02
    assert abs(a[1].std() * np.sqrt(cfg.d_ff) - 1) < 0.02
    wg, bias = wl.make_gate(cfg)
    assert bias is None and abs(wg.std() - 0.02) < 1e-3


def test_zipf_bias():
    b = wl.zipf_log_bias(128, 1.1, 2)
    w = np.exp(b.astype(np.float64))
    assert abs(w.sum() - 1) < 1e-5
    s = np.sort(w)[::-1]
    assert np.allclose(s[0] / s[1], 2 ** 1.1, rtol=1e-5)
    assert not np.array_equal(np.argsort(-w), np.arange(128))     # ranks are shuffled


def test_uniform_and_decode_histograms():
    r = counts_of(wl.CONFIGS["switch_base"])
    assert orc.activated_experts(r["counts"]) == 64 and r["counts"].max() < 64
    r = counts_of(wl.CONFIGS["nllb_decode"])
    assert r["counts"].max() <= 4 and orc.activated_experts(r["counts"]) >= 40


@pytest.mark.parametrize("name,H", [("switch_large_skew", 16), ("nllb_prefill_skew", 32)])
def test_skewed_histograms(name, H):
    cfg = wl.CONFIGS[name]
    r = counts_of(cfg)
    c = r["counts"]
    mask = orc.hot_mask_top_h(c, H)
    assert c[mask == 1].sum() >= 0.99 * c.sum()          # literal gate std: very skewed
    # matched-noise variant: a few hot experts, most experts cold (Fig. 3: 0-7 tokens)
    cm = counts_of(wl.matched_noise(cfg))["counts"]
    assert orc.activated_experts(cm) > orc.activated_experts(c)
    assert cm.max() > 20 * np.median(cm)
    assert np.count_nonzero(cm <= 7) >= 0.25 * cfg.E
