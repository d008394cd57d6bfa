"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, rejects bad arguments before launching anything, and sizes its workspace sanely."""
import ctypes
import os
import re

import pytest

import paper_2405_18832_amd as moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    names = declared_functions()
    assert sorted(moe.EXPORTS) == names
    for n in ["moe_route", "moe_select_hot", "moe_fetch_experts", "moe_expert_ffn_biased", "moe_layer_forward_biased", "moe_permute", "moe_expert_ffn", "moe_combine", "moe_layer_forward"]:
        assert n in names and callable(getattr(moe, n))


def test_library_exports_every_declared_symbol():
    lib = moe.load()
    for n in declared_functions():
        assert getattr(lib, n) is not None
    assert moe.status_string(0) == "MOE_OK"
    assert moe.status_string(3) == "MOE_ERR_WORKSPACE"


def shape(**kw):
    base = dict(T=64, d_model=64, d_ff=256, E=8, k=2, dtype="bf16", renormalize=True)
    base.update(kw)
    return moe.make_shape(**base)


def test_workspace_size():
    s = shape()
    n = moe.moe_workspace_bytes(s)
    A = 64 * 2
    assert n >= A * 256 * 2 + A * 64 * 4                   # h + y_perm at least
    assert n % 256 == 0
    assert moe.moe_workspace_bytes(shape(T=128)) > n
    assert moe.moe_packed_weight_bytes(s) == 8 * 64 * 256 * 2
    assert moe.moe_packed_weight_bytes(shape(dtype="f32")) == 8 * 64 * 256 * 4
    assert moe.moe_workspace_bytes(shape(k=9)) == 0         # bad shape -> 0


FAKE = 0x1000      # a non-null, 256-aligned address that is never dereferenced on these paths


def route_status(s, x=FAKE, wg=FAKE, idx=FAKE, w=FAKE, counts=FAKE, offsets=FAKE, H=-1, hot=None,
                 ws=FAKE, ws_bytes=None):
    lib = moe.load()
    if ws_bytes is None:
        ws_bytes = max(256, moe.moe_workspace_bytes(s))
    return lib.moe_route(ctypes.byref(s), x, wg, None, idx, w, None, counts, offsets, H, hot, ws, ws_bytes, None)


@pytest.mark.parametrize("kw,status", [
    (dict(k=0), moe.MOE_ERR_INVALID_ARG),
    (dict(k=9, E=16), moe.MOE_ERR_UNSUPPORTED),
    (dict(k=3, E=2), moe.MOE_ERR_INVALID_ARG),
    (dict(E=2048), moe.MOE_ERR_UNSUPPORTED),
    (dict(d_model=48), moe.MOE_ERR_UNSUPPORTED),        # bf16 needs multiples of 32
    (dict(d_ff=100), moe.MOE_ERR_UNSUPPORTED),
    (dict(T=-1), moe.MOE_ERR_INVALID_ARG),
    (dict(activation=2), moe.MOE_ERR_UNSUPPORTED),        # 0 = ReLU and 1 = GeLU exist
    (dict(dtype=7), moe.MOE_ERR_INVALID_ARG),
])
def test_bad_shapes_are_rejected(kw, status):
    assert route_status(shape(**kw), ws_bytes=1 << 30) == status


def test_bad_pointers_and_workspace_are_rejected():
    s = shape()
    assert route_status(s, x=None) == moe.MOE_ERR_INVALID_ARG
    assert route_status(s, idx=None) == moe.MOE_ERR_INVALID_ARG
    assert route_status(s, H=4, hot=None) == moe.MOE_ERR_INVALID_ARG
    assert route_status(s, ws=None) == moe.MOE_ERR_WORKSPACE
    assert route_status(s, ws=FAKE + 8) == moe.MOE_ERR_WORKSPACE        # misaligned
    assert route_status(s, ws_bytes=moe.moe_workspace_bytes(s) - 1) == moe.MOE_ERR_WORKSPACE
    lib = moe.load()
    n = moe.moe_workspace_bytes(s)
    assert lib.moe_permute(ctypes.byref(s), FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, n, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_permute(ctypes.byref(s), None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, n, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_expert_ffn(ctypes.byref(s), FAKE, None, FAKE, FAKE, None, FAKE, FAKE, n, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_expert_ffn(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, 16, None) == moe.MOE_ERR_WORKSPACE
    assert lib.moe_combine(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, None, None, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_layer_forward(ctypes.byref(s), FAKE, FAKE, None, FAKE, FAKE, None, -1, None, None, None, None,
                                 None, None, FAKE, n, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_pack_weights(ctypes.byref(s), 3, FAKE, FAKE + 256, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_pack_weights(ctypes.byref(s), 1, FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_route(None, FAKE, FAKE, None, FAKE, FAKE, None, FAKE, FAKE, -1, None, FAKE, n, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_select_hot(ctypes.byref(s), None, 1.0, 1.0, 1.0, FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_select_hot(ctypes.byref(s), FAKE, -1.0, 1.0, 1.0, FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_select_hot(ctypes.byref(s), FAKE, 1.0, 0.0, 1.0, FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_select_hot(ctypes.byref(s), FAKE, 1.0, 1.0, float("nan"), FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG


def test_data_movement_calculators():
    # host arithmetic of the library against the oracle's Eq. 1-2 (Section 3.2); bytes = values * storage size
    from oracle import moe_oracle as orc
    for kw, es in [(dict(), 2), (dict(dtype="f32"), 4), (dict(T=2048, d_model=768, d_ff=3072, E=64, k=1), 2)]:
        s = shape(**kw)
        assert moe.moe_parameter_movement_bytes(s) == orc.parameter_movement(s.E, s.d_model, s.d_ff) * es
        assert moe.moe_activation_movement_bytes(s) == orc.activation_movement(s.T, s.d_model) * es
    assert moe.moe_parameter_movement_bytes(shape(k=9)) == 0
    lib = moe.load()
    s = shape()
    assert lib.moe_fetch_experts(ctypes.byref(s), 3, FAKE, FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_fetch_experts(ctypes.byref(s), 1, None, FAKE, FAKE, None) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_fetch_experts(ctypes.byref(s), 1, FAKE, None, FAKE, None) == moe.MOE_ERR_INVALID_ARG


def test_plan_devices_against_oracle():
    # host arithmetic of the library against the oracle's round-robin placement (Section 3.3, last paragraph)
    import numpy as np
    from oracle import moe_oracle as orc
    rng = np.random.default_rng(5)
    for E, G in [(1, 1), (8, 2), (64, 3), (128, 4), (128, 7), (1024, 8)]:
        counts = rng.integers(0, 6, size=E) * rng.integers(0, 40, size=E)        # zeros and ties on purpose
        skip = (rng.random(E) < 0.2).astype(np.uint8)
        for sk in (None, skip):
            got = moe.moe_plan_devices(counts, sk, G)
            assert np.array_equal(got, orc.plan_devices(counts, G, sk))
    lib = moe.load()
    c = np.array([1, 2, 3], dtype=np.int32)
    out = np.full(3, 77, dtype=np.int32)
    assert lib.moe_plan_devices(3, c.ctypes.data, None, 0, out.ctypes.data) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_plan_devices(3, None, None, 2, out.ctypes.data) == moe.MOE_ERR_INVALID_ARG
    assert lib.moe_plan_devices(3, c.ctypes.data, None, 2, None) == moe.MOE_ERR_INVALID_ARG
    bad = np.array([1, -2, 3], dtype=np.int32)
    assert lib.moe_plan_devices(3, bad.ctypes.data, None, 2, out.ctypes.data) == moe.MOE_ERR_INVALID_ARG
    assert np.all(out == 77)                                                       # nothing written on error


def test_binding_raises_on_error():
    with pytest.raises(moe.MoEError) as ei:
        moe.moe_combine(shape(), FAKE, FAKE, FAKE, FAKE, None, None, stream=0)
    assert ei.value.status == moe.MOE_ERR_INVALID_ARG


def test_noalloc_entry_point_refuses_before_any_gpu_call():
    """The entry point that allocates nothing checks the shape and the size of the workspace it would need
    against its static array on the host, before anything touches a GPU."""
    lib = moe.load()
    assert moe.moe_noalloc_max_workspace() == 16 << 20

    def status(s):
        return lib.moe_layer_forward_noalloc(ctypes.byref(s), FAKE, FAKE, None, FAKE, FAKE, None, -1, FAKE, None)

    assert status(shape(k=9)) == moe.MOE_ERR_INVALID_ARG           # k > E
    assert status(shape(d_model=48)) == moe.MOE_ERR_UNSUPPORTED    # bf16 needs multiples of 32
    big = shape(T=4096, d_model=1024, d_ff=4096, E=128, k=1)
    assert moe.moe_workspace_bytes(big) > moe.moe_noalloc_max_workspace()
    assert status(big) == moe.MOE_ERR_WORKSPACE
    # decoder steps of the NLLB-shaped layer fit
    assert moe.moe_workspace_bytes(shape(T=32, d_model=2048, d_ff=8192, E=128, k=2)) < moe.moe_noalloc_max_workspace()


def test_tune_alpha_matches_the_oracle():
    """Host arithmetic of the alpha auto-tuning step (Section 3.3, after Eq. 6) against the oracle: the hand-worked
    cases, random inputs, and the refusals."""
    import json

    import numpy as np

    from oracle import moe_oracle as orc
    with open(os.path.join(ROOT, "tests", "golden", "alpha_tuning_examples.json")) as fh:
        for c in json.load(fh)["cases"]:
            a, best = moe.moe_tune_alpha(c["alpha"], c["bw_a"], c["bw_b"], c["activated"], c["times"])
            assert best == c["best"] and abs(a - c["alpha_new"]) <= 1e-15 * max(1.0, c["alpha_new"]), c
    rng = np.random.default_rng(23)
    for _ in range(200):
        B, C = int(rng.integers(1, 7)), int(rng.integers(1, 5))
        t = rng.uniform(0.5, 3.0, (B, C))
        if rng.integers(0, 3) == 0:
            t[:, rng.integers(0, C)] = t[:, 0]                # equal totals happen
        act = rng.integers(0, 130, B)
        alpha, a, b = float(rng.uniform(0, 3)), float(rng.uniform(1, 100)), float(rng.uniform(0, 1000))
        got = moe.moe_tune_alpha(alpha, a, b, act, t)
        want = orc.tune_alpha(alpha, a, b, act, t)
        assert got[1] == want[1] and got[0] == want[0], (got, want)      # same operations in the same order
    lib = moe.load()
    act = (ctypes.c_int32 * 2)(3, 4)
    t = (ctypes.c_double * 4)(1.0, 2.0, 3.0, 4.0)
    out = ctypes.c_double(-1.0)

    def status(alpha=1.0, bw_a=1.0, bw_b=1.0, nb=2, a=act, nc=2, tt=t):
        return lib.moe_tune_alpha(alpha, bw_a, bw_b, nb, a, nc, tt, ctypes.addressof(out), None)

    assert status() == moe.MOE_OK and out.value == 1.0        # totals (4, 6): offset 0
    assert status(nb=0) == moe.MOE_ERR_INVALID_ARG and status(nc=0) == moe.MOE_ERR_INVALID_ARG
    assert status(a=None) == moe.MOE_ERR_INVALID_ARG and status(tt=None) == moe.MOE_ERR_INVALID_ARG
    assert status(bw_a=0.0) == moe.MOE_ERR_INVALID_ARG and status(alpha=float("nan")) == moe.MOE_ERR_INVALID_ARG
    assert status(tt=(ctypes.c_double * 4)(1.0, 0.0, 3.0, 4.0)) == moe.MOE_ERR_INVALID_ARG
    assert status(a=(ctypes.c_int32 * 2)(3, -1)) == moe.MOE_ERR_INVALID_ARG


def test_tiled_kernel_min_rows():
    """Host arithmetic: from how many rows on an expert is run by the LDS-tiled kernel.  128, or one more than a
    streaming tile (64 rows) once the experts of 128 rows and more fill a round of the tiled kernel's 256 blocks
    in the narrower product (d_model / 256 column tiles)."""
    s = shape(T=16384, d_model=2048, d_ff=8192, E=128, k=2)          # 8 column tiles: 32 row tiles make a round
    rows = [0] * 128
    assert moe.moe_tiled_kernel_min_rows(s, rows) == 128
    rows[0] = 31 * 256                                               # 31 tiles
    assert moe.moe_tiled_kernel_min_rows(s, rows) == 128
    rows[1] = 129                                                    # the 32nd
    assert moe.moe_tiled_kernel_min_rows(s, rows) == 65
    rows[1] = 127                                                    # not large by itself: still 31
    assert moe.moe_tiled_kernel_min_rows(s, rows) == 128
    s2 = shape(T=4096, d_model=1024, d_ff=4096, E=128, k=1)          # 4 column tiles: 64 row tiles
    rows = [256] * 63 + [0] * 65
    assert moe.moe_tiled_kernel_min_rows(s2, rows) == 128
    rows[63] = 1000
    assert moe.moe_tiled_kernel_min_rows(s2, rows) == 65
    # shapes that never use the tiled kernel
    assert moe.moe_tiled_kernel_min_rows(shape(T=64), [10] * 8) == 0
    assert moe.moe_tiled_kernel_min_rows(shape(T=4096, dtype="f32"), [512] * 8) == 0
