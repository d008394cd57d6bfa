#!/usr/bin/env python3
"""Throughput of the MoE FFN layer forward on one MI355X.

A step is one pass of the whole hot path (moe_layer_forward: route -> permute -> expert FFN ->
combine) over one batch of a synthetic layer; inputs and weights are resident in HBM before the
timed region.  Prints ONE JSON line with tokens/s, the roofline figures of the dominant kernel
(measured with HIP events recorded on the launch stream), and the CPU oracle timed on the host
cores on a bounded sample of the same workload.

The headline workload is the largest preset that fits one GPU: the NLLB-MoE-shaped encoder prefill
layer (Table 2 shapes, skewed expert load as in Fig. 3).  A default run (no --workload) then measures
the other presets and the hot-only shares of the two skewed presets in the same process and reports
them under the key "configs" of the same JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

import workloads as wl

PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA, published

HEADLINE = "nllb_prefill_skew"
# what a default run measures after the headline: (workload, share)
OTHERS = [("nllb_prefill_skew", "hot"), ("nllb_decode", "full"), ("switch_large_skew", "full"),
          ("switch_large_skew", "hot"), ("switch_base", "full"), ("tiny_f32", "full")]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t handles through the HIP runtime (the library records them on its launch stream)."""

    def __init__(self):
        import torch      # the runtime torch loaded is the one the library launches on
        self.hip = ctypes.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"))
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return ev

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        if self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def record(self, ev, stream):
        if self.hip.hipEventRecord(ev, ctypes.c_void_p(stream)) != 0:
            raise RuntimeError("hipEventRecord failed")

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


# HBM-side bytes per launch of the expert-FFN kernels, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (summaries and commands: profiles/<workload>_full_layer.txt).  Valid only for the kernel sources they
# were taken with: reported as null once one of the sources below has changed.
TRAFFIC_SOURCES = {"ffn.hip": "3244c151d56e3a52", "ffn_tile.hip": "436f9bad48effd6a",
                   "tile_schedule.hpp": "9fe1793c9c6ad92e", "common.hpp": "7306a852dfe63120"}
TRAFFIC_BYTES = {
    ("switch_base", "stream_w1"): 316526015, ("switch_base", "stream_w2"): 320342552,
    ("switch_large_skew", "stream_w1"): 68335790, ("switch_large_skew", "stream_w2"): 141349222,
    ("switch_large_skew", "tile_w1"): 90878013, ("switch_large_skew", "tile_w2"): 133077616,
    ("nllb_decode", "stream_w1"): 1643615820, ("nllb_decode", "stream_w2"): 1645576598,
    ("nllb_prefill_skew", "stream_w1"): 913815377, ("nllb_prefill_skew", "stream_w2"): 972053271,
    ("nllb_prefill_skew", "tile_w1"): 2556990570, ("nllb_prefill_skew", "tile_w2"): 2389242192,
}


def recorded_traffic(workload: str, share: str, tag: str):
    import hashlib
    if share != "full":
        return None
    for fn, want in TRAFFIC_SOURCES.items():
        path = os.path.join(ROOT, "paper_2405_18832_amd", "csrc", fn)
        try:
            if hashlib.sha256(open(path, "rb").read()).hexdigest()[:16] != want:
                return None
        except OSError:
            return None
    return TRAFFIC_BYTES.get((workload, tag))


def describe(cfg) -> str:
    return (f"{cfg.name}: T={cfg.T} d_model={cfg.d_model} d_ff={cfg.d_ff} E={cfg.E} top-{cfg.k} "
            f"{'renormalised' if cfg.renormalize else 'raw-prob'} gates, {cfg.dtype}, seed {cfg.seed}"
            + (f", gate bias ln Zipf(s={cfg.zipf_s})" if cfg.zipf_s else ""))


def config_of(name: str):
    return (wl.matched_noise(wl.CONFIGS[name[:-8]]) if name.endswith("_matched")
            else wl.CONFIGS.get(name) or wl.EXTRA_CONFIGS[name])


def hot_cold_shares_context(L, H: int, steps: int) -> dict:
    """Context, not the metric: the paper's two workflows side by side (Section 3.3).  The hot share (top-H mask) and
    the cold share (its complement) as two moe_layer_forward calls, each with its own workspace and output, once on
    two streams at the same time and once back to back on one stream, against the single full call."""
    import torch

    import paper_2405_18832_amd as moe
    L.route(H=H)
    torch.cuda.synchronize()
    hot = L.hot_mask.clone()
    cold = (1 - hot).to(torch.uint8)
    ws2, out2 = torch.empty_like(L.ws), torch.empty_like(L.out)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    cur = torch.cuda.current_stream()

    def call(mask, out, ws, stream, i):
        w1, w2 = L.weight_copies[i % len(L.weight_copies)]
        moe.moe_layer_forward(L.shape, L.x, L.w_gate, L.b_gate, w1, w2, mask, -1, out, ws=ws, stream=stream.cuda_stream)

    def timed(step):
        for i in range(2):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def both_streams(i):
        call(hot, L.out, L.ws, sa, i)
        call(cold, out2, ws2, sb, i)

    def one_stream(i):
        call(hot, L.out, L.ws, cur, i)
        call(cold, out2, ws2, cur, i)

    return {"hot_experts": int(hot.sum().item()), "two_streams_ms": timed(both_streams),
            "one_stream_ms": timed(one_stream), "full_call_ms": timed(lambda i: L.forward(copy=i)), "steps": steps}


def library_gemm_context(M: int, d: int, f: int) -> dict:
    """Context, not a target: the ROCm BLAS library's dense bf16 GEMM (through torch.matmul) on the shapes of the
    two products of the large experts taken together, M rows, with normal random operands (the second product's
    row operand passed through ReLU, as the layer's is).  The chip lowers its clock under matrix load, by an
    amount that depends on the operand values, so a dense GEMM of the same shape and value distribution is the
    yardstick for what fraction of the published peak is reachable at all."""
    import torch
    out = {}
    for tag, (N, K, relu) in {"x_w1": (f, d, False), "h_w2": (d, f, True)}.items():
        a = torch.randn(M, K, device="cuda:0", dtype=torch.bfloat16)
        if relu:
            a = torch.relu(a)
        b = torch.randn(N, K, device="cuda:0", dtype=torch.bfloat16) / K ** 0.5
        for _ in range(3):
            c = a @ b.t()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            c = a @ b.t()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        tf = 2.0 * M * N * K / (us * 1e-6) / 1e12
        out[tag] = {"M": M, "N": N, "K": K, "us": us, "tflops": tf, "frac_of_peak": tf / PEAK_BF16_TFLOPS}
        del a, b, c
    torch.cuda.empty_cache()
    return out


def measure(name: str, share: str, K: int, W: int, copies_arg: int = 0, cpu_baseline: bool = False,
            measure_fetch: bool = False, breakdown: bool = True) -> dict:
    """One workload: W warm-up steps, exactly K timed steps, then the same K steps again with HIP events
    around every expert-FFN kernel.  Returns the fields of the JSON line that depend on the workload."""
    import torch

    import paper_2405_18832_amd as moe
    from paper_2405_18832_amd.device_layer import DeviceLayer

    dev = "cuda:0"
    cfg = config_of(name)
    es = 2 if cfg.dtype == "bf16" else 4
    log(f"[bench] workload {describe(cfg)}, share {share}")

    # ---- inputs into HBM --------------------------------------------------------------------
    x = wl.make_activations(cfg)
    wg, b = wl.make_gate(cfg)
    cache = {}

    def expert(e):
        if e not in cache:
            cache[e] = wl.make_expert(cfg, e)
        return cache[e]

    t0 = time.perf_counter()
    small = cfg.E * cfg.d_model * cfg.d_ff <= 400e6
    L = DeviceLayer(cfg, x, wg, b, expert, experts=None if small else [], device=dev, workers=16)
    if not small:      # route on the device, then give the experts that receive tokens their seeded weights
        L.route()
        active = [e for e, c in enumerate(L.counts.cpu().tolist()) if c > 0]
        L.upload_experts(expert, active, workers=16)
    log(f"[bench] inputs generated and uploaded in {time.perf_counter() - t0:.1f} s")

    hot = share == "hot"
    if hot and cfg.H is None:
        raise SystemExit("[bench] this workload defines no hot mask; use --share full")
    H = cfg.H if hot else -1
    L.forward(H=H, debug=True)
    torch.cuda.synchronize()
    counts = np.array(L.counts.cpu().tolist())
    mask = np.array(L.hot_mask.cpu().tolist())
    ran = (counts > 0) & (mask > 0)
    n_active = int(ran.sum())
    A_run = int(counts[ran].sum())
    w_bytes_one = n_active * cfg.d_model * cfg.d_ff * es            # one product's weights
    copies = copies_arg or max(1, min(16, int(np.ceil(2e9 / max(1, 2 * w_bytes_one)))))
    L.make_copies(copies)
    log(f"[bench] experts run {n_active}/{cfg.E}, assignments run {A_run}/{cfg.A}, max tokens/expert "
        f"{int(counts.max())}; {copies} weight copies rotated "
        f"({copies * 2 * w_bytes_one / 1e9:.2f} GB of distinct weights between reuses)")

    edges = [0, 1, 8, 64, 312, 1 << 30]                  # 312: about the rows at which an expert turns MFMA-bound
    bins = [int(((counts >= lo) & (counts < hi)).sum()) for lo, hi in zip(edges[:-1], edges[1:])]
    top = np.sort(counts)[::-1]
    Hshow = cfg.H if cfg.H is not None else max(1, cfg.E // 8)
    log(f"[bench] tokens per expert: 0: {bins[0]} experts, 1-7: {bins[1]}, 8-63: {bins[2]}, 64-311: {bins[3]}, "
        f">=312: {bins[4]}; top-{Hshow} experts hold {100.0 * top[:Hshow].sum() / max(1, counts.sum()):.1f} % of the assignments")

    # ---- pass A: the timed steps -----------------------------------------------------------------
    for i in range(W):
        L.forward(H=H, copy=i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        L.forward(H=H, copy=i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / K * 1e3
    tokens_s = cfg.T * K / dt

    # ---- pass B: same loop with HIP events around each expert-FFN kernel ------------------------
    hev = HipEvents()
    evs = [[hev.create() for _ in range(5)] for _ in range(K)]
    torch.cuda.synchronize()
    # Two events recorded back to back, with nothing between them, are already some microseconds apart (the
    # second event's own packet): that interval is measured after every step, on the same stream, and taken
    # off each kernel's interval, which then agrees with the kernel durations rocprofv3 reports.
    gap = [[hev.create(), hev.create()] for _ in range(K)]
    stream = torch.cuda.current_stream().cuda_stream
    for i in range(K):
        moe.moe_set_profile_events(evs[i])
        L.forward(H=H, copy=i)
        hev.record(gap[i][0], stream)
        hev.record(gap[i][1], stream)
    moe.moe_set_profile_events(None)
    torch.cuda.synchronize()
    seg_raw = np.array([[hev.elapsed_ms(e[j], e[j + 1]) for j in range(4)] for e in evs]) * 1e3      # us
    ev_gap = float(np.median([hev.elapsed_ms(a, z) for a, z in gap])) * 1e3
    seg = np.maximum(seg_raw - ev_gap, 0.0)
    for e5 in evs + gap:
        for e in e5:
            hev.destroy(e)

    # ---- per-entry-point breakdown (torch events on the same stream) ---------------------------
    def timed(fn, reps=50):
        fn(0)
        torch.cuda.synchronize()
        a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(reps):
            fn(i)
        z.record()
        torch.cuda.synchronize()
        return a.elapsed_time(z) / reps * 1e3

    br = {}
    if breakdown:
        mask_t = L.hot_mask.clone() if hot else None
        L.route(H=H)
        reps = 50 if ms_step < 1.0 else 10
        br = {"route_us": timed(lambda i: L.route(H=H), reps),
              "permute_us": timed(lambda i: L.permute(), reps),
              "expert_ffn_us": timed(lambda i: L.expert_ffn(mask=mask_t, copy=i), reps),
              "combine_us": timed(lambda i: L.combine(mask=mask_t), reps)}

    # ---- roofline of the dominant kernel ---------------------------------------------------------
    # Experts with at least `min_rows` rows run in the LDS-tiled kernel, the others in the weight-streaming
    # kernel (the library says where the line is for these counts; 0: everything streams).
    d, f = cfg.d_model, cfg.d_ff
    min_rows = moe.moe_tiled_kernel_min_rows(L.shape, [int(c) if r else 0 for c, r in zip(counts, ran)])
    big = ran & (counts >= min_rows) if min_rows > 0 else np.zeros_like(ran)
    smalls = ran & ~big
    rows_s, rows_b = int(counts[smalls].sum()), int(counts[big].sum())
    wb_s, wb_b = int(smalls.sum()) * d * f * es, int(big.sum()) * d * f * es
    names = ["ffn_tile_kernel (x.W1 product, large experts)", "ffn_stream_kernel (x.W1 product, small experts)",
             "ffn_tile_kernel (h.W2 product, large experts)", "ffn_stream_kernel (h.W2 product, small experts)"]
    tags = ["tile_w1", "stream_w1", "tile_w2", "stream_w2"]
    kern = []
    for j in range(4):
        rows, wb = (rows_b, wb_b) if j % 2 == 0 else (rows_s, wb_s)
        io = rows * d * (es if j < 2 else 4)                 # rows in (first product) / fp32 rows out (second)
        kern.append(dict(name=names[j], tag=tags[j], us=float(seg[:, j].mean()), us_min=float(seg[:, j].min()),
                         us_raw=float(seg_raw[:, j].mean()), bytes=wb + io, flops=2.0 * rows * d * f))
    kd = max(kern, key=lambda q: q["us"])
    t_flop = kd["flops"] / (PEAK_BF16_TFLOPS * 1e12)
    t_byte = kd["bytes"] / (PEAK_HBM_GBPS * 1e9)
    traffic = recorded_traffic(name, share, kd["tag"])
    if cfg.dtype != "bf16" or kd["us"] <= 0:
        roof = None
    elif t_flop > t_byte:
        ach = kd["flops"] / (kd["us"] * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic,
                "frac_between_events": kd["flops"] / (kd["us_raw"] * 1e-6) / 1e12 / PEAK_BF16_TFLOPS}
    else:
        ach = kd["bytes"] / (kd["us"] * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBPS, "traffic": traffic,
                "frac_between_events": kd["bytes"] / (kd["us_raw"] * 1e-6) / 1e9 / PEAK_HBM_GBPS}
    if roof is not None:
        roof.update(kernel=kd["name"], kernel_us=kd["us"], kernel_us_min=kd["us_min"],
                    kernel_us_between_events=kd["us_raw"], empty_event_interval_us=ev_gap,
                    algorithmic_bytes=kd["bytes"], flops=kd["flops"],
                    ffn_kernels_us={q["tag"]: round(q["us"], 2) for q in kern})

    layer_flops = 2.0 * cfg.T * d * cfg.E + 4.0 * A_run * d * f
    layer_bytes = 2 * w_bytes_one + 2 * cfg.T * d * es + d * cfg.E * es
    t_floor = max(layer_flops / (PEAK_BF16_TFLOPS * 1e12), layer_bytes / (PEAK_HBM_GBPS * 1e9))
    layer = {"tflops": layer_flops / (ms_step * 1e-3) / 1e12,
             "useful_GBps": layer_bytes / (ms_step * 1e-3) / 1e9,
             "useful_bytes": layer_bytes, "flops": layer_flops,
             # whole step against the larger of its two floors (all flops at the MFMA peak, all useful bytes at
             # the HBM peak)
             "frac_of_roofline": t_floor / (ms_step * 1e-3) if cfg.dtype == "bf16" else None,
             "experts_run": n_active, "assignments_run": A_run, **{k_: round(v, 2) for k_, v in br.items()}}

    # ---- optional: parameter movement on demand over the host link (Section 3.2), logged only ----------
    if measure_fetch and cfg.dtype == "bf16":
        fetch_mask = torch.from_numpy(ran.astype(np.uint8))
        host_w1 = L.w1.cpu().pin_memory()
        dst = torch.empty_like(L.w1)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for rep in range(2):                               # first pass warms the pinned pages up
            ev0.record()
            moe.moe_fetch_experts(L.shape, 1, host_w1, fetch_mask, dst)
            ev1.record()
            torch.cuda.synchronize()
        fb = int(ran.sum()) * d * f * es
        fms = ev0.elapsed_time(ev1)
        log(f"[bench] moe_fetch_experts: {int(ran.sum())} activated experts' W1, {fb / 1e6:.1f} MB from pinned host "
            f"memory in {fms:.3f} ms = {fb / fms / 1e6:.1f} GB/s (Eq. 1 for the whole layer: "
            f"{moe.moe_parameter_movement_bytes(L.shape) / 1e6:.1f} MB, Eq. 2: "
            f"{moe.moe_activation_movement_bytes(L.shape) / 1e6:.2f} MB)")
        del host_w1, dst

    # ---- CPU oracle on a bounded sample of the same workload -------------------------------------
    cpu = None
    if cpu_baseline:
        from oracle import moe_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = len(os.sched_getaffinity(0))
        S = cfg.T if cfg.T <= 2048 else 256
        xs = x[:S]
        idx_s = np.array(L.topk_idx.cpu().tolist())[:S]
        for e in sorted(set(idx_s.reshape(-1).tolist())):      # weight generation is not timed
            expert(e)
        mask_np = mask.astype(np.uint8) if hot else None
        reps, cdt = 0, 0.0
        while reps == 0 or (cdt < 10.0 and reps < 200):      # about 10 s of CPU work
            t0 = time.perf_counter()
            ref = orc.layer_forward(xs, wg, b, expert, cfg.k, cfg.renormalize, mask_np, return_intermediates=True)
            cdt += time.perf_counter() - t0
            reps += 1
        ok = ref["margin"] >= 1e-4
        got = L.out[:S].float().cpu().numpy()
        # the timed oracle never rounds the hidden activation; the second figure is against the oracle that
        # rounds it to the storage type once, as a run in that type does
        err_rows = orc.rel_error_rows(got[ok], ref["out"][ok])
        err = float(err_rows.max()) if ok.any() else 0.0
        vec = float(orc.row_error_norms(got[ok], ref["out"][ok]).max()) if ok.any() else 0.0
        err_s = None
        if cfg.dtype == "bf16":
            ref_s = orc.layer_forward(xs, wg, b, expert, cfg.k, cfg.renormalize, mask_np, h_dtype="bf16")
            err_s = float(orc.rel_error_rows(got[ok], ref_s[ok]).max()) if ok.any() else 0.0
        cpu = {"value": S * reps / cdt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"first {S} of {cfg.T} tokens, whole layer, fp64 numpy, {reps} repetitions in {cdt:.2f} s "
                         f"(host cores visible: {len(os.sched_getaffinity(0))})",
               "gpu_vs_oracle_max_rel_err": err, "gpu_vs_oracle_max_row_l2_err": vec,
               "gpu_vs_storage_precision_oracle_max_rel_err": err_s}
        log(f"[bench] oracle: {S} tokens x {reps} in {cdt:.2f} s on {threads} threads; GPU vs oracle: element-wise "
            f"max rel err {err:.3e} (per-row normalised), worst row L2 err {vec:.3e}; vs the oracle that stores the "
            f"hidden activation in bf16: {err_s if err_s is None else format(err_s, '.3e')}")

    ctx = None
    if cpu_baseline and cfg.H is not None and not hot:
        ctx = {"hot_cold_shares": hot_cold_shares_context(L, cfg.H, K)}
        hc = ctx["hot_cold_shares"]
        log(f"[bench] context: hot share ({hc['hot_experts']} experts) and cold share as two calls: "
            f"{hc['two_streams_ms']:.3f} ms on two streams at once, {hc['one_stream_ms']:.3f} ms back to back on one, "
            f"{hc['full_call_ms']:.3f} ms for the one full call")
    if cpu_baseline and rows_b > 0 and roof is not None and roof["bound"] == "mfma":
        del L
        L = None
        gc.collect()
        torch.cuda.empty_cache()
        ctx = dict(ctx or {}, library_gemm=library_gemm_context(rows_b, d, f))
        log("[bench] context: library bf16 GEMM on the large experts' rows taken together: "
            + ", ".join(f"{k_} {v['us']:.0f} us = {v['tflops']:.0f} TFLOP/s ({v['frac_of_peak']:.3f} of peak)"
                        for k_, v in ctx["library_gemm"].items()))

    res = {"value": tokens_s, "ms_per_step": ms_step, "dtype": cfg.dtype, "context": ctx,
           "config": {"workload": describe(cfg), "share": share, "weight_copies_rotated": copies},
           "roofline": roof, "cpu_baseline": cpu, "layer": layer}
    del L, cache
    gc.collect()
    torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    choices=wl.CONFIG_ORDER + [n + "_matched" for n in ("switch_large_skew", "nllb_prefill_skew")]
                    + list(wl.EXTRA_CONFIGS),
                    help=f"measure this workload only (default: {HEADLINE}, then the other presets under 'configs')")
    ap.add_argument("--share", default="full", choices=["full", "hot"],
                    help="full layer, or only the top-H hot experts' share (workloads with a hot mask)")
    ap.add_argument("--copies", type=int, default=0,
                    help="weight copies rotated through the timing loop (0 = enough for 2 GB between reuses)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--measure-fetch", action="store_true",
                    help="also time moe_fetch_experts (activated experts' W1 from pinned host memory) and log the rate")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch

    import paper_2405_18832_amd as moe

    moe.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    K, W = args.steps, args.warmup
    name = args.workload or HEADLINE

    # context, not a target: a large device-to-device copy on the same device, same run
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(4):
        cp_dst.copy_(cp_src)
    c1.record()
    torch.cuda.synchronize()
    log(f"[bench] context: device-to-device copy of 1 GiB: {4 * 2 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9:.0f} GB/s "
        f"read + written")
    del cp_src, cp_dst
    torch.cuda.empty_cache()

    head = measure(name, args.share, K, W, args.copies, cpu_baseline=not args.no_cpu_baseline,
                   measure_fetch=args.measure_fetch)
    out = {"metric": "MoE-FFN tokens/s", "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": K,
           "warmup": W, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic", "config": head["config"],
           "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"], "layer": head["layer"],
           "context": head["context"]}

    if args.workload is None:
        # the other presets and the hot-only shares: short steps, so more of them for a steady figure
        configs = {f"{name}:{args.share}": {"ms_per_step": head["ms_per_step"], "tokens_s": head["value"],
                                            "roofline": head["roofline"],
                                            "frac_of_roofline": head["layer"]["frac_of_roofline"]}}
        for oname, oshare in OTHERS:
            r = measure(oname, oshare, max(K, 50), max(W, 10), 0, cpu_baseline=False, breakdown=False)
            configs[f"{oname}:{oshare}"] = {"ms_per_step": r["ms_per_step"], "tokens_s": r["value"],
                                            "steps": max(K, 50), "roofline": r["roofline"],
                                            "frac_of_roofline": r["layer"]["frac_of_roofline"],
                                            "experts_run": r["layer"]["experts_run"],
                                            "assignments_run": r["layer"]["assignments_run"]}
        out["configs"] = configs
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
