#!/usr/bin/env python3
"""Throughput of the MoE FFN layer forward on one MI355X.

A step is one pass of the whole hot path (moe_layer_forward: route -> permute -> expert FFN ->
combine) over one batch of a synthetic layer; inputs and weights are resident in HBM before the
timed region.  Prints ONE JSON line with tokens/s, the roofline figures of the dominant kernel
(measured with HIP events recorded on the launch stream), and the CPU oracle timed on the host
cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
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
TRAFFIC_SOURCES = {"ffn.hip": "70eaa5058c3cc82c", "ffn_tile.hip": "d6e05b7ff0696246",
                   "tile_schedule.hpp": "cfb38ed553932c2c", "common.hpp": "8de102ccc6a3c46a"}
TRAFFIC_BYTES = {
    ("switch_base", "stream_w1"): 316508645, ("switch_base", "stream_w2"): 320281156,
    ("nllb_decode", "stream_w1"): 1643649720, ("nllb_decode", "stream_w2"): 1645597904,
    ("nllb_prefill_skew", "stream_w1"): 1158802682, ("nllb_prefill_skew", "stream_w2"): 1152661958,
    ("nllb_prefill_skew", "tile_w1"): 2503146561, ("nllb_prefill_skew", "tile_w2"): 2212283334,
}


def recorded_traffic(workload: str, tag: str):
    import hashlib
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="switch_base",
                    choices=wl.CONFIG_ORDER + [n + "_matched" for n in ("switch_large_skew", "nllb_prefill_skew")]
                    + list(wl.EXTRA_CONFIGS))
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
    from paper_2405_18832_amd.device_layer import DeviceLayer

    moe.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    name = args.workload
    cfg = (wl.matched_noise(wl.CONFIGS[name[:-8]]) if name.endswith("_matched")
           else wl.CONFIGS.get(name) or wl.EXTRA_CONFIGS[name])
    K, W = args.steps, args.warmup
    es = 2 if cfg.dtype == "bf16" else 4
    log(f"[bench] workload {describe(cfg)}")

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

    hot = args.share == "hot"
    if hot and cfg.H is None:
        log("[bench] this workload defines no hot mask; use --share full")
        return 2
    H = cfg.H if hot else -1
    L.forward(H=H, debug=True)
    torch.cuda.synchronize()
    counts = np.array(L.counts.cpu().tolist())
    mask = np.array(L.hot_mask.cpu().tolist())
    ran = (counts > 0) & (mask > 0)
    n_active = int(ran.sum())
    A_run = int(counts[ran].sum())
    w_bytes_one = n_active * cfg.d_model * cfg.d_ff * es            # one product's weights
    copies = args.copies or max(1, min(16, int(np.ceil(2e9 / max(1, 2 * w_bytes_one)))))
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
    # context, not a target: a large device-to-device copy on the same device, same run
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
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

    mask_t = L.hot_mask.clone() if hot else None
    L.route(H=H)
    br = {"route_us": timed(lambda i: L.route(H=H)),
          "permute_us": timed(lambda i: L.permute()),
          "expert_ffn_us": timed(lambda i: L.expert_ffn(mask=mask_t, copy=i)),
          "combine_us": timed(lambda i: L.combine(mask=mask_t))}

    # ---- roofline of the dominant kernel ---------------------------------------------------------
    # Experts with >= 128 rows run in the LDS-tiled kernel, the others in the weight-streaming kernel
    # (only when the layer has >= 128 tokens, else everything streams).
    d, f = cfg.d_model, cfg.d_ff
    big = ran & (counts >= 128) if (cfg.dtype == "bf16" and cfg.T >= 128) else np.zeros_like(ran)
    small = ran & ~big
    rows_s, rows_b = int(counts[small].sum()), int(counts[big].sum())
    wb_s, wb_b = int(small.sum()) * d * f * es, int(big.sum()) * d * f * es
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
    traffic = recorded_traffic(name, kd["tag"])
    if cfg.dtype != "bf16":
        roof = None
    elif t_flop > t_byte:
        ach = kd["flops"] / (kd["us"] * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic}
    else:
        ach = kd["bytes"] / (kd["us"] * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBPS, "traffic": traffic}
    if roof is not None:
        roof.update(kernel=kd["name"], kernel_us=kd["us"], kernel_us_min=kd["us_min"],
                    kernel_us_between_events=kd["us_raw"], empty_event_interval_us=ev_gap,
                    algorithmic_bytes=kd["bytes"], flops=kd["flops"],
                    ffn_kernels_us={q["tag"]: round(q["us"], 2) for q in kern})

    layer_flops = 2.0 * cfg.T * d * cfg.E + 4.0 * A_run * d * f
    layer_bytes = 2 * w_bytes_one + 2 * cfg.T * d * es + d * cfg.E * es
    layer = {"tflops": layer_flops / (ms_step * 1e-3) / 1e12,
             "useful_GBps": layer_bytes / (ms_step * 1e-3) / 1e9,
             "useful_bytes": layer_bytes, "flops": layer_flops,
             "experts_run": n_active, "assignments_run": A_run, **{k_: round(v, 2) for k_, v in br.items()}}

    # ---- optional: parameter movement on demand over the host link (Section 3.2), logged only ----------
    if args.measure_fetch and cfg.dtype == "bf16":
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
    if not args.no_cpu_baseline:
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
            ref = orc.layer_forward(xs, wg, b, expert, cfg.k, cfg.renormalize, mask_np,
                                    return_intermediates=True, h_dtype="bf16" if cfg.dtype == "bf16" else None)
            cdt += time.perf_counter() - t0
            reps += 1
        ok = ref["margin"] >= 1e-4
        got = L.out[:S].float().cpu().numpy()
        err = float(orc.rel_error(got[ok], ref["out"][ok]).max()) if ok.any() else 0.0
        cpu = {"value": S * reps / cdt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"first {S} of {cfg.T} tokens, whole layer, fp64 numpy, {reps} repetitions in {cdt:.2f} s "
                         f"(host cores visible: {len(os.sched_getaffinity(0))})",
               "gpu_vs_oracle_max_rel_err": err}
        log(f"[bench] oracle: {S} tokens x {reps} in {cdt:.2f} s on {threads} threads; GPU vs oracle max rel err {err:.3e}")

    out = {"metric": "MoE-FFN tokens/s", "value": tokens_s, "unit": "tokens/s", "n_gpus": 1, "steps": K,
           "warmup": W, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
           "config": {"workload": describe(cfg), "share": args.share, "weight_copies_rotated": copies},
           "roofline": roof, "cpu_baseline": cpu, "layer": layer}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
