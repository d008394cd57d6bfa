"""Thin Python binding of the MoE FFN C-ABI library for MI355X (gfx950).

Argument marshalling only: every function below has the name and the argument order of
its C counterpart in include/moe.h, takes torch CUDA tensors (or None for a nullable
pointer), passes their device addresses through ctypes and returns nothing; a status other
than MOE_OK raises MoEError.  All arithmetic runs in the HIP kernels.  There is no CPU
fallback: if the shared library has not been built, load() raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
# MOE_FFN_LIB may name another build of the same library (e.g. one compiled with other tuning constants)
LIB_PATH = os.environ.get("MOE_FFN_LIB") or os.path.join(_PKG, "libmoe_ffn_gfx950.so")

MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE, MOE_ERR_HIP = range(5)
MOE_F32, MOE_BF16 = 0, 1
MOE_MAX_K, MOE_MAX_E = 8, 1024

EXPORTS = ["moe_init", "moe_noalloc_max_workspace", "moe_layer_forward_noalloc",
           "moe_status_string", "moe_workspace_bytes", "moe_packed_weight_bytes", "moe_pack_weights",
           "moe_set_profile_events", "moe_tiled_kernel_min_rows",
           "moe_parameter_movement_bytes", "moe_activation_movement_bytes", "moe_plan_devices", "moe_fetch_experts", "moe_tune_alpha",
           "moe_route", "moe_select_hot", "moe_permute", "moe_expert_ffn", "moe_expert_ffn_biased", "moe_combine",
           "moe_layer_forward", "moe_layer_forward_biased"]


class MoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


class moe_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "d_model", "d_ff", "E", "k", "dtype", "renormalize", "activation")]


_lib = None


def load() -> ctypes.CDLL:
    """Load the built library (once).  Raises if it is missing: build it first with
    `python -m paper_2405_18832_amd.build` (or __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built; run python -m paper_2405_18832_amd.build")
    # torch ships its own HIP runtime (same soname as the system one).  Import it first so that this
    # library binds to the runtime torch's tensors and streams live in; loaded the other way round the
    # process ends up with two runtimes and every launch on a torch stream fails.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    sp = ctypes.POINTER(moe_shape)
    lib.moe_init.restype = ctypes.c_int
    lib.moe_init.argtypes = []
    lib.moe_noalloc_max_workspace.restype = sz
    lib.moe_noalloc_max_workspace.argtypes = []
    lib.moe_tiled_kernel_min_rows.restype = ctypes.c_int32
    lib.moe_tiled_kernel_min_rows.argtypes = [ctypes.POINTER(moe_shape), ctypes.POINTER(ctypes.c_int32)]
    lib.moe_layer_forward_noalloc.restype = ctypes.c_int
    lib.moe_layer_forward_noalloc.argtypes = [sp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.moe_status_string.restype = ctypes.c_char_p
    lib.moe_status_string.argtypes = [ctypes.c_int]
    lib.moe_workspace_bytes.restype = sz
    lib.moe_workspace_bytes.argtypes = [sp]
    lib.moe_packed_weight_bytes.restype = sz
    lib.moe_packed_weight_bytes.argtypes = [sp]
    lib.moe_set_profile_events.restype = None
    lib.moe_set_profile_events.argtypes = [ctypes.POINTER(vp)]
    lib.moe_pack_weights.restype = ctypes.c_int
    lib.moe_pack_weights.argtypes = [sp, i32, vp, vp, vp]
    lib.moe_route.restype = ctypes.c_int
    lib.moe_route.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.moe_permute.restype = ctypes.c_int
    lib.moe_parameter_movement_bytes.argtypes = [sp]
    lib.moe_parameter_movement_bytes.restype = sz
    lib.moe_activation_movement_bytes.argtypes = [sp]
    lib.moe_activation_movement_bytes.restype = sz
    lib.moe_plan_devices.argtypes = [i32, vp, vp, i32, vp]
    lib.moe_plan_devices.restype = ctypes.c_int
    lib.moe_tune_alpha.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double, i32, vp, i32, vp, vp, vp]
    lib.moe_tune_alpha.restype = ctypes.c_int
    lib.moe_fetch_experts.argtypes = [sp, i32, vp, vp, vp, vp]
    lib.moe_fetch_experts.restype = ctypes.c_int
    lib.moe_select_hot.argtypes = [sp, vp, ctypes.c_double, ctypes.c_double, ctypes.c_double, vp, vp, vp]
    lib.moe_select_hot.restype = ctypes.c_int
    lib.moe_permute.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_expert_ffn.restype = ctypes.c_int
    lib.moe_expert_ffn.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_combine.restype = ctypes.c_int
    lib.moe_expert_ffn_biased.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_expert_ffn_biased.restype = ctypes.c_int
    lib.moe_layer_forward_biased.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_layer_forward_biased.restype = ctypes.c_int
    lib.moe_combine.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_layer_forward.restype = ctypes.c_int
    lib.moe_layer_forward.argtypes = [sp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().moe_status_string(int(status)).decode()


def make_shape(T, d_model, d_ff, E, k, dtype, renormalize, activation=0) -> moe_shape:
    if isinstance(dtype, str):
        dtype = {"f32": MOE_F32, "bf16": MOE_BF16}[dtype]
    return moe_shape(int(T), int(d_model), int(d_ff), int(E), int(k), int(dtype),
                     int(bool(renormalize)), int(activation))


def _ptr(t) -> Optional[int]:
    """Device address of a tensor (None -> NULL).  Accepts a raw int for tests of the ABI."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("expected a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(status: int, where: str) -> None:
    if status != MOE_OK:
        raise MoEError(status, where)


def moe_init() -> None:
    _check(load().moe_init(), "moe_init")


def moe_noalloc_max_workspace() -> int:
    return int(load().moe_noalloc_max_workspace())


def moe_layer_forward_noalloc(shape, x, w_gate, gate_bias, w1, w2, mask, H, out, stream=None) -> None:
    _check(load().moe_layer_forward_noalloc(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(w1),
                                            _ptr(w2), _ptr(mask), int(H), _ptr(out), _stream(stream)),
           "moe_layer_forward_noalloc")


def moe_tiled_kernel_min_rows(shape: moe_shape, rows) -> int:
    """`rows`: per-expert row counts of the call (a sequence of E ints, 0 for experts that do not run)."""
    arr = (ctypes.c_int32 * len(rows))(*[int(r) for r in rows])
    return int(load().moe_tiled_kernel_min_rows(ctypes.byref(shape), arr))


def moe_workspace_bytes(shape: moe_shape) -> int:
    return int(load().moe_workspace_bytes(ctypes.byref(shape)))


def moe_packed_weight_bytes(shape: moe_shape) -> int:
    return int(load().moe_packed_weight_bytes(ctypes.byref(shape)))


def moe_set_profile_events(events=None) -> None:
    """`events`: sequence of five hipEvent_t handles (ints / c_void_p / None), or None to stop."""
    if events is None:
        load().moe_set_profile_events(None)
        return
    arr = (ctypes.c_void_p * 5)(*[e.value if isinstance(e, ctypes.c_void_p) else e for e in events])
    load().moe_set_profile_events(arr)


def moe_pack_weights(shape, which, src, dst, stream=None) -> None:
    _check(load().moe_pack_weights(ctypes.byref(shape), int(which), _ptr(src), _ptr(dst), _stream(stream)),
           "moe_pack_weights")


def moe_route(shape, x, w_gate, gate_bias, topk_idx, topk_w, margin, counts, offsets, H, hot_mask,
              ws, stream=None) -> None:
    _check(load().moe_route(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(topk_idx),
                            _ptr(topk_w), _ptr(margin), _ptr(counts), _ptr(offsets), int(H), _ptr(hot_mask),
                            _ptr(ws), _nbytes(ws), _stream(stream)), "moe_route")


def moe_parameter_movement_bytes(shape) -> int:
    return int(load().moe_parameter_movement_bytes(ctypes.byref(shape)))


def moe_activation_movement_bytes(shape) -> int:
    return int(load().moe_activation_movement_bytes(ctypes.byref(shape)))


def moe_plan_devices(counts, skip, n_devices: int):
    """counts, skip: host int32 / uint8 arrays (numpy or CPU tensors; skip may be None).  Returns a numpy int32
    array device_of[E]."""
    import numpy as np
    c = np.ascontiguousarray(np.asarray(counts), dtype=np.int32)
    k = None if skip is None else np.ascontiguousarray(np.asarray(skip), dtype=np.uint8)
    out = np.empty(c.shape[0], dtype=np.int32)
    _check(load().moe_plan_devices(int(c.shape[0]), c.ctypes.data, None if k is None else k.ctypes.data,
                                   int(n_devices), out.ctypes.data), "moe_plan_devices")
    return out


def moe_tune_alpha(alpha, bw_a, bw_b, activated, times):
    """activated: host ints [B]; times: host floats [B, C].  Returns (alpha_new, best_offset)."""
    import numpy as np
    act = np.ascontiguousarray(np.asarray(activated), dtype=np.int32)
    t = np.ascontiguousarray(np.asarray(times), dtype=np.float64)
    if t.ndim != 2 or act.shape != (t.shape[0],):
        raise ValueError("times must be [n_batches, n_candidates] and activated [n_batches]")
    a_out, c_out = ctypes.c_double(), ctypes.c_int32()
    _check(load().moe_tune_alpha(float(alpha), float(bw_a), float(bw_b), int(t.shape[0]), act.ctypes.data,
                                 int(t.shape[1]), t.ctypes.data, ctypes.addressof(a_out), ctypes.addressof(c_out)),
           "moe_tune_alpha")
    return float(a_out.value), int(c_out.value)


def moe_fetch_experts(shape, which, src_host, fetch_mask_host, dst_device, stream=None) -> None:
    """src_host, fetch_mask_host: CPU tensors (pinned for an asynchronous copy); dst_device: CUDA tensor."""
    _check(load().moe_fetch_experts(ctypes.byref(shape), int(which), ctypes.c_void_p(src_host.data_ptr()),
                                    ctypes.c_void_p(fetch_mask_host.data_ptr()), _ptr(dst_device), _stream(stream)),
           "moe_fetch_experts")


def moe_select_hot(shape, counts, alpha, bw_a, bw_b, H_out, hot_mask, stream=None) -> None:
    _check(load().moe_select_hot(ctypes.byref(shape), _ptr(counts), float(alpha), float(bw_a), float(bw_b),
                                 _ptr(H_out), _ptr(hot_mask), _stream(stream)), "moe_select_hot")


def moe_permute(shape, x, topk_idx, offsets, perm, inv_perm, x_perm, ws, stream=None) -> None:
    _check(load().moe_permute(ctypes.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(offsets), _ptr(perm),
                              _ptr(inv_perm), _ptr(x_perm), _ptr(ws), _nbytes(ws), _stream(stream)),
           "moe_permute")


def moe_expert_ffn(shape, x_perm, w1, w2, offsets, mask, y_perm, ws, stream=None) -> None:
    _check(load().moe_expert_ffn(ctypes.byref(shape), _ptr(x_perm), _ptr(w1), _ptr(w2), _ptr(offsets),
                                 _ptr(mask), _ptr(y_perm), _ptr(ws), _nbytes(ws), _stream(stream)),
           "moe_expert_ffn")


def moe_expert_ffn_biased(shape, x_perm, w1, b1, w2, b2, offsets, mask, y_perm, ws, stream=None) -> None:
    _check(load().moe_expert_ffn_biased(ctypes.byref(shape), _ptr(x_perm), _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2),
                                        _ptr(offsets), _ptr(mask), _ptr(y_perm), _ptr(ws), _nbytes(ws),
                                        _stream(stream)), "moe_expert_ffn_biased")


def moe_layer_forward_biased(shape, x, w_gate, gate_bias, w1, b1, w2, b2, mask, H, out, topk_idx=None, topk_w=None,
                             counts=None, perm=None, hot_mask_out=None, ws=None, stream=None) -> None:
    _check(load().moe_layer_forward_biased(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(w1),
                                           _ptr(b1), _ptr(w2), _ptr(b2), _ptr(mask), int(H), _ptr(out),
                                           _ptr(topk_idx), _ptr(topk_w), _ptr(counts), _ptr(perm),
                                           _ptr(hot_mask_out), _ptr(ws), _nbytes(ws), _stream(stream)),
           "moe_layer_forward_biased")


def moe_combine(shape, y_perm, inv_perm, topk_idx, topk_w, mask, out, stream=None) -> None:
    _check(load().moe_combine(ctypes.byref(shape), _ptr(y_perm), _ptr(inv_perm), _ptr(topk_idx),
                              _ptr(topk_w), _ptr(mask), _ptr(out), _stream(stream)), "moe_combine")


def moe_layer_forward(shape, x, w_gate, gate_bias, w1, w2, mask, H, out, topk_idx=None, topk_w=None,
                      counts=None, perm=None, hot_mask_out=None, ws=None, stream=None) -> None:
    _check(load().moe_layer_forward(ctypes.byref(shape), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(w1),
                                    _ptr(w2), _ptr(mask), int(H), _ptr(out), _ptr(topk_idx), _ptr(topk_w),
                                    _ptr(counts), _ptr(perm), _ptr(hot_mask_out), _ptr(ws), _nbytes(ws),
                                    _stream(stream)), "moe_layer_forward")
