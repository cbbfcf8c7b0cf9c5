"""Binding of the benchmark's read-only probes (libspprobe.so): what plain streaming of the K
cache achieves on this device, measured in the same run as sp_score.  Not part of the scoring path."""
from __future__ import annotations

import ctypes as C
import os

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspprobe.so")
EXPORTS = ("sp_probe_read", "sp_probe_tiled", "sp_probe_tiled_default_policy")
_lib = None


def load_library() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it first (python -m paper_2502_02789_amd.build)")
        lib = C.CDLL(LIB_PATH)
        lib.sp_probe_read.restype = C.c_int
        lib.sp_probe_read.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p]
        for fn in (lib.sp_probe_tiled, lib.sp_probe_tiled_default_policy):
            fn.restype = C.c_int
            fn.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_void_p,
                           C.c_void_p]
        _lib = lib
    return _lib


def stream_ceiling(k_layers, reps: int = 30, warmup: int = 30) -> dict:
    """Times both probes on the given per-layer K tensors (contiguous [T, H_kv, d] bf16 on the GPU)
    with HIP events on torch's current stream; returns GB/s figures for the benchmark's JSON line."""
    import torch
    lib = load_library()
    L = len(k_layers)
    T, H_kv, d = k_layers[0].shape
    arr = (C.c_void_p * L)(*[int(k.data_ptr()) for k in k_layers])
    sink = torch.zeros(64, dtype=torch.int32, device=k_layers[0].device)
    stream = torch.cuda.current_stream()
    handle = int(stream.cuda_stream) or None
    layer_bytes = T * H_kv * d * 2
    total = layer_bytes * L

    def timed(launch):
        for _ in range(warmup):
            launch()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record(stream)
            launch()
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        return ms[len(ms) // 2]

    def check(rc):
        if rc != 0:
            raise RuntimeError(f"probe launch failed with status {rc}")

    out = {}
    best = None
    for blocks in (512, 2048, 8192):
        ms = timed(lambda: check(lib.sp_probe_read(arr, L, layer_bytes, blocks, sink.data_ptr(), handle)))
        gbps = total / (ms * 1e-3) / 1e9
        out[f"plain_read_{blocks}_blocks_gbps"] = gbps
        best = gbps if best is None else max(best, gbps)
    out["stream_ceiling_gbps"] = best
    if (T, H_kv, d) == (32768, 8, 128) and all(k.is_contiguous() for k in k_layers):
        ms = timed(lambda: check(lib.sp_probe_tiled(arr, L, T, H_kv, d, H_kv * d, d, sink.data_ptr(), handle)))
        out["scorer_pattern_read_gbps"] = total / (ms * 1e-3) / 1e9
        ms = timed(lambda: check(lib.sp_probe_tiled_default_policy(arr, L, T, H_kv, d, H_kv * d, d, sink.data_ptr(), handle)))
        out["scorer_pattern_read_default_cache_policy_gbps"] = total / (ms * 1e-3) / 1e9
    return out
