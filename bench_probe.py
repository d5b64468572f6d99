"""Benchmark helper beside bench.py: builds and loads libbench_probe.so (bench_probe.hip), a
register-only loop of matrix instructions that shows what the matrix pipes of this chip sustain, as
context for the published peak.  Not part of the layer library and not imported by the package."""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "bench_probe.hip")
LIB = os.path.join(_HERE, "libbench_probe.so")
_lib = None


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    hipcc = os.environ.get("HIPCC") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", SRC, "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    return LIB


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        lib = ctypes.CDLL(LIB)
        lib.bench_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                         ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p]
        lib.bench_mfma_probe.restype = ctypes.c_int
        _lib = lib
    return _lib


def mfma_probe(workgroups: int, iters: int, out, stream=None, f64: bool = False) -> int:
    """Enqueue the loop (fp32 32x32x2, or fp64 16x16x4 with f64=True) on `stream` (a torch stream, or
    the current one); `out` is an int64 device tensor of 8*workgroups elements (per wave: core-clock
    ticks, constant-timer ticks).  Returns the rate of the constant timer in kHz."""
    import torch

    if not (isinstance(out, torch.Tensor) and out.is_cuda and out.dtype == torch.int64 and out.is_contiguous()
            and out.numel() == 8 * int(workgroups)):
        raise ValueError("mfma_probe: out must be a contiguous int64 device tensor of 8*workgroups elements")
    s = stream if stream is not None else torch.cuda.current_stream(out.device)
    khz = ctypes.c_int32(0)
    rc = load().bench_mfma_probe(int(bool(f64)), int(workgroups), int(iters), out.data_ptr(), ctypes.byref(khz),
                                 ctypes.c_void_p(s.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"bench_mfma_probe failed with status {rc}")
    return int(khz.value)


def register_loop_rate(f64: bool = False, workgroups: int = 512, iters: int = 4096, repeats: int = 3) -> dict:
    """TFLOP/s and core clock of the loop with two waves on every SIMD."""
    import torch

    dev = torch.device("cuda", torch.cuda.current_device())
    ticks = torch.zeros(8 * workgroups, dtype=torch.int64, device=dev)
    khz = mfma_probe(workgroups, iters, ticks, f64=f64)   # warm-up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(repeats):
        mfma_probe(workgroups, iters, ticks, f64=f64)
    e1.record()
    torch.cuda.synchronize()
    tk = ticks.cpu().double().reshape(-1, 2)
    flops = repeats * workgroups * 4 * iters * 4 * (2048 if f64 else 4096)
    return {"tflops": round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1),
            "core_clock_ghz": round(float((tk[:, 0] / tk[:, 1]).median()) * khz * 1e-6, 3),
            "what": "register-only loop of %s matrix instructions, two waves per SIMD, no memory traffic"
                    % ("16x16x4 fp64" if f64 else "32x32x2 fp32")}


if __name__ == "__main__":
    print(build())
