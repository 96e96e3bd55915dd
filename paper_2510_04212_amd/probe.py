"""ctypes binding over libattn_probe_gfx950.so (csrc/probe.h): measurement aids for the benchmark.

No attention arithmetic and nothing from the paper: a loop of matrix instructions on register
operands and a loop of LDS reads, each timed by the device's own counters.  Loaded by bench.py
and the probe tests only; the attention library does not depend on it.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_probe_gfx950.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first with `python -m paper_2510_04212_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)
_vp, _i = ctypes.c_void_p, ctypes.c_int
_lib.attn_probe_matrix_clock.argtypes = [_vp, _i, _i, _vp]
_lib.attn_probe_matrix_clock.restype = _i
_lib.attn_probe_lds_clock.argtypes = [_vp, _i, _i, _i, _vp]
_lib.attn_probe_lds_clock.restype = _i


def raw():
    return _lib


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status):
    if status != 0:
        raise RuntimeError(f"probe call failed with status {status}")


def matrix_clock(workgroups=512, iters=50000, stream=None):
    """Runs the matrix-instruction loop and returns a dict:
      shader_clock_ghz       mean over work-groups of (shader cycles / constant-rate time) of the loop
      shader_clock_ghz_min/max   the slowest / fastest work-group's clock
      device_ms              the longest loop, in constant-rate time (the kernel as the device saw it)
      ms                     the launch as timed by events on the stream
      tflops                 instruction rate from `ms` (4 waves x 4 iters instructions of 32768 FLOP per work-group)
      clocks_per_mfma        mean shader clock x device time / instructions per SIMD (256 CUs x 4
                             SIMDs assumed busy throughout): 32 = one instruction per 8 passes of 4 clocks
    """
    out = torch.zeros(4 + 2 * workgroups, dtype=torch.int64, device="cuda")
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    s = torch.cuda.current_stream() if stream is None else stream
    # a first, tiny launch: loading the kernel's code must not fall between the two events
    _check(_lib.attn_probe_matrix_clock(ctypes.c_void_p(out.data_ptr()), 1, 1, _stream(stream)))
    e0.record(s)
    _check(_lib.attn_probe_matrix_clock(ctypes.c_void_p(out.data_ptr()), int(workgroups), int(iters), _stream(stream)))
    e1.record(s)
    e1.synchronize()
    ms = e0.elapsed_time(e1)
    rec = out[4:].cpu().numpy().reshape(workgroups, 2).astype(np.float64)
    cyc, ticks = rec[:, 0], rec[:, 1]
    ghz = cyc / (ticks / 1e8) / 1e9
    flop = float(workgroups) * 4 * 4 * iters * 32768.0
    per_simd = float(workgroups) * 4 * 4 * iters / 1024.0
    device_s = float(ticks.max()) / 1e8
    return {"shader_clock_ghz": float(ghz.mean()), "shader_clock_ghz_min": float(ghz.min()),
            "shader_clock_ghz_max": float(ghz.max()), "device_ms": float(ticks.max() / 1e8 * 1e3),
            "ms": ms, "tflops": flop / (ms * 1e-3) / 1e12,
            "clocks_per_mfma": float(ghz.mean() * 1e9 * device_s / per_simd)}


def lds_clock(kind=0, workgroups=256, iters=20000, stream=None):
    """Runs the LDS read loop (kind 0: ds_read_b128, kind 1: ds_read_b64_tr_b16), by default one
    work-group per CU, and returns a dict: LDS read bandwidth in bytes per shader clock and CU as
    seen by the first wave's own clock, and the aggregate rate in TB/s from the launch time."""
    out = torch.zeros(4, dtype=torch.int64, device="cuda")
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    s = torch.cuda.current_stream() if stream is None else stream
    _check(_lib.attn_probe_lds_clock(ctypes.c_void_p(out.data_ptr()), int(kind), 1, 1, _stream(stream)))
    e0.record(s)
    _check(_lib.attn_probe_lds_clock(ctypes.c_void_p(out.data_ptr()), int(kind), int(workgroups), int(iters), _stream(stream)))
    e1.record(s)
    e1.synchronize()
    ms = e0.elapsed_time(e1)
    cyc, ticks = out[0].item(), out[1].item()
    per_wg = 4 * 16 * float(iters) * (1024.0 if kind == 0 else 512.0)
    return {"bytes_per_clk_per_cu": per_wg / cyc if cyc else float("nan"),
            "shader_clock_ghz": cyc / (ticks / 1e8) / 1e9 if ticks else float("nan"),
            "ms": ms, "TB/s": per_wg * workgroups / (ms * 1e-3) / 1e12}
