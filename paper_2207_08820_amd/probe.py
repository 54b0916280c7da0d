"""ctypes binding of the measurement probes (``csrc/probe.hip`` -> ``libdlrt_probe.so``).

Used by ``bench.py`` only: the probes measure, on the chip the benchmark runs on, the rates the kernels are
judged against (AND + popcount issue rate and the shader clock under that load, plain-copy HBM bandwidth, the
cost of an empty dependent launch).  Each call only enqueues on torch's current stream.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdlrt_probe.so")
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2207_08820_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int
        lib.dlrt_probe_valu.argtypes = [i32, i32, vp, vp, vp]
        lib.dlrt_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.dlrt_probe_gemm_clocks.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
        lib.dlrt_probe_empty.argtypes = [vp]
        _lib = lib
    return _lib


def _stream():
    return torch.cuda.current_stream().cuda_stream


def valu(blocks: int, iters: int, clocks: torch.Tensor, sink: torch.Tensor):
    """clocks: int64 [blocks, 2] (shader-clock cycles, constant-rate ticks of the loop); sink: int32 [blocks * 256]."""
    assert clocks.dtype == torch.int64 and clocks.numel() >= 2 * blocks and sink.dtype == torch.int32 and sink.numel() >= 256 * blocks
    if load().dlrt_probe_valu(blocks, iters, clocks.data_ptr(), sink.data_ptr(), _stream()):
        raise RuntimeError("dlrt_probe_valu: launch failed")


def gemm_clocks(A: torch.Tensor, W: torch.Tensor, C: torch.Tensor, M: int, N: int, K: int, abits: int, wbits: int,
                clocks: torch.Tensor):
    """The library's block kernel on packed A [M, abits, K/32], W [N, wbits, K/32] (unsigned activations, two's
    complement weights) with every block's lifetime on both counters in clocks (int64 [blocks, 2])."""
    rows, cols = (64 if abits <= 2 else 32), (64 if wbits <= 2 else 32)
    blocks = (M // rows) * (N // cols)
    assert A.dtype == torch.int32 and A.numel() >= M * abits * (K // 32) and W.dtype == torch.int32 and W.numel() >= N * wbits * (K // 32)
    assert C.dtype == torch.int32 and C.numel() >= M * N and clocks.dtype == torch.int64 and clocks.numel() >= 2 * blocks
    if load().dlrt_probe_gemm_clocks(A.data_ptr(), W.data_ptr(), C.data_ptr(), M, N, K, abits, wbits, clocks.data_ptr(), _stream()):
        raise RuntimeError("dlrt_probe_gemm_clocks: bad arguments or launch failed")
    return blocks


def copy(src: torch.Tensor, dst: torch.Tensor):
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes and nbytes % 16 == 0
    if load().dlrt_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()):
        raise RuntimeError("dlrt_probe_copy: launch failed")


def empty():
    if load().dlrt_probe_empty(_stream()):
        raise RuntimeError("dlrt_probe_empty: launch failed")


def wall_clock_khz() -> int:
    return int(load().dlrt_probe_wall_clock_khz())


def valu_ops_per_thread_iter() -> int:
    return int(load().dlrt_probe_valu_ops_per_thread_iter())
