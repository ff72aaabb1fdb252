"""ctypes binding of libkvfuse_probe.so (include/kvfuse_probe.h): machine probes for benchmarks.  Not part of the
hot path and not part of the method's interface; bench.py and one GPU test use it."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvfuse_probe.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_03067_amd.build` (needs hipcc)")
lib = C.CDLL(LIB_PATH)

EXPORTS = ["kvfuse_probe_last_error", "kvfuse_probe_mfma_bf16", "kvfuse_probe_copy", "kvfuse_probe_tile_loop_bf16",
           "kvfuse_probe_read2_write1"]
SCRATCH_BYTES = 65792
_vp, _i32 = C.c_void_p, C.c_int32
lib.kvfuse_probe_last_error.restype = C.c_char_p
lib.kvfuse_probe_mfma_bf16.argtypes = [_vp, _i32, _vp, C.c_size_t, C.POINTER(C.c_double)]
lib.kvfuse_probe_mfma_fp8.argtypes = [_vp, _i32, _vp, C.c_size_t, C.POINTER(C.c_double)]
lib.kvfuse_probe_copy.argtypes = [_vp, _vp, _vp, C.c_size_t, _i32, C.POINTER(C.c_double)]
lib.kvfuse_probe_tile_loop_bf16.argtypes = [_vp, _vp, C.c_size_t, _i32, _vp, C.POINTER(C.c_double)]
lib.kvfuse_probe_read2_write1.argtypes = [_vp, _vp, C.c_size_t, _i32, _i32, C.POINTER(C.c_double)]


class ProbeError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"kvfuse_probe error {code}: {text}")
        self.code = code


def _check(rc):
    if rc:
        raise ProbeError(rc, lib.kvfuse_probe_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(device):
    return C.c_void_p(torch.cuda.current_stream(torch.device(device)).cuda_stream)


def mfma_bf16(random_operands=True, device="cuda:0"):
    """Sustained bfloat16 MFMA rate of the whole GPU in TFLOP/s (operands in registers, no memory traffic)."""
    scratch = torch.empty(SCRATCH_BYTES, device=device, dtype=torch.uint8)
    out = C.c_double(0.0)
    _check(lib.kvfuse_probe_mfma_bf16(_stream(device), 1 if random_operands else 0, _ptr(scratch), scratch.numel(), C.byref(out)))
    return out.value


def mfma_fp8(random_operands=True, device="cuda:0"):
    """Sustained rate of the fp8 (e4m3) 32 x 32 x 64 MFMA of the whole GPU in TFLOP/s (operands in registers)."""
    scratch = torch.empty(SCRATCH_BYTES, device=device, dtype=torch.uint8)
    out = C.c_double(0.0)
    _check(lib.kvfuse_probe_mfma_fp8(_stream(device), 1 if random_operands else 0, _ptr(scratch), scratch.numel(), C.byref(out)))
    return out.value


def copy(src, dst, repeats=3):
    """Read + write GB/s of a plain device copy kernel from src to dst (same size, contiguous)."""
    assert src.is_contiguous() and dst.is_contiguous() and src.numel() * src.element_size() == dst.numel() * dst.element_size()
    out = C.c_double(0.0)
    _check(lib.kvfuse_probe_copy(_stream(src.device), _ptr(src), _ptr(dst), src.numel() * src.element_size(), repeats, C.byref(out)))
    return out.value


def tile_loop_bf16(src, with_loads=True):
    """TFLOP/s of the similarity kernel's stripped inner loop, LDS operands and loads taken from ``src`` (>= 4 MiB)."""
    assert src.is_contiguous()
    sink = torch.zeros(1, device=src.device, dtype=torch.float32)
    out = C.c_double(0.0)
    _check(lib.kvfuse_probe_tile_loop_bf16(_stream(src.device), _ptr(src), src.numel() * src.element_size(),
                                           1 if with_loads else 0, _ptr(sink), C.byref(out)))
    return out.value


def read2_write1(buf, block_bytes, repeats=3):
    """GB/s (read + written) of the merge step's access pattern on ``buf`` (overwritten)."""
    assert buf.is_contiguous()
    out = C.c_double(0.0)
    _check(lib.kvfuse_probe_read2_write1(_stream(buf.device), _ptr(buf), buf.numel() * buf.element_size(), int(block_bytes),
                                         repeats, C.byref(out)))
    return out.value
