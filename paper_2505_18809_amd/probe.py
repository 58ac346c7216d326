"""ctypes binding of libvorta_probe.so, a measurement aid that only the benchmark loads: the
rate the chip sustains for a bf16 matrix instruction alone, per operand distribution, per
instruction shape and per number of vector instructions issued next to it.  Not part of the
attention path or of libvorta's ABI."""
import ctypes
import os

import torch

PROBE_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvorta_probe.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(PROBE_LIB_PATH)
        _lib.mfma_probe_rate.restype = ctypes.c_int
    return _lib


def mfma_probe_rate(operands: torch.Tensor, iters: int, workgroups: int, shape: int = 32, vector_ops: int = 0,
                    stream=None):
    """shape 32: v_mfma_f32_32x32x16_bf16, 16: v_mfma_f32_16x16x32_bf16; vector_ops (0, 2, 3, 4):
    v_fma_f32 per 16 cycles of matrix-pipe time issued behind each matrix instruction.
    Returns (FLOPs issued, sink, clocks); the caller times the call with events."""
    assert operands.is_cuda and operands.is_contiguous()
    assert operands.numel() * operands.element_size() >= 16 * 64 * 16
    sink = torch.empty(workgroups * 512, dtype=torch.float32, device=operands.device)
    clocks = torch.zeros(2, dtype=torch.int64, device=operands.device)
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = _load().mfma_probe_rate(ctypes.c_void_p(operands.data_ptr()), iters, workgroups, shape, vector_ops,
                                 ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(clocks.data_ptr()),
                                 ctypes.c_void_p(st.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"mfma_probe_rate failed with code {rc}")
    return workgroups * 8 * iters * float(1 << 20), sink, clocks
