"""Binding of libskv_calib.so, the benchmark's measurement aid (include/skv_calib.h): back-to-back
MFMAs with and without the side work of an attention tile.  No part of the attention path and not
imported by the package; bench.py and its test load it."""
from __future__ import annotations

import ctypes
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libskv_calib.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from .build import build_library
            build_library()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.skv_calib_mfma_bf16.restype = ctypes.c_int32
        _lib.skv_calib_mfma_mix_bf16.restype = ctypes.c_int32
    return _lib


def _args(operands, sink, blocks, stream):
    if operands.numel() * operands.element_size() < 16384 or sink.numel() < blocks * 256 or sink.dtype != torch.float32:
        raise ValueError("operands need 16 KiB, sink blocks * 256 floats")
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(operands.data_ptr()), ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(stream)


def skv_calib_mfma_bf16(operands, sink, blocks: int, iters: int, stream=None):
    """operands: 16 KiB device tensor; sink: float32 device tensor of blocks * 256 elements."""
    o, s, st = _args(operands, sink, blocks, stream)
    rc = lib().skv_calib_mfma_bf16(o, s, blocks, iters, st)
    if rc:
        raise RuntimeError(f"skv_calib_mfma_bf16: status {rc}")


def skv_calib_mfma_mix_bf16(operands, sink, blocks: int, iters: int, mix: int, stream=None):
    """mix bit 0: four vector instructions per MFMA; bit 1: LDS operand reads at the pre-fill kernel's rate."""
    o, s, st = _args(operands, sink, blocks, stream)
    rc = lib().skv_calib_mfma_mix_bf16(o, s, blocks, iters, mix, st)
    if rc:
        raise RuntimeError(f"skv_calib_mfma_mix_bf16: status {rc}")
