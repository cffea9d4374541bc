"""Loader of the C form of the oracle's definition (oracle/amla_oracle_decode.c).  TEST INFRASTRUCTURE ONLY.

`decode_c` has the arguments and results of `amla_oracle.decode` and calls `amla_oracle_decode` through
ctypes with host arrays.  The shared object is built next to the source by `build()` (plain gcc); loading
builds it when it is not there."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "amla_oracle_decode.c")
LIBRARY = os.path.join(HERE, "libamla_oracle.so")


class Shape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("s_q", ctypes.c_int32), ("num_heads", ctypes.c_int32),
                ("num_blocks", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("q_lens", ctypes.c_void_p)]


def build() -> str:
    subprocess.run(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", LIBRARY, SOURCE, "-lm"],
                   check=True)
    return LIBRARY


_lib = None


def library():
    global _lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            build()
        _lib = ctypes.CDLL(LIBRARY)
        _lib.amla_oracle_decode.restype = ctypes.c_int
        _lib.amla_oracle_decode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(Shape)]
    return _lib


def decode_c(q_bits, kv_bits, block_table, seqlens, softmax_scale, causal=False, q_lens=None):
    """out float64 [B, T, H, 512] (not rounded), lse float64 [B, T, H]; raises ValueError with the C status on
    an argument the C routine refuses."""
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    kv = np.ascontiguousarray(kv_bits, dtype=np.uint16)
    tab = np.ascontiguousarray(block_table, dtype=np.int32)
    lens = np.ascontiguousarray(seqlens, dtype=np.int32)
    B, T, H, D = q.shape
    assert D == 576 and kv.shape[1:] == (64, 576) and tab.shape[0] == B and lens.shape == (B,)
    ql = None if q_lens is None else np.ascontiguousarray(q_lens, dtype=np.int32)
    shape = Shape(B, T, H, kv.shape[0], tab.shape[1], int(bool(causal)), None if ql is None else ql.ctypes.data)
    out = np.full((B, T, H, 512), np.nan)
    lse = np.full((B, T, H), np.nan)
    status = library().amla_oracle_decode(q.ctypes.data, kv.ctypes.data, tab.ctypes.data, lens.ctypes.data,
                                          float(softmax_scale), out.ctypes.data, lse.ctypes.data, ctypes.byref(shape))
    if status != 0:
        raise ValueError(f"amla_oracle_decode returned {status}")
    return out, lse
