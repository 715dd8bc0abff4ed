"""ctypes loader of the oracle's plain C routines (oracle/native/oracle_kernels.c).

Test infrastructure only (see the package header of ``oracle``).  The C file holds scalar-loop versions
of three bit-spec routines -- the 8-bit cast, the estimator written as a packed operand, and the
packed -> dense decode -- for the parity tests at the full workload sizes.  The numpy forms in
``oracle.formats`` / ``oracle.mvue`` / ``oracle.projection`` remain the reference; these are checked
against them element for element in ``tests/test_oracle_native.py``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_kernels.c")
_LIB = os.path.join(_HERE, "liboracle_kernels.so")
_lib = None

_FMT = {"bf16": 0, "e4m3": 1, "e5m2": 3}


def build(verbose: bool = False) -> str:
    """Compiles the C file with gcc (no fused multiply-add, OpenMP over the outer loops)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp", _SRC, "-lm", "-o", _LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return _LIB


def _library():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build()
        lib = ctypes.CDLL(_LIB)
        vp, i64, u64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
        lib.orc_cast_fp8.argtypes = [vp, i64, ctypes.c_float, ci, vp, vp]
        lib.orc_cast_fp8.restype = None
        lib.orc_mvue_pack.argtypes = [vp, i64, i64, ci, u64, u64, u64, vp, vp]
        lib.orc_mvue_pack.restype = None
        lib.orc_decode_packed.argtypes = [vp, vp, i64, i64, ci, vp]
        lib.orc_decode_packed.restype = None
        _lib = lib
    return _lib


def cast_fp8(x_bits, scale, fmt="e4m3"):
    """As ``oracle.formats.cast_fp8``: (codes uint8 of x's shape, amax float32)."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    codes = np.empty(x.shape, dtype=np.uint8)
    amax = np.zeros(1, dtype=np.float32)
    _library().orc_cast_fp8(x.ctypes.data, x.size, float(np.float32(scale)), _FMT[fmt], codes.ctypes.data, amax.ctypes.data)
    return codes, np.float32(amax[0])


def mvue_pack(dy_codes, seed, offset, dtype="bf16", first_group=0):
    """As ``oracle.mvue.mvue_pack``: vals (O, T/2), meta (O, T/8)."""
    dy = np.ascontiguousarray(dy_codes, dtype=np.uint16 if dtype == "bf16" else np.uint8)
    T, O = dy.shape
    if T % 8 != 0:
        raise ValueError("T must be a multiple of 8 (two groups per metadata byte)")
    vals = np.empty((O, T // 2), dtype=dy.dtype)
    meta = np.empty((O, T // 8), dtype=np.uint8)
    _library().orc_mvue_pack(dy.ctypes.data, T, O, _FMT[dtype], int(seed) & (2 ** 64 - 1), int(offset) & (2 ** 64 - 1),
                             int(first_group), vals.ctypes.data, meta.ctypes.data)
    return vals, meta


def decode_packed(vals, meta, val_dtype="bf16"):
    """As ``oracle.projection.decode_packed``: dense-with-zeros float64 (R, K)."""
    vals = np.ascontiguousarray(vals, dtype=np.uint16 if val_dtype == "bf16" else np.uint8)
    meta = np.ascontiguousarray(meta, dtype=np.uint8)
    R, half = vals.shape
    dense = np.empty((R, 2 * half), dtype=np.float64)
    _library().orc_decode_packed(vals.ctypes.data, meta.ctypes.data, R, 2 * half, _FMT[val_dtype], dense.ctypes.data)
    return dense
