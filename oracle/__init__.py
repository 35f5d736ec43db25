"""Python access to the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It compiles `dconv_oracle.c` with gcc into
`libdconv_oracle.so` beside the source and calls it through ctypes on host
(numpy) arrays.  It never touches HIP and imports nothing from the GPU
package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "dconv_oracle.c"
_LIB = _HERE / "libdconv_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
             "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"],
            check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.dconv_oracle_general.argtypes = [p, i64, i64, i64, i64, p, i64, i64, p, p, p,
                                             ctypes.c_int, p]
        lib.dconv_oracle_general.restype = ctypes.c_int
        lib.dconv_oracle_single_channel.argtypes = [p, i64, i64, p, i64, i64, p, p, p,
                                                    ctypes.c_int, p]
        lib.dconv_oracle_single_channel.restype = ctypes.c_int
        lib.dconv_oracle_general_at.argtypes = [p, i64, i64, i64, i64, p, i64, i64, p, i64, p, p]
        lib.dconv_oracle_general_at.restype = ctypes.c_int
        lib.dconv_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs must be float32")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().dconv_oracle_max_threads())


def general(x, filt, threads: int = 0, want32: bool = False):
    """out[n,k,y,x] = sum_{c,i,j} in[n,c,y+i,x+j] * filt[k,c,i,j] in fp64.

    Returns (acc64, mag64[, out32]) and the number of threads used as the
    last item.
    """
    x, filt = _f32(x), _f32(filt)
    N, C, H, W = x.shape
    K, C2, F, F2 = filt.shape
    if C2 != C or F2 != F:
        raise ValueError("filter shape does not match input")
    Ho, Wo = H - F + 1, W - F + 1
    if Ho <= 0 or Wo <= 0:
        raise ValueError("filter larger than image")
    acc = np.empty((N, K, Ho, Wo), np.float64)
    mag = np.empty((N, K, Ho, Wo), np.float64)
    o32 = np.empty((N, K, Ho, Wo), np.float32) if want32 else None
    used = ctypes.c_int(0)
    rc = _load().dconv_oracle_general(_ptr(x), N, C, H, W, _ptr(filt), K, F,
                                      _ptr(o32), _ptr(acc), _ptr(mag),
                                      threads, ctypes.byref(used))
    if rc != 0:
        raise RuntimeError(f"oracle rejected the arguments (code {rc})")
    return (acc, mag, o32, used.value) if want32 else (acc, mag, used.value)


def single_channel(img, filt, threads: int = 0, only32: bool = False):
    """out[k,y,x] = sum_{i,j} img[y+i,x+j] * filt[k,i,j] in fp64 -> (acc64, mag64, threads).

    With only32=True the fp64 sums are rounded to float32 and only that array
    is produced: (out32, threads).  Used to time the oracle on large inputs
    without the two fp64 result arrays.
    """
    img, filt = _f32(img), _f32(filt)
    H, W = img.shape
    K, F, F2 = filt.shape
    if F2 != F:
        raise ValueError("filters must be square")
    Ho, Wo = H - F + 1, W - F + 1
    if Ho <= 0 or Wo <= 0:
        raise ValueError("filter larger than image")
    used = ctypes.c_int(0)
    if only32:
        o32 = np.empty((K, Ho, Wo), np.float32)
        acc = mag = None
    else:
        o32 = None
        acc = np.empty((K, Ho, Wo), np.float64)
        mag = np.empty((K, Ho, Wo), np.float64)
    rc = _load().dconv_oracle_single_channel(_ptr(img), H, W, _ptr(filt), K, F,
                                             _ptr(o32), _ptr(acc), _ptr(mag),
                                             threads, ctypes.byref(used))
    if rc != 0:
        raise RuntimeError(f"oracle rejected the arguments (code {rc})")
    if only32:
        return o32, used.value
    return acc, mag, used.value


def general_at(x, filt, flat_idx):
    """The same sums for the listed flat output indices only -> (acc64, mag64)."""
    x, filt = _f32(x), _f32(filt)
    N, C, H, W = x.shape
    K, C2, F, F2 = filt.shape
    if C2 != C or F2 != F:
        raise ValueError("filter shape does not match input")
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    acc = np.empty(idx.shape, np.float64)
    mag = np.empty(idx.shape, np.float64)
    rc = _load().dconv_oracle_general_at(_ptr(x), N, C, H, W, _ptr(filt), K, F,
                                         _ptr(idx), idx.size, _ptr(acc), _ptr(mag))
    if rc != 0:
        raise RuntimeError(f"oracle rejected the arguments (code {rc})")
    return acc, mag
