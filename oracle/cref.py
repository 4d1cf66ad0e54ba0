"""ctypes access to the plain-C oracle twin (oracle/qadc_ref.c) -- TEST INFRASTRUCTURE.

`build()` compiles the C file with gcc; `lib()` loads it.  Array arguments are
NumPy arrays on the host.  Nothing here touches the HIP library.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qadc_ref.c")
_SO = os.path.join(_HERE, "libqadc_ref.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)  # compiles when the library is missing or older than its source
        _lib = ctypes.CDLL(_SO)
        _lib.ref_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().ref_num_threads())


def pq_encode(x, codebooks):
    """Section 2.1 encode; returns packed nibbles [n][m/2] for k=16, bytes [n][m] for k=256."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    cb = np.ascontiguousarray(codebooks, dtype=np.float32)
    m, k, dsub = cb.shape
    n, d = x.shape
    assert d == m * dsub and k in (16, 256)
    codes = np.zeros((n, m // 2 if k == 16 else m), dtype=np.uint8)
    lib().ref_pq_encode(_p(x), ctypes.c_int64(n), d, m, k, _p(cb), _p(codes))
    return codes


def scan_u8(codes, qlut, cap=255):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    qlut = np.ascontiguousarray(qlut, dtype=np.uint8)
    m = qlut.shape[0]
    assert codes.shape[1] == m // 2 and qlut.shape[1] == 16
    out = np.empty(len(codes), dtype=np.uint8)
    lib().ref_scan_u8(_p(codes), ctypes.c_int64(len(codes)), m, _p(qlut), cap, _p(out))
    return out


def adc_f32(codes, lut):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    m, k = lut.shape
    assert codes.shape[1] == (m // 2 if k == 16 else m)
    out = np.empty(len(codes), dtype=np.float32)
    lib().ref_adc_f32(_p(codes), ctypes.c_int64(len(codes)), m, k, _p(lut), _p(out))
    return out


def scan_topk_u8(codes, qluts, R, cap=255):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    qluts = np.ascontiguousarray(qluts, dtype=np.uint8)
    nq, m, k = qluts.shape
    assert k == 16 and codes.shape[1] == m // 2
    idx = np.empty((nq, R), dtype=np.uint32)
    dist = np.empty((nq, R), dtype=np.uint8)
    lib().ref_scan_topk_u8(_p(codes), ctypes.c_int64(len(codes)), m, _p(qluts), nq, cap, R,
                           _p(idx), _p(dist))
    return idx, dist


def scan_topk_u8_bytes(codes, qluts, R, cap=255):
    """8-bit codes uint8 [n][m], quantized tables uint8 [nq][m][256] -> (idx, dist)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    qluts = np.ascontiguousarray(qluts, dtype=np.uint8)
    nq, m, k = qluts.shape
    assert k == 256 and codes.shape[1] == m
    idx = np.empty((nq, R), dtype=np.uint32)
    dist = np.empty((nq, R), dtype=np.uint8)
    lib().ref_scan_topk_u8_bytes(_p(codes), ctypes.c_int64(len(codes)), m, _p(qluts), nq, cap, R,
                                 _p(idx), _p(dist))
    return idx, dist


def scan_topk_u8_sixbit(codes, qluts, R, cap=255):
    """6-bit codes uint8 [n][3m/4], quantized tables uint8 [nq][m][64] -> (idx, dist)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    qluts = np.ascontiguousarray(qluts, dtype=np.uint8)
    nq, m, k = qluts.shape
    assert k == 64 and codes.shape[1] == 3 * m // 4
    idx = np.empty((nq, R), dtype=np.uint32)
    dist = np.empty((nq, R), dtype=np.uint8)
    lib().ref_scan_topk_u8_sixbit(_p(codes), ctypes.c_int64(len(codes)), m, _p(qluts), nq, cap, R,
                                  _p(idx), _p(dist))
    return idx, dist


def scan_topk_f32(codes, luts, R):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    luts = np.ascontiguousarray(luts, dtype=np.float32)
    nq, m, k = luts.shape
    assert codes.shape[1] == (m // 2 if k == 16 else m)
    idx = np.empty((nq, R), dtype=np.uint32)
    dist = np.empty((nq, R), dtype=np.float32)
    lib().ref_scan_topk_f32(_p(codes), ctypes.c_int64(len(codes)), m, k, _p(luts), nq, R,
                            _p(idx), _p(dist))
    return idx, dist


if __name__ == "__main__":
    print(build())
