"""CPU oracle for masked multi-head attention -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP library and never imports it.

  attention.c   fp64 two-pass masked softmax attention over the dense mask
  formats.py    per-row (CSR) and block (BSR + bitmap) formats from a dense mask
  selector.py   the paper's kernel-selection formula (Eq. 1)
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile attention.c with gcc into liboracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_masked_attention.argtypes = [u16p, u16p, u16p, ctypes.c_int, u8p, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_double, f64p]
        lib.oracle_masked_attention.restype = ctypes.c_int
        lib.oracle_masked_attention_rect.argtypes = [u16p, u16p, u16p, ctypes.c_int, u8p, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_double, f64p]
        lib.oracle_masked_attention_rect.restype = ctypes.c_int
        lib.oracle_row_probs.argtypes = [u16p, u16p, u16p, ctypes.c_int, u8p, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, f64p, f64p]
        lib.oracle_row_probs.restype = ctypes.c_int
        lib.oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
        lib.oracle_f16_to_f64.restype = ctypes.c_double
        lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        lib.oracle_bf16_to_f64.restype = ctypes.c_double
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _check(Q, K, V, mask):
    for a in (Q, K, V):
        assert a.dtype == np.uint16 and a.ndim == 4 and a.flags.c_contiguous
    assert K.shape == V.shape and Q.shape[:2] == K.shape[:2] and Q.shape[3] == K.shape[3]
    assert mask.dtype == np.uint8 and mask.ndim == 4 and mask.flags.c_contiguous
    B, H, Sq, d = Q.shape
    Sk = K.shape[2]
    Bm, Hm = mask.shape[:2]
    assert mask.shape[2:] == (Sq, Sk)
    return B, H, Sq, Sk, d, Bm, Hm


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def masked_attention(Q, K, V, dtype: str, mask, scale: float | None = None) -> np.ndarray:
    """Q: uint16 bit patterns [B,H,Sq,d] ('f16' | 'bf16'); K, V: [B,H,Sk,d]; mask uint8
    [Bm,Hm,Sq,Sk]; returns float64 [B,H,Sq,d].  Sq = Sk is self-attention."""
    B, H, Sq, Sk, d, Bm, Hm = _check(Q, K, V, mask)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    O = np.empty((B, H, Sq, d), dtype=np.float64)
    rc = _load().oracle_masked_attention_rect(_p(Q, ctypes.c_uint16), _p(K, ctypes.c_uint16),
                                              _p(V, ctypes.c_uint16), 0 if dtype == "f16" else 1,
                                              _p(mask, ctypes.c_uint8), Bm, Hm, B, H, Sq, Sk, d,
                                              float(scale), _p(O, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("oracle_masked_attention_rect failed")
    return O


def row_probs(Q, K, V, dtype: str, mask, b: int, h: int, i: int, scale: float | None = None):
    """(probabilities[S], output[d]) of one query row, for invariant checks."""
    B, H, S, Sk, d, Bm, Hm = _check(Q, K, V, mask)
    assert S == Sk
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    probs = np.empty(S, dtype=np.float64)
    out = np.empty(d, dtype=np.float64)
    rc = _load().oracle_row_probs(_p(Q, ctypes.c_uint16), _p(K, ctypes.c_uint16),
                                  _p(V, ctypes.c_uint16), 0 if dtype == "f16" else 1,
                                  _p(mask, ctypes.c_uint8), Bm, Hm, B, H, S, d, float(scale),
                                  b, h, i, _p(probs, ctypes.c_double), _p(out, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("oracle_row_probs failed")
    return probs, out


def f16_to_f64(bits: int) -> float:
    return float(_load().oracle_f16_to_f64(int(bits)))


def bf16_to_f64(bits: int) -> float:
    return float(_load().oracle_bf16_to_f64(int(bits)))
