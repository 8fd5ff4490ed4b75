"""ctypes front end of the attention-layer oracle (``attn_oracle.c``).  TEST INFRASTRUCTURE ONLY.

NumPy in, NumPy out.  Activations are float32 values (bf16-stored inputs are widened by the
caller, exactly); weights are float32 / float64 arrays or raw bfloat16 bit patterns (uint16);
the key-value caches are bfloat16 bit patterns laid out [n_seq, Hkv, max_len, hd].
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "libattn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ka_bf16_bits.restype = C.c_uint16
        _lib.ka_bf16_bits.argtypes = [C.c_double]
    return _lib


def _wtype(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float64:
        return 2
    raise TypeError(f"weights must be float32, float64 or uint16 (bf16 bits), got {a.dtype}")


def bf16_bits(x: float) -> int:
    """Bit pattern of the bfloat16 nearest to x (ties to even)."""
    return int(lib().ka_bf16_bits(float(x)))


def rmsnorm(x, g, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g)
    out = np.empty_like(x)
    lib().ka_rmsnorm(C.c_void_p(x.ctypes.data), C.c_void_p(g.ctypes.data), _wtype(g),
                     C.c_int(x.shape[0]), C.c_double(eps), C.c_void_p(out.ctypes.data))
    return out


def rope(v, pos: int, theta: float) -> np.ndarray:
    out = np.array(v, dtype=np.float64, copy=True)
    lib().ka_rope(C.c_void_p(out.ctypes.data), C.c_int(out.shape[0]), C.c_int(pos), C.c_double(theta))
    return out


def attn_decode(x, g, wq, wk, wv, wo, kc, vc, pos: int, n_q_heads: int, n_kv_heads: int,
                head_dim: int, theta: float, eps: float) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One decoding step for one batch.  Returns (y fp64 [n_seq, d], K cache, V cache); the
    caches are copies of the inputs with row ``pos`` filled in."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n_seq, d = x.shape
    ws = [np.ascontiguousarray(a) for a in (g, wq, wk, wv, wo)]
    wt = _wtype(ws[1])
    assert all(_wtype(a) == wt for a in ws)
    dq, dkv = n_q_heads * head_dim, n_kv_heads * head_dim
    assert ws[0].shape == (d,) and ws[1].shape == (dq, d) and ws[2].shape == (dkv, d)
    assert ws[3].shape == (dkv, d) and ws[4].shape == (d, dq)
    kc = np.array(kc, dtype=np.uint16, copy=True)
    vc = np.array(vc, dtype=np.uint16, copy=True)
    max_len = kc.shape[2]
    assert kc.shape == (n_seq, n_kv_heads, max_len, head_dim) and vc.shape == kc.shape
    assert 0 <= pos < max_len and n_q_heads % n_kv_heads == 0 and head_dim % 2 == 0
    y = np.empty((n_seq, d), dtype=np.float64)
    lib().ka_attn_decode(C.c_void_p(x.ctypes.data), C.c_int(n_seq), C.c_int(d), C.c_int(n_q_heads),
                         C.c_int(n_kv_heads), C.c_int(head_dim), *[C.c_void_p(a.ctypes.data) for a in ws],
                         C.c_int(wt), C.c_void_p(kc.ctypes.data), C.c_void_p(vc.ctypes.data),
                         C.c_int(max_len), C.c_int(pos), C.c_double(theta), C.c_double(eps),
                         C.c_void_p(y.ctypes.data))
    return y, kc, vc
