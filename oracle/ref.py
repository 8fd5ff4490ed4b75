"""ctypes front end of the C oracle (``moe_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Takes NumPy arrays, returns NumPy arrays.  Activations and the gate matrix are
passed as float32 values (bf16-stored inputs are widened by the caller, which is
exact); expert weights are passed either as float32 arrays or as raw bfloat16
bit patterns (uint16), and are widened element by element inside the C code.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-std=c11", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().ko_num_threads())


def vector_width(dtype: str) -> int:
    """Elements per 16-byte vector of the storage type (part of the logit order)."""
    return 4 if dtype == "f32" else 8


def gate_logits_f32(x, wg, V: int) -> np.ndarray:
    x, wg = _f32(x), _f32(wg)
    N, d = x.shape
    E = wg.shape[0]
    out = np.empty((N, E), dtype=np.float32)
    lib().ko_gate_logits_f32(_p(x, C.c_float), _p(wg, C.c_float), N, d, E, V, _p(out, C.c_float))
    return out


def gate_logits_f64(x, wg) -> np.ndarray:
    x, wg = _f32(x), _f32(wg)
    N, d = x.shape
    E = wg.shape[0]
    out = np.empty((N, E), dtype=np.float64)
    lib().ko_gate_logits_f64(_p(x, C.c_float), _p(wg, C.c_float), N, d, E, _p(out, C.c_double))
    return out


def topk(logits, k: int) -> np.ndarray:
    logits = _f32(logits)
    N, E = logits.shape
    idx = np.empty((N, k), dtype=np.int32)
    lib().ko_topk(_p(logits, C.c_float), N, E, k, _p(idx, C.c_int32))
    return idx


def gate_weights(logits, idx, renorm: bool = True) -> np.ndarray:
    logits, idx = _f32(logits), _i32(idx)
    N, E = logits.shape
    k = idx.shape[1]
    w = np.empty((N, k), dtype=np.float64)
    lib().ko_gate_weights(_p(logits, C.c_float), _p(idx, C.c_int32), N, E, k, int(renorm),
                          _p(w, C.c_double))
    return w


@dataclass
class Dispatch:
    counts: np.ndarray
    offsets: np.ndarray
    perm: np.ndarray
    inv_perm: np.ndarray
    nbatch: np.ndarray
    exec_order: np.ndarray
    n_active: int


def dispatch(idx, E: int, batch_offsets) -> Dispatch:
    idx = _i32(idx)
    N, k = idx.shape
    bo = _i32(batch_offsets)
    B = bo.shape[0] - 1
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(N * k, np.int32)
    inv_perm = np.empty(N * k, np.int32)
    nbatch = np.empty(E, np.int32)
    order = np.empty(E, np.int32)
    n_active = C.c_int32(0)
    lib().ko_dispatch(_p(idx, C.c_int32), N, k, E, _p(bo, C.c_int32), B, _p(counts, C.c_int32),
                      _p(offsets, C.c_int32), _p(perm, C.c_int32), _p(inv_perm, C.c_int32),
                      _p(nbatch, C.c_int32), _p(order, C.c_int32), C.byref(n_active))
    return Dispatch(counts, offsets, perm, inv_perm, nbatch, order, int(n_active.value))


def _wtype(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    if a.dtype == np.float64:
        return 2
    raise TypeError(f"expert weights must be float32, float64 or uint16 (bf16 bits), got {a.dtype}")


def expert_ffn(x, w1, w3, w2) -> np.ndarray:
    """One SwiGLU expert on one token, fp64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w1, w3, w2 = (np.ascontiguousarray(a) for a in (w1, w3, w2))
    wt = _wtype(w1)
    f, d = w1.shape
    assert w3.shape == (f, d) and w2.shape == (d, f) and x.shape == (d,)
    out = np.empty(d, dtype=np.float64)
    lib().ko_expert_ffn(_p(x, C.c_double), C.c_void_p(w1.ctypes.data), C.c_void_p(w3.ctypes.data),
                        C.c_void_p(w2.ctypes.data), wt, d, f, _p(out, C.c_double))
    return out


def moe_forward(x, idx, w, w1: Sequence[np.ndarray], w3: Sequence[np.ndarray],
                w2: Sequence[np.ndarray], n_experts: int, n_shared: int = 0,
                tokens: Optional[Sequence[int]] = None, expert_kind: int = 0) -> np.ndarray:
    """Layer output (fp64) for ``tokens`` (default: all).  Weight lists hold E+S arrays."""
    x, idx = _f32(x), _i32(idx)
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, d = x.shape
    k = idx.shape[1]
    if expert_kind == 0:
        w1 = [np.ascontiguousarray(a) for a in w1]
        w3 = [np.ascontiguousarray(a) for a in w3]
        w2 = [np.ascontiguousarray(a) for a in w2]
        assert len(w1) == len(w3) == len(w2) == n_experts + n_shared
        wt = _wtype(w1[0])
        f = w1[0].shape[0]
        for a, b, c in zip(w1, w3, w2):
            assert a.shape == (f, d) and b.shape == (f, d) and c.shape == (d, f)
            assert _wtype(a) == wt and _wtype(b) == wt and _wtype(c) == wt
        arr = C.c_void_p * len(w1)
        p1 = arr(*[a.ctypes.data for a in w1])
        p3 = arr(*[a.ctypes.data for a in w3])
        p2 = arr(*[a.ctypes.data for a in w2])
    else:
        wt, f = 0, 0
        p1 = p3 = p2 = None
    if tokens is None:
        sel, n_sel, selp = None, N, None
    else:
        sel = _i32(tokens)
        n_sel = sel.shape[0]
        selp = _p(sel, C.c_int32)
    y = np.empty((n_sel, d), dtype=np.float64)
    lib().ko_moe_forward(_p(x, C.c_float), _p(idx, C.c_int32), _p(w, C.c_double), d, f,
                         n_experts, k, n_shared, p1, p3, p2, wt, expert_kind, selp, n_sel,
                         _p(y, C.c_double))
    return y


@dataclass
class LayerRef:
    logits: np.ndarray
    idx: np.ndarray
    w: np.ndarray
    disp: Dispatch
    y: Optional[np.ndarray]
    tokens: Optional[np.ndarray]


def moe_layer(x, wg, w1, w3, w2, k: int, batch_offsets, dtype: str, n_shared: int = 0,
              tokens: Optional[Sequence[int]] = None, renorm: bool = True,
              with_output: bool = True) -> LayerRef:
    """Whole layer: logits -> top-k -> weights -> dispatch arrays -> outputs."""
    E = np.asarray(wg).shape[0]
    logits = gate_logits_f32(x, wg, vector_width(dtype))
    idx = topk(logits, k)
    w = gate_weights(logits, idx, renorm)
    disp = dispatch(idx, E, batch_offsets)
    y = None
    if with_output:
        y = moe_forward(x, idx, w, w1, w3, w2, E, n_shared, tokens)
    return LayerRef(logits, idx, w, disp, y, None if tokens is None else _i32(tokens))


def round_bf16(x: float) -> float:
    lib().ko_round_bf16.restype = C.c_double
    lib().ko_round_bf16.argtypes = [C.c_double]
    return float(lib().ko_round_bf16(float(x)))


def dequant_q4(q, s_bits, z_bits, group: int = 64, to_bf16: bool = False) -> np.ndarray:
    """fp64 weights s * (code - z) of a [rows, cols/2] uint8 code array (Eq. 8); with
    ``to_bf16`` each is then rounded to bfloat16, the model's original precision."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    s_bits = np.ascontiguousarray(s_bits, dtype=np.uint16)
    z_bits = np.ascontiguousarray(z_bits, dtype=np.uint16)
    rows, cols = q.shape[0], q.shape[1] * 2
    assert cols % group == 0 and s_bits.shape == z_bits.shape == (rows, cols // group)
    out = np.empty((rows, cols), dtype=np.float64)
    lib().ko_dequant_q4(_p(q, C.c_uint8), _p(s_bits, C.c_uint16), _p(z_bits, C.c_uint16), rows, cols,
                        group, int(to_bf16), _p(out, C.c_double))
    return out


def quant_q4(w, s_bits, z_bits, group: int = 64) -> np.ndarray:
    """4-bit codes round(w / s + z), clamped, packed two per byte (Eq. 8)."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    s_bits = np.ascontiguousarray(s_bits, dtype=np.uint16)
    z_bits = np.ascontiguousarray(z_bits, dtype=np.uint16)
    rows, cols = w.shape
    q = np.empty((rows, cols // 2), dtype=np.uint8)
    lib().ko_quant_q4(_p(w, C.c_double), _p(s_bits, C.c_uint16), _p(z_bits, C.c_uint16), rows, cols,
                      group, _p(q, C.c_uint8))
    return q


def corr_update(table: np.ndarray, idx_prev, idx_cur) -> np.ndarray:
    """Add one layer transition of a batch group to an [E, E] int64 correlation table (in place)."""
    ip, ic = _i32(idx_prev), _i32(idx_cur)
    assert ip.shape == ic.shape and table.dtype == np.int64 and table.flags.c_contiguous
    N, k = ip.shape
    lib().ko_corr_update(_p(ip, C.c_int32), _p(ic, C.c_int32), N, k, table.shape[0],
                         _p(table, C.c_int64))
    return table


def corr_predict(table: np.ndarray, counts_prev, K: int):
    """(experts to prefetch, fp64 scores) for the next layer from the previous layer's counts."""
    E = table.shape[0]
    cp = _i32(counts_prev)
    score = np.zeros(E, dtype=np.float64)
    experts = np.full(max(1, K), -1, dtype=np.int32)
    n = C.c_int32(0)
    lib().ko_corr_predict(_p(np.ascontiguousarray(table), C.c_int64), _p(cp, C.c_int32), E, K,
                          _p(score, C.c_double), _p(experts, C.c_int32), C.byref(n))
    return experts[:n.value].copy(), score


def plan_batches(t_c_A, t_c_G, t_c_hotE, t_c_E, t_io_A, t_io_G, t_io_E, K: int,
                 n_max: int = 10_000_000) -> int:
    """Smallest n of the planner's inequality group by trying n = 1, 2, ...; -1 if none <= n_max."""
    q = np.ascontiguousarray(np.asarray(list(t_c_E), dtype=np.float64))
    fn = lib().ko_plan_batches
    fn.restype = C.c_int64
    fn.argtypes = [C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double), C.c_int, C.c_double,
                   C.c_double, C.c_double, C.c_int, C.c_int64]
    buf = q if q.size else np.zeros(1)
    return int(fn(t_c_A, t_c_G, t_c_hotE, _p(buf, C.c_double), int(q.size), t_io_A, t_io_G, t_io_E, K, n_max))
