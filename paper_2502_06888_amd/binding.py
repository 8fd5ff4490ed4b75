"""ctypes binding of the C-ABI library (``include/moe.h``).

Argument marshalling only: every step of the path runs in the HIP kernels behind the
library.  PyTorch tensors supply device memory and streams; their raw pointers are what
crosses the boundary.  There is no fallback: if the library is missing or cannot be
loaded, importing symbols from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libklotski_moe.so")

MOE_OK = 0
MOE_ERR_INVALID_ARG, MOE_ERR_SHAPE, MOE_ERR_STATE, MOE_ERR_OOM, MOE_ERR_NOT_PINNED, MOE_ERR_HIP = \
    1, 2, 3, 4, 5, 6
MOE_F32, MOE_BF16 = 0, 1
MOE_RESIDENT, MOE_HOST_PINNED = 0, 1
MOE_PREFETCH, MOE_ON_DEMAND = 1, 2
STATUS_NAMES = {0: "MOE_OK", 1: "MOE_ERR_INVALID_ARG", 2: "MOE_ERR_SHAPE", 3: "MOE_ERR_STATE",
                4: "MOE_ERR_OOM", 5: "MOE_ERR_NOT_PINNED", 6: "MOE_ERR_HIP"}

EXPORTS = ["moe_plan", "moe_plan_batches", "moe_create", "moe_destroy", "moe_set_gate",
           "moe_set_expert", "moe_route", "moe_route_wait", "moe_stream_experts",
           "moe_layer_forward", "moe_get_stats", "moe_reset_stats", "moe_set_tuning",
           "moe_set_profiling", "moe_get_profile", "moe_last_error", "moe_corr_enable",
           "moe_corr_reset", "moe_corr_predict", "moe_corr_table", "moe_corr_rank", "moe_measure", "moe_set_expert_q4",
           "moe_route_static"]


class MoeConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("d_model", "d_ff", "n_experts", "top_k", "n_shared", "n_layers", "window_layers",
                 "max_tokens", "max_batches", "dtype", "renormalize", "weight_bits")]


MOE_MAX_EXPERTS = 256


class MoeMeasured(C.Structure):
    _fields_ = [("t_c_gate_group_s", C.c_double), ("t_io_expert_s", C.c_double),
                ("t_c_gather_s", C.c_double), ("t_c_combine_s", C.c_double),
                ("t_c_expert_s", C.c_double * MOE_MAX_EXPERTS), ("n_active", C.c_int32),
                ("exec_order", C.c_int32 * MOE_MAX_EXPERTS), ("counts", C.c_int32 * MOE_MAX_EXPERTS)]


class MoePlan(C.Structure):
    _fields_ = [("workspace_bytes", C.c_int64), ("expert_bytes", C.c_int64),
                ("window_bytes", C.c_int64), ("n_slots", C.c_int32), ("reserved", C.c_int32),
                ("t_io_expert_s", C.c_double), ("t_c_expert_s", C.c_double),
                ("t_c_gate_s", C.c_double)]


class MoeStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("tokens", "bytes_h2d", "n_copies", "n_prefetch_hits", "n_prefetch_unused",
                 "n_forward", "n_active_sum", "h_saturated", "h_remainder_wgs", "copy_busy_ns", "compute_busy_ns",
                 "wall_ns")]


class MoeProfile(C.Structure):
    _fields_ = [(n, C.c_float) for n in
                ("router_ms", "plan_ms", "gather_ms", "up_ms", "down_ms", "combine_ms")]


class MoeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


_lib = None


def load_library():
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2502_06888_amd.build` "
                          "(hipcc, gfx950) first")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
    P = C.POINTER
    lib.moe_plan.argtypes = [P(MoeConfig), i32, dbl, dbl, dbl, P(MoePlan)]
    lib.moe_plan_batches.argtypes = [dbl, dbl, dbl, P(dbl), i32, dbl, dbl, dbl, i32, P(i32)]
    lib.moe_create.argtypes = [P(MoeConfig), vp, vp, vp, i64, vp, i64, P(vp)]
    lib.moe_destroy.argtypes = [vp]
    lib.moe_set_gate.argtypes = [vp, i32, vp]
    lib.moe_set_expert.argtypes = [vp, i32, i32, vp, vp, vp, i32, vp]
    lib.moe_set_expert_q4.argtypes = [vp, i32, i32] + [vp] * 9 + [i32, vp]
    lib.moe_route.argtypes = [vp, i32, vp, P(i32), i32] + [vp] * 8
    lib.moe_route_wait.argtypes = [vp, P(i32), P(i32), P(i32)]
    lib.moe_route_static.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, i32, P(i32), i32] + [vp] * 8
    lib.moe_stream_experts.argtypes = [vp, i32, P(i32), i32, i32]
    lib.moe_layer_forward.argtypes = [vp, i32, vp, vp]
    lib.moe_get_stats.argtypes = [vp, P(MoeStats)]
    lib.moe_reset_stats.argtypes = [vp]
    lib.moe_set_tuning.argtypes = [vp, i32, i32, i32]
    lib.moe_set_profiling.argtypes = [vp, i32]
    lib.moe_measure.argtypes = [vp, i32, vp, P(i32), i32, vp, i32, P(MoeMeasured)]
    lib.moe_corr_enable.argtypes = [vp, i32]
    lib.moe_corr_reset.argtypes = [vp]
    lib.moe_corr_predict.argtypes = [vp, i32, i32, P(i32), P(i32)]
    lib.moe_corr_table.argtypes = [vp, i32, P(i32)]
    lib.moe_corr_rank.argtypes = [P(i32), P(i32), i32, i32, P(i32), P(i32), P(dbl)]
    lib.moe_get_profile.argtypes = [vp, P(MoeProfile)]
    lib.moe_last_error.argtypes = [vp]
    lib.moe_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name != "moe_last_error":
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def corr_rank(table, counts_prev, K: int):
    """Pure host ranking of the correlation prefetcher: (expert ids, fp64 scores)."""
    E = len(counts_prev)
    flat = [int(v) for row in table for v in row]
    t = (C.c_int32 * (E * E))(*flat)
    cp = (C.c_int32 * E)(*[int(v) for v in counts_prev])
    out = (C.c_int32 * max(1, K))()
    n = C.c_int32(0)
    score = (C.c_double * E)()
    _check(load_library().moe_corr_rank(t, cp, E, K, out, C.byref(n), score))
    return [int(out[i]) for i in range(n.value)], [float(v) for v in score]


def _check(status: int, ctx=None):
    if status != MOE_OK:
        msg = load_library().moe_last_error(ctx)
        raise MoeError(status, msg.decode() if msg else "")


def make_config(d_model, d_ff, n_experts, top_k, n_shared=0, n_layers=1, window_layers=0,
                max_tokens=512, max_batches=64, dtype=MOE_BF16, renormalize=1,
                weight_bits=0) -> MoeConfig:
    return MoeConfig(d_model, d_ff, n_experts, top_k, n_shared, n_layers, window_layers,
                     max_tokens, max_batches, dtype, renormalize, weight_bits)


def moe_plan(cfg: MoeConfig, n_tokens: int, hbm_Bps: float = 8e12, link_Bps: float = 64e9,
             mfma_flops: float = 2.5e15) -> MoePlan:
    out = MoePlan()
    _check(load_library().moe_plan(C.byref(cfg), n_tokens, hbm_Bps, link_Bps, mfma_flops,
                                   C.byref(out)))
    return out


def moe_plan_batches(t_c_A, t_c_G, t_c_hotE, t_c_E: Sequence[float], t_io_A, t_io_G, t_io_E,
                     K: int) -> int:
    arr = (C.c_double * max(1, len(t_c_E)))(*t_c_E)
    n = C.c_int32(0)
    _check(load_library().moe_plan_batches(t_c_A, t_c_G, t_c_hotE, arr, len(t_c_E), t_io_A,
                                           t_io_G, t_io_E, K, C.byref(n)))
    return int(n.value)


def _ptr(t) -> Optional[int]:
    """Raw address of a torch tensor (or None)."""
    return None if t is None else t.data_ptr()


def route_static(stream, dtype: int, x, wg, top_k: int, batch_offsets: Sequence[int],
                 out: Optional["RouteOutputs"] = None, renormalize: bool = True):
    """moe_route_static: gate + dispatch plan on the library's static device scratch (no context,
    no workspace, nothing allocated by the call)."""
    out = out or RouteOutputs()
    nb = len(batch_offsets) - 1
    bo = (C.c_int32 * (nb + 1))(*[int(v) for v in batch_offsets])
    n_tokens = int(batch_offsets[-1])
    _check(load_library().moe_route_static(
        stream.cuda_stream, dtype, _ptr(x), _ptr(wg), n_tokens, int(wg.shape[1]), int(wg.shape[0]),
        top_k, 1 if renormalize else 0, bo, nb, _ptr(out.logits), _ptr(out.topk_idx), _ptr(out.topk_w),
        _ptr(out.counts), _ptr(out.offsets), _ptr(out.perm), _ptr(out.inv_perm), _ptr(out.exec_order)))


@dataclass
class RouteOutputs:
    """Optional device outputs of moe_route (torch tensors on the GPU, or None)."""
    logits: object = None
    topk_idx: object = None
    topk_w: object = None
    counts: object = None
    offsets: object = None
    perm: object = None
    inv_perm: object = None
    exec_order: object = None


class MoeContext:
    """Thin owner of a ``moe_ctx*`` plus the torch tensors it borrows."""

    def __init__(self, cfg: MoeConfig, compute_stream, copy_stream=None, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        self.plan = moe_plan(cfg, cfg.max_tokens)
        self.device = torch.device(device)
        self.compute_stream = compute_stream
        self.copy_stream = copy_stream
        self.workspace = torch.empty(self.plan.workspace_bytes, dtype=torch.uint8,
                                     device=self.device)
        self.window = None
        if self.plan.window_bytes > 0:
            self.window = torch.empty(self.plan.window_bytes, dtype=torch.uint8,
                                      device=self.device)
        self._keep = []          # tensors the context points into
        h = C.c_void_p()
        cs = compute_stream.cuda_stream
        ks = copy_stream.cuda_stream if copy_stream is not None else cs
        _check(self.lib.moe_create(C.byref(cfg), cs, ks, self.workspace.data_ptr(),
                                   self.workspace.numel(), _ptr(self.window),
                                   0 if self.window is None else self.window.numel(),
                                   C.byref(h)))
        self.h = h

    # -- placement --------------------------------------------------------------------
    def set_gate(self, layer: int, wg):
        self._keep.append(wg)
        _check(self.lib.moe_set_gate(self.h, layer, wg.data_ptr()), self.h)

    def set_expert(self, layer: int, expert: int, w1, w3, w2, where: int = MOE_RESIDENT,
                   packed=None):
        """Pack one expert.  ``packed`` (uint8 tensor of expert_bytes) is allocated here when
        not given: on the device for MOE_RESIDENT, in pinned host memory otherwise."""
        import torch
        if packed is None:
            if where == MOE_RESIDENT:
                packed = torch.empty(self.plan.expert_bytes, dtype=torch.uint8, device=self.device)
            else:
                packed = torch.empty(self.plan.expert_bytes, dtype=torch.uint8, pin_memory=True)
        self._keep.append(packed)
        _check(self.lib.moe_set_expert(self.h, layer, expert, w1.data_ptr(), w3.data_ptr(),
                                       w2.data_ptr(), where, packed.data_ptr()), self.h)
        return packed

    def set_expert_q4(self, layer: int, expert: int, q4, where: int = MOE_RESIDENT, packed=None):
        """Pack one 4-bit expert.  ``q4`` = ((q1, s1, z1), (q3, s3, z3), (q2, s2, z2)): device
        tensors, codes uint8 [rows, cols/2], scales and zero points bf16 [rows, cols/64]."""
        import torch
        if packed is None:
            if where == MOE_RESIDENT:
                packed = torch.empty(self.plan.expert_bytes, dtype=torch.uint8, device=self.device)
            else:
                packed = torch.empty(self.plan.expert_bytes, dtype=torch.uint8, pin_memory=True)
        self._keep.append(packed)
        ptrs = [t.data_ptr() for trip in q4 for t in trip]
        _check(self.lib.moe_set_expert_q4(self.h, layer, expert, *ptrs, where, packed.data_ptr()),
               self.h)
        return packed

    # -- per batch group --------------------------------------------------------------
    def route(self, layer: int, x, batch_offsets: Sequence[int],
              out: Optional[RouteOutputs] = None):
        out = out or RouteOutputs()
        nb = len(batch_offsets) - 1
        bo = (C.c_int32 * (nb + 1))(*[int(v) for v in batch_offsets])
        _check(self.lib.moe_route(self.h, layer, _ptr(x), bo, nb, _ptr(out.logits),
                                  _ptr(out.topk_idx), _ptr(out.topk_w), _ptr(out.counts),
                                  _ptr(out.offsets), _ptr(out.perm), _ptr(out.inv_perm),
                                  _ptr(out.exec_order)), self.h)

    def route_wait(self):
        E = self.cfg.n_experts
        counts = (C.c_int32 * E)()
        order = (C.c_int32 * E)()
        n = C.c_int32(0)
        _check(self.lib.moe_route_wait(self.h, counts, order, C.byref(n)), self.h)
        return list(counts), list(order), int(n.value)

    def stream_experts(self, layer: int, expert_ids: Sequence[int], flags: int):
        n = len(expert_ids)
        arr = (C.c_int32 * max(1, n))(*[int(e) for e in expert_ids])
        _check(self.lib.moe_stream_experts(self.h, layer, arr, n, flags), self.h)

    def layer_forward(self, layer: int, x, y):
        _check(self.lib.moe_layer_forward(self.h, layer, _ptr(x), _ptr(y)), self.h)

    # -- misc ---------------------------------------------------------------------------
    def stats(self) -> dict:
        s = MoeStats()
        _check(self.lib.moe_get_stats(self.h, C.byref(s)), self.h)
        return {n: int(getattr(s, n)) for n, _ in MoeStats._fields_}

    def reset_stats(self):
        _check(self.lib.moe_reset_stats(self.h), self.h)

    def set_tuning(self, split_k: int = 0, h_planes: int = 0, variant: int = 0):
        _check(self.lib.moe_set_tuning(self.h, split_k, h_planes, variant), self.h)

    def set_profiling(self, enable: bool):
        _check(self.lib.moe_set_profiling(self.h, int(enable)), self.h)

    def profile(self) -> dict:
        p = MoeProfile()
        _check(self.lib.moe_get_profile(self.h, C.byref(p)), self.h)
        return {n: float(getattr(p, n)) for n, _ in MoeProfile._fields_}

    def measure(self, layer: int, x, batch_offsets, y, reps: int = 5) -> dict:
        bo = (C.c_int32 * len(batch_offsets))(*[int(v) for v in batch_offsets])
        m = MoeMeasured()
        _check(self.lib.moe_measure(self.h, layer, x.data_ptr(), bo, len(batch_offsets) - 1,
                                    y.data_ptr(), reps, C.byref(m)), self.h)
        E = self.cfg.n_experts
        return {"t_c_gate_group_s": m.t_c_gate_group_s, "t_io_expert_s": m.t_io_expert_s,
                "t_c_gather_s": m.t_c_gather_s, "t_c_combine_s": m.t_c_combine_s,
                "t_c_expert_s": [m.t_c_expert_s[e] for e in range(E)], "n_active": m.n_active,
                "exec_order": [m.exec_order[i] for i in range(m.n_active)],
                "counts": [m.counts[e] for e in range(E)]}

    def corr_enable(self, mode: int = 1):
        """0 = off, 1 = learn and predict, 2 = predict from the table as it is."""
        _check(self.lib.moe_corr_enable(self.h, int(mode)), self.h)

    def corr_reset(self):
        _check(self.lib.moe_corr_reset(self.h), self.h)

    def corr_predict(self, layer: int, K: int) -> list:
        out = (C.c_int32 * max(1, K))()
        n = C.c_int32(0)
        _check(self.lib.moe_corr_predict(self.h, layer, K, out, C.byref(n)), self.h)
        return [int(out[i]) for i in range(n.value)]

    def corr_table(self, layer: int) -> list:
        E = self.cfg.n_experts
        out = (C.c_int32 * (E * E))()
        _check(self.lib.moe_corr_table(self.h, layer, out), self.h)
        return [[int(out[p * E + e]) for e in range(E)] for p in range(E)]

    def close(self):
        if getattr(self, "h", None):
            self.lib.moe_destroy(self.h)
            self.h = None
            self._keep = []          # the library no longer points into these
            self.workspace = None
            self.window = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
