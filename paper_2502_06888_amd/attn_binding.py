"""Thin ctypes binding of the attention-layer entry points (``include/moe_attn.h``).

Argument marshalling only: every step of the layer runs in the HIP library.  torch is used
for device memory, pinned host memory and streams.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import Sequence

from . import binding as B

ATTN_EXPORTS = ["moe_attn_workspace_bytes", "moe_attn_create", "moe_attn_destroy",
                "moe_attn_set_weights", "moe_attn_forward_group", "moe_attn_set_profiling",
                "moe_attn_get_profile", "moe_attn_last_error", "moe_attn_prefetch"]


class MoeAttnConfig(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("max_seqs", C.c_int32), ("max_len", C.c_int32),
                ("n_layers", C.c_int32), ("max_group_seqs", C.c_int32), ("rope_theta", C.c_float),
                ("rms_eps", C.c_float)]


class MoeAttnBatch(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("pos", C.c_int32), ("kv_on_host", C.c_int32),
                ("h_on_host", C.c_int32), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("h_in", C.c_void_p), ("h_out", C.c_void_p)]


class MoeAttnProfile(C.Structure):
    _fields_ = [("wall_s", C.c_double), ("load_busy_s", C.c_double), ("store_busy_s", C.c_double),
                ("compute_busy_s", C.c_double), ("kernel_s", C.c_double * 6), ("bytes_loaded", C.c_int64),
                ("bytes_stored", C.c_int64)]


_ready = False


def load_library():
    """The shared library with the attention entry points typed (fails loudly when missing)."""
    global _ready
    lib = B.load_library()
    if not _ready:
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        P = C.POINTER
        lib.moe_attn_workspace_bytes.argtypes = [P(MoeAttnConfig), P(i64)]
        lib.moe_attn_create.argtypes = [P(MoeAttnConfig), vp, i64, vp, vp, vp, P(vp)]
        lib.moe_attn_destroy.argtypes = [vp]
        lib.moe_attn_destroy.restype = None
        lib.moe_attn_set_weights.argtypes = [vp, i32] + [vp] * 5 + [i32]
        lib.moe_attn_forward_group.argtypes = [vp, i32, i32, P(MoeAttnBatch)]
        lib.moe_attn_prefetch.argtypes = [vp, P(MoeAttnBatch)]
        lib.moe_attn_set_profiling.argtypes = [vp, i32]
        lib.moe_attn_get_profile.argtypes = [vp, P(MoeAttnProfile)]
        lib.moe_attn_last_error.argtypes = [vp]
        lib.moe_attn_last_error.restype = C.c_char_p
        for name in ATTN_EXPORTS:
            if name not in ("moe_attn_last_error", "moe_attn_destroy"):
                getattr(lib, name).restype = C.c_int
        _ready = True
    return lib


def _check(status: int, ctx=None):
    if status != B.MOE_OK:
        msg = load_library().moe_attn_last_error(ctx)
        raise B.MoeError(status, msg.decode() if msg else "")


def workspace_bytes(cfg: MoeAttnConfig) -> int:
    n = C.c_int64(0)
    _check(load_library().moe_attn_workspace_bytes(C.byref(cfg), C.byref(n)))
    return int(n.value)


@dataclass
class AttnBatch:
    """One batch of the group: torch tensors, device or pinned host."""
    k_cache: object   # bf16 [n_seq, Hkv, max_len, hd]
    v_cache: object
    h_in: object      # bf16 [n_seq, d]
    h_out: object
    pos: int


class AttnContext:
    """Owner of a ``moe_attn_ctx*``, its workspace and its three streams."""

    def __init__(self, cfg: MoeAttnConfig, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.workspace = torch.empty(workspace_bytes(cfg), dtype=torch.uint8, device=self.device)
        self.compute = torch.cuda.Stream(device=self.device)
        self.load = torch.cuda.Stream(device=self.device)
        self.store = torch.cuda.Stream(device=self.device)
        h = C.c_void_p()
        _check(self.lib.moe_attn_create(C.byref(cfg), self.workspace.data_ptr(), self.workspace.numel(),
                                        self.compute.cuda_stream, self.load.cuda_stream,
                                        self.store.cuda_stream, C.byref(h)))
        self.h = h

    def set_weights(self, g, wq, wk, wv, wo, layer: int = 0):
        on_host = 0 if g.is_cuda else 1
        _check(self.lib.moe_attn_set_weights(self.h, layer, g.data_ptr(), wq.data_ptr(), wk.data_ptr(),
                                             wv.data_ptr(), wo.data_ptr(), on_host), self.h)

    @staticmethod
    def _marshal(b: AttnBatch) -> MoeAttnBatch:
        return MoeAttnBatch(b.h_in.shape[0], b.pos, 0 if b.k_cache.is_cuda else 1,
                            0 if b.h_in.is_cuda else 1, b.k_cache.data_ptr(),
                            b.v_cache.data_ptr(), b.h_in.data_ptr(), b.h_out.data_ptr())

    def prefetch(self, first: AttnBatch):
        m = self._marshal(first)
        _check(self.lib.moe_attn_prefetch(self.h, C.byref(m)), self.h)

    def forward_group(self, batches: Sequence[AttnBatch], layer: int = 0):
        arr = (MoeAttnBatch * max(1, len(batches)))()
        for i, b in enumerate(batches):
            arr[i] = self._marshal(b)
        _check(self.lib.moe_attn_forward_group(self.h, layer, len(batches), arr), self.h)

    def set_profiling(self, level: int):
        """0 off; n >= 1 on, kernels repeated n times between their events."""
        _check(self.lib.moe_attn_set_profiling(self.h, int(level)), self.h)

    def profile(self) -> MoeAttnProfile:
        out = MoeAttnProfile()
        _check(self.lib.moe_attn_get_profile(self.h, C.byref(out)), self.h)
        return out

    def synchronize(self):
        self.compute.synchronize()

    def close(self):
        if self.h:
            self.lib.moe_attn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def config_for(w, max_seqs=None, n_layers: int = 1, grouped: bool = True) -> MoeAttnConfig:
    """MoeAttnConfig of an ``inputs.AttnWorkload``; ``grouped`` sizes the buffers for the whole
    batch group so that device-resident groups run in one pass."""
    return MoeAttnConfig(w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim,
                         max_seqs or max(w.batch_seqs), w.max_len, n_layers,
                         w.n_tokens if grouped else 0, w.rope_theta, w.rms_eps)
