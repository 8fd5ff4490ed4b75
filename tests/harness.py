"""Shared helpers of the GPU parity tests: run one MoE layer through the C-ABI library and
through the CPU oracle on the same seeded inputs, and compare.  Not collected by pytest."""
from __future__ import annotations

import numpy as np
import torch

from oracle import ref
from paper_2502_06888_amd import binding as B
from paper_2502_06888_amd import inputs as I

TOL = {"bf16": (2e-2, 1e-2), "f32": (1e-5, 1e-5)}   # (rtol, atol): |gpu-ref| <= atol + rtol*|ref|


def make_ctx(w: I.Workload, compute=None, copy=None, max_tokens=None, window_layers=None,
             renorm: bool = True):
    compute = compute or torch.cuda.Stream()
    wl = w.window_layers if window_layers is None else window_layers
    if wl > 0 and copy is None:
        copy = torch.cuda.Stream()
    cfg = B.make_config(w.d_model, w.d_ff, w.n_experts, w.top_k, w.n_shared, w.n_layers, wl,
                        max_tokens or max(1, w.n_tokens), max(1, w.n_batches),
                        B.MOE_F32 if w.dtype == "f32" else B.MOE_BF16, 1 if renorm else 0)
    return B.MoeContext(cfg, compute, copy)


def place_layer(ctx, w: I.Workload, layer: int, data: I.LayerData, streamed: bool = False):
    """Upload one layer's weights and pack them (routed experts pinned when ``streamed``)."""
    dev = ctx.device
    ctx.set_gate(layer, data.wg.to(dev))
    for e in range(w.n_experts + w.n_shared):
        w1, w3, w2 = (t.to(dev) for t in (data.w1[e], data.w3[e], data.w2[e]))
        where = B.MOE_HOST_PINNED if (streamed and e < w.n_experts) else B.MOE_RESIDENT
        ctx.set_expert(layer, e, w1, w3, w2, where)
    torch.cuda.synchronize()


def alloc_route_outputs(w: I.Workload, n_tokens: int, dev) -> B.RouteOutputs:
    A = n_tokens * w.top_k
    i32 = dict(dtype=torch.int32, device=dev)
    return B.RouteOutputs(
        logits=torch.full((max(1, n_tokens), w.n_experts), float("nan"), dtype=torch.float32,
                          device=dev),
        topk_idx=torch.full((max(1, A),), -7, **i32),
        topk_w=torch.full((max(1, A),), float("nan"), dtype=torch.float32, device=dev),
        counts=torch.full((w.n_experts,), -7, **i32),
        offsets=torch.full((w.n_experts + 1,), -7, **i32),
        perm=torch.full((max(1, A),), -7, **i32),
        inv_perm=torch.full((max(1, A),), -7, **i32),
        exec_order=torch.full((w.n_experts,), -7, **i32))


def gpu_layer(ctx, w: I.Workload, layer: int, x_cpu: torch.Tensor, batch_offsets, y=None):
    """route + forward on the GPU; returns numpy views of everything."""
    dev = ctx.device
    N = x_cpu.shape[0]
    x = x_cpu.to(dev)
    out = alloc_route_outputs(w, N, dev)
    if y is None:
        y = torch.full((max(1, N), w.d_model), float("nan"), dtype=w.torch_dtype, device=dev)
    with torch.cuda.stream(ctx.compute_stream):
        ctx.route(layer, x, batch_offsets, out)
        ctx.layer_forward(layer, x, y)
    ctx.compute_stream.synchronize()
    A = N * w.top_k
    res = dict(
        logits=out.logits[:N].cpu().numpy(),
        idx=out.topk_idx[:A].cpu().numpy().reshape(N, w.top_k),
        w=out.topk_w[:A].cpu().numpy().reshape(N, w.top_k),
        counts=out.counts.cpu().numpy(), offsets=out.offsets.cpu().numpy(),
        perm=out.perm[:A].cpu().numpy(), inv_perm=out.inv_perm[:A].cpu().numpy(),
        exec_order=out.exec_order.cpu().numpy(),
        y=y[:N].to(torch.float32).cpu().numpy())
    return res


def oracle_layer(w: I.Workload, data: I.LayerData, batch_offsets, tokens=None,
                 with_output=True, renorm: bool = True) -> ref.LayerRef:
    return ref.moe_layer(I.as_f32(data.x), I.as_f32(data.wg),
                         [I.as_raw(t) for t in data.w1], [I.as_raw(t) for t in data.w3],
                         [I.as_raw(t) for t in data.w2], w.top_k, batch_offsets, w.dtype,
                         n_shared=w.n_shared, tokens=tokens, with_output=with_output,
                         renorm=renorm)


def check_routing(got: dict, want: ref.LayerRef, n_experts: int):
    """Bit-exact integer work; logits bit-exact too (same fp32 summation order)."""
    assert np.array_equal(got["logits"].view(np.uint32), want.logits.view(np.uint32)), \
        "gate logits differ bitwise"
    assert np.array_equal(got["idx"], want.idx), "top-k indices differ"
    d = want.disp
    assert np.array_equal(got["counts"], d.counts)
    assert np.array_equal(got["offsets"], d.offsets)
    assert np.array_equal(got["perm"], d.perm)
    assert np.array_equal(got["inv_perm"], d.inv_perm)
    assert np.array_equal(got["exec_order"], d.exec_order)
    assert np.allclose(got["w"], want.w, rtol=1e-5, atol=1e-6), "routing weights differ"
    assert int(got["counts"].sum()) == got["idx"].size


def check_output(got_y: np.ndarray, want_y: np.ndarray, dtype: str, tokens=None):
    rtol, atol = TOL[dtype]
    g = got_y if tokens is None else got_y[np.asarray(tokens)]
    assert np.all(np.isfinite(g)), "non-finite output"
    err = np.abs(g.astype(np.float64) - want_y)
    lim = atol + rtol * np.abs(want_y)
    worst = float((err / lim).max()) if err.size else 0.0
    if worst > 1.0:
        i = np.unravel_index(np.argmax(err / lim), err.shape)
        raise AssertionError(
            f"output outside tolerance (rtol {rtol}, atol {atol}): worst err/limit {worst:.3f} at "
            f"{i}: ref {want_y[i]:.5f} got {g[i]:.5f}; {int((err > lim).sum())} of {err.size} "
            f"elements outside; max abs err {err.max():.3e}; ref rms {np.sqrt((want_y**2).mean()):.3f}")
    return float(err.max()) if err.size else 0.0
