"""moe_route_static (the entry point that allocates nothing: its dispatch scratch is a fixed array
in the library's device image) against moe_route on the same inputs, through the C ABI: every
output bit for bit, on two calls in a row, the second with a smaller batch group, and on a group
of several plan chunks; limits are refused before anything is launched."""
import numpy as np
import pytest
import torch

from paper_2502_06888_amd import binding as B
from paper_2502_06888_amd import inputs as I

import harness as H

pytestmark = pytest.mark.gpu

FIELDS = ("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm", "exec_order")


def route_both(ctx, w, x, wg, bo):
    """Outputs of moe_route (context, workspace) and of moe_route_static for one batch group."""
    dev = ctx.device
    n = int(bo[-1])
    via_ctx = H.alloc_route_outputs(w, n, dev)
    static = H.alloc_route_outputs(w, n, dev)
    dtype = B.MOE_F32 if w.dtype == "f32" else B.MOE_BF16
    with torch.cuda.stream(ctx.compute_stream):
        ctx.route(0, x[:n], bo, via_ctx)
        before = torch.cuda.memory_allocated(dev)
        B.route_static(ctx.compute_stream, dtype, x[:n], wg, w.top_k, bo, static)
        assert torch.cuda.memory_allocated(dev) == before
    ctx.compute_stream.synchronize()
    return via_ctx, static


def assert_same(via_ctx, static, n, k):
    A = n * k
    cut = {"logits": n, "topk_idx": A, "topk_w": A, "perm": A, "inv_perm": A}
    for f in FIELDS:
        a, b = getattr(via_ctx, f), getattr(static, f)
        m = cut.get(f, a.shape[0])
        a, b = a[:m].cpu().numpy(), b[:m].cpu().numpy()
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f
    assert int(static.counts.sum()) == A


@pytest.mark.parametrize("w", [
    I.Workload("static_small", "bf16", 256, 512, 8, 2, batch_tokens=(70, 0, 130, 100)),
    I.Workload("static_f32", "f32", 64, 96, 6, 3, batch_tokens=(5, 0, 9, 23)),
    I.Workload("static_chunks", "bf16", 512, 192, 200, 8, batch_tokens=tuple([40, 0, 90, 3] * 8),
               zipf_s=1.2, corr=0.0),
], ids=lambda w: w.name)
def test_static_route_equals_route_twice_in_a_row(w):
    data, _ = I.gen_layer(w, 0, with_experts=False)
    ctx = H.make_ctx(w)
    dev = ctx.device
    wg = data.wg.to(dev)
    ctx.set_gate(0, wg)
    x = data.x.to(dev)
    bo = [int(v) for v in w.batch_offsets]
    via_ctx, static = route_both(ctx, w, x, wg, bo)
    assert_same(via_ctx, static, w.n_tokens, w.top_k)
    # second call, smaller group: the array still holds the first call's contents
    keep = max(2, w.n_batches // 2)
    bo2 = bo[:keep + 1]
    via_ctx, static = route_both(ctx, w, x, wg, bo2)
    assert_same(via_ctx, static, bo2[-1], w.top_k)
    # and with no output requested but one (everything else lands in the static array)
    only = B.RouteOutputs(perm=torch.full((max(1, bo2[-1] * w.top_k),), -7, dtype=torch.int32, device=dev))
    with torch.cuda.stream(ctx.compute_stream):
        B.route_static(ctx.compute_stream, B.MOE_F32 if w.dtype == "f32" else B.MOE_BF16, x[:bo2[-1]], wg,
                       w.top_k, bo2, only)
    ctx.compute_stream.synchronize()
    A2 = bo2[-1] * w.top_k
    assert np.array_equal(only.perm[:A2].cpu().numpy(), static.perm[:A2].cpu().numpy())
    ctx.close()


def test_static_route_refuses_sizes_beyond_its_array():
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    wg = torch.zeros((8, 256), dtype=torch.bfloat16, device=dev)
    x = torch.zeros((4, 256), dtype=torch.bfloat16, device=dev)
    for n, k in ((65537, 1), (40000, 2)):
        with pytest.raises(B.MoeError) as ei:
            B.route_static(st, B.MOE_BF16, x, wg, k, [0, n])
        assert ei.value.status == B.MOE_ERR_SHAPE
    with pytest.raises(B.MoeError) as ei:               # offsets that do not end at n_tokens
        B.load_library().moe_route_static
        B._check(B.load_library().moe_route_static(st.cuda_stream, B.MOE_BF16, x.data_ptr(), wg.data_ptr(), 4, 256,
                                                   8, 2, 1, (B.C.c_int32 * 2)(0, 3), 1, *([None] * 8)))
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    B.route_static(st, B.MOE_BF16, x, wg, 2, [0, 4])     # a legal call still works afterwards
    st.synchronize()


def test_static_route_replays_from_a_graph():
    """The callers this entry point is for include code under HIP graph capture: the call records
    nothing but its kernels, and replays reproduce the eager outputs, with eager calls (which use
    the same static array) and synchronisation between the replays."""
    w = I.Workload("static_graph", "bf16", 256, 512, 16, 4, batch_tokens=(33, 0, 60, 7))
    data, _ = I.gen_layer(w, 0, with_experts=False)
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    wg, x = data.wg.to(dev), data.x.to(dev)
    bo = [int(v) for v in w.batch_offsets]
    out = H.alloc_route_outputs(w, w.n_tokens, dev)
    with torch.cuda.stream(st):
        B.route_static(st, B.MOE_BF16, x, wg, w.top_k, bo, out)
    st.synchronize()
    want = {f: getattr(out, f).clone() for f in FIELDS}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        B.route_static(st, B.MOE_BF16, x, wg, w.top_k, bo, out)
    other = H.alloc_route_outputs(w, bo[2], dev)
    for rep in range(3):
        for f in FIELDS:
            getattr(out, f).fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for f in FIELDS:
            assert torch.equal(getattr(out, f).view(torch.int32), want[f].view(torch.int32)), (rep, f)
        with torch.cuda.stream(st):               # an eager call on a smaller group in between
            B.route_static(st, B.MOE_BF16, x[:bo[2]], wg, w.top_k, bo[:3], other)
        st.synchronize()
