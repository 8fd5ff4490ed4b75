"""The resident MoE step (moe_route + moe_layer_forward) and the device-resident attention group
are plain runs of kernels on the caller's stream, so a caller can capture them into a HIP graph.
Replays are compared with the eager result, several times, with eager work and synchronisation
between the replays."""
import pytest
import torch

from paper_2502_06888_amd import attn_binding as A
from paper_2502_06888_amd import inputs as I

import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def replay_and_compare(graph, eager_step, stream, outputs, want):
    for rep in range(3):
        for t in outputs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, w in zip(outputs, want):
            assert torch.equal(t, w), f"replay {rep} differs from the eager result"
        with torch.cuda.stream(stream):
            eager_step()
        stream.synchronize()


def test_moe_step_replays_from_a_graph():
    w = I.Workload("graph_moe", "bf16", 256, 512, 8, 2, batch_tokens=(40, 0, 25, 70), w_std=0.08)
    data, _ = I.gen_layer(w)
    ctx = H.make_ctx(w)
    H.place_layer(ctx, w, 0, data)
    x = data.x.to(DEV)
    y = torch.zeros((w.n_tokens, w.d_model), dtype=torch.bfloat16, device=DEV)
    bo = [int(v) for v in w.batch_offsets]
    st = ctx.compute_stream

    def step():
        ctx.route(0, x, bo)
        ctx.layer_forward(0, x, y)

    with torch.cuda.stream(st):
        step()
    st.synchronize()
    want = [y.clone()]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        step()
    replay_and_compare(g, step, st, [y], want)
    ctx.close()


def test_attention_group_replays_from_a_graph():
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ctx = A.AttnContext(A.config_for(w), DEV)
    ws = I.gen_attn_weights(w, 0)
    ctx.set_weights(*[ws[n].to(DEV) for n in ("norm", "wq", "wk", "wv", "wo")])
    batches, outs = [], []
    for b in range(w.n_batches):
        k, v = [t.to(DEV) for t in I.gen_kv_cache(w, 0, b)]
        h = I.gen_attn_hidden(w, 0, b).to(DEV)
        o = torch.zeros_like(h)
        batches.append(A.AttnBatch(k, v, h, o, w.batch_pos[b]))
        outs.append(o)
    st = ctx.compute

    def step():
        ctx.forward_group(batches)

    step()
    st.synchronize()
    want = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        step()
    replay_and_compare(g, step, st, outs, want)
    ctx.close()
