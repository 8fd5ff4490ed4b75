"""Attention layer and MoE layer alternating over two blocks in the order of Algorithm 1:
non-expert layer batch by batch, expert layer over the whole batch group, the first batch's
caches of the next attention layer requested while the expert layer computes.  Both libraries'
contexts live side by side on their own streams; the hidden states of the group are one tensor
whose slices are the batches.  Every stage is checked against its oracle on the very inputs the
GPU stage received (the previous stage's GPU output), so routing stays bit-exact."""
import numpy as np
import pytest
import torch

from oracle import attn_ref as AR
from paper_2502_06888_amd import attn_binding as A
from paper_2502_06888_amd import binding as B
from paper_2502_06888_amd import inputs as I

import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("kv_on_host", [False, True])
def test_two_blocks_in_schedule_order(kv_on_host):
    aw = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], batch_seqs=(5, 3, 8), batch_pos=(17, 0, 40), seed=21)
    mw = I.Workload("block_moe", "bf16", aw.d_model, 512, 8, 2, n_layers=2, batch_tokens=aw.batch_seqs,
                    w_std=0.08, seed=21)
    n_layers, N, d = 2, aw.n_tokens, aw.d_model
    actx = A.AttnContext(A.config_for(aw, n_layers=n_layers), DEV)
    mctx = H.make_ctx(mw)
    attn_w, moe_data, caches = [], [], []
    for l in range(n_layers):
        ws = I.gen_attn_weights(aw, l)
        actx.set_weights(*[ws[n].to(DEV) for n in ("norm", "wq", "wk", "wv", "wo")], layer=l)
        attn_w.append(ws)
        data, _ = I.gen_layer(mw, l)
        H.place_layer(mctx, mw, l, data)
        moe_data.append(data)
        per_batch = []
        for b in range(aw.n_batches):
            k, v = I.gen_kv_cache(aw, l, b)
            per_batch.append((k.clone().pin_memory(), v.clone().pin_memory()) if kv_on_host else (k.to(DEV), v.to(DEV)))
        caches.append(per_batch)
    cur = torch.cat([I.gen_attn_hidden(aw, 0, b) for b in range(aw.n_batches)]).to(DEV)   # [N, d]
    bo = [int(v) for v in mw.batch_offsets]

    def batches_of(l, src, dst):
        out = []
        for b in range(aw.n_batches):
            out.append(A.AttnBatch(caches[l][b][0], caches[l][b][1], src[bo[b]:bo[b + 1]], dst[bo[b]:bo[b + 1]],
                                   aw.batch_pos[b]))
        return out

    for l in range(n_layers):
        # non-expert layer, batch by batch (or in one pass when everything is on the device)
        before = [(c[0].clone(), c[1].clone()) for c in caches[l]]
        h1 = torch.zeros_like(cur)
        torch.cuda.synchronize()
        actx.forward_group(batches_of(l, cur, h1), layer=l)
        actx.synchronize()
        raw = {k: I.as_raw(v) for k, v in attn_w[l].items()}
        for b in range(aw.n_batches):
            y, k2, v2 = AR.attn_decode(I.as_f32(cur[bo[b]:bo[b + 1]]), raw["norm"], raw["wq"], raw["wk"], raw["wv"],
                                       raw["wo"], I.as_raw(before[b][0]), I.as_raw(before[b][1]), aw.batch_pos[b],
                                       aw.n_q_heads, aw.n_kv_heads, aw.head_dim, aw.rope_theta, aw.rms_eps)
            got = h1[bo[b]:bo[b + 1]].to(torch.float64).cpu().numpy()
            err = np.abs(got - y) - (1e-2 + 2e-2 * np.abs(y))
            assert err.max() <= 0, f"block {l} batch {b}: attention output off by {err.max()}"
        # expert layer over the whole group; meanwhile the next attention layer's first cache
        x_cpu = h1.cpu()
        out = H.alloc_route_outputs(mw, N, torch.device(DEV))
        y = torch.full((N, d), float("nan"), dtype=torch.bfloat16, device=DEV)
        with torch.cuda.stream(mctx.compute_stream):
            mctx.route(l, h1, bo, out)
            mctx.layer_forward(l, h1, y)
        if l + 1 < n_layers:
            nxt = batches_of(l + 1, y, y)[0]
            actx.prefetch(nxt)
        mctx.compute_stream.synchronize()
        stage = I.LayerData(x=x_cpu, wg=moe_data[l].wg, w1=moe_data[l].w1, w3=moe_data[l].w3, w2=moe_data[l].w2)
        want = H.oracle_layer(mw, stage, mw.batch_offsets)
        assert np.array_equal(out.topk_idx[:N * mw.top_k].cpu().numpy().reshape(N, mw.top_k), want.idx)
        assert np.array_equal(out.counts.cpu().numpy(), want.disp.counts)
        assert np.array_equal(out.perm[:N * mw.top_k].cpu().numpy(), want.disp.perm)
        H.check_output(y.to(torch.float32).cpu().numpy(), want.y, "bf16")
        cur = y
    actx.close()
    mctx.close()
