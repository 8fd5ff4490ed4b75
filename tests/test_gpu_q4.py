"""4-bit group-quantised experts (paper Section 7, Eq. 8): the layer computed by the HIP path from
codes, scales and zero points must match the oracle, which dequantises in fp64, rounds each weight
to the model's original precision (bf16, as the paper converts tensors back before computing) and
runs the plain definition.  Routing is untouched by the weight format (bit-exact as everywhere);
outputs within the bf16 tolerance."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2502_06888_amd import binding as B
from paper_2502_06888_amd import inputs as I

import harness as H

pytestmark = pytest.mark.gpu


def bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def make_ctx_q4(w, window_layers=0):
    compute = torch.cuda.Stream()
    copy = torch.cuda.Stream() if window_layers > 0 else None
    cfg = B.make_config(w.d_model, w.d_ff, w.n_experts, w.top_k, w.n_shared, w.n_layers, window_layers,
                        max(1, w.n_tokens), max(1, w.n_batches), B.MOE_BF16, 1, 4)
    return B.MoeContext(cfg, compute, copy)


def place_q4(ctx, w, layer, gate, experts, streamed=False):
    dev = ctx.device
    ctx.set_gate(layer, gate.to(dev))
    for e, q4 in enumerate(experts):
        q4d = tuple(tuple(t.to(dev) for t in trip) for trip in q4)
        where = B.MOE_HOST_PINNED if (streamed and e < w.n_experts) else B.MOE_RESIDENT
        ctx.set_expert_q4(layer, e, q4d, where)
    torch.cuda.synchronize()


def oracle_q4(w, data, experts, tokens=None, wdtype=np.float64):
    deq = [[ref.dequant_q4(q.numpy(), bits(s), bits(z), to_bf16=True).astype(wdtype) for q, s, z in q4]
           for q4 in experts]
    return ref.moe_layer(I.as_f32(data.x), I.as_f32(data.wg), [m[0] for m in deq], [m[1] for m in deq],
                         [m[2] for m in deq], w.top_k, w.batch_offsets, w.dtype, n_shared=w.n_shared,
                         tokens=tokens)


def run_case(w, tokens=None, wdtype=np.float64):
    data, _ = I.gen_layer(w, 0, with_experts=False)
    experts = [I.gen_expert_q4(w, 0, e) for e in range(w.n_experts + w.n_shared)]
    ctx = make_ctx_q4(w)
    assert ctx.plan.expert_bytes == w.d_model * w.d_ff * 27 // 16
    place_q4(ctx, w, 0, data.wg, experts)
    got = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
    want = oracle_q4(w, data, experts, tokens, wdtype)
    H.check_routing(got, want, w.n_experts)
    err = H.check_output(got["y"], want.y, w.dtype, tokens)
    ctx.close()
    return err, float(np.sqrt((want.y ** 2).mean()))


SMALL = I.Workload("q4_small", "bf16", 256, 512, 8, 2, batch_tokens=(70, 0, 130, 100), w_std=0.08)


@pytest.mark.parametrize("w", [
    SMALL,
    I.scaled(SMALL, name="q4_ragged_units", d_model=128, d_ff=192, batch_tokens=(33, 1, 17)),
    I.scaled(SMALL, name="q4_two_tiles", n_experts=2, top_k=1, batch_tokens=(350, 350)),
    I.scaled(SMALL, name="q4_shared", n_experts=16, top_k=3, n_shared=2, d_ff=320, batch_tokens=(40, 50)),
    I.scaled(SMALL, name="q4_one_token", batch_tokens=(1,)),
    I.scaled(SMALL, name="q4_wide", d_model=1024, d_ff=2048, batch_tokens=(64,) * 3, seed=3, w_std=0.04),
], ids=lambda w: w.name)
def test_q4_small_shapes(w):
    err, rms = run_case(w)
    assert rms > 0.05                                    # outputs are not hiding in the absolute term


def test_q4_full_size_decode_layer_sampled_tokens():
    w = I.WORKLOADS["mixtral8x7b_decode"]
    tokens = sorted(np.random.default_rng(7).choice(w.n_tokens, size=96, replace=False).tolist())
    err, rms = run_case(w, tokens=tokens, wdtype=np.float32)   # bf16-valued weights are exact in fp32


def test_q4_streamed_equals_resident_and_moves_fewer_bytes():
    w = I.Workload("q4_stream", "bf16", 256, 512, 8, 2, n_layers=3, batch_tokens=(40, 30, 50),
                   streamed=True, window_layers=2, w_std=0.08)
    layers = [I.gen_layer(w, l, with_experts=False)[0] for l in range(w.n_layers)]
    experts = [[I.gen_expert_q4(w, l, e) for e in range(w.n_experts)] for l in range(w.n_layers)]
    res = make_ctx_q4(w)
    want = []
    for l in range(w.n_layers):
        place_q4(res, w, l, layers[l].wg, experts[l])
        want.append(H.gpu_layer(res, w, l, layers[l].x, w.batch_offsets))
    res.close()
    ctx = make_ctx_q4(w, window_layers=2)
    for l in range(w.n_layers):
        place_q4(ctx, w, l, layers[l].wg, experts[l], streamed=True)
    ctx.window.fill_(0xFF)
    torch.cuda.synchronize()
    ctx.reset_stats()
    dev = ctx.device
    n_active = 0
    for l in range(w.n_layers):
        x = layers[l].x.to(dev)
        y = torch.full((w.n_tokens, w.d_model), float("nan"), dtype=torch.bfloat16, device=dev)
        with torch.cuda.stream(ctx.compute_stream):
            ctx.route(l, x, w.batch_offsets)
            ctx.layer_forward(l, x, y)
        ctx.compute_stream.synchronize()
        assert np.array_equal(y.to(torch.float32).cpu().numpy(), want[l]["y"]), f"layer {l}"
        n_active += int((want[l]["counts"] > 0).sum())
    st = ctx.stats()
    assert st["bytes_h2d"] == n_active * (256 * 512 * 27 // 16)
    assert ctx.plan.expert_bytes * 32 == 3 * 256 * 512 * 2 * 9    # 9/32 of the bf16 blob
    ctx.close()


def test_q4_context_refuses_plain_weights_and_vice_versa():
    w = SMALL
    data, _ = I.gen_layer(w, 0)
    ctx = make_ctx_q4(w)
    dev = ctx.device
    with pytest.raises(B.MoeError) as ei:
        ctx.set_expert(0, 0, data.w1[0].to(dev), data.w3[0].to(dev), data.w2[0].to(dev))
    assert ei.value.status == B.MOE_ERR_STATE
    ctx.close()
    ctx = H.make_ctx(w)
    q4 = tuple(tuple(t.to(dev) for t in trip) for trip in I.gen_expert_q4(w, 0, 0))
    with pytest.raises(B.MoeError) as ei:
        ctx.set_expert_q4(0, 0, q4)
    assert ei.value.status == B.MOE_ERR_STATE
    ctx.close()


@pytest.mark.parametrize("seed", list(range(8)))
def test_seeded_sweep_of_q4_configurations(seed):
    """Widths, expert sizes (multiples of the group of 64), expert counts, top-k, shared experts and
    batch structures drawn from a seeded generator, experts as 4-bit codes."""
    g = np.random.Generator(np.random.PCG64(4000 + seed))
    d = int(g.integers(2, 9)) * 64
    f = int(g.integers(2, 11)) * 64
    E = int(g.integers(1, 25))
    k = int(g.integers(1, min(E, 6) + 1))
    nb = int(g.integers(1, 6))
    sizes = [int(v) for v in g.integers(0, 120, size=nb)]
    if sum(sizes) == 0:
        sizes[0] = 2
    w = I.Workload(f"q4sweep{seed}", "bf16", d, f, E, k, n_shared=int(g.integers(0, 3)), batch_tokens=tuple(sizes),
                   zipf_s=1.1 if seed % 2 else 0.0, seed=seed, w_std=float(1.1 / (d * f) ** 0.25))
    run_case(w)
