"""Attention (non-expert) layer on the GPU against the CPU oracle, through the C ABI.

Tolerance: the layer output and the appended cache rows are bf16 results of contractions over
bf16 operands (the normalised activations are rounded to bf16 for the matrix cores): 2e-2
relative / 1e-2 absolute, the bar of the bf16 MoE outputs.  Cache rows the step does not
write must come back bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import attn_ref as R
from paper_2502_06888_amd import attn_binding as A
from paper_2502_06888_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def oracle_group(w, ws, hs, caches):
    raw = {k: I.as_raw(v) for k, v in ws.items()}
    out = []
    for b in range(w.n_batches):
        y, k2, v2 = R.attn_decode(I.as_f32(hs[b]), raw["norm"], raw["wq"], raw["wk"], raw["wv"], raw["wo"],
                                  I.as_raw(caches[b][0]), I.as_raw(caches[b][1]), w.batch_pos[b],
                                  w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
        out.append((y, k2, v2))
    return out


def widen(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def check_group(w, batches, want):
    for b, (bt, (y, k2, v2)) in enumerate(zip(batches, want)):
        got = bt.h_out.cpu().to(torch.float64).numpy()
        err = np.abs(got - y) - (1e-2 + 2e-2 * np.abs(y))
        assert err.max() <= 0, f"batch {b}: output off by {err.max()} beyond tolerance"
        for name, g, o in (("K", bt.k_cache, k2), ("V", bt.v_cache, v2)):
            gb = I.as_raw(g.cpu())
            pos = w.batch_pos[b]
            keep_mask = np.ones(gb.shape[2], bool)
            keep_mask[pos] = False
            assert np.array_equal(gb[:, :, keep_mask, :], o[:, :, keep_mask, :]), \
                f"batch {b}: {name} rows other than pos changed"
            # the appended row: same bar as the layer output, and much closer than that on average
            gr, orow = widen(gb[:, :, pos, :]), widen(o[:, :, pos, :])
            err = np.abs(gr - orow) - (1e-2 + 2e-2 * np.abs(orow))
            assert err.max() <= 0, f"batch {b}: new {name} row off by {err.max()} beyond tolerance"
            rms = np.sqrt((orow ** 2).mean())
            assert np.abs(gr - orow).mean() <= 4e-3 * rms, \
                f"batch {b}: new {name} row mean error {np.abs(gr - orow).mean() / rms:.2e} of rms"


def run_group(w, on_host, layer=0, ctx=None, set_weights=True, prefetch=None):
    ws = I.gen_attn_weights(w, layer)
    hs = [I.gen_attn_hidden(w, layer, b) for b in range(w.n_batches)]
    caches = [I.gen_kv_cache(w, layer, b) for b in range(w.n_batches)]
    own = ctx is None
    if own:
        ctx = A.AttnContext(A.config_for(w), DEV)
    if set_weights:
        ctx.set_weights(*[ws[n].to(DEV) for n in ("norm", "wq", "wk", "wv", "wo")], layer=layer)
    batches = []
    for b in range(w.n_batches):
        host_b = on_host[b % len(on_host)] if isinstance(on_host, (tuple, list)) else on_host
        if host_b:
            k, v = caches[b][0].clone().pin_memory(), caches[b][1].clone().pin_memory()
            h_in = hs[b].clone().pin_memory()
            h_out = torch.zeros_like(h_in).pin_memory()
        else:
            k, v = caches[b][0].to(DEV), caches[b][1].to(DEV)
            h_in = hs[b].to(DEV)
            h_out = torch.zeros_like(h_in)
        batches.append(A.AttnBatch(k, v, h_in, h_out, w.batch_pos[b]))
    torch.cuda.synchronize()
    if prefetch is not None:
        ctx.prefetch(batches[prefetch])
    ctx.forward_group(batches, layer=layer)
    ctx.synchronize()
    torch.cuda.synchronize()
    check_group(w, batches, oracle_group(w, ws, hs, caches))
    if own:
        ctx.close()


@pytest.mark.parametrize("on_host", [False, True])
def test_tiny_group_matches_oracle(on_host):
    run_group(I.ATTN_WORKLOADS["attn_tiny"], on_host)


def test_device_group_batch_by_batch():
    """A context not sized for the whole group (max_group_seqs = 0) runs a device-resident group
    batch by batch; sized for it, in one pass.  Both against the oracle."""
    w = I.ATTN_WORKLOADS["attn_tiny"]
    for grouped in (False, True):
        ctx = A.AttnContext(A.config_for(w, grouped=grouped), DEV)
        run_group(w, on_host=False, ctx=ctx)
        ctx.close()


@pytest.mark.parametrize("hd,hq,hkv", [(32, 8, 8), (64, 4, 2), (128, 8, 1), (128, 2, 1), (128, 6, 1), (64, 6, 2),
                                       (32, 20, 4), (128, 7, 1)])
def test_head_shapes(hd, hq, hkv):
    w = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], head_dim=hd, n_q_heads=hq, n_kv_heads=hkv,
                 d_model=256, batch_seqs=(33, 2), batch_pos=(70, 3), max_len=80, seed=3)
    run_group(w, on_host=True)


def test_ragged_rows_and_several_row_tiles():
    # 130 sequences: five row blocks -> two row tiles of four blocks, the last one ragged
    w = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64,
                 batch_seqs=(130, 1, 64), batch_pos=(9, 255, 128), max_len=256, seed=5)
    run_group(w, on_host=False)
    run_group(w, on_host=True)


def test_group_mixing_host_and_device_batches():
    """Batches whose caches live on the host next to batches that live on the device, in both
    alternations and with a run of device batches between two host batches."""
    w = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], batch_seqs=(4, 7, 2, 9, 3, 5), batch_pos=(11, 30, 0, 47, 8, 21), seed=11)
    ctx = A.AttnContext(A.config_for(w), DEV)
    run_group(w, on_host=(True, False), ctx=ctx)
    run_group(w, on_host=(False, True), ctx=ctx)
    run_group(w, on_host=(True, False, False, False, True, False), ctx=ctx)
    ctx.close()


@pytest.mark.parametrize("n_batches", [64, 66])
def test_many_small_batches(n_batches):
    """64 batches is the most one pass over a device-resident group takes; 66 fall back to the
    batch-by-batch loop.  One or two sequences per batch, positions all different."""
    seqs = tuple(1 + (b % 2) for b in range(n_batches))
    pos = tuple((7 * b) % 47 for b in range(n_batches))
    w = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], batch_seqs=seqs, batch_pos=pos, seed=13)
    run_group(w, on_host=False)


def test_empty_group_and_full_cache():
    w = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], batch_seqs=(8,), batch_pos=(47,), seed=17)   # last free position
    ctx = A.AttnContext(A.config_for(w), DEV)
    run_group(w, on_host=True, ctx=ctx)
    run_group(w, on_host=False, ctx=ctx)
    ctx.forward_group([])            # nothing to do, no error
    ctx.synchronize()
    ctx.close()


def test_context_reuse_with_shrinking_batches():
    big = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], batch_seqs=(8, 8, 8, 8, 8), batch_pos=(40, 41, 42, 43, 44), seed=7)
    small = I.scaled(big, batch_seqs=(3, 2), batch_pos=(5, 0), seed=8)
    ctx = A.AttnContext(A.config_for(big), DEV)
    run_group(big, True, ctx=ctx)
    run_group(small, True, ctx=ctx)
    run_group(big, False, ctx=ctx)
    ctx.close()


def test_several_layers_in_one_context():
    """Three layers' weights in one context, used out of order; inputs differ per layer."""
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ctx = A.AttnContext(A.config_for(w, n_layers=3), DEV)
    for layer in (2, 0, 1):
        ws = I.gen_attn_weights(w, layer)
        ctx.set_weights(*[ws[n].to(DEV) for n in ("norm", "wq", "wk", "wv", "wo")], layer=layer)
    for layer in (1, 2, 0, 2):
        run_group(w, on_host=(layer != 1), layer=layer, ctx=ctx, set_weights=False)
    from paper_2502_06888_amd import binding as B
    with pytest.raises(B.MoeError) as ei:
        run_group(w, on_host=False, layer=3, ctx=ctx, set_weights=False)
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    ctx.close()


def test_prefetch_of_the_first_batch():
    """The first batch's caches brought in ahead of the call (and a prefetch of some other batch,
    which the call must ignore): same results; the call then loads fewer bytes."""
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ctx = A.AttnContext(A.config_for(w), DEV)
    ctx.set_profiling(1)
    run_group(w, on_host=True, ctx=ctx)
    plain = ctx.profile().bytes_loaded
    run_group(w, on_host=True, ctx=ctx, prefetch=0)
    ahead = ctx.profile().bytes_loaded
    run_group(w, on_host=True, ctx=ctx, prefetch=2)
    other = ctx.profile().bytes_loaded
    assert plain - ahead == w.kv_bytes(0) and other == plain
    run_group(w, on_host=False, ctx=ctx, prefetch=0)   # device-resident caches: nothing to move
    ctx.close()


def test_argument_errors():
    from paper_2502_06888_amd import binding as B
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ctx = A.AttnContext(A.config_for(w), DEV)
    k, v = [t.to(DEV) for t in I.gen_kv_cache(w, 0, 0)]
    h = I.gen_attn_hidden(w, 0, 0).to(DEV)
    with pytest.raises(B.MoeError) as ei:
        ctx.forward_group([A.AttnBatch(k, v, h, h, 1)])
    assert ei.value.status == B.MOE_ERR_STATE
    ws = I.gen_attn_weights(w, 0)
    ctx.set_weights(*[ws[n] for n in ("norm", "wq", "wk", "wv", "wo")])   # plain host tensors
    with pytest.raises(B.MoeError) as ei:
        ctx.forward_group([A.AttnBatch(k, v, h, h, w.max_len)])
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    with pytest.raises(B.MoeError) as ei:   # pageable host memory where pinned is required
        ctx.forward_group([A.AttnBatch(k.cpu(), v.cpu(), h, h, 1)])
    assert ei.value.status == B.MOE_ERR_NOT_PINNED
    ctx.forward_group([A.AttnBatch(k, v, h, h, w.batch_pos[0])])          # in place, still usable
    ctx.synchronize()
    ctx.close()
    with pytest.raises(B.MoeError) as ei:
        A.workspace_bytes(A.MoeAttnConfig(200, 8, 2, 32, 4, 16, 1, 0, 1e4, 1e-5))
    assert ei.value.status == B.MOE_ERR_SHAPE


def test_full_size_sampled_sequences():
    """Mixtral-8x7B attention shape in the launch configuration the benchmark times (64 sequences
    per batch, 512 cached positions, caches streamed from pinned host memory); the oracle checks a
    sample of sequences one by one (rows of a batch are independent of each other)."""
    w = I.scaled(I.ATTN_WORKLOADS["attn_mixtral8x7b_decode"], batch_seqs=(64, 64, 37), batch_pos=(512, 512, 575))
    ws = I.gen_attn_weights(w, 0)
    hs = [I.gen_attn_hidden(w, 0, b) for b in range(w.n_batches)]
    caches = [I.gen_kv_cache(w, 0, b) for b in range(w.n_batches)]
    ctx = A.AttnContext(A.config_for(w), DEV)
    ctx.set_weights(*[ws[n].to(DEV) for n in ("norm", "wq", "wk", "wv", "wo")])
    batches = []
    for b in range(w.n_batches):
        h_in = hs[b].clone().pin_memory()
        batches.append(A.AttnBatch(caches[b][0].clone().pin_memory(), caches[b][1].clone().pin_memory(),
                                   h_in, torch.zeros_like(h_in).pin_memory(), w.batch_pos[b]))
    ctx.forward_group(batches)
    ctx.synchronize()
    raw = {k: I.as_raw(v) for k, v in ws.items()}
    for b, rows in ((0, [0, 31, 63]), (1, [32]), (2, [0, 36])):
        pos = w.batch_pos[b]
        y, k2, v2 = R.attn_decode(I.as_f32(hs[b])[rows], raw["norm"], raw["wq"], raw["wk"], raw["wv"], raw["wo"],
                                  I.as_raw(caches[b][0])[rows], I.as_raw(caches[b][1])[rows], pos,
                                  w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
        got = batches[b].h_out.to(torch.float64).numpy()[rows]
        err = np.abs(got - y) - (1e-2 + 2e-2 * np.abs(y))
        assert err.max() <= 0, f"batch {b}: output off by {err.max()} beyond tolerance"
        for name, g, o in (("K", batches[b].k_cache, k2), ("V", batches[b].v_cache, v2)):
            gr, orow = widen(I.as_raw(g)[rows][:, :, pos, :]), widen(o[:, :, pos, :])
            err = np.abs(gr - orow) - (1e-2 + 2e-2 * np.abs(orow))
            assert err.max() <= 0, f"batch {b}: new {name} row off by {err.max()} beyond tolerance"
    # properties that hold for every sequence: cache rows before pos untouched, outputs finite
    for b in range(w.n_batches):
        pos = w.batch_pos[b]
        assert torch.equal(batches[b].k_cache[:, :, :pos], caches[b][0][:, :, :pos])
        assert torch.equal(batches[b].v_cache[:, :, :pos], caches[b][1][:, :, :pos])
        assert torch.isfinite(batches[b].h_out.float()).all()
    ctx.close()


def test_full_size_one_pass_group():
    """The benchmark's device-resident configuration (8 batches x 64 sequences, 512 cached
    positions, caches in HBM, the whole group in one pass); sampled sequences against the oracle,
    properties on all."""
    w = I.ATTN_WORKLOADS["attn_mixtral8x7b_decode_hbm"]
    ws = I.gen_attn_weights(w, 0)
    hs = [I.gen_attn_hidden(w, 0, b) for b in range(w.n_batches)]
    caches = [I.gen_kv_cache(w, 0, b) for b in range(w.n_batches)]
    ctx = A.AttnContext(A.config_for(w), DEV)
    ctx.set_weights(*[ws[n].to(DEV) for n in ("norm", "wq", "wk", "wv", "wo")])
    group_in = torch.cat(hs).to(DEV)                 # hidden states of the group as one tensor
    group_out = torch.zeros_like(group_in)
    batches, r0 = [], 0
    for b in range(w.n_batches):
        n = w.batch_seqs[b]
        batches.append(A.AttnBatch(caches[b][0].to(DEV), caches[b][1].to(DEV), group_in[r0:r0 + n],
                                   group_out[r0:r0 + n], w.batch_pos[b]))
        r0 += n
    ctx.forward_group(batches)
    ctx.synchronize()
    raw = {k: I.as_raw(v) for k, v in ws.items()}
    for b, rows in ((0, [0, 63]), (3, [17]), (7, [62])):
        pos = w.batch_pos[b]
        y, k2, v2 = R.attn_decode(I.as_f32(hs[b])[rows], raw["norm"], raw["wq"], raw["wk"], raw["wv"], raw["wo"],
                                  I.as_raw(caches[b][0])[rows], I.as_raw(caches[b][1])[rows], pos,
                                  w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
        got = batches[b].h_out.cpu().to(torch.float64).numpy()[rows]
        err = np.abs(got - y) - (1e-2 + 2e-2 * np.abs(y))
        assert err.max() <= 0, f"batch {b}: output off by {err.max()} beyond tolerance"
        for name, g, o in (("K", batches[b].k_cache, k2), ("V", batches[b].v_cache, v2)):
            gr, orow = widen(I.as_raw(g[rows].cpu())[:, :, pos, :]), widen(o[:, :, pos, :])
            err = np.abs(gr - orow) - (1e-2 + 2e-2 * np.abs(orow))
            assert err.max() <= 0, f"batch {b}: new {name} row off by {err.max()} beyond tolerance"
    for b in range(w.n_batches):
        pos = w.batch_pos[b]
        assert torch.equal(batches[b].k_cache[:, :, :pos].cpu(), caches[b][0][:, :, :pos])
        assert torch.equal(batches[b].v_cache[:, :, :pos].cpu(), caches[b][1][:, :, :pos])
    assert torch.isfinite(group_out.float()).all() and (group_out != 0).any(dim=1).all()
    ctx.close()


@pytest.mark.parametrize("seed", list(range(12)))
def test_seeded_sweep_of_attention_shapes(seed):
    """Head shapes, group sizes, widths, batch structures and positions drawn from a seeded
    generator; caches on the host, on the device, or mixed."""
    g = np.random.Generator(np.random.PCG64(2000 + seed))
    hd = int(g.choice([32, 64, 128]))
    per128 = 128 // hd                       # query heads come in multiples that make Hq*hd % 128 == 0
    group = int(g.integers(1, 9))
    hkv_unit = per128 // np.gcd(per128, group) if per128 > 1 else 1
    hkv = int(hkv_unit * g.integers(1, 3))
    hq = hkv * group
    if (hq * hd) % 128 != 0 or (hkv * hd) % 32 != 0:
        pytest.skip("draw outside the supported head shapes")
    d = int(g.integers(1, 5)) * 128
    nb = int(g.integers(1, 6))
    max_len = int(g.integers(8, 200))
    seqs = tuple(int(v) for v in g.integers(1, 40, size=nb))
    pos = tuple(int(v) for v in g.integers(0, max_len, size=nb))
    w = I.AttnWorkload(f"asweep{seed}", d, hq, hkv, hd, seqs, pos, max_len, rope_theta=float(g.choice([1e4, 1e6])),
                       seed=seed)
    where = [True, False, (True, False), (False, True)][seed % 4]
    run_group(w, on_host=where)
