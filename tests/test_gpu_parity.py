"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the same
seeded inputs.  Integer results must match bit for bit (and so must the fp32 gate logits,
which decide them); outputs within the stated tolerance."""
import numpy as np
import pytest
import torch

from paper_2502_06888_amd import binding as B
from paper_2502_06888_amd import inputs as I

import harness as H

pytestmark = pytest.mark.gpu


def run_case(w: I.Workload, tokens=None, data=None, ctx=None, layer=0):
    if data is None:
        data, _ = I.gen_layer(w, layer)
    own = ctx is None
    if own:
        ctx = H.make_ctx(w)
        H.place_layer(ctx, w, layer, data)
    bo = w.batch_offsets
    got = H.gpu_layer(ctx, w, layer, data.x, bo)
    want = H.oracle_layer(w, data, bo, tokens=tokens)
    H.check_routing(got, want, w.n_experts)
    err = H.check_output(got["y"], want.y, w.dtype, tokens)
    if own:
        ctx.close()
    return got, want, err


def test_tiny_f32_config():
    w = I.WORKLOADS["tiny_f32"]
    got, want, err = run_case(w)
    assert got["counts"].sum() == 128
    # same shapes with O(1) outputs, so that the relative part of the tolerance binds
    run_case(I.scaled(w, name="tiny_f32_loud", w_std=0.1, seed=1))


# weight scale chosen so that outputs are O(1), like the full-size layer's: the absolute part of
# the tolerance must not hide a wrong result
SMALL = I.Workload("small_bf16", "bf16", 256, 512, 8, 2, batch_tokens=(70, 0, 130, 100),
                   w_std=0.08)


@pytest.mark.parametrize("w", [
    SMALL,
    I.scaled(SMALL, name="ragged_units", d_model=128, d_ff=192, batch_tokens=(33, 1, 17)),
    I.scaled(SMALL, name="two_tiles_per_expert", n_experts=2, top_k=1, batch_tokens=(350, 350)),
    I.scaled(SMALL, name="k_equals_E", n_experts=4, top_k=4, batch_tokens=(40, 24)),
    I.scaled(SMALL, name="one_token", batch_tokens=(1,)),
    I.scaled(SMALL, name="wide", d_model=1024, d_ff=2048, batch_tokens=(64,) * 3, seed=3,
             w_std=0.04),
], ids=lambda w: w.name)
def test_bf16_small_shapes(w):
    run_case(w)


@pytest.mark.parametrize("w", [
    I.scaled(SMALL, name="large_group_ragged", d_model=1024, d_ff=64, n_experts=8, top_k=3,
             batch_tokens=(4099, 0, 4096), w_std=0.04),
    I.scaled(SMALL, name="large_group_many_experts", d_model=2048, d_ff=64, n_experts=72, top_k=4,
             batch_tokens=(8193,), w_std=0.03),
    I.scaled(SMALL, name="large_group_other_router", d_model=1024, d_ff=64, n_experts=10, top_k=2,
             batch_tokens=(8200,), w_std=0.04),
    I.scaled(SMALL, name="large_group_k_equals_E", d_model=1024, d_ff=64, n_experts=8, top_k=8,
             batch_tokens=(8192,), w_std=0.04),
    I.scaled(SMALL, name="large_group_max_experts", d_model=1024, d_ff=64, n_experts=256, top_k=2,
             batch_tokens=(9000,), w_std=0.04),  # 18 chunks of assignments: two panels of the plan's scan
    I.scaled(SMALL, name="large_group_shared_experts", d_model=512, d_ff=64, n_experts=16, top_k=4,
             n_shared=2, batch_tokens=(4100, 4129), w_std=0.05),
    I.scaled(SMALL, name="mid_group_few_experts", d_model=256, d_ff=64, n_experts=6, top_k=2,
             batch_tokens=(1500, 1501)),
    I.scaled(I.WORKLOADS["tiny_f32"], name="mid_group_f32", d_model=128, d_ff=64, n_experts=5, top_k=3,
             batch_tokens=(2100,), w_std=0.1),
], ids=lambda w: w.name)
def test_large_batch_groups_route_bit_exactly(w):
    """Batch groups of 8192 tokens and more take, where the shape allows, the router in which one
    wavefront serves several tokens: token counts that leave its last wavefront partly empty,
    several expert groups and more experts than a wavefront has lanes; and a shape it does not
    serve (experts not in whole groups), which the one-token-per-wavefront router takes, as do
    groups between 2049 and 8191 tokens (there with so few experts that the selection runs in
    registers, bf16 and fp32).  One large group has always-on experts as well, so that the gather
    (several groups of reduction steps per wavefront item, shared rows behind the routed ones) and
    the combine run their large-layer paths on every kind of row.  Logits, top-k, weights and the
    whole dispatch plan bit for bit, every output within the tolerance."""
    run_case(w)


@pytest.mark.parametrize("w", [
    I.WORKLOADS["tiny_f32"], SMALL,
    I.scaled(SMALL, name="large_group_plain_softmax", d_model=1024, d_ff=64, n_experts=8, top_k=2,
             batch_tokens=(8190, 7), w_std=0.04),
], ids=lambda w: w.name)
def test_full_softmax_weights_without_renormalisation(w):
    """renormalize = 0: routing weights are the full-softmax probabilities of the winners."""
    data, _ = I.gen_layer(w, 0)
    ctx = H.make_ctx(w, renorm=False)
    H.place_layer(ctx, w, 0, data)
    got = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
    want = H.oracle_layer(w, data, w.batch_offsets, renorm=False)
    H.check_routing(got, want, w.n_experts)
    assert np.all(got["w"].sum(axis=1) < 1.0)
    H.check_output(got["y"], want.y, w.dtype)
    ctx.close()


def test_bf16_fine_grained_with_shared_experts_and_skewed_routing():
    w = I.Workload("fine_small", "bf16", 256, 192, 64, 6, n_shared=2, batch_tokens=(16,) * 12,
                   zipf_s=1.1, corr=0.6, w_std=0.08)
    got, want, _ = run_case(w)
    assert (got["counts"] == 0).any() or got["counts"].min() < got["counts"].max()


def test_f32_with_shared_experts_and_ragged_batches():
    w = I.Workload("f32_shared", "f32", 64, 96, 6, 3, n_shared=1, batch_tokens=(5, 0, 9, 23),
                   w_std=0.15)
    run_case(w)


def test_empty_batch_group_and_reuse_of_context():
    w = SMALL
    data, _ = I.gen_layer(w)
    ctx = H.make_ctx(w)
    H.place_layer(ctx, w, 0, data)
    empty = I.scaled(w, batch_tokens=(0, 0))
    x0 = data.x[:0]
    got = H.gpu_layer(ctx, empty, 0, x0, empty.batch_offsets)
    assert got["counts"].sum() == 0 and np.all(got["exec_order"] == -1)
    assert np.array_equal(got["offsets"], np.zeros(w.n_experts + 1, np.int32))
    # the same context then serves a full group, and a shorter one after it
    run_case(w, data=data, ctx=ctx)
    short = I.scaled(w, batch_tokens=(7, 12))
    d2 = I.LayerData(x=data.x[:19], wg=data.wg, w1=data.w1, w3=data.w3, w2=data.w2)
    run_case(short, data=d2, ctx=ctx)
    ctx.close()


def test_all_tokens_on_the_same_experts_ties_go_to_low_indices():
    w = I.scaled(SMALL, name="ties", batch_tokens=(300,))
    data, _ = I.gen_layer(w)
    data.wg = torch.zeros_like(data.wg)            # all logits equal -> experts 0 and 1
    got, want, _ = run_case(w, data=data)
    assert np.all(got["idx"] == np.array([0, 1]))
    assert list(got["counts"][:2]) == [300, 300] and got["counts"][2:].sum() == 0
    assert np.allclose(got["w"], 0.5)


def test_identity_expert_closed_form_on_gpu():
    # f = 2d, last coordinate of x is 1 -> FFN(x) = silu(x) - silu(-x) = x -> Y = X
    w = I.Workload("identity", "bf16", 128, 256, 8, 2, batch_tokens=(40, 24))
    data, _ = I.gen_layer(w)
    x = I.as_f32(data.x).copy()
    x[:, -1] = 1.0
    data.x = I.to_storage(x, "bf16")
    eye = np.eye(128, dtype=np.float32)
    sel = np.zeros((256, 128), np.float32)
    sel[:, -1] = 1.0
    n = w.n_experts
    data.w1 = [I.to_storage(np.concatenate([eye, -eye], 0), "bf16")] * n
    data.w3 = [I.to_storage(sel, "bf16")] * n
    data.w2 = [I.to_storage(np.concatenate([eye, -eye], 1), "bf16")] * n
    got, want, _ = run_case(w, data=data)
    assert np.allclose(got["y"], I.as_f32(data.x), rtol=2e-2, atol=1e-2)


@pytest.fixture(scope="module")
def mixtral_layer():
    w = I.WORKLOADS["mixtral8x7b_decode"]
    data, _ = I.gen_layer(w, threads=16)
    ctx = H.make_ctx(w, max_tokens=I.WORKLOADS["mixtral8x7b_prefill"].n_tokens)
    H.place_layer(ctx, w, 0, data)
    yield w, data, ctx
    ctx.close()


def test_mixtral_decode_full_size_every_output(mixtral_layer):
    """The benchmark's headline layer in the benchmark's launch configuration: every one of the
    512 x 4096 outputs against the oracle (a few seconds of CPU time), routing in full."""
    w, data, ctx = mixtral_layer
    got, want, err = run_case(w, data=data, ctx=ctx)
    assert got["counts"].sum() == 1024 and (got["counts"] > 0).all()


def test_mixtral_decode_shape_with_skewed_routing(mixtral_layer):
    """The decode layer's weights with a batch group whose routing is lopsided: every token has
    expert 3 among its two (built by repeating the layer's own tokens that route there), so that
    one expert owns 512 rows (two full tiles) while the others get ragged tiles of every size, at the
    full reduction depths (4096 and 14336).  Every output against the oracle."""
    w, data, ctx = mixtral_layer
    base = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
    mine = np.nonzero((base["idx"] == 3).any(axis=1))[0]
    assert 100 < mine.size < 200
    pick = torch.from_numpy(np.resize(mine, w.n_tokens))       # the same tokens over and over, 512 rows
    d2 = I.LayerData(x=data.x[pick], wg=data.wg, w1=data.w1, w3=data.w3, w2=data.w2)
    got, want, err = run_case(w, data=d2, ctx=ctx)
    assert got["counts"][3] == w.n_tokens and sorted(got["counts"])[-2] < 256


def test_remainder_plane_is_skipped_at_the_decode_layer_and_both_modes_agree(mixtral_layer):
    """H travels as fp16 plus an fp16 plane with its rounding remainder.  At the decode layer's
    output scale the remainders' recorded energy stays under every expert's threshold, so the
    automatic mode (the default) computes every tile from the value plane alone; forcing the
    remainder plane changes few output bits and both are inside the tolerance on the sampled
    tokens, and within it of each other everywhere."""
    w, data, ctx = mixtral_layer
    tokens = np.arange(5, w.n_tokens, 29).astype(np.int32)
    want = H.oracle_layer(w, data, w.batch_offsets, tokens=tokens)
    ys = {}
    try:
        for hp in (1, 2):
            ctx.set_tuning(h_planes=hp)
            ctx.reset_stats()
            got = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
            H.check_routing(got, want, w.n_experts)
            H.check_output(got["y"], want.y, w.dtype, tokens)
            ys[hp] = got["y"]
            st = ctx.stats()
            assert st["h_remainder_wgs"] == 0 and st["h_saturated"] == 0
    finally:
        ctx.set_tuning(h_planes=1)
    assert np.all(np.abs(ys[1] - ys[2]) <= 1e-2 + 2e-2 * np.abs(ys[1]))
    assert (ys[1] != ys[2]).mean() < 0.2             # most outputs round to the same bf16


@pytest.mark.parametrize("w", [
    SMALL,
    I.scaled(SMALL, name="one_group", d_model=128, d_ff=64, batch_tokens=(5,)),
    I.scaled(SMALL, name="ragged_192", d_model=128, d_ff=192, batch_tokens=(33, 1, 17, 300)),
    I.scaled(SMALL, name="many_rows", d_model=256, d_ff=320, batch_tokens=(700, 3)),
], ids=lambda w: w.name)
def test_both_precision_modes_on_small_shapes(w):
    """The automatic mode and the always-both-planes mode, chosen explicitly, against the oracle:
    one group of 64, a reduction that ends inside the pipeline's look-ahead, tiles of every
    row-block class, split-K 1 to 3, both launch shapes."""
    data, _ = I.gen_layer(w, 0)
    ctx = H.make_ctx(w)
    H.place_layer(ctx, w, 0, data)
    for hp in (1, 2):
        for split_k, variant in ((1, 1), (3, 1), (2, 3)):   # 8 wavefronts x 1 unit, 4 x 2
            ctx.set_tuning(split_k, hp, variant)
            run_case(w, data=data, ctx=ctx)
    ctx.close()


def test_remainder_plane_is_taken_where_the_outputs_are_large():
    """Outputs of rms ~ 50 (16 summed experts, large activations): one fp16 plane of H would leave
    errors of several times the absolute tolerance near the outputs' zero crossings.  The automatic
    mode must notice (recorded remainder energy over the threshold), multiply the remainder
    plane and land inside the tolerance; scaled down a hundredfold the same layer needs no
    remainder plane."""
    w = I.Workload("maxima", "bf16", 512, 192, 256, 8, n_shared=8,
                   batch_tokens=tuple([5, 0, 9, 3] * 16), zipf_s=1.2, corr=0.0, w_std=0.06)
    data, _ = I.gen_layer(w, 0)
    ctx = H.make_ctx(w)
    H.place_layer(ctx, w, 0, data)
    ctx.reset_stats()
    got, want, _ = run_case(w, data=data, ctx=ctx)
    assert np.sqrt((want.y ** 2).mean()) > 20
    assert ctx.stats()["h_remainder_wgs"] > 0
    ctx.close()
    quiet = I.scaled(w, name="maxima_quiet")
    dq = I.LayerData(x=data.x, wg=data.wg, w1=data.w1, w3=data.w3,
                     w2=[I.to_storage(I.as_f32(t) * 0.01, "bf16") for t in data.w2])
    ctx = H.make_ctx(quiet)
    H.place_layer(ctx, quiet, 0, dq)
    ctx.reset_stats()
    run_case(quiet, data=dq, ctx=ctx)
    assert ctx.stats()["h_remainder_wgs"] == 0
    ctx.close()


def test_full_size_outputs_do_not_depend_on_token_order_or_batch_cut(mixtral_layer):
    """Properties that hold at any size: a token's output depends on its own row and its own
    experts only.  Permuting the tokens of the decode layer permutes the outputs bit for bit, and
    cutting the same tokens into other batches (which changes the batches-per-expert counts and
    with them the execution order) leaves every output bit unchanged."""
    w, data, ctx = mixtral_layer
    base = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
    perm = np.random.Generator(np.random.PCG64(11)).permutation(w.n_tokens)
    shuffled = H.gpu_layer(ctx, w, 0, data.x[torch.from_numpy(perm)], w.batch_offsets)
    assert np.array_equal(shuffled["y"].view(np.uint32), base["y"][perm].view(np.uint32))
    assert np.array_equal(shuffled["idx"], base["idx"][perm])
    other_cut = np.array([0, 1, 2, 300, 300, 511, 512], dtype=np.int32)
    recut = H.gpu_layer(ctx, w, 0, data.x, other_cut)
    assert np.array_equal(recut["y"].view(np.uint32), base["y"].view(np.uint32))
    assert np.array_equal(recut["counts"], base["counts"]) and np.array_equal(recut["perm"], base["perm"])


def stratified_tokens(got, n_experts, top_k, tile_rows=256, blk_rows=32):
    """Tokens whose assignments cover every (expert, tile) of the dispatch plan at least once,
    plus, for the first and the last tile of every expert, every row of the tile's first and
    last row block (the ragged tail of the expert included)."""
    idx, inv_perm, offsets = got["idx"].reshape(-1), got["inv_perm"], got["offsets"]
    pos = inv_perm - offsets[idx]                       # row of the assignment inside its expert
    tile = pos // tile_rows
    picked = set()
    for e in range(n_experts):
        mine = np.nonzero(idx == e)[0]
        if mine.size == 0:
            continue
        last_tile = int(tile[mine].max())
        for t in range(last_tile + 1):                  # one row of every tile, at a varying height
            rows = mine[tile[mine] == t]
            picked.add(int(rows[(7 * t + 3 * e) % rows.size]) // top_k)
        for t in {0, last_tile}:
            rows = mine[tile[mine] == t]
            r = pos[rows] - t * tile_rows
            last_blk = int(r.max()) // blk_rows
            for a in rows[(r < blk_rows) | (r // blk_rows == last_blk)]:
                picked.add(int(a) // top_k)
    return np.array(sorted(picked), dtype=np.int32)


def test_mixtral_prefill_full_size_stratified_outputs(mixtral_layer):
    """The prefill layer (16 tiles of 256 rows per expert) in the benchmark's launch configuration.
    The compared tokens are drawn from the dispatch plan so that every (expert, tile) contributes a
    row, and the first and last row block of every expert's first and last tile contribute all of
    theirs: several hundred tokens, each checked on all 4096 outputs."""
    wd, data, ctx = mixtral_layer
    w = I.WORKLOADS["mixtral8x7b_prefill"]
    x = I.gen_x_gaussian(w)
    d2 = I.LayerData(x=x, wg=data.wg, w1=data.w1, w3=data.w3, w2=data.w2)
    got = H.gpu_layer(ctx, w, 0, x, w.batch_offsets)
    assert got["counts"].sum() == 32768
    tokens = stratified_tokens(got, w.n_experts, w.top_k)
    n_tiles = int(sum((c + 255) // 256 for c in got["counts"]))
    assert tokens.size >= n_tiles >= 128
    want = H.oracle_layer(w, d2, w.batch_offsets, tokens=tokens)
    H.check_routing(got, want, w.n_experts)
    H.check_output(got["y"], want.y, w.dtype, tokens)
    try:                                             # always both planes, on full tiles
        ctx.set_tuning(h_planes=2)
        got2 = H.gpu_layer(ctx, w, 0, x, w.batch_offsets)
        H.check_output(got2["y"], want.y, w.dtype, tokens)
        assert np.all(np.abs(got2["y"] - got["y"]) <= 1e-2 + 2e-2 * np.abs(got["y"]))
    finally:
        ctx.set_tuning(h_planes=1)


def test_prefill_size_outputs_permute_with_the_tokens_in_every_workgroup_order(mixtral_layer):
    """The same properties on full tiles (16 tiles of 256 rows per expert, panel order of the
    workgroups, two-unit shape): permuting the 16384 tokens moves every token to another row of
    another tile and permutes the outputs bit for bit; another panel shape and the one-unit shape
    change no bit either.  (Routing of a token does not depend on its neighbours, so the permuted
    run must also select the same experts with the same weights.)"""
    wd, data, ctx = mixtral_layer
    w = I.WORKLOADS["mixtral8x7b_prefill"]
    x = I.gen_x_gaussian(w)
    base = H.gpu_layer(ctx, w, 0, x, w.batch_offsets)
    perm = np.random.Generator(np.random.PCG64(12)).permutation(w.n_tokens)
    shuffled = H.gpu_layer(ctx, w, 0, x[torch.from_numpy(perm)], w.batch_offsets)
    assert np.array_equal(shuffled["idx"], base["idx"][perm])
    assert np.array_equal(shuffled["y"].view(np.uint32), base["y"][perm].view(np.uint32))
    try:
        for variant in (51, 13):                     # 16 x 2 panels with one unit, 1 x 32 with two
            ctx.set_tuning(0, 0, variant)
            other = H.gpu_layer(ctx, w, 0, x, w.batch_offsets)
            assert np.array_equal(other["y"].view(np.uint32), base["y"].view(np.uint32)), variant
    finally:
        ctx.set_tuning(0, 0, -1)


@pytest.mark.parametrize("w", [
    I.scaled(SMALL, name="shapes_ragged", d_model=192, d_ff=448, n_experts=4, batch_tokens=(33, 1, 200)),
    I.scaled(SMALL, name="shapes_full_tiles", n_experts=2, top_k=1, batch_tokens=(300, 300)),
    I.scaled(SMALL, name="shapes_many_tiles", d_model=192, d_ff=448, n_experts=3, top_k=1,
             batch_tokens=(700, 650, 300)),
], ids=lambda w: w.name)
def test_every_launch_shape_gives_the_same_bits(w):
    """The launch shapes (8 or 7 wavefronts x 1 unit, 4 x 2 units) and, on full tiles, the order
    in which the workgroups take the (tile, unit group) items (panels of 1 to 32 tiles, short
    last panels and narrow last column blocks included) only change who computes what and when:
    every accumulator still adds the same products in the same order, so the outputs must be
    identical bit for bit, and right."""
    data, _ = I.gen_layer(w, 0)
    ctx = H.make_ctx(w)
    H.place_layer(ctx, w, 0, data)
    want = H.oracle_layer(w, data, w.batch_offsets)
    base = None
    for variant in (1, 2, 3, 11, 21, 32, 43, 53, 61):
        ctx.set_tuning(1, 2, variant)
        got = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
        if base is None:
            base = got["y"]
            H.check_routing(got, want, w.n_experts)
            H.check_output(got["y"], want.y, w.dtype)
        assert np.array_equal(got["y"], base), f"variant {variant} differs from variant 1"
    for bad in (70, 104, -2):                        # tens digit past the six panel shapes, or below -1
        with pytest.raises(B.MoeError) as ei:
            ctx.set_tuning(1, 2, bad)
        assert ei.value.status == B.MOE_ERR_INVALID_ARG
    with pytest.raises(B.MoeError) as ei:            # 1 = automatic, 2 = always both planes, nothing else
        ctx.set_tuning(1, 3, 0)
    assert ei.value.status == B.MOE_ERR_INVALID_ARG
    ctx.set_tuning(1, 2, -1)                         # the defaults again
    got = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)
    assert np.array_equal(got["y"], base)
    ctx.close()


def test_maximum_experts_topk_shared_and_batches():
    """The configured maxima at once: 256 routed experts, top-8, 8 shared experts, 64 batches (some
    empty), more assignments than one plan chunk, most experts with a handful of tokens and many
    with none."""
    w = I.Workload("maxima", "bf16", 512, 192, 256, 8, n_shared=8,          # d > E: the skewed-routing
                   batch_tokens=tuple([5, 0, 9, 3] * 16), zipf_s=1.2, corr=0.0, w_std=0.06)  # inputs need it
    assert w.n_batches == 64 and w.n_tokens * w.top_k > 1024
    got, want, err = run_case(w)
    assert (got["counts"] == 0).any() and got["counts"].sum() == w.n_tokens * 8


def test_f32_maximum_topk_and_many_experts():
    w = I.Workload("maxima_f32", "f32", 64, 128, 128, 8, n_shared=2, batch_tokens=(7, 0, 11, 2, 30),
                   w_std=0.1)
    run_case(w)


def test_per_tile_choice_holds_the_tolerance_across_output_scales():
    """The same layer with W2 scaled by 1, 2, 4, ... 128: the outputs grow from rms ~1 to rms ~100,
    the absolute part of the tolerance shrinks next to them, and somewhere on the way the tiles
    start to take the remainder plane of the intermediate.  At every scale, also where some tiles
    take it and others do not, the default mode must stay inside the tolerance; the number of
    workgroups that take the remainder plane never falls as the outputs grow."""
    w = I.Workload("scales", "bf16", 512, 2048, 4, 2, n_shared=1, batch_tokens=(90, 130, 75), w_std=0.05)
    data, _ = I.gen_layer(w, 0)
    taken = []
    for scale in (1, 2, 4, 8, 16, 32, 64, 128):
        d2 = I.LayerData(x=data.x, wg=data.wg, w1=data.w1, w3=data.w3,
                         w2=[I.to_storage(I.as_f32(t) * scale, "bf16") for t in data.w2])   # exact: a power of two
        ctx = H.make_ctx(w)
        H.place_layer(ctx, w, 0, d2)
        ctx.reset_stats()
        got, want, err = run_case(w, data=d2, ctx=ctx)
        taken.append(ctx.stats()["h_remainder_wgs"])
        ctx.close()
    assert taken[0] == 0 and taken[-1] > 0, taken
    assert taken == sorted(taken), taken


def test_intermediate_values_beyond_the_fp16_range_are_clamped_and_counted():
    """Activations so large that silu(gate) * up leaves the fp16 range (|h| > 65504): the values are
    clamped, counted in the stats, and the outputs stay finite.  (No comparison with the oracle:
    a layer that saturates its intermediate is outside what the format serves.)"""
    w = SMALL
    data, _ = I.gen_layer(w, 0)
    d2 = I.LayerData(x=I.to_storage(I.as_f32(data.x) * 400.0, "bf16"), wg=data.wg, w1=data.w1, w3=data.w3, w2=data.w2)
    ctx = H.make_ctx(w)
    H.place_layer(ctx, w, 0, d2)
    ctx.reset_stats()
    got = H.gpu_layer(ctx, w, 0, d2.x, w.batch_offsets)
    assert np.all(np.isfinite(got["y"]))
    assert ctx.stats()["h_saturated"] > 0
    ctx.reset_stats()
    got = H.gpu_layer(ctx, w, 0, data.x, w.batch_offsets)      # the same context on sane inputs: nothing clamped
    assert ctx.stats()["h_saturated"] == 0
    ctx.close()


def test_weights_beyond_the_fp16_range_are_placed_scaled():
    """W2 is placed as fp16.  An expert whose W2 holds a weight beyond 65504 is stored times a
    power of two that brings it into range (exact), and the outputs are scaled back: same oracle,
    same tolerance.  Non-finite weights are refused."""
    w = SMALL
    data, _ = I.gen_layer(w, 0)
    big = data.w2[0].clone()
    big[3, 5] = 1.0e5
    big[7, 1] = -3.0e5
    d2 = I.LayerData(x=data.x, wg=data.wg, w1=data.w1, w3=data.w3, w2=[big] + list(data.w2[1:]))
    got, want, _ = run_case(w, data=d2)
    assert np.abs(want.y).max() > 1e3                # the large weights are felt
    ctx = H.make_ctx(w)
    dev = ctx.device
    bad = data.w2[0].clone()
    bad[0, 0] = float("inf")
    with pytest.raises(B.MoeError) as ei:
        ctx.set_expert(0, 0, data.w1[0].to(dev), data.w3[0].to(dev), bad.to(dev))
    assert ei.value.status == B.MOE_ERR_SHAPE
    ctx.set_expert(0, 0, data.w1[0].to(dev), data.w3[0].to(dev), data.w2[0].to(dev))   # finite: fine
    ctx.close()


@pytest.mark.parametrize("seed", list(range(16)))
def test_seeded_sweep_of_small_configurations(seed):
    """Shapes drawn from a seeded generator: widths and expert sizes that are not powers of two,
    1..40 experts, top-k up to 8, shared experts, empty and one-token batches, skewed routing; both
    precisions.  Each draw goes through the same routing (bit-exact) and output checks."""
    g = np.random.Generator(np.random.PCG64(1000 + seed))
    bf16 = bool(seed % 4 != 3)
    step = 64 if bf16 else 4
    d = int(g.integers(2, 9)) * step * (1 if bf16 else 8)
    f = int(g.integers(2, 13)) * step * (1 if bf16 else 8)
    E = int(g.integers(1, 41))
    k = int(g.integers(1, min(E, 8) + 1))
    S = int(g.integers(0, 3))
    nb = int(g.integers(1, 7))
    sizes = [int(v) for v in g.integers(0, 90, size=nb)]
    if seed % 5 == 0:
        sizes[int(g.integers(0, nb))] = 1
    if sum(sizes) == 0:
        sizes[0] = 3
    w = I.Workload(f"sweep{seed}", "bf16" if bf16 else "f32", d, f, E, k, n_shared=S,
                   batch_tokens=tuple(sizes), zipf_s=1.1 if seed % 2 else 0.0, seed=seed,
                   w_std=float(1.1 / (d * f) ** 0.25))
    run_case(w)
