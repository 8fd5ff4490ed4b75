"""The C-ABI library: loads, exports every symbol include/moe.h declares, and its host-only
entry points (sizing, the planner's inequality group, argument validation) behave.
No GPU needed, no compute call made."""
import ctypes as C
import math
import os
import re

import pytest

from paper_2502_06888_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="moe.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = declared_symbols()
    assert {"moe_plan", "moe_route", "moe_layer_forward", "moe_stream_experts"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in moe.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_library_exports_every_attention_symbol():
    from paper_2502_06888_amd import attn_binding as A
    lib = A.load_library()
    names = declared_symbols("moe_attn.h")
    assert "moe_attn_forward_group" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in moe_attn.h but not exported"
    assert sorted(A.ATTN_EXPORTS) == names
    assert C.sizeof(A.MoeAttnConfig) == 10 * 4
    assert C.sizeof(A.MoeAttnBatch) == 4 * 4 + 4 * 8
    assert C.sizeof(A.MoeAttnProfile) == 12 * 8
    # host-only sizing: Mixtral-8x7B attention with two staged caches of 64 x 8 x 576 x 128 bf16
    cfg = A.MoeAttnConfig(4096, 32, 8, 128, 64, 576, 1, 0, 1e6, 1e-5)
    need = A.workspace_bytes(cfg)
    cache = 64 * 8 * 576 * 128 * 2
    weights = (4096 + 2 * 1024) * 4096 * 2 + 4096 * 4096 * 2
    assert need > 4 * cache + weights and need < 4 * cache + weights + (200 << 20)
    cfg.n_layers = 32   # only the weights (and the norm vector, 8 KiB) scale with the number of layers
    assert A.workspace_bytes(cfg) - need == 31 * (weights + 4096 * 2)


def test_struct_sizes_match_header():
    assert C.sizeof(B.MoeConfig) == 12 * 4
    assert C.sizeof(B.MoePlan) == 3 * 8 + 2 * 4 + 3 * 8
    assert C.sizeof(B.MoeStats) == 12 * 8         # seven counters, two of the intermediate, three times


def test_plan_sizes_for_the_named_workloads():
    cfg = B.make_config(4096, 14336, 8, 2, max_tokens=512)
    p = B.moe_plan(cfg, 512, 8e12, 64e9, 2.5e15)
    assert p.expert_bytes == 3 * 4096 * 14336 * 2 == 352321536
    assert p.n_slots == 0 and p.window_bytes == 0
    assert p.workspace_bytes > 0 and p.workspace_bytes % 256 == 0
    assert math.isclose(p.t_io_expert_s, 352321536 / 64e9)
    # 128 rows per expert: memory time (44 us) dominates MFMA time (18 us)
    assert math.isclose(p.t_c_expert_s, 352321536 / 8e12)
    cfg = B.make_config(6144, 16384, 8, 2, n_layers=8, window_layers=2, max_tokens=512)
    p = B.moe_plan(cfg, 512)
    assert p.expert_bytes == 603979776 and p.n_slots == 16
    assert p.window_bytes == 16 * 603979776
    cfg = B.make_config(256, 512, 8, 2, max_tokens=64, dtype=B.MOE_F32)
    assert B.moe_plan(cfg, 64).expert_bytes == 1572864


@pytest.mark.parametrize("kw,status", [
    (dict(d_model=4100), B.MOE_ERR_SHAPE), (dict(d_ff=100), B.MOE_ERR_SHAPE),
    (dict(n_experts=0), B.MOE_ERR_SHAPE), (dict(n_experts=257), B.MOE_ERR_SHAPE),
    (dict(top_k=9), B.MOE_ERR_SHAPE), (dict(top_k=3, n_experts=2), B.MOE_ERR_SHAPE),
    (dict(n_shared=9), B.MOE_ERR_SHAPE), (dict(window_layers=2, n_layers=1), B.MOE_ERR_SHAPE),
    (dict(max_batches=65), B.MOE_ERR_SHAPE), (dict(dtype=7), B.MOE_ERR_INVALID_ARG),
    (dict(max_tokens=0), B.MOE_ERR_SHAPE),
])
def test_plan_rejects_bad_configs(kw, status):
    base = dict(d_model=4096, d_ff=14336, n_experts=8, top_k=2)
    base.update(kw)
    with pytest.raises(B.MoeError) as ei:
        B.moe_plan(B.make_config(**base), 1)
    assert ei.value.status == status and ei.value.message


def test_plan_null_and_range_arguments():
    lib = B.load_library()
    cfg = B.make_config(256, 512, 8, 2, max_tokens=64)
    out = B.MoePlan()
    assert lib.moe_plan(None, 1, 1.0, 1.0, 1.0, C.byref(out)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_plan(C.byref(cfg), 1, 1.0, 1.0, 1.0, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_plan(C.byref(cfg), 65, 1.0, 1.0, 1.0, C.byref(out)) == B.MOE_ERR_SHAPE
    assert b"max_tokens" in lib.moe_last_error(None)


def test_create_validates_before_touching_the_gpu():
    lib = B.load_library()
    cfg = B.make_config(256, 512, 8, 2, max_tokens=64)
    h = C.c_void_p()
    assert lib.moe_create(C.byref(cfg), None, None, None, 0, None, 0, C.byref(h)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_create(C.byref(cfg), None, None, 256, 1 << 30, None, 0, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_create(C.byref(cfg), None, None, 257, 1 << 30, None, 0, C.byref(h)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_create(C.byref(cfg), None, None, 256, 16, None, 0, C.byref(h)) == B.MOE_ERR_OOM
    cfgw = B.make_config(256, 512, 8, 2, n_layers=2, window_layers=1, max_tokens=64)
    assert lib.moe_create(C.byref(cfgw), None, None, 256, 1 << 30, None, 0, C.byref(h)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_create(C.byref(cfgw), None, None, 256, 1 << 30, 256, 16, C.byref(h)) == B.MOE_ERR_OOM
    assert lib.moe_create(C.byref(cfgw), None, None, 256, 1 << 30, 256, 1 << 40, C.byref(h)) == B.MOE_ERR_INVALID_ARG
    assert not h.value
    for fn in (lib.moe_destroy,):
        assert fn(None) == B.MOE_OK
    assert lib.moe_set_gate(None, 0, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_layer_forward(None, 0, None, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_stream_experts(None, 0, None, 0, 1) == B.MOE_ERR_INVALID_ARG


# ---- planner inequality group (paper Section 7): closed forms -------------------------------

def test_plan_batches_closed_forms():
    # only the gate transfer matters: n * tA >= tG_io
    assert B.moe_plan_batches(2.0, 0.0, 0.0, [], 0.0, 7.0, 0.0, 0) == 4      # ceil(3.5)
    assert B.moe_plan_batches(2.0, 0.0, 0.0, [], 0.0, 8.0, 0.0, 0) == 4      # exact -> no round up
    assert B.moe_plan_batches(2.0, 0.0, 0.0, [], 0.0, 0.0, 0.0, 0) == 1      # nothing to hide
    # second inequality: n (tA+tG) >= tG_io + K tE_io  ->  n >= (1 + 2*21)/2.7
    assert B.moe_plan_batches(2.6, 0.1, 0.0, [], 0.0, 1.0, 21.0, 2) == math.ceil(43 / 2.7)
    # best case (no cold expert queued): hot-expert compute does not enter
    assert B.moe_plan_batches(2.6, 0.1, 100.0, [], 50.0, 1.0, 21.0, 2) == math.ceil(43 / 2.7)
    # third: n(tA+tG) + t_hot >= tG_io + (K+1) tE_io ; fourth adds the queue and the next attention
    n3 = math.ceil((1 + 3 * 21 - 5.0) / 2.7)
    n4 = math.ceil((1 + (2 + 3) * 21 + 4.0 - 5.0 - 3 * 2.0) / 2.7)
    assert B.moe_plan_batches(2.6, 0.1, 5.0, [2.0, 2.0, 2.0], 4.0, 1.0, 21.0, 2) == max(n3, n4)
    # worst case of the paper: nobody picked a hot expert (t_hot = 0) needs a larger n
    assert B.moe_plan_batches(2.6, 0.1, 0.0, [2.0] * 3, 4.0, 1.0, 21.0, 2) >= max(n3, n4)
    # monotone: more compute per batch never needs more batches
    ns = [B.moe_plan_batches(t, 0.1, 1.0, [1.0] * 6, 5.0, 0.1, 21.0, 2) for t in (1.0, 2.0, 4.0, 8.0)]
    assert ns == sorted(ns, reverse=True)


def test_plan_batches_equals_the_oracle_search_on_a_seeded_sweep():
    """The library solves the inequality group with one division per row and a fix-up; the oracle
    tries n = 1, 2, 3, ... with the inequalities as printed.  Same n on drawn times, including
    the measured magnitudes of the streamed stacks (microseconds of compute against milliseconds
    of transfer) and cases built to sit exactly on a boundary."""
    import numpy as np
    from oracle import ref
    g = np.random.Generator(np.random.PCG64(2024))
    for trial in range(400):
        scale = float(10.0 ** g.uniform(-6, 0))
        tA, tG = float(g.uniform(0.0, 3.0)) * scale, float(g.uniform(0.0, 0.5)) * scale
        if tA + tG == 0.0:
            tA = scale
        thot = float(g.uniform(0.0, 4.0)) * scale
        q = [float(v) * scale for v in g.uniform(0.0, 2.0, size=int(g.integers(0, 9)))]
        io = [float(v) * scale * float(10.0 ** g.uniform(0, 3)) for v in g.uniform(0, 5, size=3)]
        K = int(g.integers(0, 7))
        if tA == 0.0:
            io[1] = 0.0                              # nothing but attention compute hides the gate transfer
        want = ref.plan_batches(tA, tG, thot, q, io[0], io[1], io[2], K)
        assert B.moe_plan_batches(tA, tG, thot, q, io[0], io[1], io[2], K) == want, trial
    for n in (1, 2, 7, 64, 1000):                    # exact boundaries in dyadic arithmetic
        assert B.moe_plan_batches(0.5, 0.25, 0.0, [], 0.0, 0.0, 0.75 * n, 1) == ref.plan_batches(0.5, 0.25, 0.0, [], 0.0, 0.0, 0.75 * n, 1) == n
        assert B.moe_plan_batches(0.5, 0.25, 1.0, [2.0], 0.25, 0.0, (0.75 * n + 3.0 - 0.25) / 2, 1) == \
            ref.plan_batches(0.5, 0.25, 1.0, [2.0], 0.25, 0.0, (0.75 * n + 3.0 - 0.25) / 2, 1)


def test_plan_batches_errors():
    with pytest.raises(B.MoeError):
        B.moe_plan_batches(0.0, 0.0, 0.0, [], 0.0, 1.0, 0.0, 0)              # nothing to overlap with
    with pytest.raises(B.MoeError):
        B.moe_plan_batches(-1.0, 0.0, 0.0, [], 0.0, 1.0, 0.0, 0)
    lib = B.load_library()
    assert lib.moe_plan_batches(1.0, 0.0, 0.0, None, 2, 0.0, 1.0, 0.0, 0, C.byref(C.c_int32())) == B.MOE_ERR_INVALID_ARG


def test_corr_rank_matches_oracle_on_cpu():
    """The prefetcher's ranking is host code: same scores (bit for bit, same fp64 order) and the
    same expert lists as the oracle, on random tables with unseen rows and tied scores."""
    import numpy as np
    from oracle import ref
    rng = np.random.default_rng(5)
    for E, K in [(8, 2), (64, 6), (5, 5), (16, 1)]:
        for trial in range(4):
            t = rng.integers(0, 40, size=(E, E)).astype(np.int64)
            t[rng.integers(0, E)] = 0                      # a previous expert never observed
            if trial == 3:
                t[:] = 3                                   # all scores equal: index order decides
            counts = rng.integers(0, 25, size=E).astype(np.int32)
            want_e, want_s = ref.corr_predict(t, counts, K)
            got_e, got_s = B.corr_rank(t.tolist(), counts.tolist(), K)
            assert got_e == want_e.tolist()
            assert np.array_equal(np.asarray(got_s).view(np.uint64), want_s.view(np.uint64))
    got_e, _ = B.corr_rank(np.zeros((4, 4), dtype=int).tolist(), [1, 2, 3, 4], 2)
    assert got_e == []                                     # empty table: nothing to prefetch


@pytest.mark.parametrize("kw", [
    dict(d_model=200), dict(d_model=8320), dict(head_dim=48), dict(n_q_heads=6, n_kv_heads=4),
    dict(n_q_heads=18, n_kv_heads=2), dict(n_kv_heads=0), dict(max_seqs=0), dict(max_len=0),
    dict(n_layers=0), dict(max_group_seqs=-1), dict(rope_theta=0.0), dict(rms_eps=-1.0),
    dict(n_q_heads=3, n_kv_heads=3, head_dim=32),   # n_q_heads*head_dim not a multiple of 128
])
def test_attention_config_rejections(kw):
    from paper_2502_06888_amd import attn_binding as A
    base = dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, max_seqs=64, max_len=576,
                n_layers=1, max_group_seqs=0, rope_theta=1e6, rms_eps=1e-5)
    assert A.workspace_bytes(A.MoeAttnConfig(**base)) > 0
    base.update(kw)
    with pytest.raises(B.MoeError) as ei:
        A.workspace_bytes(A.MoeAttnConfig(**base))
    assert ei.value.status == B.MOE_ERR_SHAPE and ei.value.message


def test_attention_null_arguments():
    from paper_2502_06888_amd import attn_binding as A
    lib = A.load_library()
    n = C.c_int64(0)
    cfg = A.MoeAttnConfig(4096, 32, 8, 128, 64, 576, 1, 0, 1e6, 1e-5)
    assert lib.moe_attn_workspace_bytes(None, C.byref(n)) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_attn_workspace_bytes(C.byref(cfg), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_attn_forward_group(None, 0, 0, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_attn_set_weights(None, 0, None, None, None, None, None, 0) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_attn_prefetch(None, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_attn_set_profiling(None, 1) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_attn_last_error(None)            # the calling thread's message
    lib.moe_attn_destroy(None)                      # no-op
