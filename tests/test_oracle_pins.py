"""Pins for the CPU oracle: each part is checked against something that is not the
oracle itself -- brute force, closed forms, library routines, a hand-worked layer.
CPU only."""
import itertools
import json
import math
import os

import numpy as np
import pytest
from scipy.special import expit, softmax

from oracle import ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- gate logits

def test_logits_exact_on_small_integers():
    # Integer inputs make every partial sum exact in fp32, so any summation order
    # must reproduce the integer matrix product exactly: pins indexing/strides.
    g = rng(1)
    for V, d in ((4, 256), (8, 512), (8, 1000), (4, 8)):
        x = g.integers(-8, 9, size=(5, d)).astype(np.float32)
        wg = g.integers(-8, 9, size=(7, d)).astype(np.float32)
        want = x.astype(np.int64) @ wg.astype(np.int64).T
        got = ref.gate_logits_f32(x, wg, V)
        assert np.array_equal(got.astype(np.int64), want)
        assert np.array_equal(ref.gate_logits_f64(x, wg), want.astype(np.float64))


def test_logits_within_fp32_bound_of_exact():
    g = rng(2)
    x = g.standard_normal((16, 4096)).astype(np.float32)
    wg = (0.02 * g.standard_normal((8, 4096))).astype(np.float32)
    exact = x.astype(np.float64) @ wg.astype(np.float64).T
    got = ref.gate_logits_f32(x, wg, 8).astype(np.float64)
    # |error| <= (depth) * eps * sum|x||w| ; depth = 64 fma + 6 adds
    bound = 70 * 2.0**-24 * (np.abs(x).astype(np.float64) @ np.abs(wg).astype(np.float64).T)
    assert np.all(np.abs(got - exact) <= bound)
    assert np.allclose(ref.gate_logits_f64(x, wg), exact, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("V", [4, 8])
def test_logit_order_lane_ownership(V):
    # Hand-derived from the stated order: element 0 and element 64*V belong to lane 0,
    # element V to lane 1.  Lane 0 computes fma(1,1,2^24) = 2^24 (tie to even), lane 1
    # holds -2^24, the butterfly gives 0.  The exact sum is 1 and a plain left-to-right
    # fp32 sum also gives 1, so only the stated lane ownership produces 0.
    d = 64 * V * 2
    x = np.zeros((1, d), np.float32)
    w = np.ones((1, d), np.float32)
    x[0, 0] = 2.0**24
    x[0, V] = -(2.0**24)
    x[0, 64 * V] = 1.0
    assert ref.gate_logits_f32(x, w, V)[0, 0] == 0.0
    assert ref.gate_logits_f64(x, w)[0, 0] == 1.0
    # elements 0 and 1 share a 16-byte vector, hence a lane: lane 0 folds 2^24 then 1 (lost to
    # rounding), lane 1 holds -2^24, the total is 0; were lanes to own single elements, the 1 would
    # sit in a lane of its own and survive
    x = np.zeros((1, d), np.float32)
    x[0, 0], x[0, 1], x[0, V] = 2.0**24, 1.0, -(2.0**24)
    assert ref.gate_logits_f32(x, w, V)[0, 0] == 0.0
    # within one lane the order is increasing i: (1 then 2^24) and (2^24 then 1) agree
    # here, but (2^24, 1, 1): ((2^24+1)->2^24)+1 -> 2^24, whereas 1+1 first gives 2^24+2.
    d3 = 64 * V * 3
    x = np.zeros((1, d3), np.float32)
    w = np.ones((1, d3), np.float32)
    x[0, 0], x[0, 64 * V], x[0, 128 * V] = 2.0**24, 1.0, 1.0
    assert ref.gate_logits_f32(x, w, V)[0, 0] == 2.0**24
    x[0, 0], x[0, 64 * V], x[0, 128 * V] = 1.0, 1.0, 2.0**24
    assert ref.gate_logits_f32(x, w, V)[0, 0] == 2.0**24 + 2


# ---------------------------------------------------------------------- top-k

def brute_topk(row, k):
    order = sorted(range(len(row)), key=lambda e: (-float(row[e]), e))
    return order[:k]


def test_topk_bruteforce_with_ties():
    g = rng(3)
    for E, k in ((8, 2), (64, 6), (5, 5), (3, 1), (16, 8)):
        logits = g.standard_normal((40, E)).astype(np.float32)
        logits[::3] = np.round(logits[::3])          # many exact ties
        logits[5] = 0.0                              # all equal -> 0,1,..,k-1
        got = ref.topk(logits, k)
        for t in range(logits.shape[0]):
            assert list(got[t]) == brute_topk(logits[t], k)
        assert list(got[5]) == list(range(k))


def test_topk_duplicate_gate_rows_lower_index_wins():
    g = rng(4)
    x = g.standard_normal((32, 512)).astype(np.float32)
    wg = (0.02 * g.standard_normal((8, 512))).astype(np.float32)
    wg[6] = wg[2]                                    # equal logits for experts 2 and 6
    logits = ref.gate_logits_f32(x, wg, 8)
    assert np.array_equal(logits[:, 2], logits[:, 6])
    idx = ref.topk(logits, 2)
    for t in range(32):
        row = list(idx[t])
        if 6 in row:
            assert 2 in row and row.index(2) < row.index(6)


# -------------------------------------------------------------------- weights

def test_weights_sum_to_one_k1_kE_and_shift():
    g = rng(5)
    E = 8
    logits = (3 * g.standard_normal((50, E))).astype(np.float32)
    for k in (1, 2, 6, 8):
        idx = ref.topk(logits, k)
        w = ref.gate_weights(logits, idx)
        assert np.all(np.abs(w.sum(1) - 1.0) <= k * 2.0**-52)
        assert np.all(np.diff(w, axis=1) <= 0)       # listed by decreasing weight
        if k == 1:
            assert np.all(w == 1.0)
        if k == E:                                   # textbook softmax (library routine)
            full = softmax(logits.astype(np.float64), axis=1)
            assert np.allclose(w, np.take_along_axis(full, idx.astype(np.int64), 1), rtol=1e-13)
        # renormalised weights == softmax restricted to the winners
        sel = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), 1)
        assert np.allclose(w, softmax(sel, axis=1), rtol=1e-13)
        # un-renormalised variant == full softmax at the winners
        w0 = ref.gate_weights(logits, idx, renorm=False)
        full = softmax(logits.astype(np.float64), axis=1)
        assert np.allclose(w0, np.take_along_axis(full, idx.astype(np.int64), 1), rtol=1e-13)
    # shift invariance (shift exactly representable)
    q = (np.round(logits * 1024) / 1024).astype(np.float32)
    idx = ref.topk(q, 2)
    shifted = (q.astype(np.float64) + 4.0).astype(np.float32)
    assert np.all(shifted.astype(np.float64) - 4.0 == q)
    assert np.allclose(ref.gate_weights(shifted, idx), ref.gate_weights(q, idx), rtol=1e-12)


# ------------------------------------------------------------------- dispatch

def test_dispatch_against_stable_sort_and_bruteforce():
    g = rng(6)
    for (N, k, E, bt) in ((37, 2, 8, (10, 0, 20, 7)), (64, 6, 64, (16,) * 4), (5, 1, 4, (5,)),
                          (0, 2, 8, (0, 0))):
        logits = g.standard_normal((N, E)).astype(np.float32)
        if N > 8:
            logits[:, E - 1] = -50.0                 # one expert never selected
        idx = ref.topk(logits, k) if N else np.empty((0, k), np.int32)
        bo = np.concatenate([[0], np.cumsum(bt)]).astype(np.int32)
        dsp = ref.dispatch(idx, E, bo)
        flat = idx.reshape(-1)
        assert np.array_equal(dsp.counts, np.bincount(flat, minlength=E))
        assert dsp.counts.sum() == N * k and dsp.offsets[E] == N * k
        assert np.array_equal(dsp.offsets, np.concatenate([[0], np.cumsum(dsp.counts)]))
        assert np.array_equal(dsp.perm, np.argsort(flat, kind="stable"))     # library routine
        assert np.array_equal(dsp.perm[dsp.inv_perm], np.arange(N * k))
        assert np.array_equal(dsp.inv_perm[dsp.perm], np.arange(N * k))
        keys = flat[dsp.perm]
        assert np.all(np.diff(keys) >= 0)
        same = np.diff(keys) == 0
        assert np.all(np.diff(dsp.perm)[same] > 0)   # stable within an expert
        # brute-force nbatch and execution order
        nb = [len({b for b in range(len(bt)) for t in range(bo[b], bo[b + 1]) if e in idx[t]})
              for e in range(E)]
        assert list(dsp.nbatch) == nb
        active = [e for e in range(E) if dsp.counts[e] > 0]
        want = sorted(active, key=lambda e: (-nb[e], -int(dsp.counts[e]), e))
        assert dsp.n_active == len(active)
        assert list(dsp.exec_order[:dsp.n_active]) == want
        assert np.all(dsp.exec_order[dsp.n_active:] == -1)


def test_exec_order_prefers_experts_shared_across_batches():
    # expert 3 has few tokens but appears in both batches; expert 1 has many tokens in one.
    idx = np.array([[1], [1], [1], [3], [3], [0]], np.int32)
    dsp = ref.dispatch(idx, 4, np.array([0, 4, 6], np.int32))
    assert list(dsp.nbatch) == [1, 1, 0, 2]
    assert list(dsp.exec_order) == [3, 1, 0, -1]


# ------------------------------------------------------------ experts + combine

def np_swiglu(x, w1, w3, w2):
    x = x.astype(np.float64)
    g = x @ w1.astype(np.float64).T
    return ((g * expit(g)) * (x @ w3.astype(np.float64).T)) @ w2.astype(np.float64).T


def make_layer(g, N, d, f, E, S=0, std=0.1):
    x = g.standard_normal((N, d)).astype(np.float32)
    wg = (0.5 * g.standard_normal((E, d))).astype(np.float32)
    w1 = [(std * g.standard_normal((f, d))).astype(np.float32) for _ in range(E + S)]
    w3 = [(std * g.standard_normal((f, d))).astype(np.float32) for _ in range(E + S)]
    w2 = [(std * g.standard_normal((d, f))).astype(np.float32) for _ in range(E + S)]
    return x, wg, w1, w3, w2


def test_handworked_layer_fixture():
    with open(os.path.join(GOLD, "handworked_layer.json")) as fh:
        G = json.load(fh)
    L = math.log(3.0)

    def arr(a):
        return np.array([[L if v == "L" else v for v in row] for row in a], dtype=np.float32)

    x = arr(G["x"])
    wg = arr(G["wg_in_L"])
    w1 = [arr(G["experts"][str(e)]["w1"]) for e in range(3)]
    w3 = [arr(G["experts"][str(e)]["w3"]) for e in range(3)]
    w2 = [arr(G["experts"][str(e)]["w2"]) for e in range(3)]
    r = ref.moe_layer(x, wg, w1, w3, w2, 2, [0, 1], "f32")
    assert r.idx.tolist() == G["expect"]["idx"]
    assert np.allclose(r.w, G["expect"]["w"], rtol=0, atol=2e-7)
    assert np.allclose(r.y, L * np.array(G["expect"]["y_in_L"]), rtol=0, atol=1e-6)


def test_identity_expert_closed_form():
    # f = 2d, last coordinate of x is 1: W1=[I;-I], W3 selects the constant, W2=[I,-I]
    # => FFN(x) = silu(x) - silu(-x) = x, so Y = X for any routing.
    g = rng(7)
    N, d, E, k = 24, 16, 8, 2
    f = 2 * d
    x = g.standard_normal((N, d)).astype(np.float32)
    x[:, -1] = 1.0
    wg = g.standard_normal((E, d)).astype(np.float32)
    eye = np.eye(d, dtype=np.float32)
    w1 = [np.concatenate([eye, -eye], 0)] * E
    sel = np.zeros((f, d), np.float32)
    sel[:, -1] = 1.0
    w3 = [sel] * E
    w2 = [np.concatenate([eye, -eye], 1)] * E
    r = ref.moe_layer(x, wg, w1, w3, w2, k, [0, N], "f32")
    assert np.allclose(r.y, x.astype(np.float64), rtol=0, atol=1e-13)
    # pluggable identity expert: the combine alone
    y = ref.moe_forward(x, r.idx, r.w, None, None, None, E, expert_kind=1)
    assert np.allclose(y, x.astype(np.float64), rtol=0, atol=1e-14)


def test_identical_experts_equal_dense_ffn():
    g = rng(8)
    N, d, f, E, k = 20, 32, 48, 8, 2
    x, wg, w1, w3, w2 = make_layer(g, N, d, f, 1)
    wg = g.standard_normal((E, d)).astype(np.float32)
    r = ref.moe_layer(x, wg, w1 * E, w3 * E, w2 * E, k, [0, N], "f32")
    assert np.allclose(r.y, np_swiglu(x, w1[0], w3[0], w2[0]), rtol=1e-12, atol=1e-14)


def test_single_live_expert():
    g = rng(9)
    N, d, f, E, k = 30, 32, 64, 8, 2
    x, wg, w1, w3, w2 = make_layer(g, N, d, f, E)
    live = 5
    w2z = [w if e == live else np.zeros_like(w) for e, w in enumerate(w2)]
    r = ref.moe_layer(x, wg, w1, w3, w2z, k, [0, N], "f32")
    dense = np_swiglu(x, w1[live], w3[live], w2[live])
    for t in range(N):
        row = list(r.idx[t])
        if live in row:
            assert np.allclose(r.y[t], r.w[t, row.index(live)] * dense[t], rtol=1e-12, atol=1e-15)
        else:
            assert np.all(r.y[t] == 0.0)
    assert any(live in list(r.idx[t]) for t in range(N))


def test_tiny_config_against_dense_numpy_mixture():
    # Independent fp64 NumPy derivation: evaluate *all* experts densely, build the
    # routing-weight matrix from the selected (idx, w), contract.
    g = rng(10)
    N, d, f, E, k, S = 64, 256, 512, 8, 2, 0
    x, wg, w1, w3, w2 = make_layer(g, N, d, f, E, S, std=0.02)
    wg = (0.02 * g.standard_normal((E, d))).astype(np.float32)
    r = ref.moe_layer(x, wg, w1, w3, w2, k, [0, 16, 32, 48, 64], "f32")
    dense = np.stack([np_swiglu(x, w1[e], w3[e], w2[e]) for e in range(E)], 1)     # [N,E,d]
    R = np.zeros((N, E))
    np.put_along_axis(R, r.idx.astype(np.int64), r.w, 1)
    assert np.allclose(r.y, np.einsum("ne,ned->nd", R, dense), rtol=1e-11, atol=1e-14)


def test_k_equals_E_is_full_softmax_mixture_with_shared_and_token_subset():
    g = rng(11)
    N, d, f, E, S = 12, 16, 32, 4, 2
    x, wg, w1, w3, w2 = make_layer(g, N, d, f, E, S)
    r = ref.moe_layer(x, wg, w1, w3, w2, E, [0, N], "f32", n_shared=S)
    p = softmax(ref.gate_logits_f32(x, wg, 4).astype(np.float64), axis=1)
    want = sum(p[:, [e]] * np_swiglu(x, w1[e], w3[e], w2[e]) for e in range(E))
    want = want + sum(np_swiglu(x, w1[E + s], w3[E + s], w2[E + s]) for s in range(S))
    assert np.allclose(r.y, want, rtol=1e-11, atol=1e-14)
    sub = np.array([7, 0, 3], np.int32)
    r2 = ref.moe_layer(x, wg, w1, w3, w2, E, [0, N], "f32", n_shared=S, tokens=sub)
    assert np.array_equal(r2.y, r.y[sub])


def test_bf16_weight_path_matches_float_path():
    import torch
    g = rng(12)
    N, d, f, E, k = 6, 64, 128, 4, 2
    x, wg, w1, w3, w2 = make_layer(g, N, d, f, E)

    def bf(a):
        t = torch.from_numpy(a).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16), t.to(torch.float32).numpy()

    raw1, f1 = zip(*[bf(a) for a in w1])
    raw3, f3 = zip(*[bf(a) for a in w3])
    raw2, f2 = zip(*[bf(a) for a in w2])
    ra = ref.moe_layer(x, wg, list(raw1), list(raw3), list(raw2), k, [0, N], "bf16")
    rb = ref.moe_layer(x, wg, list(f1), list(f3), list(f2), k, [0, N], "bf16")
    assert np.array_equal(ra.y, rb.y)
    one = ref.expert_ffn(x[0].astype(np.float64), f1[0], f3[0], f2[0])
    assert np.allclose(one, np_swiglu(x[:1], f1[0], f3[0], f2[0])[0], rtol=1e-12, atol=1e-15)


def test_output_invariant_under_expert_relabelling():
    # Reordering experts changes execution order only (Section 5): permuting the expert
    # labels consistently must leave Y unchanged up to fp64 summation order of the k slots.
    g = rng(13)
    N, d, f, E, k = 16, 32, 64, 8, 2
    x, wg, w1, w3, w2 = make_layer(g, N, d, f, E)
    r = ref.moe_layer(x, wg, w1, w3, w2, k, [0, 8, 16], "f32")
    p = g.permutation(E)
    r2 = ref.moe_layer(x, wg[p], [w1[i] for i in p], [w3[i] for i in p], [w2[i] for i in p], k,
                       [0, 8, 16], "f32")
    assert np.allclose(r.y, r2.y, rtol=1e-12, atol=1e-15)
    assert np.array_equal(np.sort(p[r2.idx], 1), np.sort(r.idx, 1))
