"""The router sums the 64 per-lane partial sums of a gate logit in the order of the xor butterfly
(32, 16, ..., 1) that the oracle's ko_gate_logits_f32 writes out.  For eight experts at a time the
kernels split the values between the lanes over the first three steps (a lane only forms the sums
it will still hold afterwards).  This test replays both orders in float32 on the CPU and checks
that the totals agree bit for bit, for every value and on adversarial magnitudes: the claim the
kernels rely on, pinned without a GPU."""
import numpy as np


def full_butterfly(v: np.ndarray) -> np.ndarray:
    """v: [64] float32 -> [64] float32, every lane ends with the total (the oracle's order)."""
    lanes = np.arange(64)
    v = v.astype(np.float32).copy()
    for m in (32, 16, 8, 4, 2, 1):
        v = (v + v[lanes ^ m]).astype(np.float32)
    return v


def halving_butterfly(a: np.ndarray) -> np.ndarray:
    """a: [8, 64] float32 (value j in lane l) -> [8] totals, by the lane-splitting order."""
    lanes = np.arange(64)
    a = a.astype(np.float32)
    h5, h4, h3 = (lanes & 32) != 0, (lanes & 16) != 0, (lanes & 8) != 0
    b = np.empty((4, 64), np.float32)
    for i in range(4):
        keep = np.where(h5, a[4 + i], a[i])
        send = np.where(h5, a[i], a[4 + i])
        b[i] = (keep + send[lanes ^ 32]).astype(np.float32)
    c = np.empty((2, 64), np.float32)
    for i in range(2):
        keep = np.where(h4, b[2 + i], b[i])
        send = np.where(h4, b[i], b[2 + i])
        c[i] = (keep + send[lanes ^ 16]).astype(np.float32)
    keep = np.where(h3, c[1], c[0])
    send = np.where(h3, c[0], c[1])
    d = (keep + send[lanes ^ 8]).astype(np.float32)
    for m in (4, 2, 1):
        d = (d + d[lanes ^ m]).astype(np.float32)
    # lane l now holds value (l >> 3) & 7; the kernels read value j from lane 8 j
    for j in range(8):
        held = d[((lanes >> 3) & 7) == j]
        assert np.all(held.view(np.uint32) == held.view(np.uint32)[0]), "lanes of one value disagree"
    return np.array([d[8 * j] for j in range(8)], np.float32)


def test_lane_splitting_sum_has_the_bits_of_the_full_butterfly():
    rng = np.random.default_rng(7)
    for trial in range(200):
        scale = np.float32(10.0 ** rng.integers(-6, 7))
        a = (rng.standard_normal((8, 64)) * scale).astype(np.float32)
        if trial % 4 == 1:   # cancellation: large terms of both signs beside small ones
            a[:, ::2] *= np.float32(1e6)
            a[:, 1::4] = -a[:, ::4]
        if trial % 4 == 2:   # many exact zeros and signed zeros
            a[rng.random((8, 64)) < 0.7] = 0.0
            a[0, :8] = -0.0
        want = np.array([full_butterfly(a[j])[0] for j in range(8)], np.float32)
        got = halving_butterfly(a)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), trial


def test_full_butterfly_leaves_the_same_total_in_every_lane():
    rng = np.random.default_rng(11)
    for _ in range(100):
        v = (rng.standard_normal(64) * 10.0 ** rng.integers(-3, 4)).astype(np.float32)
        out = full_butterfly(v)
        assert np.all(out.view(np.uint32) == out.view(np.uint32)[0])


def test_the_replayed_butterfly_is_the_oracles_order():
    """Ties the replay above to the oracle: with one element per lane (V = 1, d = 64) the oracle's
    logit is exactly the butterfly sum of the 64 products."""
    from oracle import ref
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((5, 64)) * 3.0).astype(np.float32)
    wg = rng.standard_normal((8, 64)).astype(np.float32)
    got = ref.gate_logits_f32(x, wg, 1)
    for t in range(5):
        prod = np.stack([(x[t] * wg[e]).astype(np.float32) for e in range(8)])  # fma(x, w, 0) = x * w
        want = halving_butterfly(prod)
        assert np.array_equal(got[t].view(np.uint32), want.view(np.uint32))
