"""Pins for the oracle's 4-bit group (de)quantisation, Eq. 8 of the paper's quantisation
paragraph.  The paper prints no numbers for it; the pins are a hand-worked group, a library
(NumPy broadcasting) evaluation of the same formula on other data, closed forms (code equal to the
zero point gives exactly 0; integer-valued s and z give exact integers), and the method's own
error bound: quantising with the textbook min/max parameters and dequantising again moves no
weight by more than half a step."""
import numpy as np
import torch

from oracle import ref


def bf16_bits(a) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_val(bits) -> np.ndarray:
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()


def test_hand_worked_group():
    # one row, one group of 4 (group size is a parameter): s = 0.5, z = 3.0
    q = np.array([[0x21, 0xF7]], dtype=np.uint8)             # codes by column: 1, 2, 7, 15
    w = ref.dequant_q4(q, bf16_bits([[0.5]]), bf16_bits([[3.0]]), group=4)
    assert w.tolist() == [[-1.0, -0.5, 2.0, 6.0]]


def test_matches_numpy_broadcast_and_nibble_order():
    rng = np.random.default_rng(0)
    rows, cols, group = 5, 256, 64
    codes = rng.integers(0, 16, size=(rows, cols))
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    s = bf16_bits(rng.uniform(1e-3, 1e-2, size=(rows, cols // group)))
    z = bf16_bits(rng.uniform(0, 15, size=(rows, cols // group)))
    want = np.repeat(bf16_val(s), group, axis=1) * (codes - np.repeat(bf16_val(z), group, axis=1))
    got = ref.dequant_q4(q, s, z, group)
    assert np.array_equal(got, want)                          # one fp64 product each, same operands


def test_zero_point_code_is_exact_zero_and_integers_stay_integers():
    rows, cols, group = 3, 128, 64
    codes = np.full((rows, cols), 9)
    q = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    w = ref.dequant_q4(q, bf16_bits(np.full((rows, 2), 0.0123)), bf16_bits(np.full((rows, 2), 9.0)), group)
    assert not w.any()
    w = ref.dequant_q4(q, bf16_bits(np.full((rows, 2), 2.0)), bf16_bits(np.full((rows, 2), 4.0)), group)
    assert np.array_equal(w, np.full((rows, cols), 10.0))


def test_round_trip_error_is_at_most_half_a_step():
    rng = np.random.default_rng(1)
    rows, cols, group = 16, 512, 64
    w = rng.standard_normal((rows, cols)) * 0.02
    g = w.reshape(rows, cols // group, group)
    lo, hi = g.min(axis=2), g.max(axis=2)
    s = bf16_bits((hi - lo) / 15.0 * 1.01)                    # a little wider: s and z round to bf16
    sv = bf16_val(s)
    z = bf16_bits(-lo / sv)
    q = ref.quant_q4(w, s, z, group)
    back = ref.dequant_q4(q, s, z, group)
    step = np.repeat(sv, group, axis=1)
    codes = np.stack([q & 15, q >> 4], axis=2).reshape(rows, cols)
    inner = (codes > 0) & (codes < 15)                        # not clamped
    assert inner.mean() > 0.8
    assert np.all(np.abs(back - w)[inner] <= 0.5 * step[inner] * (1 + 1e-12))
    assert np.all(np.abs(back - w) <= 1.0 * step)             # clamped ends: within one step here
    # quantising the dequantised weights again gives the same codes (fixed point)
    assert np.array_equal(ref.quant_q4(back, s, z, group), q)


def test_double_weights_feed_the_expert_like_float32_ones():
    rng = np.random.default_rng(2)
    d, f = 64, 128
    w1, w3 = rng.standard_normal((f, d)) * 0.1, rng.standard_normal((f, d)) * 0.1
    w2 = rng.standard_normal((d, f)) * 0.1
    x = rng.standard_normal(d)
    w1f, w3f, w2f = (a.astype(np.float32) for a in (w1, w3, w2))
    y64 = ref.expert_ffn(x, w1f.astype(np.float64), w3f.astype(np.float64), w2f.astype(np.float64))
    y32 = ref.expert_ffn(x, w1f, w3f, w2f)
    assert np.array_equal(y64, y32)                            # same values, two storage types
    g = w1 @ x
    want = w2 @ ((g / (1 + np.exp(-g))) * (w3 @ x))
    assert np.allclose(ref.expert_ffn(x, w1, w3, w2), want, rtol=1e-12, atol=1e-14)


def test_rounding_to_bf16_matches_the_library_conversion_and_hand_ties():
    rng = np.random.default_rng(3)
    vals = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                           [1.0, -1.0, 0.0, 3.0e38, 1e-39]]).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float64).numpy()    # library RNE
    got = np.array([ref.round_bf16(float(v)) for v in vals])
    assert np.array_equal(got, want)
    # 8 significant bits: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1); 1 + 3*2^-8 -> 1 + 2^-6
    assert ref.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert ref.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert ref.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7        # just above the tie
    # a double that rounds differently when it goes through float32 first (double rounding)
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert float(np.float32(x)) == 1.0 + 2.0 ** -8 and ref.round_bf16(x) == 1.0 + 2.0 ** -7


def test_dequant_to_original_precision_is_the_rounded_exact_value():
    rng = np.random.default_rng(4)
    rows, cols = 4, 128
    q = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
    s = bf16_bits(rng.uniform(1e-3, 1e-2, size=(rows, 2)))
    z = bf16_bits(rng.uniform(6, 9, size=(rows, 2)))
    exact = ref.dequant_q4(q, s, z)
    rounded = ref.dequant_q4(q, s, z, to_bf16=True)
    assert np.array_equal(rounded, np.vectorize(ref.round_bf16)(exact))
    assert np.all(np.abs(rounded - exact) <= np.abs(exact) * 2.0 ** -8)
    as_f32 = rounded.astype(np.float32)
    assert np.array_equal(torch.from_numpy(as_f32).to(torch.bfloat16).to(torch.float32).numpy(), as_f32)

