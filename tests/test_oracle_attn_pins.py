"""Pins of the attention-layer oracle against library routines, closed forms and invariants.

The paper takes the attention arithmetic from the models it runs (Section 2.1: a block is an
attention layer, an MoE layer and two normalisation layers); the oracle writes the textbook
definition out.  Nothing here calls the oracle to produce its own expected values.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import attn_ref as R
from paper_2502_06888_amd import inputs as I


def test_bf16_rounding_matches_library_cast():
    g = np.random.default_rng(1)
    v = np.concatenate([g.standard_normal(4000).astype(np.float32) * s for s in (1e-3, 1.0, 300.0)])
    v = np.concatenate([v, np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38])])
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([R.bf16_bits(float(a)) for a in v], dtype=np.uint16)
    assert np.array_equal(got, want)
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert R.bf16_bits(1.00390625) == 0x3F80 and R.bf16_bits(1.01171875) == 0x3F82


def test_rmsnorm_matches_library():
    g = np.random.default_rng(2)
    x = g.standard_normal(96) * 3.0
    w = 1.0 + 0.1 * g.standard_normal(96)
    want = F.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(w), eps=1e-5).numpy()
    np.testing.assert_allclose(R.rmsnorm(x, w, 1e-5), want, rtol=1e-13, atol=0)
    # a constant row c normalises to sign(c) * g / sqrt(1 + eps / c^2)
    c = np.full(8, -2.0)
    np.testing.assert_allclose(R.rmsnorm(c, np.ones(8), 0.04), -np.ones(8) / np.sqrt(1.01), rtol=1e-14)


def test_rope_properties():
    g = np.random.default_rng(3)
    hd, theta = 32, 1.0e4
    q, k = g.standard_normal(hd), g.standard_normal(hd)
    np.testing.assert_array_equal(R.rope(q, 0, theta), q)                       # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(R.rope(q, 77, theta)), np.linalg.norm(q), rtol=1e-13)
    # complex form: element pair (i, i + hd/2) is multiplied by exp(j pos theta^(-2i/hd))
    z = (q[:hd // 2] + 1j * q[hd // 2:]) * np.exp(1j * 77 * theta ** (-2.0 * np.arange(hd // 2) / hd))
    np.testing.assert_allclose(R.rope(q, 77, theta), np.concatenate([z.real, z.imag]), rtol=1e-12, atol=1e-12)
    # scores depend on the distance of the positions only
    a = R.rope(q, 50, theta) @ R.rope(k, 20, theta)
    b = R.rope(q, 130, theta) @ R.rope(k, 100, theta)
    c = R.rope(q, 30, theta) @ k
    np.testing.assert_allclose([a, b], [c, c], rtol=1e-10, atol=1e-10)
    # the first pair turns at one radian per position, the last pair almost not at all
    e = np.zeros(hd); e[0] = 1.0
    r = R.rope(e, 1, theta)
    np.testing.assert_allclose([r[0], r[hd // 2]], [np.cos(1.0), np.sin(1.0)], rtol=1e-14)


def _torch_layer(x, ws, kc, vc, pos, Hq, Hkv, hd, theta, eps):
    """The same layer from library routines (fp64): rms_norm, linear, complex rotation,
    scaled_dot_product_attention over explicitly repeated key-value heads."""
    n, d = x.shape
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    X = t(x)
    xn = F.rms_norm(X, (d,), t(ws["norm"]), eps=eps)
    q = F.linear(xn, t(ws["wq"])).view(n, Hq, hd)
    k = F.linear(xn, t(ws["wk"])).view(n, Hkv, hd)
    v = F.linear(xn, t(ws["wv"])).view(n, Hkv, hd)
    rot = torch.exp(1j * pos * torch.tensor(theta, dtype=torch.float64) ** (-2.0 * torch.arange(hd // 2, dtype=torch.float64) / hd))

    def turn(a):
        z = torch.complex(a[..., :hd // 2], a[..., hd // 2:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)

    q, k = turn(q), turn(k)
    K = t(kc).clone()
    V = t(vc).clone()
    K[:, :, pos, :] = k.to(torch.bfloat16).to(torch.float64)
    V[:, :, pos, :] = v.to(torch.bfloat16).to(torch.float64)
    Kr = K[:, :, :pos + 1, :].repeat_interleave(Hq // Hkv, dim=1)
    Vr = V[:, :, :pos + 1, :].repeat_interleave(Hq // Hkv, dim=1)
    o = F.scaled_dot_product_attention(q.unsqueeze(2), Kr, Vr)   # [n, Hq, 1, hd], scale 1/sqrt(hd)
    y = X + F.linear(o.reshape(n, Hq * hd), t(ws["wo"]))
    return y.numpy(), K.numpy(), V.numpy()


def _case(w, b, layer=0):
    ws = {k: I.as_f32(v) for k, v in I.gen_attn_weights(w, layer).items()}
    x = I.as_f32(I.gen_attn_hidden(w, layer, b))
    kc, vc = I.gen_kv_cache(w, layer, b)
    return ws, x, kc, vc


@pytest.mark.parametrize("b", [0, 1, 2])
def test_layer_matches_library_pipeline(b):
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ws, x, kc, vc = _case(w, b)
    pos = w.batch_pos[b]
    y, k2, v2 = R.attn_decode(x, ws["norm"], ws["wq"], ws["wk"], ws["wv"], ws["wo"], I.as_raw(kc), I.as_raw(vc),
                              pos, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
    yt, Kt, Vt = _torch_layer(x, ws, I.as_f32(kc), I.as_f32(vc), pos, w.n_q_heads, w.n_kv_heads, w.head_dim,
                              w.rope_theta, w.rms_eps)
    widen = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(widen(k2), Kt)     # appended rows included, older rows untouched
    np.testing.assert_array_equal(widen(v2), Vt)
    np.testing.assert_allclose(y, yt, rtol=1e-10, atol=1e-11)


def test_first_position_closed_form():
    """With an empty cache the softmax has one term: every query head returns the new value row of
    its key-value head, so y = x + Wo . repeat(bf16(Wv . norm(x)))."""
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ws, x, kc, vc = _case(w, 1)
    assert w.batch_pos[1] == 0
    y, _, v2 = R.attn_decode(x, ws["norm"], ws["wq"], ws["wk"], ws["wv"], ws["wo"], I.as_raw(kc), I.as_raw(vc),
                             0, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
    x64 = x.astype(np.float64)
    xn = x64 / np.sqrt((x64 ** 2).mean(axis=1, keepdims=True) + w.rms_eps) * ws["norm"].astype(np.float64)
    v = torch.from_numpy(xn @ ws["wv"].astype(np.float64).T).to(torch.bfloat16).to(torch.float64).numpy()
    v = v.reshape(-1, w.n_kv_heads, w.head_dim)
    o = np.repeat(v, w.n_q_heads // w.n_kv_heads, axis=1).reshape(x.shape[0], -1)
    np.testing.assert_allclose(y, x64 + o @ ws["wo"].astype(np.float64).T, rtol=1e-11, atol=1e-12)


def test_equal_keys_give_the_mean_value():
    """If every cached key (and the new one) is the same vector the weights are uniform and the
    output is the plain mean of the value rows: a zero key projection makes all keys zero."""
    w = I.ATTN_WORKLOADS["attn_tiny"]
    ws, x, kc, vc = _case(w, 0)
    pos = w.batch_pos[0]
    ws["wk"] = np.zeros_like(ws["wk"])
    kc = torch.zeros_like(kc)
    y, _, v2 = R.attn_decode(x, ws["norm"], ws["wq"], ws["wk"], ws["wv"], ws["wo"], I.as_raw(kc), I.as_raw(vc),
                             pos, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
    V = torch.from_numpy(v2.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    mean_v = V[:, :, :pos + 1, :].mean(axis=2)
    o = np.repeat(mean_v, w.n_q_heads // w.n_kv_heads, axis=1).reshape(x.shape[0], -1)
    np.testing.assert_allclose(y, x.astype(np.float64) + o @ ws["wo"].astype(np.float64).T, rtol=1e-11, atol=1e-12)


def test_one_dominant_key_selects_its_value():
    """A cached key that is a large multiple of the query direction takes all of the softmax
    weight: the head's output is that position's value row."""
    w = I.scaled(I.ATTN_WORKLOADS["attn_tiny"], n_q_heads=2, n_kv_heads=2)
    ws, x, kc, vc = _case(w, 0)
    pos, hd = w.batch_pos[0], w.head_dim
    # position-free query: with theta = 1 ... use pos such that rotation is not identity, so
    # plant the key from the oracle-independent complex rotation of the query
    x64 = x.astype(np.float64)
    xn = x64 / np.sqrt((x64 ** 2).mean(axis=1, keepdims=True) + w.rms_eps) * ws["norm"].astype(np.float64)
    q = (xn @ ws["wq"].astype(np.float64).T).reshape(-1, w.n_q_heads, hd)
    rot = np.exp(1j * pos * w.rope_theta ** (-2.0 * np.arange(hd // 2) / hd))
    z = (q[..., :hd // 2] + 1j * q[..., hd // 2:]) * rot
    qr = np.concatenate([z.real, z.imag], axis=-1)
    hit = 5
    kc[:, :, hit, :] = torch.from_numpy(qr * 200.0).to(torch.bfloat16)
    y, _, _ = R.attn_decode(x, ws["norm"], ws["wq"], ws["wk"], ws["wv"], ws["wo"], I.as_raw(kc), I.as_raw(vc),
                            pos, w.n_q_heads, w.n_kv_heads, hd, w.rope_theta, w.rms_eps)
    o = I.as_f32(vc)[:, :, hit, :].astype(np.float64).reshape(x.shape[0], -1)
    np.testing.assert_allclose(y, x64 + o @ ws["wo"].astype(np.float64).T, rtol=1e-9, atol=1e-9)
