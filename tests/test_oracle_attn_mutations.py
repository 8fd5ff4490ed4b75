"""Do the pins of the attention oracle have teeth?  Each case plants one plausible mistake in a
copy of the oracle's source (on the CPU, in a temporary directory), builds it, runs the pins
against the mutant and requires at least one of them to fail.  The unmodified source must pass
the same list."""
import ctypes as C
import os
import subprocess

import pytest

from oracle import attn_ref as R

import test_oracle_attn_pins as P

SRC = os.path.join(os.path.dirname(R.__file__), "attn_oracle.c")

PINS = [P.test_bf16_rounding_matches_library_cast, P.test_rmsnorm_matches_library, P.test_rope_properties,
        lambda: P.test_layer_matches_library_pipeline(0), lambda: P.test_layer_matches_library_pipeline(1),
        lambda: P.test_layer_matches_library_pipeline(2), P.test_first_position_closed_form,
        P.test_equal_keys_give_the_mean_value, P.test_one_dominant_key_selects_its_value]

MUTATIONS = {
    "eps dropped from the norm": ("ss / d + eps", "ss / d"),
    "mean replaced by sum in the norm": ("1.0 / sqrt(ss / d + eps)", "1.0 / sqrt(ss + eps)"),
    "norm weight not applied": ("x[i] * r * wat(g, wtype, i)", "x[i] * r"),
    "rotation sign": ("v[i] = a * c - b * s;", "v[i] = a * c + b * s;"),
    "rotation frequency exponent": ("pow(theta, -2.0 * i / hd)", "pow(theta, -1.0 * i / hd)"),
    "rotation pairs adjacent elements": ("const double a = v[i], b = v[i + half];", "const double a = v[i], b = v[(i + 1) % hd];"),
    "keys not rotated": ("for (int h = 0; h < Hkv; ++h) ka_rope(k + (size_t)h * hd, hd, pos, theta);", ""),
    "query heads mapped round-robin to key-value heads": ("const int gk = h / group;", "const int gk = h % Hkv;"),
    "scale 1/hd instead of 1/sqrt(hd)": ("p[t] = acc / sqrt((double)hd);", "p[t] = acc / (double)hd;"),
    "new token left out of the scores": ("for (int t = 0; t <= pos; ++t) {\n                double acc = 0.0;\n                for (int i = 0; i < hd; ++i) acc += q",
                                          "for (int t = 0; t < pos + (pos == 0); ++t) {\n                double acc = 0.0;\n                for (int i = 0; i < hd; ++i) acc += q"),
    "weights transposed": ("acc += wat(w, wtype, (size_t)r * cols + c) * x[c];", "acc += wat(w, wtype, (size_t)c * rows + r) * x[c];"),
    "residual dropped": ("y[(size_t)s * d + i] = xd[i] + out[i];", "y[(size_t)s * d + i] = out[i];"),
    "softmax not normalised": ("o[(size_t)h * hd + i] = acc / den;", "o[(size_t)h * hd + i] = acc;"),
    "values read from the key cache": ("const uint16_t *V = vc + ((size_t)s * Hkv + gk) * max_len * hd;", "const uint16_t *V = kc + ((size_t)s * Hkv + gk) * max_len * hd;"),
    "new rows truncated instead of rounded": ("const double r = nearbyint(x / ulp) * ulp;", "const double r = trunc(x / ulp) * ulp;"),
}


def build_variant(tmp_path, name, old, new):
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, f"mutation '{name}': pattern occurs {text.count(old)} times"
        text = text.replace(old, new)
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", str(lib),
                    str(src), "-lm"], check=True)
    h = C.CDLL(str(lib))
    h.ka_bf16_bits.restype = C.c_uint16
    h.ka_bf16_bits.argtypes = [C.c_double]
    return h


def failures(handle, monkeypatch):
    R.lib()                               # the real one is loaded first, then shadowed
    monkeypatch.setattr(R, "_lib", handle)
    failed = 0
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            failed += 1
    return failed


def test_unmodified_source_passes_every_pin(tmp_path, monkeypatch):
    assert failures(build_variant(tmp_path, "none", None, None), monkeypatch) == 0


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    assert failures(build_variant(tmp_path, name, old, new), monkeypatch) >= 1, f"no pin notices: {name}"
