"""Checks that the pins have teeth: each plausible mistake planted in a copy of the oracle source
(on the CPU, never in the GPU code) must make at least one pin test fail."""
import os
import types

import pytest

import test_oracle_attention as pins_attn
import test_oracle_layout_placement as pins_misc
import test_oracle_recurrent as pins_rec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "mixers.py")).read()

RECURRENT_MUTATIONS = {
    "wrong sign of the write": ("S = Sbar + k[:, t, :, :, None] * delta[:, :, None, :]",
                                "S = Sbar - k[:, t, :, :, None] * delta[:, :, None, :]"),
    "prediction from the undecayed state": ('u = np.einsum("bhkv,bhk->bhv", Sbar, k[:, t])',
                                            'u = np.einsum("bhkv,bhk->bhv", S, k[:, t])'),
    "read-out before the write": ('out[:, t] = scale * np.einsum("bhkv,bhk->bhv", S, q[:, t])',
                                  'out[:, t] = scale * np.einsum("bhkv,bhk->bhv", Sbar, q[:, t])'),
    "beta dropped": ("delta = beta[:, t, :, None] * (v[:, t] - u)", "delta = (v[:, t] - u)"),
    "channel gate on value columns": ("Sbar = alpha[:, t, :, :, None] * S", "Sbar = alpha[:, t, :, None, :] * S"),
    "transposed state product": ('u = np.einsum("bhkv,bhk->bhv", Sbar, k[:, t])',
                                 'u = np.einsum("bhvk,bhk->bhv", Sbar, k[:, t])'),
    "decay applied after the write": ("S = Sbar + k[:, t, :, :, None] * delta[:, :, None, :]",
                                      "S = Sbar + (alpha[:, t, :, :, None] if per_channel else alpha[:, t, :, None, None]) "
                                      "* k[:, t, :, :, None] * delta[:, :, None, :]"),
    "scale dropped": ('out[:, t] = scale * np.einsum("bhkv,bhk->bhv", S, q[:, t])',
                      'out[:, t] = np.einsum("bhkv,bhk->bhv", S, q[:, t])'),
    "key heads interleaved instead of grouped": ("return np.repeat(x, H // Hk, axis=2)",
                                                 "return np.tile(x, (1, 1, H // Hk, 1))"),
    "commit point off by one": ("if t + 1 == n_commit:", "if t == n_commit:"),
}

ATTENTION_MUTATIONS = {
    "window one token too long": ("lo = max(0, hi - window) if window > 0 else 0", "lo = max(0, hi - window - 1) if window > 0 else 0"),
    "window excludes the newest token": ("hi = L - T + i + 1                       # new token", "hi = L - T + i                       # new token"),
    "query heads interleaved over KV heads": ("        g = h // group\n        key = (b, g, lo, hi)", "        g = h % Hkv\n        key = (b, g, lo, hi)"),
    "softmax scale dropped": ("s = scale * (K @ q[b, i, h])", "s = (K @ q[b, i, h])"),
    "weights not normalised": ("        p = p / np.sum(p)\n        out[b, i, h] = p @ V", "        out[b, i, h] = p @ V"),
    "in-page slot ignored": ("cache[key] = (widen(kpool[phys, g, pos % PAGE]), widen(vpool[phys, g, pos % PAGE]))",
                             "cache[key] = (widen(kpool[phys, g, pos % PAGE]), widen(vpool[phys, g, (pos + 1) % PAGE]))"),
    "keys used as values": ("        out[b, i, h] = p @ V", "        out[b, i, h] = p @ K"),
}

PLACEMENT_MUTATIONS = {
    "window passed to full attention": ('io["seq_lens"][r:r + 1], window if m == "S" else 0, attn_scale)',
                                        'io["seq_lens"][r:r + 1], window, attn_scale)'),
    "KDA and GDN swapped": ('fn = kda_steps if m == "K" else gdn_steps\n                a = io["alpha_vec"] if m == "K" else io["alpha_scalar"]',
                            'fn = kda_steps if m == "G" else gdn_steps\n                a = io["alpha_vec"] if m == "G" else io["alpha_scalar"]'),
}


def mutated_module(old, new):
    assert SOURCE.count(old) >= 1, "mutation target not found: %r" % old
    mod = types.ModuleType("oracle_mutant")
    exec(compile(SOURCE.replace(old, new), "oracle_mutant", "exec"), mod.__dict__)
    return mod


def any_pin_fails(pins, mutant, monkeypatch):
    monkeypatch.setattr(pins, "om", mutant)
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [()]
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            cases = [c + (v if len(names) > 1 else (v,)) for c in cases for v in m.args[1]]
        for case in cases:
            try:
                fn(*case)
            except Exception:
                return True
    return False


@pytest.mark.parametrize("what", sorted(RECURRENT_MUTATIONS))
def test_recurrent_pins_catch(what, monkeypatch):
    assert any_pin_fails(pins_rec, mutated_module(*RECURRENT_MUTATIONS[what]), monkeypatch), what


@pytest.mark.parametrize("what", sorted(ATTENTION_MUTATIONS))
def test_attention_pins_catch(what, monkeypatch):
    assert any_pin_fails(pins_attn, mutated_module(*ATTENTION_MUTATIONS[what]), monkeypatch), what


@pytest.mark.parametrize("what", sorted(PLACEMENT_MUTATIONS))
def test_placement_pins_catch(what, monkeypatch):
    assert any_pin_fails(pins_misc, mutated_module(*PLACEMENT_MUTATIONS[what]), monkeypatch), what


def test_unmutated_oracle_passes_through_the_same_runner(monkeypatch):
    clean = mutated_module("PAGE = 16", "PAGE = 16")
    assert not any_pin_fails(pins_rec, clean, monkeypatch)
    assert not any_pin_fails(pins_attn, clean, monkeypatch)
    assert not any_pin_fails(pins_misc, clean, monkeypatch)
