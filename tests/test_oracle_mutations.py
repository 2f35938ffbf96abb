"""Checks that the pins have teeth: each plausible mistake planted in a copy of the oracle source
(on the CPU, never in the GPU code) must make at least one pin test fail."""
import os
import types

import pytest

import test_oracle_attention as pins_attn
import test_oracle_block as pins_block
import test_oracle_chunked as pins_chunk
import test_oracle_layout_placement as pins_misc
import test_oracle_recurrent as pins_rec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = open(os.path.join(ROOT, "oracle", "mixers.py")).read()
CHUNK_SOURCE = open(os.path.join(ROOT, "oracle", "chunked.py")).read().replace("from .mixers import", "from oracle.mixers import")
LAYOUT_SOURCE = open(os.path.join(ROOT, "oracle", "kv_layout.py")).read()
BLOCK_SOURCE = open(os.path.join(ROOT, "oracle", "recurrent_block.py")).read().replace("from .mixers import", "from oracle.mixers import")

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


BLOCK_MUTATIONS = {
    "convolution taps reversed": ('acc = np.einsum("bjc,jc->bc", window, weight)', 'acc = np.einsum("bjc,jc->bc", window, weight[::-1])'),
    "history drops the newest input": ("return silu(acc), window[:, 1:, :].copy()", "return silu(acc), window[:, :-1, :].copy()"),
    "sigmoid instead of SiLU after the convolution": ("return silu(acc), window[:, 1:, :].copy()",
                                                      "return sigmoid(acc), window[:, 1:, :].copy()"),
    "decay grows instead of shrinking": ("return np.exp(-np.exp(widen(A_log))", "return np.exp(np.exp(widen(A_log))"),
    "A_log used without the exponential": ("return np.exp(-np.exp(widen(A_log))", "return np.exp(-(widen(A_log))"),
    "dt_bias dropped": ("softplus(widen(alpha_raw) + widen(dt_bias))", "softplus(widen(alpha_raw))"),
    "softplus replaced by relu": ("softplus(widen(alpha_raw) + widen(dt_bias))", "np.maximum(widen(alpha_raw) + widen(dt_bias), 0.0)"),
    "sum instead of mean in the RMS norm": ("np.sqrt(np.mean(o * o, axis=-1, keepdims=True) + eps)",
                                            "np.sqrt(np.sum(o * o, axis=-1, keepdims=True) + eps)"),
    "output gate activations swapped": ('act = silu(z) if gate_act == "silu" else sigmoid(z)',
                                        'act = sigmoid(z) if gate_act == "silu" else silu(z)'),
    "norm weight dropped": ("return weight * o / np.sqrt(", "return o / np.sqrt("),
    "L2 norm without the root": ("return x / np.sqrt(np.sum(x * x, axis=-1, keepdims=True) + L2_EPS)",
                                 "return x / (np.sum(x * x, axis=-1, keepdims=True) + L2_EPS)"),
    "queries not normalised": ("    q = l2_normalise(q.reshape(B, Hk, dk))", "    q = q.reshape(B, Hk, dk)"),
    "keys not normalised": ("    k = l2_normalise(k.reshape(B, Hk, dk))", "    k = k.reshape(B, Hk, dk)"),
    "beta not activated": ("    beta = sigmoid(widen(beta_raw))", "    beta = widen(beta_raw)"),
    "value stream skips its convolution": ("    v, conv_v = causal_conv_silu_step(np.asarray(xv).reshape(B, -1), conv_v, wv)",
                                           "    v, conv_v = widen(np.asarray(xv).reshape(B, -1)), conv_v"),
    "KDA gate bias shared over channels": ("alpha = decay_gate(alpha_raw, widen(A_log)[None, :, None], widen(dt_bias)[None])",
                                           "alpha = decay_gate(alpha_raw, widen(A_log)[None, :, None], widen(dt_bias)[None, :, :1])"),
}


CHUNK_MUTATIONS = {
    "earlier tokens' corrections ignored": ("Delta = solve_triangular(np.eye(T) + A, rhs, lower=True, unit_diagonal=True)", "Delta = rhs"),
    "read-out misses the token's own write": ("np.tril(Qhat @ Ktil.T) @ Delta)", "np.tril(Qhat @ Ktil.T, -1) @ Delta)"),
    "beta missing on the right-hand side": ("rhs = be[:, None] * (V - Khat @ S0[b, h])", "rhs = (V - Khat @ S0[b, h])"),
    "prediction without the decay": ("rhs = be[:, None] * (V - Khat @ S0[b, h])", "rhs = be[:, None] * (V - K @ S0[b, h])"),
    "state carried without the decay": ("S_out[b, h] = gam[-1][:, None] * S0[b, h] + (gam[-1] * Ktil).T @ Delta",
                                        "S_out[b, h] = S0[b, h] + (gam[-1] * Ktil).T @ Delta"),
    "decay of later tokens dropped from the update": ("(gam[-1] * Ktil).T @ Delta", "K.T @ Delta"),
    "upper instead of lower triangle": ("A = np.tril(be[:, None] * (Khat @ Ktil.T), -1)", "A = np.triu(be[:, None] * (Khat @ Ktil.T), 1)"),
}

LAYOUT_MUTATIONS = {
    "K chunks of 16 dims": ("    return ((d // 8) * PAGE + j) * 8 + d % 8", "    return ((d // 16) * PAGE + j) * 16 + d % 16"),
    "K token-major": ("    return ((d // 8) * PAGE + j) * 8 + d % 8", "    return j * 128 + d"),
    "V groups of 8 tokens": ("    return (((d // 16) * 4 + j // 4) * 16 + d % 16) * 4 + j % 4",
                             "    return (((d // 16) * 2 + j // 8) * 16 + d % 16) * 8 + j % 8"),
    "V dims and token groups swapped": ("    return (((d // 16) * 4 + j // 4) * 16 + d % 16) * 4 + j % 4",
                                        "    return (((j // 4) * 8 + d // 16) * 16 + d % 16) * 4 + j % 4"),
    "gather map differs from the scalar formula": ("    vmap = (((dd // 16) * 4 + jj // 4) * 16 + dd % 16) * 4 + jj % 4",
                                                   "    vmap = (((dd // 16) * 4 + jj % 4) * 16 + dd % 16) * 4 + jj // 4"),
    "append lands one slot late": ("            j = pos % PAGE\n", "            j = (pos + 1) % PAGE\n"),
}


def mutated_module(old, new, source=None):
    source = SOURCE if source is None else source
    assert source.count(old) >= 1, "mutation target not found: %r" % old
    mod = types.ModuleType("oracle_mutant")
    exec(compile(source.replace(old, new), "oracle_mutant", "exec"), mod.__dict__)
    return mod


def any_pin_fails(pins, mutant, monkeypatch, attr="om"):
    monkeypatch.setattr(pins, attr, mutant)
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [{}]
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            cases = [dict(c, **dict(zip(names, v if len(names) > 1 else (v,)))) for c in cases for v in m.args[1]]
        for case in cases:
            try:
                fn(**case)
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


@pytest.mark.parametrize("what", sorted(BLOCK_MUTATIONS))
def test_block_pins_catch(what, monkeypatch):
    assert any_pin_fails(pins_block, mutated_module(*BLOCK_MUTATIONS[what], source=BLOCK_SOURCE), monkeypatch, attr="ob"), what


@pytest.mark.parametrize("what", sorted(CHUNK_MUTATIONS))
def test_chunked_form_pins_catch(what, monkeypatch):
    assert any_pin_fails(pins_chunk, mutated_module(*CHUNK_MUTATIONS[what], source=CHUNK_SOURCE), monkeypatch, attr="oc"), what


@pytest.mark.parametrize("what", sorted(LAYOUT_MUTATIONS))
def test_layout_pins_catch(what, monkeypatch):
    assert any_pin_fails(pins_misc, mutated_module(*LAYOUT_MUTATIONS[what], source=LAYOUT_SOURCE), monkeypatch, attr="kl"), what


def test_unmutated_block_oracle_passes_through_the_same_runner(monkeypatch):
    assert not any_pin_fails(pins_chunk, mutated_module("import numpy as np", "import numpy as np", source=CHUNK_SOURCE), monkeypatch,
                             attr="oc")
    assert not any_pin_fails(pins_misc, mutated_module("PAGE = 16", "PAGE = 16", source=LAYOUT_SOURCE), monkeypatch, attr="kl")
    clean = mutated_module("L2_EPS = 1e-6", "L2_EPS = 1e-6", source=BLOCK_SOURCE)
    assert not any_pin_fails(pins_block, clean, monkeypatch, attr="ob")


def test_unmutated_oracle_passes_through_the_same_runner(monkeypatch):
    clean = mutated_module("PAGE = 16", "PAGE = 16")
    assert not any_pin_fails(pins_rec, clean, monkeypatch)
    assert not any_pin_fails(pins_attn, clean, monkeypatch)
    assert not any_pin_fails(pins_misc, clean, monkeypatch)
