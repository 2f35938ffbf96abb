"""The fp64 C / OpenMP twin of the oracle (oracle/mixers_omp.c) is admitted only while it agrees with the numpy
oracle to 1e-12, and it has to pass the hand examples of the printed recurrences and closed forms on its own as well."""
import os

import numpy as np
import pytest

from oracle import kv_layout as kl
from oracle import mixers as om
from oracle import omp
from paper_2604_19877_amd import inputs as gen
from test_oracle_recurrent import read_golden

TOL = 1e-12

if not os.path.exists(omp.LIB_PATH):      # the checker's own library: a second of gcc
    from oracle import build as _build
    _build.build()


def close(a, b):
    np.testing.assert_allclose(a, b, rtol=0, atol=TOL)


@pytest.mark.parametrize("kda", [False, True])
@pytest.mark.parametrize("shape", [(2, 16, 4, 4, 64, 64), (3, 5, 4, 2, 16, 24), (1, 1, 2, 1, 128, 128)])
def test_recurrent_steps_match_the_numpy_oracle(kda, shape):
    B, T, H, Hk, dk, dv = shape
    p = gen.recurrent_inputs(700 + kda, B, T, H, Hk, dk, dv, kda)
    S0 = gen.recurrent_state(701, B * H, dk, dv).reshape(B, H, dk, dv)
    ref_fn, fn = (om.kda_steps, omp.kda_steps) if kda else (om.gdn_steps, omp.gdn_steps)
    for n_commit in (None, 0, 1, T):
        o_ref, s_ref = ref_fn(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 0.3, n_commit)
        o, s = fn(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 0.3, n_commit)
        close(o, o_ref)
        close(s, s_ref)


def test_recurrent_hand_examples():
    """Appendix B recurrences on the 2 x 2 examples worked by hand (tests/golden/gdn_kda_hand_example.txt)."""
    g = read_golden("gdn_kda_hand_example.txt")
    bits = lambda x: gen.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))     # all values are exact in bf16
    for name, fn in (("gdn", omp.gdn_steps), ("kda", omp.kda_steps)):
        alpha = g[name + "_alpha"].reshape((1, 1, 1) if name == "gdn" else (1, 1, 1, 2))
        o, s = fn(bits(g[name + "_q"]).reshape(1, 1, 1, 2), bits(g[name + "_k"]).reshape(1, 1, 1, 2),
                  bits(g[name + "_v"]).reshape(1, 1, 1, 2), alpha, g[name + "_beta"].reshape(1, 1, 1),
                  g[name + "_S0"].reshape(1, 1, 2, 2))
        close(s.reshape(-1), g[name + "_S1"])
        close(o.reshape(-1), g[name + "_o"])


def test_unit_learning_rate_recalls_the_value_exactly():
    """beta = 1 and a basis key: after the write S^T k = v, whatever the state and the gates were."""
    rng = np.random.default_rng(5)
    dk, dv = 8, 6
    S0 = rng.standard_normal((1, 1, dk, dv)).astype(np.float32)
    k = np.zeros((1, 1, 1, dk), dtype=np.float32)
    k[..., 3] = 1.0
    v = gen.f32_to_bf16_bits(rng.standard_normal((1, 1, 1, dv)).astype(np.float32))
    alpha = rng.uniform(0.1, 1.0, (1, 1, 1, dk)).astype(np.float32)
    o, s = omp.kda_steps(gen.f32_to_bf16_bits(k), gen.f32_to_bf16_bits(k), v, alpha, np.ones((1, 1, 1), dtype=np.float32), S0)
    close(s[0, 0, 3], om.widen(v)[0, 0, 0])
    close(o[0, 0, 0], om.widen(v)[0, 0, 0])
    other = [i for i in range(dk) if i != 3]
    close(s[0, 0, other], alpha[0, 0, 0, other, None].astype(np.float64) * S0[0, 0, other])    # gate on rows, others only decay


def problem(seed, lens, T, Hq=8, Hkv=2, D=16, max_pages=8):
    lens = np.array(lens, dtype=np.int32)
    p = gen.attention_inputs(seed, len(lens), T, Hq, Hkv, D, lens, max_pages)
    kp, vp = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    return p, kp, vp


@pytest.mark.parametrize("window", [0, 5, 16, 33, 4096])
@pytest.mark.parametrize("T", [1, 3])
def test_attention_matches_the_numpy_oracle(window, T):
    p, kp, vp = problem(710 + T, [100, 37, 16, T, 0, 1], T)
    ref = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], window, 0.3)
    close(omp.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], window, 0.3), ref)
    kphys, vphys = kl.to_physical(kp, vp)
    close(omp.attn_decode(p["q"], kphys, vphys, p["page_table"], p["seq_lens"], window, 0.3, physical=True), ref)


def test_attention_closed_forms():
    """Equal keys give equal weights, so the output is the mean of the visible values (the window's, for a window);
    a context of one token returns its value."""
    p, kp, vp = problem(715, [40, 1], 1)
    kp = kp.copy()
    kp[:] = gen.f32_to_bf16_bits(np.float32(0.75))
    for window in (0, 7):
        out = omp.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], window, 0.9)
        lo = 40 - window if window else 0
        for h in range(8):
            close(out[0, 0, h], om.widen(p["v_tok"][0, lo:40, h // 4]).mean(0))
            close(out[1, 0, h], om.widen(p["v_tok"][1, 0, h // 4]))


def test_unmapped_live_page_is_an_error():
    p, kp, vp = problem(720, [40], 1)
    table = p["page_table"].copy()
    table[0, 1] = -1
    with pytest.raises(ValueError):
        omp.attn_decode(p["q"], kp, vp, table, p["seq_lens"])
    assert omp.threads() >= 1
