"""Pins for the GDN/KDA block oracle (convolution, gates, norms around the state update)."""
import numpy as np
import pytest
from scipy.signal import lfilter

from oracle import mixers as om
from oracle import recurrent_block as ob


def test_conv_steps_equal_a_causal_fir_filter_followed_by_silu():
    """Feeding tokens one at a time = scipy's FIR filter over the whole sequence (zero history)."""
    rng = np.random.default_rng(1)
    T, C, taps = 9, 5, 4
    x = rng.standard_normal((T, C))
    w = rng.standard_normal((taps, C))
    state = np.zeros((1, taps - 1, C))
    ys = []
    for t in range(T):
        y, state = ob.causal_conv_silu_step(x[t][None], state, w)
        ys.append(y[0])
    for c in range(C):
        fir = lfilter(w[::-1, c], [1.0], x[:, c])            # lag 0 <- last tap
        np.testing.assert_allclose(np.array(ys)[:, c], fir / (1 + np.exp(-fir)), atol=1e-13)
    np.testing.assert_array_equal(state[0], x[-(taps - 1):])   # the state is the last Kc-1 inputs, oldest first


def test_initial_convolution_of_the_paper_halves_the_input():
    """Appendix C (DIL/KIL init): 0.5 on the last tap, zeros elsewhere -> y = SiLU(x / 2) whatever the history."""
    rng = np.random.default_rng(2)
    x, hist = rng.standard_normal((2, 6)), rng.standard_normal((2, 3, 6))
    w = np.zeros((4, 6))
    w[-1] = 0.5
    y, new = ob.causal_conv_silu_step(x, hist, w)
    np.testing.assert_allclose(y, (x / 2) / (1 + np.exp(-x / 2)), atol=1e-15)
    np.testing.assert_array_equal(new[:, :2], hist[:, 1:])
    np.testing.assert_array_equal(new[:, 2], x)


def test_initial_gates_of_the_paper():
    """A_log = log 0.1, dt_bias = 0, zero gate projections: beta = 0.5 and the state halves every 10 steps
    (the paper: slow decay, retains state about 10 steps)."""
    a = ob.decay_gate(np.zeros(3), np.full(3, np.log(0.1)), np.zeros(3))
    np.testing.assert_allclose(a ** 10, 0.5, atol=1e-15)
    assert ob.sigmoid(0.0) == 0.5
    # monotone: a larger raw gate or a larger A_log forgets faster, and alpha stays inside (0,1)
    raw = np.linspace(-6, 6, 9)
    al = ob.decay_gate(raw, 0.0, 0.5)
    assert np.all(np.diff(al) < 0) and np.all((al > 0) & (al < 1))
    assert ob.decay_gate(0.3, 1.0, 0.0) < ob.decay_gate(0.3, 0.0, 0.0)
    np.testing.assert_allclose(ob.decay_gate(0.3, 0.0, 0.2), np.exp(-np.log1p(np.exp(0.5))), atol=1e-15)


def test_norms():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 7))
    n = ob.l2_normalise(x * 1e3)
    np.testing.assert_allclose(np.sum(n * n, -1), 1.0, atol=1e-9)
    np.testing.assert_allclose(ob.l2_normalise(x * 5.0), ob.l2_normalise(x), atol=1e-6)
    o, z, w = rng.standard_normal((4, 8)), rng.standard_normal((4, 8)), rng.uniform(0.5, 2, 8)
    y = ob.gated_rms_norm(o, z, w, 0.0, "silu")
    # scale invariance in o, linear in the weight, gate applied elementwise
    np.testing.assert_allclose(ob.gated_rms_norm(3.7 * o, z, w, 0.0, "silu"), y, atol=1e-13)
    np.testing.assert_allclose(np.sqrt(np.mean((y / (w * z / (1 + np.exp(-z)))) ** 2, -1)), 1.0, atol=1e-12)
    np.testing.assert_allclose(ob.gated_rms_norm(o, z, w, 0.0, "sigmoid"), y / z, atol=1e-12)
    assert not ob.gated_rms_norm(o, np.zeros_like(z), w, 1e-6, "silu").any()      # SiLU(0) = 0 closes the gate
    # hand example: o = (3,4), mean square 12.5, weight 1, z large -> SiLU(z) ~ z
    np.testing.assert_allclose(ob.gated_rms_norm(np.array([3.0, 4.0]), np.array([50.0, 50.0]), np.ones(2), 0.0, "silu"),
                               np.array([3.0, 4.0]) / np.sqrt(12.5) * 50.0, rtol=1e-12)


@pytest.mark.parametrize("kind", ["gdn", "kda"])
def test_block_step_is_the_composition_of_its_pinned_parts(kind):
    rng = np.random.default_rng(4)
    B, H, Hk, dk, dv, taps = 2, 4, 2, 6, 5, 4
    xq, xk, xv = rng.standard_normal((B, Hk, dk)), rng.standard_normal((B, Hk, dk)), rng.standard_normal((B, H, dv))
    cq, ck, cv = (rng.standard_normal((B, taps - 1, c)) for c in (Hk * dk, Hk * dk, H * dv))
    wq, wk, wv = (rng.standard_normal((taps, c)) for c in (Hk * dk, Hk * dk, H * dv))
    beta_raw = rng.standard_normal((B, H))
    alpha_raw = rng.standard_normal((B, H, dk) if kind == "kda" else (B, H))
    A_log = rng.standard_normal(H) * 0.3
    dt_bias = rng.standard_normal((H, dk) if kind == "kda" else H)
    z, nw, S0 = rng.standard_normal((B, H, dv)), rng.uniform(0.5, 2, dv), rng.standard_normal((B, H, dk, dv))
    r = ob.block_decode_step(kind, xq, xk, xv, cq, ck, cv, wq, wk, wv, beta_raw, alpha_raw, A_log, dt_bias, z, nw, 1e-5,
                             "silu", S0, 0.4)
    # parts, each pinned above or in test_oracle_recurrent.py
    q = ob.l2_normalise(ob.causal_conv_silu_step(xq.reshape(B, -1), cq, wq)[0].reshape(B, Hk, dk))
    k = ob.l2_normalise(ob.causal_conv_silu_step(xk.reshape(B, -1), ck, wk)[0].reshape(B, Hk, dk))
    v = ob.causal_conv_silu_step(xv.reshape(B, -1), cv, wv)[0].reshape(B, H, dv)
    for b in range(B):
        for h in range(H):
            a = np.exp(-np.exp(A_log[h]) * np.log1p(np.exp(alpha_raw[b, h] + dt_bias[h])))
            fn = om.kda_steps if kind == "kda" else om.gdn_steps
            o, S = fn(q[b:b + 1, None, h // 2:h // 2 + 1], k[b:b + 1, None, h // 2:h // 2 + 1], v[b:b + 1, None, h:h + 1],
                      np.reshape(a, (1, 1, 1) + np.shape(a)), np.reshape(1 / (1 + np.exp(-beta_raw[b, h])), (1, 1, 1)),
                      S0[b:b + 1, h:h + 1], 0.4)
            np.testing.assert_allclose(r["state"][b, h], S[0, 0], atol=1e-13)
            want = ob.gated_rms_norm(o[0, 0, 0], z[b, h], nw, 1e-5, "silu")
            np.testing.assert_allclose(r["out"][b, h], want, atol=1e-12)
    np.testing.assert_array_equal(r["conv_v"][:, -1], xv.reshape(B, -1))


def test_block_with_paper_initial_values_reduces_to_plain_gdn_on_half_inputs():
    """DIL init end to end: conv = 0.5 * identity tap, zero gate projections, A_log = log 0.1: the block
    is a GDN step on q,k = normalised SiLU(x/2), v = SiLU(x/2), beta = 0.5, alpha = 2^-0.1."""
    rng = np.random.default_rng(5)
    B, H, dk, dv = 1, 2, 4, 4
    xq, xk, xv = rng.standard_normal((B, H, dk)), rng.standard_normal((B, H, dk)), rng.standard_normal((B, H, dv))
    w = np.zeros((4, H * dk))
    w[-1] = 0.5
    hist = rng.standard_normal((B, 3, H * dk))
    S0 = rng.standard_normal((B, H, dk, dv))
    r = ob.block_decode_step("gdn", xq, xk, xv, hist, hist, hist, w, w, w, np.zeros((B, H)), np.zeros((B, H)),
                             np.full(H, np.log(0.1)), np.zeros(H), np.full((B, H, dv), 30.0), np.ones(dv), 0.0, "sigmoid",
                             S0, 1.0)
    half = lambda x: (x / 2) / (1 + np.exp(-x / 2))
    q, k = ob.l2_normalise(half(xq)), ob.l2_normalise(half(xk))
    o, S = om.gdn_steps(q[:, None], k[:, None], half(xv)[:, None], np.full((B, 1, H), 2 ** -0.1), np.full((B, 1, H), 0.5), S0)
    np.testing.assert_allclose(r["state"], S, atol=1e-13)
    np.testing.assert_allclose(r["out"], o[:, 0] / np.sqrt(np.mean(o[:, 0] ** 2, -1, keepdims=True)), atol=1e-12)
