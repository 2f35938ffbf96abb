"""Pins for the GDN/KDA oracle: hand example, closed forms and invariants fixed by the
recurrences of Appendix B.  Shapes use dk != dv so that a transposed operand cannot pass."""
import os

import numpy as np
import pytest

from oracle import mixers as om
from paper_2604_19877_amd import inputs as gen

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    vals = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rest = line.split(":")
            vals[key.strip()] = np.array([float(x) for x in rest.split()])
    return vals


def rand_problem(seed, B=2, T=3, H=4, Hk=4, dk=6, dv=5, per_channel=False, unit_k=False):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, T, Hk, dk))
    k = rng.standard_normal((B, T, Hk, dk))
    if unit_k:
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, T, H, dv))
    beta = rng.uniform(0.1, 0.9, (B, T, H))
    alpha = rng.uniform(0.2, 0.95, (B, T, H, dk) if per_channel else (B, T, H))
    S = rng.standard_normal((B, H, dk, dv))
    return q, k, v, alpha, beta, S


def test_hand_example_gdn():
    g = read_golden("gdn_kda_hand_example.txt")
    o, S = om.gdn_steps(g["gdn_q"].reshape(1, 1, 1, 2), g["gdn_k"].reshape(1, 1, 1, 2), g["gdn_v"].reshape(1, 1, 1, 2),
                        g["gdn_alpha"].reshape(1, 1, 1), g["gdn_beta"].reshape(1, 1, 1), g["gdn_S0"].reshape(1, 1, 2, 2))
    np.testing.assert_allclose(S.reshape(-1), g["gdn_S1"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(o.reshape(-1), g["gdn_o"], rtol=0, atol=1e-15)


def test_hand_example_kda():
    g = read_golden("gdn_kda_hand_example.txt")
    o, S = om.kda_steps(g["kda_q"].reshape(1, 1, 1, 2), g["kda_k"].reshape(1, 1, 1, 2), g["kda_v"].reshape(1, 1, 1, 2),
                        g["kda_alpha"].reshape(1, 1, 1, 2), g["kda_beta"].reshape(1, 1, 1), g["kda_S0"].reshape(1, 1, 2, 2))
    np.testing.assert_allclose(S.reshape(-1), g["kda_S1"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(o.reshape(-1), g["kda_o"], rtol=0, atol=1e-15)


@pytest.mark.parametrize("per_channel", [False, True])
def test_rank1_form_equals_printed_transition(per_channel):
    q, k, v, a, b, S = rand_problem(1, per_channel=per_channel)
    fast = om.kda_steps if per_channel else om.gdn_steps
    dense = om.kda_steps_dense if per_channel else om.gdn_steps_dense
    o1, S1 = fast(q, k, v, a, b, S, 0.7)
    o2, S2 = dense(q, k, v, a, b, S, 0.7)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(S1, S2, rtol=0, atol=1e-13)


@pytest.mark.parametrize("per_channel", [False, True])
def test_no_gate_no_write_leaves_state(per_channel):
    q, k, v, a, b, S = rand_problem(2, per_channel=per_channel)
    fn = om.kda_steps if per_channel else om.gdn_steps
    o, S1 = fn(q, k, v, np.ones_like(a), np.zeros_like(b), S)
    assert np.array_equal(S1, S)
    # read-out of an unchanged state is a plain matrix-vector product
    for bb in range(2):
        for h in range(4):
            np.testing.assert_allclose(o[bb, 0, h], S[bb, h].T @ q[bb, 0, h], atol=1e-13)


def test_beta_zero_is_pure_decay():
    q, k, v, a, b, S = rand_problem(3, T=2)
    _, S1 = om.gdn_steps(q, k, v, a, np.zeros_like(b), S)
    np.testing.assert_allclose(S1, (a[:, 0] * a[:, 1])[:, :, None, None] * S, atol=1e-15)
    q, k, v, a, b, S = rand_problem(3, T=2, per_channel=True)
    _, S1 = om.kda_steps(q, k, v, a, np.zeros_like(b), S)
    np.testing.assert_allclose(S1, (a[:, 0] * a[:, 1])[:, :, :, None] * S, atol=1e-15)


@pytest.mark.parametrize("per_channel", [False, True])
def test_full_write_stores_value_exactly(per_channel):
    """beta = 1 and |k| = 1: the projection erases the k-component, so S_t^T k = v whatever the gate,
    and reading out with q = k returns v (this needs the state after the write)."""
    q, k, v, a, b, S = rand_problem(4, T=1, per_channel=per_channel, unit_k=True)
    fn = om.kda_steps if per_channel else om.gdn_steps
    o, S1 = fn(k, k, v, a, np.ones_like(b), S)
    got = np.einsum("bhkv,bhk->bhv", S1, k[:, 0])
    np.testing.assert_allclose(got, v[:, 0], atol=1e-13)
    np.testing.assert_allclose(o[:, 0], v[:, 0], atol=1e-13)


def test_uniform_channel_gate_is_gdn():
    q, k, v, a, b, S = rand_problem(5)
    avec = np.repeat(a[..., None], 6, axis=-1)
    o1, S1 = om.gdn_steps(q, k, v, a, b, S, 0.3)
    o2, S2 = om.kda_steps(q, k, v, avec, b, S, 0.3)
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    np.testing.assert_allclose(S1, S2, atol=1e-14)


def test_orthonormal_keys_closed_form_gdn():
    """Orthonormal keys, beta = 1, S_0 = 0: S_n = sum_j (prod_{m>j} alpha_m) k_j v_j^T, and the read-out
    at step j with q = k_j is v_j (an outer-product associative memory with global forgetting)."""
    rng = np.random.default_rng(6)
    dk, dv, n = 7, 4, 5
    Q, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    keys = Q[:, :n].T                                     # n orthonormal keys
    v = rng.standard_normal((n, dv))
    a = rng.uniform(0.3, 0.9, n)
    o, S = om.gdn_steps(keys.reshape(1, n, 1, dk), keys.reshape(1, n, 1, dk), v.reshape(1, n, 1, dv),
                        a.reshape(1, n, 1), np.ones((1, n, 1)), np.zeros((1, 1, dk, dv)))
    want = sum(np.prod(a[j + 1:]) * np.outer(keys[j], v[j]) for j in range(n))
    np.testing.assert_allclose(S[0, 0], want, atol=1e-13)
    np.testing.assert_allclose(o[0, :, 0], v, atol=1e-13)


def test_basis_keys_closed_form_kda():
    """Keys are distinct basis vectors e_i, beta = 1, S_0 = 0: row i of S_n is v_j decayed by the gates
    of channel i alone from the steps after j.  A gate applied to columns, or after the write, fails."""
    rng = np.random.default_rng(7)
    dk, dv, n = 6, 5, 4
    rows = [3, 0, 5, 2]
    keys = np.eye(dk)[rows]
    v = rng.standard_normal((n, dv))
    a = rng.uniform(0.3, 0.9, (n, dk))
    _, S = om.kda_steps(keys.reshape(1, n, 1, dk), keys.reshape(1, n, 1, dk), v.reshape(1, n, 1, dv),
                        a.reshape(1, n, 1, dk), np.ones((1, n, 1)), np.zeros((1, 1, dk, dv)))
    want = np.zeros((dk, dv))
    for j, r in enumerate(rows):
        want[r] = np.prod(a[j + 1:, r]) * v[j]
    np.testing.assert_allclose(S[0, 0], want, atol=1e-14)


def test_update_is_rank_one_and_key_component_follows_delta_rule():
    q, k, v, a, b, S = rand_problem(8, T=1, unit_k=True)
    _, S1 = om.gdn_steps(q, k, v, a, b, S)
    for bb in range(2):
        for h in range(4):
            Sbar = a[bb, 0, h] * S[bb, h]
            diff = S1[bb, h] - Sbar
            assert np.linalg.matrix_rank(diff, tol=1e-10) == 1
            # along k the state moves a fraction beta of the way from its old answer to v
            kk = k[bb, 0, h]
            np.testing.assert_allclose(S1[bb, h].T @ kk, (1 - b[bb, 0, h]) * (Sbar.T @ kk) + b[bb, 0, h] * v[bb, 0, h],
                                       atol=1e-13)
            # directions orthogonal to k are untouched
            w = np.linalg.svd(kk.reshape(1, -1))[2][1:]
            np.testing.assert_allclose(w @ S1[bb, h], w @ Sbar, atol=1e-13)


@pytest.mark.parametrize("per_channel", [False, True])
def test_multi_step_call_is_chained_single_steps_and_n_commit(per_channel):
    q, k, v, a, b, S = rand_problem(9, T=4, per_channel=per_channel)
    fn = om.kda_steps if per_channel else om.gdn_steps
    o_all, S_all = fn(q, k, v, a, b, S, 0.5)
    cur = S
    for t in range(4):
        o_t, cur = fn(q[:, t:t + 1], k[:, t:t + 1], v[:, t:t + 1], a[:, t:t + 1], b[:, t:t + 1], cur, 0.5)
        assert np.array_equal(o_t[:, 0], o_all[:, t])
        _, S_c = fn(q, k, v, a, b, S, 0.5, n_commit=t + 1)
        assert np.array_equal(S_c, cur)
    assert np.array_equal(cur, S_all)
    _, S_0 = fn(q, k, v, a, b, S, 0.5, n_commit=0)
    assert np.array_equal(S_0, S)


def test_grouped_key_heads_map_contiguously():
    """H = 4 state heads over Hk = 2 q/k heads: heads 0,1 use q/k head 0 and heads 2,3 use head 1.
    With basis keys the written row tells which key head was used."""
    dk, dv = 4, 3
    k = np.zeros((1, 1, 2, dk))
    k[0, 0, 0, 1] = 1.0
    k[0, 0, 1, 3] = 1.0
    v = np.arange(12, dtype=float).reshape(1, 1, 4, dv) + 1
    _, S = om.gdn_steps(k, k, v, np.ones((1, 1, 4)), np.ones((1, 1, 4)), np.zeros((1, 4, dk, dv)))
    for h, row in enumerate([1, 1, 3, 3]):
        want = np.zeros((dk, dv))
        want[row] = v[0, 0, h]
        assert np.array_equal(S[0, h], want)


def test_bf16_inputs_are_widened_exactly():
    x = np.array([1.0, -2.5, 0.33203125, 3.0e-5], dtype=np.float32)
    bits = gen.f32_to_bf16_bits(x)
    assert np.array_equal(om.widen(bits), gen.bf16_bits_to_f32(bits).astype(np.float64))
    assert om.widen(np.array([0x3F80, 0xC020], dtype=np.uint16)).tolist() == [1.0, -2.5]


def test_config1_recipe_runs_and_state_stays_bounded():
    """B=2, H=4, dk=dv=64, T=256 from zero state with the benchmark's value recipe: with |k| ~ 1 and
    gates in (0,1) the transition is a contraction, so the state cannot blow up."""
    p = gen.recurrent_inputs(1001, 2, 256, 4, 4, 64, 64, False)
    S0 = gen.recurrent_state(0, 8, 64, 64, std=0.0).reshape(2, 4, 64, 64)
    o, S = om.gdn_steps(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 64 ** -0.5)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(S))
    assert 0.05 < np.sqrt(np.mean(S ** 2)) < 1.0
