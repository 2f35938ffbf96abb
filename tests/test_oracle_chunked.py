"""The chunk-parallel (triangular-solve) form and the step-by-step form are two independent routes from the
printed recurrences to the same numbers; they must agree, on random problems and on the benchmark recipe."""
import numpy as np
import pytest

from oracle import chunked as oc
from oracle import mixers as om
from paper_2604_19877_amd import inputs as gen


@pytest.mark.parametrize("per_channel", [False, True])
@pytest.mark.parametrize("T", [1, 2, 16, 37])
def test_chunk_form_equals_sequential_form(per_channel, T):
    rng = np.random.default_rng(11 + T)
    B, H, Hk, dk, dv = 2, 4, 2, 6, 5
    q, k, v = rng.standard_normal((B, T, Hk, dk)), rng.standard_normal((B, T, Hk, dk)), rng.standard_normal((B, T, H, dv))
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    beta = rng.uniform(0.1, 0.9, (B, T, H))
    alpha = rng.uniform(0.6, 0.99, (B, T, H, dk) if per_channel else (B, T, H))
    S0 = rng.standard_normal((B, H, dk, dv))
    seq = om.kda_steps if per_channel else om.gdn_steps
    o1, S1 = seq(q, k, v, alpha, beta, S0, 0.7)
    o2, S2 = oc.chunk_steps(q, k, v, alpha, beta, S0, 0.7, per_channel)
    np.testing.assert_allclose(o2, o1, rtol=0, atol=1e-10)
    np.testing.assert_allclose(S2, S1, rtol=0, atol=1e-10)


@pytest.mark.parametrize("per_channel", [False, True])
def test_chunks_chain_like_steps_on_the_benchmark_recipe(per_channel):
    """64 tokens of the benchmark's value recipe (bf16 operands, 128x128 state) as four chunks of 16."""
    p = gen.recurrent_inputs(77, 1, 64, 2, 2, 128, 128, per_channel)
    S0 = gen.recurrent_state(78, 2, 128, 128).reshape(1, 2, 128, 128)
    seq = om.kda_steps if per_channel else om.gdn_steps
    o1, S1 = seq(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 128 ** -0.5)
    S, outs = S0, []
    for c in range(4):
        sl = slice(16 * c, 16 * c + 16)
        o, S = oc.chunk_steps(p["q"][:, sl], p["k"][:, sl], p["v"][:, sl], p["alpha"][:, sl], p["beta"][:, sl], S, 128 ** -0.5,
                              per_channel)
        outs.append(o)
    np.testing.assert_allclose(np.concatenate(outs, 1), o1, rtol=0, atol=1e-9)
    np.testing.assert_allclose(S, S1, rtol=0, atol=1e-9)
