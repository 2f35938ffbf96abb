"""GPU parity of the chunk-parallel recurrent entry points against the step-by-step fp64 oracle (the printed
recurrence), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, STATE_TOL, Guarded, dev, host, rel_err

pytestmark = pytest.mark.gpu

FN = {False: (sa.gdn_chunk_steps, om.gdn_steps)}
if hasattr(sa, "kda_chunk_steps"):
    FN[True] = (sa.kda_chunk_steps, om.kda_steps)
KINDS = sorted(FN)


def run_chunked(kda, p, S0, B, T, H, Hk, scale, slot_idx=None, req_idx=None, n_slots=None):
    d = {n: dev(a) for n, a in p.items()}
    state = dev(S0.copy())
    out = torch.full((B, T, H, 128), float("nan"), dtype=torch.float32, device="cuda")
    FN[kda][0](d["q"], d["k"], d["v"], d["alpha"], d["beta"], state, state, out,
               None if slot_idx is None else dev(slot_idx), None if req_idx is None else dev(req_idx),
               0 if req_idx is None else len(req_idx), B, T, H, Hk, 128, 128, scale)
    torch.cuda.synchronize()
    return host(out), host(state)


@pytest.mark.parametrize("kda", KINDS)
@pytest.mark.parametrize("T", [1, 5, 16, 17, 40, 64])
@pytest.mark.parametrize("Hk", [4, 2])
def test_chunked_call_equals_the_recurrence(kda, T, Hk):
    """One call over T tokens (full chunks, a ragged tail, less than one chunk) against T oracle steps."""
    B, H = 3, 4
    p = gen.recurrent_inputs(4100 + T + 7 * Hk + kda, B, T, H, Hk, 128, 128, kda)
    S0 = gen.recurrent_state(4200 + T, B * H, 128, 128).reshape(B, H, 128, 128)
    scale = 128 ** -0.5
    o, S = run_chunked(kda, p, S0, B, T, H, Hk, scale)
    o_ref, S_ref = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, scale)
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(S, S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", KINDS)
def test_256_tokens_in_four_calls_state_tolerance(kda):
    """The state tolerance is stated after 256 steps: 4 calls of 64 tokens, state carried in place."""
    B, H, T, calls = 2, 4, 64, 4
    p = gen.recurrent_inputs(4300 + kda, B, T * calls, H, H, 128, 128, kda)
    S0 = gen.recurrent_state(4301, B * H, 128, 128).reshape(B, H, 128, 128)
    scale = 128 ** -0.5
    d = {n: dev(a) for n, a in p.items()}
    state = dev(S0.copy())
    outs = []
    for c in range(calls):
        sl = slice(c * T, (c + 1) * T)
        out = torch.empty((B, T, H, 128), dtype=torch.float32, device="cuda")
        FN[kda][0](d["q"][:, sl].contiguous(), d["k"][:, sl].contiguous(), d["v"][:, sl].contiguous(),
                   d["alpha"][:, sl].contiguous(), d["beta"][:, sl].contiguous(), state, state, out, None, None, 0,
                   B, T, H, H, 128, 128, scale)
        outs.append(out)
    torch.cuda.synchronize()
    o = np.concatenate([host(x) for x in outs], axis=1)
    o_ref, S_ref = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, scale)
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(host(state), S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", KINDS)
def test_slow_decay_and_strong_writes(kda):
    """Gates near 1 (the state remembers the whole call) and beta near 1 with repeated keys: the triangular
    system is then far from the identity."""
    B, H, T = 2, 2, 48
    p = gen.recurrent_inputs(4400 + kda, B, T, H, H, 128, 128, kda)
    rng = np.random.default_rng(4401)
    p["alpha"] = rng.uniform(0.97, 1.0, p["alpha"].shape).astype(np.float32)
    p["beta"] = rng.uniform(0.9, 1.0, p["beta"].shape).astype(np.float32)
    p["k"][:, 1::2] = p["k"][:, 0:-1:2]   # every second token repeats the key before it
    S0 = gen.recurrent_state(4402, B * H, 128, 128).reshape(B, H, 128, 128)
    o, S = run_chunked(kda, p, S0, B, T, H, H, 1.0)
    o_ref, S_ref = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 1.0)
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(S, S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", KINDS)
def test_vanishing_gates_stay_finite(kda):
    """Gates so small that their product over a chunk underflows fp32: the result must stay finite and right."""
    B, H, T = 1, 2, 32
    p = gen.recurrent_inputs(4500 + kda, B, T, H, H, 128, 128, kda)
    p["alpha"] = np.full(p["alpha"].shape, 1e-4, dtype=np.float32)
    S0 = gen.recurrent_state(4501, B * H, 128, 128).reshape(B, H, 128, 128)
    o, S = run_chunked(kda, p, S0, B, T, H, H, 1.0)
    o_ref, S_ref = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 1.0)
    assert np.isfinite(o).all() and np.isfinite(S).all()
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(S, S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", KINDS)
@pytest.mark.parametrize("n_commit", [None, 0, 603, 608])
def test_moderate_decay_over_many_chunks(kda, n_commit):
    """Gates around 0.9 over 44 chunks: the decay accumulated since the call's start passes 2^-96 once and is far
    from 1 where the committed prefix ends (inside a chunk, and on a chunk's boundary)."""
    B, H, T = 1, 2, 700
    p = gen.recurrent_inputs(4560 + kda, B, T, H, H, 128, 128, kda)
    rng = np.random.default_rng(4561)
    p["alpha"] = rng.uniform(0.85, 0.95, p["alpha"].shape).astype(np.float32)
    S0 = gen.recurrent_state(4562, B * H, 128, 128).reshape(B, H, 128, 128)
    d = {n: dev(a) for n, a in p.items()}
    s_in, s_out = dev(S0.copy()), dev(np.full_like(S0, np.nan))
    out = torch.full((B, T, H, 128), float("nan"), dtype=torch.float32, device="cuda")
    FN[kda][0](d["q"], d["k"], d["v"], d["alpha"], d["beta"], s_in, s_out, out, None, None, 0, B, T, H, H, 128, 128, 0.25,
               T if n_commit is None else n_commit)
    torch.cuda.synchronize()
    o_ref, S_ref = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 0.25)
    if n_commit is not None:
        cut = {n: a[:, :n_commit] for n, a in p.items()}
        S_ref = FN[kda][1](cut["q"], cut["k"], cut["v"], cut["alpha"], cut["beta"], S0, 0.25)[1] if n_commit else S0
    assert rel_err(host(out), o_ref) <= OUT_TOL
    assert rel_err(host(s_out), S_ref) <= STATE_TOL
    assert np.array_equal(host(s_in), S0)


def test_kda_few_channels_with_tiny_gates_split_the_chunk():
    """A handful of key channels decay by 1e-9 per token while the rest follow the recipe: the product of
    gates over a chunk leaves the range in which it can be divided by, so chunks run in several passes."""
    if True not in FN:
        pytest.skip("no chunked KDA entry point")
    B, H, T = 2, 2, 40
    p = gen.recurrent_inputs(4550, B, T, H, H, 128, 128, True)
    rng = np.random.default_rng(4551)
    tiny = rng.random(p["alpha"].shape) < 0.03
    p["alpha"] = np.where(tiny, np.float32(1e-9), p["alpha"]).astype(np.float32)
    S0 = gen.recurrent_state(4552, B * H, 128, 128).reshape(B, H, 128, 128)
    o, S = run_chunked(True, p, S0, B, T, H, H, 1.0)
    o_ref, S_ref = om.kda_steps(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 1.0)
    assert np.isfinite(o).all() and np.isfinite(S).all()
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(S, S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", KINDS)
def test_slots_request_list_and_untouched_rows(kda):
    """State slots differ from batch rows, only listed rows run, everything else keeps its bytes."""
    B, H, T, n_slots = 5, 2, 20, 7
    p = gen.recurrent_inputs(4600 + kda, B, T, H, H, 128, 128, kda)
    pool = gen.recurrent_state(4601, n_slots * H, 128, 128).reshape(n_slots, H, 128, 128)
    slot_idx = np.array([6, 2, 0, 5, 3], dtype=np.int32)
    req_idx = np.array([3, 0, 4], dtype=np.int32)
    d = {n: dev(a) for n, a in p.items()}
    gs = Guarded(pool.copy())
    go = Guarded(np.full((B, T, H, 128), 7.0, dtype=np.float32))
    FN[kda][0](d["q"], d["k"], d["v"], d["alpha"], d["beta"], gs.ptr(), gs.ptr(), go.ptr(), dev(slot_idx), dev(req_idx),
               len(req_idx), B, T, H, H, 128, 128, 0.5)
    torch.cuda.synchronize()
    S, o = gs.read(), go.read()
    assert gs.bands_intact() and go.bands_intact()
    for b in range(B):
        sl = slice(b, b + 1)
        if b in req_idx:
            o_ref, S_ref = FN[kda][1](p["q"][sl], p["k"][sl], p["v"][sl], p["alpha"][sl], p["beta"][sl],
                                      pool[slot_idx[b]:slot_idx[b] + 1], 0.5)
            assert rel_err(o[b], o_ref[0]) <= OUT_TOL
            assert rel_err(S[slot_idx[b]], S_ref[0]) <= STATE_TOL
        else:
            assert (o[b] == 7.0).all()
            assert np.array_equal(S[slot_idx[b]], pool[slot_idx[b]])
    for s in set(range(n_slots)) - set(slot_idx.tolist()):
        assert np.array_equal(S[s], pool[s])


@pytest.mark.parametrize("kda", KINDS)
def test_chunked_full_shape_every_tile_against_the_oracle(kda):
    """Batch 64 x 32 heads, 64 tokens in one chunked call: every tile against the fp64 C form of the oracle (admitted at
    1e-12 from the numpy oracle by tests/test_oracle_omp.py) at the tolerances of the decode steps.  Why they hold: every
    fp32 operand of a matrix product enters as two bf16 terms rounded to nearest, a relative error of 2^-18 = 3.8e-6 per
    operand; a token's correction passes through three such products and 64 tokens of them add up with random signs.
    Measured here over all 2048 tiles, worst tile: outputs 6.4e-5 (GDN) / 7.2e-5 (KDA), states 2.3e-5 / 4.2e-5 (the fp32
    one-token kernels: below 1e-6).  Outputs get a second bound at a tenth of their tolerance as a guard on the
    arithmetic: a single bf16 term anywhere (2^-9 per operand) would show as about 1e-3."""
    from oracle import omp
    B, H, T = 64, 32, 64
    p = gen.recurrent_inputs(4700 + kda, B, T, H, H, 128, 128, kda)
    S0 = gen.recurrent_state(4701, B * H, 128, 128).reshape(B, H, 128, 128)
    scale = 128 ** -0.5
    o, S = run_chunked(kda, p, S0, B, T, H, H, scale)
    o_ref, S_ref = (omp.kda_steps if kda else omp.gdn_steps)(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, scale)
    err_o = max(rel_err(o[b, :, h], o_ref[b, :, h]) for b in range(B) for h in range(H))
    err_s = max(rel_err(S[b, h], S_ref[b, h]) for b in range(B) for h in range(H))
    print("chunked %s, 64 tokens, worst tile: outputs %.2e, states %.2e" % ("kda" if kda else "gdn", err_o, err_s))
    assert err_o <= OUT_TOL and err_s <= STATE_TOL
    assert err_o <= 2e-4


@pytest.mark.parametrize("kda", KINDS)
def test_prefill_with_chunks_then_decode_token_by_token(kda):
    """The two kernel families share the state layout: 100 tokens go through the chunked call, the next 12 through
    the one-token decode kernel on the same state buffer; the oracle runs all 112 steps in one go."""
    B, H, Hk, T0, T1 = 2, 4, 2, 100, 12
    p = gen.recurrent_inputs(4800 + kda, B, T0 + T1, H, Hk, 128, 128, kda)
    S0 = gen.recurrent_state(4801, B * H, 128, 128).reshape(B, H, 128, 128)
    scale = 128 ** -0.5
    d = {n: dev(a) for n, a in p.items()}
    state = dev(S0.copy())
    out0 = torch.empty((B, T0, H, 128), dtype=torch.float32, device="cuda")
    FN[kda][0](*[d[n][:, :T0].contiguous() for n in ("q", "k", "v", "alpha", "beta")], state, state, out0, None, None, 0,
               B, T0, H, Hk, 128, 128, scale)
    step = sa.kda_decode_step if kda else sa.gdn_decode_step
    outs = []
    for t in range(T0, T0 + T1):
        o = torch.empty((B, 1, H, 128), dtype=torch.float32, device="cuda")
        step(*[d[n][:, t:t + 1].contiguous() for n in ("q", "k", "v", "alpha", "beta")], state, state, o, None, None, 0,
             B, 1, H, Hk, 128, 128, scale, 1)
        outs.append(o)
    torch.cuda.synchronize()
    o_all = np.concatenate([host(out0)] + [host(x) for x in outs], axis=1)
    o_ref, S_ref = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, scale)
    assert rel_err(o_all, o_ref) <= OUT_TOL
    assert rel_err(host(state), S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", KINDS)
@pytest.mark.parametrize("n_commit", [0, 1, 7, 16, 21, 32, 39])
@pytest.mark.parametrize("in_place", [False, True])
def test_committed_prefix_of_a_chunked_call(kda, n_commit, in_place):
    """All 40 outputs are produced, the state written is the one after n_commit tokens (inside a chunk, at a chunk
    boundary, nothing at all); out of place the input state keeps its bytes."""
    B, H, T = 2, 2, 40
    p = gen.recurrent_inputs(4900 + kda + n_commit, B, T, H, H, 128, 128, kda)
    S0 = gen.recurrent_state(4901, B * H, 128, 128).reshape(B, H, 128, 128)
    d = {n: dev(a) for n, a in p.items()}
    s_in = dev(S0.copy())
    s_out = s_in if in_place else torch.full_like(s_in, float("nan"))
    out = torch.empty((B, T, H, 128), dtype=torch.float32, device="cuda")
    FN[kda][0](d["q"], d["k"], d["v"], d["alpha"], d["beta"], s_in, s_out, out, None, None, 0, B, T, H, H, 128, 128, 0.25,
               n_commit)
    torch.cuda.synchronize()
    o_ref, _ = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 0.25)
    cut = {n: a[:, :n_commit] for n, a in p.items()}
    S_ref = FN[kda][1](cut["q"], cut["k"], cut["v"], cut["alpha"], cut["beta"], S0, 0.25)[1] if n_commit else S0
    assert rel_err(host(out), o_ref) <= OUT_TOL
    assert rel_err(host(s_out), S_ref) <= STATE_TOL
    if not in_place:
        assert np.array_equal(host(s_in), S0)


@pytest.mark.parametrize("kda", KINDS)
def test_decode_step_with_eight_tokens_runs_on_the_chunk_kernels_and_keeps_its_contract(kda):
    """gdn_decode_step / kda_decode_step hand longer calls (from 7 / 8 tokens) to the chunk-parallel kernels: an 8-token
    verify with 3 accepted tokens, out of place."""
    B, H, T, n_commit = 3, 4, 8, 3
    p = gen.recurrent_inputs(4950 + kda, B, T, H, H, 128, 128, kda)
    S0 = gen.recurrent_state(4951, B * H, 128, 128).reshape(B, H, 128, 128)
    d = {n: dev(a) for n, a in p.items()}
    s_in, s_out = dev(S0.copy()), torch.empty((B, H, 128, 128), dtype=torch.float32, device="cuda")
    out = torch.empty((B, T, H, 128), dtype=torch.float32, device="cuda")
    step, kid = (sa.kda_decode_step, sa.SA_K_KDA_CHUNK) if kda else (sa.gdn_decode_step, sa.SA_K_GDN_CHUNK)
    sa.sa_prof_read(kid)
    sa.sa_prof_enable(True)
    step(d["q"], d["k"], d["v"], d["alpha"], d["beta"], s_in, s_out, out, None, None, 0, B, T, H, H, 128, 128, 1.0, n_commit)
    torch.cuda.synchronize()
    sa.sa_prof_enable(False)
    assert sa.sa_prof_read(kid)[0] == 1
    o_ref, _ = FN[kda][1](p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 1.0)
    S_ref = FN[kda][1](*[p[n][:, :n_commit] for n in ("q", "k", "v", "alpha", "beta")], S0, 1.0)[1]
    assert rel_err(host(out), o_ref) <= OUT_TOL
    assert rel_err(host(s_out), S_ref) <= STATE_TOL
    assert np.array_equal(host(s_in), S0)


@pytest.mark.parametrize("kda", KINDS)
def test_long_prefill_full_batch_sampled_tiles(kda):
    """64 sequences x 32 heads x 512 tokens in one call (the shape bench.py --prefill times); the oracle follows a
    seeded sample of tiles through all 512 steps."""
    B, H, T = 64, 32, 512
    g = torch.Generator(device="cuda")
    g.manual_seed(4990 + kda)
    nrm = lambda x: (x / x.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    q = nrm(torch.empty((B, T, H, 128), device="cuda").normal_(generator=g))
    k = nrm(torch.empty((B, T, H, 128), device="cuda").normal_(generator=g))
    v = torch.empty((B, T, H, 128), device="cuda").normal_(generator=g).bfloat16()
    beta = torch.sigmoid(torch.empty((B, T, H), device="cuda").normal_(generator=g))
    alpha = torch.exp(-torch.nn.functional.softplus(
        torch.empty((B, T, H, 128) if kda else (B, T, H), device="cuda").normal_(generator=g) + 2.0))
    S0 = torch.empty((B, H, 128, 128), device="cuda").normal_(0.0, 0.02, generator=g)
    state = S0.clone()
    out = torch.empty((B, T, H, 128), dtype=torch.float32, device="cuda")
    FN[kda][0](q, k, v, alpha, beta, state, state, out, None, None, 0, B, T, H, H, 128, 128, 128 ** -0.5)
    torch.cuda.synchronize()
    rng = np.random.default_rng(4991)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    for b, h in [(0, 0), (B - 1, H - 1)] + [(int(rng.integers(B)), int(rng.integers(H))) for _ in range(6)]:
        sl = (slice(b, b + 1), slice(None), slice(h, h + 1))
        o_ref, S_ref = FN[kda][1](bits(q[sl]), bits(k[sl]), bits(v[sl]), alpha[sl].cpu().numpy(), beta[sl].cpu().numpy(),
                                  S0[b:b + 1, h:h + 1].cpu().numpy(), 128 ** -0.5)
        assert rel_err(host(out[sl]), o_ref) <= OUT_TOL, (b, h)
        assert rel_err(host(state[b:b + 1, h:h + 1]), S_ref) <= STATE_TOL, (b, h)
