"""GPU parity of gdn_block_decode / kda_block_decode (conv + SiLU, L2 norm, gates, state update, gated
RMS norm in one launch) against the block oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import recurrent_block as ob
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, STATE_TOL, Guarded, dev, host, rel_err

pytestmark = pytest.mark.gpu

FN = {False: (sa.gdn_block_decode, "gdn"), True: (sa.kda_block_decode, "kda")}


def run_block(kda, p, S0, B, H, Hk, dk, dv, taps, gate_act, scale, slot=None, req=None, in_place=True, eps=1e-5):
    """One fused launch; returns (out, state, conv_q, conv_k, conv_v) as host arrays plus the guards."""
    d = {n: dev(a) for n, a in p.items()}
    state = Guarded(S0)
    conv_in = {n: Guarded(p[n]) for n in ("conv_q", "conv_k", "conv_v")}
    conv_out = conv_in if in_place else {n: Guarded(np.full_like(p[n], 0x7FC0)) for n in conv_in}
    out = Guarded(np.full((B, H, dv), 77.0, dtype=np.float32))
    io = sa.make_block_io(xq=d["xq"], xk=d["xk"], xv=d["xv"], wq=d["wq"], wk=d["wk"], wv=d["wv"],
                          conv_q_in=conv_in["conv_q"].ptr(), conv_k_in=conv_in["conv_k"].ptr(), conv_v_in=conv_in["conv_v"].ptr(),
                          conv_q_out=conv_out["conv_q"].ptr(), conv_k_out=conv_out["conv_k"].ptr(), conv_v_out=conv_out["conv_v"].ptr(),
                          conv_taps=taps, beta_raw=d["beta_raw"], alpha_raw=d["alpha_raw"], A_log=d["A_log"], dt_bias=d["dt_bias"],
                          z=d["z"], norm_weight=d["norm_weight"], norm_eps=eps, gate_act=gate_act)
    FN[kda][0](io, state.ptr(), state.ptr(), out.ptr(), None if slot is None else dev(slot), None if req is None else dev(req),
               0 if req is None else len(req), B, H, Hk, dk, dv, scale)
    torch.cuda.synchronize()
    guards = [state, out] + list(conv_in.values()) + list(conv_out.values())
    assert all(g.bands_intact() for g in guards)
    return out.read(), state.read(), {n: conv_out[n].read() for n in conv_out}, {n: conv_in[n].read() for n in conv_in}


def oracle_block(kda, p, S0, rows, slots, taps, gate_act, scale, eps=1e-5):
    return ob.block_decode_step(FN[kda][1], p["xq"][rows], p["xk"][rows], p["xv"][rows], p["conv_q"][slots], p["conv_k"][slots],
                                p["conv_v"][slots], p["wq"], p["wk"], p["wv"], p["beta_raw"][rows], p["alpha_raw"][rows],
                                p["A_log"], p["dt_bias"], p["z"][rows], p["norm_weight"], eps,
                                "silu" if gate_act == 0 else "sigmoid", S0[slots], scale)


@pytest.mark.parametrize("kda", [False, True])
@pytest.mark.parametrize("dk,taps,gate_act", [(128, 4, 0), (128, 2, 1), (64, 3, 0)])
def test_block_step_in_place(kda, dk, taps, gate_act):
    B, H = 5, 8
    p = gen.block_inputs(7001 + kda + taps, B, H, H, dk, dk, taps, kda)
    S0 = gen.recurrent_state(7002, B * H, dk, dk, std=0.3).reshape(B, H, dk, dk)
    out, S, conv, _ = run_block(kda, p, S0, B, H, H, dk, dk, taps, gate_act, dk ** -0.5)
    ref = oracle_block(kda, p, S0, slice(None), slice(None), taps, gate_act, dk ** -0.5)
    assert rel_err(out, ref["out"]) <= OUT_TOL
    assert rel_err(S, ref["state"]) <= STATE_TOL
    for n in ("conv_q", "conv_k", "conv_v"):           # histories are moved bit for bit
        assert np.array_equal(conv[n], gen.f32_to_bf16_bits(ref[n].astype(np.float32)))


@pytest.mark.parametrize("kda", [False, True])
def test_shared_key_heads_slots_and_request_list(kda):
    """Hk < H (4 state heads per q/k head), permuted slots, a request sub-list, out-of-place histories:
    unlisted rows, unlisted slots and the input histories stay untouched."""
    B, H, Hk, dk, taps, n_slots = 6, 8, 2, 128, 4, 9
    p = gen.block_inputs(7011 + kda, B, H, Hk, dk, dk, taps, kda, n_slots=n_slots)
    S0 = gen.recurrent_state(7012, n_slots * H, dk, dk, std=0.3).reshape(n_slots, H, dk, dk)
    slot = np.array([4, 0, 8, 2, 7, 5], dtype=np.int32)
    req = np.array([5, 1, 3], dtype=np.int32)
    out, S, conv, conv_in_after = run_block(kda, p, S0, B, H, Hk, dk, dk, taps, 0, 0.1, slot=slot, req=req, in_place=False)
    ref = oracle_block(kda, p, S0, req, slot[req], taps, 0, 0.1)
    assert rel_err(out[req], ref["out"]) <= OUT_TOL
    assert rel_err(S[slot[req]], ref["state"]) <= STATE_TOL
    for n in ("conv_q", "conv_k", "conv_v"):
        assert np.array_equal(conv[n][slot[req]], gen.f32_to_bf16_bits(ref[n].astype(np.float32)))
        assert np.array_equal(conv_in_after[n], p[n])
        others = [s for s in range(n_slots) if s not in slot[req]]
        assert (conv[n][others] == 0x7FC0).all()
    assert (out[[0, 2, 4]] == 77.0).all()
    others = [s for s in range(n_slots) if s not in slot[req]]
    assert np.array_equal(S[others], S0[others])


def test_argument_errors():
    p = gen.block_inputs(7021, 2, 4, 2, 128, 128, 4, False)
    d = {n: dev(a) for n, a in p.items()}
    st = torch.zeros((2 * 4, 128, 128), device="cuda")
    out = torch.zeros((2, 4, 128), device="cuda")
    base = dict(xq=d["xq"], xk=d["xk"], xv=d["xv"], wq=d["wq"], wk=d["wk"], wv=d["wv"], conv_q_in=d["conv_q"], conv_k_in=d["conv_k"],
                conv_v_in=d["conv_v"], conv_q_out=d["conv_q"], conv_k_out=d["conv_k"], conv_v_out=d["conv_v"], conv_taps=4,
                beta_raw=d["beta_raw"], alpha_raw=d["alpha_raw"], A_log=d["A_log"], dt_bias=d["dt_bias"], z=d["z"],
                norm_weight=d["norm_weight"], norm_eps=1e-5, gate_act=0)
    for change, code in ((dict(), sa.SA_EINVAL),                       # in-place q/k histories with Hk < H
                         (dict(conv_taps=5), sa.SA_EUNSUPPORTED), (dict(gate_act=2), sa.SA_EINVAL), (dict(z=None), sa.SA_EINVAL)):
        with pytest.raises(sa.SaError) as e:
            sa.gdn_block_decode(sa.make_block_io(**{**base, **change}), st, st, out, None, None, 0, 2, 4, 2, 128, 128, 1.0)
        assert e.value.status == code, change
    assert (out == 0).all()


@pytest.mark.parametrize("kda", [False, True])
def test_decode_loop_of_eight_tokens_carries_state_and_histories(kda):
    """Eight consecutive tokens through the fused block, state and histories updated in place each step,
    against the oracle fed the same way."""
    B, H, dk, taps = 2, 4, 128, 4
    first = gen.block_inputs(7031 + kda, B, H, H, dk, dk, taps, kda)
    S = np.zeros((B, H, dk, dk), dtype=np.float32)
    conv = {n: first[n].copy() for n in ("conv_q", "conv_k", "conv_v")}
    S_ref, conv_ref = S.astype(np.float64), {n: c.copy() for n, c in conv.items()}
    for t in range(8):
        p = dict(first)
        step = gen.block_inputs(7040 + 3 * t + kda, B, H, H, dk, dk, taps, kda)
        for n in ("xq", "xk", "xv", "z", "beta_raw", "alpha_raw"):
            p[n] = step[n]
        out, S, conv, _ = run_block(kda, {**p, **conv}, S, B, H, H, dk, dk, taps, 0, dk ** -0.5)
        ref = ob.block_decode_step(FN[kda][1], p["xq"], p["xk"], p["xv"], conv_ref["conv_q"], conv_ref["conv_k"], conv_ref["conv_v"],
                                   p["wq"], p["wk"], p["wv"], p["beta_raw"], p["alpha_raw"], p["A_log"], p["dt_bias"], p["z"],
                                   p["norm_weight"], 1e-5, "silu", S_ref, dk ** -0.5)
        S_ref = ref["state"]
        conv_ref = {n: gen.f32_to_bf16_bits(ref[n].astype(np.float32)) for n in conv_ref}
        assert rel_err(out, ref["out"]) <= OUT_TOL, t
    assert rel_err(S, S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", [False, True])
def test_full_shape_batch64_sampled_rows(kda):
    """Batch 64, 32 heads, 128x128 states, 4 taps: every tile on the GPU, the oracle on sampled rows."""
    B, H, dk, taps = 64, 32, 128, 4
    p = gen.block_inputs(7051 + kda, B, H, H, dk, dk, taps, kda)
    S0 = gen.recurrent_state(7052, B * H, dk, dk).reshape(B, H, dk, dk)
    out, S, conv, _ = run_block(kda, p, S0, B, H, H, dk, dk, taps, 0, dk ** -0.5)
    assert np.isfinite(out).all() and np.isfinite(S).all()
    rows = np.array([0, 17, 40, 63])
    ref = oracle_block(kda, p, S0, rows, rows, taps, 0, dk ** -0.5)
    assert rel_err(out[rows], ref["out"]) <= OUT_TOL
    assert rel_err(S[rows], ref["state"]) <= STATE_TOL
    for n in ("conv_q", "conv_k", "conv_v"):
        assert np.array_equal(conv[n][rows], gen.f32_to_bf16_bits(ref[n].astype(np.float32)))
