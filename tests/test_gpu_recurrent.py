"""GPU parity of gdn_decode_step / kda_decode_step against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, STATE_TOL, Guarded, dev, host, rel_err

pytestmark = pytest.mark.gpu

FN = {False: (sa.gdn_decode_step, om.gdn_steps), True: (sa.kda_decode_step, om.kda_steps)}


def stepwise_inputs(seed, steps, B, T, H, Hk, dk, dv, kda):
    """Operands for `steps` consecutive calls of T tokens: arrays [steps,B,T,...]."""
    p = gen.recurrent_inputs(seed, steps * B, T, H, Hk, dk, dv, kda)
    return {n: a.reshape((steps, B) + a.shape[1:]) for n, a in p.items()}


def as_sequence(p, name):
    """[steps,B,T,...] -> [B,steps*T,...] for the oracle."""
    a = p[name]
    a = np.moveaxis(a, 0, 1)
    return a.reshape((a.shape[0], a.shape[1] * a.shape[2]) + a.shape[3:])


def run_gpu(kda, p, state0, B, T, H, Hk, dk, dv, scale):
    fn = FN[kda][0]
    steps = p["q"].shape[0]
    d = {n: dev(a) for n, a in p.items()}
    state = dev(state0.copy())
    out = torch.empty((steps, B, T, H, dv), dtype=torch.float32, device="cuda")
    for s in range(steps):
        fn(d["q"][s], d["k"][s], d["v"][s], d["alpha"][s], d["beta"][s], state, state, out[s], None, None, 0,
           B, T, H, Hk, dk, dv, scale, T)
    torch.cuda.synchronize()
    o = host(out)
    o = np.moveaxis(o, 0, 1).reshape(B, steps * T, H, dv)
    return o, host(state)


@pytest.mark.parametrize("kda", [False, True])
@pytest.mark.parametrize("T", [1, 8, 16])
def test_config1_256_tokens_from_zero_state(kda, T):
    """B=2, H=4, dk=dv=64, 256 tokens, zero initial state; fed 1, 8 and 16 tokens per call."""
    B, H, dk, dv, n_tok = 2, 4, 64, 64, 256
    p = stepwise_inputs(1001 + kda, n_tok // T, B, T, H, H, dk, dv, kda)
    S0 = np.zeros((B, H, dk, dv), dtype=np.float32)
    scale = dk ** -0.5
    o, S = run_gpu(kda, p, S0, B, T, H, H, dk, dv, scale)
    o_ref, S_ref = FN[kda][1](as_sequence(p, "q"), as_sequence(p, "k"), as_sequence(p, "v"), as_sequence(p, "alpha"),
                              as_sequence(p, "beta"), S0, scale)
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(S, S_ref) <= STATE_TOL


@pytest.mark.parametrize("kda", [False, True])
@pytest.mark.parametrize("tiny", [False, True])
def test_four_tokens_per_call_256_tokens(kda, tiny):
    """128x128 states, 4 tokens per call (the register-resident multi-token kernel), 64 calls: the state tolerance
    after 256 steps; with `tiny`, a third of the gates are 1e-7, so that the product of a call's gates leaves the
    range in which the GDN kernel carries it as a common factor of the tile."""
    B, H, Hk, d, T, n_tok = 2, 4, 2, 128, 4, 256
    p = stepwise_inputs(1101 + kda, n_tok // T, B, T, H, Hk, d, d, kda)
    if tiny:
        rng = np.random.default_rng(1102)
        p["alpha"] = np.where(rng.random(p["alpha"].shape) < 0.33, np.float32(1e-7), p["alpha"]).astype(np.float32)
    S0 = gen.recurrent_state(1103, B * H, d, d).reshape(B, H, d, d)
    scale = d ** -0.5
    o, S = run_gpu(kda, p, S0, B, T, H, Hk, d, d, scale)
    o_ref, S_ref = FN[kda][1](as_sequence(p, "q"), as_sequence(p, "k"), as_sequence(p, "v"), as_sequence(p, "alpha"),
                              as_sequence(p, "beta"), S0, scale)
    assert np.isfinite(o).all() and np.isfinite(S).all()
    assert rel_err(o, o_ref) <= OUT_TOL
    assert rel_err(S, S_ref) <= STATE_TOL


def per_tile_rel_err(got, ref, head_axis):
    """max_i |g_i - r_i| / (|r_i| + rms(r)) per (sequence, head), the metric of gpu_util.rel_err tile by tile."""
    got = np.moveaxis(np.asarray(got, dtype=np.float64), head_axis, 1)
    ref = np.moveaxis(np.asarray(ref, dtype=np.float64), head_axis, 1)
    B, H = ref.shape[:2]
    got, ref = got.reshape(B, H, -1), ref.reshape(B, H, -1)
    rms = np.sqrt(np.mean(ref ** 2, axis=2, keepdims=True))
    return np.max(np.abs(got - ref) / (np.abs(ref) + rms), axis=2)


@pytest.mark.parametrize("kda,B", [(False, 64), (True, 64), (True, 256)])
def test_full_shape_256_steps_every_tile(kda, B):
    """BASELINE configs 2 and 3 (and 3's batch 256): 15B-class shape (32 heads, 128x128 fp32 states ~ N(0, 0.02^2)), 256
    consecutive steps on the GPU.  Every tile and every step is checked against the oracle's fp64 C form (plain loops,
    admitted at 1e-12 from the numpy oracle by tests/test_oracle_omp.py); a seeded sample of tiles is also followed by the
    numpy oracle itself, which the C form must match on those tiles at this size too."""
    from oracle import omp
    H, dk, dv, steps = 32, 128, 128, 256
    p = stepwise_inputs(1002 + kda + B, steps, B, 1, H, H, dk, dv, kda)
    S0 = gen.recurrent_state(7, B * H, dk, dv).reshape(B, H, dk, dv)
    scale = dk ** -0.5
    o, S = run_gpu(kda, p, S0, B, 1, H, H, dk, dv, scale)
    assert np.isfinite(o).all() and np.isfinite(S).all()
    seq = {n: as_sequence(p, n) for n in p}
    o_all, S_all = (omp.kda_steps if kda else omp.gdn_steps)(seq["q"], seq["k"], seq["v"], seq["alpha"], seq["beta"], S0, scale)
    err_o, err_s = per_tile_rel_err(o, o_all, 2), per_tile_rel_err(S, S_all, 1)
    assert err_o.max() <= OUT_TOL, np.unravel_index(err_o.argmax(), err_o.shape)
    assert err_s.max() <= STATE_TOL, np.unravel_index(err_s.argmax(), err_s.shape)
    rng = np.random.default_rng(5)
    tiles = [(int(rng.integers(B)), int(rng.integers(H))) for _ in range(30)] + [(0, 0), (B - 1, H - 1)]
    for (b, h) in tiles:
        sl = (slice(b, b + 1), slice(None), slice(h, h + 1))
        o_ref, S_ref = FN[kda][1](seq["q"][sl], seq["k"][sl], seq["v"][sl], seq["alpha"][sl], seq["beta"][sl],
                                  S0[b:b + 1, h:h + 1], scale)
        assert rel_err(o[b, :, h], o_ref[0, :, 0]) <= OUT_TOL, (b, h)
        assert rel_err(S[b, h], S_ref[0, 0]) <= STATE_TOL, (b, h)
        assert np.max(np.abs(o_all[b, :, h] - o_ref[0, :, 0])) <= 1e-12 and np.max(np.abs(S_all[b, h] - S_ref[0, 0])) <= 1e-12


@pytest.mark.parametrize("kda", [False, True])
def test_grouped_key_heads_slots_request_lists_and_commit_prefix(kda):
    """Hk < H, a permuted slot map, a request sub-list, out-of-place state with n_commit < T; rows that
    are not listed and all guard bands must stay untouched."""
    fn, ref = FN[kda]
    B, T, H, Hk, dk, dv = 5, 4, 8, 2, 128, 128
    p = gen.recurrent_inputs(2001 + kda, B, T, H, Hk, dk, dv, kda)
    n_slots = 7
    S0 = gen.recurrent_state(8, n_slots * H, dk, dv, std=0.5).reshape(n_slots, H, dk, dv)
    slot = np.array([3, 0, 6, 1, 4], dtype=np.int32)
    req = np.array([4, 1, 2], dtype=np.int32)
    d = {n: dev(a) for n, a in p.items()}
    for n_commit in (0, 2, 4):
        s_in, s_out = Guarded(S0), Guarded(np.full_like(S0, 7.0))
        out = Guarded(np.full((B, T, H, dv), 9.0, dtype=np.float32))
        fn(d["q"], d["k"], d["v"], d["alpha"], d["beta"], s_in.ptr(), s_out.ptr(), out.ptr(), dev(slot), dev(req), len(req),
           B, T, H, Hk, dk, dv, 0.25, n_commit)
        torch.cuda.synchronize()
        got_o, got_s = out.read(), s_out.read()
        assert np.array_equal(s_in.read(), S0)
        assert s_in.bands_intact() and s_out.bands_intact() and out.bands_intact()
        o_ref, S_ref = ref(p["q"][req], p["k"][req], p["v"][req], p["alpha"][req], p["beta"][req], S0[slot[req]], 0.25,
                           n_commit=n_commit)
        assert rel_err(got_o[req], o_ref) <= OUT_TOL
        if n_commit == 0:
            assert np.array_equal(got_s[slot[req]], S0[slot[req]])
        else:
            assert rel_err(got_s[slot[req]], S_ref) <= STATE_TOL
        untouched_rows = [b for b in range(B) if b not in req]
        assert (got_o[untouched_rows] == 9.0).all()
        untouched_slots = [s for s in range(n_slots) if s not in slot[req]]
        assert (got_s[untouched_slots] == 7.0).all()


@pytest.mark.parametrize("kda", [False, True])
def test_identities_on_the_gpu(kda):
    """alpha = 1, beta = 0 leaves the state bit-identical; a uniform channel gate makes KDA equal GDN
    bit for bit (same kernel arithmetic)."""
    fn, _ = FN[kda]
    B, H, dk, dv = 3, 4, 128, 128
    p = gen.recurrent_inputs(2003, B, 1, H, H, dk, dv, kda)
    S0 = gen.recurrent_state(9, B * H, dk, dv, std=1.0).reshape(B, H, dk, dv)
    d = {n: dev(a) for n, a in p.items()}
    state = dev(S0.copy())
    out = torch.empty((B, 1, H, dv), dtype=torch.float32, device="cuda")
    fn(d["q"], d["k"], d["v"], torch.ones_like(d["alpha"]), torch.zeros_like(d["beta"]), state, state, out, None, None, 0,
       B, 1, H, H, dk, dv, 1.0, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host(state), S0)
    if kda:
        g = gen.recurrent_inputs(2003, B, 1, H, H, dk, dv, False)
        a_vec = np.repeat(g["alpha"][..., None], dk, axis=-1).astype(np.float32)
        s1, s2 = dev(S0.copy()), dev(S0.copy())
        o1, o2 = torch.empty_like(out), torch.empty_like(out)
        dg = {n: dev(a) for n, a in g.items()}
        sa.gdn_decode_step(dg["q"], dg["k"], dg["v"], dg["alpha"], dg["beta"], s1, s1, o1, None, None, 0, B, 1, H, H, dk, dv, 0.5, 1)
        sa.kda_decode_step(dg["q"], dg["k"], dg["v"], dev(a_vec), dg["beta"], s2, s2, o2, None, None, 0, B, 1, H, H, dk, dv, 0.5, 1)
        torch.cuda.synchronize()
        assert torch.equal(s1, s2) and torch.equal(o1, o2)


def test_state_pack_and_unpack_round_trip_and_feed_a_step():
    """A state written through sa_state_pack steps exactly like the same numbers uploaded directly, and
    sa_state_unpack returns the row-major [dk][dv] matrices the oracle works with."""
    B, H, dk, dv = 2, 4, 128, 128
    p = gen.recurrent_inputs(1500, B, 1, H, H, dk, dv, False)
    S0 = gen.recurrent_state(1501, B * H, dk, dv).reshape(B, H, dk, dv)
    assert sa.sa_state_tile_bytes(dk, dv) == dk * dv * 4
    rowmajor, tiles, back = dev(S0.copy()), torch.empty((B, H, dk, dv), device="cuda"), torch.empty((B, H, dk, dv), device="cuda")
    sa.sa_state_pack(rowmajor, tiles, B * H, dk, dv)
    d = {n: dev(a) for n, a in p.items()}
    out = torch.empty((B, 1, H, dv), dtype=torch.float32, device="cuda")
    sa.gdn_decode_step(d["q"], d["k"], d["v"], d["alpha"], d["beta"], tiles, tiles, out, None, None, 0, B, 1, H, H, dk, dv, 1.0, 1)
    sa.sa_state_unpack(tiles, back, B * H, dk, dv)
    torch.cuda.synchronize()
    o_ref, S_ref = om.gdn_steps(p["q"], p["k"], p["v"], p["alpha"], p["beta"], S0, 1.0)
    assert rel_err(host(out), o_ref) <= OUT_TOL
    assert rel_err(host(back), S_ref) <= STATE_TOL


def test_stream_tiles_calibration_kernel_touches_exactly_its_tiles():
    """The bandwidth-calibration kernel reads, fills or rescales n_tiles tiles of 128x128 and nothing beyond them."""
    n, guard = 5, 1024
    buf = torch.empty(n * 128 * 128 + 2 * guard, dtype=torch.float32, device="cuda").normal_()
    before = buf.clone()
    tiles = buf[guard:guard + n * 128 * 128]
    sa.sa_stream_tiles(0, tiles, n)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
    sa.sa_stream_tiles(2, tiles, n)
    torch.cuda.synchronize()
    assert torch.equal(tiles, before[guard:-guard] * 0.999)
    sa.sa_stream_tiles(1, tiles, n - 1)
    torch.cuda.synchronize()
    assert torch.equal(tiles[:(n - 1) * 128 * 128], torch.full(((n - 1) * 128 * 128,), 0.01, device="cuda"))
    assert torch.equal(tiles[(n - 1) * 128 * 128:], before[guard + (n - 1) * 128 * 128:-guard] * 0.999)
    assert torch.equal(buf[:guard], before[:guard]) and torch.equal(buf[-guard:], before[-guard:])


@pytest.mark.parametrize("kda", [False, True])
@pytest.mark.parametrize("T,dk", [(4, 128), (5, 128), (6, 128), (7, 128), (8, 128), (13, 128), (3, 64), (16, 64), (1, 128)])
def test_per_request_commit_counts(kda, T, dk):
    """Every request commits its own number of drafted tokens in one call (short calls on the register-resident kernel,
    longer ones, from 7 tokens for GDN and 8 for KDA at 128x128, on the chunk-parallel one); counts outside [0, T] are
    clamped; unlisted rows stay untouched."""
    B, H, Hk, dv = 7, 4, 2, dk
    p = gen.recurrent_inputs(1600 + T + kda, B, T, H, Hk, dk, dv, kda)
    S0 = gen.recurrent_state(1601, B * H, dk, dv, std=0.3).reshape(B, H, dk, dv)
    counts = np.array([0, T, 1, T - 1, T + 5, -3, T // 2], dtype=np.int32)
    req = np.array([6, 0, 1, 2, 3, 4], dtype=np.int32)            # row 5 is not processed
    fn, ref_fn = (sa.kda_decode_step_var, om.kda_steps) if kda else (sa.gdn_decode_step_var, om.gdn_steps)
    d = {n: dev(a) for n, a in p.items()}
    for in_place in (False, True):
        s_in = dev(S0.copy())
        s_out = s_in if in_place else dev(np.full_like(S0, 3.0))
        out = torch.full((B, T, H, dv), -7.0, dtype=torch.float32, device="cuda")
        fn(d["q"], d["k"], d["v"], d["alpha"], d["beta"], s_in, s_out, out, None, dev(req), len(req), B, T, H, Hk, dk, dv, 0.4,
           dev(counts))
        torch.cuda.synchronize()
        got_o, got_s = host(out), host(s_out)
        for b in req:
            n = int(min(max(counts[b], 0), T))
            sl = slice(b, b + 1)
            o_ref, S_ref = ref_fn(p["q"][sl], p["k"][sl], p["v"][sl], p["alpha"][sl], p["beta"][sl], S0[sl], 0.4, n_commit=n)
            assert rel_err(got_o[b], o_ref[0]) <= OUT_TOL, (b, n)
            if n == 0:
                assert np.array_equal(got_s[b], S0[b]), b          # nothing committed: the tile is copied
            else:
                assert rel_err(got_s[b], S_ref[0]) <= STATE_TOL, (b, n)
        assert (got_o[5] == -7.0).all()
        assert np.array_equal(got_s[5], S0[5]) if in_place else (got_s[5] == 3.0).all()
        if not in_place:
            assert np.array_equal(host(s_in), S0)
