"""Seeded random valid configurations (shapes, lengths, windows, token counts, request lists) of the
attention and recurrent entry points against the oracle: a sweep over the planner's and the kernels'
parameter space, not of invalid inputs."""
import numpy as np
import pytest
import torch

from oracle import kv_layout as kl
from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, STATE_TOL, dev, host, rel_err

pytestmark = pytest.mark.gpu
D = 128


@pytest.mark.parametrize("case", range(10))
def test_attention_random_configuration(case):
    rng = np.random.default_rng(9100 + case)
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 2, 4, 8]))
    T = int(rng.integers(1, min(8, 32 // group) + 1))
    hq = hkv * group
    B = int(rng.integers(1, 7))
    max_len = int(rng.choice([64, 300, 1500, 4000]))
    lens = rng.integers(0, max_len + 1, size=B).astype(np.int32)
    lens[rng.integers(B)] = max_len
    window = int(rng.choice([0, 0, 17, 128, 1000]))
    max_pages = (max_len + 15) // 16 + int(rng.integers(0, 3))
    p = gen.attention_inputs(9200 + case, B, T, hq, hkv, D, lens, max_pages)
    klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    kphys, vphys = kl.to_physical(klog, vlog)
    req = np.sort(rng.choice(B, size=int(rng.integers(1, B + 1)), replace=False)).astype(np.int32)
    rng.shuffle(req)
    ws_bytes = sa.attn_decode_workspace_bytes(len(req), T, hq, hkv, D, max_pages * 16, window)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    out = torch.full((B, T, hq, D), -7.0, dtype=torch.float32, device="cuda")
    sa.attn_decode(dev(p["q"]), dev(kphys), dev(vphys), p["n_pages"], dev(p["page_table"]), max_pages, dev(lens), dev(req), len(req),
                   out, B, T, hq, hkv, D, 16, max_pages * 16, window, D ** -0.5, ws, ws_bytes)
    torch.cuda.synchronize()
    got = host(out)
    ref = om.attn_decode(p["q"], klog, vlog, p["page_table"], lens, window, D ** -0.5)
    for b in range(B):
        if b in req:
            assert rel_err(got[b], ref[b]) <= OUT_TOL, (case, b, int(lens[b]), window, T, hq, hkv)
        else:
            assert (got[b] == -7.0).all()


@pytest.mark.parametrize("case", range(8))
def test_recurrent_random_configuration(case):
    rng = np.random.default_rng(9300 + case)
    kda = bool(rng.integers(2))
    dk = int(rng.choice([64, 128]))
    Hk = int(rng.choice([1, 2, 4]))
    H = Hk * int(rng.choice([1, 2, 4]))
    T = int(rng.integers(1, 9))
    B = int(rng.integers(1, 6))
    n_slots = B + int(rng.integers(0, 4))
    n_commit = int(rng.integers(0, T + 1))
    p = gen.recurrent_inputs(9400 + case, B, T, H, Hk, dk, dk, kda)
    S0 = gen.recurrent_state(9500 + case, n_slots * H, dk, dk, std=0.4).reshape(n_slots, H, dk, dk)
    slot = rng.permutation(n_slots)[:B].astype(np.int32)
    req = rng.permutation(B)[:int(rng.integers(1, B + 1))].astype(np.int32)
    fn, ref_fn = (sa.kda_decode_step, om.kda_steps) if kda else (sa.gdn_decode_step, om.gdn_steps)
    d = {n: dev(a) for n, a in p.items()}
    s_in, s_out = dev(S0.copy()), dev(np.full_like(S0, 3.0))
    out = torch.full((B, T, H, dk), -7.0, dtype=torch.float32, device="cuda")
    fn(d["q"], d["k"], d["v"], d["alpha"], d["beta"], s_in, s_out, out, dev(slot), dev(req), len(req), B, T, H, Hk, dk, dk, 0.3,
       n_commit)
    torch.cuda.synchronize()
    o_ref, S_ref = ref_fn(p["q"][req], p["k"][req], p["v"][req], p["alpha"][req], p["beta"][req], S0[slot[req]], 0.3,
                          n_commit=n_commit)
    got_o, got_s = host(out), host(s_out)
    assert rel_err(got_o[req], o_ref) <= OUT_TOL, (case, kda, dk, H, Hk, T, n_commit)
    assert rel_err(got_s[slot[req]], S_ref) <= STATE_TOL
    assert np.array_equal(host(s_in), S0)
    untouched = [s for s in range(n_slots) if s not in slot[req]]
    assert (got_s[untouched] == 3.0).all()
