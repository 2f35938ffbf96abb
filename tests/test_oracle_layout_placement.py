"""Pins for the KV page layout reference and the placement oracle."""
import numpy as np
import pytest

from oracle import kv_layout as kl
from oracle import mixers as om
from paper_2604_19877_amd import inputs as gen


def test_layout_offsets_are_bijections_and_match_stated_examples():
    D = 128
    ks = {kl.k_offset(j, d) for j in range(16) for d in range(D)}
    vs = {kl.v_offset(j, d) for j in range(16) for d in range(D)}
    assert ks == set(range(16 * D)) and vs == set(range(16 * D))
    # K: 8 consecutive dims of one token are contiguous, consecutive tokens of a chunk are 8 apart,
    # chunks are 128 apart.
    assert [kl.k_offset(0, d) for d in (0, 7, 8, 127)] == [0, 7, 128, 15 * 128 + 7]
    assert kl.k_offset(1, 0) == 8 and kl.k_offset(15, 127) == 2047
    # V: 4 consecutive tokens of one dim are contiguous, dims of a 16-block are 4 apart, token
    # groups 64 apart, dim blocks 256 apart.
    assert [kl.v_offset(j, 0) for j in (0, 3, 4, 15)] == [0, 3, 64, 195]
    assert kl.v_offset(0, 1) == 4 and kl.v_offset(0, 16) == 256 and kl.v_offset(15, 127) == 2047


def test_append_then_decode_round_trip():
    lens = np.array([37, 20], dtype=np.int32)
    p = gen.attention_inputs(31, 2, 1, 4, 2, 32, lens, 4)
    kp = np.zeros((p["n_pages"], 2, 16 * 32), dtype=np.uint16)
    vp = np.zeros_like(kp)
    # feed the tokens in two calls with different T
    kl.kv_append(p["k_tok"][:, :16], p["v_tok"][:, :16], kp, vp, p["page_table"], [0, 0])
    kl.kv_append(p["k_tok"][:, 16:20], p["v_tok"][:, 16:20], kp, vp, p["page_table"], [16, 16])
    kl.kv_append(p["k_tok"][:1, 20:37], p["v_tok"][:1, 20:37], kp, vp, p["page_table"], [20])
    klog, vlog = kl.to_logical(kp, vp, 32)
    want_k, want_v = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    for b in range(2):
        for j in range(int(lens[b])):
            pg = p["page_table"][b, j // 16]
            assert np.array_equal(klog[pg, :, j % 16], want_k[pg, :, j % 16])
            assert np.array_equal(vlog[pg, :, j % 16], want_v[pg, :, j % 16])
    kp2, vp2 = kl.to_physical(klog, vlog)
    assert np.array_equal(kp2, kp) and np.array_equal(vp2, vp)


def _stack(seed, B, L, placements):
    layers = []
    dk = dv = 8
    H = 4
    lens = np.full(B, 21, dtype=np.int32)
    for l in range(L):
        r = gen.recurrent_inputs(seed + l, B, 1, H, H, dk, dv, False)
        rv = gen.recurrent_inputs(seed + 100 + l, B, 1, H, H, dk, dv, True)
        a = gen.attention_inputs(seed + 200 + l, B, 1, H, 2, dv, lens, 2)
        kp, vp = gen.logical_pools(a["k_tok"], a["v_tok"], a["page_table"], lens, a["n_pages"])
        layers.append({"q": r["q"], "k": r["k"], "v": r["v"], "alpha_scalar": r["alpha"], "alpha_vec": rv["alpha"],
                       "beta": r["beta"], "state": gen.recurrent_state(seed + 300 + l, B * H, dk, dv).reshape(B, H, dk, dv),
                       "qa": a["q"], "kpool": kp, "vpool": vp, "page_table": a["page_table"], "seq_lens": lens})
    return layers


def test_placement_dispatch_equals_direct_calls():
    placements = ["FSKG", "GKSF", "KKFF"]
    pid = np.array([0, 1, 2, 1, 0], dtype=np.int32)
    layers = _stack(41, 5, 4, placements)
    outs, states = om.placement_decode(placements, pid, layers, 6, 0.3, 0.5)
    for l, io in enumerate(layers):
        for r in range(5):
            m = placements[pid[r]][l]
            sl = slice(r, r + 1)
            if m == "F":
                want = om.attn_decode(io["qa"][sl], io["kpool"], io["vpool"], io["page_table"][sl], io["seq_lens"][sl], 0, 0.3)
            elif m == "S":
                want = om.attn_decode(io["qa"][sl], io["kpool"], io["vpool"], io["page_table"][sl], io["seq_lens"][sl], 6, 0.3)
            elif m == "K":
                want, s = om.kda_steps(io["q"][sl], io["k"][sl], io["v"][sl], io["alpha_vec"][sl], io["beta"][sl], io["state"][sl], 0.5)
            else:
                want, s = om.gdn_steps(io["q"][sl], io["k"][sl], io["v"][sl], io["alpha_scalar"][sl], io["beta"][sl], io["state"][sl], 0.5)
            assert np.array_equal(outs[l][r], want[0])
            if m in "KG":
                assert np.array_equal(states[l][r], s[0])
            else:
                assert np.array_equal(states[l][r], om.widen(io["state"][r]))


def test_placement_parse_errors():
    with pytest.raises(ValueError):
        om.parse_placements(["FSK"], 4)
    with pytest.raises(ValueError):
        om.parse_placements(["FSKX"], 4)
    assert om.parse_placements(["FSKG"], 4) == [["F", "S", "K", "G"]]


def test_placement_string_generator():
    s = gen.placement_string(5001, 48)
    assert len(s) == 48 and all(s.count(c) == 12 for c in "FSKG")
    assert s == gen.placement_string(5001, 48) and s != gen.placement_string(5002, 48)
