"""Pins for the paged GQA attention oracle: hand example, scalar-loop brute force, scipy's softmax,
and the identities the FA / SWA definitions of Appendix B fix."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import mixers as om
from paper_2604_19877_amd import inputs as gen
from test_oracle_recurrent import read_golden


def small_problem(seed, B=2, T=1, Hq=4, Hkv=2, D=8, lens=(37, 20), max_pages=4):
    lens = np.array(lens, dtype=np.int32)
    p = gen.attention_inputs(seed, B, T, Hq, Hkv, D, lens, max_pages)
    kp, vp = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    return p, kp, vp


def test_hand_example():
    g = read_golden("attention_hand_example.txt")
    kp = np.zeros((1, 1, 16, 1))
    vp = np.zeros((1, 1, 16, 1))
    kp[0, 0, :2, 0], vp[0, 0, :2, 0] = g["k"], g["v"]
    kp[0, 0, 2, 0], vp[0, 0, 2, 0] = g["k3"][0], g["v3"][0]
    q = g["q"].reshape(1, 1, 1, 1)
    table = np.zeros((1, 1), dtype=np.int32)
    assert om.attn_decode(q, kp, vp, table, [2])[0, 0, 0, 0] == pytest.approx(g["o"][0], abs=1e-14)
    assert om.attn_decode(q, kp, vp, table, [3], window=2)[0, 0, 0, 0] == pytest.approx(g["o_window2"][0], abs=1e-13)
    assert om.attn_decode(q, kp, vp, table, [3])[0, 0, 0, 0] == pytest.approx(g["o_full3"][0], abs=1e-13)


@pytest.mark.parametrize("window,T", [(0, 1), (9, 1), (0, 3), (9, 3)])
def test_matches_scalar_loops(window, T):
    p, kp, vp = small_problem(11, T=T)
    a = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], window, 0.35)
    b = om.attn_decode_loops(p["q"], kp, vp, p["page_table"], p["seq_lens"], window, 0.35)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_matches_scipy_softmax_on_contiguous_cache():
    p, kp, vp = small_problem(12)
    out = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 0.5)
    for b in range(2):
        L = int(p["seq_lens"][b])
        for h in range(4):
            K = om.widen(p["k_tok"][b, :L, h // 2])
            V = om.widen(p["v_tok"][b, :L, h // 2])
            w = softmax(0.5 * K @ om.widen(p["q"][b, 0, h]))
            np.testing.assert_allclose(out[b, 0, h], w @ V, atol=1e-14)


def test_window_at_least_context_is_full_attention():
    p, kp, vp = small_problem(13)
    full = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 0.4)
    for w in (37, 38, 4096):
        assert np.array_equal(om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], w, 0.4), full)


def test_window_equals_full_attention_on_truncated_cache():
    """SWA(W) over a long cache = FA over a cache that only ever held the last W tokens."""
    p, kp, vp = small_problem(14)
    W = 11
    swa = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], W, 0.4)
    for b in range(2):
        L = int(p["seq_lens"][b])
        lens1 = np.array([W], dtype=np.int32)
        k_tok = p["k_tok"][b:b + 1, L - W:L]
        v_tok = p["v_tok"][b:b + 1, L - W:L]
        table, n = gen.page_table(99, lens1, 1)
        kp1, vp1 = gen.logical_pools(k_tok, v_tok, table, lens1, n)
        fa = om.attn_decode(p["q"][b:b + 1], kp1, vp1, table, lens1, 0, 0.4)
        np.testing.assert_allclose(swa[b], fa[0], atol=1e-14)


def test_equal_keys_give_mean_value_and_single_token_gives_its_value():
    p, kp, vp = small_problem(15)
    kp[:] = kp[0, 0, 0, 0]
    out = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 7, 1.0)
    for b in range(2):
        L = int(p["seq_lens"][b])
        for h in range(4):
            np.testing.assert_allclose(out[b, 0, h], om.widen(p["v_tok"][b, L - 7:L, h // 2]).mean(0), atol=1e-14)
    p, kp, vp = small_problem(16, lens=(1, 1))
    out = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 1.0)
    for b in range(2):
        for h in range(4):
            assert np.array_equal(out[b, 0, h], om.widen(p["v_tok"][b, 0, h // 2]))


def test_physical_page_order_does_not_matter():
    p, kp, vp = small_problem(17)
    a = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 0.4)
    table2, n2 = gen.page_table(4242, p["seq_lens"], 4, n_spare_pages=9)
    kp2, vp2 = gen.logical_pools(p["k_tok"], p["v_tok"], table2, p["seq_lens"], n2)
    assert not np.array_equal(table2, p["page_table"])
    assert np.array_equal(om.attn_decode(p["q"], kp2, vp2, table2, p["seq_lens"], 0, 0.4), a)


def test_split_and_merge_identity():
    """Attention over [0,L) = merge of attention over [0,c) and [c,L) weighted by exp(logsumexp)."""
    p, kp, vp = small_problem(18, B=1, lens=(37,))
    full = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 0.4)
    c = 21
    left = om.attn_decode(p["q"], kp, vp, p["page_table"], [c], 0, 0.4)
    right = om.attn_decode(p["q"], kp, vp, p["page_table"], [37], 37 - c, 0.4)
    for h in range(4):
        K = om.widen(p["k_tok"][0, :37, h // 2])
        s = 0.4 * K @ om.widen(p["q"][0, 0, h])
        l1, l2 = logsumexp(s[:c]), logsumexp(s[c:])
        merged = (np.exp(l1) * left[0, 0, h] + np.exp(l2) * right[0, 0, h]) / (np.exp(l1) + np.exp(l2))
        np.testing.assert_allclose(merged, full[0, 0, h], atol=1e-13)


@pytest.mark.parametrize("window", [0, 9])
def test_multi_token_is_causal_single_token_calls(window):
    """T new tokens: token i behaves like a one-token call on the cache cut at its own position."""
    p, kp, vp = small_problem(19, T=4)
    out = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], window, 0.4)
    for i in range(4):
        one = om.attn_decode(p["q"][:, i:i + 1], kp, vp, p["page_table"], p["seq_lens"] - 3 + i, window, 0.4)
        assert np.array_equal(one[:, 0], out[:, i])


def test_empty_context_gives_zeros_and_unmapped_live_page_raises():
    p, kp, vp = small_problem(20, lens=(0, 5))
    out = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 1.0)
    assert not out[0].any() and out[1].any()
    bad = p["page_table"].copy()
    bad[1, 0] = -1
    with pytest.raises(ValueError):
        om.attn_decode(p["q"], kp, vp, bad, p["seq_lens"], 0, 1.0)


def test_bounded_window_cache_never_reads_outside_the_window():
    """Pages wholly before the window are unmapped (-1) and unwritten slots hold NaN: the result must
    still be finite and equal to the full-cache SWA result."""
    lens = np.array([61, 40], dtype=np.int32)
    W = 20
    p = gen.attention_inputs(21, 2, 1, 4, 2, 8, lens, 4)
    kp, vp = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    ref = om.attn_decode(p["q"], kp, vp, p["page_table"], lens, W, 0.4)
    tb, nb = gen.page_table(22, lens, 4, window_only=W)
    assert (tb[0, :2] == -1).all() and tb[0, 2] >= 0
    kpb, vpb = gen.logical_pools(p["k_tok"], p["v_tok"], tb, lens, nb)
    got = om.attn_decode(p["q"], kpb, vpb, tb, lens, W, 0.4)
    assert np.isfinite(got).all()
    assert np.array_equal(got, ref)


def test_rows_argument_selects_outputs():
    p, kp, vp = small_problem(23)
    full = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 0.4)
    some = om.attn_decode(p["q"], kp, vp, p["page_table"], p["seq_lens"], 0, 0.4, rows=[(1, 0, 3)])
    assert np.array_equal(some[1, 0, 3], full[1, 0, 3]) and not some[0].any()
