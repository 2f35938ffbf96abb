"""GPU parity of attn_decode / kv_append against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import kv_layout as kl
from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, Guarded, dev, host, rel_err

pytestmark = pytest.mark.gpu

HQ, HKV, D = 32, 8, 128
SCALE = D ** -0.5


def gpu_attention(q, kphys, vphys, table, lens, T, window, max_seq_len, req=None, n_pages=None, HQ=HQ, HKV=HKV):
    """kphys/vphys: device tensors or host uint16 arrays [n_pages,Hkv,2048]."""
    B = len(lens)
    kd = kphys if torch.is_tensor(kphys) else dev(kphys)
    vd = vphys if torch.is_tensor(vphys) else dev(vphys)
    n_pages = n_pages or kd.shape[0]
    n_req = B if req is None else len(req)
    ws_bytes = sa.attn_decode_workspace_bytes(n_req, T, HQ, HKV, D, max_seq_len, window)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    out = torch.full((B, T, HQ, D), 123.0, dtype=torch.float32, device="cuda")
    sa.attn_decode(dev(q), kd, vd, n_pages, dev(table), table.shape[1], dev(np.asarray(lens, dtype=np.int32)),
                   None if req is None else dev(np.asarray(req, dtype=np.int32)), n_req, out, B, T, HQ, HKV, D, 16,
                   max_seq_len, window, SCALE, ws, ws_bytes)
    torch.cuda.synchronize()
    return host(out)


def host_problem(seed, lens, T, max_pages, window_only=0):
    lens = np.asarray(lens, dtype=np.int32)
    p = gen.attention_inputs(seed, len(lens), T, HQ, HKV, D, lens, max_pages, window_only=window_only)
    klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])  # NaN in dead slots
    kphys, vphys = kl.to_physical(klog, vlog)
    return p, klog, vlog, kphys, vphys


@pytest.mark.parametrize("window", [0, 64, 100, 4096])
@pytest.mark.parametrize("T", [1, 4])
def test_ragged_lengths_against_oracle(window, T):
    """Lengths from a single token to several page ranges, page tails of every kind, dead slots full
    of NaN; full attention and windows that are shorter, unaligned and longer than the context."""
    lens = [T, 16, 17, 31, 100, 1000, 2047, 5000, 5013]
    p, klog, vlog, kphys, vphys = host_problem(3001 + T, lens, T, 320)
    got = gpu_attention(p["q"], kphys, vphys, p["page_table"], lens, T, window, 5120)
    ref = om.attn_decode(p["q"], klog, vlog, p["page_table"], p["seq_lens"], window, SCALE)
    assert np.isfinite(got).all()
    for b in range(len(lens)):
        assert rel_err(got[b], ref[b]) <= OUT_TOL, (b, lens[b])


def test_short_and_empty_contexts_and_request_list():
    """L = 0 and L < T give zeros for the tokens that do not exist yet; only listed rows are written."""
    T = 4
    lens = [0, 2, 4, 40, 300]
    p, klog, vlog, kphys, vphys = host_problem(3010, lens, T, 32)
    req = [4, 0, 1, 3]
    got = gpu_attention(p["q"], kphys, vphys, p["page_table"], lens, T, 0, 512, req=req)
    ref = om.attn_decode(p["q"], klog, vlog, p["page_table"], p["seq_lens"], 0, SCALE)
    assert not got[0].any()
    assert not got[1, :2].any() and got[1, 2:].any()
    assert (got[2] == 123.0).all()
    for b in (1, 3, 4):
        assert rel_err(got[b], ref[b]) <= OUT_TOL


def test_bounded_window_cache_with_unmapped_pages():
    """A sliding-window cache that only maps the pages the window touches (-1 elsewhere)."""
    lens, W, T = [5000, 4100, 333], 256, 1
    full, klog, vlog, kphys, vphys = host_problem(3020, lens, T, 320)
    ref = om.attn_decode(full["q"], klog, vlog, full["page_table"], full["seq_lens"], W, SCALE)
    tb, nb = gen.page_table(3021, np.asarray(lens, dtype=np.int32), 320, window_only=W)
    assert (tb[0, :290] == -1).all()
    klog_b, vlog_b = gen.logical_pools(full["k_tok"], full["v_tok"], tb, lens, nb)
    kp, vp = kl.to_physical(klog_b, vlog_b)
    got = gpu_attention(full["q"], kp, vp, tb, lens, T, W, 5120)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= OUT_TOL


def test_runs_are_bit_reproducible_and_a_window_covering_the_context_equals_full_attention():
    lens = [777, 3000]
    p, klog, vlog, kphys, vphys = host_problem(3030, lens, 1, 192)
    a = gpu_attention(p["q"], kphys, vphys, p["page_table"], lens, 1, 0, 3072)
    b = gpu_attention(p["q"], kphys, vphys, p["page_table"], lens, 1, 0, 3072)
    assert np.array_equal(a, b)
    c = gpu_attention(p["q"], kphys, vphys, p["page_table"], lens, 1, 3000, 3072)
    assert rel_err(c, a) <= 1e-5


def test_kv_append_is_bit_exact_and_respects_bounds():
    """Appending through the library gives the byte layout the header states: compared with the
    index-formula reference after appends of T = 1 and T = 5 that cross page boundaries."""
    B, max_pages = 3, 6
    lens = np.array([40, 60, 77], dtype=np.int32)
    table, n_pages = gen.page_table(3041, np.array([96, 96, 96], dtype=np.int32), max_pages)
    table[1, 4] = -1                                  # an unmapped page: tokens landing there are skipped
    rng = np.random.default_rng(3040)
    kp = rng.integers(0, 2 ** 16, (n_pages, HKV, 16 * D), dtype=np.uint16)
    vp = rng.integers(0, 2 ** 16, (n_pages, HKV, 16 * D), dtype=np.uint16)
    kg, vg = Guarded(kp), Guarded(vp)
    k_ref, v_ref = kp.copy(), vp.copy()
    pos = lens.copy()
    for T in (1, 5, 1, 16):
        k_new = rng.integers(0, 2 ** 16, (B, T, HKV, D), dtype=np.uint16)
        v_new = rng.integers(0, 2 ** 16, (B, T, HKV, D), dtype=np.uint16)
        sa.kv_append(dev(k_new), dev(v_new), kg.ptr(), vg.ptr(), n_pages, dev(table), max_pages, dev(pos), B, T, HKV, D, 16)
        torch.cuda.synchronize()
        for b in range(B):
            for i in range(T):
                pg = (pos[b] + i) // 16
                if pg >= max_pages or table[b, pg] < 0:
                    continue
                kl.kv_append(k_new[b:b + 1, i:i + 1], v_new[b:b + 1, i:i + 1], k_ref, v_ref, table[b:b + 1], [pos[b] + i])
        pos += T
    assert np.array_equal(kg.read(), k_ref) and np.array_equal(vg.read(), v_ref)
    assert kg.bands_intact() and vg.bands_intact()


def test_append_then_attend_round_trip():
    """Decode loop: append one token, attend, repeat; every step equals the oracle on the grown cache."""
    B, max_pages, n_steps = 2, 8, 6
    lens = np.array([30, 45], dtype=np.int32)
    p = gen.attention_inputs(3050, B, 1, HQ, HKV, D, lens + n_steps, max_pages)
    klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    kd, vd = (dev(a) for a in kl.to_physical(klog, vlog))
    for step in range(n_steps):
        cur = lens + step
        k_new = np.stack([p["k_tok"][b, cur[b]] for b in range(B)])[:, None]
        v_new = np.stack([p["v_tok"][b, cur[b]] for b in range(B)])[:, None]
        sa.kv_append(dev(k_new), dev(v_new), kd, vd, p["n_pages"], dev(p["page_table"]), max_pages, dev(cur), B, 1, HKV, D, 16)
        got = gpu_attention(p["q"], kd, vd, p["page_table"], cur + 1, 1, 0, max_pages * 16)
        klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], cur + 1, p["n_pages"])
        ref = om.attn_decode(p["q"], klog, vlog, p["page_table"], cur + 1, 0, SCALE)
        assert rel_err(got, ref) <= OUT_TOL


@pytest.mark.parametrize("hq,hkv,T", [(8, 8, 1), (8, 8, 8), (16, 8, 2), (24, 8, 3), (32, 4, 2), (16, 1, 1), (5, 5, 3),
                                       (32, 8, 8), (32, 8, 5), (16, 8, 12), (16, 1, 2)])
def test_other_head_groupings_and_token_counts(hq, hkv, T):
    """Group sizes 1..16 and 1..8 new tokens (up to 32 query rows per KV head: one or two MFMA tiles), windowed and full."""
    lens = np.array([T + 3, 70, 555, 1300], dtype=np.int32)
    p = gen.attention_inputs(3060 + hq + T, len(lens), T, hq, hkv, D, lens, 96)
    klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    kphys, vphys = kl.to_physical(klog, vlog)
    for window in (0, 200):
        got = gpu_attention(p["q"], kphys, vphys, p["page_table"], lens, T, window, 1536, HQ=hq, HKV=hkv)
        ref = om.attn_decode(p["q"], klog, vlog, p["page_table"], lens, window, SCALE)
        assert rel_err(got, ref) <= OUT_TOL, window


def _device_pools(seed, n_pages):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    kp = torch.empty((n_pages, HKV, 16 * D), dtype=torch.bfloat16, device="cuda")
    vp = torch.empty((n_pages, HKV, 16 * D), dtype=torch.bfloat16, device="cuda")
    kp.normal_(generator=g)
    vp.normal_(generator=g)
    return kp, vp


def _per_row_rel_err(got, ref):
    """gpu_util.rel_err for every (sequence, token, head) output row at once: [B,T,Hq]."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    return np.max(np.abs(got - ref) / (np.abs(ref) + rms + (rms == 0)), axis=-1)


def _check_every_row(got, q, kp, vp, table, lens, window, T, groups):
    """Every output row against the oracle's fp64 C form (plain loops over the pools copied to the host in the library's
    in-page order; admitted at 1e-12 from the numpy oracle by tests/test_oracle_omp.py), and the (sequence, KV head) groups
    listed in `groups`, two query heads each, against the numpy oracle itself, which the C form must match there too."""
    from oracle import omp
    kph = kp.view(torch.int16).cpu().numpy().view(np.uint16)
    vph = vp.view(torch.int16).cpu().numpy().view(np.uint16)
    ref_all = omp.attn_decode(q, kph, vph, table, lens, window, SCALE, physical=True)
    err = _per_row_rel_err(got, ref_all)
    assert err.max() <= OUT_TOL, (np.unravel_index(err.argmax(), err.shape), err.max())
    G = HQ // HKV
    for n, (b, g) in enumerate(groups):
        L = int(lens[b])
        pages = table[b, :(L + 15) // 16]
        klog, vlog = kl.to_logical(kph[pages, g][:, None], vph[pages, g][:, None], D)
        ident = np.arange(len(pages), dtype=np.int32)[None]
        heads = [g * G + n % G, g * G + (n % G + 1 + (n // G) % (G - 1)) % G]     # two different heads of the group
        ref = om.attn_decode(q[b:b + 1][:, :, heads], klog, vlog, ident, [L], window, SCALE)     # both heads sit on this KV head
        for i, h in enumerate(heads):
            assert rel_err(got[b, :, h], ref[0, :, i]) <= OUT_TOL, (b, h, L)
            assert np.max(np.abs(ref_all[b, :, h] - ref[0, :, i])) <= 1e-12, (b, h, L)


@pytest.fixture(scope="module")
def batch64_cache():
    """Batch 64, 32768-token caches (8 GiB of K+V, N(0,1) bf16 drawn on the device), shuffled page table."""
    B, max_len = 64, 32768
    table, n_pages = gen.page_table(4005, np.full(B, max_len, dtype=np.int32), max_len // 16)
    kp, vp = _device_pools(4006, n_pages)
    yield table, n_pages, kp, vp
    del kp, vp
    torch.cuda.empty_cache()


@pytest.mark.parametrize("mode", ["fa_32k", "swa_4096", "fa_ragged"])
def test_full_size_batch64_every_row(mode, batch64_cache):
    """BASELINE config 4: batch 64, 32 query / 8 KV heads, 32768-token caches, in the launch configuration the benchmark
    times.  All 2048 (sequence, head) rows are checked against the C form of the oracle and 128 of them (every sequence
    once, every KV head 8 times, two heads of the group) against the numpy oracle."""
    B, max_len = 64, 32768
    table, n_pages, kp, vp = batch64_cache
    if mode == "fa_32k":
        lens = np.full(B, max_len, dtype=np.int32)
        window = 0
    else:
        lens = gen.context_lengths(4004, B, 8192, max_len)
        window = 4096 if mode == "swa_4096" else 0
    q = gen.attention_inputs(4007, B, 1, HQ, HKV, D, np.ones(B, dtype=np.int32), 1)["q"]
    got = gpu_attention(q, kp, vp, table, lens, 1, window, max_len, n_pages=n_pages)
    assert np.isfinite(got).all()
    _check_every_row(got, q, kp, vp, table, lens, window, 1, [(b, (b + b // HKV) % HKV) for b in range(B)])


def test_verify_four_tokens_full_size_every_row():
    """4-token verify step (16 query rows per KV head) on long contexts, FA and SWA."""
    B, max_len, T = 16, 16384, 4
    max_pages = max_len // 16
    lens = gen.context_lengths(4014, B, 4096, max_len)
    table, n_pages = gen.page_table(4015, np.full(B, max_len, dtype=np.int32), max_pages)
    kp, vp = _device_pools(4016, n_pages)
    q = gen.attention_inputs(4017, B, T, HQ, HKV, D, np.ones(B, dtype=np.int32), 1)["q"]
    for window in (0, 4096):
        got = gpu_attention(q, kp, vp, table, lens, T, window, max_len, n_pages=n_pages)
        assert np.isfinite(got).all()
        _check_every_row(got, q, kp, vp, table, lens, window, T, [(0, 0), (3, 4), (15, 7), (7, 2)])


@pytest.mark.parametrize("window", [0, 300])
def test_regular_page_tables_and_many_ranges(window):
    """Pages of a sequence in a row, sequences at a fixed distance (a freshly filled cache) and, second, pages
    interleaved over the sequences (caches that grew together): every workgroup visits its range from its own
    starting point, so the result must not depend on how regular the table is."""
    B, T, max_len = 5, 2, 3000
    max_pages = (max_len + 15) // 16
    lens = np.array([3000, 2999, 1, 1717, 48], dtype=np.int32)
    p = gen.attention_inputs(4100, B, T, HQ, HKV, D, lens, max_pages)
    for kind in ("rows", "interleaved"):
        if kind == "rows":
            table = np.arange(B * max_pages, dtype=np.int32).reshape(B, max_pages)
        else:
            table = (np.arange(max_pages, dtype=np.int32)[None, :] * B + np.arange(B, dtype=np.int32)[:, None])
        n_pages = B * max_pages
        klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], table, lens, n_pages)
        kphys, vphys = kl.to_physical(klog, vlog)
        got = gpu_attention(p["q"], dev(kphys), dev(vphys), table, lens, T, window, max_len, n_pages=n_pages)
        ref = om.attn_decode(p["q"], klog, vlog, table, lens, window, D ** -0.5)
        for b in range(B):
            assert rel_err(got[b], ref[b]) <= OUT_TOL, (kind, b)
