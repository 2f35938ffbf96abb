"""attn_decode_static (the entry point for callers that cannot allocate: its partial results live in a device array inside
the library) against attn_decode with a caller workspace, through the C ABI: same kernels, same split plan, so the
outputs must agree bit for bit; and both against the oracle.  Two calls in a row share the array, the second smaller."""
import numpy as np
import pytest
import torch

from oracle import kv_layout as kl
from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, dev, host, rel_err

pytestmark = pytest.mark.gpu

HQ, HKV, D = 32, 8, 128
SCALE = D ** -0.5


def problem(seed, lens, T, max_pages):
    lens = np.asarray(lens, dtype=np.int32)
    p = gen.attention_inputs(seed, len(lens), T, HQ, HKV, D, lens, max_pages)
    klog, vlog = gen.logical_pools(p["k_tok"], p["v_tok"], p["page_table"], lens, p["n_pages"])
    kphys, vphys = kl.to_physical(klog, vlog)
    return p, klog, vlog, dev(kphys), dev(vphys)


def both(p, kd, vd, lens, T, window, max_seq_len):
    """(output of attn_decode_static, output of attn_decode with a workspace, workspace bytes)."""
    B = len(lens)
    q, table, ln = dev(p["q"]), dev(p["page_table"]), dev(np.asarray(lens, dtype=np.int32))
    mp = p["page_table"].shape[1]
    outs = []
    ws_bytes = sa.attn_decode_workspace_bytes(B, T, HQ, HKV, D, max_seq_len, window)
    for static in (True, False):
        out = torch.full((B, T, HQ, D), 321.0, dtype=torch.float32, device="cuda")
        if static:
            sa.attn_decode_static(q, kd, vd, kd.shape[0], table, mp, ln, None, 0, out, B, T, HQ, HKV, D, 16, max_seq_len, window, SCALE)
        else:
            ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
            sa.attn_decode(q, kd, vd, kd.shape[0], table, mp, ln, None, 0, out, B, T, HQ, HKV, D, 16, max_seq_len, window, SCALE, ws, ws_bytes)
        torch.cuda.synchronize()
        outs.append(host(out))
    return outs[0], outs[1], ws_bytes


def test_two_calls_in_a_row_the_second_smaller():
    assert sa.attn_decode_static_max_bytes() == 16 << 20
    cases = [([5000, 4999, 2047, 100, 16, 3000], 4, 0, 5120, 4001),      # several page ranges per (request, KV head), 16 query rows
             ([1500, 700, 3], 1, 0, 2048, 4002),                         # smaller: fewer rows, fewer and shorter ranges
             ([5000, 4100, 333], 1, 256, 5120, 4003)]                    # a window: one range, no partial results at all
    for lens, T, window, max_seq_len, seed in cases:
        p, klog, vlog, kd, vd = problem(seed, lens, T, max_seq_len // 16)
        got_static, got_ws, ws_bytes = both(p, kd, vd, lens, T, window, max_seq_len)
        assert (ws_bytes > 0) == (window == 0)
        assert np.isfinite(got_static).all()
        assert np.array_equal(got_static, got_ws), (lens, T, window)
        ref = om.attn_decode(p["q"], klog, vlog, p["page_table"], p["seq_lens"], window, SCALE)
        for b in range(len(lens)):
            assert rel_err(got_static[b], ref[b]) <= OUT_TOL, (b, lens[b])


def test_sizes_beyond_the_array_are_refused_before_anything_runs():
    # 512 requests of up to 32768 tokens would need ~65 MiB of partial results
    B, max_seq_len = 512, 32768
    assert sa.attn_decode_workspace_bytes(B, 1, HQ, HKV, D, max_seq_len, 0) > sa.attn_decode_static_max_bytes()
    small = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    out = torch.full((B, 1, HQ, D), 7.0, dtype=torch.float32, device="cuda")
    q = torch.zeros((B, 1, HQ, D), dtype=torch.int16, device="cuda")
    table = torch.zeros((B, max_seq_len // 16), dtype=torch.int32, device="cuda")
    lens = torch.zeros(B, dtype=torch.int32, device="cuda")
    with pytest.raises(sa.SaError) as e:
        sa.attn_decode_static(q, small, small, 1, table, max_seq_len // 16, lens, None, 0, out, B, 1, HQ, HKV, D, 16, max_seq_len, 0, SCALE)
    assert e.value.status == sa.SA_EWORKSPACE and "attn_decode_static" in str(e.value)
    torch.cuda.synchronize()
    assert (out == 7.0).all()
    # the ordinary argument checks still apply
    with pytest.raises(sa.SaError) as e:
        sa.attn_decode_static(q, small, small, 1, table, max_seq_len // 16, lens, None, 0, out, B, 1, HQ, HKV, 64, 16, max_seq_len, 0, SCALE)
    assert e.value.status == sa.SA_EUNSUPPORTED
