"""End to end on the GPU: one arena managed by the unified page pool serves the KV caches of FA and SWA
layers and the states of KDA and GDN layers of three sequences on different placements; a few decode
steps (reserve -> tables -> kv_append -> placement_decode) are checked against the oracle."""
import numpy as np
import pytest
import torch

from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, STATE_TOL, dev, rel_err

pytestmark = pytest.mark.gpu

H, DK, DV, HQ, HKV, D = 32, 128, 128, 32, 8, 128


def test_decode_loop_on_a_pooled_arena():
    placements = ["FSKG", "GKSF", "SFFK"]
    L, B, window, max_pages, n_unified = 4, 3, 256, 96, 24
    lens = np.array([600, 1100, 50], dtype=np.int32)
    n_steps = 3
    shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
    pool = sa.sa_pool_create(n_unified, shapes, L)
    page_bytes = sa.sa_pool_page_bytes(pool)
    stride = sa.sa_pool_kv_id_stride(pool)
    arena = torch.zeros((n_unified, page_bytes), dtype=torch.uint8, device="cuda")
    arena[:] = 0xFF                                              # NaN patterns everywhere until written
    kpool_ptr, vpool_ptr = arena.data_ptr(), arena.data_ptr() + page_bytes // 2
    state_view = arena.view(torch.float32).view(n_unified, H, DK, DV)
    seqs = [sa.sa_pool_seq_create(pool, p) for p in placements]
    pid = np.arange(B, dtype=np.int32)
    plan = sa.placement_plan_create(placements, pid)

    # token history per layer (attention layers) and fp64 reference states (recurrent layers)
    total = lens + n_steps
    hist = [gen.attention_inputs(9000 + l, B, 1, HQ, HKV, D, total, max_pages) for l in range(L)]
    ref_state = {}
    for l in range(L):
        _, slot = sa.sa_pool_layer_tables(pool, seqs, l, 0)
        for b in range(B):
            if slot[b] >= 0:
                state_view[slot[b]].zero_()                      # a new sequence starts from the zero state
                ref_state[(l, b)] = np.zeros((1, H, DK, DV))

    # prefill: make the context addressable, then append it layer by layer, sequence by sequence
    for b in range(B):
        sa.sa_pool_seq_reserve(pool, seqs[b], int(lens[b]), window)
    for l in range(L):
        table, _ = sa.sa_pool_layer_tables(pool, seqs, l, max_pages)
        for b in range(B):
            n = int(lens[b])
            sa.kv_append(dev(hist[l]["k_tok"][b:b + 1, :n]), dev(hist[l]["v_tok"][b:b + 1, :n]), kpool_ptr, vpool_ptr,
                         sa.sa_pool_kernel_pages(pool), dev(table[b:b + 1]), max_pages, dev(np.zeros(1, dtype=np.int32)), 1, n, HKV, D, 16)
    torch.cuda.synchronize()
    free_after_prefill = sa.sa_pool_free_pages(pool)
    # FSKG@600: F 2 + S 2(blocks 0..1 both touch [344,600)) + 2 states; GKSF@1100: 2 + S 2 + F 3; SFFK@50: 1+1+1+1
    assert n_unified - free_after_prefill == (2 + 2 + 2) + (2 + 2 + 3) + 4

    ws_bytes = sa.placement_workspace_bytes(plan, shapes, 1, max_pages * 16, window)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    for step in range(n_steps):
        cur = lens + step                                        # position of the new token
        for b in range(B):
            sa.sa_pool_seq_reserve(pool, seqs[b], int(cur[b]) + 1, window)
        keep, ios, rec_ops = [], [], []
        for l in range(L):
            table, slot = sa.sa_pool_layer_tables(pool, seqs, l, max_pages)
            t_table, t_slot, t_len = dev(table), dev(np.maximum(slot, 0)), dev(cur + 1)
            k_new = np.stack([hist[l]["k_tok"][b, cur[b]] for b in range(B)])[:, None]
            v_new = np.stack([hist[l]["v_tok"][b, cur[b]] for b in range(B)])[:, None]
            sa.kv_append(dev(k_new), dev(v_new), kpool_ptr, vpool_ptr, sa.sa_pool_kernel_pages(pool), t_table, max_pages, dev(cur), B, 1,
                         HKV, D, 16)
            r = gen.recurrent_inputs(9100 + 10 * step + l, B, 1, H, H, DK, DV, False)
            rv = gen.recurrent_inputs(9200 + 10 * step + l, B, 1, H, H, DK, DV, True)
            qa = gen.attention_inputs(9300 + 10 * step + l, B, 1, HQ, HKV, D, np.ones(B, dtype=np.int32), 1)["q"]
            t = {n: dev(a) for n, a in (("q", r["q"]), ("k", r["k"]), ("v", r["v"]), ("a_s", r["alpha"]), ("a_v", rv["alpha"]),
                                        ("beta", r["beta"]), ("qa", qa))}
            t["out"] = torch.zeros((B, 1, H, DV), dtype=torch.float32, device="cuda")
            t.update(table=t_table, slot=t_slot, len=t_len)
            keep.append(t)
            rec_ops.append((r, rv, qa, slot))
            ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["a_s"], alpha_vec=t["a_v"], beta=t["beta"],
                                        state=arena.data_ptr(), slot_idx=t_slot, q_attn=t["qa"], kpool=kpool_ptr, vpool=vpool_ptr,
                                        n_pages=sa.sa_pool_kernel_pages(pool), page_table=t_table, seq_lens=t_len, max_pages=max_pages,
                                        max_seq_len=max_pages * 16, out=t["out"]))
        sa.placement_decode(plan, ios, shapes, 1, window, D ** -0.5, DK ** -0.5, ws, ws_bytes)
        torch.cuda.synchronize()
        for l in range(L):
            r, rv, qa, slot = rec_ops[l]
            got = keep[l]["out"].cpu().numpy()
            assert np.isfinite(got).all()
            for b in range(B):
                m = placements[b][l]
                if m in "FS":
                    n = int(cur[b]) + 1
                    ident = np.arange(max_pages, dtype=np.int32)[None]
                    klog, vlog = gen.logical_pools(hist[l]["k_tok"][b:b + 1], hist[l]["v_tok"][b:b + 1], ident, [n], max_pages)
                    ref = om.attn_decode(qa[b:b + 1], klog, vlog, ident, [n], window if m == "S" else 0, D ** -0.5)
                    assert rel_err(got[b], ref[0]) <= OUT_TOL, (step, l, b, m)
                else:
                    fn, a = (om.kda_steps, rv["alpha"]) if m == "K" else (om.gdn_steps, r["alpha"])
                    o, s = fn(r["q"][b:b + 1], r["k"][b:b + 1], r["v"][b:b + 1], a[b:b + 1], r["beta"][b:b + 1],
                              ref_state[(l, b)], DK ** -0.5)
                    ref_state[(l, b)] = s
                    assert rel_err(got[b], o[0]) <= OUT_TOL, (step, l, b, m)
                    assert rel_err(state_view[slot[b]].cpu().numpy(), s[0]) <= STATE_TOL, (step, l, b, m)
    for s in seqs:
        sa.sa_pool_seq_free(pool, s)
    assert sa.sa_pool_free_pages(pool) == n_unified
    sa.placement_plan_destroy(plan)
    sa.sa_pool_destroy(pool)
