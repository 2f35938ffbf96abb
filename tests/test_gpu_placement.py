"""GPU parity of placement_decode against the oracle: a 48-layer mixers-only stack, three seeded
placements of 12 FA / 12 SWA / 12 KDA / 12 GDN layers, a different placement per request."""
import numpy as np
import pytest
import torch

from oracle import kv_layout as kl
from oracle import mixers as om
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import OUT_TOL, STATE_TOL, dev, host, rel_err

pytestmark = pytest.mark.gpu

H, DK, DV, HQ, HKV, D = 32, 128, 128, 32, 8, 128


def build_stack(seed, L, B, T, ctx, max_pages, lens=None):
    """Host-side operands of every layer for the whole batch (each layer has its own)."""
    lens = np.full(B, ctx, dtype=np.int32) if lens is None else np.asarray(lens, dtype=np.int32)
    layers = []
    for l in range(L):
        r = gen.recurrent_inputs(seed + 10 * l, B, T, H, H, DK, DV, False)
        rv = gen.recurrent_inputs(seed + 10 * l + 1, B, T, H, H, DK, DV, True)
        a = gen.attention_inputs(seed + 10 * l + 2, B, T, HQ, HKV, D, lens, max_pages)
        klog, vlog = gen.logical_pools(a["k_tok"], a["v_tok"], a["page_table"], lens, a["n_pages"])
        state = gen.recurrent_state(seed + 10 * l + 3, B * H, DK, DV).reshape(B, H, DK, DV)
        layers.append({"q": r["q"], "k": r["k"], "v": r["v"], "alpha_scalar": r["alpha"], "alpha_vec": rv["alpha"],
                       "beta": r["beta"], "state": state, "qa": a["q"], "kpool": klog, "vpool": vlog,
                       "page_table": a["page_table"], "seq_lens": lens, "n_pages": a["n_pages"]})
    return layers


@pytest.mark.parametrize("T", [1, 4])
def test_48_layer_stack_three_placements(T):
    L, B, ctx, window, max_pages = 48, 6, 1024, 256, 64
    placements = [gen.placement_string(5001 + i, L) for i in range(3)]
    pid = np.arange(B, dtype=np.int32) % 3
    layers = build_stack(5100 + T, L, B, T, ctx, max_pages)
    attn_scale, rec_scale = D ** -0.5, DK ** -0.5

    plan = sa.placement_plan_create(placements, pid)
    try:
        for l in range(L):
            counts = {m: sa.placement_plan_count(plan, l, m) for m in "FSKG"}
            assert sum(counts.values()) == B
            for m in "FSKG":
                assert counts[m] == sum(placements[p][l] == m for p in pid)
        shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
        ws_bytes = sa.placement_workspace_bytes(plan, shapes, T, ctx, window)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        keep, ios, outs, states = [], [], [], []
        for io in layers:
            kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
            t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
            t["state"] = dev(io["state"].copy())
            t["kpool"], t["vpool"] = dev(kphys), dev(vphys)
            t["out"] = torch.full((B, T, H, DV), 55.0, dtype=torch.float32, device="cuda")
            keep.append(t)
            outs.append(t["out"])
            states.append(t["state"])
            ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                                        beta=t["beta"], state=t["state"], slot_idx=None, q_attn=t["qa"], kpool=t["kpool"],
                                        vpool=t["vpool"], n_pages=io["n_pages"], page_table=t["page_table"],
                                        seq_lens=t["seq_lens"], max_pages=max_pages, max_seq_len=ctx, out=t["out"]))
        sa.placement_decode(plan, ios, shapes, T, window, attn_scale, rec_scale, ws, ws_bytes)
        torch.cuda.synchronize()
    finally:
        sa.placement_plan_destroy(plan)

    ref_outs, ref_states = om.placement_decode(placements, pid, layers, window, attn_scale, rec_scale)
    for l in range(L):
        got_o, got_s = host(outs[l]), host(states[l])
        assert np.isfinite(got_o).all()
        for r in range(B):
            m = placements[pid[r]][l]
            assert rel_err(got_o[r], ref_outs[l][r]) <= OUT_TOL, (l, r, m)
            if m in "KG":
                assert rel_err(got_s[r], ref_states[l][r]) <= STATE_TOL, (l, r, m)
            else:
                assert np.array_equal(got_s[r], layers[l]["state"][r]), (l, r, m)   # attention rows leave the state alone


def test_all_four_mixers_in_every_layer_ragged_and_empty_contexts():
    """Four placements rotated against each other: every layer runs all four mixers in one fused launch, over
    contexts of very different lengths (one empty, one of a single token, one ending mid-page)."""
    L, B, ctx, window, max_pages = 8, 9, 1500, 200, 96
    placements = ["FSKGFSKG", "SKGFSKGF", "KGFSKGFS", "GFSKGFSK"]
    pid = np.array([0, 1, 2, 3, 3, 2, 1, 0, 2], dtype=np.int32)
    lens = [1500, 0, 1, 777, 16, 1203, 15, 450, 1499]
    layers = build_stack(5300, L, B, 1, ctx, max_pages, lens)
    plan = sa.placement_plan_create(placements, pid)
    shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
    ws_bytes = sa.placement_workspace_bytes(plan, shapes, 1, ctx, window)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    keep, ios = [], []
    for io in layers:
        kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
        t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
        t["state"], t["kpool"], t["vpool"] = dev(io["state"].copy()), dev(kphys), dev(vphys)
        t["out"] = torch.full((B, 1, H, DV), 55.0, dtype=torch.float32, device="cuda")
        keep.append(t)
        ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                                    beta=t["beta"], state=t["state"], q_attn=t["qa"], kpool=t["kpool"], vpool=t["vpool"],
                                    n_pages=io["n_pages"], page_table=t["page_table"], seq_lens=t["seq_lens"],
                                    max_pages=max_pages, max_seq_len=ctx, out=t["out"]))
    for l in range(L):
        assert all(sa.placement_plan_count(plan, l, m) >= 2 for m in "FSKG")
    sa.placement_decode(plan, ios, shapes, 1, window, D ** -0.5, DK ** -0.5, ws, ws_bytes)
    torch.cuda.synchronize()
    sa.placement_plan_destroy(plan)
    ref_outs, ref_states = om.placement_decode(placements, pid, layers, window, D ** -0.5, DK ** -0.5)
    for l in range(L):
        got_o, got_s = host(keep[l]["out"]), host(keep[l]["state"])
        for r in range(B):
            m = placements[pid[r]][l]
            if m in "FS" and lens[r] == 0:
                assert not got_o[r].any(), (l, r)          # an empty context reads nothing and returns zeros
                continue
            assert rel_err(got_o[r], ref_outs[l][r]) <= OUT_TOL, (l, r, m)
            if m in "KG":
                assert rel_err(got_s[r], ref_states[l][r]) <= STATE_TOL, (l, r, m)
            else:
                assert np.array_equal(got_s[r], layers[l]["state"][r]), (l, r, m)


def run_stack(placements, pid, layers, T, window, ctx, max_pages, slot=None, n_slots=None, n_commit_rows=None):
    """One placement_decode step over host-side layers; returns the outputs and states as numpy arrays."""
    B = len(pid)
    plan = sa.placement_plan_create(placements, pid)
    try:
        shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
        ws_bytes = sa.placement_workspace_bytes(plan, shapes, T, ctx, window)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        keep, ios = [], []
        for io in layers:
            kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
            t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
            state = io["state"].copy()
            if slot is not None:                      # states live in a larger slot array, addressed through slot_idx
                pool = np.full((n_slots,) + state.shape[1:], 9.0, dtype=np.float32)
                pool[slot] = state
                state = pool
            t["state"], t["kpool"], t["vpool"] = dev(state), dev(kphys), dev(vphys)
            t["slot"] = dev(slot) if slot is not None else None
            t["commit"] = dev(n_commit_rows) if n_commit_rows is not None else None
            t["out"] = torch.full((B, T, H, DV), 55.0, dtype=torch.float32, device="cuda")
            keep.append(t)
            ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                                        beta=t["beta"], state=t["state"], slot_idx=t["slot"], q_attn=t["qa"], kpool=t["kpool"],
                                        vpool=t["vpool"], n_pages=io["n_pages"], page_table=t["page_table"],
                                        seq_lens=t["seq_lens"], max_pages=max_pages, max_seq_len=ctx, out=t["out"],
                                        n_commit_rows=t["commit"]))
        sa.placement_decode(plan, ios, shapes, T, window, D ** -0.5, DK ** -0.5, ws, ws_bytes)
        torch.cuda.synchronize()
    finally:
        sa.placement_plan_destroy(plan)
    return [host(t["out"]) for t in keep], [host(t["state"]) for t in keep]


@pytest.mark.parametrize("T", [1, 4, 8])
def test_verify_pass_then_commit_of_accepted_prefixes(T):
    """Self-speculative decoding over a stack: a verify pass scores T drafted tokens per request and leaves every
    recurrent state alone (all counts zero); the second pass commits each request's own accepted prefix."""
    L, B, ctx, window, max_pages = 6, 5, 300, 64, 20
    placements = ["FKGSKG", "GGKFSK", "KSFGGF"]
    pid = np.array([0, 1, 2, 0, 1], dtype=np.int32)
    layers = build_stack(5400 + T, L, B, T, ctx, max_pages)
    ref_outs, _ = om.placement_decode(placements, pid, layers, window, D ** -0.5, DK ** -0.5)
    accepted = np.array([T, 0, T // 2, 1, max(T - 1, 0)], dtype=np.int32)
    for counts in (np.zeros(B, dtype=np.int32), accepted):
        outs, states = run_stack(placements, pid, layers, T, window, ctx, max_pages, n_commit_rows=counts)
        for l in range(L):
            for r in range(B):
                m = placements[pid[r]][l]
                assert rel_err(outs[l][r], ref_outs[l][r]) <= OUT_TOL, (l, r, m)       # all T read-outs either way
                if m in "KG" and counts[r] > 0:
                    fn = om.kda_steps if m == "K" else om.gdn_steps
                    io, sl = layers[l], slice(r, r + 1)
                    a = io["alpha_vec"] if m == "K" else io["alpha_scalar"]
                    _, s_ref = fn(io["q"][sl], io["k"][sl], io["v"][sl], a[sl], io["beta"][sl], io["state"][sl], DK ** -0.5,
                                  n_commit=int(counts[r]))
                    assert rel_err(states[l][r], s_ref[0]) <= STATE_TOL, (l, r, m, int(counts[r]))
                else:
                    assert np.array_equal(states[l][r], layers[l]["state"][r]), (l, r, m)


@pytest.mark.parametrize("placements", [
    ["FKF", "SGS"],            # fused (FA + SWA) -> fused recurrent-only layer, which merges layer 0 -> fused, last layer
    ["FFKF", "KFGF", "SFKF"],  # fused -> a single-mixer layer (stand-alone launches) -> recurrent-only -> single mixer
    ["FF", "SF", "KF"],        # fused -> single mixer
    ["FFFF", "SSSS"],          # four fused layers in a row with both attention kinds: the workspace halves alternate
])
def test_partial_results_merged_by_the_next_layers_launch(placements):
    """A fused layer leaves the merge of its attention ranges to the launch of the layer after it, whatever that
    layer runs; the window is long enough for the sliding-window calls to split into ranges as well."""
    L, B, ctx, window, max_pages = len(placements[0]), 7, 2100, 1100, 136
    pid = (np.arange(B) % len(placements)).astype(np.int32)
    lens = [2100, 1, 333, 2099, 1200, 16, 1999]
    layers = build_stack(5600 + L, L, B, 1, ctx, max_pages, lens)
    outs, states = run_stack(placements, pid, layers, 1, window, ctx, max_pages)
    ref_outs, ref_states = om.placement_decode(placements, pid, layers, window, D ** -0.5, DK ** -0.5)
    for l in range(L):
        for r in range(B):
            m = placements[pid[r]][l]
            assert rel_err(outs[l][r], ref_outs[l][r]) <= OUT_TOL, (l, r, m)
            if m in "KG":
                assert rel_err(states[l][r], ref_states[l][r]) <= STATE_TOL, (l, r, m)
            else:
                assert np.array_equal(states[l][r], layers[l]["state"][r]), (l, r, m)


@pytest.mark.parametrize("T", [1, 4])
def test_fused_layers_against_the_stand_alone_entry_points(T):
    """The fused per-layer launches run the bodies of the stand-alone kernels over the same request lists and page
    ranges: attention rows must come out bit for bit as from attn_decode; a recurrent tile sums its rows in an order
    that depends on where its workgroup sits in the grid, so those rows agree to rounding only."""
    L, B, ctx, window, max_pages = 3, 7, 2100, 1100, 136
    placements = ["FKS", "SGF", "KFG", "GSK"]
    pid = (np.arange(B) % 4).astype(np.int32)
    lens = [2100, T, 333, 2099, 1200, 16, 1999]
    layers = build_stack(5700 + T, L, B, T, ctx, max_pages, lens)
    outs, states = run_stack(placements, pid, layers, T, window, ctx, max_pages)
    for l, io in enumerate(layers):
        kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
        t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
        kd, vd = dev(kphys), dev(vphys)
        state = dev(io["state"].copy())
        out = torch.full((B, T, H, DV), 55.0, dtype=torch.float32, device="cuda")
        for m in "FSKG":
            req = np.array([r for r in range(B) if placements[pid[r]][l] == m], dtype=np.int32)
            if len(req) == 0:
                continue
            if m in "FS":
                w = 0 if m == "F" else window
                ws_bytes = sa.attn_decode_workspace_bytes(len(req), T, HQ, HKV, D, ctx, w)
                ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
                sa.attn_decode(t["qa"], kd, vd, io["n_pages"], t["page_table"], max_pages, t["seq_lens"], dev(req), len(req), out,
                               B, T, HQ, HKV, D, 16, ctx, w, D ** -0.5, ws, ws_bytes)
            else:
                fn = sa.kda_decode_step if m == "K" else sa.gdn_decode_step
                alpha = t["alpha_vec"] if m == "K" else t["alpha_scalar"]
                fn(t["q"], t["k"], t["v"], alpha, t["beta"], state, state, out, None, dev(req), len(req), B, T, H, H, DK, DV,
                   DK ** -0.5, T)
        torch.cuda.synchronize()
        alone_o, alone_s = host(out), host(state)
        for r in range(B):
            if placements[pid[r]][l] in "FS":
                assert np.array_equal(outs[l][r], alone_o[r]), (l, r)
                assert np.array_equal(states[l][r], alone_s[r]), (l, r)
            else:
                assert rel_err(outs[l][r], alone_o[r]) <= 2e-6, (l, r)
                assert rel_err(states[l][r], alone_s[r]) <= 2e-6, (l, r)


@pytest.mark.parametrize("case", range(8))
def test_random_stacks(case):
    """Seeded random stacks: number of layers, batch, placements, mixers per layer, ragged lengths, window, token
    count and state slots all vary, so layers with one, two, three and four mixers present all occur."""
    rng = np.random.default_rng(9700 + case)
    L, B = int(rng.integers(2, 7)), int(rng.integers(1, 11))
    n_pl = int(rng.integers(1, 5))
    T = int(rng.choice([1, 1, 1, 2, 4]))
    placements = ["".join(rng.choice(list("FSKG"), size=L)) for _ in range(n_pl)]
    pid = rng.integers(0, n_pl, size=B).astype(np.int32)
    ctx = int(rng.choice([96, 700, 2100]))
    max_pages = (ctx + 15) // 16 + int(rng.integers(0, 3))
    lens = rng.integers(T, ctx + 1, size=B).astype(np.int32)
    lens[rng.integers(B)] = ctx
    window = int(rng.choice([16, 100, 512, 5000]))
    n_slots = B + int(rng.integers(0, 3))
    slot = rng.permutation(n_slots)[:B].astype(np.int32)
    layers = build_stack(9800 + 100 * case, L, B, T, ctx, max_pages, lens)
    outs, states = run_stack(placements, pid, layers, T, window, ctx, max_pages, slot, n_slots)
    ref_outs, ref_states = om.placement_decode(placements, pid, layers, window, D ** -0.5, DK ** -0.5)
    for l in range(L):
        for r in range(B):
            m = placements[pid[r]][l]
            assert rel_err(outs[l][r], ref_outs[l][r]) <= OUT_TOL, (case, l, r, m)
            if m in "KG":
                assert rel_err(states[l][slot[r]], ref_states[l][r]) <= STATE_TOL, (case, l, r, m)
            else:
                assert np.array_equal(states[l][slot[r]], layers[l]["state"][r]), (case, l, r, m)
        unused = [x for x in range(n_slots) if x not in slot]
        assert (states[l][unused] == 9.0).all()


def test_one_output_buffer_shared_by_all_layers():
    """A caller may hand every layer the same output buffer (each layer's result is consumed before the next layer
    writes): the merge of a layer's partial results then cannot ride on the next layer's launch, and the buffer must end
    up holding the last layer's rows.  Contexts long enough for several page ranges per (request, KV head)."""
    L, B, ctx, window, max_pages = 4, 4, 1500, 700, 96
    placements = ["FSFF", "SFKF", "FFSG"]
    pid = np.array([0, 1, 2, 0], dtype=np.int32)
    lens = np.array([1500, 1301, 1499, 1100], dtype=np.int32)
    layers = build_stack(5600, L, B, 1, ctx, max_pages, lens)
    ref_outs, _ = om.placement_decode(placements, pid, layers, window, D ** -0.5, DK ** -0.5)
    plan = sa.placement_plan_create(placements, pid)
    shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
    ws_bytes = sa.placement_workspace_bytes(plan, shapes, 1, ctx, window)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    shared = torch.full((B, 1, H, DV), 55.0, dtype=torch.float32, device="cuda")
    keep, ios = [], []
    for io in layers:
        kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
        t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
        t["state"], t["kpool"], t["vpool"] = dev(io["state"].copy()), dev(kphys), dev(vphys)
        keep.append(t)
        ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                                    beta=t["beta"], state=t["state"], q_attn=t["qa"], kpool=t["kpool"], vpool=t["vpool"],
                                    n_pages=io["n_pages"], page_table=t["page_table"], seq_lens=t["seq_lens"],
                                    max_pages=max_pages, max_seq_len=ctx, out=shared))
    sa.placement_decode(plan, ios, shapes, 1, window, D ** -0.5, DK ** -0.5, ws, ws_bytes)
    torch.cuda.synchronize()
    sa.placement_plan_destroy(plan)
    got = host(shared)
    for r in range(B):
        assert rel_err(got[r], ref_outs[L - 1][r]) <= OUT_TOL, r


def test_same_placement_for_all_requests_and_empty_batch():
    """All requests on one placement: every layer is a single launch over the whole batch."""
    L, B, ctx, window, max_pages = 4, 3, 200, 64, 16
    layers = build_stack(5200, L, B, 1, ctx, max_pages)
    placements = ["FKSG", "GGGG"]
    pid = np.zeros(B, dtype=np.int32)
    plan = sa.placement_plan_create(placements, pid)
    shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
    ws_bytes = sa.placement_workspace_bytes(plan, shapes, 1, ctx, window)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    keep, ios = [], []
    for io in layers:
        kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
        t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
        t["state"], t["kpool"], t["vpool"] = dev(io["state"].copy()), dev(kphys), dev(vphys)
        t["out"] = torch.zeros((B, 1, H, DV), dtype=torch.float32, device="cuda")
        keep.append(t)
        ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                                    beta=t["beta"], state=t["state"], q_attn=t["qa"], kpool=t["kpool"], vpool=t["vpool"],
                                    n_pages=io["n_pages"], page_table=t["page_table"], seq_lens=t["seq_lens"],
                                    max_pages=max_pages, max_seq_len=ctx, out=t["out"]))
    sa.placement_decode(plan, ios, shapes, 1, window, D ** -0.5, DK ** -0.5, ws, ws_bytes)
    torch.cuda.synchronize()
    sa.placement_plan_destroy(plan)
    ref_outs, _ = om.placement_decode(placements, pid, layers, window, D ** -0.5, DK ** -0.5)
    for l in range(L):
        assert rel_err(host(keep[l]["out"]), ref_outs[l]) <= OUT_TOL
    empty = sa.placement_plan_create(placements, [])
    assert sa.placement_plan_count(empty, 0, "F") == 0
    sa.placement_decode(empty, ios, shapes, 1, window, 1.0, 1.0, ws, ws_bytes)
    sa.placement_plan_destroy(empty)


def test_full_size_stack_batch128_ctx16384():
    """BASELINE config 5: 48 layers, batch 128, 16384-token contexts, three placements (about 126 GiB of KV cache and
    state): one placement_decode step in the configuration the benchmark times.  Against the fp64 C form of the oracle
    (admitted at 1e-12 from the numpy oracle by tests/test_oracle_omp.py): every recurrent tile of every layer (all 128
    requests), and every query head of four seeded requests per placement on every attention layer.  Against the numpy
    oracle itself: two of those requests per placement through all 48 layers (all heads of a recurrent layer, one seeded
    query head of an attention layer)."""
    from oracle import omp
    from paper_2604_19877_amd.workloads import PlacementWorkload, fetch_logical_kv
    w = PlacementWorkload(B=128, L=48, ctx=16384, window=4096, T=1, seed=5000)
    try:
        rng = np.random.default_rng(6)
        wide, requests = [], []
        for p in range(3):
            chosen = [int(r) for r in rng.choice(np.flatnonzero(w.pid == p), size=4, replace=False)]
            wide += chosen
            requests += chosen[:2]
        before = [w.layers[l]["state"].view(-1, H, DK, DV).cpu().numpy() for l in range(w.L)]
        w.step()
        torch.cuda.synchronize()
        seen = set()
        for l in range(w.L):
            hl = w.host[l]
            got_l = w.layers[l]["out"].cpu().numpy()
            got_state = w.layers[l]["state"].view(-1, H, DK, DV).cpu().numpy()
            assert np.isfinite(got_l).all()
            # every recurrent tile of the layer
            for m, fn, gate in (("K", omp.kda_steps, "alpha_vec"), ("G", omp.gdn_steps, "alpha_scalar")):
                rows = np.flatnonzero(w.mixer[l] == m)
                if len(rows) == 0:
                    continue
                slots = hl["slot"][rows]
                o_ref, s_ref = fn(hl["q"][rows], hl["k"][rows], hl["v"][rows], hl[gate][rows], hl["beta"][rows], before[l][slots],
                                  w.rec_scale)
                for i, r in enumerate(rows):
                    assert rel_err(got_l[r], o_ref[i]) <= OUT_TOL, (l, r, m)
                    assert rel_err(got_state[slots[i]], s_ref[i]) <= STATE_TOL, (l, r, m)
            # every query head of the widely sampled requests on the attention mixers of the layer
            for m in "FS":
                rows = [r for r in wide if w.mixer[l, r] == m]
                if not rows:
                    continue
                first = 0 if m == "F" else (w.ctx - w.window) // 16
                n = w.max_pages - first
                table = np.full((len(rows), w.max_pages), -1, dtype=np.int32)
                ks, vs = [], []
                for i, r in enumerate(rows):
                    pages = torch.as_tensor(hl["page_table"][r, first:], device="cuda").long()
                    ks.append(w.kpool[pages].view(torch.int16).cpu().numpy().view(np.uint16))
                    vs.append(w.vpool[pages].view(torch.int16).cpu().numpy().view(np.uint16))
                    table[i, first:] = np.arange(i * n, (i + 1) * n)
                ref = omp.attn_decode(hl["q"][rows], np.concatenate(ks), np.concatenate(vs), table, np.full(len(rows), w.ctx, dtype=np.int32),
                                      w.window if m == "S" else 0, w.attn_scale, physical=True)
                for i, r in enumerate(rows):
                    for h in range(HQ):
                        assert rel_err(got_l[r][:, h], ref[i][:, h]) <= OUT_TOL, (l, r, m, h)
            # the numpy oracle on its sample
            for r in requests:
                m = str(w.mixer[l, r])
                seen.add(m)
                got = got_l[r]
                if m in "KG":
                    fn = om.kda_steps if m == "K" else om.gdn_steps
                    a = hl["alpha_vec"] if m == "K" else hl["alpha_scalar"]
                    sl = slice(r, r + 1)
                    slot = int(hl["slot"][r])
                    o_ref, s_ref = fn(hl["q"][sl], hl["k"][sl], hl["v"][sl], a[sl], hl["beta"][sl], before[l][slot][None], w.rec_scale)
                    assert rel_err(got, o_ref[0]) <= OUT_TOL, (l, r, m)
                    assert rel_err(got_state[slot], s_ref[0]) <= STATE_TOL, (l, r, m)
                else:
                    window = w.window if m == "S" else 0
                    first = 0 if m == "F" else (w.ctx - w.window) // 16
                    pages = hl["page_table"][r, first:]
                    assert (pages >= 0).all()
                    h = int(rng.integers(HQ))
                    kph, vph = fetch_logical_kv(w.kpool, w.vpool, pages, h // (HQ // HKV))
                    klog, vlog = kl.to_logical(kph, vph, D)
                    ident = np.full((1, w.max_pages), -1, dtype=np.int32)
                    ident[0, first:] = np.arange(len(pages))
                    ref = om.attn_decode(hl["q"][r:r + 1, :, h:h + 1], klog, vlog, ident, [w.ctx], window, w.attn_scale)
                    assert rel_err(got[:, h], ref[0, :, 0]) <= OUT_TOL, (l, r, m, h)
        assert seen == set("FSKG")
    finally:
        w.close()


def test_bad_descriptor_in_the_last_layer_enqueues_nothing():
    """Every launch of the stack is checked before the first one is enqueued."""
    L, B, ctx, window, max_pages = 3, 2, 100, 64, 8
    layers = build_stack(5300, L, B, 1, ctx, max_pages)
    plan = sa.placement_plan_create(["FGK"], np.zeros(B, dtype=np.int32))
    shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    keep, ios = [], []
    for l, io in enumerate(layers):
        kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
        t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
        t["state"], t["kpool"], t["vpool"] = dev(io["state"].copy()), dev(kphys), dev(vphys)
        t["out"] = torch.full((B, 1, H, DV), 55.0, dtype=torch.float32, device="cuda")
        keep.append(t)
        ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"],
                                    alpha_vec=None if l == L - 1 else t["alpha_vec"],          # the KDA layer lacks its gate
                                    beta=t["beta"], state=t["state"], q_attn=t["qa"], kpool=t["kpool"], vpool=t["vpool"],
                                    n_pages=io["n_pages"], page_table=t["page_table"], seq_lens=t["seq_lens"],
                                    max_pages=max_pages, max_seq_len=ctx, out=t["out"]))
    with pytest.raises(sa.SaError) as e:
        sa.placement_decode(plan, ios, shapes, 1, window, 1.0, 1.0, ws, ws.numel())
    assert e.value.status == sa.SA_EINVAL and "kda_decode_step" in str(e.value)
    torch.cuda.synchronize()
    for l, t in enumerate(keep):
        assert (t["out"] == 55.0).all()
        assert np.array_equal(host(t["state"]), layers[l]["state"])
    sa.placement_plan_destroy(plan)
