"""The hot calls only enqueue kernels (no allocation, no synchronisation, no memset), so a decode step can
be captured into a HIP graph once per placement assignment and replayed, as the paper's serving stack
pre-captures one graph per placement.  Replays are interleaved with eager work and each is checked."""
import numpy as np
import pytest
import torch

from oracle import kv_layout as kl
from paper_2604_19877_amd import binding as sa
from paper_2604_19877_amd import inputs as gen
from gpu_util import dev, host
from test_gpu_placement import D, DK, DV, H, HKV, HQ, build_stack

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T", [1, 4, 8])
def test_placement_step_replays_from_a_graph(T):
    """T = 4 is a verify pass on the fused per-layer launches (partial results merged by the next layer's launch);
    T = 8 a longer one: two query tiles in attention, the chunk-parallel kernels for the recurrent mixers."""
    L, B, ctx, window, max_pages = 8, 6, 700, 128, 48
    placements = [gen.placement_string(8001 + i, L) for i in range(3)]
    pid = np.arange(B, dtype=np.int32) % 3
    layers = build_stack(8100, L, B, T, ctx, max_pages)
    plan = sa.placement_plan_create(placements, pid)
    shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, 16)
    ws_bytes = sa.placement_workspace_bytes(plan, shapes, T, ctx, window)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    keep, ios = [], []
    for io in layers:
        kphys, vphys = kl.to_physical(io["kpool"], io["vpool"])
        t = {n: dev(io[n]) for n in ("q", "k", "v", "alpha_scalar", "alpha_vec", "beta", "qa", "page_table", "seq_lens")}
        t["state0"] = dev(io["state"].copy())
        t["state"], t["kpool"], t["vpool"] = dev(io["state"].copy()), dev(kphys), dev(vphys)
        t["out"] = torch.zeros((B, T, H, DV), dtype=torch.float32, device="cuda")
        keep.append(t)
        ios.append(sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                                    beta=t["beta"], state=t["state"], q_attn=t["qa"], kpool=t["kpool"], vpool=t["vpool"],
                                    n_pages=io["n_pages"], page_table=t["page_table"], seq_lens=t["seq_lens"],
                                    max_pages=max_pages, max_seq_len=ctx, out=t["out"]))
    io_arr = (sa.sa_layer_io * L)(*ios)

    def reset():
        for t in keep:
            t["state"].copy_(t["state0"])
            t["out"].zero_()

    def step(stream=None):
        sa.placement_decode(plan, io_arr, shapes, T, window, D ** -0.5, DK ** -0.5, ws, ws_bytes, stream)

    reset()
    step()
    torch.cuda.synchronize()
    want_out = [host(t["out"]).copy() for t in keep]
    want_state = [host(t["state"]).copy() for t in keep]

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())
    for replay in range(3):
        reset()
        scratch = torch.randn(1 << 20, device="cuda").cumsum(0)      # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l, t in enumerate(keep):
            assert np.array_equal(host(t["out"]), want_out[l]), (replay, l)
            assert np.array_equal(host(t["state"]), want_state[l]), (replay, l)
        del scratch
    sa.placement_plan_destroy(plan)
