"""Device-resident synthetic workloads at the paper's 15B-class shapes, shared by bench.py and the
full-size GPU tests.  Only allocation, seeded random fills and table building: no mixer arithmetic.
"""
from __future__ import annotations

import numpy as np

from . import binding as sa
from . import inputs as gen

H, DK, DV = 32, 128, 128
HQ, HKV, D, PAGE = 32, 8, 128, 16


def dev(a):
    """Host array -> device tensor; bf16 bit patterns (uint16) travel as int16."""
    import torch
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def fetch_logical_kv(kpool, vpool, pages, kv_head):
    """Physical blocks of the given pages and one KV head, copied to the host as uint16
    [n, 1, 16*D] (the caller decodes the in-page layout)."""
    import torch
    idx = torch.as_tensor(pages, device="cuda").long()
    k = kpool[idx, kv_head].view(torch.int16).cpu().numpy().view(np.uint16)[:, None]
    v = vpool[idx, kv_head].view(torch.int16).cpu().numpy().view(np.uint16)[:, None]
    return k, v


class PlacementWorkload:
    """A mixers-only stack of L layers for B requests, each request on one of three seeded placements
    (12 FA / 12 SWA / 12 KDA / 12 GDN per 48 layers, shuffled), all contexts `ctx` tokens long.

    One global K pool and one global V pool serve every attention layer (per-layer page tables point
    into them); sliding-window layers map only the pages their window touches.  Recurrent layers hold
    state only for the requests that run a recurrent mixer there (slot maps).

    page_scatter = "layer": every layer's cache is a region of its own in the pools (a serving engine allocates one
    KV tensor per layer) and the pages of its requests are a seeded shuffle inside that region.  "global": the
    pages of all layers are one seeded shuffle over the whole pools, which costs the attention kernels several per
    cent at pools of 100 GiB (address translation reaches further).
    """

    def __init__(self, B=128, L=48, ctx=16384, window=4096, T=1, seed=5000, n_placements=3, placements=None,
                 page_scatter="layer"):
        import torch
        self.B, self.L, self.ctx, self.window, self.T = B, L, ctx, window, T
        if placements is None:
            placements = [gen.placement_string(seed + 1 + i, L) for i in range(n_placements)]
        self.placements, n_placements = list(placements), len(placements)
        self.pid = (np.arange(B) % n_placements).astype(np.int32)
        self.max_pages = (ctx + PAGE - 1) // PAGE
        first_win = max(0, ctx - T + 1 - window) // PAGE
        mixer = np.array([[self.placements[p][l] for p in self.pid] for l in range(L)])     # [L,B]
        self.mixer = mixer
        n_f = int((mixer == "F").sum())
        n_s = int((mixer == "S").sum())
        self.n_pages = n_f * self.max_pages + n_s * (self.max_pages - first_win) + 3
        rng = np.random.default_rng(seed)
        if page_scatter == "global":
            perm = rng.permutation(self.n_pages).astype(np.int32)
        elif page_scatter == "layer":
            perm, start = np.empty(self.n_pages, dtype=np.int32), 0
            for l in range(L):
                n = int((mixer[l] == "F").sum()) * self.max_pages + int((mixer[l] == "S").sum()) * (self.max_pages - first_win)
                perm[start:start + n] = start + rng.permutation(n)
                start += n
            perm[start:] = np.arange(start, self.n_pages)          # the spare pages
        else:
            raise ValueError("page_scatter must be 'layer' or 'global'")
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        self.kpool = torch.empty((self.n_pages, HKV, PAGE * D), dtype=torch.bfloat16, device="cuda")
        self.vpool = torch.empty((self.n_pages, HKV, PAGE * D), dtype=torch.bfloat16, device="cuda")
        self.kpool.normal_(generator=g)
        self.vpool.normal_(generator=g)
        self.shapes = sa.sa_shapes(H, H, DK, DV, HQ, HKV, D, PAGE)
        self.attn_scale, self.rec_scale = D ** -0.5, DK ** -0.5
        self.seq_lens_h = np.full(B, ctx, dtype=np.int32)
        self.seq_lens = dev(self.seq_lens_h)
        self.layers, self.host = [], []
        at = 0
        for l in range(L):
            table = np.full((B, self.max_pages), -1, dtype=np.int32)
            for r in range(B):
                if mixer[l, r] == "F":
                    table[r, :] = perm[at:at + self.max_pages]
                    at += self.max_pages
                elif mixer[l, r] == "S":
                    n = self.max_pages - first_win
                    table[r, first_win:] = perm[at:at + n]
                    at += n
            rec_rows = np.flatnonzero((mixer[l] == "K") | (mixer[l] == "G"))
            slot = np.full(B, 0, dtype=np.int32)
            slot[rec_rows] = np.arange(len(rec_rows), dtype=np.int32)
            ops = gen.recurrent_inputs(seed + 100 + 2 * l, B, T, H, H, DK, DV, False)
            ops_vec = gen.recurrent_inputs(seed + 101 + 2 * l, B, T, H, H, DK, DV, True)
            state = torch.empty((max(len(rec_rows), 1) * H, DK, DV), dtype=torch.float32, device="cuda")
            if len(rec_rows):
                state.normal_(0.0, 0.02, generator=g)
            t = {"q": dev(ops["q"]), "k": dev(ops["k"]), "v": dev(ops["v"]), "alpha_scalar": dev(ops["alpha"]),
                 "alpha_vec": dev(ops_vec["alpha"]), "beta": dev(ops["beta"]), "state": state, "slot_idx": dev(slot),
                 "page_table": dev(table), "out": torch.zeros((B, T, H, DV), dtype=torch.float32, device="cuda")}
            self.layers.append(t)
            self.host.append({"q": ops["q"], "k": ops["k"], "v": ops["v"], "alpha_scalar": ops["alpha"],
                              "alpha_vec": ops_vec["alpha"], "beta": ops["beta"], "slot": slot, "page_table": table})
        self.plan = sa.placement_plan_create(self.placements, self.pid)
        self.io = (sa.sa_layer_io * L)(*[
            sa.make_layer_io(q=t["q"], k=t["k"], v=t["v"], alpha_scalar=t["alpha_scalar"], alpha_vec=t["alpha_vec"],
                             beta=t["beta"], state=t["state"], slot_idx=t["slot_idx"], q_attn=t["q"], kpool=self.kpool,
                             vpool=self.vpool, n_pages=self.n_pages, page_table=t["page_table"], seq_lens=self.seq_lens,
                             max_pages=self.max_pages, max_seq_len=ctx, out=t["out"]) for t in self.layers])
        self.ws_bytes = sa.placement_workspace_bytes(self.plan, self.shapes, T, ctx, window)
        self.ws = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device="cuda")

    def step(self, stream=None):
        sa.placement_decode(self.plan, self.io, self.shapes, self.T, self.window, self.attn_scale, self.rec_scale, self.ws,
                            self.ws_bytes, stream)

    def algorithmic_bytes(self) -> int:
        """Bytes one step must move: K/V of every attended token, state read + write of every recurrent tile."""
        n_f = int((self.mixer == "F").sum())
        n_s = int((self.mixer == "S").sum())
        n_rec = int(((self.mixer == "K") | (self.mixer == "G")).sum())
        per_token = 2 * HKV * D * 2
        return (n_f * self.ctx + n_s * min(self.ctx, self.window)) * per_token + n_rec * H * 2 * DK * DV * 4

    def close(self):
        if self.plan is not None:
            sa.placement_plan_destroy(self.plan)
            self.plan = None
