"""Seeded synthetic inputs for the mixer decode path.

This module only draws numbers and formats them (bf16 bit patterns, page tables, placement
strings).  It holds none of the mixers' arithmetic and is the one piece shared by the tests of the
CPU oracle and of the HIP library: both consume exactly the arrays produced here.

Value recipes follow the workload shapes of the paper's 15B model (48 layers, 32 query / 8 KV
heads, head dim 128, window 4096; Section 2 "Teacher" and "Mixer vocabulary", Appendix B):
  * q, k ~ N(0,1), rounded to bf16, L2-normalised per head in fp32, rounded to bf16 again
    (Appendix B: queries and keys of GDN/KDA are L2-normalised);
  * v ~ N(0,1) in bf16;
  * beta = sigmoid(N(0,1)), alpha = exp(-softplus(N(0,1) + 2)), fp32, alpha per head (GDN) or per
    key channel (KDA);
  * attention q/K/V ~ N(0,1) in bf16, 16-token pages, page table = seeded permutation.
All small tensors come from numpy's default_rng(seed) on the host so the same bits exist on the
CPU-only box and on the GPU machine.
"""
from __future__ import annotations

import numpy as np

PAGE_SIZE = 16
MIXER_CHARS = "FSKG"  # full attention, sliding window, KDA, GDN


# ----------------------------------------------------------------------------- bf16 formatting
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even) and return the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def _unit_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    x = bf16_bits_to_f32(_normal_bf16(rng, shape))
    n = np.sqrt(np.sum(x.astype(np.float32) ** 2, axis=-1, keepdims=True, dtype=np.float32))
    return f32_to_bf16_bits(x / np.maximum(n, np.float32(1e-12)))


def _softplus(x):
    return np.logaddexp(0.0, x)


# ----------------------------------------------------------------------------- recurrent mixers
def recurrent_inputs(seed: int, B: int, T: int, H: int, Hk: int, dk: int, dv: int, per_channel_gate: bool):
    """Operands of T consecutive tokens for B sequences of a GDN (scalar gate) or KDA
    (per-key-channel gate) layer.

    Returns a dict: q, k uint16 [B,T,Hk,dk]; v uint16 [B,T,H,dv]; alpha fp32 [B,T,H] or
    [B,T,H,dk]; beta fp32 [B,T,H].
    """
    rng = np.random.default_rng(seed)
    q = _unit_bf16(rng, (B, T, Hk, dk))
    k = _unit_bf16(rng, (B, T, Hk, dk))
    v = _normal_bf16(rng, (B, T, H, dv))
    beta = (1.0 / (1.0 + np.exp(-rng.standard_normal((B, T, H))))).astype(np.float32)
    ashape = (B, T, H, dk) if per_channel_gate else (B, T, H)
    alpha = np.exp(-_softplus(rng.standard_normal(ashape) + 2.0)).astype(np.float32)
    return {"q": q, "k": k, "v": v, "alpha": alpha, "beta": beta}


def recurrent_state(seed: int, n_tiles: int, dk: int, dv: int, std: float = 0.02) -> np.ndarray:
    """Resident fp32 states, row-major [n_tiles, dk, dv], N(0, std^2); std=0 gives zeros."""
    if std == 0.0:
        return np.zeros((n_tiles, dk, dv), dtype=np.float32)
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n_tiles, dk, dv), dtype=np.float32) * np.float32(std)).astype(np.float32)


def block_inputs(seed: int, B: int, H: int, Hk: int, dk: int, dv: int, taps: int, per_channel_gate: bool, n_slots=None):
    """Operands of one decode token of a whole GDN / KDA block (before the convolution): projection
    outputs xq, xk [B,Hk,dk], xv and z [B,H,dv] ~ N(0,1) bf16; convolution histories (the taps-1
    previous inputs, oldest first) [n_slots,taps-1,C] ~ N(0,1) bf16; depthwise taps fp32 [taps,C] ~
    N(0, 1/taps); raw gates ~ N(0,1); A_log ~ log 0.1 + N(0, 0.3^2) per head; dt_bias ~ N(0,1) per head
    (GDN) or per (head, channel) (KDA); norm weight 1 + 0.1 N(0,1)."""
    rng = np.random.default_rng(seed)
    n_slots = B if n_slots is None else n_slots
    Cqk, Cv = Hk * dk, H * dv
    nb = lambda shape: _normal_bf16(rng, shape)
    f32 = lambda shape, scale=1.0: (rng.standard_normal(shape) * scale).astype(np.float32)
    return {
        "xq": nb((B, Hk, dk)), "xk": nb((B, Hk, dk)), "xv": nb((B, H, dv)), "z": nb((B, H, dv)),
        "conv_q": nb((n_slots, taps - 1, Cqk)), "conv_k": nb((n_slots, taps - 1, Cqk)), "conv_v": nb((n_slots, taps - 1, Cv)),
        "wq": f32((taps, Cqk), taps ** -0.5), "wk": f32((taps, Cqk), taps ** -0.5), "wv": f32((taps, Cv), taps ** -0.5),
        "beta_raw": f32((B, H)), "alpha_raw": f32((B, H, dk) if per_channel_gate else (B, H)),
        "A_log": (np.log(0.1) + rng.standard_normal(H) * 0.3).astype(np.float32),
        "dt_bias": f32((H, dk) if per_channel_gate else (H,)),
        "norm_weight": (1.0 + 0.1 * rng.standard_normal(dv)).astype(np.float32),
    }


# ----------------------------------------------------------------------------- paged attention
def context_lengths(seed: int, B: int, lo: int, hi: int) -> np.ndarray:
    """Context lengths uniform in [lo, hi], int32 (not page aligned)."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=B, dtype=np.int64).astype(np.int32)


def page_table(seed: int, seq_lens: np.ndarray, max_pages: int, n_spare_pages: int = 3,
               window_only: int = 0, n_new: int = 1):
    """A shuffled logical->physical page map.

    Every page a sequence needs gets a distinct physical page drawn from a seeded permutation of
    the pool; unmapped entries are -1.  With window_only=W>0 only the pages that intersect the
    last W + n_new - 1 tokens are mapped (a bounded sliding-window cache).
    Returns (table int32 [B,max_pages], n_pages_in_pool).
    """
    rng = np.random.default_rng(seed)
    B = len(seq_lens)
    need = []
    for L in seq_lens:
        L = int(L)
        last = (L + PAGE_SIZE - 1) // PAGE_SIZE
        first = 0
        if window_only > 0:
            first = max(0, L - n_new + 1 - window_only) // PAGE_SIZE
        need.append((first, last))
    total = sum(b - a for a, b in need)
    n_pages = total + n_spare_pages
    perm = rng.permutation(n_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    at = 0
    for b, (a, e) in enumerate(need):
        table[b, a:e] = perm[at:at + (e - a)]
        at += e - a
    return table, n_pages


def attention_inputs(seed: int, B: int, T: int, Hq: int, Hkv: int, D: int, seq_lens: np.ndarray,
                     max_pages: int, window_only: int = 0):
    """Small-scale paged-attention problem held entirely on the host.

    Returns a dict: q uint16 [B,T,Hq,D]; k_tok, v_tok uint16 [B,Lmax,Hkv,D] (token-major logical
    content, rows >= seq_lens[b] are unused); page_table int32 [B,max_pages]; n_pages; seq_lens.
    """
    rng = np.random.default_rng(seed)
    Lmax = int(max(1, int(np.max(seq_lens)) if len(seq_lens) else 1))
    q = _normal_bf16(rng, (B, T, Hq, D))
    k_tok = _normal_bf16(rng, (B, Lmax, Hkv, D))
    v_tok = _normal_bf16(rng, (B, Lmax, Hkv, D))
    table, n_pages = page_table(seed + 1, seq_lens, max_pages, window_only=window_only, n_new=T)
    return {"q": q, "k_tok": k_tok, "v_tok": v_tok, "page_table": table, "n_pages": n_pages,
            "seq_lens": np.asarray(seq_lens, dtype=np.int32)}


def logical_pools(k_tok: np.ndarray, v_tok: np.ndarray, table: np.ndarray, seq_lens: np.ndarray, n_pages: int):
    """Scatter token-major K/V into logical page pools [n_pages,Hkv,16,D] (uint16) through the table.
    Unwritten slots hold the bf16 NaN pattern 0x7FC0 so that any read of them shows up."""
    B, _, Hkv, D = k_tok.shape
    kp = np.full((n_pages, Hkv, PAGE_SIZE, D), 0x7FC0, dtype=np.uint16)
    vp = np.full((n_pages, Hkv, PAGE_SIZE, D), 0x7FC0, dtype=np.uint16)
    for b in range(B):
        for j in range(int(seq_lens[b])):
            p = table[b, j // PAGE_SIZE]
            if p < 0:
                continue
            kp[p, :, j % PAGE_SIZE, :] = k_tok[b, j]
            vp[p, :, j % PAGE_SIZE, :] = v_tok[b, j]
    return kp, vp


# ----------------------------------------------------------------------------- placements
def placement_string(seed: int, n_layers: int, counts=None) -> str:
    """A seeded shuffle of a mixer allocation, one character per layer (F, S, K, G)."""
    if counts is None:
        counts = {c: n_layers // 4 for c in MIXER_CHARS}
    chars = [c for c in MIXER_CHARS for _ in range(counts.get(c, 0))]
    if len(chars) != n_layers:
        raise ValueError("allocation does not sum to the number of layers")
    rng = np.random.default_rng(seed)
    return "".join(rng.permutation(np.array(chars)).tolist())
