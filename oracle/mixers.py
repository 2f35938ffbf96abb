"""CPU fp64 oracle for the decode step of the four token mixers (test infrastructure only).

This file is the parity reference for the HIP library and nothing else: only the tests, the smoke
check and the cpu_baseline leg of the benchmark may import it.  It shares no code with the GPU
path.  Everything is numpy in float64; bf16 inputs arrive as 16-bit patterns and are widened
exactly.

What each function follows
  * gdn_steps / kda_steps       -- the GDN and KDA state recurrences of Appendix B ("Gated DeltaNet
                                   (GDN)", "Kimi Delta Attention (KDA)"), evaluated in the rank-1
                                   form  S <- Sbar + beta k (v - Sbar^T k)^T  with Sbar the decayed
                                   state.  The paper prints no read-out; the reading taken is
                                   o_t = scale * S_t^T q_t with the state after the write.
  * gdn_steps_dense / kda_steps_dense -- the same recurrences with the transition matrix built
                                   explicitly, term by term as printed; used to pin the rank-1 form.
  * attn_decode                 -- grouped-query softmax attention of the newest T tokens over a
                                   paged cache: the definition of Appendix B "Full Attention (FA)"
                                   (window <= 0) and "Sliding Window Attention (SWA)" (each token
                                   sees the w most recent positions, itself included).
  * attn_decode_loops           -- the same definition as scalar Python loops for tiny inputs.
  * placement_decode            -- Section 6 "Per-request placement switching": request r runs, at
                                   layer l, the mixer named by its placement string.

Pinned by tests/test_oracle_*.py against closed forms and invariants (see those files); no value in
the paper can be reproduced numerically (it prints no worked example for any mixer).
"""
from __future__ import annotations

import math

import numpy as np

PAGE = 16


def widen(x) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly; float arrays -> float64."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


# ----------------------------------------------------------------------------- GDN / KDA
def _expand_heads(x: np.ndarray, H: int) -> np.ndarray:
    """[B,T,Hk,d] -> [B,T,H,d]: state head h uses q/k head h // (H/Hk) (contiguous groups)."""
    Hk = x.shape[2]
    if H % Hk:
        raise ValueError("H must be a multiple of Hk")
    return np.repeat(x, H // Hk, axis=2)


def _delta_steps(q, k, v, alpha, beta, state, scale, per_channel, n_commit):
    q, k, v = widen(q), widen(k), widen(v)
    alpha, beta = widen(alpha), widen(beta)
    S = widen(state).copy()                      # [B,H,dk,dv]
    B, T, H, dv = v.shape
    q, k = _expand_heads(q, H), _expand_heads(k, H)
    if n_commit is None:
        n_commit = T
    out = np.zeros((B, T, H, dv))
    S_commit = S.copy()
    for t in range(T):
        if per_channel:
            Sbar = alpha[:, t, :, :, None] * S                       # row i (key channel i) scaled by alpha_i
        else:
            Sbar = alpha[:, t, :, None, None] * S
        u = np.einsum("bhkv,bhk->bhv", Sbar, k[:, t])                # Sbar^T k
        delta = beta[:, t, :, None] * (v[:, t] - u)
        S = Sbar + k[:, t, :, :, None] * delta[:, :, None, :]        # + k delta^T
        out[:, t] = scale * np.einsum("bhkv,bhk->bhv", S, q[:, t])   # S_t^T q_t
        if t + 1 == n_commit:
            S_commit = S.copy()
    return out, S_commit


def gdn_steps(q, k, v, alpha, beta, state, scale=1.0, n_commit=None):
    """T sequential GDN steps.  q,k [B,T,Hk,dk]; v [B,T,H,dv]; alpha, beta [B,T,H]; state [B,H,dk,dv].
    Returns (out [B,T,H,dv], state after n_commit steps)."""
    return _delta_steps(q, k, v, alpha, beta, state, scale, False, n_commit)


def kda_steps(q, k, v, alpha, beta, state, scale=1.0, n_commit=None):
    """T sequential KDA steps; alpha is [B,T,H,dk] (one gate per key channel)."""
    return _delta_steps(q, k, v, alpha, beta, state, scale, True, n_commit)


def _dense_steps(q, k, v, alpha, beta, state, scale, per_channel):
    q, k, v = widen(q), widen(k), widen(v)
    alpha, beta = widen(alpha), widen(beta)
    S = widen(state).copy()
    B, T, H, dv = v.shape
    dk = k.shape[-1]
    q, k = _expand_heads(q, H), _expand_heads(k, H)
    out = np.zeros((B, T, H, dv))
    eye = np.eye(dk)
    for b in range(B):
        for h in range(H):
            for t in range(T):
                kk, vv, bt = k[b, t, h], v[b, t, h], beta[b, t, h]
                proj = eye - bt * np.outer(kk, kk)
                if per_channel:
                    A = proj @ np.diag(alpha[b, t, h])
                else:
                    A = alpha[b, t, h] * proj
                S[b, h] = A @ S[b, h] + bt * np.outer(kk, vv)
                out[b, t, h] = scale * (S[b, h].T @ q[b, t, h])
    return out, S


def gdn_steps_dense(q, k, v, alpha, beta, state, scale=1.0):
    """GDN with A_t = alpha_t (I - beta_t k k^T) formed as a dk x dk matrix."""
    return _dense_steps(q, k, v, alpha, beta, state, scale, False)


def kda_steps_dense(q, k, v, alpha, beta, state, scale=1.0):
    """KDA with A_t = (I - beta_t k k^T) diag(alpha_t) formed as a dk x dk matrix."""
    return _dense_steps(q, k, v, alpha, beta, state, scale, True)


# ----------------------------------------------------------------------------- attention
def _token_range(L: int, T: int, i: int, window: int):
    hi = L - T + i + 1                       # new token i sits at position hi-1 and sees itself
    lo = max(0, hi - window) if window > 0 else 0
    return lo, hi


def attn_decode(q, kpool, vpool, page_table, seq_lens, window=0, scale=1.0, rows=None):
    """GQA softmax attention of the newest T tokens of each sequence over its paged cache.

    q [B,T,Hq,D]; kpool, vpool logical pools [n_pages,Hkv,16,D]; page_table int [B,max_pages];
    seq_lens [B] counts the T new tokens.  window <= 0 is full attention.  rows: optional iterable
    of (b, i, h) triples to evaluate (others are left zero).  Returns out [B,T,Hq,D] float64.
    """
    q = widen(q)
    B, T, Hq, D = q.shape
    Hkv = kpool.shape[1]
    group = Hq // Hkv
    out = np.zeros((B, T, Hq, D))
    if rows is None:
        rows = [(b, i, h) for b in range(B) for i in range(T) for h in range(Hq)]
    cache = {}
    for (b, i, h) in rows:
        L = int(seq_lens[b])
        lo, hi = _token_range(L, T, i, window)
        if hi <= lo or hi <= 0:
            continue
        g = h // group
        key = (b, g, lo, hi)
        if key not in cache:
            if len(cache) > 8:
                cache.clear()
            pos = np.arange(lo, hi)
            phys = np.asarray(page_table[b])[pos // PAGE]
            if np.any(phys < 0):
                raise ValueError("live token maps to an unmapped page")
            cache[key] = (widen(kpool[phys, g, pos % PAGE]), widen(vpool[phys, g, pos % PAGE]))
        K, V = cache[key]
        s = scale * (K @ q[b, i, h])
        p = np.exp(s - np.max(s))
        p = p / np.sum(p)
        out[b, i, h] = p @ V
    return out


def attn_decode_loops(q, kpool, vpool, page_table, seq_lens, window=0, scale=1.0):
    """The same definition written as scalar loops (tiny inputs only)."""
    q = widen(q)
    kpool, vpool = widen(kpool), widen(vpool)
    B, T, Hq, D = q.shape
    Hkv = kpool.shape[1]
    group = Hq // Hkv
    out = np.zeros((B, T, Hq, D))
    for b in range(B):
        L = int(seq_lens[b])
        for i in range(T):
            hi = L - T + i + 1
            lo = 0
            if window > 0 and hi - window > 0:
                lo = hi - window
            if hi <= 0:
                continue
            for h in range(Hq):
                g = h // group
                scores = []
                for j in range(lo, hi):
                    page = int(page_table[b][j // PAGE])
                    acc = 0.0
                    for d in range(D):
                        acc += q[b, i, h, d] * kpool[page, g, j % PAGE, d]
                    scores.append(scale * acc)
                biggest = max(scores)
                weights = [math.exp(s - biggest) for s in scores]
                total = sum(weights)
                for d in range(D):
                    acc = 0.0
                    for n, j in enumerate(range(lo, hi)):
                        page = int(page_table[b][j // PAGE])
                        acc += weights[n] * vpool[page, g, j % PAGE, d]
                    out[b, i, h, d] = acc / total
    return out


# ----------------------------------------------------------------------------- placement
def parse_placements(placements, n_layers):
    for s in placements:
        if len(s) != n_layers:
            raise ValueError("placement length differs from the layer count")
        for c in s:
            if c not in "FSKG":
                raise ValueError("unknown mixer character %r" % c)
    return [list(s) for s in placements]


def placement_decode(placements, placement_id, layers, window, attn_scale, rec_scale):
    """Run one decode step of a mixers-only stack with a per-request placement.

    placements: list of strings over {F,S,K,G}, one character per layer.  placement_id: [B] ints.
    layers: list (one per layer) of dicts holding every operand of that layer for the whole batch:
      q,k,v,alpha_scalar,alpha_vec,beta,state  (recurrent; state [B,H,dk,dv])
      qa,kpool,vpool,page_table,seq_lens        (attention)
    Only the entries of the mixer a request actually runs are read.  Returns
    (outs: list of [B,T,H,dv] float64, states: list of [B,H,dk,dv] float64 with non-participating
    rows unchanged).
    """
    table = parse_placements(placements, len(layers))
    outs, states = [], []
    for l, io in enumerate(layers):
        B = len(placement_id)
        out = None
        new_state = widen(io["state"]).copy() if io.get("state") is not None else None
        for r in range(B):
            m = table[int(placement_id[r])][l]
            if m in "FS":
                o = attn_decode(io["qa"][r:r + 1], io["kpool"], io["vpool"], io["page_table"][r:r + 1],
                                io["seq_lens"][r:r + 1], window if m == "S" else 0, attn_scale)
            else:
                fn = kda_steps if m == "K" else gdn_steps
                a = io["alpha_vec"] if m == "K" else io["alpha_scalar"]
                o, s = fn(io["q"][r:r + 1], io["k"][r:r + 1], io["v"][r:r + 1], a[r:r + 1],
                          io["beta"][r:r + 1], io["state"][r:r + 1], rec_scale)
                new_state[r] = s[0]
            if out is None:
                out = np.zeros((B,) + o.shape[1:])
            out[r] = o[0]
        outs.append(out)
        states.append(new_state)
    return outs, states
