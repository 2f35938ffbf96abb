"""Chunk-parallel form of the GDN / KDA recurrences in fp64 (test infrastructure only).

Appendix B of the paper names the parallel forms the mixers train with (GDN: chunk by chunk on a WY
representation; KDA: diagonal-plus-low-rank transition matrices) and Section 6 uses such kernels for
prefill.  The paper prints neither, so this is a derivation from the printed recurrences:

with Gamma_t = prod_{i<=t} alpha_i inside the chunk (a scalar for GDN, a vector over key channels for
KDA), the state after t steps is  S_t = Gamma_t * S_0 + sum_{i<=t} (Gamma_t / Gamma_i) * k_i delta_i^T
(row-wise scaling), and the corrections delta_t = beta_t (v_t - (alpha_t S_{t-1})^T k_t) solve the
unit lower-triangular system
    delta_t + beta_t sum_{i<t} ((Gamma_t/Gamma_i) k_i . k_t) delta_i = beta_t (v_t - S_0^T (Gamma_t k_t)).
Everything is then matrix products over the chunk:
    Khat = Gamma * K, Ktil = K / Gamma,  A = tril(diag(beta) Khat Ktil^T, -1),
    Delta = (I + A)^{-1} diag(beta) (V - Khat S_0),
    O = scale * ((Gamma * Q) S_0 + tril(Qhat Ktil^T) Delta),   S_C = Gamma_C * S_0 + (Gamma_C * Ktil)^T Delta.
It must agree with the step-by-step oracle; tests/test_oracle_chunked.py checks that, which pins both.
"""
from __future__ import annotations

import numpy as np
from scipy.linalg import solve_triangular

from .mixers import _expand_heads, widen


def chunk_steps(q, k, v, alpha, beta, state, scale=1.0, per_channel=False):
    """Same interface and results as mixers.gdn_steps / kda_steps for one chunk of T tokens."""
    q, k, v, alpha, beta = widen(q), widen(k), widen(v), widen(alpha), widen(beta)
    S0 = widen(state)
    B, T, H, dv = v.shape
    q, k = _expand_heads(q, H), _expand_heads(k, H)
    dk = k.shape[-1]
    out = np.zeros((B, T, H, dv))
    S_out = np.zeros_like(S0)
    for b in range(B):
        for h in range(H):
            a = alpha[b, :, h]
            gam = np.cumprod(a, axis=0)                                  # [T] or [T,dk]
            gam = gam[:, None] * np.ones((1, dk)) if not per_channel else gam
            K, Q, V, be = k[b, :, h], q[b, :, h], v[b, :, h], beta[b, :, h]
            Khat, Ktil, Qhat = gam * K, K / gam, gam * Q
            A = np.tril(be[:, None] * (Khat @ Ktil.T), -1)
            rhs = be[:, None] * (V - Khat @ S0[b, h])
            Delta = solve_triangular(np.eye(T) + A, rhs, lower=True, unit_diagonal=True)
            out[b, :, h] = scale * (Qhat @ S0[b, h] + np.tril(Qhat @ Ktil.T) @ Delta)
            S_out[b, h] = gam[-1][:, None] * S0[b, h] + (gam[-1] * Ktil).T @ Delta
    return out, S_out
