"""CPU fp64 oracle for the decode step of a whole GDN / KDA mixer block around the state update
(test infrastructure only; shares no code with the GPU path).

Appendix B of the paper lists, for GDN: a short causal 1-D convolution with SiLU on Q, K and V before
the recurrence, L2-normalised queries and keys, beta = sigmoid(beta_raw),
g = -exp(A_log) * softplus(alpha_raw + dt_bias) as the log-decay (alpha = exp(g)), and a gated RMS
normalisation of the read-out with z as the gate; for KDA: the same with one convolution per stream,
a per-key-channel gate that comes out of one fused gate computation, and a separate output gate.  The paper gives
no formula for the normalisation or for KDA's gate; the readings taken are
  * L2 norm:   x / sqrt(sum(x^2) + 1e-6) per head,
  * KDA gate:  the GDN formula per channel, A_log per head and dt_bias per (head, channel),
  * out norm:  y = weight * o / sqrt(mean(o^2) + eps) * act(z), per head, act = SiLU (GDN) or
               sigmoid (KDA output gate), chosen by the caller.
Depthwise convolution: tap Kc-1 multiplies the newest input; the state holds the Kc-1 previous inputs,
oldest first.  Pinned in tests/test_oracle_block.py (scipy's FIR filter, the paper's initial values,
closed forms).
"""
from __future__ import annotations

import numpy as np

from .mixers import _delta_steps, widen

L2_EPS = 1e-6


def silu(x):
    return x / (1.0 + np.exp(-x))


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def softplus(x):
    return np.logaddexp(0.0, x)


def causal_conv_silu_step(x_new, conv_state, weight, bias=None):
    """One token of a depthwise causal convolution followed by SiLU.
    x_new [B,C]; conv_state [B,Kc-1,C] (oldest first); weight [Kc,C].  Returns (y [B,C], new state)."""
    x_new, conv_state, weight = widen(x_new), widen(conv_state), widen(weight)
    taps = weight.shape[0]
    window = np.concatenate([conv_state, x_new[:, None, :]], axis=1)          # [B,Kc,C], oldest first
    assert window.shape[1] == taps
    acc = np.einsum("bjc,jc->bc", window, weight)
    if bias is not None:
        acc = acc + widen(bias)
    return silu(acc), window[:, 1:, :].copy()


def l2_normalise(x):
    return x / np.sqrt(np.sum(x * x, axis=-1, keepdims=True) + L2_EPS)


def decay_gate(alpha_raw, A_log, dt_bias):
    """alpha = exp(-exp(A_log) * softplus(alpha_raw + dt_bias)); A_log broadcasts per head."""
    return np.exp(-np.exp(widen(A_log)) * softplus(widen(alpha_raw) + widen(dt_bias)))


def gated_rms_norm(o, z, weight, eps, gate_act):
    o, z, weight = widen(o), widen(z), widen(weight)
    act = silu(z) if gate_act == "silu" else sigmoid(z)
    return weight * o / np.sqrt(np.mean(o * o, axis=-1, keepdims=True) + eps) * act


def block_decode_step(kind, xq, xk, xv, conv_q, conv_k, conv_v, wq, wk, wv, beta_raw, alpha_raw, A_log, dt_bias,
                      z, norm_weight, norm_eps, gate_act, state, scale):
    """One decode token through a GDN ("gdn") or KDA ("kda") block.

    xq, xk [B,Hk,dk]; xv [B,H,dv] (bf16 patterns or floats): projection outputs before the convolution.
    conv_q, conv_k [B,Kc-1,Hk*dk]; conv_v [B,Kc-1,H*dv]; wq, wk [Kc,Hk*dk]; wv [Kc,H*dv].
    beta_raw [B,H]; alpha_raw [B,H] (gdn) or [B,H,dk] (kda); A_log [H]; dt_bias [H] or [H,dk].
    z [B,H,dv]; norm_weight [dv]; state [B,H,dk,dv].
    Returns dict(out [B,H,dv], state, conv_q, conv_k, conv_v, q, k, v, alpha, beta).
    """
    B, Hk, dk = np.asarray(xq).shape
    _, H, dv = np.asarray(xv).shape
    q, conv_q = causal_conv_silu_step(np.asarray(xq).reshape(B, -1), conv_q, wq)
    k, conv_k = causal_conv_silu_step(np.asarray(xk).reshape(B, -1), conv_k, wk)
    v, conv_v = causal_conv_silu_step(np.asarray(xv).reshape(B, -1), conv_v, wv)
    q = l2_normalise(q.reshape(B, Hk, dk))
    k = l2_normalise(k.reshape(B, Hk, dk))
    v = v.reshape(B, H, dv)
    beta = sigmoid(widen(beta_raw))
    if kind == "kda":
        alpha = decay_gate(alpha_raw, widen(A_log)[None, :, None], widen(dt_bias)[None])
    else:
        alpha = decay_gate(alpha_raw, widen(A_log)[None], widen(dt_bias)[None])
    o, S = _delta_steps(q[:, None], k[:, None], v[:, None], alpha[:, None], beta[:, None], state, scale, kind == "kda", 1)
    out = gated_rms_norm(o[:, 0], z, norm_weight, norm_eps, gate_act)
    return {"out": out, "state": S, "conv_q": conv_q, "conv_k": conv_k, "conv_v": conv_v,
            "q": q, "k": k, "v": v, "alpha": alpha, "beta": beta}
