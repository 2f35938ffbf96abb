"""ctypes front of oracle/mixers_omp.c, the fp64 C / OpenMP twin of oracle/mixers.py (test infrastructure only).

Same call shapes as gdn_steps / kda_steps / attn_decode of the numpy oracle, which stays the parity authority:
tests/test_oracle_omp.py admits this twin only while it agrees with it to 1e-12, and bench.py times it as the
all-cores CPU baseline.  Build with `python -m oracle.build`; loading raises if the library is missing.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import kv_layout as kl

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmixers_omp.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s is missing: build it with `python -m oracle.build`" % LIB_PATH)
        h = ctypes.CDLL(LIB_PATH)
        P, I, D = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        h.sa_oracle_threads.restype = I
        h.sa_oracle_threads.argtypes = []
        h.sa_oracle_delta_steps.restype = I
        h.sa_oracle_delta_steps.argtypes = [P] * 8 + [I] * 6 + [D, I, I]
        h.sa_oracle_attn_decode.restype = I
        h.sa_oracle_attn_decode.argtypes = [P, P, P, I, P, P, P, I, P, P] + [I] * 6 + [D]
        _lib = h
    return _lib


def threads() -> int:
    """OpenMP threads a call will use."""
    return lib().sa_oracle_threads()


def _arr(x, dtype):
    return np.ascontiguousarray(np.asarray(x), dtype=dtype)


def _delta(q, k, v, alpha, beta, state, scale, per_channel, n_commit):
    q, k, v = _arr(q, np.uint16), _arr(k, np.uint16), _arr(v, np.uint16)
    alpha, beta, state = _arr(alpha, np.float32), _arr(beta, np.float32), _arr(state, np.float32)
    B, T, Hk, dk = q.shape
    _, _, H, dv = v.shape
    if n_commit is None:
        n_commit = T
    out = np.empty((B, T, H, dv), dtype=np.float64)
    state_out = np.empty((B, H, dk, dv), dtype=np.float64)
    rc = lib().sa_oracle_delta_steps(q.ctypes.data, k.ctypes.data, v.ctypes.data, alpha.ctypes.data, beta.ctypes.data,
                                     state.ctypes.data, out.ctypes.data, state_out.ctypes.data, B, T, H, Hk, dk, dv,
                                     float(scale), int(per_channel), int(n_commit))
    if rc != 0:
        raise ValueError("sa_oracle_delta_steps failed (%d)" % rc)
    return out, state_out


def gdn_steps(q, k, v, alpha, beta, state, scale=1.0, n_commit=None):
    return _delta(q, k, v, alpha, beta, state, scale, False, n_commit)


def kda_steps(q, k, v, alpha, beta, state, scale=1.0, n_commit=None):
    return _delta(q, k, v, alpha, beta, state, scale, True, n_commit)


def attn_decode(q, kpool, vpool, page_table, seq_lens, window=0, scale=1.0, physical=False):
    """kpool, vpool: uint16 pools, logical [n_pages,Hkv,16,D] or, with physical=True, the library's in-page order
    [n_pages,Hkv,16*D] (decoded through the index maps of oracle/kv_layout.py)."""
    q = _arr(q, np.uint16)
    B, T, Hq, D = q.shape
    kpool, vpool = _arr(kpool, np.uint16), _arr(vpool, np.uint16)
    n_pages, Hkv = kpool.shape[0], kpool.shape[1]
    if physical:
        kmap, vmap = kl._index_maps(D)
    else:
        kmap = vmap = np.arange(kl.PAGE * D).reshape(kl.PAGE, D)
    kmap, vmap = _arr(kmap, np.int32), _arr(vmap, np.int32)
    table, lens = _arr(page_table, np.int32), _arr(seq_lens, np.int32)
    out = np.empty((B, T, Hq, D), dtype=np.float64)
    rc = lib().sa_oracle_attn_decode(q.ctypes.data, kpool.ctypes.data, vpool.ctypes.data, n_pages, kmap.ctypes.data,
                                     vmap.ctypes.data, table.ctypes.data, table.shape[1], lens.ctypes.data, out.ctypes.data,
                                     B, T, Hq, Hkv, D, int(window), float(scale))
    if rc == -2:
        raise ValueError("live token maps to an unmapped page")
    if rc != 0:
        raise ValueError("sa_oracle_attn_decode failed (%d)" % rc)
    return out
