"""ctypes binding of libsamixers.so: argument marshalling only.

Every function has the name and the argument order of its C entry point (include/samixers.h) and
takes torch tensors (device memory) or None where the C side takes pointers.  Nothing is computed
here; there is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char, c_char_p, c_float, c_int, c_int32, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsamixers.so")

SA_OK, SA_EINVAL, SA_EUNSUPPORTED, SA_EHIP, SA_EWORKSPACE, SA_ENOMEM = 0, -1, -2, -3, -4, -5
(SA_K_GDN, SA_K_KDA, SA_K_ATTN_SPLIT, SA_K_ATTN_MERGE, SA_K_KV_APPEND, SA_K_COPY, SA_K_GDN_BLOCK, SA_K_KDA_BLOCK,
 SA_K_GDN_CHUNK, SA_K_KDA_CHUNK, SA_K_STREAM, SA_K_LAYER) = range(12)


class SaError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("samixers status %d: %s" % (status, message))
        self.status = status


class sa_shapes(ctypes.Structure):
    _fields_ = [("H", c_int), ("Hk", c_int), ("dk", c_int), ("dv", c_int),
                ("Hq", c_int), ("Hkv", c_int), ("D", c_int), ("page_size", c_int)]


class sa_layer_io(ctypes.Structure):
    _fields_ = [("q", c_void_p), ("k", c_void_p), ("v", c_void_p),
                ("alpha_scalar", c_void_p), ("alpha_vec", c_void_p), ("beta", c_void_p),
                ("state", c_void_p), ("slot_idx", c_void_p),
                ("q_attn", c_void_p), ("kpool", c_void_p), ("vpool", c_void_p), ("n_pages", c_int),
                ("page_table", c_void_p), ("seq_lens", c_void_p), ("max_pages", c_int), ("max_seq_len", c_int),
                ("out", c_void_p), ("n_commit_rows", c_void_p)]


class sa_block_io(ctypes.Structure):
    _fields_ = [("xq", c_void_p), ("xk", c_void_p), ("xv", c_void_p), ("wq", c_void_p), ("wk", c_void_p), ("wv", c_void_p),
                ("conv_q_in", c_void_p), ("conv_k_in", c_void_p), ("conv_v_in", c_void_p),
                ("conv_q_out", c_void_p), ("conv_k_out", c_void_p), ("conv_v_out", c_void_p), ("conv_taps", c_int),
                ("beta_raw", c_void_p), ("alpha_raw", c_void_p), ("A_log", c_void_p), ("dt_bias", c_void_p),
                ("z", c_void_p), ("norm_weight", c_void_p), ("norm_eps", c_float), ("gate_act", c_int)]


_BLOCK_ARGS = [ctypes.POINTER(sa_block_io)] + [c_void_p] * 5 + [c_int] * 6 + [c_float, c_void_p]
_RECURRENT_ARGS = [c_void_p] * 10 + [c_int] * 7 + [c_float, c_int, c_void_p]
_RECURRENT_VAR_ARGS = [c_void_p] * 10 + [c_int] * 7 + [c_float, c_void_p, c_void_p]
_SIGNATURES = {
    "sa_last_error": (c_char_p, []),
    "sa_version": (c_int, []),
    "gdn_decode_step": (c_int, _RECURRENT_ARGS),
    "kda_decode_step": (c_int, _RECURRENT_ARGS),
    "gdn_decode_step_var": (c_int, _RECURRENT_VAR_ARGS),
    "kda_decode_step_var": (c_int, _RECURRENT_VAR_ARGS),
    "gdn_chunk_steps": (c_int, _RECURRENT_ARGS),
    "kda_chunk_steps": (c_int, _RECURRENT_ARGS),
    "gdn_block_decode": (c_int, _BLOCK_ARGS),
    "kda_block_decode": (c_int, _BLOCK_ARGS),
    "kv_append": (c_int, [c_void_p] * 4 + [c_int, c_void_p, c_int, c_void_p] + [c_int] * 5 + [c_void_p]),
    "attn_decode_workspace_bytes": (c_size_t, [c_int] * 7),
    "attn_decode": (c_int, [c_void_p] * 3 + [c_int, c_void_p, c_int, c_void_p, c_void_p, c_int, c_void_p] + [c_int] * 8
                    + [c_float, c_void_p, c_size_t, c_void_p]),
    "attn_decode_static_max_bytes": (c_size_t, []),
    "attn_decode_static": (c_int, [c_void_p] * 3 + [c_int, c_void_p, c_int, c_void_p, c_void_p, c_int, c_void_p] + [c_int] * 8
                           + [c_float, c_void_p]),
    "placement_plan_create": (c_int, [ctypes.POINTER(c_char_p), c_int, c_int, ctypes.POINTER(c_int32), c_int,
                                      ctypes.POINTER(c_void_p)]),
    "placement_plan_destroy": (None, [c_void_p]),
    "placement_plan_count": (c_int, [c_void_p, c_int, c_char]),
    "placement_workspace_bytes": (c_size_t, [c_void_p, ctypes.POINTER(sa_shapes), c_int, c_int, c_int]),
    "placement_decode": (c_int, [c_void_p, ctypes.POINTER(sa_layer_io), ctypes.POINTER(sa_shapes), c_int, c_int, c_float,
                                 c_float, c_void_p, c_size_t, c_void_p]),
    "sa_pool_create": (c_int, [c_int, ctypes.POINTER(sa_shapes), c_int, ctypes.POINTER(c_void_p)]),
    "sa_pool_destroy": (None, [c_void_p]),
    "sa_pool_page_bytes": (c_size_t, [c_void_p]),
    "sa_pool_tokens_per_page": (c_int, [c_void_p]),
    "sa_pool_kv_id_stride": (c_int, [c_void_p]),
    "sa_pool_kernel_pages": (c_int, [c_void_p]),
    "sa_pool_free_pages": (c_int, [c_void_p]),
    "sa_pool_seq_create": (c_int, [c_void_p, c_char_p, ctypes.POINTER(c_int)]),
    "sa_pool_seq_reserve": (c_int, [c_void_p, c_int, c_int, c_int, c_int]),
    "sa_pool_seq_free": (c_int, [c_void_p, c_int]),
    "sa_pool_seq_pages": (c_int, [c_void_p, c_int]),
    "sa_pool_layer_tables": (c_int, [c_void_p, ctypes.POINTER(c_int32), c_int, c_int, c_void_p, c_int, c_void_p]),
    "sa_prof_enable": (None, [c_int]),
    "sa_prof_read": (c_int, [c_int, ctypes.POINTER(c_int), ctypes.POINTER(c_float), ctypes.POINTER(c_float), c_int]),
    "sa_copy_bytes": (c_int, [c_void_p, c_void_p, c_size_t, c_void_p]),
    "sa_stream_tiles": (c_int, [c_int, c_void_p, c_int, c_void_p]),
    "sa_state_tile_bytes": (c_size_t, [c_int, c_int]),
    "sa_state_pack": (c_int, [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p]),
    "sa_state_unpack": (c_int, [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p]),
}
EXPORTS = tuple(_SIGNATURES)

_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2604_19877_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s is missing: build it with `python -m paper_2604_19877_amd.build`" % LIB_PATH)
        # PyTorch ships its own HIP runtime; it must be in the process before this library is
        # loaded so that both resolve to the same runtime (two runtimes cannot share the device).
        import torch  # noqa: F401
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status):
    if status != SA_OK:
        raise SaError(status, lib().sa_last_error().decode())


def sa_last_error() -> str:
    return lib().sa_last_error().decode()


def sa_version() -> int:
    return lib().sa_version()


def _recurrent(fn, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
               n_commit, stream):
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(alpha), _ptr(beta), _ptr(state_in), _ptr(state_out), _ptr(out),
              _ptr(slot_idx), _ptr(req_idx), n_req, B, T, H, Hk, dk, dv, scale, n_commit, _stream(stream)))


def gdn_decode_step(q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
                    n_commit, stream=None):
    _recurrent(lib().gdn_decode_step, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
               Hk, dk, dv, scale, n_commit, stream)


def kda_decode_step(q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
                    n_commit, stream=None):
    _recurrent(lib().kda_decode_step, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
               Hk, dk, dv, scale, n_commit, stream)


def gdn_decode_step_var(q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
                        n_commit_rows, stream=None):
    _check(lib().gdn_decode_step_var(_ptr(q), _ptr(k), _ptr(v), _ptr(alpha), _ptr(beta), _ptr(state_in), _ptr(state_out),
                                     _ptr(out), _ptr(slot_idx), _ptr(req_idx), n_req, B, T, H, Hk, dk, dv, scale,
                                     _ptr(n_commit_rows), _stream(stream)))


def kda_decode_step_var(q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
                        n_commit_rows, stream=None):
    _check(lib().kda_decode_step_var(_ptr(q), _ptr(k), _ptr(v), _ptr(alpha), _ptr(beta), _ptr(state_in), _ptr(state_out),
                                     _ptr(out), _ptr(slot_idx), _ptr(req_idx), n_req, B, T, H, Hk, dk, dv, scale,
                                     _ptr(n_commit_rows), _stream(stream)))


def gdn_chunk_steps(q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
                    n_commit=None, stream=None):
    _recurrent(lib().gdn_chunk_steps, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
               Hk, dk, dv, scale, T if n_commit is None else n_commit, stream)


def kda_chunk_steps(q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv, scale,
                    n_commit=None, stream=None):
    _recurrent(lib().kda_chunk_steps, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
               Hk, dk, dv, scale, T if n_commit is None else n_commit, stream)


def make_block_io(**kw):
    """Fills an sa_block_io from tensors / numbers given by field name."""
    io = sa_block_io()
    for name, _ in sa_block_io._fields_:
        val = kw.get(name)
        if name in ("conv_taps", "gate_act"):
            setattr(io, name, int(val or 0))
        elif name == "norm_eps":
            io.norm_eps = float(val or 0.0)
        else:
            setattr(io, name, _ptr(val))
    return io


def gdn_block_decode(io, state_in, state_out, out, slot_idx, req_idx, n_req, B, H, Hk, dk, dv, scale, stream=None):
    _check(lib().gdn_block_decode(ctypes.byref(io), _ptr(state_in), _ptr(state_out), _ptr(out), _ptr(slot_idx), _ptr(req_idx),
                                  n_req, B, H, Hk, dk, dv, scale, _stream(stream)))


def kda_block_decode(io, state_in, state_out, out, slot_idx, req_idx, n_req, B, H, Hk, dk, dv, scale, stream=None):
    _check(lib().kda_block_decode(ctypes.byref(io), _ptr(state_in), _ptr(state_out), _ptr(out), _ptr(slot_idx), _ptr(req_idx),
                                  n_req, B, H, Hk, dk, dv, scale, _stream(stream)))


def kv_append(k_new, v_new, kpool, vpool, n_pages, page_table, max_pages, positions, B, T, Hkv, D, page_size, stream=None):
    _check(lib().kv_append(_ptr(k_new), _ptr(v_new), _ptr(kpool), _ptr(vpool), n_pages, _ptr(page_table), max_pages,
                           _ptr(positions), B, T, Hkv, D, page_size, _stream(stream)))


def attn_decode_workspace_bytes(n_req, T, Hq, Hkv, D, max_seq_len, window) -> int:
    return lib().attn_decode_workspace_bytes(n_req, T, Hq, Hkv, D, max_seq_len, window)


def attn_decode(q, kpool, vpool, n_pages, page_table, max_pages, seq_lens, req_idx, n_req, out, B, T, Hq, Hkv, D,
                page_size, max_seq_len, window, scale, workspace, workspace_bytes, stream=None):
    _check(lib().attn_decode(_ptr(q), _ptr(kpool), _ptr(vpool), n_pages, _ptr(page_table), max_pages, _ptr(seq_lens),
                             _ptr(req_idx), n_req, _ptr(out), B, T, Hq, Hkv, D, page_size, max_seq_len, window, scale,
                             _ptr(workspace), workspace_bytes, _stream(stream)))


def attn_decode_static_max_bytes() -> int:
    return lib().attn_decode_static_max_bytes()


def attn_decode_static(q, kpool, vpool, n_pages, page_table, max_pages, seq_lens, req_idx, n_req, out, B, T, Hq, Hkv, D,
                       page_size, max_seq_len, window, scale, stream=None):
    _check(lib().attn_decode_static(_ptr(q), _ptr(kpool), _ptr(vpool), n_pages, _ptr(page_table), max_pages, _ptr(seq_lens),
                                    _ptr(req_idx), n_req, _ptr(out), B, T, Hq, Hkv, D, page_size, max_seq_len, window, scale,
                                    _stream(stream)))


def placement_plan_create(placements, placement_id):
    """placements: list of str; placement_id: sequence of ints (host).  Returns an opaque plan handle."""
    n = len(placements)
    L = len(placements[0]) if n else 0
    strings = (c_char_p * max(n, 1))(*[s.encode() for s in placements])
    ids = (c_int32 * max(len(placement_id), 1))(*[int(x) for x in placement_id])
    plan = c_void_p()
    _check(lib().placement_plan_create(strings, n, L, ids, len(placement_id), ctypes.byref(plan)))
    return plan


def placement_plan_destroy(plan):
    lib().placement_plan_destroy(plan)


def placement_plan_count(plan, layer, mixer) -> int:
    return lib().placement_plan_count(plan, layer, mixer.encode())


def placement_workspace_bytes(plan, shapes, T, max_seq_len, window) -> int:
    return lib().placement_workspace_bytes(plan, ctypes.byref(shapes), T, max_seq_len, window)


def make_layer_io(**kw):
    """Fills an sa_layer_io from tensors / ints given by field name; missing fields are NULL / 0."""
    io = sa_layer_io()
    for name, _ in sa_layer_io._fields_:
        val = kw.get(name)
        if name in ("n_pages", "max_pages", "max_seq_len"):
            setattr(io, name, int(val or 0))
        else:
            setattr(io, name, _ptr(val))
    return io


def placement_decode(plan, io, shapes, T, window, attn_scale, rec_scale, workspace, workspace_bytes, stream=None):
    """io: a ctypes array (sa_layer_io * L) or a list of sa_layer_io."""
    if isinstance(io, (list, tuple)):
        io = (sa_layer_io * len(io))(*io)
    _check(lib().placement_decode(plan, io, ctypes.byref(shapes), T, window, attn_scale, rec_scale, _ptr(workspace),
                                  workspace_bytes, _stream(stream)))


def sa_pool_create(n_pages, shapes, n_layers):
    pool = c_void_p()
    _check(lib().sa_pool_create(n_pages, ctypes.byref(shapes), n_layers, ctypes.byref(pool)))
    return pool


def sa_pool_destroy(pool):
    lib().sa_pool_destroy(pool)


def sa_pool_page_bytes(pool) -> int:
    return lib().sa_pool_page_bytes(pool)


def sa_pool_tokens_per_page(pool) -> int:
    return lib().sa_pool_tokens_per_page(pool)


def sa_pool_kv_id_stride(pool) -> int:
    return lib().sa_pool_kv_id_stride(pool)


def sa_pool_kernel_pages(pool) -> int:
    return lib().sa_pool_kernel_pages(pool)


def sa_pool_free_pages(pool) -> int:
    return lib().sa_pool_free_pages(pool)


def sa_pool_seq_create(pool, placement) -> int:
    seq = c_int(-1)
    _check(lib().sa_pool_seq_create(pool, placement.encode(), ctypes.byref(seq)))
    return seq.value


def sa_pool_seq_reserve(pool, seq_id, length, window, slack=0):
    _check(lib().sa_pool_seq_reserve(pool, seq_id, length, window, slack))


def sa_pool_seq_free(pool, seq_id):
    _check(lib().sa_pool_seq_free(pool, seq_id))


def sa_pool_seq_pages(pool, seq_id) -> int:
    return lib().sa_pool_seq_pages(pool, seq_id)


def sa_pool_layer_tables(pool, seq_ids, layer, max_pages):
    """Returns (page_table int32 [B,max_pages], slot int32 [B]) as numpy arrays (host)."""
    import numpy as np
    B = len(seq_ids)
    ids = (c_int32 * max(B, 1))(*[int(x) for x in seq_ids])
    table = np.empty((B, max_pages), dtype=np.int32)
    slot = np.empty(B, dtype=np.int32)
    _check(lib().sa_pool_layer_tables(pool, ids, B, layer, table.ctypes.data, max_pages, slot.ctypes.data))
    return table, slot


def sa_prof_enable(on):
    lib().sa_prof_enable(int(bool(on)))


def sa_prof_read(kernel, capacity=0):
    """Returns (n_launches, total_ms) or, with capacity > 0, (n_launches, total_ms, [ms of each launch])."""
    n, ms = c_int(0), c_float(0.0)
    each = (c_float * capacity)() if capacity > 0 else None
    _check(lib().sa_prof_read(kernel, ctypes.byref(n), ctypes.byref(ms), each, capacity))
    if capacity > 0:
        return n.value, ms.value, list(each)[:min(n.value, capacity)]
    return n.value, ms.value


def sa_copy_bytes(src, dst, n_bytes, stream=None):
    _check(lib().sa_copy_bytes(_ptr(src), _ptr(dst), n_bytes, _stream(stream)))


def sa_stream_tiles(kind, tiles, n_tiles, stream=None):
    _check(lib().sa_stream_tiles(kind, _ptr(tiles), n_tiles, _stream(stream)))


def sa_state_tile_bytes(dk, dv) -> int:
    return lib().sa_state_tile_bytes(dk, dv)


def sa_state_pack(rowmajor, tiles, n_tiles, dk, dv, stream=None):
    _check(lib().sa_state_pack(_ptr(rowmajor), _ptr(tiles), n_tiles, dk, dv, _stream(stream)))


def sa_state_unpack(tiles, rowmajor, n_tiles, dk, dv, stream=None):
    _check(lib().sa_state_unpack(_ptr(tiles), _ptr(rowmajor), n_tiles, dk, dv, _stream(stream)))
