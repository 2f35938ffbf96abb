"""Byte-level reference for the library's in-page KV layout (test infrastructure only).

The paged cache keeps 16-token pages (the paper's serving stack pads per-layer state to a common
page size, Section 6 "Heterogeneous state"; it fixes no in-page order, so the order is this
library's own and is stated in include/samixers.h).  Per (page, kv head) there is one 4 KiB K block
and one 4 KiB V block of bf16:

  K block: [D/8 chunks][16 tokens][8 dims]     element (token j, dim d) at ((d//8)*16 + j)*8 + d%8
  V block: [D/16 blocks][4 token groups][16 dims][4 tokens]
                                               element (j, d) at (((d//16)*4 + j//4)*16 + d%16)*4 + j%4

Pools are [n_pages][Hkv][16*D] uint16.  The functions below move bf16 bit patterns only; there is
no arithmetic to get wrong beyond the index formulas, which tests pin by spot values and round trip.
"""
from __future__ import annotations

import numpy as np

PAGE = 16


def k_offset(j: int, d: int) -> int:
    return ((d // 8) * PAGE + j) * 8 + d % 8


def v_offset(j: int, d: int) -> int:
    return (((d // 16) * 4 + j // 4) * 16 + d % 16) * 4 + j % 4


def kv_append(k_new, v_new, kpool, vpool, page_table, positions):
    """Write T new tokens per sequence.  k_new, v_new uint16 [B,T,Hkv,D]; token i of sequence b goes
    to position positions[b] + i.  Pools uint16 [n_pages,Hkv,16*D] are modified in place."""
    B, T, Hkv, D = k_new.shape
    for b in range(B):
        for i in range(T):
            pos = int(positions[b]) + i
            page = int(page_table[b][pos // PAGE])
            j = pos % PAGE
            for g in range(Hkv):
                for d in range(D):
                    kpool[page, g, k_offset(j, d)] = k_new[b, i, g, d]
                    vpool[page, g, v_offset(j, d)] = v_new[b, i, g, d]


def _index_maps(D: int):
    jj, dd = np.meshgrid(np.arange(PAGE), np.arange(D), indexing="ij")
    kmap = ((dd // 8) * PAGE + jj) * 8 + dd % 8
    vmap = (((dd // 16) * 4 + jj // 4) * 16 + dd % 16) * 4 + jj % 4
    return kmap, vmap


def to_logical(kpool_phys, vpool_phys, D: int):
    """Physical pools [n,Hkv,16*D] -> logical pools [n,Hkv,16,D] (vectorised gather of the maps above)."""
    kmap, vmap = _index_maps(D)
    return np.asarray(kpool_phys)[..., kmap], np.asarray(vpool_phys)[..., vmap]


def to_physical(kpool_log, vpool_log):
    """Logical pools [n,Hkv,16,D] -> physical pools [n,Hkv,16*D]."""
    n, Hkv, _, D = kpool_log.shape
    kmap, vmap = _index_maps(D)
    kp = np.empty((n, Hkv, PAGE * D), dtype=kpool_log.dtype)
    vp = np.empty((n, Hkv, PAGE * D), dtype=vpool_log.dtype)
    kp[..., kmap] = kpool_log
    vp[..., vmap] = vpool_log
    return kp, vp
