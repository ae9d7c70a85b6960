"""Token-by-token brute force of pack / unpack / convert over dict-addressed
pools, used to pin the C oracle on tiny inputs.

Nothing here uses byte strides or buffer offsets.  A pool is a dict keyed by
the tuple (layer, kv, page, slot) holding one token row (bytes); the transfer
buffer is the plain concatenation of rows "one after another" in the order
section 3.6 of the paper gives (per request: layers ascending, K rows then V
rows, tokens ascending).  The bridge to flat memory is numpy's own N-d
indexing on an array shaped like the layout's name.
"""
from __future__ import annotations

import numpy as np

LAYER_MAJOR, PAGE_MAJOR = 0, 1


def table(ids, offs, r):
    return [int(x) for x in ids[int(offs[r]):int(offs[r + 1])]]


def _page_view(flat: np.ndarray, L, NP, P, row, layout, inner, heads, elem=1):
    """The pool as an N-d array whose leading axes are (layer, kv, page) and
    whose page-internal axes are spelled as the arrangement's name says; the
    returned function picks one token row out of it as [head][dim] bytes."""
    lead = (L, 2, NP) if layout == LAYER_MAJOR else (NP, L, 2)
    hb = row // heads                                   # bytes of one head of one token
    if inner == 0:                                      # [token][head][dim]
        a = flat.reshape(*lead, P, row)
        pick = lambda pg, s: pg[s]
    elif inner == 1:                                    # [head][token][dim]
        a = flat.reshape(*lead, heads, P, hb)
        pick = lambda pg, s: pg[:, s, :]
    elif inner == 2:                                    # [head][dim/x][token][x], x elements = 16 bytes
        a = flat.reshape(*lead, heads, hb // 16, P, 16)
        pick = lambda pg, s: pg[:, :, s, :]
    else:                                               # [head][dim][token], elements of `elem` bytes
        a = flat.reshape(*lead, heads, hb // elem, P, elem)
        pick = lambda pg, s: pg[:, :, s, :]
    if layout == LAYER_MAJOR:
        page = lambda l, c, p: a[l, c, p]
    else:
        page = lambda l, c, p: a[p, l, c]
    return a, page, pick


def flat_to_dict(flat: np.ndarray, L, NP, P, row, layout, inner=0, heads=1, elem=1):
    _, page, pick = _page_view(flat, L, NP, P, row, layout, inner, heads, elem)
    return {(l, c, p, s): bytes(np.ascontiguousarray(pick(page(l, c, p), s)).reshape(-1))
            for l in range(L) for c in range(2) for p in range(NP) for s in range(P)}


def dict_to_flat(d: dict, L, NP, P, row, layout, inner=0, heads=1, elem=1) -> np.ndarray:
    flat = np.zeros(L * 2 * NP * P * row, dtype=np.uint8)
    a, page, pick = _page_view(flat, L, NP, P, row, layout, inner, heads, elem)
    for (l, c, p, s), v in d.items():
        tgt = pick(page(l, c, p), s)
        tgt[...] = np.frombuffer(v, dtype=np.uint8).reshape(tgt.shape)
    return a.reshape(-1)


def pack(pool: dict, P, seq_lens, ids, offs, l0, l1) -> bytes:
    out = []
    for r, n in enumerate(seq_lens):
        bt = table(ids, offs, r)
        for l in range(l0, l1):
            for c in range(2):
                for t in range(int(n)):
                    out.append(pool[(l, c, bt[t // P], t % P)])
    return b"".join(out)


def unpack(buf: bytes, row, pool: dict, P, seq_lens, ids, offs, l0, l1) -> None:
    """Consumes `buf` row by row in the same order and writes into `pool`."""
    k = 0
    for r, n in enumerate(seq_lens):
        bt = table(ids, offs, r)
        for l in range(l0, l1):
            for c in range(2):
                for t in range(int(n)):
                    pool[(l, c, bt[t // P], t % P)] = buf[k * row:(k + 1) * row]
                    k += 1
    assert k * row == len(buf)


def convert(src: dict, Ps, ids_s, offs_s, dst: dict, Pd, ids_d, offs_d, seq_lens, l0, l1) -> None:
    for r, n in enumerate(seq_lens):
        bs, bd = table(ids_s, offs_s, r), table(ids_d, offs_d, r)
        for l in range(l0, l1):
            for c in range(2):
                for t in range(int(n)):
                    dst[(l, c, bd[t // Pd], t % Pd)] = src[(l, c, bs[t // Ps], t % Ps)]
