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


def flat_to_dict(flat: np.ndarray, L, NP, P, row, layout):
    if layout == LAYER_MAJOR:
        a = flat.reshape(L, 2, NP, P, row)
        get = lambda l, c, p, s: a[l, c, p, s]
    else:
        a = flat.reshape(NP, L, 2, P, row)
        get = lambda l, c, p, s: a[p, l, c, s]
    return {(l, c, p, s): bytes(get(l, c, p, s))
            for l in range(L) for c in range(2) for p in range(NP) for s in range(P)}


def dict_to_flat(d: dict, L, NP, P, row, layout) -> np.ndarray:
    if layout == LAYER_MAJOR:
        a = np.zeros((L, 2, NP, P, row), dtype=np.uint8)
        for (l, c, p, s), v in d.items():
            a[l, c, p, s] = np.frombuffer(v, dtype=np.uint8)
    else:
        a = np.zeros((NP, L, 2, P, row), dtype=np.uint8)
        for (l, c, p, s), v in d.items():
            a[p, l, c, s] = np.frombuffer(v, dtype=np.uint8)
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
