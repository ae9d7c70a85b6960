"""Pins for the CPU oracle: what the paper and the arithmetic fix, checked
without reference to the oracle's own formulas.

 1. brute force over dict-addressed pools on tiny inputs (tests/bruteforce.py)
 2. round trip: unpack(pack(S)) read through the receiver's table == S read
    through the sender's (the receiver "recovers the bytes to desired discrete
    blocks", sections 1 and 2.2.3)
 3. closed-form size (section 2.1) and the paper's printed GPT-3 numbers
 4. bytes outside the live slots of listed pages are never written
 5. coordinate stamps: indexing checked independently of copying
 6. reduction to numpy.take / numpy.transpose on identity block tables
 7. algebra: convert == unpack o pack; a whole-range buffer is the per-layer
    buffers placed at `segment` offsets (section 3.6: per-layer or whole-model
    transfer by different offsets and lengths); permuting the batch permutes
    buffer segments and leaves the destination image unchanged
"""
import os

import numpy as np
import pytest

from oracle import kvxo
from tests import bruteforce as bf

LM, PM = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_tables(rng, seq_lens, P, num_pages, *, unique, extra=0):
    """CSR block table; `unique` = no page used twice (a receiver must not be
    asked to write one page from two places).  `extra` appends unused ids."""
    need = [(int(n) + P - 1) // P for n in seq_lens]
    if unique:
        perm = rng.permutation(num_pages)
        assert sum(need) + extra * len(seq_lens) <= num_pages
        it = iter(perm)
        rows = [[int(next(it)) for _ in range(k + extra)] for k in need]
    else:
        rows = [[int(x) for x in rng.integers(0, num_pages, size=k + extra)] for k in need]
    offs = np.zeros(len(seq_lens) + 1, dtype=np.uint64)
    offs[1:] = np.cumsum([len(x) for x in rows])
    ids = np.array([x for row in rows for x in row], dtype=np.uint32)
    return ids, offs


def rand_pool(rng, pool: kvxo.Pool):
    return rng.integers(0, 256, size=pool.nbytes, dtype=np.uint8)


# ---------------------------------------------------------------- 1. brute force
TINY = []
for L, H, D, e in [(1, 1, 3, 1), (2, 2, 4, 2), (2, 1, 8, 1)]:
    for Ps, Pd in [(1, 1), (2, 3), (3, 2), (4, 4), (4, 1), (1, 4), (3, 4)]:
        for ls, ld in [(LM, LM), (LM, PM), (PM, LM), (PM, PM)]:
            TINY.append((L, H, D, e, Ps, Pd, ls, ld))


# page-internal arrangements (0 rows, 1 head-major, 2 token axis inside 16-byte dim groups, 3 token axis
# innermost element by element) on either side
INNER = []
for H, D, e in [(2, 16, 1), (3, 8, 2), (1, 8, 4)]:
    for Ps, Pd in [(4, 4), (2, 3), (4, 1), (3, 8)]:
        for (ls, ins), (ld, ind) in [((LM, 1), (LM, 0)), ((LM, 0), (PM, 2)), ((PM, 2), (LM, 1)),
                                      ((PM, 1), (PM, 1)), ((LM, 2), (LM, 2)), ((LM, 0), (LM, 1)),
                                      ((LM, 0), (LM, 3)), ((PM, 3), (LM, 0)), ((LM, 3), (PM, 3)),
                                      ((PM, 2), (LM, 3)), ((LM, 3), (LM, 1))]:
            INNER.append((2, H, D, e, Ps, Pd, ls, ld, ins, ind))
# token-innermost pages whose head dimension is not a multiple of 16 bytes (nothing in that arrangement needs it)
INNER += [(2, 2, 3, 2, 4, 3, LM, PM, 3, 0), (1, 1, 5, 1, 3, 3, PM, LM, 0, 3), (2, 3, 3, 4, 2, 5, LM, LM, 3, 3)]


@pytest.mark.parametrize("L,H,D,e,Ps,Pd,ls,ld,ins,ind", INNER)
def test_bruteforce_tiny_inner_arrangements(L, H, D, e, Ps, Pd, ls, ld, ins, ind):
    test_bruteforce_tiny(L, H, D, e, Ps, Pd, ls, ld, ins, ind)


@pytest.mark.parametrize("L,H,D,e,Ps,Pd,ls,ld", TINY)
def test_bruteforce_tiny(L, H, D, e, Ps, Pd, ls, ld, ins=0, ind=0):
    rng = np.random.default_rng(hash((L, H, D, e, Ps, Pd, ls, ld, ins, ind)) & 0xFFFFFFFF)
    P = max(Ps, Pd)
    lens = np.array([0, 1, P - 1, P, P + 1, 2 * P, 2 * P + 1, int(rng.integers(0, 5 * P))],
                    dtype=np.uint32)
    rng.shuffle(lens)
    row = H * D * e
    NPs, NPd = 40, 64
    ps = kvxo.Pool(L, H, D, e, Ps, NPs, ls, inner=ins)
    pd = kvxo.Pool(L, H, D, e, Pd, NPd, ld, inner=ind)
    ids_s, offs_s = make_tables(rng, lens, Ps, NPs, unique=False, extra=1)   # shared source pages allowed
    ids_d, offs_d = make_tables(rng, lens, Pd, NPd, unique=True, extra=1)
    bs, bd = kvxo.Batch(lens, ids_s, offs_s), kvxo.Batch(lens, ids_d, offs_d)
    src = rand_pool(rng, ps)
    src_d = bf.flat_to_dict(src, L, NPs, Ps, row, ls, ins, H, e)

    for l0, l1 in [(0, L), (L - 1, L), (0, 0)]:
        want = bf.pack(src_d, Ps, lens, ids_s, offs_s, l0, l1)
        assert kvxo.total_bytes(ps, bs, l0, l1) == len(want)
        buf = np.full(len(want) + 7, 0xA5, dtype=np.uint8)
        kvxo.pack(ps, bs, l0, l1, src, buf)
        assert bytes(buf[:len(want)]) == want
        assert (buf[len(want):] == 0xA5).all()

        canary = rng.integers(0, 256, size=pd.nbytes, dtype=np.uint8)
        dst = canary.copy()
        kvxo.unpack(pd, bd, l0, l1, buf, dst)
        dst_d = bf.flat_to_dict(canary, L, NPd, Pd, row, ld, ind, H, e)
        bf.unpack(want, row, dst_d, Pd, lens, ids_d, offs_d, l0, l1)
        assert np.array_equal(dst, bf.dict_to_flat(dst_d, L, NPd, Pd, row, ld, ind, H, e))

        dst2 = canary.copy()
        kvxo.convert(ps, bs, pd, bd, l0, l1, src, dst2)
        dst2_d = bf.flat_to_dict(canary, L, NPd, Pd, row, ld, ind, H, e)
        bf.convert(src_d, Ps, ids_s, offs_s, dst2_d, Pd, ids_d, offs_d, lens, l0, l1)
        assert np.array_equal(dst2, bf.dict_to_flat(dst2_d, L, NPd, Pd, row, ld, ind, H, e))


# ---------------------------------------------------------------- 3. closed form + paper numbers
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "kv_size_paper.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                L, hid, e, n, val, unit, tol = line.split()
                rows.append((int(L), int(hid), int(e), int(n), float(val), unit, float(tol)))
    return rows


@pytest.mark.parametrize("L,hid,e,n,val,unit,tol", _golden_rows())
def test_paper_kv_sizes(L, hid, e, n, val, unit, tol):
    scale = {"MiB": 2 ** 20, "GiB": 2 ** 30}[unit]
    heads, dim = 96, hid // 96
    pool = kvxo.Pool(L, heads, dim, e, 16, 1)
    batch = kvxo.Batch([n], np.zeros((n + 15) // 16, np.uint32), [0, (n + 15) // 16])
    got = kvxo.total_bytes(pool, batch, 0, L)
    assert abs(got - val * scale) <= tol * val * scale
    # a single layer is 1/L of it, and so is that layer's segment length
    assert kvxo.total_bytes(pool, batch, 3, 4) * L == got
    assert kvxo.segment(pool, batch, 0, L, 0, 5) == (5 * got // L, got // L)


@pytest.mark.parametrize("seed", range(6))
def test_closed_form_and_segments_tile_buffer(seed):
    rng = np.random.default_rng(seed)
    L, H, D, e, P = int(rng.integers(1, 7)), int(rng.integers(1, 9)), 16 * int(rng.integers(1, 9)), \
        int(rng.choice([1, 2])), int(rng.choice([1, 16, 128]))
    R = int(rng.integers(1, 40))
    lens = rng.integers(0, 700, size=R).astype(np.uint32)
    ids, offs = make_tables(rng, lens, P, 40000, unique=True)
    pool, batch = kvxo.Pool(L, H, D, e, P, 40000), kvxo.Batch(lens, ids, offs)
    l0 = int(rng.integers(0, L))
    l1 = int(rng.integers(l0, L + 1))
    total = kvxo.total_bytes(pool, batch, l0, l1)
    assert total == (l1 - l0) * 2 * H * D * e * int(lens.sum())
    cursor = 0
    for r in range(R):
        for l in range(l0, l1):
            off, ln = kvxo.segment(pool, batch, l0, l1, r, l)
            assert off == cursor and ln == 2 * int(lens[r]) * H * D * e
            cursor += ln
    assert cursor == total
    with pytest.raises(ValueError):
        kvxo.segment(pool, batch, l0, l1, R, l0)
    with pytest.raises(ValueError):
        kvxo.segment(pool, batch, l0, l1, 0, l1)


# ---------------------------------------------------------------- 2, 4, 5. round trip, canary, stamps
def stamp_pool(pool: kvxo.Pool):
    """Each row's first 16 bytes encode its own (layer, kv, page, slot) and the
    remaining bytes a position-dependent pattern, written through numpy N-d
    indexing of an array shaped like the layout's name."""
    L, NP, P, row = pool.num_layers, pool.num_pages, pool.page_tokens, pool.row
    assert row >= 16
    l, c, p, s = np.meshgrid(np.arange(L), np.arange(2), np.arange(NP), np.arange(P), indexing="ij")
    rows = np.zeros((L, 2, NP, P, row), dtype=np.uint8)
    hdr = np.stack([l, c, p, s], axis=-1).astype("<u4").view(np.uint8).reshape(L, 2, NP, P, 16)
    rows[..., :16] = hdr
    j = np.arange(16, row, dtype=np.int64)
    rows[..., 16:] = ((l + 3 * c + 7 * p + 11 * s)[..., None] + 13 * j) & 0xFF
    if pool.layout == PM:
        rows = rows.transpose(2, 0, 1, 3, 4)
    return np.ascontiguousarray(rows).reshape(-1)


def read_row(flat, pool: kvxo.Pool, l, c, p, s):
    L, NP, P, row = pool.num_layers, pool.num_pages, pool.page_tokens, pool.row
    if pool.layout == LM:
        return flat.reshape(L, 2, NP, P, row)[l, c, p, s]
    return flat.reshape(NP, L, 2, P, row)[p, l, c, s]


@pytest.mark.parametrize("ls,ld,Ps,Pd", [(LM, LM, 16, 16), (LM, PM, 128, 16), (PM, LM, 16, 128),
                                          (PM, PM, 8, 24), (LM, LM, 5, 7)])
def test_roundtrip_stamps_and_canaries(ls, ld, Ps, Pd):
    rng = np.random.default_rng(Ps * 131 + Pd)
    L, H, D, e = 3, 2, 16, 2
    lens = np.array([0, 1, 257, 128, 300, 15, 16, 17], dtype=np.uint32)
    ps = kvxo.Pool(L, H, D, e, Ps, 2 * int(sum((n + Ps - 1) // Ps for n in lens)) + 3, ls)
    pd = kvxo.Pool(L, H, D, e, Pd, 2 * int(sum((n + Pd - 1) // Pd for n in lens)) + 3, ld)
    ids_s, offs_s = make_tables(rng, lens, Ps, ps.num_pages, unique=True)
    ids_d, offs_d = make_tables(rng, lens, Pd, pd.num_pages, unique=True)
    bs, bd = kvxo.Batch(lens, ids_s, offs_s), kvxo.Batch(lens, ids_d, offs_d)
    src = stamp_pool(ps)
    buf = np.full(kvxo.total_bytes(ps, bs, 0, L) + 64, 0xEE, dtype=np.uint8)
    kvxo.pack(ps, bs, 0, L, src, buf)
    assert (buf[-64:] == 0xEE).all()

    for how in ("unpack", "convert"):
        dst = np.full(pd.nbytes, 0xC3, dtype=np.uint8)
        if how == "unpack":
            kvxo.unpack(pd, bd, 0, L, buf, dst)
        else:
            kvxo.convert(ps, bs, pd, bd, 0, L, src, dst)
        live = np.zeros(pd.nbytes // pd.row, dtype=bool).reshape(
            (L, 2, pd.num_pages, Pd) if ld == LM else (pd.num_pages, L, 2, Pd))
        for r, n in enumerate(lens):
            ts, td = bf.table(ids_s, offs_s, r), bf.table(ids_d, offs_d, r)
            for l in range(L):
                for c in range(2):
                    for t in range(int(n)):
                        got = read_row(dst, pd, l, c, td[t // Pd], t % Pd)
                        # the stamp names the source coordinates it must have come from
                        assert tuple(got[:16].view("<u4")) == (l, c, ts[t // Ps], t % Ps)
                        assert np.array_equal(got, read_row(src, ps, l, c, ts[t // Ps], t % Ps))
                        if ld == LM:
                            live[l, c, td[t // Pd], t % Pd] = True
                        else:
                            live[td[t // Pd], l, c, t % Pd] = True
        dead = ~np.repeat(live.reshape(-1), pd.row)
        assert (dst[dead] == 0xC3).all(), "a byte outside the live slots of listed pages was written"
        assert live.sum() == L * 2 * int(lens.sum())


# ---------------------------------------------------------------- 6. reduction to library routines
@pytest.mark.parametrize("seed", range(3))
def test_pack_reduces_to_numpy_take(seed):
    rng = np.random.default_rng(100 + seed)
    L, H, D, e, P, NP = 3, 2, 16, 2, 8, 50
    pool = kvxo.Pool(L, H, D, e, P, NP, LM)
    src = rand_pool(rng, pool)
    bt = rng.permutation(NP)[:12].astype(np.uint32)
    n = 12 * P - int(rng.integers(0, P))           # ragged tail handled by slicing the take
    batch = kvxo.Batch([n], bt, [0, 12])
    buf = np.zeros(kvxo.total_bytes(pool, batch, 0, L), dtype=np.uint8)
    kvxo.pack(pool, batch, 0, L, src, buf)
    want = np.take(src.reshape(L, 2, NP, P, pool.row), bt, axis=2).reshape(L, 2, -1, pool.row)[:, :, :n]
    assert np.array_equal(buf, want.reshape(-1))


def test_convert_reduces_to_transpose():
    rng = np.random.default_rng(7)
    L, H, D, e, P, NP = 4, 1, 16, 1, 4, 9
    ps, pd = kvxo.Pool(L, H, D, e, P, NP, LM), kvxo.Pool(L, H, D, e, P, NP, PM)
    src = rand_pool(rng, ps)
    ident = np.arange(NP, dtype=np.uint32)
    b = kvxo.Batch([NP * P], ident, [0, NP])
    dst = np.zeros(pd.nbytes, dtype=np.uint8)
    kvxo.convert(ps, b, pd, b, 0, L, src, dst)
    want = np.transpose(src.reshape(L, 2, NP, P, ps.row), (2, 0, 1, 3, 4))
    assert np.array_equal(dst, np.ascontiguousarray(want).reshape(-1))
    back = np.zeros(ps.nbytes, dtype=np.uint8)
    kvxo.convert(pd, b, ps, b, 0, L, dst, back)
    assert np.array_equal(back, src)


@pytest.mark.parametrize("e,D", [(2, 16), (1, 32), (4, 8)])
def test_inner_arrangements_reduce_to_transposes(e, D):
    """Identity block tables, full pages: converting between page-internal
    arrangements is a plain axis permutation of the page."""
    rng = np.random.default_rng(8 + e)
    L, H, P, NP = 2, 3, 4, 5
    x = 16 // e
    rows = kvxo.Pool(L, H, D, e, P, NP, LM, inner=0)
    heads = kvxo.Pool(L, H, D, e, P, NP, LM, inner=1)
    split = kvxo.Pool(L, H, D, e, P, NP, LM, inner=2)
    tinner = kvxo.Pool(L, H, D, e, P, NP, LM, inner=3)
    src = rand_pool(rng, rows)
    b = kvxo.Batch([NP * P], np.arange(NP, dtype=np.uint32), [0, NP])
    as_elems = src.reshape(L, 2, NP, P, H, D // x, x * e)           # [token][head][dim/x][x]
    out = np.zeros(rows.nbytes, dtype=np.uint8)
    kvxo.convert(rows, b, heads, b, 0, L, src, out)
    assert np.array_equal(out, np.ascontiguousarray(as_elems.transpose(0, 1, 2, 4, 3, 5, 6)).reshape(-1))
    kvxo.convert(rows, b, split, b, 0, L, src, out)
    want_split = np.ascontiguousarray(as_elems.transpose(0, 1, 2, 4, 5, 3, 6)).reshape(-1)
    assert np.array_equal(out, want_split)
    back = np.zeros(rows.nbytes, dtype=np.uint8)
    kvxo.convert(split, b, rows, b, 0, L, want_split, back)
    assert np.array_equal(back, src)
    # token axis innermost: [token][head][dim][e] -> [head][dim][token][e], a transposed page
    by_elem = src.reshape(L, 2, NP, P, H, D, e)
    want_tinner = np.ascontiguousarray(by_elem.transpose(0, 1, 2, 4, 5, 3, 6)).reshape(-1)
    kvxo.convert(rows, b, tinner, b, 0, L, src, out)
    assert np.array_equal(out, want_tinner)
    kvxo.convert(split, b, tinner, b, 0, L, want_split, out)
    assert np.array_equal(out, want_tinner)
    kvxo.convert(tinner, b, rows, b, 0, L, want_tinner, back)
    assert np.array_equal(back, src)
    # pack out of any arrangement gives the same buffer as out of rows
    bufs = []
    for pool, data in ((rows, src), (split, want_split), (tinner, want_tinner)):
        buf = np.zeros(kvxo.total_bytes(pool, b, 0, L), dtype=np.uint8)
        kvxo.pack(pool, b, 0, L, data, buf)
        bufs.append(buf)
    assert np.array_equal(bufs[0], bufs[1]) and np.array_equal(bufs[0], bufs[2])
    with pytest.raises(ValueError):                                  # 16-byte groups need head_dim*e % 16 == 0
        kvxo.pack(kvxo.Pool(1, 1, 4, 2, 4, 2, LM, inner=2), kvxo.Batch([1], [0], [0, 1]), 0, 1,
                  np.zeros(64, np.uint8), np.zeros(64, np.uint8))


def test_explicit_strides_match_padded_numpy_view():
    """Caller-given strides: a pool embedded in a larger, padded array."""
    rng = np.random.default_rng(11)
    L, H, D, e, P, NP = 2, 2, 8, 2, 4, 6
    row = H * D * e
    padded = rng.integers(0, 256, size=(L, 2, NP + 1, P + 2, row + 16), dtype=np.uint8)
    st = padded.strides
    pool = kvxo.Pool(L, H, D, e, P, NP, LM, stride_layer=st[0], stride_kv=st[1], stride_page=st[2],
                     stride_token=st[3])
    lens = np.array([5, 9], dtype=np.uint32)
    ids, offs = make_tables(rng, lens, P, NP, unique=True)
    batch = kvxo.Batch(lens, ids, offs)
    buf = np.zeros(kvxo.total_bytes(pool, batch, 0, L), dtype=np.uint8)
    kvxo.pack(pool, batch, 0, L, padded.reshape(-1), buf)
    rows = []
    for r, n in enumerate(lens):
        t = bf.table(ids, offs, r)
        for l in range(L):
            for c in range(2):
                for k in range(int(n)):
                    rows.append(padded[l, c, t[k // P], k % P, :row])
    assert np.array_equal(buf, np.concatenate(rows))


# ---------------------------------------------------------------- 7. algebra
def _mid_case(rng, ls=LM, ld=PM, Ps=16, Pd=4):
    L, H, D, e = 4, 2, 8, 2
    lens = rng.integers(0, 90, size=9).astype(np.uint32)
    ps = kvxo.Pool(L, H, D, e, Ps, 80, ls)
    pd = kvxo.Pool(L, H, D, e, Pd, 300, ld)
    ids_s, offs_s = make_tables(rng, lens, Ps, 80, unique=False)
    ids_d, offs_d = make_tables(rng, lens, Pd, 300, unique=True)
    return L, lens, ps, pd, (ids_s, offs_s), (ids_d, offs_d)


def test_convert_equals_unpack_of_pack():
    rng = np.random.default_rng(21)
    L, lens, ps, pd, ts, td = _mid_case(rng)
    bs, bd = kvxo.Batch(lens, *ts), kvxo.Batch(lens, *td)
    src = rand_pool(rng, ps)
    for l0, l1 in [(0, L), (1, 3)]:
        buf = np.zeros(kvxo.total_bytes(ps, bs, l0, l1), dtype=np.uint8)
        kvxo.pack(ps, bs, l0, l1, src, buf)
        a = np.full(pd.nbytes, 0x5A, dtype=np.uint8)
        b = a.copy()
        kvxo.unpack(pd, bd, l0, l1, buf, a)
        kvxo.convert(ps, bs, pd, bd, l0, l1, src, b)
        assert np.array_equal(a, b)


def test_whole_range_is_per_layer_ranges_at_segment_offsets():
    rng = np.random.default_rng(22)
    L, lens, ps, pd, ts, td = _mid_case(rng)
    bs = kvxo.Batch(lens, *ts)
    src = rand_pool(rng, ps)
    whole = np.zeros(kvxo.total_bytes(ps, bs, 0, L), dtype=np.uint8)
    kvxo.pack(ps, bs, 0, L, src, whole)
    rebuilt = np.zeros_like(whole)
    for l in range(L):
        part = np.zeros(kvxo.total_bytes(ps, bs, l, l + 1), dtype=np.uint8)
        kvxo.pack(ps, bs, l, l + 1, src, part)
        for r in range(len(lens)):
            o_w, n_w = kvxo.segment(ps, bs, 0, L, r, l)
            o_p, n_p = kvxo.segment(ps, bs, l, l + 1, r, l)
            assert n_w == n_p
            rebuilt[o_w:o_w + n_w] = part[o_p:o_p + n_p]
    assert np.array_equal(whole, rebuilt)


def test_batch_permutation():
    rng = np.random.default_rng(23)
    L, lens, ps, pd, (ids_s, offs_s), (ids_d, offs_d) = _mid_case(rng)
    R = len(lens)
    perm = rng.permutation(R)

    def permuted(ids, offs):
        rows = [bf.table(ids, offs, r) for r in perm]
        o = np.zeros(R + 1, dtype=np.uint64)
        o[1:] = np.cumsum([len(x) for x in rows])
        return np.array([x for row in rows for x in row], dtype=np.uint32), o

    bs, bd = kvxo.Batch(lens, ids_s, offs_s), kvxo.Batch(lens, ids_d, offs_d)
    bs2, bd2 = kvxo.Batch(lens[perm], *permuted(ids_s, offs_s)), kvxo.Batch(lens[perm], *permuted(ids_d, offs_d))
    src = rand_pool(rng, ps)
    buf = np.zeros(kvxo.total_bytes(ps, bs, 0, L), dtype=np.uint8)
    buf2 = np.zeros_like(buf)
    kvxo.pack(ps, bs, 0, L, src, buf)
    kvxo.pack(ps, bs2, 0, L, src, buf2)
    bpt = L * 2 * ps.row
    seg = {}
    cur = 0
    for r in range(R):
        seg[r] = buf[cur:cur + bpt * int(lens[r])]
        cur += bpt * int(lens[r])
    assert np.array_equal(buf2, np.concatenate([seg[int(r)] for r in perm]))
    d1 = np.full(pd.nbytes, 1, dtype=np.uint8)
    d2 = d1.copy()
    kvxo.unpack(pd, bd, 0, L, buf, d1)
    kvxo.unpack(pd, bd2, 0, L, buf2, d2)
    assert np.array_equal(d1, d2)


def test_threads_change_nothing():
    rng = np.random.default_rng(24)
    L, lens, ps, pd, ts, td = _mid_case(rng)
    bs, bd = kvxo.Batch(lens, *ts), kvxo.Batch(lens, *td)
    src = rand_pool(rng, ps)
    out = []
    for th in (1, 4):
        buf = np.zeros(kvxo.total_bytes(ps, bs, 0, L), dtype=np.uint8)
        kvxo.pack(ps, bs, 0, L, src, buf, threads=th)
        d = np.full(pd.nbytes, 9, dtype=np.uint8)
        kvxo.unpack(pd, bd, 0, L, buf, d, threads=th)
        e = np.full(pd.nbytes, 9, dtype=np.uint8)
        kvxo.convert(ps, bs, pd, bd, 0, L, src, e, threads=th)
        out.append((buf, d, e))
    for a, b in zip(*out):
        assert np.array_equal(a, b)


def test_bad_tables_are_reported():
    pool = kvxo.Pool(1, 1, 16, 1, 4, 8)
    src = np.zeros(pool.nbytes, dtype=np.uint8)
    buf = np.zeros(4096, dtype=np.uint8)
    with pytest.raises(ValueError):                       # table too short for the length
        kvxo.pack(pool, kvxo.Batch([9], [0, 1], [0, 2]), 0, 1, src, buf)
    with pytest.raises(ValueError):                       # page id outside the pool
        kvxo.pack(pool, kvxo.Batch([4], [8], [0, 1]), 0, 1, src, buf)
