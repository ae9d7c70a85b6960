"""Property tests (hypothesis, CPU only): random geometries, lengths and block
tables.  The oracle against the dict brute force; the library's host arithmetic
(totals, segments, error codes) against the oracle and against first
principles."""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

from oracle import kvxo
from paper_2408_08147_amd import kvx
from tests import bruteforce as bf

SET = dict(max_examples=60, deadline=None, suppress_health_check=[HealthCheck.too_slow])


@st.composite
def geometry(draw):
    e = draw(st.sampled_from([1, 2, 4]))
    inner_s = draw(st.sampled_from([0, 1, 2]))
    inner_d = draw(st.sampled_from([0, 1, 2]))
    x = 16 // e
    D = x * draw(st.integers(1, 2)) if (inner_s or inner_d) else draw(st.integers(1, 9))
    H = draw(st.integers(1, 3))
    L = draw(st.integers(1, 3))
    Ps, Pd = draw(st.integers(1, 6)), draw(st.integers(1, 6))
    ls, ld = draw(st.sampled_from([0, 1])), draw(st.sampled_from([0, 1]))
    lens = draw(st.lists(st.integers(0, 20), min_size=0, max_size=5))
    seed = draw(st.integers(0, 2 ** 31))
    return L, H, D, e, Ps, Pd, ls, ld, inner_s, inner_d, lens, seed


def tables(rng, lens, P, num_pages, unique, extra):
    need = [(n + P - 1) // P for n in lens]
    if unique:
        it = iter(rng.permutation(num_pages))
        rows = [[int(next(it)) for _ in range(k + extra)] for k in need]
    else:
        rows = [[int(v) for v in rng.integers(0, num_pages, size=k + extra)] for k in need]
    offs = np.zeros(len(lens) + 1, dtype=np.uint64)
    offs[1:] = np.cumsum([len(r) for r in rows])
    return np.array([v for r in rows for v in r], dtype=np.uint32), offs


@settings(**SET)
@given(geometry())
def test_oracle_equals_bruteforce(g):
    L, H, D, e, Ps, Pd, ls, ld, ins, ind, lens, seed = g
    rng = np.random.default_rng(seed)
    row = H * D * e
    lens = np.array(lens, dtype=np.uint32)
    NPs = 2 * int(sum((n + Ps - 1) // Ps + 1 for n in lens)) + 2
    NPd = 2 * int(sum((n + Pd - 1) // Pd + 1 for n in lens)) + 2
    ps = kvxo.Pool(L, H, D, e, Ps, NPs, ls, inner=ins)
    pd = kvxo.Pool(L, H, D, e, Pd, NPd, ld, inner=ind)
    ids_s, offs_s = tables(rng, lens, Ps, NPs, unique=False, extra=1)
    ids_d, offs_d = tables(rng, lens, Pd, NPd, unique=True, extra=1)
    bs, bd = kvxo.Batch(lens, ids_s, offs_s), kvxo.Batch(lens, ids_d, offs_d)
    src = rng.integers(0, 256, size=ps.nbytes, dtype=np.uint8)
    src_d = bf.flat_to_dict(src, L, NPs, Ps, row, ls, ins, H)
    l0 = int(rng.integers(0, L))
    l1 = int(rng.integers(l0, L + 1))
    want = bf.pack(src_d, Ps, lens, ids_s, offs_s, l0, l1)
    assert kvxo.total_bytes(ps, bs, l0, l1) == len(want)
    buf = np.zeros(len(want), dtype=np.uint8)
    kvxo.pack(ps, bs, l0, l1, src, buf)
    assert bytes(buf) == want
    canary = rng.integers(0, 256, size=pd.nbytes, dtype=np.uint8)
    for how in ("unpack", "convert"):
        dst = canary.copy()
        dd = bf.flat_to_dict(canary, L, NPd, Pd, row, ld, ind, H)
        if how == "unpack":
            kvxo.unpack(pd, bd, l0, l1, buf, dst)
            bf.unpack(want, row, dd, Pd, lens, ids_d, offs_d, l0, l1)
        else:
            kvxo.convert(ps, bs, pd, bd, l0, l1, src, dst)
            bf.convert(src_d, Ps, ids_s, offs_s, dd, Pd, ids_d, offs_d, lens, l0, l1)
        assert np.array_equal(dst, bf.dict_to_flat(dd, L, NPd, Pd, row, ld, ind, H))


@st.composite
def big_geometry(draw):
    H = draw(st.integers(1, 64))
    D = 16 * draw(st.integers(1, 16))
    e = draw(st.sampled_from([1, 2, 4]))
    L = draw(st.integers(1, 96))
    P = draw(st.sampled_from([1, 8, 16, 100, 128, 1024]))
    lens = draw(st.lists(st.integers(0, 200000), min_size=0, max_size=12))
    seed = draw(st.integers(0, 2 ** 31))
    return L, H, D, e, P, lens, seed


@settings(**SET)
@given(big_geometry())
def test_library_totals_and_segments(g):
    """Host-only plans at sizes up to tens of GB: 64-bit totals and segments
    equal the closed form and the oracle's, and segments tile the buffer."""
    L, H, D, e, P, lens, seed = g
    rng = np.random.default_rng(seed)
    lens = np.array(lens, dtype=np.uint32)
    need = [(int(n) + P - 1) // P for n in lens]
    NP = max(sum(need), 1)
    ids = rng.permutation(NP).astype(np.uint32)[:sum(need)]
    offs = np.concatenate([[0], np.cumsum(need)]).astype(np.uint64)
    if H * D * e * P >= 2 ** 32:
        return
    pool = kvx.pool_desc(L, H, D, e, P, NP)
    batch = kvx.BatchDesc(lens, ids, offs)
    l0 = int(rng.integers(0, L))
    l1 = int(rng.integers(l0, L + 1))
    plan = kvx.kvx_plan(pool, batch, pool, batch, l0, l1)
    row = H * D * e
    assert kvx.kvx_plan_total_bytes(plan) == (l1 - l0) * 2 * row * int(lens.astype(np.int64).sum())
    op, ob = kvxo.Pool(L, H, D, e, P, NP), kvxo.Batch(lens, ids, offs)
    cursor = 0
    for r in range(len(lens)):
        assert kvx.kvx_plan_request_segment(plan, r) == (cursor, (l1 - l0) * 2 * row * int(lens[r]))
        for l in range(l0, l1) if l1 - l0 <= 4 else (l0, l1 - 1):
            assert kvx.kvx_plan_segment(plan, r, l) == kvxo.segment(op, ob, l0, l1, r, l)
        cursor += (l1 - l0) * 2 * row * int(lens[r])
    plan.destroy()


@settings(**SET)
@given(st.integers(0, 2 ** 31), st.sampled_from(["short", "range", "dup", "ok"]))
def test_block_table_validation(seed, flaw):
    """One planted flaw in an otherwise valid receiver table is always reported
    as KVX_ERR_BLOCK_TABLE; the unflawed table is accepted."""
    rng = np.random.default_rng(seed)
    P = int(rng.choice([1, 4, 16]))
    lens = rng.integers(1, 100, size=int(rng.integers(1, 6))).astype(np.uint32)
    need = [(int(n) + P - 1) // P for n in lens]
    NP = sum(need) + 5
    ids = rng.permutation(NP).astype(np.uint32)[:sum(need)]
    offs = np.concatenate([[0], np.cumsum(need)]).astype(np.uint64)
    if flaw == "short":
        r = int(rng.integers(0, len(lens)))
        lens = lens.copy()
        lens[r] += P                                       # one page more than the table holds
    elif flaw == "range":
        ids = ids.copy()
        ids[int(rng.integers(0, len(ids)))] = NP + int(rng.integers(0, 10))
    elif flaw == "dup":
        if len(ids) < 2:
            return
        ids = ids.copy()
        i, j = rng.choice(len(ids), size=2, replace=False)
        ids[i] = ids[j]
    pool = kvx.pool_desc(2, 1, 16, 1, P, NP)
    batch = kvx.BatchDesc(lens, ids, offs)
    if flaw == "ok":
        kvx.kvx_plan(None, None, pool, batch, 0, 2).destroy()
        return
    with pytest.raises(kvx.KvxError) as e:
        kvx.kvx_plan(None, None, pool, batch, 0, 2)
    assert e.value.status == kvx.ERR_BLOCK_TABLE
    if flaw == "dup":                                      # the same table is fine on a sender
        kvx.kvx_plan(pool, batch, None, None, 0, 2).destroy()
