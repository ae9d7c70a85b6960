"""Seeded random geometries on the GPU against the oracle: layouts, page arrangements, page sizes that
need not divide, shared sender pages, unused table entries, layer sub-ranges and launch knobs all drawn
together.  Deterministic: the case list is a function of the seeds below."""
import numpy as np
import pytest

from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def draw_case(seed, token_innermost=False):
    rng = np.random.default_rng(seed)
    e = int(rng.choice([1, 2, 4, 8] if token_innermost else [1, 2, 4]))
    ins, ind = int(rng.integers(0, 3)), int(rng.integers(0, 3))
    if token_innermost:      # on one side or on both; the other side keeps any of the four arrangements
        which = int(rng.integers(0, 3))
        ins, ind = (3, int(rng.integers(0, 4))) if which == 0 else ((int(rng.integers(0, 4)), 3) if which == 1 else (3, 3))
    # head_dim*e must be a multiple of 16 for the non-row arrangements, the row always
    D = int(rng.choice([16, 32, 48, 64, 128])) if (ins or ind) else int(rng.choice([8, 16, 24, 64, 128]))
    H = int(rng.integers(1, 9))
    if (H * D * e) % 16:
        H *= 2
    if (H * D * e) % 16:
        H *= 2
    L = int(rng.integers(1, 5))
    Ps = int(rng.choice([1, 2, 3, 8, 16, 33, 64, 128]))
    Pd = int(rng.choice([1, 4, 5, 16, 32, 100, 128]))
    R = int(rng.integers(0, 9))
    lens = rng.integers(0, 400, size=R).astype(np.uint32)
    if R and rng.random() < 0.5:
        lens[int(rng.integers(0, R))] = 0
    case = G.make_case(rng, L, H, D, e, lens, Ps, Pd, int(rng.integers(0, 2)), int(rng.integers(0, 2)),
                       shared_src=bool(rng.integers(0, 2)), extra=int(rng.integers(0, 3)),
                       inner_s=ins, inner_d=ind)
    l0 = int(rng.integers(0, L))
    l1 = int(rng.integers(l0, L + 1))
    launch = None
    if rng.random() < 0.6:
        launch = dict(order=int(rng.integers(0, 4)), xcd_swizzle=int(rng.integers(1, 3)),
                      nontemporal=int(rng.integers(0, 4)), threads=int(rng.choice([0, 64, 128, 256, 512, 1024])),
                      unroll=int(rng.choice([0, 1, 2, 4, 8])), max_workgroups=int(rng.choice([0, 0, 3, 40, 1000])),
                      xcd_block_tiles=int(rng.choice([0, 0, 1, 4, 64])), workgroups_per_cu=int(rng.choice([0, 0, 2, 5])))
    return case, (l0, l1), launch, rng


@pytest.mark.parametrize("seed", range(1000, 1300))
def test_random_case(seed):
    case, (l0, l1), launch, rng = draw_case(seed)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, l0, l1)
    got = G.run_gpu(case, src, l0, l1, launch=launch)
    G.assert_same(got, want, f"seed {seed} layers [{l0},{l1}) launch {launch}")


@pytest.mark.parametrize("seed", range(2000, 2150))
def test_random_case_with_token_innermost_pages(seed):
    case, (l0, l1), launch, rng = draw_case(seed, token_innermost=True)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, l0, l1)
    got = G.run_gpu(case, src, l0, l1, launch=launch)
    G.assert_same(got, want, f"seed {seed} layers [{l0},{l1}) launch {launch}")


HOST_PLANNED = {"seeds": 0, "sender": 0, "receiver": 0}


@pytest.mark.parametrize("seed", range(1000, 1300))
def test_random_case_one_sided_plans(seed):
    """The same cases as two machines see them: a sender-only plan for the pack, a receiver-only plan for the
    unpack, each without a workspace where that is allowed (run records built on the host)."""
    case, (l0, l1), launch, rng = draw_case(seed)
    src = rng.integers(0, 256, size=case.pool_bytes(case.s), dtype=np.uint8)
    want = G.run_oracle(case, src, l0, l1)
    total, buf, dst, how = G.run_gpu_one_sided(case, src, l0, l1, launch=launch)
    what = f"seed {seed} layers [{l0},{l1}) launch {launch} without workspace {how}"
    assert total == want.total, what
    assert np.array_equal(buf, want.buf), what
    assert np.array_equal(dst, want.dst_unpack), what
    HOST_PLANNED["seeds"] += 1
    HOST_PLANNED["sender"] += how[0]
    HOST_PLANNED["receiver"] += how[1]


def test_random_cases_did_cover_both_kinds_of_one_sided_plans():
    """Runs after the 300 cases above (same file, collected in order): a good share of them were planned on
    the host, and a good share on the device."""
    if HOST_PLANNED["seeds"] < 300:
        pytest.skip("only meaningful after the whole list has run in this process")
    for side in ("sender", "receiver"):
        assert 30 <= HOST_PLANNED[side] <= 270, HOST_PLANNED
