"""The seeded input recipe: drawn sizes stay what the design notes state, block tables are valid and
maximally scattered, value generators produce what their names say."""
import numpy as np
import pytest

from paper_2408_08147_amd import workloads as W

DRAWN_TOKENS = {1: 1456, 2: 46172, 3: 161473, 4: 466885, 5: 286830}


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_seeded_draws_and_tables(idx):
    w = W.CONFIGS[idx]
    b = W.draw_batch(w)
    assert b.total_tokens == DRAWN_TOKENS[idx]
    assert np.array_equal(b.seq_lens, W.draw_batch(w).seq_lens)            # same seed, same draw
    assert b.seq_lens.min() >= max(w.len_lo, 1) and b.seq_lens.max() <= w.len_hi
    for ids, offs, page, num_pages in ((b.ids_s, b.offs_s, w.page_s, b.num_pages_s),
                                       (b.ids_d, b.offs_d, w.page_d, b.num_pages_d)):
        need = (b.seq_lens.astype(np.int64) + page - 1) // page
        assert np.array_equal(np.diff(offs.astype(np.int64)), need)        # exactly the pages each length needs
        assert len(ids) == need.sum() and len(np.unique(ids)) == len(ids)   # no page used twice
        assert ids.max() < num_pages
        if w.pool_pages_fixed:
            assert num_pages == w.pool_pages_fixed
        else:
            assert num_pages == int(np.ceil(w.pool_factor * need.sum()))
        # scattered: hardly any logical neighbours are physical neighbours
        adjacent = np.mean(np.diff(ids.astype(np.int64)) == 1)
        assert adjacent < max(0.02, 10.0 / num_pages)
    assert not np.array_equal(b.ids_s[:50], b.ids_d[:50])                   # the two sides are drawn independently


def test_lognormal_lengths_have_the_stated_median():
    w = W.CONFIGS[3].scaled(num_requests=20000)
    n = W.draw_lengths(w, np.random.default_rng(1))
    assert abs(np.median(n) - 2048) < 60 and n.max() <= 8192 and n.min() >= 1


def test_value_generators():
    rng = np.random.default_rng(0)
    fp8 = W.values_numpy("fp8e4m3", 1 << 16, rng)
    assert fp8.dtype == np.uint8 and not np.isin(fp8, [0x7F, 0xFF]).any() and len(np.unique(fp8)) == 254
    f16 = W.values_numpy("fp16", 1 << 16, rng).view(np.float16).astype(np.float64)
    assert abs(f16.mean()) < 0.05 and abs(f16.std() - 1) < 0.05
    bf = W.values_numpy("bf16", 1 << 16, rng).view(np.uint16)
    as_f32 = (bf.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert abs(as_f32.mean()) < 0.05 and abs(as_f32.std() - 1) < 0.05
    # round to nearest even on the dropped 16 bits
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5], dtype=np.float32)    # 1 + 2^-8 is a tie: stays 1.0
    got = W._f32_to_bf16_bits(x)
    assert list(got) == [0x3F80, 0x3F80, 0x3F82, 0xC020]


def test_torch_fill_matches_kinds_on_cpu():
    torch = pytest.importorskip("torch")
    out = torch.empty(1 << 14, dtype=torch.uint8)
    W.fill_values_torch("fp8e4m3", out, seed=3, slab_bytes=5000)
    a = out.numpy()
    assert not np.isin(a, [0x7F, 0xFF]).any()
    W.fill_values_torch("bf16", out, seed=3, slab_bytes=4096)
    v = (out.numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    assert np.isfinite(v).all() and abs(float(v.std()) - 1) < 0.1
