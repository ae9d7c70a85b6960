"""Seeded synthetic workloads for KV-cache transfer between paged pools.

This module only *draws inputs*: request lengths, block tables (which physical
page holds which logical page of a request), pool sizes and KV values.  It
contains none of the transfer method's arithmetic (no buffer offsets, no pool
addressing, no copying) so that both the HIP library and the CPU oracle can be
fed from it without sharing any code of the method itself.

The inputs stand in for the private production traces and models the paper
evaluated on (section 4.1, "Setup"): the shapes follow common GQA decoder
models, the lengths follow the stated distributions, and the block tables are
random permutations of a pool's pages, i.e. a maximally fragmented block-fixed
(PagedAttention-style) pool as described in section 2.2.3.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 240808147

LAYER_MAJOR = 0  # [layer][K,V][page][token][head][dim]
PAGE_MAJOR = 1   # [page][layer][K,V][token][head][dim]


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic batch.  `dist` names the length distribution."""
    name: str
    index: int                 # 1-based config number; seed = BASE_SEED + index
    num_layers: int
    num_kv_heads: int
    head_dim: int
    elem_bytes: int
    value_kind: str            # "fp16" | "bf16" | "fp8e4m3"
    page_s: int                # sender page size, tokens
    page_d: int                # receiver page size, tokens
    layout_s: int
    layout_d: int
    num_requests: int
    dist: str                  # "uniform" | "lognormal"
    len_lo: int
    len_hi: int                # inclusive upper bound / cap
    ln_median: float = 0.0
    ln_sigma: float = 0.0
    pool_pages_fixed: int = 0  # >0: fixed pool size in pages (both sides)
    pool_factor: float = 2.0   # else pages = ceil(factor * used pages)
    inner_s: int = 0           # arrangement inside a page, per side: 0 [token][head][dim],
    inner_d: int = 0           # 1 [head][token][dim], 2 [head][dim/x][token][x] (x elements = 16 bytes)

    @property
    def row_bytes(self) -> int:
        return self.num_kv_heads * self.head_dim * self.elem_bytes

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def scaled(self, **kw) -> "Workload":
        """A smaller variant of the same recipe (fewer layers / requests /
        shorter lengths) for cases a CPU check finishes in seconds."""
        return dataclasses.replace(self, **kw)


CONFIGS = {
    1: Workload("tiny", 1, 2, 8, 128, 2, "fp16", 16, 16, LAYER_MAJOR, LAYER_MAJOR,
                4, "uniform", 100, 600, pool_pages_fixed=256),
    2: Workload("llama3-8b-shape", 2, 32, 8, 128, 2, "bf16", 128, 128, LAYER_MAJOR, LAYER_MAJOR,
                16, "uniform", 1024, 4096),
    3: Workload("70b-shape-tp8-share", 3, 80, 1, 128, 2, "bf16", 128, 128, LAYER_MAJOR, LAYER_MAJOR,
                64, "lognormal", 1, 8192, ln_median=2048.0, ln_sigma=0.6),
    4: Workload("convert-128-to-16", 4, 40, 8, 128, 2, "bf16", 128, 16, LAYER_MAJOR, PAGE_MAJOR,
                32, "uniform", 1, 32768, pool_factor=1.0625),
    5: Workload("tidal-burst-fp8", 5, 40, 8, 128, 1, "fp8e4m3", 16, 16, LAYER_MAJOR, LAYER_MAJOR,
                1024, "uniform", 32, 512),
}


@dataclass
class Batch:
    """One drawn batch: lengths and CSR block tables for both sides."""
    workload: Workload
    seq_lens: np.ndarray        # uint32 [R]
    ids_s: np.ndarray           # uint32 [sum pages_s]
    offs_s: np.ndarray          # uint64 [R+1]
    ids_d: np.ndarray           # uint32 [sum pages_d]
    offs_d: np.ndarray          # uint64 [R+1]
    num_pages_s: int
    num_pages_d: int

    @property
    def total_tokens(self) -> int:
        return int(self.seq_lens.astype(np.int64).sum())


def draw_lengths(w: Workload, rng: np.random.Generator) -> np.ndarray:
    if w.dist == "uniform":
        n = rng.integers(w.len_lo, w.len_hi + 1, size=w.num_requests)
    elif w.dist == "lognormal":
        x = np.exp(rng.normal(np.log(w.ln_median), w.ln_sigma, size=w.num_requests))
        n = np.clip(np.rint(x), max(w.len_lo, 1), w.len_hi)
    else:
        raise ValueError(w.dist)
    return n.astype(np.uint32)


def _pages_needed(seq_lens: np.ndarray, page: int) -> np.ndarray:
    return (seq_lens.astype(np.int64) + page - 1) // page


def _deal_tables(seq_lens: np.ndarray, page: int, fixed: int, factor: float,
                 rng: np.random.Generator) -> Tuple[np.ndarray, np.ndarray, int]:
    """Pool size, then the first sum(pages) ids of a random permutation of all
    pages, dealt to the requests in order."""
    need = _pages_needed(seq_lens, page)
    used = int(need.sum())
    if fixed > 0:
        num_pages = fixed
    else:
        num_pages = max(int(np.ceil(factor * used)), 1)
    if used > num_pages:
        raise ValueError(f"pool of {num_pages} pages cannot hold {used}")
    perm = rng.permutation(num_pages).astype(np.uint32)
    offs = np.zeros(len(seq_lens) + 1, dtype=np.uint64)
    offs[1:] = np.cumsum(need).astype(np.uint64)
    return perm[:used].copy(), offs, num_pages


def draw_batch(w: Workload, seed: Optional[int] = None) -> Batch:
    rng = np.random.default_rng(w.seed if seed is None else seed)
    n = draw_lengths(w, rng)
    ids_s, offs_s, np_s = _deal_tables(n, w.page_s, w.pool_pages_fixed, w.pool_factor, rng)
    ids_d, offs_d, np_d = _deal_tables(n, w.page_d, w.pool_pages_fixed, w.pool_factor, rng)
    return Batch(w, n, ids_s, offs_s, ids_d, offs_d, np_s, np_d)


# ---------------------------------------------------------------------------
# Values.  All of these return raw bytes (uint8): the transfer treats the KV
# element type as opaque, and every comparison downstream is on bytes.
# ---------------------------------------------------------------------------

def _f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)          # round to nearest even
    return (u >> 16).astype(np.uint16)


def values_numpy(kind: str, nbytes: int, rng: np.random.Generator) -> np.ndarray:
    """`nbytes` bytes of KV values of the given kind, as a uint8 array."""
    if kind == "fp16":
        v = rng.standard_normal(nbytes // 2, dtype=np.float32).astype(np.float16)
        return v.view(np.uint8)
    if kind == "bf16":
        v = _f32_to_bf16_bits(rng.standard_normal(nbytes // 2, dtype=np.float32))
        return v.view(np.uint8)
    if kind == "fp8e4m3":
        b = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
        # e4m3 (finite-only variant): S.1111.111 are the two NaN encodings.
        b[b == 0x7F] = 0x7E
        b[b == 0xFF] = 0xFE
        return b
    raise ValueError(kind)


def fill_values_torch(kind: str, out_u8, seed: int, slab_bytes: int = 1 << 28) -> None:
    """Fill a 1-D uint8 torch tensor (any device) with KV values of `kind`,
    generated slab by slab on the tensor's own device."""
    import torch
    g = torch.Generator(device=out_u8.device)
    g.manual_seed(seed)
    n = out_u8.numel()
    for lo in range(0, n, slab_bytes):
        hi = min(lo + slab_bytes, n)
        dst = out_u8[lo:hi]
        if kind in ("fp16", "bf16"):
            dt = torch.float16 if kind == "fp16" else torch.bfloat16
            cnt = (hi - lo) // 2
            v = torch.randn(cnt, generator=g, device=out_u8.device, dtype=torch.float32).to(dt)
            dst[: cnt * 2].copy_(v.view(torch.uint8))
        elif kind == "fp8e4m3":
            b = torch.randint(0, 256, (hi - lo,), generator=g, device=out_u8.device,
                              dtype=torch.int16).to(torch.uint8)
            b[b == 0x7F] = 0x7E
            b[b == 0xFF] = 0xFE
            dst.copy_(b)
        else:
            raise ValueError(kind)
