"""Synthetic multi-turn workloads: shapes, length mixes, values and page tables.

The five configurations mirror the shapes the benchmark contract names (a tiny
MHA check case, LLaMA-7B/13B-shaped MHA stacks, a context-overflow case and a
LLaMA-70B-shaped GQA stack).  They stand in for the ShareGPT trace the paper
(Section 4.1) replays: only length *distributions* are used, no dataset item.

Nothing here knows about RoPE, attention, truncation rules or KV layouts: the
module only produces seeded random lengths, bf16 bit patterns and permutations.
Lengths come from numpy.random.default_rng(seed) with history lengths drawn
before new-turn lengths.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# index 1..5 follow the benchmark contract's order; index 0 is unused padding
CONFIGS = {
    1: dict(name="cfg1-tiny-mha", n_layers=1, n_q_heads=4, n_kv_heads=4, head_dim=64,
            batch=1, window=4096, page_size=16, lengths="fixed", hist=256, new=32,
            truncate=False),
    2: dict(name="cfg2-llama7b-b16", n_layers=32, n_q_heads=32, n_kv_heads=32, head_dim=128,
            batch=16, window=4096, page_size=16, lengths="uniform",
            hist_range=(512, 2048), new_range=(32, 256), truncate=False),
    3: dict(name="cfg3-llama13b-b32", n_layers=40, n_q_heads=40, n_kv_heads=40, head_dim=128,
            batch=32, window=4096, page_size=16, lengths="lognormal",
            hist_mu_sigma=(7.0, 0.6), hist_clip=(64, 3800),
            new_mu_sigma=(4.5, 0.8), new_clip=(8, 512), truncate=False),
    4: dict(name="cfg4-overflow-7b-b8", n_layers=32, n_q_heads=32, n_kv_heads=32, head_dim=128,
            batch=8, window=4096, page_size=16, lengths="overflow",
            total_range=(5000, 6000), new_range=(64, 512), truncate=True, ratio=0.5),
    5: dict(name="cfg5-llama70b-gqa-b64", n_layers=80, n_q_heads=64, n_kv_heads=8, head_dim=128,
            batch=64, window=8192, page_size=16, lengths="uniform",
            hist_range=(1024, 4096), new_range=(64, 512), truncate=False),
}


def draw_lengths(cfg: dict, seed: int) -> tuple[np.ndarray, np.ndarray]:
    """History and new-turn token counts per conversation (int32 arrays)."""
    rng = np.random.default_rng(seed)
    b = cfg["batch"]
    kind = cfg["lengths"]
    if kind == "fixed":
        hist = np.full(b, cfg["hist"], dtype=np.int64)
        new = np.full(b, cfg["new"], dtype=np.int64)
    elif kind == "uniform":
        lo, hi = cfg["hist_range"]
        hist = rng.integers(lo, hi + 1, b)
        lo, hi = cfg["new_range"]
        new = rng.integers(lo, hi + 1, b)
    elif kind == "lognormal":
        mu, sg = cfg["hist_mu_sigma"]
        lo, hi = cfg["hist_clip"]
        hist = np.clip(np.rint(rng.lognormal(mu, sg, b)), lo, hi).astype(np.int64)
        mu, sg = cfg["new_mu_sigma"]
        lo, hi = cfg["new_clip"]
        new = np.clip(np.rint(rng.lognormal(mu, sg, b)), lo, hi).astype(np.int64)
    elif kind == "overflow":
        lo, hi = cfg["total_range"]
        total = rng.integers(lo, hi + 1, b)
        lo, hi = cfg["new_range"]
        new = rng.integers(lo, hi + 1, b)
        hist = total - new
    else:
        raise ValueError(kind)
    return hist.astype(np.int32), new.astype(np.int32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float64 exactly."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def draw_values_bf16(shape, seed: int, stream: int, scale: float = 1.0) -> np.ndarray:
    """~N(0, scale^2) values rounded to bf16, as uint16 bits.  (seed, stream) picks an
    independent generator, one per (layer, tensor)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(stream)])))
    x = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return f32_to_bf16_bits(x)


def draw_block_table(pages_per_seq, num_pages: int, seed: int) -> np.ndarray:
    """[n_seqs][max_pages] int32 physical page ids: a seeded random permutation of the pool
    dealt to the sequences in order; unused entries are -1.  Never the identity for pools
    larger than a couple of pages, so paging is really exercised."""
    pages_per_seq = [int(p) for p in pages_per_seq]
    need = sum(pages_per_seq)
    if need > num_pages:
        raise ValueError("pool too small")
    rng = np.random.default_rng([int(seed), 0xB10C])
    perm = rng.permutation(num_pages)[:need].astype(np.int32)
    max_pages = max(pages_per_seq) if pages_per_seq else 0
    table = np.full((len(pages_per_seq), max(max_pages, 1)), -1, dtype=np.int32)
    at = 0
    for c, p in enumerate(pages_per_seq):
        table[c, :p] = perm[at:at + p]
        at += p
    return table


@dataclass
class Workload:
    """Shapes + lengths of one batch; values are drawn on demand per (layer, tensor)."""
    index: int
    cfg: dict
    seed: int
    hist_len: np.ndarray
    new_len: np.ndarray
    _stream_ids: dict = field(default_factory=dict)

    @property
    def n_seqs(self) -> int:
        return int(self.hist_len.shape[0])

    def stream(self, layer: int, tensor: str, conv: int = 0) -> int:
        tid = {"q": 0, "k_hist": 1, "v_hist": 2, "k_new": 3, "v_new": 4}[tensor]
        return (layer * 8 + tid) * 4096 + conv

    def values(self, layer: int, tensor: str, conv: int, scale: float = 1.0) -> np.ndarray:
        """bf16 bits, shape [tokens][heads][head_dim] for one conversation."""
        c = self.cfg
        heads = c["n_q_heads"] if tensor == "q" else c["n_kv_heads"]
        toks = int(self.hist_len[conv]) if tensor in ("k_hist", "v_hist") else int(self.new_len[conv])
        return draw_values_bf16((toks, heads, c["head_dim"]), self.seed,
                                self.stream(layer, tensor, conv), scale)


def make_workload(index: int, seed: int | None = None, batch: int | None = None) -> Workload:
    cfg = dict(CONFIGS[index])
    if batch is not None:
        cfg["batch"] = batch
    if seed is None:
        seed = 0
    hist, new = draw_lengths(cfg, seed)
    return Workload(index=index, cfg=cfg, seed=seed, hist_len=hist, new_len=new)
