"""Shared plumbing of the GPU parity tests: builds seeded inputs, drives the HIP library through
its Python binding (which only marshals into the C ABI) and evaluates the fp64 oracle on the
same bits.  Nothing here is computed by the HIP path for the oracle or vice versa."""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

import oracle
import paper_2403_19708_amd as ca
from synth import bf16_bits_to_f64, draw_block_table, draw_values_bf16

P = 16


def bits_to_torch(bits: np.ndarray, device=None, pin=False) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    if pin:
        p = torch.empty(t.shape, dtype=torch.bfloat16, pin_memory=True)
        p.copy_(t)
        return p
    if device is not None:
        return t.to(device)
    return t


def torch_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


@dataclass
class Case:
    hist_len: list
    new_len: list
    keep_start: list
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seed: int = 0
    n_layers: int = 1
    q_scale: float = 1.0
    window: int = 4096
    style: int = 0
    spare_pages: int = 7
    data: dict = field(default_factory=dict)

    def __post_init__(self):
        self.hist_len = np.asarray(self.hist_len, np.int32)
        self.new_len = np.asarray(self.new_len, np.int32)
        self.keep_start = np.asarray(self.keep_start, np.int32)
        self.B = len(self.hist_len)
        self.n_keep = self.hist_len - self.keep_start
        self.ctx_len = self.n_keep + self.new_len
        self.pages = (self.ctx_len + P - 1) // P
        self.num_pages = int(self.pages.sum()) + self.spare_pages
        self.block_table = draw_block_table(self.pages, self.num_pages, self.seed + 17)
        self.cu_q = np.concatenate([[0], np.cumsum(self.new_len)]).astype(np.int64)

    def tensor(self, layer: int, name: str, conv: int) -> np.ndarray:
        """bf16 bits [tokens][heads][D] for one conversation (cached)."""
        key = (layer, name, conv)
        if key not in self.data:
            heads = self.n_q_heads if name == "q" else self.n_kv_heads
            toks = int(self.hist_len[conv]) if name in ("k_hist", "v_hist") else int(self.new_len[conv])
            tid = {"q": 0, "k_hist": 1, "v_hist": 2, "k_new": 3, "v_new": 4}[name]
            scale = self.q_scale if name == "q" else 1.0
            self.data[key] = draw_values_bf16((toks, heads, self.head_dim), self.seed,
                                              (layer * 8 + tid) * 4096 + conv, scale)
        return self.data[key]

    def flat_new(self, layer: int, name: str) -> np.ndarray:
        return np.concatenate([self.tensor(layer, name, c) for c in range(self.B)], axis=0)

    def config(self, **kw) -> ca.Config:
        base = dict(n_layers=self.n_layers, n_q_heads=self.n_q_heads, n_kv_heads=self.n_kv_heads,
                    head_dim=self.head_dim, max_positions=self.window, rope_style=self.style,
                    max_seqs=max(self.B, 1), max_batch_kv_tokens=int(self.ctx_len.sum()) + 64,
                    max_batch_q_tokens=int(self.new_len.sum()) + 16)
        base.update(kw)
        return ca.Config(**base)

    # ---- oracle ---------------------------------------------------------------------------
    def oracle_out(self, layer: int, conv: int, heads=None) -> np.ndarray:
        """fp64 [Ln][Hq or len(heads)][D]; `heads` restricts to some query heads (and the KV heads
        they read) so that big cases can be sampled."""
        w = bf16_bits_to_f64
        kh, vh = self.tensor(layer, "k_hist", conv), self.tensor(layer, "v_hist", conv)
        q, kn, vn = self.tensor(layer, "q", conv), self.tensor(layer, "k_new", conv), self.tensor(layer, "v_new", conv)
        if heads is not None:
            G = self.n_q_heads // self.n_kv_heads
            outs = []
            for h in heads:
                g = h // G
                outs.append(oracle.cached_attention(w(kh[:, g:g + 1]), w(vh[:, g:g + 1]), w(q[:, h:h + 1]),
                                                    w(kn[:, g:g + 1]), w(vn[:, g:g + 1]),
                                                    keep_start=int(self.keep_start[conv]), style=self.style))
            return np.concatenate(outs, axis=1)
        return oracle.cached_attention(w(kh), w(vh), w(q), w(kn), w(vn),
                                       keep_start=int(self.keep_start[conv]), style=self.style)

    def oracle_pool(self, layer: int, which: str, sentinel: int = 0x7FC0) -> np.ndarray:
        """What the pool must hold after load + append: uint16 [num_pages][Hkv][P][D]."""
        pool = np.full((self.num_pages, self.n_kv_heads, P, self.head_dim), sentinel, np.uint16)
        for c in range(self.B):
            hist = self.tensor(layer, f"{which}_hist", c)
            new = self.tensor(layer, f"{which}_new", c)
            oracle.unpack(hist, int(self.keep_start[c]), pool, self.block_table[c], P, self.n_kv_heads,
                          self.head_dim, 0, int(self.n_keep[c]))
            oracle.unpack(new, 0, pool, self.block_table[c], P, self.n_kv_heads, self.head_dim,
                          int(self.n_keep[c]), int(self.new_len[c]))
        return pool


class GpuRun:
    """One context + the device/pinned tensors of a Case.  tier: 'pinned' or 'device'."""

    def __init__(self, case: Case, tier="pinned", sentinel=0x7FC0, **cfg_kw):
        self.case = case
        self.dev = torch.device("cuda:0")
        self.ctx = ca.Context(case.config(**cfg_kw))
        self.tier = tier
        c = case
        shape = (c.num_pages, c.n_kv_heads, P, c.head_dim)
        self.k_pool, self.v_pool = [], []
        for _ in range(c.n_layers):
            for lst in (self.k_pool, self.v_pool):
                t = torch.empty(shape, dtype=torch.bfloat16, device=self.dev)
                t.view(torch.int16).fill_(np.array(sentinel, np.uint16).view(np.int16).item())
                lst.append(t)
        self.host_k, self.host_v = [], []   # [layer][conv] tier tensors with room for the new turn
        for layer in range(c.n_layers):
            hk, hv = [], []
            for conv in range(c.B):
                for name, lst in (("k_hist", hk), ("v_hist", hv)):
                    bits = c.tensor(layer, name, conv)
                    room = np.full((int(c.hist_len[conv] + c.new_len[conv]), c.n_kv_heads, c.head_dim), sentinel, np.uint16)
                    room[:c.hist_len[conv]] = bits
                    lst.append(bits_to_torch(room, pin=True) if tier == "pinned" else bits_to_torch(room, self.dev))
            self.host_k.append(hk)
            self.host_v.append(hv)
        self.q = [bits_to_torch(c.flat_new(layer, "q"), self.dev) for layer in range(c.n_layers)]
        self.k_new = [bits_to_torch(c.flat_new(layer, "k_new"), self.dev) for layer in range(c.n_layers)]
        self.v_new = [bits_to_torch(c.flat_new(layer, "v_new"), self.dev) for layer in range(c.n_layers)]
        self.out = [torch.zeros_like(q) for q in self.q]
        torch.cuda.synchronize()

    def rebase(self, stream=None):
        c = self.case
        self.ctx.rope_rebase(c.hist_len, c.keep_start, c.new_len, c.block_table, c.num_pages, stream)

    def load(self, layer):
        self.ctx.kv_load_layer(layer, self.host_k[layer], self.host_v[layer], self.k_pool[layer], self.v_pool[layer])

    def append(self, layer, stream=None):
        self.ctx.kv_append_layer(layer, self.k_new[layer], self.v_new[layer], self.k_pool[layer], self.v_pool[layer], stream)

    def attn(self, layer, stream=None, scale=None):
        s = scale if scale is not None else 1.0 / np.sqrt(self.case.head_dim)
        self.ctx.cached_prefill_attn(layer, self.q[layer], self.k_pool[layer], self.v_pool[layer], self.out[layer], s, stream)

    def save(self, layer, after_stream=None, **kw):
        self.ctx.kv_save_layer(layer, self.k_pool[layer], self.v_pool[layer], self.host_k[layer], self.host_v[layer],
                               after_stream=after_stream, **kw)

    def run_layer(self, layer):
        self.load(layer)
        self.append(layer)
        self.attn(layer)
        self.save(layer)

    def finish(self):
        self.ctx.sync()
        torch.cuda.synchronize()

    def out_f64(self, layer, conv) -> np.ndarray:
        c = self.case
        bits = torch_to_bits(self.out[layer][int(c.cu_q[conv]):int(c.cu_q[conv + 1])])
        return bf16_bits_to_f64(bits)

    def close(self):
        self.ctx.close()


def err_stats(got: np.ndarray, want: np.ndarray):
    d = np.abs(got - want)
    return float(d.max()), float(d.mean()), float(np.sqrt(np.mean(want ** 2)))
