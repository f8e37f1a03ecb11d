#!/usr/bin/env python3
"""Benchmark of the cached-prefill hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic conversations, for every
layer of the stack:  rebase (once)  ->  per layer: load the kept history from the KV tier into the
paged pool (read stream), append the new turn's K/V, fused rotary + causal attention of the new
tokens, save the new turn's K/V (without positions) back to the tier (write stream).

Default workload: the largest one-GPU configuration (config 5, LLaMA-70B-shaped grouped-query
attention, 80 layers, batch 64) with the KV tier where the method keeps it, in PINNED HOST memory
(Section 3.2.1), streamed layer by layer over the host link while attention runs.  `value` = new
tokens per second of that pipeline (sum of new tokens / step time).  Q, the new K/V, the pools and
all metadata are resident in HBM when the timed region starts; the tier is not an input hand-over
but the storage level the method loads from.  The same step with the tier placed in HBM (no host
link) is reported under "hbm_resident_tier", each kernel alone under "isolated", smaller
configurations under "configs", the read-buffer experiments of Sections 3.2.1 / 4.3.2 under
"pipeline_depth_sweep" and "preload_sweep", the decode phase under "decode".

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
P = 16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def release_pinned(torch):
    """hands cached pinned host blocks back to the system (the boxes pin only so much at a time)"""
    import gc
    gc.collect()
    fn = getattr(torch._C, "_host_emptyCache", None)
    if fn is not None:
        fn()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=5, help="workload index 1..5 (default 5: LLaMA-70B-shaped GQA, 80 layers, batch 64)")
    ap.add_argument("--tier", choices=["pinned", "hbm"], default="pinned",
                    help="where the KV tier of the headline leg lives (pinned host memory is the method's tier)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--hbm-steps", type=int, default=3, help="timed steps of the HBM-resident-tier leg")
    ap.add_argument("--summary-configs", type=str, default="2,3,4", help="configurations for the compact per-config summary ('' = none)")
    ap.add_argument("--no-hbm-leg", action="store_true")
    ap.add_argument("--no-sweeps", action="store_true", help="skip the pipeline-depth and preload sweeps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-phase leg")
    ap.add_argument("--decode-steps", type=int, default=20)
    ap.add_argument("--no-check", action="store_true", help="skip the sampled parity check against the oracle")
    ap.add_argument("--load-mode", type=int, default=0, help="library load_mode (0 staged copies for a host tier, 2 kernels read the tier in place)")
    ap.add_argument("--save-mode", type=int, default=0)
    ap.add_argument("--loads-ahead", type=int, default=0, help="layers whose loads are queued ahead of the compute calls (0: all first)")
    ap.add_argument("--two-call-save", action="store_true", help="append and save the new turn with the two separate calls in every leg")
    ap.add_argument("--depth", type=int, default=4, help="staging slots of the read stream (pipeline_depth) in the headline leg")
    ap.add_argument("--timeline-file", type=str, default="", help="write the per-interval timeline of the instrumented step here")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debugging only; marks the result invalid)")
    return ap.parse_args()


# ----------------------------------------------------------------------------------------------------
# one workload on the device
# ----------------------------------------------------------------------------------------------------
class Job:
    """Device (and optionally pinned-host) tensors of one batch of conversations for every layer, and the
    step that drives them through the library.  Layer 0 carries the seeded bits of synth/ (so that sampled
    outputs can be checked against the oracle); the other layers are filled by the device generator:
    distinct buffers per layer, so all traffic is real."""

    def __init__(self, torch, ca, index, seed, layers=0, with_layer0_bits=True, lengths=None, model=None):
        from synth import CONFIGS, draw_block_table, draw_values_bf16, make_workload
        self.torch, self.ca = torch, ca
        self.dev = torch.device("cuda:0")
        if lengths is None:
            wl = make_workload(index, seed=seed)
            cfg, hist, new = wl.cfg, wl.hist_len, wl.new_len
            self.wl = wl
        else:                                   # fixed lengths on a configuration's model shape
            cfg = dict(CONFIGS[model]); hist, new = lengths
            cfg["batch"] = len(hist); cfg["truncate"] = False
            self.wl = None
            with_layer0_bits = False
        self.cfg, self.index, self.seed = cfg, index, seed
        self.L = layers or cfg["n_layers"]
        self.Hq, self.Hkv, self.D, self.B, self.W = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["batch"], cfg["window"]
        self.hist, self.new = hist, new
        self.keep_start = ca.truncate_plan(hist, new, self.W, cfg["ratio"], policy=0) if cfg["truncate"] else np.zeros(self.B, np.int32)
        self.n_keep = hist - self.keep_start
        self.ctx_len = self.n_keep + new
        pages = (self.ctx_len + P - 1) // P
        self.num_pages = int(pages.sum()) + 8
        self.block_table = draw_block_table(pages, self.num_pages, seed + 17)
        self.tot_q, self.tot_n, self.tot_k = int(new.sum()), int(self.n_keep.sum()), int(self.ctx_len.sum())
        self.cu_q = np.concatenate([[0], np.cumsum(new)]).astype(np.int64)
        self.row = self.Hkv * self.D            # elements per token on the KV side
        self.scale = 1.0 / float(np.sqrt(self.D))
        # algorithmic work per layer = one launch of each kernel
        newf, keepf = new.astype(np.float64), self.n_keep.astype(np.float64)
        self.flops_layer = 4.0 * self.D * self.Hq * float(np.sum(newf * keepf + newf * (newf + 1) / 2))
        self.attn_bytes = 2.0 * self.tot_k * self.row * 2 + 2.0 * self.tot_q * self.Hq * self.D * 2   # K,V once + Q in + O out
        self.unpack_bytes = 2.0 * (2.0 * self.tot_n * self.row * 2)                                   # read + write, K and V
        self.append_bytes = 2.0 * (2.0 * self.tot_q * self.row * 2)
        self.pack_bytes = 2.0 * (2.0 * self.tot_q * self.row * 2)
        self.link_in_bytes = 2.0 * self.tot_n * self.row * 2
        self.link_out_bytes = 2.0 * self.tot_q * self.row * 2
        self.t_mfma_us = self.flops_layer / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6
        self.t_hbm_us = self.attn_bytes / (HBM_PEAK_GBS * 1e9) * 1e6
        self.attn_bound = "mfma" if self.t_mfma_us > self.t_hbm_us else "hbm"
        self.attn_floor_us = max(self.t_mfma_us, self.t_hbm_us)

        gen = torch.Generator(device=self.dev)
        gen.manual_seed(1234 + seed + 1000 * index)
        self._gen = gen
        L, B = self.L, self.B
        self.tier_off = np.concatenate([[0], np.cumsum(hist.astype(np.int64) + new)])
        self.layer0 = {}
        if with_layer0_bits:
            for name, toks in (("k_hist", hist), ("v_hist", hist), ("q", new), ("k_new", new), ("v_new", new)):
                heads = self.Hq if name == "q" else self.Hkv
                self.layer0[name] = [draw_values_bf16((int(toks[c]), heads, self.D), seed, self.wl.stream(0, name, c)) for c in range(B)]
        self.k_pool, self.v_pool, self.q, self.k_new, self.v_new, self.out = [], [], [], [], [], []
        bf = torch.bfloat16
        for l in range(L):
            if l == 0 and with_layer0_bits:
                self.q.append(self.bits_to_dev(np.concatenate(self.layer0["q"])))
                self.k_new.append(self.bits_to_dev(np.concatenate(self.layer0["k_new"])))
                self.v_new.append(self.bits_to_dev(np.concatenate(self.layer0["v_new"])))
            else:
                self.q.append(self.randn((self.tot_q, self.Hq, self.D)))
                self.k_new.append(self.randn((self.tot_q, self.Hkv, self.D)))
                self.v_new.append(self.randn((self.tot_q, self.Hkv, self.D)))
            self.k_pool.append(torch.zeros((self.num_pages, self.Hkv, P, self.D), dtype=bf, device=self.dev))
            self.v_pool.append(torch.zeros((self.num_pages, self.Hkv, P, self.D), dtype=bf, device=self.dev))
            self.out.append(torch.zeros((self.tot_q, self.Hq, self.D), dtype=bf, device=self.dev))
        self.dev_tier = None
        self.pin_tier = None

    def bits_to_dev(self, bits):
        t = self.torch
        return t.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(t.bfloat16).to(self.dev)

    def randn(self, shape):
        t = self.torch
        return t.randn(shape, generator=self._gen, device=self.dev, dtype=t.float32).to(t.bfloat16)

    def _fill_tier_layer(self, l, tk, tv):
        """values of the tier of layer l into the device tensors tk, tv ([all conversations' hist+new tokens][Hkv][D])"""
        if l == 0 and self.layer0:
            tk.zero_(); tv.zero_()
            for c in range(self.B):
                a = int(self.tier_off[c])
                tk[a:a + int(self.hist[c])] = self.bits_to_dev(self.layer0["k_hist"][c])
                tv[a:a + int(self.hist[c])] = self.bits_to_dev(self.layer0["v_hist"][c])
        else:
            tk.copy_(self.randn(tk.shape)); tv.copy_(self.randn(tv.shape))

    def make_device_tier(self):
        t = self.torch
        shape = (int(self.tier_off[-1]), self.Hkv, self.D)
        self.dev_tier = ([], [])
        for l in range(self.L):
            tk = t.empty(shape, dtype=t.bfloat16, device=self.dev); tv = t.empty_like(tk)
            self._fill_tier_layer(l, tk, tv)
            self.dev_tier[0].append(tk); self.dev_tier[1].append(tv)
        t.cuda.synchronize()

    def make_pinned_tier(self, cap_gib=40.0):
        """The tier in pinned host memory, one K and one V buffer per layer (filled through the device).  The
        boxes refuse to pin much more than ~50 GiB: when the whole stack does not fit under cap_gib (or pinning
        fails earlier), the layers cycle through the n_distinct buffers that could be pinned (layer l uses buffer
        l % n_distinct); every byte still crosses the host link, from distinct memory within any window of
        n_distinct layers."""
        t = self.torch
        shape = (int(self.tier_off[-1]), self.Hkv, self.D)
        per_layer = 2 * int(self.tier_off[-1]) * self.row * 2
        want = max(1, min(self.L, int(cap_gib * 2**30 // per_layer)))
        pk_list, pv_list = [], []
        tk = t.empty(shape, dtype=t.bfloat16, device=self.dev); tv = t.empty_like(tk)
        t0 = time.time()
        for l in range(want):
            try:
                pk = t.empty(shape, dtype=t.bfloat16, pin_memory=True); pv = t.empty(shape, dtype=t.bfloat16, pin_memory=True)
            except Exception as e:                     # the box will not pin more: keep a margin and cycle
                log(f"[bench]   pinning stopped at layer {l}: {type(e).__name__}")
                for lst in (pk_list, pv_list):
                    del lst[-2:]
                release_pinned(t)
                try:                                   # the refused allocation may leave its error to the next call
                    t.cuda.synchronize()
                except Exception:
                    pass
                break
            if self.dev_tier is not None:
                sk, sv = self.dev_tier[0][l], self.dev_tier[1][l]
            else:
                self._fill_tier_layer(l, tk, tv); sk, sv = tk, tv
            pk.copy_(sk); pv.copy_(sv)
            pk_list.append(pk); pv_list.append(pv)
        t.cuda.synchronize()
        del tk, tv
        n = len(pk_list)
        if n == 0:
            raise RuntimeError("no pinned host memory available")
        self.pin_distinct = n
        self.pin_gib = n * per_layer / 2**30
        self.pin_tier = ([pk_list[l % n] for l in range(self.L)], [pv_list[l % n] for l in range(self.L)])
        log(f"[bench]   pinned tier: {n} distinct layer buffers of {self.L} layers, {self.pin_gib:.1f} GiB, {time.time() - t0:.1f}s")

    def tier_ptrs(self, bufs):
        """per layer, the library's pointer array of the conversations' saved token 0"""
        esz = self.row * 2
        return [self.ca.pointer_array([bufs[l].data_ptr() + int(self.tier_off[c]) * esz for c in range(self.B)]) for l in range(self.L)]

    def config(self, **kw):
        base = dict(n_layers=self.L, n_q_heads=self.Hq, n_kv_heads=self.Hkv, head_dim=self.D, max_positions=self.W, pipeline_depth=2,
                    max_seqs=self.B, max_batch_kv_tokens=self.tot_k + 64, max_batch_q_tokens=self.tot_q + 16)
        base.update(kw)
        return self.ca.Config(**base)

    def rebase(self, ctx, stream):
        ctx.rope_rebase(self.hist, self.keep_start, self.new, self.block_table, self.num_pages, stream)

    loads_ahead = 0        # layers whose loads are queued before the first compute call (0: all of them)
    fused_save = True      # the new turn is appended and saved by one call that reads it once (False: the two calls)

    def compute_layer(self, ctx, l, src_k, src_v, stream, save=True):
        if save and self.fused_save:
            ctx.kv_append_save_layer(l, self.k_new[l], self.v_new[l], self.k_pool[l], self.v_pool[l], src_k[l], src_v[l], stream)
            ctx.cached_prefill_attn(l, self.q[l], self.k_pool[l], self.v_pool[l], self.out[l], self.scale, stream)
            return
        ctx.kv_append_layer(l, self.k_new[l], self.v_new[l], self.k_pool[l], self.v_pool[l], stream)
        ctx.cached_prefill_attn(l, self.q[l], self.k_pool[l], self.v_pool[l], self.out[l], self.scale, stream)
        if save:
            ctx.kv_save_layer(l, self.k_pool[l], self.v_pool[l], src_k[l], src_v[l], after_stream=stream)

    def step(self, ctx, src_k, src_v, stream):
        """the whole path for one batch: the read stream runs ahead as far as its staging slots allow"""
        self.rebase(ctx, stream)
        # All loads are queued first.  That keeps the host busy for about 6 ms before the first attention is queued (a
        # load is 2 copies per conversation), but queueing them a few layers ahead of the compute calls instead was
        # measured to lower the link rate of the whole step (config 5: 1030-1036 ms per step against 1073-1119 ms with
        # 6 or 12 layers ahead): the copy queues run dry whenever the host is busy with the other calls.
        ahead = min(self.L, self.loads_ahead) if self.loads_ahead > 0 else self.L
        for l in range(ahead):
            ctx.kv_load_layer(l, src_k[l], src_v[l], self.k_pool[l], self.v_pool[l])
        for l in range(self.L):
            if l + ahead < self.L:
                ctx.kv_load_layer(l + ahead, src_k[l + ahead], src_v[l + ahead], self.k_pool[l + ahead], self.v_pool[l + ahead])
            self.compute_layer(ctx, l, src_k, src_v, stream)
        ctx.join(stream)

    def timed(self, ctx, src_k, src_v, stream, warmup, steps, tag, kinds=None, timeline=False):
        """kinds: which of the library's kernels/copies are bracketed by HIP events during the timed steps
        (None = all; the events cost a few per cent of a step made of short kernels)"""
        torch, ca = self.torch, self.ca
        for _ in range(warmup):
            self.step(ctx, src_k, src_v, stream)
        ctx.sync(); torch.cuda.synchronize()
        for k in ca.Context.PROFILE_KINDS:
            ctx.profile_read(k)              # drop what the warm-up recorded
        ctx.profile_enable(True, kinds)
        t = time.perf_counter()
        for _ in range(steps):
            self.step(ctx, src_k, src_v, stream)
        ctx.sync(); torch.cuda.synchronize()
        dt = time.perf_counter() - t
        ctx.profile_enable(False)
        tl = ctx.profile_timeline() if timeline else None
        prof = {k: ctx.profile_read(k) for k in ca.Context.PROFILE_KINDS}
        if timeline:
            prof["timeline"] = tl
        log(f"[bench] {tag}: {steps} steps in {dt * 1e3:.1f} ms")
        return dt, prof

    def isolated(self, ctx, src_k, src_v, stream):
        """each kernel alone (nothing else on the GPU), a few layers"""
        torch = self.torch
        n_iso = min(self.L, 4)
        for k in self.ca.Context.PROFILE_KINDS:
            ctx.profile_read(k)
        ctx.profile_enable(True)
        sync = lambda: (ctx.sync(), torch.cuda.synchronize())
        for l in range(n_iso):
            sync(); self.rebase(ctx, stream)
            sync(); ctx.kv_load_layer(l, src_k[l], src_v[l], self.k_pool[l], self.v_pool[l])
            sync(); ctx.kv_append_layer(l, self.k_new[l], self.v_new[l], self.k_pool[l], self.v_pool[l], stream)
            sync(); ctx.cached_prefill_attn(l, self.q[l], self.k_pool[l], self.v_pool[l], self.out[l], self.scale, stream)
            sync(); ctx.kv_save_layer(l, self.k_pool[l], self.v_pool[l], src_k[l], src_v[l], after_stream=stream)
            sync()
        ctx.profile_enable(False)
        iso = {}
        sep = {k: ctx.profile_read(k) for k in ("append", "pack")}
        ctx.profile_enable(True, ["append"])
        for l in range(n_iso):
            sync(); ctx.kv_append_save_layer(l, self.k_new[l], self.v_new[l], self.k_pool[l], self.v_pool[l], src_k[l], src_v[l], stream)
            sync()
        ctx.profile_enable(False)
        f_ms, f_n = ctx.profile_read("append")
        ctx.profile_read("copy_out")
        fused_us = f_ms / f_n * 1e3 if f_n else None
        for kname, nbytes in (("attn", self.attn_bytes), ("unpack", self.unpack_bytes), ("append", self.append_bytes), ("pack", self.pack_bytes)):
            ms, cnt = sep[kname] if kname in sep else ctx.profile_read(kname)
            us = ms / cnt * 1e3 if cnt else None
            iso[kname] = {"avg_launch_us": us, "gbs": nbytes / (us * 1e-6) / 1e9 if us else None,
                          "frac_hbm_peak": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS if us else None}
        for k in ("copy_in", "copy_out"):
            ctx.profile_read(k)
        if fused_us:
            nb = self.append_bytes * 1.5
            iso["append_save_fused"] = {"avg_launch_us": fused_us, "gbs": nb / (fused_us * 1e-6) / 1e9,
                                        "frac_hbm_peak": nb / (fused_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                        "vs_two_calls": fused_us / (iso["append"]["avg_launch_us"] + iso["pack"]["avg_launch_us"]) - 1.0
                                        if iso["append"]["avg_launch_us"] and iso["pack"]["avg_launch_us"] else None}
        a = iso["attn"]
        a["tflops"] = self.flops_layer / (a["avg_launch_us"] * 1e-6) / 1e12
        a["frac_mfma_peak"] = a["tflops"] / MFMA_BF16_PEAK_TFLOPS
        a["binding_roofline"] = self.attn_bound
        a["roofline_floor_us"] = self.attn_floor_us
        a["frac_binding_roofline"] = self.attn_floor_us / a["avg_launch_us"]
        return iso

    def attn_figures(self, us):
        tf = self.flops_layer / (us * 1e-6) / 1e12
        gbs = self.attn_bytes / (us * 1e-6) / 1e9
        return {"avg_launch_us": us, "tflops": tf, "frac_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS, "gbs": gbs,
                "frac_hbm_peak": gbs / HBM_PEAK_GBS, "binding_roofline": self.attn_bound, "roofline_floor_us": self.attn_floor_us,
                "frac_binding_roofline": self.attn_floor_us / us}

    def move_figures(self, prof, fused_device_tier=False):
        """fused_device_tier: the append figure is the one-pass append + save kernel (read N, write 2N bytes)"""
        out = {}
        app = self.append_bytes * 1.5 if fused_device_tier else self.append_bytes
        for k, nbytes in (("unpack", self.unpack_bytes), ("append", app), ("pack", self.pack_bytes)):
            ms, n = prof[k]
            us = ms / n * 1e3 if n else None
            out[k] = {"avg_launch_us": us, "gbs": nbytes / (us * 1e-6) / 1e9 if us else None,
                      "frac_hbm_peak": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS if us else None}
        return out

    def parity(self, layer0_out):
        """sampled (conversation, head) outputs of layer 0 against the oracle, element by element"""
        import oracle
        from synth import bf16_bits_to_f64 as w
        torch = self.torch
        got_all = layer0_out.detach().cpu().view(torch.int16).numpy().view(np.uint16)
        rng = np.random.default_rng(5)
        samples = [(int(rng.integers(self.B)), int(rng.integers(self.Hq))) for _ in range(6)]
        G = self.Hq // self.Hkv
        worst_max, worst_mean = 0.0, 0.0
        l0 = self.layer0
        for c, h in samples:
            g = h // G
            want = oracle.cached_attention(w(l0["k_hist"][c][:, g:g + 1]), w(l0["v_hist"][c][:, g:g + 1]), w(l0["q"][c][:, h:h + 1]),
                                           w(l0["k_new"][c][:, g:g + 1]), w(l0["v_new"][c][:, g:g + 1]), keep_start=int(self.keep_start[c]))
            got = w(got_all[int(self.cu_q[c]):int(self.cu_q[c + 1]), h:h + 1])
            err = np.abs(got - want)
            worst_max, worst_mean = max(worst_max, float(err.max())), max(worst_mean, float(err.mean()))
        ok = bool(worst_max <= 2e-2 and worst_mean <= 2e-3)
        log(f"[bench] sampled parity vs oracle (layer 0): max-abs {worst_max:.2e} mean-abs {worst_mean:.2e}")
        return dict(samples=len(samples), max_abs=worst_max, mean_abs=worst_mean, ok=ok)

    def free(self):
        for name in ("k_pool", "v_pool", "q", "k_new", "v_new", "out"):
            setattr(self, name, None)
        self.dev_tier = self.pin_tier = None
        self.torch.cuda.empty_cache()
        release_pinned(self.torch)


# ----------------------------------------------------------------------------------------------------
# legs
# ----------------------------------------------------------------------------------------------------
def pipeline_figures(job, dt, steps, prof):
    """Section 3.2.1's quantities from the events of the timed steps of a host-tier run"""
    t_pipe = dt / steps
    cin_ms, cin_n = prof["copy_in"]; cout_ms, cout_n = prof["copy_out"]; att_ms, att_n = prof["attn"]
    wb_kind = "copies out of a staging slot"
    if cout_n == 0 and prof.get("pack", (0.0, 0))[1]:
        cout_ms, cout_n = prof["pack"]          # the pack kernel writes the pinned tier in place: its run time is the write-back
        wb_kind = "pack kernel storing to the pinned tier in place"
    t_in, t_out, t_attn = cin_ms / steps / 1e3, cout_ms / steps / 1e3, att_ms / steps / 1e3
    L = job.L
    # per token and layer, as the paper defines them: T_load = access time of one token's K/V, T_pref = prefill
    # time of one new token (here: its attention, the only compute on this path)
    t_load_tok = t_in / L / max(job.tot_n, 1)
    t_pref_tok = t_attn / L / max(job.tot_q, 1)
    lhs, rhs = t_load_tok * job.tot_n, t_pref_tok * job.tot_q        # = per-layer load time, per-layer compute time
    link_gbs = job.link_in_bytes * cin_n / (cin_ms * 1e-3) / 1e9 if cin_ms else None
    s_buf = (link_gbs or 0.0) * 1e9 * max(0.0, lhs - rhs) * L        # bytes for the whole stack
    return dict(
        ms_per_step=t_pipe * 1e3, tokens_per_s=job.tot_q / t_pipe, context_tokens_per_s=job.tot_k / t_pipe,
        h2d_gbs=link_gbs, d2h_gbs=job.link_out_bytes * cout_n / (cout_ms * 1e-3) / 1e9 if cout_ms else None,
        copy_in_ms=t_in * 1e3, copy_out_ms=cout_ms / steps, write_back=wb_kind, attn_ms=t_attn * 1e3,
        # (T_copy + T_attn - T_pipe) / min(T_copy, T_attn): 1.0 = the shorter one is completely hidden
        overlap_efficiency=(t_in + t_attn - t_pipe) / min(t_in, t_attn) if min(t_in, t_attn) > 0 else None,
        not_under_copy_ms=(t_pipe - t_in) * 1e3,
        overlap_condition=dict(
            T_load_x_L_hist_ms_per_layer=lhs * 1e3, T_pref_x_L_new_ms_per_layer=rhs * 1e3, imperfect=bool(lhs > rhs),
            S_buf_bytes=s_buf, S_buf_layers=s_buf / job.link_in_bytes if job.link_in_bytes else None,
            note="Section 3.2.1 with attention as the only compute: loading a layer takes longer than computing it, so the "
                 "pipeline is bound by the host link and the formula asks for a read buffer of nearly the whole stack"),
    )


def mfma_rate_probe():
    """the matrix-core rate the card sustains on zero and on random operands (a stand-alone program built with the
    library, run as a child process); None when it is not built"""
    exe = os.path.join(ROOT, "paper_2403_19708_amd", "mfma_rate_probe")
    if not os.path.exists(exe):
        return None
    try:
        import subprocess
        out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
        return json.loads(out.stdout.strip().splitlines()[-1]) if out.returncode == 0 else None
    except Exception:
        return None


def link_probe(torch):
    """the host link by itself: one 320 MiB copy from pinned host memory to the device, best of five"""
    n = 320 * 1024 * 1024 // 2
    h = torch.empty(n, dtype=torch.bfloat16, pin_memory=True)
    d = torch.empty(n, dtype=torch.bfloat16, device="cuda:0")
    d.copy_(h, non_blocking=True); torch.cuda.synchronize()
    best = 0.0
    for _ in range(5):
        t = time.perf_counter()
        d.copy_(h, non_blocking=True); torch.cuda.synchronize()
        best = max(best, n * 2 / (time.perf_counter() - t) / 1e9)
    del h, d
    return best


def _union(iv):
    """sorted disjoint union of intervals"""
    out = []
    for a, b in sorted(iv):
        if out and a <= out[-1][1]:
            out[-1][1] = max(out[-1][1], b)
        else:
            out.append([a, b])
    return out


def _common(u, v):
    """total length of the intersection of two disjoint sorted interval lists"""
    i = j = 0
    tot = 0.0
    while i < len(u) and j < len(v):
        lo, hi = max(u[i][0], v[j][0]), min(u[i][1], v[j][1])
        if hi > lo:
            tot += hi - lo
        if u[i][1] < v[j][1]:
            i += 1
        else:
            j += 1
    return tot


def timeline_figures(tl, path=None):
    """Where the time of one step with a host tier goes, from the library's own event pairs around every copy
    batch and kernel (all on one clock): how much of the attention runs while the read stream is copying, and
    what is left uncovered at the head and the tail of the step."""
    by = {}
    for kind, a, b in tl:
        by.setdefault(kind, []).append((a, b))
    length = lambda u: sum(b - a for a, b in u)
    cin, att = _union(by.get("copy_in", [])), _union(by.get("attn", []))
    comp = _union(by.get("attn", []) + by.get("unpack", []) + by.get("append", []))
    cout = _union(by.get("copy_out", []) or by.get("pack", []))
    t0, t1 = min(a for _, a, _ in tl), max(b for _, _, b in tl)
    res = dict(span_ms=t1 - t0, copy_in_busy_ms=length(cin), attn_busy_ms=length(att), compute_busy_ms=length(comp),
               copy_out_busy_ms=length(cout), attn_under_copy_in_ms=_common(att, cin), copy_in_under_compute_ms=_common(cin, comp),
               head_before_first_attn_ms=(att[0][0] - t0) if att else None,
               tail_after_last_copy_in_ms=(t1 - cin[-1][1]) if cin else None,
               read_stream_idle_ms=(t1 - t0) - length(cin),
               note="one step with every copy batch and kernel bracketed by events; head = the first layer's load, which nothing can "
                    "hide; tail = the last layer's unpack, attention, save and write-back after the read stream has finished")
    if att:
        res["attn_under_copy_in_frac"] = res["attn_under_copy_in_ms"] / res["attn_busy_ms"]
    if path:
        with open(path, "w") as f:
            f.write("# kind index start_ms stop_ms (index = order within the kind = layer for copy_in, attn, copy_out)\n")
            seen = {}
            for kind, a, b in tl:
                i = seen.get(kind, 0); seen[kind] = i + 1
                f.write(f"{kind} {i} {a:.4f} {b:.4f}\n")
    return res


def depth_sweep(torch, ca, job, host_k, host_v, stream, depths, args):
    """the same host-tier step with 1, 2, 4, ... staging slots on the read stream"""
    out = []
    for d in depths:
        ctx = ca.Context(job.config(pipeline_depth=d, load_mode=args.load_mode, save_mode=args.save_mode))
        try:
            dt, prof = job.timed(ctx, host_k, host_v, stream, 1, 2, f"pinned tier, pipeline_depth {d}", kinds=["copy_in", "attn"])
            cin_ms, _ = prof["copy_in"]
            out.append(dict(pipeline_depth=d, ms_per_step=dt / 2 * 1e3, copy_in_ms=cin_ms / 2))
        finally:
            ctx.close()
    return out


def preload_sweep(torch, ca, seed):
    """Section 4.3.2's pre-loading experiment at its shape (LLaMA-13B shapes, batch 16, 1K history, 100 new tokens,
    host tier): the time from the moment the previous job releases the GPU to the end of this job's last layer,
    when d layers of this job were already loaded into the read buffer while the previous job ran."""
    B, L_hist, L_new = 16, 1000, 100
    lengths = (np.full(B, L_hist, np.int32), np.full(B, L_new, np.int32))
    job = Job(torch, ca, 3, seed, lengths=lengths, model=3)
    job.make_pinned_tier()
    host_k, host_v = job.tier_ptrs(job.pin_tier[0]), job.tier_ptrs(job.pin_tier[1])
    stream = torch.cuda.current_stream()
    L = job.L
    ctx = ca.Context(job.config(pipeline_depth=2))
    res = []
    try:
        def run(depth, preload):
            """depth None: no pre-loading at all (every layer loaded, then computed)"""
            job.rebase(ctx, stream)
            n_pre = 0 if depth is None else min(depth, L)
            for l in range(n_pre):
                ctx.kv_load_layer(l, host_k[l], host_v[l], job.k_pool[l], job.v_pool[l])
            ctx.sync(); torch.cuda.synchronize()              # the previous job ends here; the read buffer holds n_pre layers
            t0 = time.perf_counter()
            for l in range(n_pre, L):
                ctx.kv_load_layer(l, host_k[l], host_v[l], job.k_pool[l], job.v_pool[l])
            if not preload:
                ctx.sync()
            for l in range(L):
                job.compute_layer(ctx, l, host_k, host_v, stream, save=False)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3

        run(0, True)                                          # warm-up
        for name, depth, pre in (("NO-PL", None, False), ("PL-B0", 0, True), ("PL-B5", 5, True), ("PL-B15", 15, True),
                                 ("PL-B30", 30, True), (f"PL-B{L}", L, True)):
            ms = min(run(depth, pre) for _ in range(2))
            res.append(dict(name=name, layers_in_read_buffer=0 if depth is None else depth, ms=ms))
        # the two sides of the overlap condition from measured per-layer times
        dt, prof = job.timed(ctx, host_k, host_v, stream, 0, 1, "preload shape, one step", kinds=["copy_in", "attn"])
        fig = pipeline_figures(job, dt, 1, {**prof, "copy_out": (0.0, 0)})
    finally:
        ctx.close()
    t_load, t_pref = fig["overlap_condition"]["T_load_x_L_hist_ms_per_layer"], fig["overlap_condition"]["T_pref_x_L_new_ms_per_layer"]
    knee_formula = fig["overlap_condition"]["S_buf_layers"]
    # measured knee: the smallest buffer whose time is within 5 % of the fully pre-loaded run
    full = res[-1]["ms"]
    knee_measured = next((r["layers_in_read_buffer"] for r in res[1:] if r["ms"] <= 1.05 * full), L)
    no_pl = res[0]["ms"]
    for r in res:
        r["vs_no_preload"] = r["ms"] / no_pl - 1.0
    job.free()
    return dict(shape=dict(model="LLaMA-13B shapes (40 layers, 40 heads, head_dim 128)", batch=B, history=L_hist, new=L_new),
                runs=res, T_load_x_L_hist_ms_per_layer=t_load, T_pref_x_L_new_ms_per_layer=t_pref, h2d_gbs=fig["h2d_gbs"],
                S_buf_bytes=fig["overlap_condition"]["S_buf_bytes"], knee_formula_layers=knee_formula, knee_measured_layers=knee_measured,
                note="compute here is attention only, so T_load*L_hist >> T_pref*L_new: the time falls linearly with the layers "
                     "already in the read buffer and only (nearly) the whole stack hides the loads; the paper's 35 % / 61 % at "
                     "B0 / B15 have whole-layer prefill (projections, FFN) on the compute side")


def decode_leg(torch, ca, cfg, n_steps, seed):
    """Decode phase of a turn (Section 3.2.2) at the shape of the paper's saving experiment (Section 4.3.2:
    batch 16, prompts of 1K..1.6K tokens, 20 decoding steps) on the given model: every step appends
    one K/V token per conversation and layer, attends it over the whole context, and writes the
    step's K/V back to the tier on the save stream while the next step runs.  The contexts are already in
    the pool (as after the turn's prefill); the tier is device memory."""
    from synth import draw_block_table
    dev = torch.device("cuda:0")
    L, Hq, Hkv, D = cfg["n_layers"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    B = 16
    rng = np.random.default_rng(seed + 77)
    prompt = rng.integers(1000, 1601, B).astype(np.int32)
    pages = (prompt + n_steps + P - 1) // P
    num_pages = int(pages.sum()) + 4
    bt = draw_block_table(pages, num_pages, seed + 78)
    g = torch.Generator(device=dev); g.manual_seed(seed + 79)
    randn = lambda shape: torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_pool = [randn((num_pages, Hkv, P, D)) for _ in range(L)]
    v_pool = [randn((num_pages, Hkv, P, D)) for _ in range(L)]
    q = [randn((B, Hq, D)) for _ in range(L)]
    kn = [randn((B, Hkv, D)) for _ in range(L)]
    vn = [randn((B, Hkv, D)) for _ in range(L)]
    out = [torch.zeros((B, Hq, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
    # tier rows of the generated tokens only (the prompt's rows were written by the prefill's save)
    tier_k = [torch.zeros((B, n_steps, Hkv, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
    tier_v = [torch.zeros((B, n_steps, Hkv, D), dtype=torch.bfloat16, device=dev) for _ in range(L)]
    row = Hkv * D * 2
    ptrs = lambda t: [t.data_ptr() + c * n_steps * row for c in range(B)]
    tk_ptr = [ca.pointer_array(ptrs(t)) for t in tier_k]; tv_ptr = [ca.pointer_array(ptrs(t)) for t in tier_v]
    conf = ca.Config(n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, max_positions=cfg["window"], max_seqs=B,
                     max_batch_kv_tokens=int((prompt + n_steps).sum()) + 64, max_batch_q_tokens=B + 16, require_load=0)
    scale = 1.0 / float(np.sqrt(D))
    stream = torch.cuda.current_stream()
    one, zero = np.ones(B, np.int32), np.zeros(B, np.int32)

    def run(ctx, write_back):
        t0 = time.perf_counter()
        for s in range(n_steps):
            have = prompt + s
            nxt, off = have + 1, np.full(B, s, np.int64)
            ctx.rope_rebase(have, zero, one, bt, num_pages, stream)
            for l in range(L):
                ctx.kv_append_layer(l, kn[l], vn[l], k_pool[l], v_pool[l], stream)
                ctx.cached_prefill_attn(l, q[l], k_pool[l], v_pool[l], out[l], scale, stream)
                if write_back:
                    ctx.kv_save_layer(l, k_pool[l], v_pool[l], tk_ptr[l], tv_ptr[l], tok_begin=have, tok_end=nxt,
                                      dst_tok_offset=off, after_stream=stream)
        host = time.perf_counter() - t0
        ctx.sync(); torch.cuda.synchronize()
        return time.perf_counter() - t0, host

    with ca.Context(conf) as ctx:
        run(ctx, True)                                        # warm-up
        t_plain, _ = run(ctx, False)
        t_wb, host_wb = run(ctx, True)
        ctx.profile_enable(True, ["attn"])
        run(ctx, True)
        att_ms, att_n = ctx.profile_read("attn")
        ctx.profile_enable(False)
        # the write-back must have delivered the bits of the last pass: spot check, layer 0
        ok = bool(torch.equal(tier_k[0][:, -1], kn[0]) and torch.equal(tier_v[0][:, 0], vn[0]))
    kv_bytes = 2.0 * float((prompt + (n_steps + 1) / 2.0).sum()) * row       # K and V of the mean context, per layer
    att_us = att_ms / att_n * 1e3
    return dict(model=cfg["name"], batch=B, prompt_tokens=[int(prompt.min()), int(prompt.max())], steps=n_steps, layers=L,
                ms_per_step=t_wb / n_steps * 1e3, tokens_per_s=B * n_steps / t_wb,
                ms_per_step_without_write_back=t_plain / n_steps * 1e3, host_ms_per_step=host_wb / n_steps * 1e3,
                attn_avg_launch_us=att_us, attn_kv_read_gbs=kv_bytes / att_us / 1e3,
                attn_frac_hbm_peak=kv_bytes / att_us / 1e3 / HBM_PEAK_GBS, write_back_ok=ok,
                attn_kernel="attn_decode_kernel" if Hq // Hkv <= 2 else "attn_dma_kernel",
                note="one token per conversation and step through the same entry points; each step's K/V is written back "
                     "on the save stream while the next step runs (device tier)")


def cpu_baseline(job):
    """the oracle as it stands on the host cores, on a bounded sample of the same workload"""
    import oracle
    from synth import bf16_bits_to_f64 as w
    l0 = job.layer0
    budget_s, used, convs, fl = 15.0, 0.0, 0, 0.0
    t_start = time.perf_counter()
    order = np.argsort(job.new.astype(np.int64) * job.ctx_len)      # cheapest conversations first: several fit the budget
    done = []
    for c in order:
        c = int(c)
        tk = time.perf_counter()
        oracle.cached_attention(w(l0["k_hist"][c]), w(l0["v_hist"][c]), w(l0["q"][c]), w(l0["k_new"][c]), w(l0["v_new"][c]),
                                keep_start=int(job.keep_start[c]))
        used += time.perf_counter() - tk
        convs += 1; done.append(c)
        fl += 4.0 * job.D * job.Hq * (float(job.new[c]) * float(job.n_keep[c]) + float(job.new[c]) * (float(job.new[c]) + 1) / 2)
        if time.perf_counter() - t_start > budget_s:
            break
    step_s = used * (job.flops_layer * job.L) / fl        # the sample scaled to one whole step by attention flops
    cpu = dict(value=job.tot_q / step_s, unit="tokens/s", cores=oracle.n_threads(), kind="oracle",
               sample=f"attention of layer 0 of {job.cfg['name']}, the {convs} cheapest of {job.B} conversations (all heads), {used:.1f} s of "
                      f"oracle time, scaled to {job.L} layers x {job.B} conversations by attention flops; data movement not included",
               gflops=fl / used / 1e9)
    c0 = done[0]
    rows = np.ascontiguousarray(np.concatenate([l0["k_hist"][c0][int(job.keep_start[c0]):], l0["k_new"][c0]]))
    pool_cpu = np.zeros((job.num_pages, job.Hkv, 16, job.D), np.uint16)
    back = np.zeros_like(rows)
    tk = time.perf_counter()
    oracle.unpack(rows, 0, pool_cpu, job.block_table[c0], 16, job.Hkv, job.D, 0, len(rows))
    t_unpack = time.perf_counter() - tk
    tk = time.perf_counter()
    oracle.pack(pool_cpu, job.block_table[c0], 16, job.Hkv, job.D, 0, len(rows), back, 0)
    t_pack = time.perf_counter() - tk
    assert np.array_equal(back, rows)
    cpu["move_gbs"] = {"unpack": 2.0 * rows.nbytes / t_unpack / 1e9, "pack": 2.0 * rows.nbytes / t_pack / 1e9,
                       "sample": f"K of conversation {c0}, layer 0: {rows.nbytes / 1e6:.1f} MB each way, one thread"}
    log(f"[bench] oracle: {convs} conversations of one layer in {used:.1f}s on {cpu['cores']} threads; "
        f"unpack {cpu['move_gbs']['unpack']:.2f} GB/s, pack {cpu['move_gbs']['pack']:.2f} GB/s")
    return cpu


def config_summary(torch, ca, index, seed):
    """compact figures of a smaller configuration with its tier in HBM: attention and load kernels alone and
    inside a step, against the roofline that binds them"""
    t0 = time.time()
    job = Job(torch, ca, index, seed, with_layer0_bits=False)
    job.make_device_tier()
    dev_k, dev_v = job.tier_ptrs(job.dev_tier[0]), job.tier_ptrs(job.dev_tier[1])
    stream = torch.cuda.current_stream()
    ctx = ca.Context(job.config())
    try:
        dt, prof = job.timed(ctx, dev_k, dev_v, stream, 1, 3, f"{job.cfg['name']}: tier in HBM, every kernel timed")
        iso = job.isolated(ctx, dev_k, dev_v, stream)
    finally:
        ctx.close()
    att_us = prof["attn"][0] / prof["attn"][1] * 1e3
    mv = job.move_figures(prof, fused_device_tier=True)
    res = dict(workload=job.cfg["name"], layers=job.L, new_tokens=job.tot_q, kept_history_tokens=job.tot_n,
               ms_per_step_hbm_tier=dt / 3 * 1e3, tokens_per_s_hbm_tier=job.tot_q / (dt / 3),
               attn_binding_roofline=job.attn_bound, attn_roofline_floor_us=job.attn_floor_us,
               attn_isolated_us=iso["attn"]["avg_launch_us"], attn_isolated_frac_binding_roofline=iso["attn"]["frac_binding_roofline"],
               attn_isolated_tflops=iso["attn"]["tflops"], attn_isolated_gbs=iso["attn"]["gbs"],
               attn_in_step_us=att_us, attn_in_step_frac_binding_roofline=job.attn_floor_us / att_us,
               unpack_isolated_gbs=iso["unpack"]["gbs"], unpack_isolated_frac_hbm_peak=iso["unpack"]["frac_hbm_peak"],
               unpack_in_step_gbs=mv["unpack"]["gbs"], append_isolated_gbs=iso["append"]["gbs"], pack_isolated_gbs=iso["pack"]["gbs"],
               append_in_step_us=mv["append"]["avg_launch_us"], pack_in_step_us=mv["pack"]["avg_launch_us"])
    job.free()
    log(f"[bench] {job.cfg['name']}: attention {res['attn_isolated_us']:.1f} us alone ({res['attn_isolated_frac_binding_roofline']:.2f} of its "
        f"{job.attn_bound} roofline), {att_us:.1f} us in step; unpack {res['unpack_isolated_gbs']:.0f} GB/s alone ({time.time() - t0:.0f}s)")
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2403_19708_amd as ca
    from synth import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    t_begin = time.time()
    stream = torch.cuda.current_stream()

    job = Job(torch, ca, args.config, args.seed, layers=args.layers)
    if args.two_call_save:
        job.fused_save = False
    job.loads_ahead = args.loads_ahead
    cfg = job.cfg
    L = job.L
    log(f"[bench] {cfg['name']}: L={L} B={job.B} Hq={job.Hq} Hkv={job.Hkv} D={job.D} kept-history={job.tot_n} new={job.tot_q} tokens, "
        f"attention {job.attn_bound}-bound (floor {job.attn_floor_us:.0f} us per layer)")
    want_hbm = (not args.no_hbm_leg) or args.tier == "hbm"
    if want_hbm:
        job.make_device_tier()
    log(f"[bench] device tensors ready after {time.time() - t_begin:.0f}s, {torch.cuda.memory_allocated() / 2**30:.1f} GiB on device")
    pinned_ok = args.tier == "pinned" or not args.no_sweeps
    host_k = host_v = None
    if pinned_ok:
        try:
            job.make_pinned_tier()
            host_k, host_v = job.tier_ptrs(job.pin_tier[0]), job.tier_ptrs(job.pin_tier[1])
            log(f"[bench] pinned tier ready after {time.time() - t_begin:.0f}s")
        except Exception as e:
            pinned_ok = False
            log(f"[bench] pinned tier failed: {e!r}")
            if args.tier == "pinned":
                raise
    dev_k = dev_v = None
    if want_hbm:
        dev_k, dev_v = job.tier_ptrs(job.dev_tier[0]), job.tier_ptrs(job.dev_tier[1])

    ctx = ca.Context(job.config(pipeline_depth=args.depth, load_mode=args.load_mode, save_mode=args.save_mode))

    # ---- headline leg ---------------------------------------------------------------------------------------
    # the events around the attention call and the copies cost nothing measurable next to a link-bound step
    if args.tier == "pinned":
        src_k, src_v, tier_name = host_k, host_v, "pinned-host"
        kinds = ["attn", "copy_in", "copy_out", "pack"]
    else:
        src_k, src_v, tier_name = dev_k, dev_v, "HBM-resident"
        kinds = ["attn"]
    dt, prof = job.timed(ctx, src_k, src_v, stream, args.warmup, args.steps, f"{tier_name} tier, timed", kinds=kinds)
    ms_step = dt / args.steps * 1e3
    value = job.tot_q / (dt / args.steps)
    att_us_live = prof["attn"][0] / prof["attn"][1] * 1e3
    attn_live = job.attn_figures(att_us_live)
    pipeline = pipeline_figures(job, dt, args.steps, prof) if args.tier == "pinned" else None
    if pipeline is not None:
        # the step is bound by the read stream, so what bounds the headline value is the host link, not a kernel
        peak = link_probe(torch)
        step_gbs = L * job.link_in_bytes / (dt / args.steps) / 1e9
        pipeline["link"] = dict(step_gbs=step_gbs, single_copy_gbs=peak, frac_of_single_copy=step_gbs / peak,
                                pcie5_x16_gbs=63.0, frac_of_pcie5_x16=step_gbs / 63.0,
                                note="step_gbs = tier bytes read per step / step time (everything else hidden or not); "
                                     "single_copy_gbs = one 320 MiB pinned-to-device copy on an idle GPU, measured in this run")
        log(f"[bench] host link: {step_gbs:.1f} GB/s over the whole step, {peak:.1f} GB/s for one large copy alone")

    parity = None
    if not args.no_check and job.layer0:
        parity = job.parity(job.out[0])
        if not parity["ok"]:
            log("[bench] PARITY FAILED: the numbers below are not valid")

    # every kernel bracketed, same tier: in-step durations of the move kernels
    dt_i, prof_i = job.timed(ctx, src_k, src_v, stream, 0, 1, f"{tier_name} tier, every kernel timed", timeline=True)
    kv_move = job.move_figures(prof_i)
    if pipeline is not None and prof_i.get("timeline"):
        pipeline["timeline"] = timeline_figures(prof_i["timeline"], args.timeline_file or None)
        pipeline["timeline"]["ms_step_instrumented"] = dt_i * 1e3

    # the dominant kernel of the step by GPU time: the attention call
    attn_kernel = "attn_dma_kernel"
    G = job.Hq // job.Hkv
    # the library rotates the keys once per layer when on average three or more 256-row tiles share them
    prerot = job.W <= 32768 and int(np.sum((job.new.astype(np.int64) * G + 255) // 256)) >= 3 * job.B
    if job.attn_bound == "mfma":
        roof = dict(kernel=attn_kernel, bound="mfma", achieved=attn_live["tflops"], peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=attn_live["frac_mfma_peak"], traffic=None, algorithmic_flops_per_launch=job.flops_layer)
    else:
        roof = dict(kernel=attn_kernel, bound="hbm", achieved=attn_live["gbs"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=attn_live["frac_hbm_peak"], traffic=None)
    roof["avg_launch_us"] = att_us_live
    roof["algorithmic_bytes_per_launch"] = job.attn_bytes
    roof["launch"] = ("one ca_cached_prefill_attn call inside the timed steps: rotate_keys_kernel + attn_dma_kernel (+ combine_kernel "
                      "when keys are split)" if prerot else "one ca_cached_prefill_attn call inside the timed steps")
    sustained = mfma_rate_probe()
    if sustained:
        log(f"[bench] matrix cores alone: {sustained['zero_operands_tflops']:.0f} TFLOP/s on zero operands, "
            f"{sustained['random_operands_tflops']:.0f} TFLOP/s on random operands")
    if sustained and job.attn_bound == "mfma":
        # context for frac: what back-to-back matrix instructions alone reach on this card (clock under load)
        roof["mfma_sustained"] = dict(sustained, frac_of_random_operand_rate=attn_live["tflops"] / sustained["random_operands_tflops"],
                                      note="measured by paper_2403_19708_amd/mfma_rate_probe in this run: v_mfma_f32_32x32x16_bf16 "
                                           "back to back, nothing else; peak above stays the published figure")
    traffic_file = os.path.join(ROOT, "profiles", f"hbm_traffic_cfg{args.config}.txt")
    if os.path.exists(traffic_file):
        kv = {}
        for line in open(traffic_file):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                kv[k.strip()] = v.split("#")[0].strip()
        if "attn_bytes_per_launch" in kv:
            roof["traffic"] = float(kv["attn_bytes_per_launch"])
            roof["traffic_source"] = f"profiles/hbm_traffic_cfg{args.config}.txt (rocprofv3 counter runs of this command)"

    # ---- the same step with the tier in HBM -----------------------------------------------------------------------
    hbm = None
    if want_hbm and args.tier == "pinned":
        hdt, hprof = job.timed(ctx, dev_k, dev_v, stream, 1, args.hbm_steps, "HBM-resident tier, every kernel timed")
        h_att = hprof["attn"][0] / hprof["attn"][1] * 1e3
        job.fused_save = False
        sdt, sprof = job.timed(ctx, dev_k, dev_v, stream, 0, 1, "HBM-resident tier, append and save as two calls")
        job.fused_save = True
        two = job.move_figures(sprof)
        one = job.move_figures(hprof, fused_device_tier=True)
        hbm = dict(ms_per_step=hdt / args.hbm_steps * 1e3, tokens_per_s=job.tot_q / (hdt / args.hbm_steps),
                   context_tokens_per_s=job.tot_k / (hdt / args.hbm_steps), attn=job.attn_figures(h_att), kv_move=one,
                   append_save=dict(one_call_in_step_us=one["append"]["avg_launch_us"],
                                    two_calls_in_step_us=(two["append"]["avg_launch_us"] or 0) + (two["pack"]["avg_launch_us"] or 0),
                                    ms_per_step_two_calls=sdt * 1e3,
                                    note="the new turn appended and saved by one kernel that reads it once (N in, 2N out), "
                                         "against the append kernel plus the pack kernel (2N in, 2N out)"),
                   note="same entry points; the load kernel reads the tier in place from device memory, no host link in the step")
    iso = job.isolated(ctx, dev_k if want_hbm else src_k, dev_v if want_hbm else src_v, stream)
    log("[bench] isolated: " + ", ".join(f"{k} {v['avg_launch_us']:.1f} us" for k, v in iso.items()))

    # ---- a plain device copy of known size: the reference the HBM byte counters are scaled by ---------------
    cal_n = 256 * 1024 * 1024 // 2
    cal_src = torch.empty(cal_n, dtype=torch.bfloat16, device=job.dev).normal_()
    cal_dst = torch.empty_like(cal_src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    cal_dst.copy_(cal_src)
    e0.record(); cal_dst.copy_(cal_src); e1.record(); torch.cuda.synchronize()
    copy_gbs = 2 * cal_n * 2 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del cal_src, cal_dst
    ctx.close()

    # ---- read-buffer experiments ------------------------------------------------------------------------------------
    sweep = None
    if not args.no_sweeps and pinned_ok:
        try:
            sweep = depth_sweep(torch, ca, job, host_k, host_v, stream, [1, 2, 4, 8], args)
        except Exception as e:
            log(f"[bench] depth sweep failed: {e!r}")
            sweep = dict(error=repr(e))

    cpu = None
    if not args.no_cpu_baseline and job.layer0:
        cpu = cpu_baseline(job)

    result_config = {"workload": cfg["name"], "index": args.config, "tier": tier_name, "n_layers": L, "batch": job.B, "n_q_heads": job.Hq,
                     "n_kv_heads": job.Hkv, "head_dim": job.D, "new_tokens": job.tot_q, "kept_history_tokens": job.tot_n,
                     "pipeline_depth": args.depth, "load_mode": args.load_mode,
                     "pinned_tier_gib": getattr(job, "pin_gib", 0.0) if args.tier == "pinned" else 0.0,
                     "pinned_tier_distinct_layers": getattr(job, "pin_distinct", 0) if args.tier == "pinned" else 0,
                     "tier_bytes_streamed_per_step_gib": L * job.link_in_bytes / 2**30,
                     "valid": not bool(args.layers)}
    context_tps = job.tot_k / (dt / args.steps)
    job.free()
    del job

    preload = None
    if not args.no_sweeps:
        try:
            preload = preload_sweep(torch, ca, args.seed)
            log("[bench] preload sweep: " + ", ".join(f"{r['name']} {r['ms']:.1f} ms" for r in preload["runs"]))
        except Exception as e:
            log(f"[bench] preload sweep failed: {e!r}")
            preload = dict(error=repr(e))

    decode = None
    if not args.no_decode:
        try:
            decode = decode_leg(torch, ca, dict(CONFIGS[2]), args.decode_steps, args.seed)
            log(f"[bench] decode leg: {decode['ms_per_step']:.2f} ms per step ({decode['ms_per_step_without_write_back']:.2f} without "
                f"write-back), attention {decode['attn_avg_launch_us']:.1f} us, {decode['attn_kv_read_gbs']:.0f} GB/s of K/V")
        except Exception as e:
            log(f"[bench] decode leg failed: {e!r}")
            decode = dict(error=repr(e))

    configs = []
    for tok in [t for t in args.summary_configs.split(",") if t.strip()]:
        idx = int(tok)
        if idx == args.config:
            continue
        try:
            configs.append(config_summary(torch, ca, idx, args.seed))
        except Exception as e:
            log(f"[bench] summary of config {idx} failed: {e!r}")
            configs.append(dict(index=idx, error=repr(e)))

    result = {
        "metric": "cached-prefill tokens/s + attn TFLOP/s (% bf16 MFMA peak); KV load/pack GB/s",
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": result_config,
        "context_tokens_per_s": context_tps,
        "attn": attn_live,
        "kv_move": kv_move,
        "roofline": roof,
        "cpu_baseline": cpu,
        "pipeline": pipeline,
        "hbm_resident_tier": hbm,
        "isolated": iso,
        "device_copy_gbs": copy_gbs,
        "mfma_sustained": sustained,
        "pipeline_depth_sweep": sweep,
        "preload_sweep": preload,
        "configs": configs,
        "decode": decode,
        "parity": parity,
        "wall_s": time.time() - t_begin,
    }
    print(json.dumps(result), flush=True)
    return 0 if (parity is None or parity["ok"]) else 1


if __name__ == "__main__":
    sys.exit(main())
