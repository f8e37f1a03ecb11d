"""Decode phase through the same entry points (Section 3.2.2): after the prefill of a turn every
step appends one token per conversation behind the context, attends it over the whole context with
rotary-on-load, and the generated tokens' keys/values are written back to the tier asynchronously,
a few steps at a time, without the host waiting.  Each step must equal the oracle, and at the end the
tier must hold the pre-rotary bits of every token, prompt and generated alike."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_19708_amd as ca
from synth import bf16_bits_to_f64, draw_block_table, draw_values_bf16

from harness import P, bits_to_torch, torch_to_bits
from test_gpu_parity import check_contract, check_tight

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(8, 2, 128, 0), (4, 4, 64, 1)], ids=["gqa4-d128", "mha-d64-interleaved"])
def test_decode_steps_with_asynchronous_write_back(shape):
    Hq, Hkv, D, style = shape
    prompt = np.array([200, 37, 500], np.int32)
    steps, flush_every = 7, 3
    B, W, seed = len(prompt), 1024, 71
    total = prompt + steps
    full_k = [draw_values_bf16((int(total[c]), Hkv, D), seed, 10 + c) for c in range(B)]
    full_v = [draw_values_bf16((int(total[c]), Hkv, D), seed, 20 + c) for c in range(B)]
    full_q = [draw_values_bf16((int(total[c]), Hq, D), seed, 30 + c) for c in range(B)]
    tier_k = [torch.zeros((int(total[c]), Hkv, D), dtype=torch.bfloat16).pin_memory() for c in range(B)]
    tier_v = [torch.zeros((int(total[c]), Hkv, D), dtype=torch.bfloat16).pin_memory() for c in range(B)]
    dev = torch.device("cuda:0")
    pages = (total + P - 1) // P
    num_pages = int(pages.sum()) + 3
    bt = draw_block_table(pages, num_pages, seed)              # pages for the whole generation, fixed
    k_pool = torch.zeros((num_pages, Hkv, P, D), dtype=torch.bfloat16, device=dev)
    v_pool = torch.zeros_like(k_pool)
    w = bf16_bits_to_f64
    scale = 1.0 / np.sqrt(D)
    # the context already in the pool plays the part of the kept history; nothing is loaded for it
    cfg = ca.Config(n_layers=1, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, max_positions=W, max_seqs=B, rope_style=style,
                    max_batch_kv_tokens=int(total.sum()) + 64, max_batch_q_tokens=int(prompt.sum()) + 16, require_load=0)

    def run_turn(ctx, have, new):
        """have[c] tokens are in the pool; process the next new[c] tokens; returns bf16 bits of the output"""
        take = lambda full: bits_to_torch(np.concatenate([full[c][have[c]:have[c] + new[c]] for c in range(B)]), dev)
        q, kn, vn = take(full_q), take(full_k), take(full_v)
        out = torch.zeros_like(q)
        ctx.rope_rebase(have, np.zeros(B, np.int32), new, bt, num_pages)
        ctx.kv_append_layer(0, kn, vn, k_pool, v_pool)
        ctx.cached_prefill_attn(0, q, k_pool, v_pool, out, scale)
        return out, (q, kn, vn)

    def check(out, have, new, tight):
        got = torch_to_bits(out)
        at = 0
        for c in range(B):
            h, n = int(have[c]), int(new[c])
            want = oracle.cached_attention(w(full_k[c][:h]), w(full_v[c][:h]), w(full_q[c][h:h + n]),
                                           w(full_k[c][h:h + n]), w(full_v[c][h:h + n]), keep_start=0, style=style)
            check_contract(w(got[at:at + n]), want, (have.tolist(), c))
            if tight:
                check_tight(w(got[at:at + n]), want, h, (have.tolist(), c))
            at += n

    with ca.Context(cfg) as ctx:
        have = np.zeros(B, np.int32)
        out, keep_alive = run_turn(ctx, have, prompt)                       # prefill of the prompt (no history)
        ctx.kv_save_layer(0, k_pool, v_pool, tier_k, tier_v)                # prompt tokens -> tier rows [0, prompt)
        ctx.sync(); torch.cuda.synchronize()
        check(out, have, prompt, tight=True)
        have = prompt.copy()
        saved = prompt.copy()
        one = np.ones(B, np.int32)
        pending = []
        for s in range(steps):
            out, bufs = run_turn(ctx, have, one)
            pending.append((out, bufs, have.copy()))
            have = have + 1
            if (s + 1) % flush_every == 0 or s == steps - 1:
                # write back what was generated since the last flush; the host does not wait for it
                ctx.kv_save_layer(0, k_pool, v_pool, tier_k, tier_v, tok_begin=saved, tok_end=have,
                                  dst_tok_offset=saved.astype(np.int64))
                saved = have.copy()
        ctx.sync(); torch.cuda.synchronize()
        for out, _, had in pending:
            check(out, had, one, tight=False)
        for c in range(B):
            assert np.array_equal(torch_to_bits(tier_k[c]), full_k[c]), c
            assert np.array_equal(torch_to_bits(tier_v[c]), full_v[c]), c
