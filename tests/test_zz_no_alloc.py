"""The attention entry point that allocates nothing (ca_cached_prefill_attn_static): the shares of split row
tiles go to a fixed array inside the library instead of the context's buffer.  Called through the C ABI twice
in a row, the second time with a smaller batch, each against the ordinary entry point on the same inputs (same
kernels, same order of operations: identical bits) and against the oracle at the contract tolerance.  A plan
whose shares exceed the array is refused and nothing is launched."""
import numpy as np
import pytest
import torch

import paper_2403_19708_amd as ca
from harness import Case, GpuRun, err_stats, torch_to_bits

pytestmark = pytest.mark.gpu


def one_call(case, check_oracle_convs):
    run = GpuRun(case, tier="device")
    try:
        run.rebase()
        items = run.ctx.rebase_read(6).reshape(-1, 8)
        n_shares = int((items[:, 6] >= 0).sum())
        assert n_shares > 0, "the case must split keys, or the scratch array is never used"
        run.load(0)
        run.append(0)
        run.attn(0)
        run.finish()
        want_bits = torch_to_bits(run.out[0]).copy()
        run.out[0].view(torch.int16).fill_(0x7FC0)          # NaN pattern: every element must be rewritten
        s = 1.0 / np.sqrt(case.head_dim)
        run.ctx.cached_prefill_attn_static(0, run.q[0], run.k_pool[0], run.v_pool[0], run.out[0], s, None)
        run.finish()
        got_bits = torch_to_bits(run.out[0])
        assert np.array_equal(got_bits, want_bits)
        for c in check_oracle_convs:
            mx, mean, _ = err_stats(run.out_f64(0, c), case.oracle_out(0, c))
            assert mx <= 2e-2 and mean <= 2e-3, (c, mx, mean)
        return n_shares
    finally:
        run.close()


def test_two_calls_in_a_row_the_second_smaller():
    # few, long row tiles: the planner splits their keys over workgroups
    big = Case(hist_len=[3900, 2500], new_len=[180, 97], keep_start=[0, 13], n_q_heads=8, n_kv_heads=4, head_dim=128, seed=31)
    small = Case(hist_len=[1500], new_len=[40], keep_start=[100], n_q_heads=4, n_kv_heads=2, head_dim=128, seed=32)
    n_big = one_call(big, [0, 1])
    n_small = one_call(small, [0])
    assert n_small < n_big                                   # stale shares of the first call stay in the array behind it


def test_a_plan_beyond_the_array_is_refused():
    # 64 kv heads x one long conversation: hundreds of shares of 256-row tiles, more than 32 MiB of partial results
    case = Case(hist_len=[7900], new_len=[200], keep_start=[0], n_q_heads=64, n_kv_heads=64, head_dim=128, seed=33, window=8192)
    run = GpuRun(case, tier="device")
    try:
        run.rebase()
        items = run.ctx.rebase_read(6).reshape(-1, 8)
        n_shares = int((items[:, 6] >= 0).sum())
        tile_rows = 256 if case.new_len.max() * (case.n_q_heads // case.n_kv_heads) > 128 else 128
        if n_shares * tile_rows * (case.head_dim + 2) * 4 <= 32 << 20:
            pytest.skip(f"planner made only {n_shares} shares")
        run.load(0)
        run.append(0)
        run.finish()
        run.out[0].view(torch.int16).fill_(0x7FC0)
        with pytest.raises(ca.CaError) as e:
            run.ctx.cached_prefill_attn_static(0, run.q[0], run.k_pool[0], run.v_pool[0], run.out[0], 0.088, None)
        assert e.value.status_name == "CA_ERR_OUT_OF_RANGE"
        run.finish()
        assert np.all(torch_to_bits(run.out[0]) == 0x7FC0)   # nothing was launched
        run.attn(0)                                          # the ordinary entry point serves the same plan
        run.finish()
        mx, mean, _ = err_stats(run.out_f64(0, 0)[:, :2], case.oracle_out(0, 0, heads=[0, 1]))
        assert mx <= 2e-2 and mean <= 2e-3
    finally:
        run.close()
