"""The one-call append + save of the new turn (Sections 3.2.2, 3.4): the pool and the tier must hold, bit for bit,
what the oracle's unpack puts into the pages and the pre-rotary rows of the new turn behind the saved history --
exactly what ca_kv_append_layer followed by ca_kv_save_layer produce."""
import numpy as np
import pytest
import torch

from harness import Case, GpuRun, torch_to_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tier,save_mode", [("device", 0), ("pinned", 0), ("pinned", 1), ("pinned", 2), ("device", 1)])
def test_append_save_bit_exact(tier, save_mode):
    # non-page-aligned kept histories, a conversation without history, one whose new turn is a single token
    case = Case([333, 0, 90, 515], [17, 129, 1, 64], [77, 0, 90, 3], 8, 2, 128, seed=41)
    run = GpuRun(case, tier=tier, save_mode=save_mode)
    try:
        run.rebase()
        run.load(0)
        run.ctx.kv_append_save_layer(0, run.k_new[0], run.v_new[0], run.k_pool[0], run.v_pool[0], run.host_k[0], run.host_v[0])
        run.attn(0)
        run.finish()
        for which, pool, host in (("k", run.k_pool[0], run.host_k[0]), ("v", run.v_pool[0], run.host_v[0])):
            assert np.array_equal(torch_to_bits(pool), case.oracle_pool(0, which)), which
            for c in range(case.B):
                got = torch_to_bits(host[c])
                hist, new = case.tensor(0, f"{which}_hist", c), case.tensor(0, f"{which}_new", c)
                assert np.array_equal(got[:case.hist_len[c]], hist), (which, c)      # history untouched
                assert np.array_equal(got[case.hist_len[c]:], new), (which, c)       # new turn behind it, pre-rotary bits
        for c in range(case.B):
            err = np.abs(run.out_f64(0, c) - case.oracle_out(0, c))
            assert err.max() <= 2e-2 and err.mean() <= 2e-3, c
    finally:
        run.close()


def test_append_save_equals_the_two_calls_on_a_d64_stack():
    case = Case([70, 200], [65, 9], [5, 0], 4, 4, 64, seed=42, n_layers=3, style=1)
    outs = []
    for fused in (False, True):
        run = GpuRun(case, tier="pinned")
        try:
            run.rebase()
            for l in range(case.n_layers):
                run.load(l)
            for l in range(case.n_layers):
                if fused:
                    run.ctx.kv_append_save_layer(l, run.k_new[l], run.v_new[l], run.k_pool[l], run.v_pool[l], run.host_k[l], run.host_v[l])
                    run.attn(l)
                else:
                    run.append(l); run.attn(l); run.save(l)
            run.finish()
            outs.append(([torch_to_bits(o).copy() for o in run.out],
                         [[torch_to_bits(t).copy() for t in run.host_k[l]] + [torch_to_bits(t).copy() for t in run.host_v[l]] for l in range(case.n_layers)],
                         [torch_to_bits(p).copy() for p in run.k_pool + run.v_pool]))
        finally:
            run.close()
    for a, b in zip(outs[0][0], outs[1][0]):
        assert np.array_equal(a, b)
    for la, lb in zip(outs[0][1], outs[1][1]):
        for a, b in zip(la, lb):
            assert np.array_equal(a, b)
    for a, b in zip(outs[0][2], outs[1][2]):
        assert np.array_equal(a, b)


def test_default_save_mode_picks_the_write_back_by_the_plan():
    """save_mode 0 on a pinned tier: copies out of a staging slot while the tokens to save are fewer than a fifth of
    the kept history loaded per layer, the pack kernel storing in place beyond that; the saved bits are the same."""
    few = Case([600, 500], [20, 30], [0, 0], 4, 2, 128, seed=43)          # 50 new against 1100 kept
    many = Case([100, 90], [60, 70], [0, 0], 4, 2, 128, seed=44)          # 130 new against 190 kept
    for case, staged in ((few, True), (many, False)):
        run = GpuRun(case, tier="pinned")
        try:
            run.rebase()
            run.load(0)
            run.ctx.profile_enable(True)
            run.ctx.kv_append_save_layer(0, run.k_new[0], run.v_new[0], run.k_pool[0], run.v_pool[0], run.host_k[0], run.host_v[0])
            run.finish()
            run.ctx.profile_enable(False)
            n_copy_out, n_pack = run.ctx.profile_read("copy_out")[1], run.ctx.profile_read("pack")[1]
            assert (n_copy_out, n_pack) == ((1, 0) if staged else (0, 1)), (staged, n_copy_out, n_pack)
            for which, host in (("k", run.host_k[0]), ("v", run.host_v[0])):
                for c in range(case.B):
                    got = torch_to_bits(host[c])
                    assert np.array_equal(got[:case.hist_len[c]], case.tensor(0, f"{which}_hist", c)), (which, c)
                    assert np.array_equal(got[case.hist_len[c]:], case.tensor(0, f"{which}_new", c)), (which, c)
        finally:
            run.close()
