"""The streaming kernel that serves decode steps (every (conversation, kv head) has one or two stacked
query rows): outputs against the oracle for both head sizes and pair conventions, grouped heads, two
new tokens, truncated and empty histories, contexts that end anywhere inside a page, and long contexts
whose keys the host splits over several workgroups.  attn_variant 4 refuses any other kind of batch,
so a pass here is a pass of that kernel and not of the matrix-core one."""
import numpy as np
import pytest

import oracle  # noqa: F401  (Case uses it)
import paper_2403_19708_amd as ca
from harness import Case, GpuRun, torch_to_bits
from test_gpu_parity import check_contract, check_tight

pytestmark = pytest.mark.gpu


def run_case(case, **knobs):
    run = GpuRun(case, tier="device", attn_variant=4, **knobs)
    try:
        run.rebase()
        run.run_layer(0)
        run.finish()
        for c in range(case.B):
            check_contract(run.out_f64(0, c), case.oracle_out(0, c), c)
            check_tight(run.out_f64(0, c), case.oracle_out(0, c), int(case.n_keep[c]), c)
        # the kernel writes nothing but its output: the pools hold exactly what load and append put there
        for which, pool in (("k", run.k_pool[0]), ("v", run.v_pool[0])):
            assert np.array_equal(torch_to_bits(pool), case.oracle_pool(0, which)), which
        return run.ctx.rebase_read(6).reshape(-1, 8)
    finally:
        run.close()


SHAPES = [  # Hq, Hkv, D, style
    (4, 4, 128, 0), (4, 4, 128, 1), (4, 4, 64, 0), (4, 4, 64, 1), (4, 2, 128, 0), (6, 3, 64, 1),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "hq%d-hkv%d-d%d-style%d" % s)
def test_one_new_token_per_conversation(shape):
    Hq, Hkv, D, style = shape
    hist = [0, 1, 15, 16, 17, 63, 64, 200, 333, 1000, 1027]
    keep = [0, 0, 3, 0, 16, 0, 1, 77, 0, 500, 0]
    case = Case(hist, [1] * len(hist), keep, Hq, Hkv, D, seed=40 + D + style, style=style, window=2048)
    run_case(case)


@pytest.mark.parametrize("shape", [(2, 2, 128, 0), (2, 2, 64, 1)], ids=["d128-half", "d64-interleaved"])
def test_two_new_tokens_have_their_own_causal_ends(shape):
    Hq, Hkv, D, style = shape
    case = Case([0, 30, 129, 700], [2, 2, 1, 2], [0, 7, 0, 0], Hq, Hkv, D, seed=51, style=style, window=1024)
    run_case(case)


@pytest.mark.parametrize("split", [0, 1], ids=["split", "whole"])
def test_long_contexts_are_split_over_workgroups_and_merged(split):
    case = Case([9000, 4100], [1, 1], [0, 37], 2, 2, 128, seed=52, window=16384)
    items = run_case(case, attn_split=split)
    live = items[items[:, 0] >= 0]
    if split == 0:
        assert len(live) > 4 and (live[:, 6] >= 0).all()          # every item is a share of a split unit
        for c in range(2):
            for g in range(2):
                mine = live[(live[:, 0] == c) & (live[:, 1] == g)]
                order = np.argsort(mine[:, 4])
                assert mine[order[0], 4] == 0 and (mine[order[1:], 4] == mine[order[:-1], 5]).all()   # shares tile the keys
    else:
        assert len(live) == 4 and (live[:, 6] < 0).all()


def test_peaky_scores():
    """queries scaled up so that a few keys carry the whole softmax: masking or indexing slips cannot hide"""
    case = Case([500, 77], [1, 1], [0, 0], 2, 2, 128, seed=53, window=1024, q_scale=6.0)
    run_case(case)


def test_any_other_batch_is_refused():
    case = Case([100], [3], [0], 2, 2, 128, seed=54, window=512)
    run = GpuRun(case, tier="device", attn_variant=4)
    try:
        run.rebase()
        run.load(0)
        run.append(0)
        with pytest.raises(ca.CaError) as e:
            run.attn(0)
        assert e.value.status_name == "CA_ERR_UNSUPPORTED"
        run.finish()
    finally:
        run.close()
