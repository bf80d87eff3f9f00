"""GPU mirror of the tie pin: two vocabulary elements whose Philox noise words are equal get equal
weights, so their Gumbel keys are bit-identical and only the lowest-index rule decides the draw
(correction, bonus and excluded-token draws of adasd_verify; the drafted token of adasd_draft_step).
Expected values are the oracle's, which tests/test_oracle_tiebreak.py pins on the CPU."""
import numpy as np
import pytest
import torch

import philox_ref
from test_oracle_tiebreak import KNOWN, SEED, V, tied_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def am():
    import paper_2512_11280_amd as am
    am.load_library()
    assert torch.cuda.is_available()
    return am


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", ["residual", "bonus", "excluded"])
def test_verify_keeps_the_lowest_index_on_an_exact_tie(am, oracle, kind, dtype):
    ws = am.Workspace(1, 1, V, dtype)
    for i, j in KNOWN[1]:
        t, d, x, k = tied_rows(i, j, kind)
        t, d = torch.tensor(t).to(dtype), torch.tensor(d).to(dtype)
        opt = am.Options(relaxed_off=1, base_test=1 if kind == "excluded" else 0)
        ref = oracle.verify(t, d, x, draft_len=np.int32([k]), seed=SEED, relaxed_off=1, base_test=opt.base_test)
        assert ref["next_token"][0] == i and ref["top2_gap"][0] == 0.0
        out = am.verify(t.cuda(), d.cuda(), torch.tensor(x).cuda(), ws, draft_len=torch.tensor([k], dtype=torch.int32).cuda(),
                        seed=SEED, options=opt)
        torch.cuda.synchronize()
        assert out.n_accept.item() == 0
        assert out.next_token.item() == i, (kind, i, j, out.next_token.item())
        assert out.status.item() & am.binding.ST_EXACT_PATH      # a tie is a close call: settled in float64


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_draft_step_keeps_the_lowest_index_on_an_exact_tie(am, oracle, dtype):
    ws = am.Workspace(1, 1, V, dtype)
    for i, j in KNOWN[2]:
        z = torch.full((1, V), -40.0)
        z[0, [i, j]] = 1.5
        z = z.to(dtype)
        tok, gap = oracle.draft_sample(z, step=0, seed=SEED)
        assert tok[0] == i and gap[0] == 0.0
        _, _, x, st = am.draft_step(z.cuda(), ws, step=0, k_max=20, seed=SEED)
        torch.cuda.synchronize()
        assert x.item() == i, (i, j, x.item())


def test_the_noise_words_of_the_pairs_are_equal_on_the_device_too(am, oracle):
    """If the kernels' Philox differed from the oracle's on these counters, the tie cases above would
    pass for the wrong reason: three elements with the SAME weight, two of them a pair; the draw must be
    what the oracle says for every pair (a pair member wins only if its word beats the third one's)."""
    ws = am.Workspace(1, 1, V, torch.float32)
    for i, j in KNOWN[1]:
        t = np.full((1, 2, V), -40.0, np.float32)
        third = (i + j) // 2
        t[0, :, [i, j, third]] = 3.0
        d = np.full((1, 1, V), -40.0, np.float32)
        x = np.int32([[77]])
        ref = oracle.verify(t, d, x, draft_len=np.int32([0]), seed=SEED, relaxed_off=1)
        out = am.verify(torch.tensor(t).cuda(), torch.tensor(d).cuda(), torch.tensor(x).cuda(), ws,
                        draft_len=torch.zeros(1, dtype=torch.int32).cuda(), seed=SEED, options=am.Options(relaxed_off=1))
        torch.cuda.synchronize()
        assert out.next_token.item() == ref["next_token"][0]


@pytest.mark.parametrize("kind", ["residual", "bonus", "excluded"])
def test_column_sharded_round_keeps_the_lowest_index_on_an_exact_tie(am, oracle, kind):
    """The same tied rows through the column-sharded calls: the two elements of a pair sit in different
    holders' columns (or both in one), their records travel through the pick and settle calls with equal
    keys, and every replica must name the lower index."""
    from paper_2512_11280_amd import workloads as wl
    from test_gpu_parity import _sharded_decisions, _sharded_tokens
    for i, j in KNOWN[1]:
        t, d, x, k = tied_rows(i, j, kind)
        opt = dict(relaxed_off=1, base_test=1 if kind == "excluded" else 0)
        ref = oracle.verify(t, d, x, draft_len=np.int32([k]), seed=SEED, **opt)
        assert ref["next_token"][0] == i and ref["top2_gap"][0] == 0.0
        batch = wl.VerifyBatch(torch.tensor(t), torch.tensor(d), torch.tensor(x), torch.tensor([k], dtype=torch.int32),
                               wl.empty_state(1, 8), SEED)
        options = am.Options(**opt)
        ctx = _sharded_decisions(am, batch, 4, options=options)
        outs = ctx[0]
        _sharded_tokens(am, batch, ctx, outs)
        for o in outs:
            st = int(o.status.item())
            assert o.next_token.item() == i, (kind, i, j, o.next_token.item())
            assert st & am.binding.ST_EXACT_PATH and not st & am.binding.ST_UNSETTLED, (kind, i, j, st)
