"""CPU checks of the seeded input generators (shapes, dtypes, determinism, intended structure)."""
import numpy as np
import torch

from paper_2512_11280_amd import workloads as wl


def test_tiny_config_shape_and_determinism():
    a, b = wl.config_tiny(), wl.config_tiny()
    assert a.target.shape == (1, 5, 32000) and a.draft.shape == (1, 4, 32000)
    assert a.target.dtype == torch.float32 and a.draft_tokens.dtype == torch.int32
    assert torch.equal(a.target, b.target) and torch.equal(a.draft_tokens, b.draft_tokens)
    assert a.state["nA"].sum() == 0 and a.state["T_G"][0] == 0           # paper-default state
    c = wl.config_tiny(seed=1)
    assert not torch.equal(a.target, c.target)


def test_single_stream_has_two_entropy_regimes():
    b = wl.config_single_stream(V=20000)
    assert b.target.dtype == torch.bfloat16 and b.draft.shape == (1, 8, 20000)
    sd = b.target[0].float().std(dim=-1)
    assert sd[:4].min() > 5 and sd[4:8].max() < 1.2


def test_batched_state_encodes_per_sequence_thresholds():
    b = wl.config_batched(B=4, k=2, V=1000)
    st = b.state
    assert st["nA"].tolist() == [64] * 4 and st["LA"].shape == (4, 128)
    la = st["LA"][:, :64].mean(1)
    lr = st["LR"][:, :64].mean(1)
    assert np.all(la < lr)
    assert np.all((st["LA"][:, :64] > 0) & (st["LA"][:, :64] < 1))
    assert np.allclose((la + lr) / 2, st["tau"], atol=0.05)


def test_large_config_has_independent_rows():
    b = wl.config_large(B=6, k=8, V=3000)
    t, d = b.target[:, :8].float(), b.draft.float()
    corr = ((t - t.mean(-1, keepdim=True)) * (d - d.mean(-1, keepdim=True))).mean(-1) / (t.std(-1) * d.std(-1))
    assert (corr > 0.9).any() and (corr < 0.2).any()


def test_closed_loop_source_walks_alpha():
    s = wl.ClosedLoopSource(3, 500, 4, seed=5)
    a0 = s.alpha.clone()
    t, d, x = s.next_round()
    assert t.shape == (3, 5, 500) and d.shape == (3, 4, 500) and x.shape == (3, 4)
    assert torch.allclose((s.alpha - a0).abs(), torch.full((3,), 0.02), atol=1e-6) or \
        ((s.alpha == 0.4) | (s.alpha == 0.99)).any()
    assert ((x >= 0) & (x < 500)).all()
