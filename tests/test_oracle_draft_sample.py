"""Pins for the oracle's draft-token draw, "x_i ~ q_i" of Algorithm 1's generation loop (CPU only).

What fixes the expected values: the Gumbel-max theorem (the argmax of ln q_v + Gumbel noise follows
q), an independent pure-Python evaluation of the same argmax from the published Philox algorithm
(which pins the counter layout), and the independence of the draw from the verification step's
streams."""
import math

import numpy as np

from philox_ref import philox4x32_10

NEG_INF = float("-inf")


def softmax(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def test_draft_tokens_follow_the_softmax_of_the_row(oracle):
    V, B = 9, 60000
    z = np.float32([2.0, 1.0, 0.0, -1.0, NEG_INF, 0.5, 0.5, -3.0, 1.5])
    rows = np.broadcast_to(z, (B, V)).copy()
    tok, gap = oracle.draft_sample(rows, seed=12, step=3)
    q = softmax(z)
    counts = np.bincount(tok, minlength=V).astype(np.float64)
    assert counts[4] == 0                                            # masked token is never drawn
    keep = q > 0
    chi2 = float((((counts - B * q) ** 2)[keep] / (B * q[keep])).sum())
    assert chi2 < 31.8                                               # 7 dof, ~4e-5
    assert abs(counts[5] - counts[6]) < 5 * math.sqrt(counts[5] + counts[6])
    assert (gap > 0).all()


def test_draw_equals_an_independent_evaluation_from_the_published_generator(oracle):
    rng = np.random.default_rng(5)
    V, B = 37, 6
    rows = np.float32(rng.normal(0, 2, (B, V)))
    rows[2, 5:9] = NEG_INF
    seed, step, round0 = 0x1234567887654321, 11, 7
    seq = np.uint32([3, 9, 27, 81, 243, 4000000000])
    tok, gap = oracle.draft_sample(rows, seed=seed, step=step, seq_id=seq, round0=round0)
    for b in range(B):
        lq = np.log(softmax(rows[b].astype(np.float64)), where=rows[b] > NEG_INF,
                    out=np.full(V, NEG_INF))
        keys = []
        for v in range(V):
            w = philox4x32_10([v >> 2, step | (2 << 16), round0, int(seq[b])],
                              [seed & 0xFFFFFFFF, seed >> 32])[v & 3]
            u = (w + 0.5) / 2.0 ** 32
            keys.append(lq[v] - math.log(-math.log(u)))
        order = np.argsort(keys)
        assert tok[b] == order[-1]
        assert gap[b] == np.float64(keys[order[-1]]) - np.float64(keys[order[-2]]) or \
            abs(gap[b] - (keys[order[-1]] - keys[order[-2]])) < 1e-12


def test_draw_depends_on_every_counter_field_and_not_on_the_verification_streams(oracle):
    rng = np.random.default_rng(1)
    V, B = 50, 400
    z = np.float32(rng.normal(0, 1, V))
    rows = np.broadcast_to(z, (B, V)).copy()
    base, _ = oracle.draft_sample(rows, seed=1, step=0, round0=0)
    for kw in (dict(seed=2), dict(step=1), dict(round0=1), dict(seq_id=np.arange(B) + B)):
        other, _ = oracle.draft_sample(rows, **{**dict(seed=1, step=0, round0=0), **kw})
        agree = (other == base).mean()
        assert agree < 0.2, kw                                       # sum q^2 ~ 0.05 for this row
    per_seq, _ = oracle.draft_sample(rows, seed=1, step=0, rounds=np.full(B, 5, np.uint32))
    scalar, _ = oracle.draft_sample(rows, seed=1, step=0, round0=5)
    assert np.array_equal(per_seq, scalar)
    # the verification step's token for the same row, position, round and sequence uses stream 1
    target = np.broadcast_to(z, (B, 1, V)).copy()
    out = oracle.verify(target, np.zeros((B, 0, V), np.float32), np.zeros((B, 0), np.int32), seed=1)
    assert (out["next_token"] == base).mean() < 0.2


def test_inactive_and_broken_rows_give_no_token(oracle):
    V = 12
    rows = np.zeros((5, V), np.float32)
    rows[1, 3] = np.nan
    rows[2, :] = NEG_INF
    rows[3, 7] = np.inf
    tok, _ = oracle.draft_sample(rows, active=[1, 1, 1, 1, 0], seed=3)
    assert tok[0] >= 0 and list(tok[1:]) == [-1, -1, -1, -1]
    onehot = np.full((1, V), NEG_INF, np.float32); onehot[0, 9] = 2.0
    tok, gap = oracle.draft_sample(onehot, seed=3)
    assert tok[0] == 9 and gap[0] == math.inf
