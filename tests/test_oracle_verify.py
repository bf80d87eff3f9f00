"""Pins for the oracle's verification, sampling and update steps (CPU only).

What fixes the expected values: the theorem that speculative sampling emits tokens
distributed exactly as the target (Section 2.1.3), the Gumbel-max theorem, inputs
constructed so that every decision is forced, and the initial conditions and update
lines of Algorithm 1."""
import itertools
import math

import numpy as np
import pytest

from oracle import new_state

NEG_INF = float("-inf")


def softmax(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def chi2_stat(counts, probs):
    n = counts.sum()
    exp = n * probs
    keep = exp > 0
    return float(((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum())


# --------------------------------------------------------------- laws of the emitted tokens
def test_speculative_sampling_emits_the_target_distribution(oracle):
    """k=1, Bayesian test off.  First emitted token = draft token if accepted, else the
    re-sampled token; its law must be p exactly, and P(accept) = sum_v min(p_v, q_v)."""
    rng = np.random.default_rng(11)
    V, B = 6, 60000
    zp = np.float32([1.2, -0.3, 0.4, 2.0, -1.5, 0.0])
    zq = np.float32([0.1, 1.4, 0.4, 0.5, -0.2, NEG_INF])       # one token the draft never proposes
    zp2 = np.float32([0.0, 0.5, -0.5, 1.0, 0.2, -1.0])         # bonus row
    p, q, p2 = softmax(zp), softmax(zq), softmax(zp2)
    target = np.broadcast_to(np.stack([zp, zp2]), (B, 2, V)).copy()
    draft = np.broadcast_to(zq, (B, 1, V)).copy()
    x = rng.choice(V, size=(B, 1), p=q).astype(np.int32)
    out = oracle.verify(target, draft, x, seed=2024, relaxed_off=1)

    acc = out["n_accept"] == 1
    assert acc.mean() == pytest.approx(np.minimum(p, q).sum(), abs=4 * 0.5 / math.sqrt(B))
    first = np.where(acc, x[:, 0], out["next_token"])
    c1 = np.bincount(first, minlength=V).astype(np.float64)
    assert chi2_stat(c1, p) < 25.7            # 5 dof, P(chi2 > 25.7) ~ 1e-4
    # after a full acceptance the extra token follows the next target row
    c2 = np.bincount(out["next_token"][acc], minlength=V).astype(np.float64)
    assert chi2_stat(c2, p2) < 25.7
    # a re-sampled token always comes from where the target puts more mass than the draft
    rej_tok = out["next_token"][~acc]
    assert np.all(p[rej_tok] > q[rej_tok])
    resid = np.maximum(p - q, 0)
    c3 = np.bincount(rej_tok, minlength=V).astype(np.float64)
    assert chi2_stat(c3, resid / resid.sum()) < 25.7


def test_bonus_token_follows_softmax_with_no_drafts(oracle):
    """k_b = 0: the step degenerates to sampling one token from the target row (Gumbel-max)."""
    V, B = 8, 50000
    z = np.float32([2.0, 1.0, 0.0, -1.0, NEG_INF, 0.5, 0.5, -3.0])
    target = np.broadcast_to(z, (B, 3, V)).copy()
    draft = np.zeros((B, 2, V), np.float32)
    out = oracle.verify(target, draft, np.zeros((B, 2), np.int32), draft_len=np.zeros(B, np.int32),
                        seed=5)
    assert np.all(out["n_accept"] == 0)
    counts = np.bincount(out["next_token"], minlength=V).astype(np.float64)
    assert counts[4] == 0                                     # masked token is never drawn
    assert chi2_stat(counts, softmax(z)) < 29.9               # 6 dof, ~4e-5
    # equal logits are drawn equally often (no index bias away from exact ties)
    assert abs(counts[5] - counts[6]) < 5 * math.sqrt(counts[5] + counts[6])


def test_draws_depend_on_seed_sequence_round_and_position(oracle):
    V = 64
    rng = np.random.default_rng(0)
    t = np.float32(rng.normal(0, 1, (1, 2, V)))
    d = np.float32(rng.normal(0, 1, (1, 1, V)))
    x = np.int32([[3]])
    runs = {}
    for name, kw in dict(a=dict(seed=1), b=dict(seed=2), c=dict(seed=1, seq_id=[9]),
                         d=dict(seed=1, round0=4), e=dict(seed=1, rounds=[4])).items():
        toks = []
        for trial in range(40):  # vary the round to collect a sequence of draws
            kw2 = dict(kw)
            if "rounds" in kw2:
                kw2["rounds"] = [kw2["rounds"][0] + trial]
            else:
                kw2["round0"] = kw2.get("round0", 0) + trial
            toks.append(int(oracle.verify(t, d, x, relaxed_off=1, **kw2)["next_token"][0]))
        runs[name] = toks
    assert runs["a"] != runs["b"] and runs["a"] != runs["c"] and runs["a"] != runs["d"]
    assert runs["d"] == runs["e"]                     # per-sequence round array == scalar round
    assert runs["a"][4:] == runs["d"][:-4]            # round0=4 is the same stream shifted


# --------------------------------------------------------------- forced decisions
def _forced_rows(V=6):
    """Row pairs whose decisions do not depend on the random numbers.
    S : p == q                    -> ratio 1, base test always accepts, d = 0
    D1: p(x)=0, small distance    -> base test always rejects
    D2: p(x)=0, large distance    -> base test always rejects"""
    base = np.float32([0.5, 0.0, -0.5, 1.0, 0.2, -1.0])
    x = 1
    s = (base, base)
    p1 = base.copy(); p1[x] = NEG_INF
    q1 = base.copy()
    p2 = np.float32([0.0, NEG_INF, 4.0, NEG_INF, NEG_INF, 0.0])
    q2 = np.float32([0.0, 3.0, NEG_INF, NEG_INF, NEG_INF, -2.0])
    return dict(S=s, D1=(p1, q1), D2=(p2, q2)), x


def test_truth_table_of_the_two_tests_and_first_reject(oracle):
    rows, x = _forced_rows()
    V = 6
    d1 = math.sqrt(oracle.jsd(*rows["D1"]) / math.log(2))
    d2 = math.sqrt(oracle.jsd(*rows["D2"]) / math.log(2))
    assert 0 < d1 < 0.5 < d2 < 1
    # history: accepted distances tightly around d1, rejected tightly around d2
    LA = np.float32([[d1 - 0.01, d1, d1 + 0.01, d1 + 0.005]])
    LR = np.float32([[d2 - 0.01, d2, d2 + 0.01, d2 - 0.005]])
    assert oracle.posterior(d1, LA[0], LR[0]) > 1 - 1e-12
    assert oracle.posterior(d2, LA[0], LR[0]) < 1e-12
    bonus = np.float32([0, 1, 2, 3, 4, 5])
    for k in (1, 2, 3, 4):
        for pattern in itertools.product("S D1 D2".split(), repeat=k):
            t = np.stack([rows[c][0] for c in pattern] + [bonus])[None]
            d = np.stack([rows[c][1] for c in pattern])[None]
            out = oracle.verify(t, d, np.full((1, k), x, np.int32), LA=LA, LR=LR,
                                nA=[4], nR=[4], seed=77, round0=k)
            expect = next((i for i, c in enumerate(pattern) if c == "D2"), k)
            assert out["n_accept"][0] == expect, pattern
            for i, c in enumerate(pattern):
                m = int(out["accept_mask"][0, i])
                assert (m & 1) == (1 if c == "S" else 0), (pattern, i)
                if c == "D1":
                    assert m == 2
                if c == "D2":
                    assert m == 0
            tok = int(out["next_token"][0])
            if expect < k:   # re-sampled from max(0, p - q) of the D2 pair: support is {2, 5}
                assert tok in (2, 5)
            else:
                assert 0 <= tok < V
            assert out["status"][0] == 0
            # with the Bayesian test off every D1 is a rejection too
            out2 = oracle.verify(t, d, np.full((1, k), x, np.int32), LA=LA, LR=LR, nA=[4], nR=[4],
                                 seed=77, relaxed_off=1)
            expect2 = next((i for i, c in enumerate(pattern) if c != "S"), k)
            assert out2["n_accept"][0] == expect2
            # MAP rule gives the same decisions here (posteriors are ~0 or ~1)
            out3 = oracle.verify(t, d, np.full((1, k), x, np.int32), LA=LA, LR=LR, nA=[4], nR=[4],
                                 seed=77, reject_rule=1)
            assert out3["n_accept"][0] == expect


def test_statistics_are_reported_for_every_drafted_position_and_padding_is_zero(oracle):
    rows, x = _forced_rows()
    bonus = np.float32([0, 1, 2, 3, 4, 5])
    pattern = ["D2", "S", "D1", "S"]                       # rejected at position 0
    t = np.stack([rows[c][0] for c in pattern] + [bonus])[None]
    d = np.stack([rows[c][1] for c in pattern])[None]
    out = oracle.verify(t, d, np.full((1, 4), x, np.int32), draft_len=[3], seed=1)
    assert out["n_accept"][0] == 0
    assert out["d_js"][0, 2] > 0 and out["H_q"][0, 1] > 0          # after the rejection: still computed
    assert out["d_js"][0, 1] == 0.0
    for name in ("H_p", "H_q", "d_js", "p_accept", "accept_mask"):
        assert out[name][0, 3] == 0                                  # beyond draft_len: filler
    for i, c in enumerate(pattern[:3]):
        assert out["H_p"][0, i] == pytest.approx(oracle.row_stats(rows[c][0])[1], rel=1e-14)
        assert out["H_q"][0, i] == pytest.approx(oracle.row_stats(rows[c][1])[1], rel=1e-14)
        assert out["d_js"][0, i] == pytest.approx(
            math.sqrt(oracle.jsd(*rows[c]) / math.log(2)), rel=1e-14)


def test_ragged_draft_lengths_use_the_right_bonus_row(oracle):
    # all positions identical rows -> everything accepted -> bonus row index = draft_len[b]
    V, K = 5, 3
    same = np.float32([0.0, 0.1, 0.2, 0.3, 0.4])
    t = np.tile(same, (4, K + 1, 1))
    for b in range(4):
        for i in range(K + 1):
            t[b, i] = NEG_INF
            t[b, i, i] = 0.0                   # row i of the target is one-hot on token i
    d = t[:, :K].copy()
    x = np.tile(np.arange(K, dtype=np.int32), (4, 1))
    out = oracle.verify(t, d, x, draft_len=[0, 1, 2, 3], seed=3)
    assert list(out["n_accept"]) == [0, 1, 2, 3]
    assert list(out["next_token"]) == [0, 1, 2, 3]
    with pytest.raises(ValueError):
        oracle.verify(t, d, x, draft_len=[0, 1, 2, 4])


def test_status_bits(oracle):
    from oracle.pyoracle import ST_BAD_TOKEN, ST_NONFINITE, ST_ZERO_MASS
    z = np.float32([0.3, -0.2, 1.0, 0.0])
    t = np.stack([z, z])[None]
    d = z[None, None]
    # out-of-range token: base test fails; residual of identical rows has no mass -> sample p
    out = oracle.verify(t, d, np.int32([[7]]), seed=1)
    assert out["n_accept"][0] == 0 and out["status"][0] == ST_BAD_TOKEN | ST_ZERO_MASS
    assert 0 <= out["next_token"][0] < 4
    out = oracle.verify(t, d, np.int32([[-1]]), seed=1)
    assert out["status"][0] & ST_BAD_TOKEN
    # NaN in the draft row: position rejected, statistics NaN, no token can be drawn from it
    dn = d.copy(); dn[0, 0, 2] = float("nan")
    out = oracle.verify(t, dn, np.int32([[0]]), seed=1)
    assert out["status"][0] & ST_NONFINITE and out["n_accept"][0] == 0
    assert math.isnan(out["d_js"][0, 0]) and out["next_token"][0] == -1
    # +inf in the bonus row only: statistics fine, token unavailable
    tn = t.copy(); tn[0, 1, 0] = float("inf")
    out = oracle.verify(tn, d, np.int32([[0]]), seed=1)
    assert out["n_accept"][0] == 1 and out["next_token"][0] == -1 and out["status"][0] & ST_NONFINITE


def test_margins_are_consistent_with_decisions(oracle):
    rng = np.random.default_rng(5)
    B, K, V = 64, 4, 50
    t = np.float32(rng.normal(0, 2, (B, K + 1, V)))
    d = np.float32(0.8 * t[:, :K] + 0.2 * rng.normal(0, 2, (B, K, V)))
    x = rng.integers(0, V, (B, K)).astype(np.int32)
    LA = np.float32(rng.uniform(0.05, 0.3, (B, 16)))
    LR = np.float32(rng.uniform(0.2, 0.6, (B, 16)))
    out = oracle.verify(t, d, x, LA=LA, LR=LR, nA=np.full(B, 16), nR=np.full(B, 16), seed=8)
    base = out["base_margin"] < 0
    relaxed = out["relaxed_margin"] < 0
    assert np.array_equal(out["accept_mask"] & 1, base.astype(np.uint8))
    assert np.array_equal(out["accept_mask"] >> 1, relaxed.astype(np.uint8))
    acc = base | relaxed
    expect = np.where(acc.all(1), K, np.argmin(acc, axis=1))
    assert np.array_equal(out["n_accept"], expect)
    assert 0 < out["n_accept"].mean() < K         # both outcomes occur
    assert (out["accept_mask"] == 2).any()        # the Bayesian test rescued some tokens


# --------------------------------------------------------------- update + draft rule (Algorithm 1)
def test_algorithm_trace_from_the_initial_state(oracle):
    rng = np.random.default_rng(6)
    B, K, cap = 3, 4, 32
    st = new_state(B, cap)
    # initial threshold 0: any row with positive entropy stops the draft loop at its first token
    z = np.float32(rng.normal(0, 1, (B, 40)))
    H, stop = oracle.draft_entropy(z, T_G=st["T_G"], step=0, k_max=20)
    assert np.all(H > 0) and np.all(stop == 1)
    # a one-hot draft row has entropy 0, which is not > 0: drafting continues ...
    onehot = np.full((1, 40), NEG_INF, np.float32); onehot[0, 5] = 1.0
    H1, stop1 = oracle.draft_entropy(onehot, T_G=np.float32([0.0]), step=0, k_max=20)
    assert H1[0] == 0.0 and stop1[0] == 0
    # ... until the window cap
    _, stop2 = oracle.draft_entropy(onehot, T_G=np.float32([0.0]), step=19, k_max=20)
    assert stop2[0] == 1
    # inactive rows are skipped
    Hm, stopm = oracle.draft_entropy(z, T_G=st["T_G"], active=[1, 0, 1], step=0, k_max=20)
    assert Hm[1] == 0.0 and stopm[1] == 0 and Hm[0] == H[0]

    explicit_E = [[] for _ in range(B)]
    explicit_A = [[] for _ in range(B)]
    explicit_R = [[] for _ in range(B)]
    for rnd in range(12):
        n_acc = rng.integers(0, K + 1, B).astype(np.int32)
        dl = np.int32([K, K - 1, K])
        n_acc = np.minimum(n_acc, dl)
        Hq = rng.uniform(0.5, 5.0, (B, K))
        dj = rng.uniform(0.0, 1.0, (B, K))
        dj[0, 0] = 0.0            # exact agreement: never recorded
        dj[1, 1] = 1.0            # exact disagreement: never recorded
        dj[2, 2] = 5e-7           # inside the exclusion band
        oracle.update(st, n_acc, dl, Hq, dj, K, d_eps=1e-6)
        for b in range(B):
            r = int(n_acc[b])
            for i in range(r):
                if 1e-6 < dj[b, i] < 1 - 1e-6:
                    explicit_A[b].append(np.float32(dj[b, i]))
            if r < dl[b]:
                explicit_E[b].append(Hq[b, r])
                if 1e-6 < dj[b, r] < 1 - 1e-6:
                    explicit_R[b].append(np.float32(dj[b, r]))
            tg = np.float32(np.mean(explicit_E[b])) if explicit_E[b] else np.float32(0)
            assert st["T_G"][b] == pytest.approx(tg, rel=1e-6)
            assert st["ent_cnt"][b] == len(explicit_E[b])
            assert list(st["LA"][b, :st["nA"][b]]) == explicit_A[b]
            assert list(st["LR"][b, :st["nR"][b]]) == explicit_R[b]
    assert all(len(e) > 0 for e in explicit_E)


def test_first_rejection_sets_threshold_to_that_entropy_and_full_accept_changes_nothing(oracle):
    st = new_state(1, 8)
    Hq = np.array([[1.5, 2.5, 3.5]])
    dj = np.array([[0.2, 0.4, 0.6]])
    oracle.update(st, [3], None, Hq, dj, 3)                     # all accepted
    assert st["T_G"][0] == 0.0 and st["ent_cnt"][0] == 0 and st["nA"][0] == 3 and st["nR"][0] == 0
    oracle.update(st, [1], None, Hq, dj, 3)                     # rejected at position 1
    assert st["T_G"][0] == np.float32(2.5) and st["nR"][0] == 1 and st["LR"][0, 0] == np.float32(0.4)
    assert st["nA"][0] == 4 and st["LA"][0, 3] == np.float32(0.2)
    oracle.update(st, [0], None, Hq, dj, 3)
    assert st["T_G"][0] == np.float32(2.0)                      # mean(2.5, 1.5)


def test_list_overflow_is_flagged_and_drops_the_append(oracle):
    from oracle.pyoracle import ST_OVERFLOW
    st = new_state(1, 2)
    Hq = np.ones((1, 4)); dj = np.array([[0.1, 0.2, 0.3, 0.4]])
    status = oracle.update(st, [4], None, Hq, dj, 4)
    assert status[0] == ST_OVERFLOW and st["nA"][0] == 2
    assert list(st["LA"][0]) == [np.float32(0.1), np.float32(0.2)]
