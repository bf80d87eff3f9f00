"""Pins for the oracle's Algorithm-1-literal options (CPU only): the verification loop's own
acceptance test (a token y_i drawn from the target, accepted iff it equals the drafted one) and
the appends to the accepted-distance list inside the loop.

What fixes the expected values: the law of the emitted token (it is y_i, so it follows the target
distribution whatever the draft proposes), elementary probability for the acceptance rate and the
conditional law of the replacement token, and the composition of single-position rounds with the
update step between them, which is what a list that grows inside the loop means."""
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


# --------------------------------------------------------------- the loop's own acceptance test
def test_exact_match_test_emits_the_target_distribution(oracle):
    """k = 1, Bayesian test off.  The emitted token is y ~ p: the drafted token where the two agree,
    y itself otherwise.  Its law is p for ANY proposal law; P(accept) = sum_v q_v p_v; a replacement
    never repeats the drafted token and follows p restricted to the other tokens."""
    rng = np.random.default_rng(3)
    V, B = 6, 80000
    zp = np.float32([1.2, -0.3, 0.4, 2.0, -1.5, 0.0])
    zq = np.float32([0.1, 1.4, 0.4, 0.5, -0.2, NEG_INF])
    zp2 = np.float32([0.0, 0.5, -0.5, 1.0, 0.2, -1.0])
    p, q, p2 = softmax(zp), softmax(zq), softmax(zp2)
    target = np.broadcast_to(np.stack([zp, zp2]), (B, 2, V)).copy()
    draft = np.broadcast_to(zq, (B, 1, V)).copy()
    x = rng.choice(V, size=(B, 1), p=q).astype(np.int32)
    out = oracle.verify(target, draft, x, seed=77, relaxed_off=1, base_test=1)

    acc = out["n_accept"] == 1
    assert acc.mean() == pytest.approx(float((p * q).sum()), abs=4 * 0.5 / math.sqrt(B))
    first = np.where(acc, x[:, 0], out["next_token"])
    assert chi2_stat(np.bincount(first, minlength=V).astype(np.float64), p) < 25.7     # 5 dof, ~1e-4
    # after an acceptance the extra token follows the next target row
    assert chi2_stat(np.bincount(out["next_token"][acc], minlength=V).astype(np.float64), p2) < 25.7
    # replacements: never the drafted token; given the drafted token, p renormalised without it
    rej = ~acc
    assert np.all(out["next_token"][rej] != x[rej, 0])
    for xv in range(V - 1):                               # token 5 is never drafted
        sel = rej & (x[:, 0] == xv)
        cond = p.copy(); cond[xv] = 0.0; cond /= cond.sum()
        counts = np.bincount(out["next_token"][sel], minlength=V).astype(np.float64)
        assert chi2_stat(counts, cond) < 23.5             # 4 dof, ~1e-4
    # the acceptance bit does not look at the draft's probabilities: same decisions for another q
    draft2 = np.float32(rng.normal(0, 2, (B, 1, V)))
    out2 = oracle.verify(target, draft2, x, seed=77, relaxed_off=1, base_test=1)
    assert np.array_equal(out2["n_accept"], out["n_accept"])
    assert np.array_equal(out2["next_token"], out["next_token"])
    # and it differs from the ratio test on the same inputs (which accepts more often)
    out0 = oracle.verify(target, draft, x, seed=77, relaxed_off=1, base_test=0)
    assert (out0["n_accept"] == 1).mean() > acc.mean() + 0.05


def test_exact_match_margin_and_forced_cases(oracle):
    V = 5
    z = np.float32([0.0, 1.0, 2.0, NEG_INF, -1.0])
    onehot = np.full(V, NEG_INF, np.float32); onehot[2] = 0.0
    target = np.stack([np.stack([z, z]), np.stack([onehot, z]), np.stack([onehot, z])])
    draft = np.zeros((3, 1, V), np.float32)
    x = np.int32([[3], [2], [1]])         # p(x) = 0 | p(x) = 1 | p(x) = 0 with all mass elsewhere
    out = oracle.verify(target, draft, x, seed=1, relaxed_off=1, base_test=1)
    assert list(out["n_accept"]) == [0, 1, 0]
    assert out["base_margin"][0, 0] == math.inf            # ln u - ln 0
    assert out["next_token"][2] == 2                       # the only token with mass
    assert out["status"][2] == 0
    lp = math.log(softmax(z)[1])
    # margin = ln u1 - ln p(x): the decision is its sign
    for s in range(40):
        o = oracle.verify(target[:1], draft[:1], np.int32([[1]]), seed=s, relaxed_off=1, base_test=1)
        m = o["base_margin"][0, 0]
        assert (m < 0) == bool(o["accept_mask"][0, 0] & 1)
        assert m + lp <= 0.0                               # ln u1 <= 0


def test_a_rejected_position_always_leaves_mass_outside_the_drafted_token(oracle):
    """A rejection needs ln u1 >= ln p(x) with u1 < 1, so p(x) < 1 and the other tokens hold mass: the
    replacement is always defined.  Extreme rows: the drafted token holds all of the mass (always
    accepted) or none of it (always rejected, the replacement is the token that holds it all)."""
    V = 4
    z = np.float32([0.0, -2000.0, -2000.0, -2000.0])      # p(0) = 1 to the last bit
    target = np.stack([z, z])[None]
    draft = np.zeros((1, 1, V), np.float32)
    for s in range(20):
        out = oracle.verify(target, draft, np.int32([[0]]), seed=s, relaxed_off=1, base_test=1)
        assert out["n_accept"][0] == 1 and out["status"][0] == 0
        out = oracle.verify(target, draft, np.int32([[1]]), seed=s, relaxed_off=1, base_test=1)
        assert out["n_accept"][0] == 0 and out["next_token"][0] == 0 and out["status"][0] == 0


# --------------------------------------------------------------- appends inside the loop
def _random_round(rng, B, K, V, scale=1.5):
    t = np.float32(rng.normal(0, scale, (B, K + 1, V)))
    d = np.float32(t[:, :K] + rng.normal(0, 1.0, (B, K, V)))
    x = rng.integers(0, V, (B, K)).astype(np.int32)
    return t, d, x


def _seeded_state(rng, B, cap, nA, nR):
    st = new_state(B, cap)
    for b in range(B):
        st["LA"][b, :nA[b]] = rng.uniform(0.05, 0.5, nA[b])
        st["LR"][b, :nR[b]] = rng.uniform(0.3, 0.9, nR[b])
    st["nA"][:] = nA
    st["nR"][:] = nR
    return st


def test_in_loop_appends_equal_single_position_rounds_with_the_update_between(oracle):
    """Position i of a round with in-loop appends must see what a chain of one-position rounds sees
    when every earlier position was accepted and the update step ran after each."""
    rng = np.random.default_rng(21)
    B, K, V, cap = 5, 6, 40, 64
    t, d, x = _random_round(rng, B, K, V)
    nA = np.int32([0, 1, 2, 7, 20]); nR = np.int32([5, 3, 2, 9, 1])
    st = _seeded_state(rng, B, cap, nA, nR)
    before = {k: v.copy() for k, v in st.items()}
    full = oracle.verify(t, d, x, LA=st["LA"], LR=st["LR"], nA=st["nA"], nR=st["nR"], seed=5,
                         list_update=1)
    for k in before:                                      # the state is only read
        assert np.array_equal(st[k], before[k])

    chain = {k: v.copy() for k, v in st.items()}
    for i in range(K):
        ti = np.ascontiguousarray(t[:, [i, i + 1]])
        one = oracle.verify(ti, d[:, i:i + 1], x[:, i:i + 1], LA=chain["LA"], LR=chain["LR"],
                            nA=chain["nA"], nR=chain["nR"], seed=5)
        assert np.array_equal(one["d_js"][:, 0], full["d_js"][:, i])
        assert np.array_equal(one["p_accept"][:, 0], full["p_accept"][:, i]), i
        # as if accepted
        oracle.update(chain, np.ones(B, np.int32), None, one["H_q"], one["d_js"], 1)
    # with every position accepted the chain's lists are what the update step leaves after the round
    ref = {k: v.copy() for k, v in st.items()}
    oracle.update(ref, np.full(B, K, np.int32), None, full["H_q"], full["d_js"], K)
    assert np.array_equal(ref["LA"], chain["LA"]) and np.array_equal(ref["nA"], chain["nA"])
    # the growing list matters: without it the later posteriors differ
    flat = oracle.verify(t, d, x, LA=st["LA"], LR=st["LR"], nA=st["nA"], nR=st["nR"], seed=5)
    assert np.array_equal(flat["p_accept"][:, 0], full["p_accept"][:, 0])
    assert not np.allclose(flat["p_accept"][:, 1:], full["p_accept"][:, 1:], rtol=1e-3, atol=0)
    # a list that starts with 0 or 1 samples becomes usable inside the round
    assert full["p_accept"][0, 1] == 0.0 and full["p_accept"][0, 2] > 0.0
    assert flat["p_accept"][0].max() == 0.0


def test_in_loop_posterior_on_explicit_lists_with_filter_and_capacity(oracle):
    rng = np.random.default_rng(8)
    K, V, cap = 7, 24, 12
    t, d, x = _random_round(rng, 1, K, V)
    d[0, 2] = t[0, 2]                                     # identical rows: distance 0, never recorded
    st = _seeded_state(rng, 1, cap, np.int32([9]), np.int32([4]))
    out = oracle.verify(t, d, x, LA=st["LA"], LR=st["LR"], nA=st["nA"], nR=st["nR"], seed=1,
                        list_update=1)
    assert out["d_js"][0, 2] == 0.0
    la = list(st["LA"][0, :9])
    lr = st["LR"][0, :4]
    for i in range(K):
        want = oracle.posterior(out["d_js"][0, i], np.float32(la), lr)
        assert out["p_accept"][0, i] == want, i
        di = out["d_js"][0, i]
        if 1e-6 < di < 1 - 1e-6 and len(la) < cap:        # the update step's filter and capacity
            la.append(np.float32(di))
    assert len(la) == cap                                 # 9 + 6 candidates > 12: the cap was hit


def test_in_loop_appends_do_not_change_the_round_without_history_lists(oracle):
    rng = np.random.default_rng(2)
    t, d, x = _random_round(rng, 3, 4, 16)
    a = oracle.verify(t, d, x, seed=3, list_update=1)
    b = oracle.verify(t, d, x, seed=3)
    for k in ("n_accept", "next_token", "p_accept", "accept_mask"):
        assert np.array_equal(a[k], b[k])
