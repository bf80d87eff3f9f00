"""Pin of the lowest-index rule on exact ties of the Gumbel-max draws (CPU only).

The re-sampled token of Section 2.1.3 and the drafted token of Algorithm 1 (x_i ~ q_i) are drawn by
Gumbel-max; the paper gives no rule for equal keys, this build takes the lowest index.  A row of
128256 32-bit Philox words holds about n^2 / 2^33 = 2 pairs of elements with the SAME word: two such
elements with equal weights have bit-identical keys, so the rule decides the draw.  The pairs are
found here with an independent numpy Philox and confirmed word by word through the oracle and the
pure-Python implementation; an oracle that kept the later of two equal keys would return the higher
index and fail every case below."""
import numpy as np
import pytest

import philox_ref

V = 128256
SEED = 1                     # (seed, sequence 0, round 0, position 0) holds three pairs on stream 1, four on stream 2
KNOWN = {1: [(6825, 109521), (18339, 45018), (50415, 52012)],
         2: [(6024, 80251), (18530, 43784), (61492, 125679), (68895, 113803)]}


@pytest.fixture(scope="module")
def pairs():
    found = {s: philox_ref.equal_word_pairs(philox_ref.noise_words_of_row(SEED, 0, 0, 0, s, V)) for s in (1, 2)}
    assert found == KNOWN
    return found


def test_the_pairs_really_share_a_word(oracle, pairs):
    for i, j in pairs[1]:
        wi, wj = oracle.gumbel_word(SEED, 0, 0, 0, i), oracle.gumbel_word(SEED, 0, 0, 0, j)
        assert wi == wj == philox_ref.gumbel_word(SEED, 0, 0, 0, i) == philox_ref.gumbel_word(SEED, 0, 0, 0, j)
    for i, j in pairs[2]:
        wi = philox_ref.philox4x32_10([i >> 2, 2 << 16, 0, 0], [SEED, 0])[i & 3]
        wj = philox_ref.philox4x32_10([j >> 2, 2 << 16, 0, 0], [SEED, 0])[j & 3]
        assert wi == wj
        assert int(oracle.philox([i >> 2, 2 << 16, 0, 0], [SEED, 0])[i & 3]) == wi


def tied_rows(i, j, kind):
    """One position whose draw is decided between elements i and j alone: everything else sits 40 nats
    lower (the Gumbel noise of a 32-bit word spans less than 26 nats).  Returns target [1,2,V], draft
    [1,1,V], the drafted token, the window length."""
    t = np.full((1, 2, V), -40.0, np.float32)
    d = np.full((1, 1, V), -40.0, np.float32)
    x = 77                                     # the drafted token: neither i nor j
    t[0, :, [i, j]] = 3.0                      # equal target logits on the pair, in the bonus row too
    if kind == "residual":
        d[0, 0, [i, j]] = 0.0                  # equal draft logits, below the target's: equal residual mass
        d[0, 0, x] = 30.0                      # the draft is sure of x, the target is not: the ratio test rejects
    elif kind == "excluded":
        d[0, 0, x] = 30.0                      # (the match test only looks at p(x) = e^-43.7)
    return t, d, np.int32([[x]]), (0 if kind == "bonus" else 1)


@pytest.mark.parametrize("kind", ["residual", "bonus", "excluded"])
def test_lowest_index_wins_an_exact_tie_of_the_replacement_draw(oracle, pairs, kind):
    for i, j in pairs[1]:
        t, d, x, k = tied_rows(i, j, kind)
        out = oracle.verify(t, d, x, draft_len=np.int32([k]), seed=SEED, relaxed_off=1,
                            base_test=1 if kind == "excluded" else 0)
        assert out["n_accept"][0] == 0
        assert out["top2_gap"][0] == 0.0, "the two keys are not bit-identical: the case does not test the rule"
        assert out["next_token"][0] == i, (kind, i, j, out["next_token"][0])
        # the same with the pair's weights swapped onto other elements: no tie, no special role of i
        t2 = t.copy()
        t2[0, :, j] = 3.5
        out2 = oracle.verify(t2, d, x, draft_len=np.int32([k]), seed=SEED, relaxed_off=1,
                             base_test=1 if kind == "excluded" else 0)
        assert out2["next_token"][0] == j and out2["top2_gap"][0] > 0


def test_lowest_index_wins_an_exact_tie_of_the_drafted_token(oracle, pairs):
    for i, j in pairs[2]:
        z = np.full((1, V), -40.0, np.float32)
        z[0, [i, j]] = 1.5
        tok, gap = oracle.draft_sample(z, step=0, seed=SEED)
        assert gap[0] == 0.0
        assert tok[0] == i
        z[0, j] = 2.0
        tok, gap = oracle.draft_sample(z, step=0, seed=SEED)
        assert tok[0] == j and gap[0] > 0
