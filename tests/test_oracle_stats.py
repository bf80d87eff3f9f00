"""Pins for the oracle's entropy and Jensen-Shannon statistics (CPU only).

Expected values never come from the oracle: closed forms, brute force written from
the definitions (Appendix A; Section 2.2), library routines (scipy), and the
properties the paper states (symmetry, [0,1] bound under log2, metric)."""
import itertools
import math

import numpy as np
import pytest
import torch
from scipy.spatial.distance import jensenshannon
from scipy.special import log_softmax
from scipy.stats import entropy as scipy_entropy

LN2 = math.log(2.0)
NEG_INF = float("-inf")


def f32(x):
    return np.asarray(x, dtype=np.float32)


def bf16_bits(x):
    return torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)


def brute_entropy(z):
    """-sum p ln p from the definition, with exact-ish fsum."""
    z = [float(v) for v in z]
    m = max(z)
    S = math.fsum(math.exp(v - m) for v in z)
    p = [math.exp(v - m) / S for v in z]
    return -math.fsum(pi * math.log(pi) for pi in p if pi > 0.0)


def brute_jsd(zp, zq):
    def sm(z):
        z = [float(v) for v in z]
        m = max(z)
        S = math.fsum(math.exp(v - m) for v in z)
        return [math.exp(v - m) / S for v in z]
    p, q = sm(zp), sm(zq)
    terms = []
    for a, b in zip(p, q):
        m = 0.5 * (a + b)
        if a > 0:
            terms.append(0.5 * a * math.log(a / m))
        if b > 0:
            terms.append(0.5 * b * math.log(b / m))
    return math.fsum(terms)


# ----------------------------------------------------------------------------- entropy
@pytest.mark.parametrize("V", [1, 2, 7, 1000, 32000, 128256, 152064])
@pytest.mark.parametrize("c", [0.0, -3.25, 17.5])
def test_entropy_of_uniform_row_is_ln_V(oracle, V, c):
    lse, H, bad = oracle.row_stats(f32(np.full(V, c)))
    assert bad == 0
    assert H == pytest.approx(math.log(V), rel=1e-10, abs=1e-13)  # index-order fp64 sums
    assert lse == pytest.approx(c + math.log(V), rel=1e-10)


def test_entropy_of_uniform_bf16_row(oracle):
    lse, H, bad = oracle.row_stats(bf16_bits(np.full(128256, 2.5)))
    assert H == pytest.approx(math.log(128256), rel=1e-10)


def test_entropy_of_one_hot_row_is_zero(oracle):
    z = np.full(100, NEG_INF, dtype=np.float32)
    z[37] = 1.25
    lse, H, bad = oracle.row_stats(z)
    assert bad == 0 and H == 0.0 and lse == 1.25


@pytest.mark.parametrize("a", [0.5, 0.9, 0.999, 1e-6])
def test_entropy_two_point_closed_form(oracle, a):
    # probabilities (a, 1-a) <=> logits (ln a, ln(1-a)); fp32 rounding of the logits changes a
    z = f32([math.log(a), math.log1p(-a)])
    pa = math.exp(float(z[0])) / (math.exp(float(z[0])) + math.exp(float(z[1])))
    expect = -pa * math.log(pa) - (1 - pa) * math.log1p(-pa)
    _, H, _ = oracle.row_stats(z)
    assert H == pytest.approx(expect, rel=1e-12, abs=1e-15)


def test_entropy_brute_force_small_vocab(oracle):
    rng = np.random.default_rng(0)
    for V in range(1, 9):
        for _ in range(20):
            z = f32(rng.normal(0, 4, V))
            _, H, _ = oracle.row_stats(z)
            assert H == pytest.approx(brute_entropy(z), rel=1e-12, abs=1e-14)


def test_entropy_matches_scipy_on_llm_sized_rows(oracle):
    rng = np.random.default_rng(1)
    for V, sd in [(32000, 3.0), (128256, 1.0), (128256, 6.0)]:
        z = f32(rng.normal(0, sd, V))
        z[rng.integers(V)] += 8.0
        _, H, _ = oracle.row_stats(z)
        p = np.exp(log_softmax(z.astype(np.float64)))
        assert H == pytest.approx(float(scipy_entropy(p)), rel=1e-11)
        lse, _, _ = oracle.row_stats(z)
        assert lse == pytest.approx(float(np.logaddexp.reduce(z.astype(np.float64))), rel=1e-13)


def test_entropy_invariances_and_bounds(oracle):
    rng = np.random.default_rng(2)
    z = f32(rng.normal(0, 3, 5000))
    _, H, _ = oracle.row_stats(z)
    assert 0.0 <= H <= math.log(5000)
    # adding a constant that is exact in fp32 (power of two, values stay on the same grid)
    zs = f32(np.round(z * 1024) / 1024)
    _, H0, _ = oracle.row_stats(zs)
    _, H1, _ = oracle.row_stats(f32(zs + 8.0))
    assert H1 == pytest.approx(H0, rel=1e-12)
    _, Hp, _ = oracle.row_stats(z[rng.permutation(5000)])
    assert Hp == pytest.approx(H, rel=1e-12)


def test_entropy_small_sigma_lognormal_sanity(oracle):
    # i.i.d. N(0, s^2) logits, small s: H ~ ln V - s^2/2 (log-normal sum); sanity only
    rng = np.random.default_rng(3)
    V, s = 128256, 0.5
    _, H, _ = oracle.row_stats(f32(rng.normal(0, s, V)))
    assert H == pytest.approx(math.log(V) - s * s / 2, rel=2e-3)


def test_masked_logits_are_ignored(oracle):
    z = f32([0.3, NEG_INF, -1.2, NEG_INF, 2.0])
    _, H, bad = oracle.row_stats(z)
    assert bad == 0
    assert H == pytest.approx(brute_entropy(z[[0, 2, 4]]), rel=1e-13)


@pytest.mark.parametrize("poison", [float("nan"), float("inf")])
def test_nonfinite_rows_are_flagged(oracle, poison):
    z = f32([0.0, 1.0, poison, 2.0])
    lse, H, bad = oracle.row_stats(z)
    assert bad == 1 and math.isnan(H) and math.isnan(lse)
    lse, H, bad = oracle.row_stats(f32([NEG_INF, NEG_INF]))
    assert bad == 1 and math.isnan(H)


def test_bf16_rows_are_read_exactly(oracle):
    rng = np.random.default_rng(4)
    zb = bf16_bits(rng.normal(0, 3, 999))
    _, Hb, _ = oracle.row_stats(zb)
    _, Hf, _ = oracle.row_stats(zb.float().numpy())
    assert Hb == Hf


# ----------------------------------------------------------------------------- JSD
def test_jsd_identical_rows_is_zero(oracle):
    rng = np.random.default_rng(5)
    z = f32(rng.normal(0, 3, 4096))
    assert oracle.jsd(z, z) == 0.0
    zg = f32(np.round(z * 1024) / 1024)          # on a grid where +4 is exact in fp32
    assert oracle.jsd(zg, f32(zg + 4.0)) == pytest.approx(0.0, abs=1e-15)  # shift only


def test_jsd_disjoint_supports_is_ln2(oracle):
    V = 64
    zp = np.full(V, NEG_INF, dtype=np.float32)
    zq = np.full(V, NEG_INF, dtype=np.float32)
    zp[:20] = np.linspace(-1, 1, 20)
    zq[30:] = np.linspace(2, -2, 34)
    assert oracle.jsd(zp, zq) == pytest.approx(LN2, rel=1e-14)


def test_jsd_two_point_closed_form(oracle):
    for a, b in [(0.5, 0.5), (0.9, 0.1), (0.7, 0.2), (0.999, 0.5)]:
        zp = f32([math.log(a), math.log1p(-a)])
        zq = f32([math.log(b), math.log1p(-b)])
        assert oracle.jsd(zp, zq) == pytest.approx(brute_jsd(zp, zq), rel=1e-12, abs=1e-16)


def test_jsd_brute_force_small_vocab(oracle):
    rng = np.random.default_rng(6)
    for V in range(2, 9):
        for _ in range(20):
            zp, zq = f32(rng.normal(0, 3, V)), f32(rng.normal(0, 3, V))
            assert oracle.jsd(zp, zq) == pytest.approx(brute_jsd(zp, zq), rel=1e-12, abs=1e-16)


def test_jsd_symmetric_bounded_and_both_forms_agree(oracle):
    rng = np.random.default_rng(7)
    for V, sd in [(50, 3.0), (5000, 3.0), (32000, 1.0), (128256, 6.0)]:
        zp = f32(rng.normal(0, sd, V))
        zq = f32(0.7 * zp + 0.3 * rng.normal(0, sd, V))
        D = oracle.jsd(zp, zq)
        assert 0.0 < D < LN2
        assert oracle.jsd(zq, zp) == pytest.approx(D, rel=1e-12)
        # second line of the definition: H(m) - (H(p)+H(q))/2
        assert oracle.jsd(zp, zq, entropy_form=True) == pytest.approx(D, rel=1e-9, abs=1e-13)


def test_jsd_matches_scipy(oracle):
    rng = np.random.default_rng(8)
    for V in (100, 32000, 128256):
        zp = f32(rng.normal(0, 3, V))
        zq = f32(0.8 * zp + 0.2 * rng.normal(0, 3, V))
        p = np.exp(log_softmax(zp.astype(np.float64)))
        q = np.exp(log_softmax(zq.astype(np.float64)))
        d_nats = float(jensenshannon(p, q))           # sqrt of JSD, natural log
        d_bits = float(jensenshannon(p, q, base=2))   # in [0,1]
        D = oracle.jsd(zp, zq)
        assert math.sqrt(D) == pytest.approx(d_nats, rel=1e-10)
        assert math.sqrt(D / LN2) == pytest.approx(d_bits, rel=1e-10)


def test_js_distance_satisfies_triangle_inequality(oracle):
    rng = np.random.default_rng(9)
    for _ in range(50):
        V = int(rng.integers(2, 200))
        a, b, c = (f32(rng.normal(0, 3, V)) for _ in range(3))
        dab, dbc, dac = (math.sqrt(oracle.jsd(x, y)) for x, y in ((a, b), (b, c), (a, c)))
        assert dac <= dab + dbc + 1e-12


def test_jsd_permutation_invariance(oracle):
    rng = np.random.default_rng(10)
    zp, zq = f32(rng.normal(0, 3, 777)), f32(rng.normal(0, 3, 777))
    perm = rng.permutation(777)
    assert oracle.jsd(zp[perm], zq[perm]) == pytest.approx(oracle.jsd(zp, zq), rel=1e-12)


def test_jsd_partial_overlap_with_masks(oracle):
    zp = f32([0.0, 1.0, NEG_INF, 0.5])
    zq = f32([NEG_INF, 1.0, 0.2, 0.5])
    assert oracle.jsd(zp, zq) == pytest.approx(brute_jsd(zp, zq), rel=1e-13)


def test_jsd_nonfinite_row(oracle):
    assert math.isnan(oracle.jsd(f32([0.0, float("nan")]), f32([0.0, 1.0])))


def test_exhaustive_tiny_grid(oracle):
    # every pair of 3-element rows on a small logit grid: oracle == brute force
    grid = [-2.0, 0.0, 1.5]
    rows = [f32(r) for r in itertools.product(grid, repeat=3)]
    for zp in rows:
        _, H, _ = oracle.row_stats(zp)
        assert H == pytest.approx(brute_entropy(zp), rel=1e-12, abs=1e-15)
        for zq in rows:
            assert oracle.jsd(zp, zq) == pytest.approx(brute_jsd(zp, zq), rel=1e-11, abs=1e-15)
