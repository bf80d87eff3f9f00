"""GPU parity tests: the HIP library against the CPU oracle, through the C ABI (run with -m gpu)."""
import math

import numpy as np
import pytest
import torch

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def am():
    import paper_2512_11280_amd as am
    am.load_library()          # fails loudly if libadasd.so is not built
    assert torch.cuda.is_available()
    return am


@pytest.fixture(scope="module")
def wl():
    from paper_2512_11280_amd import workloads
    return workloads


@pytest.fixture(params=[2, 1], ids=["singleread", "twokernel"])
def path(request):
    """Both implementations of the statistics stage must meet the same bar."""
    return request.param


def _no_flips(rep):
    """On the five configurations of the benchmark no decision sits within 1e-5 of its threshold: every
    sequence is compared bit for bit."""
    assert rep["flips"] == 0 and rep["member_flips"] == 0 and rep["seq_skipped"] == 0, rep


def _report(name, rep):
    print(f"[parity] {name}: flips={rep['flips']} member_flips={rep['member_flips']} "
          f"skipped_seq={rep['seq_skipped']} exact_path={rep['exact_path']} max_rel_H={rep['max_rel_H']:.2e} "
          f"max_rel_d={rep['max_rel_d']:.2e}", flush=True)


# ------------------------------------------------------------------------------- the five shapes
def test_config_tiny_fp32(am, wl, oracle, path):
    batch = wl.config_tiny()
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    rep = G.compare_verify(out, G.run_oracle(oracle, batch))
    _report("tiny", rep)
    _no_flips(rep)


@pytest.mark.parametrize("with_state", [True, False])
def test_config_single_stream_bf16(am, wl, oracle, with_state, path):
    batch = wl.config_single_stream(with_state=with_state)
    ws = am.Workspace(8, 8, batch.V, torch.bfloat16)      # also serves the 8-row draft-entropy call
    out, _, _ = G.run_gpu(am, batch, stats_path=path, ws=ws)
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref)
    _report(f"single_stream(state={with_state})", rep)
    _no_flips(rep)
    # both entropy regimes are present
    assert ref["H_q"][0, :4].max() < ref["H_q"][0, 4:].min()
    # draft-side entropy of each draft row, with a threshold in the middle of the two regimes
    rows = batch.draft[0].cuda()
    tg = torch.full((rows.shape[0],), 6.0, device="cuda")
    H, stop = am.draft_entropy(rows, ws, T_G=tg, step=0, k_max=20)
    torch.cuda.synchronize()
    Href, stop_ref = oracle.draft_entropy(batch.draft[0], T_G=tg.cpu().numpy(), step=0, k_max=20)
    assert G.close(H.cpu().numpy(), Href).all()
    assert np.array_equal(stop.cpu().numpy(), stop_ref)
    assert stop_ref.min() == 0 and stop_ref.max() == 1


def test_config_batched_reduced(am, wl, oracle, path):
    # same generator and vocabulary as the headline shape, fewer sequences so the oracle takes seconds
    batch = wl.config_batched(B=8, k=8)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref)
    _report("batched(B=8)", rep)
    _no_flips(rep)
    assert 0 < ref["n_accept"].mean() < 8
    assert (ref["accept_mask"] == 2).any()      # the Bayesian test decides some positions


def test_config_large_reduced(am, wl, oracle, path):
    batch = wl.config_large(B=6, k=16)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref)
    _report("large(B=6,k=16,V=152064)", rep)
    _no_flips(rep)


def test_headline_workload_full_size(am, wl, oracle, path):
    """The exact shape, generator, list capacity and launch configuration that bench.py times
    (B=32, k=8, V=128256, bf16): every output of every sequence against the oracle."""
    batch = wl.config_batched(seed=wl.DEFAULT_SEED + 2, B=32, k=8, V=128256, cap=8192)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref)
    _report("headline(B=32,k=8,V=128256)", rep)
    _no_flips(rep)
    assert 0 < ref["n_accept"].mean() < 8


def test_large_workload_full_size_sampled_sequences(am, wl, oracle):
    """B=128, k=16, V=152064 on the GPU in one call; the oracle redoes every 16th sequence (sequences
    are independent: own lists, own Philox stream selected by the sequence id)."""
    batch = wl.config_large(B=128, k=16)
    out, _, _ = G.run_gpu(am, batch)
    pick = list(range(0, 128, 16))
    sub = wl.VerifyBatch(target=batch.target[pick], draft=batch.draft[pick],
                         draft_tokens=batch.draft_tokens[pick],
                         draft_len=None if batch.draft_len is None else batch.draft_len[pick],
                         state={k: v[pick] for k, v in batch.state.items()},
                         seed=batch.seed, round0=batch.round0)
    ref = G.run_oracle(oracle, sub, seq_id=pick)

    class Picked:
        pass
    got = Picked()
    for name in ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept", "accept_mask", "status"):
        setattr(got, name, getattr(out, name)[pick])
    rep = G.compare_verify(got, ref)
    _report("large(B=128,k=16,V=152064), 8 sampled sequences", rep)
    _no_flips(rep)


def test_largest_window(am, wl, oracle, path):
    """k_max = 64, the compiled limit: every decision group loops eight times, the update step uses
    all 64 lanes."""
    batch = wl.config_batched(B=3, k=64, V=2048, seed=64)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    rep = G.compare_verify(out, G.run_oracle(oracle, batch))
    _report("k=64", rep)


def test_largest_vocabulary(am, wl, oracle):
    """V = 2^24, the compiled limit, one position: 64 slices of 32768 vectors each, i.e. sixteen
    batches per thread in both streaming kernels and 128 slices in the sampling kernel."""
    batch = wl.config_batched(B=1, k=1, V=1 << 24, seed=24)
    out, _, _ = G.run_gpu(am, batch)
    rep = G.compare_verify(out, G.run_oracle(oracle, batch))
    _report("V=2^24", rep)


def test_ragged_lengths_sequence_ids_and_rounds(am, wl, oracle, path):
    batch = wl.config_batched(B=6, k=5, V=32003, seed=99)       # V not a multiple of 8: scalar tail
    batch.draft_len = torch.tensor([0, 1, 5, 3, 2, 5], dtype=torch.int32)
    seq_id = [7, 1 << 31, 3, 3, 0xFFFFFFFF, 12]
    rounds = [0, 5, 1000, 1001, 2, 3]
    out, _, _ = G.run_gpu(am, batch, stats_path=path, seq_id=seq_id, rounds=rounds)
    ref = G.run_oracle(oracle, batch, seq_id=seq_id, rounds=rounds)
    rep = G.compare_verify(out, ref)
    _report("ragged", rep)
    assert out.n_accept[0].item() == 0 and out.H_q[0].abs().sum().item() == 0


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_entropy_of_rows_with_nearly_all_mass_on_one_token(am, wl, oracle, dtype, path):
    """Entropies far below 1 nat: the heaviest token sits late in the row, so a reference taken from the
    start of the row is far below the maximum (the single-read kernel starts from such a reference and
    has to notice; a randomised sweep once found 2e-6 nats of error on a row with H = 0.067)."""
    batch = wl.config_batched(B=3, k=4, V=4104, seed=77, dtype=dtype)
    g = torch.Generator().manual_seed(5)
    for b in range(3):
        for i in range(5):
            at = int(torch.randint(2000, 4104, (1,), generator=g))
            batch.target[b, i, at] += 14.0 + 2.0 * i
            if i < 4:
                batch.draft[b, i, at] += 12.0
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    assert ref["H_p"].min() < 0.05                   # the case is what it says
    rep = G.compare_verify(out, ref)
    _report(f"peaked rows {dtype} path {path}", rep)


@pytest.mark.parametrize("B,K,V", [(70, 9, 1032), (130, 3, 520), (1100, 2, 264), (64, 16, 2056), (3, 64, 520),
                                   (32767, 1, 16), (16383, 2, 24)])
def test_ragged_windows_of_many_sequences(am, wl, oracle, B, K, V):
    """Ragged windows go through a packed list of the positions that have work: one wavefront of
    sequences, several wavefronts, more sequences than one workgroup has threads, the longest window;
    lengths from 0 to k_max and beyond (clamped and flagged)."""
    batch = wl.config_batched(B=B, k=K, V=V, seed=B * 1000 + K, cap=64)
    rng = np.random.default_rng(B + K)
    lens = rng.integers(0, K + 1, B)
    lens[0] = 0
    lens[-1] = K
    if B > 2:
        lens[1] = K + 3                     # out of range: clamped to k_max, flagged
    batch.draft_len = torch.tensor(np.minimum(lens, K), dtype=torch.int32)
    ref = G.run_oracle(oracle, batch)
    batch.draft_len = torch.tensor(lens, dtype=torch.int32)
    out, _, _ = G.run_gpu(am, batch)
    st = out.status.cpu().numpy()
    if B > 2:
        assert st[1] & am.binding.ST_BAD_LENGTH
        st[1] &= ~am.binding.ST_BAD_LENGTH
        out.status = torch.tensor(st, device="cuda")
    rep = G.compare_verify(out, ref, info_bits=16 | 8)
    _report(f"ragged B={B} K={K}", rep)
    # positions past a window's end hold the filler, never a stale value
    H = out.H_q.cpu().numpy()
    for b in range(B):
        assert (H[b, min(lens[b], K):] == 0).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [8, 100, 1001, 4096, 20011])
def test_small_and_ragged_vocabularies(am, wl, oracle, dtype, V, path):
    batch = wl.config_batched(B=5, k=3, V=V, dtype=dtype, seed=V)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    rep = G.compare_verify(out, G.run_oracle(oracle, batch))
    _report(f"V={V},{dtype}", rep)


def test_unaligned_rows_take_the_elementwise_path(am, wl, oracle):
    # an odd vocabulary stride makes most rows start off a 16-byte boundary
    batch = wl.config_batched(B=4, k=3, V=3001, seed=5)
    t = torch.zeros(4, 4, 3003, dtype=torch.bfloat16)
    d = torch.zeros(4, 3, 3003, dtype=torch.bfloat16)
    t[:, :, :3001] = batch.target
    d[:, :, :3001] = batch.draft
    tg, dg = t.cuda()[:, :, :3001], d.cuda()[:, :, :3001]
    ws = am.Workspace(4, 3, 3001, torch.bfloat16)
    st = G.state_to_device(am, batch.state, 4, batch.state["LA"].shape[1])
    out = am.verify(tg, dg, batch.draft_tokens.cuda(), ws, state=st, seed=batch.seed)
    torch.cuda.synchronize()
    rep = G.compare_verify(out, G.run_oracle(oracle, batch))
    _report("unaligned", rep)


def test_nearly_identical_distributions(am, wl, oracle, path):
    """Small JS distances: flat rows with a slightly perturbed draft, and peaked rows where both
    models put ~0.999 on one token (the regime the paper reports as distances 'equal to 0')."""
    V, K = 128256, 6
    g = torch.Generator().manual_seed(12)
    t = torch.randn(1, K + 1, V, generator=g)
    d = torch.empty(1, K, V)
    for i, noise in enumerate([0.2, 0.05, 0.01]):                     # flat, std 1
        d[0, i] = t[0, i] + noise * torch.randn(V, generator=g)
    for i, (zt, zd) in enumerate([(19.0, 18.0), (22.0, 21.875), (25.0, 25.0)], start=3):   # peaked
        d[0, i] = t[0, i] + 0.3 * torch.randn(V, generator=g)
        t[0, i, 1000 + i] = zt
        d[0, i, 1000 + i] = zd
    tok = torch.full((1, K), 1003, dtype=torch.int32)
    batch = wl.VerifyBatch(t.to(torch.bfloat16), d.to(torch.bfloat16), tok, None, wl.empty_state(1, 8), 3)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    print("[small d] oracle d:", ref["d_js"][0], "gpu d:", out.d_js[0].cpu().numpy(), flush=True)
    rep = G.compare_verify(out, ref)
    _report("nearly identical", rep)
    assert ref["d_js"].min() < 1e-3
    # small distances keep RELATIVE accuracy (no absolute floor): the per-element term is taken from its
    # series in the exactly formed log ratio where that ratio is small
    rel = np.abs(out.d_js[0].cpu().numpy().astype(np.float64) - ref["d_js"][0]) / ref["d_js"][0]
    print("[small d] relative error of the distance:", rel, flush=True)
    assert rel.max() < 1e-5


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rows_with_normalisers_far_apart(am, wl, oracle, dtype, path):
    """Softmax does not see a row's offset, so the two rows of a position may carry very different ones
    (hundreds of nats in float32; in bf16 as far as its grid still resolves the row).  The log ratio of an
    element is then formed from each logit relative to its own row's offset, with the rounding error of the
    difference carried along, so the distance keeps its accuracy, also where the distributions are close."""
    V, K = 32768, 4
    g = torch.Generator().manual_seed(40)
    t = 3.0 * torch.randn(1, K + 1, V, generator=g)
    d = torch.empty(1, K, V)
    cases = [(600.0, 0.5), (-450.0, 0.05), (90.0, 1.5), (1000.0, 0.01)] if dtype == torch.float32 else \
        [(64.0, 0.5), (-96.0, 0.3), (24.0, 1.0), (-40.0, 0.2)]
    for i, (shift, noise) in enumerate(cases):
        d[0, i] = t[0, i] + noise * torch.randn(V, generator=g) + shift
    tok = torch.full((1, K), 17, dtype=torch.int32)
    batch = wl.VerifyBatch(t.to(dtype), d.to(dtype), tok, None, wl.empty_state(1, 8), 5)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    rel = np.abs(out.d_js[0].cpu().numpy().astype(np.float64) - ref["d_js"][0]) / ref["d_js"][0]
    print(f"[offset rows {dtype}] d:", ref["d_js"][0], "relative error:", rel, flush=True)
    rep = G.compare_verify(out, ref)
    _report("offset rows", rep)
    assert rel.max() < 1e-5


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_nearly_one_hot_rows_with_offsets_far_apart(am, wl, oracle, dtype, path):
    """Both rows put (nearly) all their mass on the same token while their offsets differ by hundreds of
    nats: the distance is a few 1e-8 or less, and an inconsistency of 1e-8 of an OFFSET in the log ratios
    would show as 1e-6.  Found by a randomised sweep (rows scaled by 12 and shifted by +-80): the factor
    log2(e) has to be the same float constant in the normalisers and in the log ratios."""
    V, K = 4104, 6
    g = torch.Generator().manual_seed(41)
    t = 36.0 * torch.randn(1, K + 1, V, generator=g)
    d = torch.empty(1, K, V)
    shifts = [(193.0, 6.6), (-250.0, 120.0), (40.0, -35.0), (209.0, 5.7), (0.0, 300.0), (-60.0, -58.0)]
    for i, (sp, sq) in enumerate(shifts):
        top = int(torch.argmax(t[0, i]))
        t[0, i] += sp - t[0, i, top]                     # the largest logit sits at the offset itself
        d[0, i] = 0.9 * (t[0, i] - sp) + sq              # same ranking, other scale and offset
    tok = torch.full((1, K), 17, dtype=torch.int32)
    batch = wl.VerifyBatch(t.to(dtype), d.to(dtype), tok, None, wl.empty_state(1, 8), 5)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    print(f"[one-hot rows {dtype}] d gpu:", out.d_js[0].cpu().numpy(), "oracle:", ref["d_js"][0], flush=True)
    rep = G.compare_verify(out, ref)
    _report("one-hot rows", rep)
    err = np.abs(out.d_js[0].cpu().numpy().astype(np.float64) - ref["d_js"][0])
    assert (err <= 1e-5 * ref["d_js"][0] + 2e-7).all(), err        # well inside the contract's 1e-6
    assert (out.H_p >= 0).all() and (out.H_q >= 0).all()


# ------------------------------------------------------------------------------- options
@pytest.mark.parametrize("opt", [dict(reject_rule=1), dict(relaxed_off=1), dict(bw_rule=1),
                                 dict(kde_min_n=100)])
def test_option_variants(am, wl, oracle, opt):
    batch = wl.config_batched(B=6, k=6, V=32000, seed=17)
    options = am.Options(**opt)
    out, _, _ = G.run_gpu(am, batch, options=options)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref)
    _report(f"options {opt}", rep)
    if opt.get("relaxed_off") or opt.get("kde_min_n"):
        assert (out.p_accept == 0).all()


# ------------------------------------------------------------------------------- Algorithm 1 as written
LITERAL = [dict(base_test=1), dict(list_update=1), dict(base_test=1, list_update=1),
           dict(base_test=1, list_update=1, reject_rule=1), dict(list_update=1, bw_rule=1)]


def _short_and_full_lists(batch, cap):
    """History lists from empty to nearly full, so that a list becomes usable inside the round and
    another one fills up inside it."""
    st = batch.state
    B = batch.B
    nA = [0, 1, 2, cap - 2, cap, 64][:B] + [64] * max(B - 6, 0)
    for b in range(B):
        st["nA"][b] = nA[b]
        if nA[b] > 64:
            st["LA"][b, 64:nA[b]] = st["LA"][b, :nA[b] - 64]
    return batch


@pytest.mark.parametrize("opt", LITERAL, ids=lambda o: "+".join(f"{k}{v}" for k, v in o.items()))
def test_literal_variant_of_the_verification_loop(am, wl, oracle, opt, path):
    """The loop's own match test with the replacement drawn without the drafted token, and the accepted
    list growing inside the loop."""
    cap = 70
    batch = _short_and_full_lists(wl.config_batched(B=7, k=6, V=32000, seed=23, cap=cap), cap)
    options = am.Options(**opt)
    out, _, _ = G.run_gpu(am, batch, options=options, stats_path=path)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref)
    _report(f"literal {opt}", rep)
    pa = ref["p_accept"]
    if opt.get("list_update"):
        assert pa[0, 0] == 0 and pa[0, 1] == 0 and pa[0, 2:].max() > 0      # empty list: usable from the third position
        assert pa[1, 0] == 0 and pa[1, 1:].max() > 0
        flat = G.run_oracle(oracle, batch, options=am.Options(**{**opt, "list_update": 0}))
        assert not np.allclose(flat["p_accept"], pa, rtol=1e-3, atol=1e-6)
    if opt.get("base_test"):
        rej = ref["n_accept"] < batch.k
        tok = batch.draft_tokens.numpy()
        nt = out.next_token.cpu().numpy()
        assert rej.any()
        assert all(nt[b] != tok[b, ref["n_accept"][b]] for b in np.flatnonzero(rej))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [8, 100, 1001, 20011])
def test_literal_variant_small_and_ragged_vocabularies(am, wl, oracle, dtype, V):
    batch = wl.config_batched(B=5, k=5, V=V, seed=100 + V, dtype=dtype, cap=80)
    batch.draft_len = torch.tensor([5, 0, 3, 5, 1], dtype=torch.int32)
    options = am.Options(base_test=1, list_update=1)
    out, _, _ = G.run_gpu(am, batch, options=options)
    rep = G.compare_verify(out, G.run_oracle(oracle, batch, options=options))
    _report(f"literal V={V} {dtype}", rep)


def test_literal_variant_largest_window_and_unaligned_rows(am, wl, oracle):
    # 64 positions, a list with room for 10 more samples: the in-loop appends stop at the capacity
    batch = wl.config_batched(B=2, k=64, V=4099, seed=5, cap=74)
    options = am.Options(base_test=1, list_update=1)
    out, _, _ = G.run_gpu(am, batch, options=options)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref)
    _report("literal K=64", rep)
    assert (ref["p_accept"][:, 11:] > 0).any()


def test_literal_variant_with_the_update_in_the_same_call(am, wl, oracle):
    """The state after the round does not depend on when the posteriors saw the appends."""
    batch = wl.config_batched(B=6, k=7, V=8192, seed=78, cap=70)
    batch.draft_len = torch.tensor([7, 0, 3, 7, 5, 1], dtype=torch.int32)
    options = am.Options(base_test=1, list_update=1, apply_update=1)
    out, st, _ = G.run_gpu(am, batch, options=options)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref, info_bits=16 | 8)
    host = {k: np.array(v, copy=True) for k, v in batch.state.items()}
    oracle.update(host, ref["n_accept"], batch.draft_len.numpy(), ref["H_q"], ref["d_js"], batch.k, d_eps=1e-6)
    got = st.to_host()
    if rep["flips"] == 0 and rep["member_flips"] == 0:
        for k in ("nA", "nR", "ent_cnt"):
            assert np.array_equal(got[k], host[k]), k


def test_literal_variant_status_and_float64_path(am, wl, oracle):
    """Broken draft token at the rejected position (nothing to exclude), and replacement draws whose two
    best keys nearly tie, found with the oracle: those take the float64 path, exclusion included."""
    V = 256
    g = torch.Generator().manual_seed(9)
    n = 150000
    t = (torch.randn(1, 2, V, generator=g) * 2).repeat(n, 1, 1).contiguous()
    d = (torch.randn(1, 1, V, generator=g) * 2).repeat(n, 1, 1).contiguous()
    tok = torch.full((n, 1), 3, dtype=torch.int32)
    ref = oracle.verify(t.numpy(), d.numpy(), tok.numpy(), seed=31, relaxed_off=1, base_test=1)
    rej = ref["n_accept"] == 0
    close_call = np.flatnonzero(rej & (ref["top2_gap"] < 5e-5))[:6]
    assert len(close_call) >= 2, "no near tie among the draws: widen the search"
    ids = np.concatenate([close_call, np.flatnonzero(rej)[:2]]).astype(np.uint32)
    B = len(ids)
    tok_b = tok[:B].clone()
    tok_b[-1, 0] = V + 7                                   # broken token: rejected, the row is sampled as it is
    batch = wl.VerifyBatch(t[:B].contiguous(), d[:B].contiguous(), tok_b, None, wl.empty_state(B, 8), 31)
    options = am.Options(base_test=1, relaxed_off=1)
    out, _, _ = G.run_gpu(am, batch, options=options, seq_id=ids)
    refb = G.run_oracle(oracle, batch, options=options, seq_id=ids)
    rep = G.compare_verify(out, refb)
    _report("literal exact path", rep)
    assert np.array_equal(refb["next_token"][:len(close_call)], ref["next_token"][close_call])
    st = out.status.cpu().numpy()
    assert rep["exact_path"] >= 1
    assert st[-1] & am.binding.ST_BAD_TOKEN and out.n_accept[-1].item() == 0
    assert (out.next_token.cpu().numpy()[:-1] != 3).all()


# ------------------------------------------------------------------------------- long histories
@pytest.mark.parametrize("n_hist,cap,path", [(64, 512, 1), (700, 1024, 1), (700, 1024, 2), (5000, 5003, 1), (40000, 40100, 1),
                                             (64, 20000, 1), (5000, 20000, 1), (17000, 20000, 1), (131072, 131100, 2)])
@pytest.mark.parametrize("opt", [dict(), dict(list_update=1, base_test=1), dict(bw_rule=1, reject_rule=1)],
                         ids=["default", "literal", "scott-map"])
def test_long_history_lists_take_the_workgroup_per_position_path(am, wl, oracle, n_hist, cap, opt, path):
    """From a list capacity of 512 on, the decision stage gives every position a workgroup of its own
    (path: which statistics kernels ran before it)."""
    batch = wl.config_batched(B=5, k=6, V=8192, seed=300 + n_hist, cap=cap)
    g = torch.Generator().manual_seed(n_hist)
    batch.state = wl.threshold_state(batch.B, cap, g, n_hist=n_hist)
    batch.state["nA"][1] = max(n_hist - 37, 0)                 # lists of different lengths
    batch.state["nR"][2] = max(n_hist // 2, 2)
    batch.state["nA"][3] = cap - 2                             # nearly full: in-loop appends hit the capacity
    batch.state["LA"][3, n_hist:cap - 2] = batch.state["LA"][3, :cap - 2 - n_hist] if cap - 2 - n_hist <= n_hist else 0.3
    batch.draft_len = torch.tensor([6, 6, 4, 6, 0], dtype=torch.int32)
    options = am.Options(**opt)
    out, _, _ = G.run_gpu(am, batch, options=options, stats_path=path)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref)
    _report(f"long history n={n_hist} {opt}", rep)
    assert (ref["p_accept"] > 0).any()


def test_long_history_with_the_update_in_the_same_call_and_status_bits(am, wl, oracle):
    cap = 600
    batch = wl.config_batched(B=6, k=7, V=8192, seed=91, cap=cap)
    g = torch.Generator().manual_seed(2)
    batch.state = wl.threshold_state(batch.B, cap, g, n_hist=cap - 3)      # three free slots: appends overflow
    batch.draft_len = torch.tensor([7, 0, 3, 7, 5, 9], dtype=torch.int32)  # 9: out of range, clamped and flagged
    batch.draft[2, 1, 5] = float("nan")
    batch.draft_tokens[3, 2] = -4
    oracle_len = batch.draft_len.clamp(0, 7)
    a, st_a, _ = G.run_gpu(am, batch)
    am.update_thresholds(st_a, batch.k, a.n_accept, a.H_q, a.d_js, draft_len=batch.draft_len.cuda(), status=a.status)
    b, st_b, _ = G.run_gpu(am, batch, options=am.Options(apply_update=1))
    torch.cuda.synchronize()
    for name in ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept", "accept_mask", "status"):
        ga, gb = getattr(a, name), getattr(b, name)
        assert torch.equal(torch.nan_to_num(ga.float(), nan=-7.0), torch.nan_to_num(gb.float(), nan=-7.0)), name
    ha, hb = st_a.to_host(), st_b.to_host()
    for k in ha:
        assert np.array_equal(ha[k], hb[k]), k
    st = b.status.cpu().numpy()
    assert st[5] & am.binding.ST_BAD_LENGTH and st[2] & am.binding.ST_NONFINITE and st[3] & am.binding.ST_BAD_TOKEN
    ref_batch = wl.VerifyBatch(batch.target, batch.draft, batch.draft_tokens, oracle_len, batch.state, batch.seed)
    ref = G.run_oracle(oracle, ref_batch)
    G.compare_verify(b, ref, info_bits=16 | 8 | am.binding.ST_BAD_LENGTH)
    host = {k: np.array(v, copy=True) for k, v in batch.state.items() if k != "tau"}
    oracle.update(host, ref["n_accept"], oracle_len.numpy(), ref["H_q"], ref["d_js"], batch.k, d_eps=1e-6)
    for k in ("nA", "nR", "ent_cnt"):
        assert np.array_equal(hb[k], host[k]), k


def test_many_sequences_with_long_histories(am, wl, oracle):
    """More sequences than the arrival-counter arrays have cache lines: the counters of neighbouring
    sequences share lines again, in the sampling kernel and in the per-position decision kernel."""
    B, cap = 1200, 600
    batch = wl.config_batched(B=B, k=2, V=520, seed=12, cap=cap)
    g = torch.Generator().manual_seed(3)
    batch.state = wl.threshold_state(B, cap, g, n_hist=500)
    out, _, _ = G.run_gpu(am, batch, options=am.Options(apply_update=1))
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref, info_bits=16 | 8)
    _report("many sequences", rep)


def test_long_history_largest_window(am, wl, oracle):
    cap = 2000
    batch = wl.config_batched(B=2, k=64, V=4099, seed=6, cap=cap)
    g = torch.Generator().manual_seed(4)
    batch.state = wl.threshold_state(batch.B, cap, g, n_hist=1990)          # room for 10 in-loop appends
    options = am.Options(list_update=1)
    out, _, _ = G.run_gpu(am, batch, options=options)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref)
    _report("long history K=64", rep)


# ------------------------------------------------------------------------------- column-sharded verification
def _column_cuts(V, G):
    """G column ranges that tile [0, V): starts are multiples of 8, sizes deliberately uneven."""
    cuts = [0]
    for g in range(1, G):
        c = (V * g // G) // 8 * 8 + (8 if g % 2 else 0)
        cuts.append(min(max(c, cuts[-1] + 8), V - 8 * (G - g)))
    return cuts + [V]


def _sharded_decisions(am, batch, n_sh, options=None, seq_id=None):
    """Stages 1-3 of the column-sharded path on one device: G calls on column slices per stage."""
    B, K, V = batch.B, batch.k, batch.V
    t, d, x = batch.target.cuda(), batch.draft.cuda(), batch.draft_tokens.cuda()
    dl = G.to_dev(batch.draft_len)
    cuts = _column_cuts(V, n_sh)
    wss = [am.Workspace(B, max(K, 1), V, batch.target.dtype) for _ in range(n_sh)]      # one per holder
    shards = [am.Shard(n_sh, g, V, cuts[g]) for g in range(n_sh)]
    views = [(t[:, :, cuts[g]:cuts[g + 1]], d[:, :, cuts[g]:cuts[g + 1]]) for g in range(n_sh)]
    rows, P = B * K * 2, B * K
    triples_all = torch.empty(n_sh, rows, 4, device="cuda")
    pos_all = torch.empty(n_sh, P, 4, device="cuda")
    for g in range(n_sh):
        am.verify_shard_stats(views[g][0], views[g][1], x, wss[g], shards[g], draft_len=dl, triples_out=triples_all[g])
    for g in range(n_sh):
        am.verify_shard_jsd(views[g][0], views[g][1], x, wss[g], shards[g], triples_all, draft_len=dl, pos_out=pos_all[g])
    cap = batch.state["LA"].shape[1]
    outs, states = [], []
    sid = None if seq_id is None else torch.tensor(np.asarray(seq_id, dtype=np.uint32).view(np.int32)).cuda()
    for g in range(n_sh):                                # replicated: every holder must get the same
        st = G.state_to_device(am, batch.state, B, cap)
        outs.append(am.verify_shard_decide(B, K, batch.target.dtype, x, wss[g], shards[g], triples_all, pos_all,
                                           state=st, draft_len=dl, seed=batch.seed, seq_id=sid,
                                           round0=batch.round0, options=options))
        states.append(st)
    torch.cuda.synchronize()
    return outs, states, wss, shards, views, (triples_all, pos_all)


@pytest.mark.parametrize("G_", [1, 2, 5, 8])
@pytest.mark.parametrize("opt", [dict(), dict(base_test=1, list_update=1), dict(apply_update=1)],
                         ids=["default", "literal", "update"])
def test_column_sharded_statistics_and_decisions(am, wl, oracle, G_, opt):
    batch = wl.config_batched(B=5, k=6, V=32000, seed=400 + G_, cap=96)
    batch.draft_len = torch.tensor([6, 0, 3, 6, 5], dtype=torch.int32)
    batch.draft_tokens[3, 1] = 32000 + 5                       # out of range: no holder owns it
    batch.draft[2, 1, 31999] = float("nan")                    # broken row, seen by the last holder only
    options = am.Options(**opt)
    outs, states, *_ = _sharded_decisions(am, batch, G_, options=options)
    ref = G.run_oracle(oracle, batch, options=options)
    names = ("n_accept", "H_p", "H_q", "d_js", "p_accept", "accept_mask", "status")
    for o in outs[1:]:                                         # the replicas agree bit for bit
        for n in names:
            assert torch.equal(torch.nan_to_num(getattr(o, n).float(), nan=-7.0),
                               torch.nan_to_num(getattr(outs[0], n).float(), nan=-7.0)), n
    got = outs[0]
    got.next_token = torch.tensor(ref["next_token"], dtype=torch.int32).cuda()      # (not produced by this stage)
    sampled_bits = am.binding.ST_ZERO_MASS | am.binding.ST_EXACT_PATH
    ref_status = ref["status"].copy()
    ref["status"] = ref_status & ~np.uint32(sampled_bits)      # bits that only the sampling stage sets
    rep = G.compare_verify(got, ref, info_bits=16 | 8)
    _report(f"sharded G={G_} {opt}", rep)
    assert rep["flips"] == 0
    if opt.get("apply_update"):
        host = {k: np.array(v, copy=True) for k, v in batch.state.items() if k != "tau"}
        oracle.update(host, ref["n_accept"], batch.draft_len.numpy(), ref["H_q"], ref["d_js"], batch.k, d_eps=1e-6)
        hb = states[0].to_host()
        for k in ("nA", "nR", "ent_cnt"):
            assert np.array_equal(hb[k], host[k]), k


def _sharded_tokens(am, batch, ctx, outs, seq_id=None):
    """Stages 4-7 on one device, after _sharded_decisions: the token of every sequence on every replica."""
    outs_, states, wss, shards, views, _ = ctx
    B, K = batch.B, batch.k
    n_sh = len(shards)
    x = batch.draft_tokens.cuda()
    dl = G.to_dev(batch.draft_len)
    sid = None if seq_id is None else torch.tensor(np.asarray(seq_id, dtype=np.uint32).view(np.int32)).cuda()
    kw = dict(draft_len=dl, seed=batch.seed, seq_id=sid, round0=batch.round0)
    top_all = torch.empty(n_sh, B, 4, device="cuda")
    cand_all = torch.empty(n_sh, B, am.binding.SHARD_CAND_BYTES, dtype=torch.uint8, device="cuda")
    for g in range(n_sh):
        am.verify_shard_sample(views[g][0], views[g][1], x, wss[g], shards[g], top_out=top_all[g], **kw)
    taus = [am.verify_shard_pick(B, K, batch.target.dtype, x, wss[g], shards[g], top_all, outs[g], draft_len=dl)
            for g in range(n_sh)]
    open_after_pick = int(torch.isfinite(taus[0]).sum())
    for exact in (0, 1):               # the second pass (float64-exact sums) only works on what the first left open
        for g in range(n_sh):
            am.verify_shard_refine(views[g][0], views[g][1], x, wss[g], shards[g], taus[g], cand_out=cand_all[g],
                                   exact_sums=exact, **kw)
        for g in range(n_sh):
            am.verify_shard_settle(B, K, batch.target.dtype, x, wss[g], shards[g], taus[g], cand_all, outs[g], **kw)
        torch.cuda.synchronize()
        if exact == 0:
            open_after_first = int(torch.isfinite(taus[0]).sum())
    return open_after_pick, open_after_first


@pytest.mark.parametrize("n_sh", [1, 3, 8])
@pytest.mark.parametrize("opt", [dict(), dict(base_test=1, list_update=1)], ids=["default", "literal"])
def test_column_sharded_round_gives_the_oracles_tokens(am, wl, oracle, n_sh, opt):
    batch = wl.config_batched(B=8, k=6, V=32000, seed=500 + n_sh, cap=96)
    batch.draft_len = torch.tensor([6, 0, 3, 6, 5, 6, 1, 6], dtype=torch.int32)
    batch.target[5, 6, 17] = float("inf")                      # broken bonus row (only matters if it is sampled)
    options = am.Options(**opt)
    ctx = _sharded_decisions(am, batch, n_sh, options=options)
    outs = ctx[0]
    _sharded_tokens(am, batch, ctx, outs)
    ref = G.run_oracle(oracle, batch, options=options)
    for o in outs[1:]:
        assert torch.equal(o.next_token, outs[0].next_token) and torch.equal(o.status, outs[0].status)
    rep = G.compare_verify(outs[0], ref)
    _report(f"sharded round G={n_sh} {opt}", rep)
    assert rep["flips"] == 0
    assert (outs[0].status & am.binding.ST_UNSETTLED == 0).all()
    # the whole-vocabulary call gives the same integers
    whole, _, _ = G.run_gpu(am, batch, options=options)
    assert torch.equal(whole.next_token, outs[0].next_token) and torch.equal(whole.n_accept, outs[0].n_accept)


@pytest.mark.parametrize("mode", ["residual", "bonus", "exclude"])
@pytest.mark.parametrize("dtype,V", [(torch.bfloat16, 4104), (torch.float32, 2056)], ids=["bf16", "f32"])
def test_column_sharded_near_ties_are_settled_from_the_exchanged_candidates(am, wl, oracle, mode, dtype, V):
    g = torch.Generator().manual_seed(V)
    t = (torch.randn(1, 2, V, generator=g) * 2.5).to(dtype)
    d = (t[:, :1].float() + torch.randn(1, 1, V, generator=g)).to(dtype)
    p = torch.softmax(t[0, 0].double(), -1)
    q = torch.softmax(d[0, 0].double(), -1)
    n = 100000
    x = int(torch.argmax(q - p)) if mode == "residual" else int(torch.argmax(p - q))
    opt = dict(relaxed_off=1)
    if mode == "exclude":
        opt["base_test"] = 1
        x = int(torch.argmin(p))
    ref = oracle.verify(t, d, np.full((n, 1), x, np.int32), seed=41, shared_rows=True, **opt)
    sel = (ref["n_accept"] == (1 if mode == "bonus" else 0))
    close_call = np.flatnonzero(sel & (ref["top2_gap"] < 1e-4))[:16]
    assert len(close_call) >= 2
    ids = close_call.astype(np.uint32)
    B = len(ids)
    batch = wl.VerifyBatch(t.repeat(B, 1, 1).contiguous(), d.repeat(B, 1, 1).contiguous(),
                           torch.full((B, 1), x, dtype=torch.int32), None, wl.empty_state(B, 8), 41)
    options = am.Options(**opt)
    ctx = _sharded_decisions(am, batch, 4, options=options, seq_id=ids)
    outs = ctx[0]
    n_open, n_open2 = _sharded_tokens(am, batch, ctx, outs, seq_id=ids)
    refb = G.run_oracle(oracle, batch, options=options, seq_id=ids)
    assert np.array_equal(refb["next_token"], ref["next_token"][close_call])
    rep = G.compare_verify(outs[0], refb)
    st = outs[0].status.cpu().numpy()
    print(f"[sharded near ties] {mode} V={V}: {B} draws, {n_open} open after the pick, {n_open2} after the first "
          f"settle, {(st & 16 != 0).sum()} settled in float64", flush=True)
    assert rep["flips"] == 0 and (st & am.binding.ST_UNSETTLED == 0).all() and (st & 16 != 0).sum() >= 1


def test_column_sharded_draw_without_certain_mass_is_flagged(am, wl, oracle):
    """Identical target and draft rows with a broken draft token: the rejection leaves a residual without
    mass, which only the whole-row float64 path of the unsharded call can turn into a draw."""
    V = 2048
    g = torch.Generator().manual_seed(4)
    z = (torch.randn(V, generator=g) * 2).to(torch.bfloat16)
    t = z.repeat(2, 2, 1).clone()
    d = z.repeat(2, 1, 1).clone()
    tok = torch.tensor([[V + 5], [3]], dtype=torch.int32)
    batch = wl.VerifyBatch(t, d, tok, None, wl.empty_state(2, 8), 11)
    ctx = _sharded_decisions(am, batch, 2)
    outs = ctx[0]
    _sharded_tokens(am, batch, ctx, outs)
    st = outs[0].status.cpu().numpy()
    assert st[0] & am.binding.ST_UNSETTLED and st[0] & am.binding.ST_BAD_TOKEN
    ref = G.run_oracle(oracle, batch)
    assert st[1] == 0 and outs[0].next_token[1].item() == ref["next_token"][1]       # accepted: bonus token as usual


def test_column_sharded_round_with_long_histories_and_without_drafts(am, wl, oracle):
    cap = 600
    batch = wl.config_batched(B=4, k=5, V=8192, seed=77, cap=cap)
    g = torch.Generator().manual_seed(9)
    batch.state = wl.threshold_state(batch.B, cap, g, n_hist=520)            # the per-position decision kernel
    options = am.Options(base_test=1, list_update=1)
    ctx = _sharded_decisions(am, batch, 3, options=options)
    _sharded_tokens(am, batch, ctx, ctx[0])
    rep = G.compare_verify(ctx[0][0], G.run_oracle(oracle, batch, options=options))
    _report("sharded long history", rep)
    # no drafted positions at all: only the bonus token is drawn
    b0 = wl.VerifyBatch(batch.target[:, :1].contiguous(), batch.draft[:, :0].contiguous(),
                        batch.draft_tokens[:, :0].contiguous(), None, wl.empty_state(batch.B, 8), batch.seed)
    ctx0 = _sharded_decisions(am, b0, 2)
    _sharded_tokens(am, b0, ctx0, ctx0[0])
    ref0 = G.run_oracle(oracle, b0)
    assert np.array_equal(ctx0[0][0].next_token.cpu().numpy(), ref0["next_token"])
    assert (ctx0[0][0].n_accept == 0).all()


def test_literal_variant_without_a_state(am, wl, oracle):
    batch = wl.config_batched(B=4, k=5, V=8192, seed=78)
    batch.state = {}
    t, d, x = batch.target.cuda(), batch.draft.cuda(), batch.draft_tokens.cuda()
    ws = am.Workspace(batch.B, batch.k, batch.V, torch.bfloat16)
    options = am.Options(base_test=1, list_update=1)
    out = am.verify(t, d, x, ws, seed=batch.seed, options=options)
    torch.cuda.synchronize()
    ref = oracle.verify(batch.target, batch.draft, x.cpu().numpy(), seed=batch.seed, base_test=1, list_update=1)
    ref["posterior_at"] = lambda b, i, dd: 0.0
    rep = G.compare_verify(out, ref)
    assert rep["flips"] == 0 and (out.p_accept == 0).all()


def test_column_sharded_argument_errors(am):
    ws = am.Workspace(2, 2, 64, torch.float32)
    t = torch.zeros(2, 3, 64, device="cuda")
    d = torch.zeros(2, 2, 64, device="cuda")
    tok = torch.zeros(2, 2, dtype=torch.int32, device="cuda")
    for bad in (am.Shard(2, 2, 64, 0), am.Shard(2, 1, 64, 4), am.Shard(2, 1, 64, 32), am.Shard(65, 0, 64, 0)):
        with pytest.raises(am.AdasdError):
            am.verify_shard_stats(t[:, :, :40], d[:, :, :40], tok, ws, bad)


# ------------------------------------------------------------------------------- seeded random shapes
@pytest.mark.parametrize("case", range(48))
def test_random_shapes_and_options(am, wl, oracle, case):
    """Seeded draws of shape, dtype, lengths, history sizes and options: whatever combination comes up has
    to meet the same bar."""
    rng = np.random.default_rng(9000 + case)
    B = int(rng.integers(1, 7))
    K = int(rng.choice([1, 2, 3, 5, 8, 13, 20]))
    V = int(rng.choice([9, 64, 257, 1000, 2048, 4099, 8200, 12345]))
    dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
    cap = int(rng.choice([8, 40, 300, 600, 5000]))
    n_hist = int(min(cap, rng.choice([0, 1, 2, 30, 200, 450, 4200])))
    batch = wl.config_batched(B=B, k=K, V=V, seed=1000 + case, dtype=dtype, cap=64)
    g = torch.Generator().manual_seed(case)
    st = wl.threshold_state(B, cap, g, n_hist=max(n_hist, 1))
    st["nA"][:] = np.minimum(n_hist, rng.integers(0, n_hist + 1, B) + n_hist // 2)
    st["nR"][:] = np.minimum(n_hist, rng.integers(0, n_hist + 1, B) + n_hist // 2)
    batch.state = st
    if rng.random() < 0.5:
        batch.draft_len = torch.tensor(rng.integers(0, K + 1, B), dtype=torch.int32)
    if rng.random() < 0.3:
        batch.draft_tokens[rng.integers(0, B), rng.integers(0, K)] = V + 3        # a broken token
    if rng.random() < 0.3:
        batch.target[rng.integers(0, B), rng.integers(0, K + 1), : V // 2] = float("-inf")
    opt = dict(base_test=int(rng.integers(0, 2)), list_update=int(rng.integers(0, 2)),
               reject_rule=int(rng.integers(0, 2)), bw_rule=int(rng.integers(0, 2)),
               apply_update=int(rng.integers(0, 2)), kde_min_n=int(rng.choice([0, 2, 5])))
    options = am.Options(**opt)
    seq_id = rng.integers(0, 2 ** 32, B, dtype=np.uint64).astype(np.uint32)
    out, _, _ = G.run_gpu(am, batch, options=options, seq_id=seq_id, stats_path=int(rng.integers(1, 3)))
    ref = G.run_oracle(oracle, batch, options=options, seq_id=seq_id)
    rep = G.compare_verify(out, ref, info_bits=16 | 8)
    print(f"[random {case}] B={B} K={K} V={V} {dtype} cap={cap} n={n_hist} {opt}: flips={rep['flips']}", flush=True)
    assert rep["flips"] <= 1


def _extreme_rows(rng, batch, B, K, V, dtype, mode):
    """Rows far from the configurations' recipe: 0 nearly all mass on one token (target and mostly also draft),
    1 large offsets and scales, 2 draft rows next to the target rows (tiny distances), 3 flat rows."""
    t, d = batch.target.float(), batch.draft.float()
    if mode == 0:
        for b in range(B):
            for i in range(K + 1):
                at = int(rng.integers(0, V)); amp = float(rng.uniform(8, 40))
                t[b, i, at] += amp
                if i < K and rng.random() < 0.7:
                    d[b, i, at] += amp * float(rng.uniform(0.5, 1.1))
    elif mode == 1:
        t = t * float(rng.uniform(0.1, 12)) + float(rng.uniform(-80, 80))
        d = d * float(rng.uniform(0.1, 12)) + float(rng.uniform(-80, 80))
    elif mode == 2:
        d = t[:, :K] + torch.randn(B, K, V) * float(rng.choice([1e-3, 1e-2, 0.05]))
    else:
        t = t * 0.01; d = d * 0.01
    batch.target, batch.draft = t.to(dtype), d.to(dtype)


@pytest.mark.parametrize("case", [257, 413, 626] + list(range(1000, 1021)))
def test_rows_with_extreme_shapes_and_random_options(am, wl, oracle, case):
    """Seeded draws of peaked, shifted and scaled, near-identical and flat rows with random options, history
    sizes, window lengths and statistics path (the first three seeds are cases a randomised sweep once
    failed on: posteriors after in-loop appends of distances below the floor of the divergence)."""
    rng = np.random.default_rng(41000 + case)
    B = int(rng.integers(1, 6)); K = int(rng.choice([1, 3, 6, 11])); V = int(rng.choice([64, 1000, 2048, 4104, 8200, 32768]))
    dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
    batch = wl.config_batched(B=B, k=K, V=V, seed=5000 + case, dtype=dtype, cap=64)
    mode = int(rng.integers(0, 4))
    _extreme_rows(rng, batch, B, K, V, dtype, mode)
    path = int(rng.integers(1, 3))
    opt = dict(base_test=int(rng.integers(0, 2)), list_update=int(rng.integers(0, 2)), reject_rule=int(rng.integers(0, 2)),
               apply_update=int(rng.integers(0, 2)))
    options = am.Options(**opt)
    if rng.random() < 0.5:
        g = torch.Generator().manual_seed(case)
        cap = int(rng.choice([100, 600, 3000]))
        n_hist = int(rng.choice([2, 64, 90, 450, 2500])) if cap >= 2500 else int(rng.choice([2, 64, 90]))
        batch.state = wl.threshold_state(B, cap, g, n_hist=n_hist)
    if rng.random() < 0.4:
        batch.draft_len = torch.tensor(rng.integers(0, K + 1, B), dtype=torch.int32)
    out, _, _ = G.run_gpu(am, batch, options=options, stats_path=path)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref, info_bits=16 | 8)
    _report(f"extreme rows {case}: mode {mode} path {path} {opt}", rep)


# ------------------------------------------------------------------------------- close calls of the argmax
@pytest.mark.parametrize("dtype,V", [(torch.bfloat16, 4104), (torch.float32, 2056), (torch.bfloat16, 4107)],
                         ids=["bf16-2slices", "f32-2slices", "bf16-unaligned"])
@pytest.mark.parametrize("mode", ["residual", "bonus", "exclude"])
def test_near_ties_of_the_gumbel_argmax_are_settled_in_float64(am, wl, oracle, mode, dtype, V):
    """Draws whose two best keys lie closer than the float keys can tell apart, found with the oracle
    among many draws on one pair of rows; the GPU must return the oracle's token for every one."""
    g = torch.Generator().manual_seed(V)
    t = (torch.randn(1, 2, V, generator=g) * 2.5).to(dtype)
    d = (t[:, :1].float() + torch.randn(1, 1, V, generator=g)).to(dtype)
    p = torch.softmax(t[0, 0].double(), -1)
    q = torch.softmax(d[0, 0].double(), -1)
    n = 100000
    x = int(torch.argmax(q - p)) if mode == "residual" else int(torch.argmax(p - q))   # mostly rejected | always accepted
    opt = dict(relaxed_off=1)
    if mode == "exclude":
        opt["base_test"] = 1
        x = int(torch.argmin(p))
    tok = np.full((n, 1), x, np.int32)
    ref = oracle.verify(t, d, tok, seed=41, shared_rows=True, **opt)
    want_reject = mode != "bonus"
    sel = (ref["n_accept"] == (0 if want_reject else 1))
    close_call = np.flatnonzero(sel & (ref["top2_gap"] < 1e-4))[:16]
    assert len(close_call) >= 2, "no near tie among the draws: widen the search"
    ids = close_call.astype(np.uint32)
    B = len(ids)
    batch = wl.VerifyBatch(t.repeat(B, 1, 1).contiguous(), d.repeat(B, 1, 1).contiguous(),
                           torch.full((B, 1), x, dtype=torch.int32), None, wl.empty_state(B, 8), 41)
    options = am.Options(**opt)
    out, _, _ = G.run_gpu(am, batch, options=options, seq_id=ids)
    refb = G.run_oracle(oracle, batch, options=options, seq_id=ids)
    assert np.array_equal(refb["next_token"], ref["next_token"][close_call])
    rep = G.compare_verify(out, refb)
    _report(f"near ties {mode} V={V}", rep)
    assert rep["flips"] == 0 and rep["exact_path"] >= 1       # too close for the float keys


# ------------------------------------------------------------------------------- degenerate inputs
def test_masked_identical_and_disjoint_rows(am, wl, oracle, path):
    V, K = 4100, 4
    g = torch.Generator().manual_seed(3)
    t = torch.randn(1, K + 1, V, generator=g) * 3
    d = torch.randn(1, K, V, generator=g) * 3
    ninf = float("-inf")
    d[0, 0] = t[0, 0]                                  # identical rows: d = 0, always accepted
    t[0, 1, : V // 2] = ninf; d[0, 1, V // 2:] = ninf  # disjoint supports: d = 1
    t[0, 2, 5:900] = ninf                              # partially masked target
    d[0, 3, 17] = ninf
    tok = torch.tensor([[3, V // 2 - 1, 7, 17]], dtype=torch.int32)   # q(x)>0,p(x)=0 | p=0 | q(x)=0
    batch = wl.VerifyBatch(t.to(torch.bfloat16), d.to(torch.bfloat16), tok, None, wl.empty_state(1, 8), 5)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref)
    _report("masked", rep)
    assert out.d_js[0, 0].item() == 0.0 and ref["d_js"][0, 0] == 0.0
    assert out.d_js[0, 1].item() == pytest.approx(1.0, abs=1e-6) and ref["d_js"][0, 1] == pytest.approx(1.0)
    assert ref["n_accept"][0] == 1


def test_status_bits_and_exact_path(am, wl, oracle, path):
    V = 2048
    g = torch.Generator().manual_seed(4)
    z = (torch.randn(V, generator=g) * 2).to(torch.bfloat16)
    B = 5
    t = z.repeat(B, 2, 1).clone()
    d = z.repeat(B, 1, 1).clone()
    tok = torch.tensor([[V + 5], [-1], [3], [3], [3]], dtype=torch.int32)
    d[2, 0, 100] = float("nan")          # NaN in a draft row
    t[3, 1, 7] = float("inf")            # +inf in the bonus row only
    t[4, 1, :] = float("-inf")           # bonus row without any finite logit
    batch = wl.VerifyBatch(t, d, tok, None, wl.empty_state(B, 8), 11)
    out, _, _ = G.run_gpu(am, batch, stats_path=path)
    ref = G.run_oracle(oracle, batch)
    rep = G.compare_verify(out, ref)
    _report("status", rep)
    st = out.status.cpu().numpy()
    # sequences 0,1: bad token -> rejected at identical rows -> residual has no mass -> float64 path
    assert st[0] == am.binding.ST_BAD_TOKEN | am.binding.ST_ZERO_MASS | am.binding.ST_EXACT_PATH
    assert st[1] == st[0]
    assert st[2] & am.binding.ST_NONFINITE and out.next_token[2].item() == -1
    assert math.isnan(out.d_js[2, 0].item()) and math.isnan(out.H_p[2, 0].item())
    assert st[3] & am.binding.ST_NONFINITE and out.next_token[3].item() == -1 and out.n_accept[3].item() == 1
    assert st[4] & am.binding.ST_NONFINITE and out.next_token[4].item() == -1


def test_no_drafts_and_empty_batch(am, wl, oracle):
    batch = wl.config_batched(B=3, k=2, V=5000, seed=8)
    batch.draft_len = torch.zeros(3, dtype=torch.int32)
    out, _, ws = G.run_gpu(am, batch)
    ref = G.run_oracle(oracle, batch)
    G.compare_verify(out, ref)
    assert (out.n_accept == 0).all()
    # k_max = 0: only the bonus row exists
    t0 = batch.target[:, :1].contiguous()
    b0 = wl.VerifyBatch(t0, batch.draft[:, :0].contiguous(), batch.draft_tokens[:, :0].contiguous(),
                        None, batch.state, batch.seed)
    out0, _, _ = G.run_gpu(am, b0)
    ref0 = G.run_oracle(oracle, b0)
    assert np.array_equal(out0.next_token.cpu().numpy(), ref0["next_token"])
    # B = 0 is a no-op
    e = torch.empty(0, 3, 64, dtype=torch.bfloat16, device="cuda")
    am.verify(e, e[:, :2], torch.empty(0, 2, dtype=torch.int32, device="cuda"), ws)


def test_argument_errors_are_reported_before_any_launch(am):
    ws = am.Workspace(2, 2, 64, torch.float32)
    t = torch.zeros(2, 3, 64, device="cuda")
    d = torch.zeros(2, 2, 64, device="cuda")
    tok = torch.zeros(2, 2, dtype=torch.int32, device="cuda")
    with pytest.raises(am.AdasdError) as e:
        am.verify(t, d, tok, ws, options=am.Options(base_test=2))
    assert e.value.code == -1
    with pytest.raises(am.AdasdError) as e:
        am.verify(t, d, tok, ws, options=am.Options(list_update=3))
    assert e.value.code == -1
    small = am.Workspace(1, 1, 64, torch.float32)
    with pytest.raises(am.AdasdError) as e:
        am.verify(t, d, tok, small)
    assert e.value.code == -4
    with pytest.raises(am.AdasdError) as e:
        am.verify(torch.zeros(2, 80, 64, device="cuda"), torch.zeros(2, 79, 64, device="cuda"),
                  torch.zeros(2, 79, dtype=torch.int32, device="cuda"), ws)
    assert e.value.code == -5
    with pytest.raises(am.AdasdError) as e:
        am.verify(t, d, tok, ws, options=am.Options(reject_rule=7))
    assert e.value.code == -1


# ------------------------------------------------------------------------------- draft side
def test_draft_entropy_rule(am, wl, oracle):
    g = torch.Generator().manual_seed(21)
    B, V = 37, 128256
    z = (torch.randn(B, V, generator=g) * torch.linspace(0.5, 6, B).reshape(B, 1)).to(torch.bfloat16)
    z[5] = 1.5                                     # uniform row: H = ln V
    z[6] = float("-inf"); z[6, 77] = 2.0           # one-hot: H = 0
    z[7, 3] = float("nan")
    active = torch.ones(B, dtype=torch.uint8); active[11] = 0
    tg = torch.rand(B, generator=g) * 12
    tg[6] = 0.0                                    # H = 0 is not > 0: keep drafting
    ws = am.Workspace(B, 1, V, torch.bfloat16)
    H, stop = am.draft_entropy(z.cuda(), ws, T_G=tg.cuda(), active=active.cuda(), step=3, k_max=20)
    torch.cuda.synchronize()
    Href, sref = oracle.draft_entropy(z, T_G=tg.numpy(), active=active.numpy(), step=3, k_max=20)
    Hg, sg = H.cpu().numpy(), stop.cpu().numpy()
    ok = [b for b in range(B) if b != 7]
    assert G.close(Hg[ok], Href[ok]).all()
    assert Hg[5] == pytest.approx(math.log(V), rel=1e-6) and Hg[6] == 0.0 and Hg[11] == 0.0
    assert math.isnan(Hg[7]) and sg[7] == 1
    near = np.abs(Href - tg.numpy()) < 1e-5 * np.abs(Href) + 1e-6
    cmp = [b for b in ok if not near[b]]
    assert np.array_equal(sg[cmp], sref[cmp])
    assert sg[6] == 0 and sg[11] == 0
    # window cap forces the stop
    _, stop2 = am.draft_entropy(z.cuda(), ws, T_G=tg.cuda(), active=active.cuda(), step=19, k_max=20)
    s2 = stop2.cpu().numpy()
    assert s2[6] == 1 and s2[11] == 0 and s2[ok].sum() == len(ok) - 1
    # no threshold given: only the cap can stop
    _, stop3 = am.draft_entropy(z.cuda(), ws, step=0, k_max=20)
    assert stop3.cpu().numpy()[ok].sum() == 0


# ------------------------------------------------------------------------------- drafting step with the token draw
def _draft_step_case(am, oracle, z, **kw):
    B, V = z.shape
    ws = am.Workspace(B, 1, V, z.dtype)
    dev = {k: (None if v is None else torch.as_tensor(v).cuda()) for k, v in kw.items()
           if k in ("T_G", "active", "seq_id", "rounds")}
    if dev.get("seq_id") is not None:
        dev["seq_id"] = torch.tensor(np.asarray(kw["seq_id"], np.uint32).view(np.int32)).cuda()
    if dev.get("rounds") is not None:
        dev["rounds"] = torch.tensor(np.asarray(kw["rounds"], np.uint32).view(np.int32)).cuda()
    scal = {k: kw[k] for k in ("step", "k_max", "seed", "round0") if k in kw}
    H, stop, tok, st = am.draft_step(z.cuda(), ws, **dev, **scal)
    He, stope = am.draft_entropy(z.cuda(), ws, T_G=dev.get("T_G"), active=dev.get("active"),
                                 step=scal.get("step", 0), k_max=scal.get("k_max", 1 << 30))
    torch.cuda.synchronize()
    # entropy and stop flag are those of the entropy-only call, bit for bit
    assert torch.equal(H.view(torch.int32), He.view(torch.int32)) and torch.equal(stop, stope)
    ref_tok, gap = oracle.draft_sample(z, active=kw.get("active"), step=scal.get("step", 0),
                                       seed=scal.get("seed", 0), seq_id=kw.get("seq_id"),
                                       rounds=kw.get("rounds"), round0=scal.get("round0", 0))
    return H.cpu().numpy(), stop.cpu().numpy(), tok.cpu().numpy(), st.cpu().numpy(), ref_tok, gap


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [8, 100, 1001, 4096, 20011, 128256])
def test_draft_step_draws_the_oracles_tokens(am, wl, oracle, dtype, V):
    g = torch.Generator().manual_seed(V + 1)
    B = 19
    z = (torch.randn(B, V, generator=g) * torch.linspace(0.5, 5, B).reshape(B, 1)).to(dtype)
    z[3, : V // 2] = float("-inf")                       # masked tokens are never drawn
    active = np.ones(B, np.uint8); active[4] = 0
    seq = np.arange(B, dtype=np.uint32) * 7919 + 4000000000 % 977
    rounds = np.arange(B, dtype=np.uint32) % 3
    tg = (torch.rand(B, generator=g) * 10).numpy().astype(np.float32)
    H, stop, tok, st, ref_tok, gap = _draft_step_case(am, oracle, z, T_G=tg, active=active, seq_id=seq,
                                                      rounds=rounds, step=5, k_max=20, seed=0xABCDEF0123)
    assert np.array_equal(tok, ref_tok), (tok, ref_tok, gap)
    assert tok[4] == -1 and H[4] == 0 and stop[4] == 0
    assert tok[3] >= V // 2
    assert (st & ~16 == 0).all()
    Href, sref = oracle.draft_entropy(z, T_G=tg, active=active, step=5, k_max=20)
    assert G.close(H, Href).all()


@pytest.mark.parametrize("B,V", [(2000, 20011), (3000, 4099)], ids=["fewer-slices", "dense-counters"])
def test_draft_step_many_rows(am, wl, oracle, B, V):
    """Many rows: the slices per row are halved until the grid fits, and the arrival counters of the rows
    no longer get a cache line each."""
    g = torch.Generator().manual_seed(B)
    z = (torch.randn(B, V, generator=g) * 2).to(torch.bfloat16)
    H, stop, tok, st, ref_tok, gap = _draft_step_case(am, oracle, z, step=1, k_max=9, seed=5, round0=2)
    assert np.array_equal(tok, ref_tok), np.flatnonzero(tok != ref_tok)
    Href, _ = oracle.draft_entropy(z, step=1, k_max=9)
    assert G.close(H, Href).all()


def test_draft_step_unaligned_rows_and_broken_rows(am, wl, oracle):
    g = torch.Generator().manual_seed(3)
    B, V = 6, 4099                                       # odd row length: most rows are not 16-byte aligned
    z = (torch.randn(B, V, generator=g) * 2).to(torch.bfloat16)
    z[1, 7] = float("nan")
    z[2] = float("-inf")
    z[3, 9] = float("inf")
    z[4] = float("-inf"); z[4, 4000] = 1.0               # one-hot
    H, stop, tok, st, ref_tok, gap = _draft_step_case(am, oracle, z, step=0, k_max=4, seed=9)
    assert np.array_equal(tok, ref_tok)
    assert list(tok[1:5]) == [-1, -1, -1, 4000]
    assert all(st[b] & am.binding.ST_NONFINITE for b in (1, 2, 3)) and st[0] & ~16 == 0
    assert all(stop[b] == 1 for b in (1, 2, 3)) and H[4] == 0.0


@pytest.mark.parametrize("dtype,V", [(torch.bfloat16, 128256), (torch.float32, 4104), (torch.bfloat16, 4107)],
                         ids=["bf16-headline", "f32-small", "bf16-unaligned"])
def test_draft_step_near_ties_are_settled_in_float64(am, wl, oracle, dtype, V):
    g = torch.Generator().manual_seed(V + 5)
    z = (torch.randn(1, V, generator=g) * 2.5).to(dtype)
    n = 200000 if V < 10000 else 6000
    ref_tok, gap = oracle.draft_sample(z, step=2, seed=77, round0=3, shared_row=n)
    close_call = np.flatnonzero(gap < (1e-4 if V < 10000 else 1e-3))[:24]
    assert len(close_call) >= 2, "no near tie among the draws: widen the search"
    B = len(close_call)
    rows = z.repeat(B, 1).contiguous()
    H, stop, tok, st, ref_b, gap_b = _draft_step_case(am, oracle, rows, seq_id=close_call.astype(np.uint32),
                                                      step=2, seed=77, round0=3)
    assert np.array_equal(ref_b, ref_tok[close_call])
    assert np.array_equal(tok, ref_b), (tok, ref_b, gap_b)
    print(f"[draft near ties] V={V}: {B} draws, {(st & 16 != 0).sum()} settled in float64, gaps {np.sort(gap_b)[:4]}", flush=True)
    assert V > 10000 or (st & 16 != 0).sum() >= 1        # the closest draws of the short search at the large V may still be decidable in float


def test_draft_step_argument_errors(am):
    ws = am.Workspace(2, 1, 64, torch.float32)
    z = torch.zeros(2, 64, device="cuda")
    with pytest.raises(am.AdasdError) as e:
        am.draft_step(z, ws, step=70000)
    assert e.value.code == -1
    small = am.Workspace(1, 1, 64, torch.float32)
    with pytest.raises(am.AdasdError) as e:
        am.draft_step(torch.zeros(4, 64, device="cuda"), small)
    assert e.value.code == -4
    am.draft_step(torch.zeros(0, 64, device="cuda"), ws)          # B = 0 is a no-op


# ------------------------------------------------------------------------------- update + closed loop
@pytest.mark.parametrize("B,K,cap", [(9, 6, 12), (7, 64, 100)])   # 64: the largest window, every lane a position
def test_update_matches_oracle_and_state_round_trip(am, wl, oracle, B, K, cap):
    from oracle import new_state
    rng = np.random.default_rng(31)
    host = new_state(B, cap)
    dev = am.State(B, cap)
    for rnd in range(8):
        dl = rng.integers(0, K + 1, B).astype(np.int32)
        na = np.minimum(rng.integers(0, K + 1, B), dl).astype(np.int32)
        if rnd == 0:
            dl[0], na[0] = K, K                 # whole window accepted
        Hq = rng.uniform(0.1, 6.0, (B, K)).astype(np.float32)
        dj = rng.uniform(0.0, 1.0, (B, K)).astype(np.float32)
        dj[0, 0], dj[1, 1], dj[2, 2] = 0.0, 1.0, 5e-7
        dj[3, 0], dj[4, 0], dj[5, 0] = 1.0 - 1e-6, 1e-6, 0.99999905   # the floats next to the ends of the open interval
        if rnd == 3:
            Hq[4, :] = np.nan
            dj[5, :] = np.nan
        status = torch.zeros(B, dtype=torch.int32, device="cuda")
        am.update_thresholds(dev, K, torch.tensor(na).cuda(), torch.tensor(Hq).cuda(),
                             torch.tensor(dj).cuda(), draft_len=torch.tensor(dl).cuda(), status=status)
        st_ref = oracle.update(host, na, dl, Hq.astype(np.float64), dj.astype(np.float64), K, d_eps=1e-6)
        got = dev.to_host()
        for k in ("nA", "nR", "ent_cnt"):
            assert np.array_equal(got[k], host[k]), k
        for b in range(B):
            assert np.array_equal(got["LA"][b, :host["nA"][b]], host["LA"][b, :host["nA"][b]])
            assert np.array_equal(got["LR"][b, :host["nR"][b]], host["LR"][b, :host["nR"][b]])
        assert np.allclose(got["T_G"], host["T_G"], rtol=1e-6)
        assert np.allclose(got["ent_sum"], host["ent_sum"], rtol=1e-12)
        assert np.array_equal(status.cpu().numpy(), st_ref.astype(np.int32))
    assert (host["nA"] == cap).any()          # overflow was exercised


def test_running_sums_of_long_lists_follow_every_update(am, wl, oracle):
    """adasd_state.mom: from 4096 samples on, the sums of a list are kept by the update step (added up from
    scratch in the call that crosses the mark) and equal the sums recomputed from the list; a state without
    running sums (the decision stage adds the lists up itself) gives the same decisions."""
    B, K, V, cap = 6, 7, 4096, 4130
    g = torch.Generator().manual_seed(8)
    host = wl.threshold_state(B, cap, g, n_hist=4080)            # sixteen samples short of the mark
    host["nA"][1] = 4096; host["nR"][1] = 4096                   # already there (refresh makes the sums)
    host["nA"][2] = 100; host["nR"][2] = 4095                    # a short accepted list stays without sums
    host["nA"][3] = cap - 3                                      # overflows: dropped appends are not summed
    host["LA"][:, 4080:] = host["LA"][:, :cap - 4080]
    host["LR"][:, 4080:] = host["LR"][:, :cap - 4080]
    st = am.State(B, cap).load(host)
    plain = am.State(B, cap, running_sums=False).load(host)
    ws = am.Workspace(B, K, V, torch.bfloat16)
    src = wl.ClosedLoopSource(B, V, K, dtype=torch.bfloat16, seed=5)
    crossed = set()
    for rnd in range(9):
        t, d, x = src.next_round()
        outs = []
        for state in (st, plain):
            outs.append(am.verify(t.cuda(), d.cuda(), x.cuda(), ws, state=state, seed=3, round0=rnd,
                                  options=am.Options(apply_update=1 if rnd % 2 else 0)))
            if rnd % 2 == 0:
                am.update_thresholds(state, K, outs[-1].n_accept, outs[-1].H_q, outs[-1].d_js)
        torch.cuda.synchronize()
        for name in ("n_accept", "next_token", "accept_mask"):
            assert torch.equal(getattr(outs[0], name), getattr(outs[1], name)), (rnd, name)
        assert torch.allclose(outs[0].p_accept, outs[1].p_accept, rtol=0, atol=1e-6)
        h = st.to_host()
        mom = st.mom.cpu().numpy()
        for b in range(B):
            for which, (L, n) in enumerate((("LA", "nA"), ("LR", "nR"))):
                cnt = int(h[n][b])
                if cnt < 4096:
                    continue
                crossed.add((b, which))
                v = h[L][b, :cnt].astype(np.float64)
                want = [(v - v[0]).sum(), ((v - v[0]) ** 2).sum()]
                assert np.allclose(mom[b, 2 * which:2 * which + 2], want, rtol=1e-12, atol=1e-15), (rnd, b, which)
    assert len(crossed) >= 6 and (2, 0) not in crossed and h["nA"][3] == cap


def test_verify_with_fused_update_matches_verify_then_update(am, wl, oracle):
    """options.apply_update: the decision kernel applies the round to the state; outputs and state must
    equal those of adasd_verify followed by adasd_update_thresholds, and the oracle's."""
    batch = wl.config_batched(B=6, k=7, V=8192, seed=77, cap=70)      # lists 64 long: some overflow at 70
    batch.draft_len = torch.tensor([7, 0, 3, 7, 5, 1], dtype=torch.int32)
    a, st_a, _ = G.run_gpu(am, batch)
    am.update_thresholds(st_a, batch.k, a.n_accept, a.H_q, a.d_js, draft_len=batch.draft_len.cuda(), status=a.status)
    b, st_b, _ = G.run_gpu(am, batch, options=am.Options(apply_update=1))
    torch.cuda.synchronize()
    for name in ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept", "accept_mask", "status"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    ha, hb = st_a.to_host(), st_b.to_host()
    for k in ha:
        assert np.array_equal(ha[k], hb[k]), k
    ref = G.run_oracle(oracle, batch)
    G.compare_verify(b, ref, info_bits=16 | 8)         # overflow bits come from the update step
    host = {k: np.array(v, copy=True) for k, v in batch.state.items()}
    oracle.update(host, ref["n_accept"], batch.draft_len.numpy(), ref["H_q"], ref["d_js"], batch.k, d_eps=1e-6)
    for k in ("nA", "nR", "ent_cnt"):
        assert np.array_equal(hb[k], host[k]), k


@pytest.mark.parametrize("mode", ["default", "literal", "gen_only", "verify_only", "drawn_tokens"])
def test_closed_loop_rounds_against_oracle(am, wl, oracle, mode):
    """Draft-entropy stop rule -> verify -> update for several rounds; the oracle runs its own
    trajectory and the GPU is fed the oracle's state each round (never the other way round).
    literal: the verification loop as Algorithm 1 writes it, from the empty lists on.
    gen_only / verify_only: the two ablations of Section 5.3 (adaptive window with plain speculative
    sampling; fixed window of 5 with the adaptive acceptance test).
    drawn_tokens: the drafted tokens come from adasd_draft_step (x_i ~ q_i) instead of the input source."""
    options = {"literal": am.Options(base_test=1, list_update=1),
               "gen_only": am.Options(relaxed_off=1)}.get(mode, am.Options())
    fixed_window = 5 if mode == "verify_only" else 0
    from oracle import new_state
    B, V, W, cap, n_rounds = 4, 32000, 6, 256, 12
    src = wl.ClosedLoopSource(B, V, W, dtype=torch.bfloat16, seed=77)
    host = new_state(B, cap)
    ws = am.Workspace(B, W, V, torch.bfloat16)
    dev = am.State(B, cap)
    total_flips = 0
    lens = []
    for rnd in range(n_rounds):
        t, d, x = src.next_round()
        dev.load(host)
        # generation: one draft-entropy call per drafted token until every sequence has stopped
        active = torch.ones(B, dtype=torch.uint8, device="cuda")
        dl_gpu = torch.zeros(B, dtype=torch.int32, device="cuda")
        act_ref = np.ones(B, dtype=np.uint8)
        dl_ref = np.zeros(B, dtype=np.int32)
        dg = d.cuda()
        tg_gpu, tg_ref, k_cap = (None, None, fixed_window) if fixed_window else (dev.T_G, host["T_G"], W)
        for step in range(W):
            if mode == "drawn_tokens":
                H, stop, x_gpu, _ = am.draft_step(dg[:, step], ws, T_G=tg_gpu, active=active, step=step, k_max=k_cap,
                                                  seed=src.seed, round0=rnd)
                x_ref, _ = oracle.draft_sample(d[:, step].contiguous(), active=act_ref, step=step, seed=src.seed,
                                               round0=rnd)
                assert np.array_equal(x_gpu.cpu().numpy(), x_ref)
                x[:, step] = torch.tensor(np.maximum(x_ref, 0))        # (inactive rows keep a valid placeholder)
            else:
                H, stop = am.draft_entropy(dg[:, step], ws, T_G=tg_gpu, active=active, step=step, k_max=k_cap)
            dl_gpu += active.to(torch.int32)
            active = active & (1 - stop)
            Href, sref = oracle.draft_entropy(d[:, step].contiguous(), T_G=tg_ref, active=act_ref,
                                              step=step, k_max=k_cap)
            dl_ref += act_ref
            # compare flags unless the entropy sits on the threshold
            live = act_ref.astype(bool)
            near = (np.abs(Href - host["T_G"]) < 1e-5 * np.abs(Href) + 1e-6) if not fixed_window else np.zeros(B, bool)
            assert G.close(H.cpu().numpy()[live], Href[live]).all()
            assert np.array_equal(stop.cpu().numpy()[live & ~near], sref[live & ~near])
            act_ref = act_ref & (1 - sref)
            active = torch.tensor(act_ref, device="cuda")     # follow the oracle's trajectory
            if not act_ref.any():
                break
        dl_gpu = torch.tensor(dl_ref, device="cuda")
        lens.append(dl_ref.copy())
        batch = wl.VerifyBatch(t, d, x, torch.tensor(dl_ref), host, src.seed, rnd)
        out = am.verify(t.cuda(), dg, x.cuda(), ws, state=dev, draft_len=dl_gpu, seed=src.seed, round0=rnd,
                        options=options)
        torch.cuda.synchronize()
        ref = G.run_oracle(oracle, batch, options=options)
        rep = G.compare_verify(out, ref)
        total_flips += rep["flips"]
        if mode == "gen_only":
            assert (out.p_accept == 0).all() and ((out.accept_mask & 2) == 0).all()
        am.update_thresholds(dev, W, out.n_accept, out.H_q, out.d_js, draft_len=dl_gpu)
        got_before = dev.to_host()
        oracle.update(host, ref["n_accept"], dl_ref, ref["H_q"], ref["d_js"], W)
        if rep["flips"] == 0 and rep["member_flips"] == 0:
            assert np.array_equal(got_before["nA"], host["nA"]) and np.array_equal(got_before["nR"], host["nR"])
            assert np.allclose(got_before["T_G"], host["T_G"], rtol=1e-5)
            for b in range(B):
                assert np.allclose(got_before["LA"][b, :host["nA"][b]], host["LA"][b, :host["nA"][b]],
                                   rtol=1e-5, atol=1e-6)
    lens = np.array(lens)
    print(f"[closed loop] mean window {lens.mean():.2f}, flips {total_flips}, T_G {host['T_G']}", flush=True)
    if fixed_window:
        assert (lens == fixed_window).all()
    else:
        assert lens[0].max() == 1            # initial threshold 0: the first window has length 1
        assert lens.max() > 1                # the threshold has adapted upwards since


@pytest.mark.parametrize("n_hist,cap", [(64, 300), (4060, 4400)], ids=["short_lists", "lists_crossing_the_running_sum_mark"])
def test_snapshot_then_resume_twice_gives_identical_state(am, wl, n_hist, cap):
    """Checkpoint and resume of a decoding run: the state copied to the host after five rounds and loaded
    into a fresh device state twice must give, both times, bit for bit the same outputs and the same final
    state, and the same decisions, tokens and lists as the run that was never interrupted (whose running
    sums of long lists were carried from round to round rather than added up again at the load)."""
    B, K, V, n_rounds, cut = 6, 6, 8192, 10, 5
    g = torch.Generator().manual_seed(21)
    host0 = wl.threshold_state(B, cap, g, n_hist=n_hist)
    src = wl.ClosedLoopSource(B, V, K, dtype=torch.bfloat16, seed=33)
    rounds = [tuple(x.cuda() for x in src.next_round()) for _ in range(n_rounds)]
    ws = am.Workspace(B, K, V, torch.bfloat16)
    names = ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept", "accept_mask", "status")

    def bits(v):
        return v.view(torch.int32) if v.dtype == torch.float32 else v

    def run(state, first, last):
        outs = []
        for r in range(first, last):
            t, d, x = rounds[r]
            o = am.verify(t, d, x, ws, state=state, seed=5, round0=r, options=am.Options(apply_update=1))
            torch.cuda.synchronize()
            outs.append({k: getattr(o, k).clone() for k in names})
        return outs

    whole = am.State(B, cap).load(host0)
    run(whole, 0, cut)
    snapshot = {k: np.array(v, copy=True) for k, v in whole.to_host().items()}
    rest = run(whole, cut, n_rounds)
    final = whole.to_host()
    resumed = []
    for _ in range(2):
        st = am.State(B, cap).load(snapshot)
        outs = run(st, cut, n_rounds)
        resumed.append((outs, st.to_host(), st.mom.cpu().numpy()))
    (o1, f1, m1), (o2, f2, m2) = resumed
    for a, b in zip(o1, o2):
        for k in names:
            assert torch.equal(bits(a[k]), bits(b[k])), k
    for k in f1:
        assert np.array_equal(f1[k], f2[k]), k
    assert np.array_equal(m1, m2)
    # against the uninterrupted run: integers, tokens and the state's lists bit for bit; the posterior to the
    # rounding of the two ways of forming the lists' sums
    for a, b in zip(rest, o1):
        for k in ("n_accept", "next_token", "accept_mask", "status", "H_p", "H_q", "d_js"):
            assert torch.equal(a[k], b[k]), k
        assert torch.allclose(a["p_accept"], b["p_accept"], rtol=0, atol=1e-6)
    for k in final:
        assert np.array_equal(final[k], f1[k]), k
    assert (f1["nA"] + f1["nR"] > snapshot["nA"] + snapshot["nR"]).all()      # the lists did grow after the cut
    if n_hist >= 4000:
        assert (f1["nA"] >= 4096).any() and (snapshot["nA"] < 4096).all()


def test_verify_and_draft_step_replay_from_a_hip_graph(am, wl):
    """The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
    memset), so a round can be captured once and replayed.  Every replay, with eager work and
    synchronisations in between, must reproduce the eager results for the same round counter."""
    batch = wl.config_batched(B=6, k=5, V=32000, seed=55, cap=640)
    B, K, V = batch.B, batch.k, batch.V
    t, d, x = batch.target.cuda(), batch.draft.cuda(), batch.draft_tokens.cuda()
    ws = am.Workspace(B, K, V, torch.bfloat16)
    st = am.State(B, 640).load(batch.state)
    rounds = torch.zeros(B, dtype=torch.int32, device="cuda")
    out = am.binding.alloc_verify_result(B, K)
    H = torch.empty(B, dtype=torch.float32, device="cuda")
    stop = torch.empty(B, dtype=torch.uint8, device="cuda")
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    dst = torch.empty(B, dtype=torch.int32, device="cuda")
    one = torch.ones(B, dtype=torch.int32, device="cuda")
    opts = am.Options(apply_update=1)

    def round_():
        am.draft_step(d[:, 0], ws, T_G=st.T_G, step=0, k_max=K, seed=9, rounds=rounds, H_out=H, stop_out=stop,
                      token_out=tok, status_out=dst)
        am.verify(t, d, x, ws, state=st, seed=batch.seed, rounds=rounds, options=opts, out=out)
        rounds.add_(one)

    def snapshot():
        torch.cuda.synchronize()
        r = {k: getattr(out, k).clone() for k in ("n_accept", "next_token", "H_q", "d_js", "p_accept", "status")}
        r.update(H=H.clone(), stop=stop.clone(), tok=tok.clone(), state={k: torch.as_tensor(v).clone() for k, v in st.to_host().items()})
        return r

    eager = []
    for _ in range(4):                                  # rounds 0..3 eagerly, from the initial state
        round_()
        eager.append(snapshot())
    st.load(batch.state)
    rounds.zero_()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up on the capture stream, then rewind
        round_()
    torch.cuda.current_stream().wait_stream(side)
    st.load(batch.state)
    rounds.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        round_()
    st.load(batch.state)                                # capture does not run anything, but be explicit
    rounds.zero_()
    for i in range(4):
        graph.replay()
        got = snapshot()
        junk = torch.randn(1 << 16, device="cuda").sum().item()      # eager work between replays
        assert junk == junk
        for k, v in eager[i].items():
            if k == "state":
                for name, ref in v.items():
                    assert torch.equal(torch.nan_to_num(got["state"][name].double()), torch.nan_to_num(ref.double())), (i, name)
            else:
                assert torch.equal(torch.nan_to_num(got[k].double(), nan=-7.0), torch.nan_to_num(v.double(), nan=-7.0)), (i, k)


@pytest.mark.parametrize("n_bytes", [16, 32768, 32768 + 16, 5 * 32768 - 4096, 131334144 // 8])
def test_stream_read_touches_every_byte_once(am, n_bytes):
    """The diagnostic read leaves the xor of every 32-bit word of each 32 KiB piece: integer work, exact."""
    g = torch.Generator().manual_seed(n_bytes)
    host = torch.randint(-2**31, 2**31 - 1, (n_bytes // 4,), dtype=torch.int32, generator=g)
    pieces = (n_bytes + 32767) // 32768
    sink = torch.full((pieces + 2,), 0x5a5a5a5a, dtype=torch.int32, device="cuda")
    am.stream_read(host.cuda(), sink)
    torch.cuda.synchronize()
    got = sink.cpu().numpy()
    words = host.numpy()
    want = [int(np.bitwise_xor.reduce(words[p * 8192:(p + 1) * 8192])) for p in range(pieces)]
    assert got[:pieces].tolist() == want
    assert (got[pieces:] == 0x5a5a5a5a).all()           # nothing written past the last piece
    with pytest.raises(am.AdasdError):
        am.stream_read(host.cuda(), sink[:pieces - 1] if pieces > 1 else sink[:0])


def test_bounded_wait_expiry_gives_identical_results(am, wl):
    """With options.wait_polls < 0 every workgroup of the single-read kernel stops waiting at once and
    recomputes the other slices' results itself; the outputs must not change by a single bit."""
    batch = wl.config_batched(B=4, k=4, V=128256, seed=321)
    a, _, ws = G.run_gpu(am, batch, stats_path=2)
    snap = {k: getattr(a, k).clone() for k in ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept")}
    b, _, _ = G.run_gpu(am, batch, ws=ws, options=am.Options(wait_polls=-1), stats_path=2)
    for k, v in snap.items():
        assert torch.equal(getattr(b, k), v, ), k
    c, _, _ = G.run_gpu(am, batch, ws=ws, stats_path=2)   # and the workspace is clean afterwards
    for k, v in snap.items():
        assert torch.equal(getattr(c, k), v), k


def test_results_are_bitwise_reproducible(am, wl, path):
    batch = wl.config_batched(B=4, k=4, V=50000, seed=123)
    a, _, ws = G.run_gpu(am, batch, stats_path=path)
    snap = {k: getattr(a, k).clone() for k in ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept")}
    for _ in range(3):
        b, _, _ = G.run_gpu(am, batch, ws=ws, stats_path=path)
        for k, v in snap.items():
            assert torch.equal(getattr(b, k), v), k
