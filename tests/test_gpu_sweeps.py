"""Seeded sweeps of the HIP library against the CPU oracle (run with -m gpu): update step, drafting calls,
history-list shapes, strided views.  Every case draws shapes, options and data from its seed; whatever comes
up has to meet the bar of the parity tests.  (Longer runs of the same generators found: the filter of the
lists at the float just below its upper end; nothing else in these areas.)"""
import numpy as np
import pytest
import torch

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def am():
    import paper_2512_11280_amd as am
    am.load_library()
    assert torch.cuda.is_available()
    return am


@pytest.fixture(scope="module")
def wl():
    from paper_2512_11280_amd import workloads
    return workloads


# ------------------------------------------------------------------------------------------ update step
@pytest.mark.parametrize("case", range(16))
def test_update_step_sweep(am, oracle, case):
    """Lists next to their capacity and next to the length from which running sums are kept, window lengths
    and accepted counts out of range, distances on and next to the ends of the open interval, non-finite
    values: lists bit for bit, counts, status and running sums after each of four rounds."""
    from oracle import new_state
    rng = np.random.default_rng(63000 + case)
    B = int(rng.integers(1, 40)); K = int(rng.choice([1, 2, 5, 8, 16, 33, 64]))
    cap = int(rng.choice([1, 3, 16, 100, 4090, 4100, 4200]))
    host = new_state(B, cap)
    for b in range(B):
        nA = int(min(cap, rng.choice([0, 1, cap - 1, cap, max(cap - K, 0), 4090, 4095, 4096])))
        nR = int(min(cap, rng.choice([0, 2, cap - 1, cap, 4094, 4095, 4096])))
        host["LA"][b, :nA] = rng.uniform(0.01, 0.99, nA)
        host["LR"][b, :nR] = rng.uniform(0.01, 0.99, nR)
        host["nA"][b], host["nR"][b] = nA, nR
    dev = am.State(B, cap).load(host)
    for rnd in range(4):
        use_len = rng.random() < 0.7
        dl = rng.integers(-1, K + 3, B).astype(np.int32) if use_len else None
        dlc = np.clip(dl, 0, K) if use_len else np.full(B, K, np.int32)
        na = rng.integers(-1, K + 2, B).astype(np.int32)
        Hq = rng.uniform(0.0, 12.0, (B, K)).astype(np.float32)
        dj = rng.choice([0.0, 1.0, 5e-7, 1e-6, 1.0000001e-6, 1 - 1e-6, 0.99999905, 0.3, 0.5, 0.77], (B, K)).astype(np.float32)
        mask = rng.random((B, K)) < 0.5
        dj[mask] = rng.uniform(0, 1, mask.sum()).astype(np.float32)
        if rng.random() < 0.3:
            Hq[rng.integers(0, B), :] = rng.choice([np.nan, np.inf, -np.inf])
        if rng.random() < 0.3:
            dj[rng.integers(0, B), :] = rng.choice([np.nan, np.inf, -1.0, 2.0])
        status = torch.zeros(B, dtype=torch.int32, device="cuda")
        am.update_thresholds(dev, K, torch.tensor(na).cuda(), torch.tensor(Hq).cuda(), torch.tensor(dj).cuda(),
                             draft_len=None if dl is None else torch.tensor(dl).cuda(), status=status)
        st_ref = oracle.update(host, np.clip(na, 0, dlc), dlc if use_len else None, Hq.astype(np.float64),
                               dj.astype(np.float64), K, d_eps=float(np.float32(1e-6)))
        got = dev.to_host()
        for k in ("nA", "nR", "ent_cnt"):
            assert np.array_equal(got[k], host[k]), (k, rnd)
        for b in range(B):
            assert np.array_equal(got["LA"][b, :host["nA"][b]], host["LA"][b, :host["nA"][b]]), ("LA", b, rnd)
            assert np.array_equal(got["LR"][b, :host["nR"][b]], host["LR"][b, :host["nR"][b]]), ("LR", b, rnd)
        assert np.allclose(got["T_G"], host["T_G"], rtol=1e-6)
        assert np.allclose(got["ent_sum"], host["ent_sum"], rtol=1e-12)
        assert np.array_equal(status.cpu().numpy() & ~am.binding.ST_BAD_LENGTH, st_ref.astype(np.int32))
        mom = dev.mom.cpu().numpy()
        for b in range(B):
            for off, (L, n) in enumerate(((host["LA"][b], host["nA"][b]), (host["LR"][b], host["nR"][b]))):
                if n >= 4096:                                    # kept from 4096 samples on
                    e = L[:n].astype(np.float64) - np.float64(L[0])
                    assert np.allclose(mom[b, 2 * off], e.sum(), rtol=1e-9, atol=1e-9), ("sum", b, off, rnd)
                    assert np.allclose(mom[b, 2 * off + 1], (e * e).sum(), rtol=1e-9), ("sum of squares", b, off, rnd)


# ------------------------------------------------------------------------------------------ drafting calls
@pytest.mark.parametrize("case", range(16))
def test_drafting_calls_sweep(am, oracle, case):
    """Rows of very different scale and offset, lifted and masked tokens, active masks, thresholds, sequence
    ids and rounds: the drawn tokens are the oracle's, entropy and stop flag within tolerance, and the
    entropy-only call returns the same bits."""
    rng = np.random.default_rng(87000 + case)
    B = int(rng.integers(1, 80)); V = int(rng.choice([8, 9, 64, 257, 1000, 2048, 4099, 8200, 12344, 40000]))
    dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
    g = torch.Generator().manual_seed(case)
    scale = torch.tensor(rng.choice([0.01, 0.3, 3.0, 12.0, 40.0], B), dtype=torch.float32).reshape(B, 1)
    z = torch.randn(B, V, generator=g) * scale + float(rng.uniform(-90, 90))
    if rng.random() < 0.5:
        z[torch.arange(B), torch.tensor(rng.integers(0, V, B))] += float(rng.uniform(5, 60))
    if rng.random() < 0.3:
        z[int(rng.integers(0, B)), : V // 2] = float("-inf")
    z = z.to(dtype)
    active = (rng.random(B) < 0.7).astype(np.uint8) if rng.random() < 0.6 else None
    tg = rng.uniform(0, 10, B).astype(np.float32)
    seq = rng.integers(0, 2 ** 32, B, dtype=np.uint64).astype(np.uint32)
    rounds = rng.integers(0, 1000, B).astype(np.uint32)
    step = int(rng.integers(0, 20)); k_max = int(rng.integers(step + 1, 40)); seed = int(rng.integers(0, 2 ** 62))
    ws = am.Workspace(B, 1, V, dtype)
    dev = dict(T_G=torch.tensor(tg).cuda(), active=None if active is None else torch.tensor(active).cuda(),
               seq_id=torch.tensor(seq.view(np.int32)).cuda(), rounds=torch.tensor(rounds.view(np.int32)).cuda())
    H, stop, tok, st = am.draft_step(z.cuda(), ws, step=step, k_max=k_max, seed=seed, **dev)
    He, stope = am.draft_entropy(z.cuda(), ws, T_G=dev["T_G"], active=dev["active"], step=step, k_max=k_max)
    torch.cuda.synchronize()
    assert torch.equal(H.view(torch.int32), He.view(torch.int32)) and torch.equal(stop, stope)
    ref_tok, gap = oracle.draft_sample(z, active=active, step=step, seed=seed, seq_id=seq, rounds=rounds)
    assert np.array_equal(tok.cpu().numpy(), ref_tok), (np.flatnonzero(tok.cpu().numpy() != ref_tok), gap)
    Href, sref = oracle.draft_entropy(z, T_G=tg, active=active, step=step, k_max=k_max)
    live = np.ones(B, bool) if active is None else active.astype(bool)
    Hn, sn = H.cpu().numpy(), stop.cpu().numpy()
    assert G.close(Hn[live], Href[live]).all()
    near = np.abs(Href - tg) < 1e-5 * np.abs(Href) + 1e-6
    assert np.array_equal(sn[live & ~near], sref[live & ~near])


# ------------------------------------------------------------------------------------------ history lists
def _fill_list(rng, n, kind):
    if kind == 0:
        x = rng.normal(rng.uniform(0.05, 0.9), rng.choice([1e-4, 1e-3, 0.01, 0.05, 0.2]), n)
    elif kind == 1:
        x = np.full(n, rng.uniform(0.01, 0.99))                                    # no spread: the test is off
    elif kind == 2:
        x = rng.uniform(1e-5, 1 - 1e-5, n)
    elif kind == 3:
        x = rng.choice([0.1, 0.1000001, 0.9], n)                                   # duplicates
    else:
        x = np.concatenate([rng.normal(0.2, 0.01, n // 2), rng.normal(0.8, 0.01, n - n // 2)])
    return np.clip(x, 2e-6, 1 - 2e-6).astype(np.float32)


@pytest.mark.parametrize("case", [c for c in range(25) if c != 20])    # 20: both lists alike, P(A|d) = 1/2 to the last bit
def test_history_list_shapes_sweep(am, wl, oracle, case):
    """Lists from empty to 8000 samples (both forms of the decision kernel, lengths around the switches
    between them), tight clusters, no spread, duplicates, two clusters; all options of the Bayesian test."""
    rng = np.random.default_rng(52000 + case)
    B = int(rng.integers(1, 5)); K = int(rng.choice([1, 4, 9])); V = int(rng.choice([64, 1000, 4104]))
    cap = int(rng.choice([8, 64, 511, 512, 1500, 4200, 9000]))
    batch = wl.config_batched(B=B, k=K, V=V, seed=7000 + case, dtype=torch.bfloat16, cap=64)
    st = wl.empty_state(B, cap)
    for b in range(B):
        nA = int(min(cap, rng.choice([0, 1, 2, 3, 40, 383, 384, 500, 1100, 4095, 4096, 4100, 8000])))
        nR = int(min(cap, rng.choice([0, 1, 2, 3, 40, 383, 384, 500, 1100, 4095, 4096, 4100, 8000])))
        st["LA"][b, :nA] = _fill_list(rng, nA, int(rng.integers(0, 5)))
        st["LR"][b, :nR] = _fill_list(rng, nR, int(rng.integers(0, 5)))
        st["nA"][b], st["nR"][b] = nA, nR
    batch.state = st
    if rng.random() < 0.4:
        batch.draft_len = torch.tensor(rng.integers(0, K + 1, B), dtype=torch.int32)
    opt = dict(list_update=int(rng.integers(0, 2)), reject_rule=int(rng.integers(0, 2)), bw_rule=int(rng.integers(0, 2)),
               apply_update=int(rng.integers(0, 2)), kde_min_n=int(rng.choice([0, 2, 5])), base_test=int(rng.integers(0, 2)))
    options = am.Options(**opt)
    out, dev, _ = G.run_gpu(am, batch, options=options)
    ref = G.run_oracle(oracle, batch, options=options)
    rep = G.compare_verify(out, ref, info_bits=16 | 8)
    if opt["apply_update"] and rep["flips"] == 0 and rep["member_flips"] == 0:
        host = {k: np.array(v, copy=True) for k, v in st.items()}
        dl = None if batch.draft_len is None else batch.draft_len.numpy()
        oracle.update(host, ref["n_accept"], dl, ref["H_q"], ref["d_js"], K, d_eps=1e-6)
        got = dev.to_host()
        assert np.array_equal(got["nA"], host["nA"]) and np.array_equal(got["nR"], host["nR"])


# ------------------------------------------------------------------------------------------ strided views
def _strided(x, pad_pos, pad_seq, off):
    B, P, V = x.shape
    buf = torch.full((off + B * (P * (V + pad_pos) + pad_seq) + 64,), 7.0, dtype=x.dtype, device="cuda")
    v = buf[off:].as_strided((B, P, V), (P * (V + pad_pos) + pad_seq, V + pad_pos, 1))
    v.copy_(x.cuda())
    return v


@pytest.mark.parametrize("case", range(16))
def test_strided_and_misaligned_views_sweep(am, wl, oracle, case):
    """Logits as views into larger buffers: padding between rows and between sequences, a base that is not
    16-byte aligned; verification on both statistics paths and the drafting call on a strided row block."""
    rng = np.random.default_rng(93000 + case)
    B = int(rng.integers(1, 6)); K = int(rng.choice([1, 2, 5, 9]))
    V = int(rng.choice([8, 63, 64, 257, 1000, 2048, 4099, 4104, 8200]))
    dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
    batch = wl.config_batched(B=B, k=K, V=V, seed=8000 + case, dtype=dtype, cap=64)
    if rng.random() < 0.5:
        batch.draft_len = torch.tensor(rng.integers(0, K + 1, B), dtype=torch.int32)
    opt = dict(base_test=int(rng.integers(0, 2)), list_update=int(rng.integers(0, 2)), apply_update=int(rng.integers(0, 2)))
    options = am.Options(stats_path=int(rng.integers(1, 3)), **opt)
    t = _strided(batch.target, int(rng.choice([0, 1, 3, 8, 24])), int(rng.choice([0, 2, 8])), int(rng.choice([0, 1, 5, 8])))
    d = _strided(batch.draft, int(rng.choice([0, 1, 3, 8, 24])), int(rng.choice([0, 2, 8])), int(rng.choice([0, 1, 5, 8])))
    ws = am.Workspace(B, K, V, dtype)
    st = G.state_to_device(am, batch.state, B, batch.state["LA"].shape[1])
    out = am.verify(t, d, batch.draft_tokens.cuda(), ws, state=st, draft_len=G.to_dev(batch.draft_len), seed=batch.seed,
                    round0=batch.round0, options=options)
    torch.cuda.synchronize()
    G.compare_verify(out, G.run_oracle(oracle, batch, options=options), info_bits=16 | 8)
    H, stop, tok, _ = am.draft_step(d[:, 0], ws, step=0, k_max=9, seed=5, round0=case)
    ref_tok, gap = oracle.draft_sample(batch.draft[:, 0].contiguous(), step=0, seed=5, round0=case)
    assert np.array_equal(tok.cpu().numpy(), ref_tok), (tok.cpu().numpy(), ref_tok, gap)
    Href, _ = oracle.draft_entropy(batch.draft[:, 0].contiguous(), step=0, k_max=9)
    assert G.close(H.cpu().numpy(), Href).all()


# ------------------------------------------------------------------------------------------ one workspace, many shapes
def test_one_workspace_serves_calls_of_different_shapes(am, wl, oracle):
    """The regions of a workspace only depend on its size, and every kernel leaves the arrival counters it
    used at zero: verification calls of different shapes, window lengths, history sizes and options and
    drafting calls in between, all on ONE workspace, each against the oracle."""
    rng = np.random.default_rng(4242)
    dtype = torch.bfloat16
    ws = am.Workspace(40, 9, 8200, dtype)
    for call in range(40):
        B = int(rng.integers(1, 41)); K = int(rng.choice([1, 2, 5, 9])); V = int(rng.choice([64, 1000, 4099, 4104, 8200]))
        batch = wl.config_batched(B=B, k=K, V=V, seed=9000 + call, dtype=dtype, cap=64)
        if rng.random() < 0.5:
            g = torch.Generator().manual_seed(call)
            batch.state = wl.threshold_state(B, 700, g, n_hist=int(rng.choice([64, 500])))    # both forms of the decision kernel
        if rng.random() < 0.5:
            batch.draft_len = torch.tensor(rng.integers(0, K + 1, B), dtype=torch.int32)
        options = am.Options(stats_path=int(rng.integers(1, 3)), list_update=int(rng.integers(0, 2)),
                             apply_update=int(rng.integers(0, 2)))
        out, _, _ = G.run_gpu(am, batch, options=options, ws=ws)
        G.compare_verify(out, G.run_oracle(oracle, batch, options=options), info_bits=16 | 8)
        rows = batch.draft[:, 0].contiguous()
        H, stop, tok, _ = am.draft_step(rows.cuda(), ws, step=0, k_max=4, seed=call, round0=call)
        ref_tok, gap = oracle.draft_sample(rows, step=0, seed=call, round0=call)
        assert np.array_equal(tok.cpu().numpy(), ref_tok), (call, tok.cpu().numpy(), ref_tok, gap)
        Href, _ = oracle.draft_entropy(rows, step=0, k_max=4)
        assert G.close(H.cpu().numpy(), Href).all(), call
