"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded inputs and compare element by element, with the tolerances of the build's contract:

  * entropies and JS distance: |gpu - oracle| <= 1e-5 |oracle| + 1e-6
  * accepted lengths and sampled token ids: bit-exact
  * an acceptance bit may differ only where the deciding statistic lies within 1e-5 of its
    threshold (ln u1 vs the log ratio; u2 vs P(A|d)), and a distance may fall on the other side of
    the open-interval filter of the history lists only within 1e-5 of that filter's bounds; every
    such flip is counted and the sequence's downstream integers are then not compared.
"""
from __future__ import annotations

import numpy as np
import torch

RTOL, ATOL = 1e-5, 1e-6
FLIP_BAND = 1e-5
PA_ATOL = 2e-5          # posterior moves by dP/dd * 1e-5*d; slope of the KDE ratio can reach ~1/h


def to_dev(x):
    return None if x is None else x.cuda()


def state_to_device(am, host_state, B, cap):
    st = am.State(B, cap)
    st.load({k: host_state[k] for k in ("T_G", "ent_sum", "ent_cnt", "LA", "LR", "nA", "nR")})
    return st


def run_gpu(am, batch, options=None, seq_id=None, rounds=None, ws=None, stats_path=0):
    B, K, V = batch.B, batch.k, batch.V
    if stats_path:
        import dataclasses
        options = dataclasses.replace(options or am.Options(), stats_path=stats_path)
    ws = ws or am.Workspace(B, max(K, 1), V, batch.target.dtype)
    cap = batch.state["LA"].shape[1]
    st = state_to_device(am, batch.state, B, cap)
    sid = None if seq_id is None else torch.tensor(np.asarray(seq_id, dtype=np.uint32).view(np.int32)).cuda()
    rnd = None if rounds is None else torch.tensor(np.asarray(rounds, dtype=np.uint32).view(np.int32)).cuda()
    out = am.verify(batch.target.cuda(), batch.draft.cuda(), batch.draft_tokens.cuda(), ws, state=st,
                    draft_len=to_dev(batch.draft_len), seed=batch.seed, seq_id=sid, rounds=rnd,
                    round0=batch.round0, options=options)
    torch.cuda.synchronize()
    return out, st, ws


def run_oracle(oracle, batch, options=None, seq_id=None, rounds=None):
    kw = {}
    if options is not None:
        kw = dict(reject_rule=options.reject_rule, kde_min_n=options.kde_min_n,
                  bw_rule=options.bw_rule, relaxed_off=options.relaxed_off,
                  base_test=options.base_test, list_update=options.list_update,
                  d_eps=float(np.float32(options.d_eps)) if options.d_eps > 0 else 1e-6)
    s = batch.state
    ref = oracle.verify(batch.target, batch.draft, batch.draft_tokens.numpy(),
                        draft_len=None if batch.draft_len is None else batch.draft_len.numpy(),
                        LA=s["LA"], LR=s["LR"], nA=s["nA"], nR=s["nR"], seed=batch.seed,
                        seq_id=seq_id, rounds=rounds, round0=batch.round0, **kw)

    def posterior_at(b, i, d, earlier=None):
        """The oracle's posterior of sequence b, position i, at a given distance (for the p_accept
        check).  With appends inside the loop the list is the state's followed by the distances of the
        earlier positions that pass the filter and fit the capacity: the oracle's own, or `earlier`
        (the ones another implementation found, within their tolerance)."""
        la = list(s["LA"][b, :int(s["nA"][b])])
        if kw.get("list_update", 0):
            eps, cap = kw["d_eps"], s["LA"].shape[1]
            for j in range(i):
                dj = float(ref["d_js"][b, j] if earlier is None else earlier[j])   # (a float32 scalar would pull 1 - eps down to float32)
                if eps < dj < 1.0 - eps and len(la) < cap:
                    la.append(np.float32(dj))
        return oracle.posterior(float(d), np.float32(la), s["LR"][b, :int(s["nR"][b])],
                                min_n=kw.get("kde_min_n", 2), bw_rule=kw.get("bw_rule", 0))
    ref["posterior_at"] = posterior_at
    ref["d_eps"] = kw.get("d_eps", 1e-6)
    return ref


def close(gpu, ref, rtol=RTOL, atol=ATOL):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    both_nan = np.isnan(gpu) & np.isnan(ref)
    ok = np.abs(gpu - ref) <= rtol * np.abs(ref) + atol
    return ok | both_nan


def compare_verify(gpu, ref, info_bits=16):
    """Returns a report dict; raises AssertionError on any disagreement outside the contract."""
    g = {k: getattr(gpu, k).cpu().numpy() for k in
         ("n_accept", "next_token", "H_p", "H_q", "d_js", "p_accept", "accept_mask", "status")}
    rep = dict(flips=0, exact_path=int(((g["status"] & info_bits) != 0).sum()), seq_skipped=0)
    for name in ("H_p", "H_q", "d_js"):
        ok = close(g[name], ref[name])
        if not ok.all():
            bad = np.argwhere(~ok)[0]
            raise AssertionError(f"{name} mismatch at {tuple(bad)}: gpu {g[name][tuple(bad)]!r} "
                                 f"oracle {ref[name][tuple(bad)]!r}")
    # A distance that passes the comparison above can still sit on the other side of the open-interval
    # filter (d_eps, 1 - d_eps) of the history lists than the oracle's, if the oracle's is within FLIP_BAND
    # of one of the filter's bounds: a membership flip, counted like an acceptance flip.
    d_eps = ref.get("d_eps", 1e-6)
    dg, dr = g["d_js"].astype(np.float64), np.asarray(ref["d_js"], dtype=np.float64)
    with np.errstate(invalid="ignore"):
        member_flip = ((dg > d_eps) & (dg < 1 - d_eps)) != ((dr > d_eps) & (dr < 1 - d_eps))
        near_bound = (np.abs(dr - d_eps) <= FLIP_BAND) | (np.abs(dr - (1 - d_eps)) <= FLIP_BAND)
    assert not (member_flip & ~near_bound).any(), \
        f"list membership differs outside the 1e-5 band: gpu {dg[member_flip & ~near_bound]} oracle {dr[member_flip & ~near_bound]}"
    # The posterior is a steep function of the distance where the kernel bandwidth is small, so an
    # admissible error of the distance can move it by more than PA_ATOL.  Where the direct comparison
    # fails, the posterior must still agree with the oracle's evaluated at the distance the GPU found.
    # With appends inside the loop an earlier position's distance is part of the list: after a membership
    # flip the sequence's later posteriors belong to another list and must agree with the oracle's posterior
    # on THAT list; the rest of such a sequence is not compared.
    member_seq = np.zeros(g["n_accept"].shape[0], dtype=bool)
    okp = close(g["p_accept"], ref["p_accept"], rtol=0.0, atol=PA_ATOL)
    for b, i in np.argwhere(~okp):
        if member_seq[b]:
            continue
        at_gpu_d = ref["posterior_at"](b, i, g["d_js"][b, i])
        if abs(g["p_accept"][b, i] - at_gpu_d) <= PA_ATOL:
            continue
        # With appends inside the loop the earlier distances of the round are samples of the list, and far
        # from the stored samples the nearest of them carries the whole kernel sum: the posterior is then as
        # steep in an EARLIER distance as in its own.  The posterior must agree with the oracle's on the list
        # built from the distances the GPU found (each of them within its own tolerance, checked above).
        with_own = ref["posterior_at"](b, i, g["d_js"][b, i], earlier=g["d_js"][b, :i])
        if abs(g["p_accept"][b, i] - with_own) <= PA_ATOL:
            if member_flip[b, :i].any():
                member_seq[b] = True
            continue
        raise AssertionError(
            f"p_accept mismatch at {(b, i)}: gpu {g['p_accept'][b, i]!r}, oracle at the same distance "
            f"{at_gpu_d!r}, on the list with the GPU's earlier distances {with_own!r}, oracle at its own distance "
            f"{ref['p_accept'][b, i]!r}")
    member_seq |= member_flip.any(axis=1)
    rep["member_flips"] = int(np.nansum(member_flip))
    rep["max_rel_H"] = float(np.nanmax(np.abs(g["H_q"] - ref["H_q"]) / np.maximum(np.abs(ref["H_q"]), 1e-30),
                                       initial=0.0))
    rep["max_rel_d"] = float(np.nanmax(np.abs(g["d_js"] - ref["d_js"]) / np.maximum(np.abs(ref["d_js"]), 1e-30),
                                       initial=0.0))

    B = g["n_accept"].shape[0]
    gm, rm = g["accept_mask"], ref["accept_mask"]
    flipped_seq = member_seq.copy()
    for bit, margin in ((1, ref["base_margin"]), (2, ref["relaxed_margin"])):
        diff = ((gm & bit) != (rm & bit)) & ~member_seq[:, None]
        if diff.any():
            assert (np.abs(margin[diff]) <= FLIP_BAND).all(), \
                f"acceptance bit {bit} differs outside the 1e-5 band: margins {margin[diff]}"
            rep["flips"] += int(diff.sum())
            flipped_seq |= diff.any(axis=1)
    rep["seq_skipped"] = int(flipped_seq.sum())
    keep = ~flipped_seq
    assert np.array_equal(g["n_accept"][keep], ref["n_accept"][keep]), \
        (g["n_accept"][keep], ref["n_accept"][keep])
    if not np.array_equal(g["next_token"][keep], ref["next_token"][keep]):
        bad = np.flatnonzero(g["next_token"][keep] != ref["next_token"][keep])
        raise AssertionError(f"next_token differs for sequences {bad}: gpu {g['next_token'][keep][bad]} "
                             f"oracle {ref['next_token'][keep][bad]} top2 gaps {ref['top2_gap'][keep][bad]}")
    assert np.array_equal(g["status"][keep] & ~info_bits, ref["status"][keep].astype(np.int64)), \
        (g["status"][keep], ref["status"][keep])
    return rep
