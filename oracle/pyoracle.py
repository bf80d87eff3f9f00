"""ctypes loader for the float64 C oracle (test infrastructure, not product code).

The arithmetic lives in ``adasd_oracle.c``; this file only compiles it with gcc,
marshals numpy arrays and returns plain dicts.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adasd_oracle.c")
_LIB = os.path.join(_HERE, "libadasd_oracle.so")

F32, BF16 = 0, 1
ST_BAD_TOKEN, ST_NONFINITE, ST_ZERO_MASS, ST_OVERFLOW = 1, 2, 4, 8


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with plain gcc -O2 (no fast-math, no intrinsics).

    With ADASD_ORACLE_SANITIZE set to a -fsanitize= list ("undefined" or "address,undefined") a second,
    instrumented library is built at -O1 instead and returned: the sanitizer leg of the CPU tests loads
    the oracle through it (AddressSanitizer needs its runtime preloaded into the interpreter)."""
    san = os.environ.get("ADASD_ORACLE_SANITIZE", "")
    lib = _LIB if not san else os.path.join(_HERE, "libadasd_oracle_san_" + san.replace(",", "_") + ".so")
    stale = (not os.path.exists(lib)) or os.path.getmtime(lib) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "adasd_oracle.h")))
    if force or stale:
        opt = ["-O2"] if not san else ["-O1", "-g", "-fsanitize=" + san, "-fno-sanitize-recover=all"]
        cmd = ["gcc"] + opt + ["-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared", "-fopenmp",
                               "-o", lib, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return lib


class _VerifyArgs(C.Structure):
    _fields_ = [
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p),
        ("dtype", C.c_int32), ("B", C.c_int32), ("k_max", C.c_int32), ("V", C.c_int32),
        ("t_seq_stride", C.c_int64), ("t_pos_stride", C.c_int64),
        ("d_seq_stride", C.c_int64), ("d_pos_stride", C.c_int64),
        ("draft_tokens", C.c_void_p), ("draft_len", C.c_void_p),
        ("cap", C.c_int32),
        ("LA", C.c_void_p), ("LR", C.c_void_p), ("nA", C.c_void_p), ("nR", C.c_void_p),
        ("seed", C.c_uint64), ("seq_id", C.c_void_p), ("round", C.c_void_p),
        ("round0", C.c_uint32),
        ("reject_rule", C.c_int32), ("kde_min_n", C.c_int32), ("bw_rule", C.c_int32),
        ("relaxed_off", C.c_int32), ("base_test", C.c_int32), ("list_update", C.c_int32),
        ("d_eps", C.c_double),
        ("n_accept", C.c_void_p), ("next_token", C.c_void_p),
        ("H_p", C.c_void_p), ("H_q", C.c_void_p), ("d_js", C.c_void_p),
        ("p_accept", C.c_void_p), ("accept_mask", C.c_void_p), ("status", C.c_void_p),
        ("base_margin", C.c_void_p), ("relaxed_margin", C.c_void_p), ("top2_gap", C.c_void_p),
    ]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _as_logit_array(x):
    """Accept numpy float32, numpy uint16 (raw bf16 bits) or a torch CPU tensor."""
    if hasattr(x, "detach"):  # torch tensor, imported lazily by the caller
        import torch
        x = x.detach().cpu().contiguous()
        if x.dtype == torch.bfloat16:
            return x.view(torch.int16).numpy().view(np.uint16), BF16
        if x.dtype == torch.float32:
            return x.numpy(), F32
        raise TypeError(f"unsupported logit dtype {x.dtype}")
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.uint16:
        return x, BF16
    raise TypeError(f"unsupported logit dtype {x.dtype}")


class Oracle:
    def __init__(self, lib_path: str):
        L = C.CDLL(lib_path)
        self.L = L
        L.adasd_oracle_philox4x32_10.argtypes = [C.c_void_p] * 3
        L.adasd_oracle_uniform24.restype = C.c_double
        L.adasd_oracle_uniform24.argtypes = [C.c_uint32]
        L.adasd_oracle_uniform32.restype = C.c_double
        L.adasd_oracle_uniform32.argtypes = [C.c_uint32]
        L.adasd_oracle_accept_words.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                                C.c_void_p, C.c_void_p]
        L.adasd_oracle_gumbel_word.restype = C.c_uint32
        L.adasd_oracle_gumbel_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                               C.c_uint32]
        L.adasd_oracle_row_stats.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.adasd_oracle_jsd.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.adasd_oracle_jsd_entropy_form.argtypes = L.adasd_oracle_jsd.argtypes
        L.adasd_oracle_kde_logpdf.restype = C.c_double
        L.adasd_oracle_kde_logpdf.argtypes = [C.c_double, C.c_void_p, C.c_int, C.c_int]
        L.adasd_oracle_posterior.restype = C.c_double
        L.adasd_oracle_posterior.argtypes = [C.c_double, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                             C.c_int, C.c_int]
        L.adasd_oracle_draft_entropy.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64,
                                                 C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                 C.c_void_p, C.c_void_p]
        L.adasd_oracle_draft_sample.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64,
                                                C.c_void_p, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p,
                                                C.c_uint32, C.c_void_p, C.c_void_p]
        L.adasd_oracle_verify.argtypes = [C.c_void_p]
        L.adasd_oracle_update.argtypes = [C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 4 + \
            [C.c_double] + [C.c_void_p] * 8
        L.adasd_oracle_num_threads.restype = C.c_int

    # -- randomness -------------------------------------------------------
    def philox(self, ctr, key):
        c = np.asarray(ctr, dtype=np.uint32)
        k = np.asarray(key, dtype=np.uint32)
        out = np.zeros(4, dtype=np.uint32)
        self.L.adasd_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
        return out

    def uniform24(self, x):
        return self.L.adasd_oracle_uniform24(int(x))

    def uniform32(self, x):
        return self.L.adasd_oracle_uniform32(int(x))

    def accept_words(self, seed, seq, rnd, pos):
        a, b = C.c_uint32(), C.c_uint32()
        self.L.adasd_oracle_accept_words(seed, seq, rnd, pos, C.byref(a), C.byref(b))
        return a.value, b.value

    def gumbel_word(self, seed, seq, rnd, pos, v):
        return self.L.adasd_oracle_gumbel_word(seed, seq, rnd, pos, v)

    # -- statistics -------------------------------------------------------
    def row_stats(self, row):
        r, dt = _as_logit_array(row)
        lse, H = C.c_double(), C.c_double()
        bad = self.L.adasd_oracle_row_stats(_ptr(r), dt, r.shape[-1], C.byref(lse), C.byref(H))
        return lse.value, H.value, bad

    def jsd(self, prow, qrow, entropy_form=False):
        p, dt = _as_logit_array(prow)
        q, dt2 = _as_logit_array(qrow)
        assert dt == dt2 and p.shape == q.shape
        D = C.c_double()
        f = self.L.adasd_oracle_jsd_entropy_form if entropy_form else self.L.adasd_oracle_jsd
        f(_ptr(p), _ptr(q), dt, p.shape[-1], C.byref(D))
        return D.value

    def kde_logpdf(self, d, samples, bw_rule=0):
        s = np.ascontiguousarray(samples, dtype=np.float32)
        return self.L.adasd_oracle_kde_logpdf(float(d), _ptr(s), len(s), bw_rule)

    def posterior(self, d, LA, LR, min_n=2, bw_rule=0):
        a = np.ascontiguousarray(LA, dtype=np.float32)
        r = np.ascontiguousarray(LR, dtype=np.float32)
        return self.L.adasd_oracle_posterior(float(d), _ptr(a), len(a), _ptr(r), len(r), min_n,
                                             bw_rule)

    def draft_entropy(self, logits, T_G=None, active=None, step=0, k_max=1 << 30):
        z, dt = _as_logit_array(logits)
        B, V = z.shape
        H = np.zeros(B, dtype=np.float64)
        stop = np.zeros(B, dtype=np.uint8)
        tg = None if T_G is None else np.ascontiguousarray(T_G, dtype=np.float32)
        act = None if active is None else np.ascontiguousarray(active, dtype=np.uint8)
        self.L.adasd_oracle_draft_entropy(_ptr(z), dt, B, V, V, _ptr(tg), _ptr(act), step, k_max,
                                          _ptr(H), _ptr(stop))
        return H, stop

    def draft_sample(self, logits, active=None, step=0, seed=0, seq_id=None, rounds=None, round0=0,
                     shared_row=0):
        """x ~ softmax(row) for every active row; returns (tokens, top2_gap).
        shared_row = n > 0: logits hold ONE row [1, V] that n draws (sequences 0..n-1 unless seq_id is
        given) refer to (row stride 0)."""
        z, dt = _as_logit_array(logits)
        B, V = z.shape
        stride = V
        if shared_row:
            assert B == 1
            B, stride = int(shared_row), 0
        act = None if active is None else np.ascontiguousarray(active, dtype=np.uint8)
        sid = None if seq_id is None else np.ascontiguousarray(seq_id, dtype=np.uint32)
        rnd = None if rounds is None else np.ascontiguousarray(rounds, dtype=np.uint32)
        tok = np.zeros(B, np.int32)
        gap = np.zeros(B, np.float64)
        self.L.adasd_oracle_draft_sample(_ptr(z), dt, B, V, stride, _ptr(act), step, seed, _ptr(sid),
                                         _ptr(rnd), round0, _ptr(tok), _ptr(gap))
        return tok, gap

    # -- verification -----------------------------------------------------
    def verify(self, target_logits, draft_logits, draft_tokens, draft_len=None, LA=None, LR=None,
               nA=None, nR=None, seed=0, seq_id=None, rounds=None, round0=0, reject_rule=0,
               kde_min_n=2, bw_rule=0, relaxed_off=0, base_test=0, list_update=0, d_eps=1e-6,
               shared_rows=False):
        """shared_rows: the logits hold ONE sequence ([1, k+1, V], [1, k, V]) that every row of
        draft_tokens refers to (sequence stride 0): many draws on the same rows without copies."""
        t, dt = _as_logit_array(target_logits)
        d, dt2 = _as_logit_array(draft_logits)
        assert dt == dt2
        B, K1, V = t.shape
        K = K1 - 1
        assert d.shape == (B, K, V), (d.shape, t.shape)
        seq = 1
        if shared_rows:
            assert B == 1
            B = int(np.asarray(draft_tokens).shape[0])
            seq = 0
        tok = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, K)
        dl = None if draft_len is None else np.ascontiguousarray(draft_len, dtype=np.int32)
        cap = 0
        if LA is not None:
            LA = np.ascontiguousarray(LA, dtype=np.float32)
            LR = np.ascontiguousarray(LR, dtype=np.float32)
            nA = np.ascontiguousarray(nA, dtype=np.int32)
            nR = np.ascontiguousarray(nR, dtype=np.int32)
            cap = LA.shape[1]
            assert LA.shape == (B, cap) and LR.shape == (B, cap)
        sid = None if seq_id is None else np.ascontiguousarray(seq_id, dtype=np.uint32)
        rnd = None if rounds is None else np.ascontiguousarray(rounds, dtype=np.uint32)
        out = dict(
            n_accept=np.zeros(B, np.int32), next_token=np.zeros(B, np.int32),
            H_p=np.zeros((B, K), np.float64), H_q=np.zeros((B, K), np.float64),
            d_js=np.zeros((B, K), np.float64), p_accept=np.zeros((B, K), np.float64),
            accept_mask=np.zeros((B, K), np.uint8), status=np.zeros(B, np.uint32),
            base_margin=np.zeros((B, K), np.float64), relaxed_margin=np.zeros((B, K), np.float64),
            top2_gap=np.zeros(B, np.float64))
        a = _VerifyArgs(
            _ptr(t), _ptr(d), dt, B, K, V, seq * K1 * V, V, seq * K * V, V, _ptr(tok), _ptr(dl), cap,
            _ptr(LA), _ptr(LR), _ptr(nA), _ptr(nR), seed, _ptr(sid), _ptr(rnd), round0,
            reject_rule, kde_min_n, bw_rule, relaxed_off, base_test, list_update, d_eps,
            _ptr(out["n_accept"]), _ptr(out["next_token"]), _ptr(out["H_p"]), _ptr(out["H_q"]),
            _ptr(out["d_js"]), _ptr(out["p_accept"]), _ptr(out["accept_mask"]),
            _ptr(out["status"]), _ptr(out["base_margin"]), _ptr(out["relaxed_margin"]),
            _ptr(out["top2_gap"]))
        rc = self.L.adasd_oracle_verify(C.byref(a))
        if rc != 0:
            raise ValueError("oracle: invalid arguments")
        return out

    def update(self, state, n_accept, draft_len, H_q, d_js, k_max, d_eps=1e-6):
        """In-place update of ``state`` = dict(LA, LR, nA, nR, ent_sum, ent_cnt, T_G)."""
        B, cap = state["LA"].shape
        na = np.ascontiguousarray(n_accept, dtype=np.int32)
        dl = None if draft_len is None else np.ascontiguousarray(draft_len, dtype=np.int32)
        hq = np.ascontiguousarray(H_q, dtype=np.float64)
        dj = np.ascontiguousarray(d_js, dtype=np.float64)
        status = np.zeros(B, np.uint32)
        self.L.adasd_oracle_update(B, k_max, cap, _ptr(na), _ptr(dl), _ptr(hq), _ptr(dj),
                                   float(d_eps), _ptr(state["LA"]), _ptr(state["LR"]),
                                   _ptr(state["nA"]), _ptr(state["nR"]), _ptr(state["ent_sum"]),
                                   _ptr(state["ent_cnt"]), _ptr(state["T_G"]), _ptr(status))
        return status

    def num_threads(self):
        return self.L.adasd_oracle_num_threads()


def new_state(B, cap):
    """Initial state of Algorithm 1: empty lists, T_G = 0."""
    return dict(LA=np.zeros((B, cap), np.float32), LR=np.zeros((B, cap), np.float32),
                nA=np.zeros(B, np.int32), nR=np.zeros(B, np.int32),
                ent_sum=np.zeros(B, np.float64), ent_cnt=np.zeros(B, np.int32),
                T_G=np.zeros(B, np.float32))


_cached = None


def load_oracle() -> Oracle:
    global _cached
    if _cached is None:
        _cached = Oracle(build_oracle())
    return _cached
