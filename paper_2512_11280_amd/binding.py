"""Thin ctypes binding of ``libadasd.so``: argument marshalling only.

Function names mirror the C ABI in ``include/adasd.h`` (``adasd_draft_entropy`` ->
``draft_entropy`` and so on).  Tensors are torch CUDA tensors (PyTorch is used for device memory
and streams only); all arithmetic happens in the HIP kernels.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

F32, BF16 = 0, 1
ST_BAD_TOKEN, ST_NONFINITE, ST_ZERO_MASS, ST_OVERFLOW, ST_EXACT_PATH, ST_BAD_LENGTH, ST_UNSETTLED = 1, 2, 4, 8, 16, 32, 64
SHARD_CAND_BYTES = 128

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libadasd.so")
_lib = None


class AdasdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load_library().adasd_strerror(code).decode()
        super().__init__(f"{where}: {msg} ({code})")


class _State(C.Structure):
    _fields_ = [("B", C.c_int32), ("cap", C.c_int32), ("T_G", C.c_void_p), ("ent_sum", C.c_void_p),
                ("ent_cnt", C.c_void_p), ("LA", C.c_void_p), ("LR", C.c_void_p),
                ("nA", C.c_void_p), ("nR", C.c_void_p), ("mom", C.c_void_p)]


class _Options(C.Structure):
    _fields_ = [("base_test", C.c_int32), ("reject_rule", C.c_int32), ("kde_min_n", C.c_int32),
                ("bw_rule", C.c_int32), ("relaxed_off", C.c_int32), ("d_eps", C.c_float),
                ("stats_path", C.c_int32), ("apply_update", C.c_int32), ("list_update", C.c_int32),
                ("wait_polls", C.c_int32)]


class _VerifyArgs(C.Structure):
    _fields_ = [
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p), ("dt", C.c_int),
        ("B", C.c_int32), ("k_max", C.c_int32), ("V", C.c_int32),
        ("t_seq_stride", C.c_int64), ("t_pos_stride", C.c_int64),
        ("d_seq_stride", C.c_int64), ("d_pos_stride", C.c_int64),
        ("draft_tokens", C.c_void_p), ("draft_len", C.c_void_p), ("state", C.POINTER(_State)),
        ("seed", C.c_uint64), ("seq_id", C.c_void_p), ("round", C.c_void_p), ("round0", C.c_uint32),
        ("n_accept", C.c_void_p), ("next_token", C.c_void_p), ("H_p", C.c_void_p),
        ("H_q", C.c_void_p), ("d_js", C.c_void_p), ("p_accept", C.c_void_p),
        ("accept_mask", C.c_void_p), ("status", C.c_void_p),
        ("workspace", C.c_void_p), ("ws_bytes", C.c_size_t)]


class _Shard(C.Structure):
    _fields_ = [("n_shards", C.c_int32), ("shard", C.c_int32), ("V_total", C.c_int32), ("col_begin", C.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libadasd.so; raises (never falls back to a CPU path) if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2512_11280_amd.build`")
    L = C.CDLL(_LIB_PATH)
    L.adasd_version.restype = C.c_int
    L.adasd_strerror.restype = C.c_char_p
    L.adasd_strerror.argtypes = [C.c_int]
    L.adasd_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.adasd_workspace_init.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
    L.adasd_state_init.argtypes = [C.POINTER(_State), C.c_void_p]
    L.adasd_state_refresh.argtypes = [C.POINTER(_State), C.c_void_p]
    L.adasd_draft_step.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_void_p,
                                   C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint32,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                   C.c_void_p]
    L.adasd_draft_entropy.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_void_p,
                                      C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
    L.adasd_verify.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Options), C.c_void_p]
    L.adasd_verify_noalloc.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Options), C.c_void_p]
    L.adasd_verify_shard_stats.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_void_p]
    L.adasd_verify_shard_jsd.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_void_p,
                                         C.c_void_p]
    L.adasd_verify_shard_decide.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_void_p,
                                            C.POINTER(_Options), C.c_void_p]
    L.adasd_verify_shard_sample.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_void_p]
    L.adasd_verify_shard_pick.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_void_p, C.c_void_p]
    L.adasd_verify_shard_refine.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_int, C.c_void_p,
                                            C.c_void_p]
    L.adasd_verify_shard_settle.argtypes = [C.POINTER(_VerifyArgs), C.POINTER(_Shard), C.c_void_p, C.c_void_p, C.c_void_p]
    L.adasd_update_thresholds.argtypes = [C.POINTER(_State), C.c_int, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.POINTER(_Options), C.c_void_p,
                                          C.c_void_p]
    L.adasd_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]
    L.adasd_profile_enable.argtypes = [C.c_int]
    L.adasd_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    _lib = L
    return L


def _check(rc: int, where: str):
    if rc != 0:
        raise AdasdError(rc, where)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"logits must be bfloat16 or float32, got {t.dtype}")


def _p(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _need(t: Optional[torch.Tensor], dtype, name: str, optional: bool = False):
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous CUDA tensor of {dtype}")


@dataclass
class Options:
    base_test: int = 0
    reject_rule: int = 0
    kde_min_n: int = 2
    bw_rule: int = 0
    relaxed_off: int = 0
    d_eps: float = 1e-6
    stats_path: int = 0
    apply_update: int = 0
    list_update: int = 0
    wait_polls: int = 0

    def _c(self) -> _Options:
        return _Options(self.base_test, self.reject_rule, self.kde_min_n, self.bw_rule,
                        self.relaxed_off, self.d_eps, self.stats_path, self.apply_update,
                        self.list_update, self.wait_polls)


def workspace_bytes(B: int, k_max: int, V: int, dtype: torch.dtype) -> int:
    n = C.c_size_t()
    code = BF16 if dtype == torch.bfloat16 else F32
    _check(load_library().adasd_workspace_bytes(B, k_max, V, code, C.byref(n)), "adasd_workspace_bytes")
    return n.value


class Workspace:
    """Device scratch for adasd_verify / adasd_draft_entropy (allocated through torch)."""

    def __init__(self, B: int, k_max: int, V: int, dtype: torch.dtype, device="cuda"):
        self.bytes = workspace_bytes(B, k_max, V, dtype)
        self.buf = torch.empty(self.bytes + 256, dtype=torch.uint8, device=device)
        off = (-self.buf.data_ptr()) % 256
        self.ptr = self.buf.data_ptr() + off
        _check(load_library().adasd_workspace_init(self.ptr, self.bytes, _stream()), "adasd_workspace_init")


class State:
    """Per-sequence adaptive state (history lists, rejected-entropy sum, generation threshold)."""

    def __init__(self, B: int, cap: int, device="cuda", running_sums: bool = True):
        """running_sums: keep adasd_state.mom (sums of the lists for the bandwidths); without it the
        decision stage adds the lists up in every call."""
        self.B, self.cap = B, cap
        self.mom = torch.empty(B, 4, dtype=torch.float64, device=device) if running_sums else None
        self.T_G = torch.empty(B, dtype=torch.float32, device=device)
        self.ent_sum = torch.empty(B, dtype=torch.float64, device=device)
        self.ent_cnt = torch.empty(B, dtype=torch.int32, device=device)
        self.LA = torch.zeros(B, cap, dtype=torch.float32, device=device)
        self.LR = torch.zeros(B, cap, dtype=torch.float32, device=device)
        self.nA = torch.empty(B, dtype=torch.int32, device=device)
        self.nR = torch.empty(B, dtype=torch.int32, device=device)
        _check(load_library().adasd_state_init(C.byref(self._c()), _stream()), "adasd_state_init")

    def _c(self) -> _State:
        return _State(self.B, self.cap, _p(self.T_G), _p(self.ent_sum), _p(self.ent_cnt),
                      _p(self.LA), _p(self.LR), _p(self.nA), _p(self.nR), _p(self.mom))

    def load(self, host: dict):
        """Copy a host-side state (numpy arrays keyed like the fields) onto the device."""
        for k in ("T_G", "ent_sum", "ent_cnt", "LA", "LR", "nA", "nR"):
            getattr(self, k).copy_(torch.from_numpy(host[k]))
        _check(load_library().adasd_state_refresh(C.byref(self._c()), _stream()), "adasd_state_refresh")
        return self

    def to_host(self) -> dict:
        return {k: getattr(self, k).cpu().numpy()
                for k in ("T_G", "ent_sum", "ent_cnt", "LA", "LR", "nA", "nR")}


def draft_entropy(draft_logits: torch.Tensor, workspace: Workspace, T_G: Optional[torch.Tensor] = None,
                  active: Optional[torch.Tensor] = None, step: int = 0, k_max: int = 1 << 30,
                  H_out: Optional[torch.Tensor] = None, stop_out: Optional[torch.Tensor] = None):
    """adasd_draft_entropy: H(q) of every row of draft_logits [B, V] and the stop flag."""
    if draft_logits.dim() != 2 or not draft_logits.is_cuda or draft_logits.stride(1) != 1:
        raise ValueError("draft_logits must be a CUDA tensor [B, V] with contiguous vocabulary")
    B, V = draft_logits.shape
    dev = draft_logits.device
    if H_out is None:
        H_out = torch.empty(B, dtype=torch.float32, device=dev)
    if stop_out is None:
        stop_out = torch.empty(B, dtype=torch.uint8, device=dev)
    _need(T_G, torch.float32, "T_G", optional=True)
    _need(active, torch.uint8, "active", optional=True)
    _need(H_out, torch.float32, "H_out")
    _need(stop_out, torch.uint8, "stop_out")
    rc = load_library().adasd_draft_entropy(
        draft_logits.data_ptr(), _dtype_code(draft_logits), B, V, draft_logits.stride(0) if B > 1 else V,
        _p(T_G), _p(active), step, k_max, H_out.data_ptr(), stop_out.data_ptr(), workspace.ptr,
        workspace.bytes, _stream())
    _check(rc, "adasd_draft_entropy")
    return H_out, stop_out


def draft_step(draft_logits: torch.Tensor, workspace: Workspace, T_G: Optional[torch.Tensor] = None,
               active: Optional[torch.Tensor] = None, step: int = 0, k_max: int = 1 << 30, seed: int = 0,
               seq_id: Optional[torch.Tensor] = None, rounds: Optional[torch.Tensor] = None, round0: int = 0,
               H_out: Optional[torch.Tensor] = None, stop_out: Optional[torch.Tensor] = None,
               token_out: Optional[torch.Tensor] = None, status_out: Optional[torch.Tensor] = None):
    """adasd_draft_step: H(q), the stop flag and a token drawn from softmax(row) for every row of
    draft_logits [B, V].  Returns (H, stop, token, status)."""
    if draft_logits.dim() != 2 or not draft_logits.is_cuda or draft_logits.stride(1) != 1:
        raise ValueError("draft_logits must be a CUDA tensor [B, V] with contiguous vocabulary")
    B, V = draft_logits.shape
    dev = draft_logits.device
    if H_out is None:
        H_out = torch.empty(B, dtype=torch.float32, device=dev)
    if stop_out is None:
        stop_out = torch.empty(B, dtype=torch.uint8, device=dev)
    if token_out is None:
        token_out = torch.empty(B, dtype=torch.int32, device=dev)
    if status_out is None:
        status_out = torch.empty(B, dtype=torch.int32, device=dev)
    _need(T_G, torch.float32, "T_G", optional=True)
    _need(active, torch.uint8, "active", optional=True)
    _need(seq_id, torch.int32, "seq_id", optional=True)
    _need(rounds, torch.int32, "rounds", optional=True)
    _need(H_out, torch.float32, "H_out")
    _need(stop_out, torch.uint8, "stop_out")
    _need(token_out, torch.int32, "token_out")
    _need(status_out, torch.int32, "status_out")
    rc = load_library().adasd_draft_step(
        draft_logits.data_ptr(), _dtype_code(draft_logits), B, V, draft_logits.stride(0) if B > 1 else V,
        _p(T_G), _p(active), step, k_max, seed & 0xFFFFFFFFFFFFFFFF, _p(seq_id), _p(rounds),
        round0 & 0xFFFFFFFF, H_out.data_ptr(), stop_out.data_ptr(), token_out.data_ptr(),
        status_out.data_ptr(), workspace.ptr, workspace.bytes, _stream())
    _check(rc, "adasd_draft_step")
    return H_out, stop_out, token_out, status_out


@dataclass
class VerifyResult:
    n_accept: torch.Tensor
    next_token: torch.Tensor
    H_p: torch.Tensor
    H_q: torch.Tensor
    d_js: torch.Tensor
    p_accept: torch.Tensor
    accept_mask: torch.Tensor
    status: torch.Tensor


def alloc_verify_result(B: int, K: int, device="cuda") -> VerifyResult:
    f = dict(dtype=torch.float32, device=device)
    return VerifyResult(torch.empty(B, dtype=torch.int32, device=device),
                        torch.empty(B, dtype=torch.int32, device=device),
                        torch.empty(B, K, **f), torch.empty(B, K, **f), torch.empty(B, K, **f),
                        torch.empty(B, K, **f), torch.empty(B, K, dtype=torch.uint8, device=device),
                        torch.empty(B, dtype=torch.int32, device=device))


def verify(target_logits: torch.Tensor, draft_logits: torch.Tensor, draft_tokens: torch.Tensor,
           workspace: Optional[Workspace], state: Optional[State] = None, draft_len: Optional[torch.Tensor] = None,
           seed: int = 0, seq_id: Optional[torch.Tensor] = None, rounds: Optional[torch.Tensor] = None,
           round0: int = 0, options: Optional[Options] = None,
           out: Optional[VerifyResult] = None) -> VerifyResult:
    """adasd_verify on target_logits [B, k+1, V], draft_logits [B, k, V], draft_tokens [B, k].
    workspace=None: adasd_verify_noalloc (the library's built-in scratch array; `out` should then be
    given too, so that the call allocates nothing at all)."""
    if target_logits.dim() != 3 or draft_logits.dim() != 3:
        raise ValueError("logits must be [B, k(+1), V]")
    B, K1, V = target_logits.shape
    K = K1 - 1
    if tuple(draft_logits.shape) != (B, K, V):
        raise ValueError(f"draft_logits must be [{B}, {K}, {V}]")
    if target_logits.stride(2) != 1 or (K > 0 and draft_logits.stride(2) != 1):
        raise ValueError("vocabulary dimension must be contiguous")
    if draft_logits.dtype != target_logits.dtype:
        raise TypeError("target and draft logits must share a dtype")
    _need(draft_tokens, torch.int32, "draft_tokens")
    _need(draft_len, torch.int32, "draft_len", optional=True)
    _need(seq_id, torch.int32, "seq_id", optional=True)
    _need(rounds, torch.int32, "rounds", optional=True)
    if out is None:
        out = alloc_verify_result(B, K, target_logits.device)
    st = state._c() if state is not None else None
    a = _VerifyArgs(
        target_logits.data_ptr(), draft_logits.data_ptr(), _dtype_code(target_logits), B, K, V,
        target_logits.stride(0), target_logits.stride(1),
        draft_logits.stride(0) if K > 0 else V, draft_logits.stride(1) if K > 0 else V,
        draft_tokens.data_ptr(), _p(draft_len), C.pointer(st) if st is not None else None,
        seed & 0xFFFFFFFFFFFFFFFF, _p(seq_id), _p(rounds), round0 & 0xFFFFFFFF,
        out.n_accept.data_ptr(), out.next_token.data_ptr(), out.H_p.data_ptr(), out.H_q.data_ptr(),
        out.d_js.data_ptr(), out.p_accept.data_ptr(), out.accept_mask.data_ptr(),
        out.status.data_ptr(), workspace.ptr if workspace is not None else None,
        workspace.bytes if workspace is not None else 0)
    opt = options._c() if options is not None else None
    if workspace is None:
        rc = load_library().adasd_verify_noalloc(C.byref(a), C.byref(opt) if opt is not None else None, _stream())
        _check(rc, "adasd_verify_noalloc")
        return out
    rc = load_library().adasd_verify(C.byref(a), C.byref(opt) if opt is not None else None, _stream())
    _check(rc, "adasd_verify")
    return out


@dataclass
class Shard:
    """adasd_shard: which columns of the vocabulary a column-sharded call is given."""
    n_shards: int
    shard: int
    V_total: int
    col_begin: int

    def _c(self) -> _Shard:
        return _Shard(self.n_shards, self.shard, self.V_total, self.col_begin)


def _local_args(target_local, draft_local, draft_tokens, workspace, draft_len, seed=0, seq_id=None, rounds=None,
                round0=0, next_token=None, status=None) -> _VerifyArgs:
    """adasd_verify_args of a local (column slice) call: logits and strides of the slice, no outputs."""
    B, K1, V = target_local.shape
    K = K1 - 1
    if tuple(draft_local.shape) != (B, K, V) or target_local.stride(2) != 1 or (K > 0 and draft_local.stride(2) != 1):
        raise ValueError("local logits must be [B, k(+1), V_local] with the vocabulary contiguous")
    _need(draft_tokens, torch.int32, "draft_tokens")
    _need(draft_len, torch.int32, "draft_len", optional=True)
    _need(seq_id, torch.int32, "seq_id", optional=True)
    _need(rounds, torch.int32, "rounds", optional=True)
    return _VerifyArgs(
        target_local.data_ptr(), draft_local.data_ptr(), _dtype_code(target_local), B, K, V,
        target_local.stride(0), target_local.stride(1),
        draft_local.stride(0) if K > 0 else V, draft_local.stride(1) if K > 0 else V,
        draft_tokens.data_ptr(), _p(draft_len), None, seed & 0xFFFFFFFFFFFFFFFF, _p(seq_id), _p(rounds),
        round0 & 0xFFFFFFFF, None, _p(next_token), None, None, None, None, None, _p(status),
        workspace.ptr, workspace.bytes)


def verify_shard_stats(target_local, draft_local, draft_tokens, workspace: Workspace, shard: Shard,
                       draft_len=None, triples_out=None):
    """adasd_verify_shard_stats: one (reference, sum, weighted sum) triple per row over the local columns."""
    a = _local_args(target_local, draft_local, draft_tokens, workspace, draft_len)
    if triples_out is None:
        triples_out = torch.empty(a.B * a.k_max * 2, 4, dtype=torch.float32, device=target_local.device)
    sh = shard._c()
    _check(load_library().adasd_verify_shard_stats(C.byref(a), C.byref(sh), triples_out.data_ptr(), _stream()),
           "adasd_verify_shard_stats")
    return triples_out


def verify_shard_jsd(target_local, draft_local, draft_tokens, workspace: Workspace, shard: Shard,
                     triples_all: torch.Tensor, draft_len=None, pos_out=None):
    """adasd_verify_shard_jsd: per position the local partial JS sum and the drafted token's logits."""
    a = _local_args(target_local, draft_local, draft_tokens, workspace, draft_len)
    _need(triples_all, torch.float32, "triples_all")
    if pos_out is None:
        pos_out = torch.empty(a.B * a.k_max, 4, dtype=torch.float32, device=target_local.device)
    sh = shard._c()
    _check(load_library().adasd_verify_shard_jsd(C.byref(a), C.byref(sh), triples_all.data_ptr(),
                                                 pos_out.data_ptr(), _stream()), "adasd_verify_shard_jsd")
    return pos_out


def _meta_args(B, k, dtype, draft_tokens, workspace, shard, out, state=None, draft_len=None, seed=0, seq_id=None,
               rounds=None, round0=0):
    """adasd_verify_args of a replicated call: whole-vocabulary shape, no logits, the outputs."""
    _need(draft_tokens, torch.int32, "draft_tokens")
    _need(draft_len, torch.int32, "draft_len", optional=True)
    _need(seq_id, torch.int32, "seq_id", optional=True)
    _need(rounds, torch.int32, "rounds", optional=True)
    st = state._c() if state is not None else None
    V = shard.V_total
    a = _VerifyArgs(
        None, None, BF16 if dtype == torch.bfloat16 else F32, B, k, V, (k + 1) * V, V, k * V, V,
        draft_tokens.data_ptr(), _p(draft_len), C.pointer(st) if st is not None else None,
        seed & 0xFFFFFFFFFFFFFFFF, _p(seq_id), _p(rounds), round0 & 0xFFFFFFFF,
        out.n_accept.data_ptr(), out.next_token.data_ptr(), out.H_p.data_ptr(), out.H_q.data_ptr(),
        out.d_js.data_ptr(), out.p_accept.data_ptr(), out.accept_mask.data_ptr(),
        out.status.data_ptr(), workspace.ptr, workspace.bytes)
    a._keep = st            # the struct only holds a pointer to it
    return a


def verify_shard_decide(B: int, k: int, dtype, draft_tokens, workspace: Workspace, shard: Shard,
                        triples_all: torch.Tensor, pos_all: torch.Tensor, state: Optional[State] = None,
                        draft_len=None, seed: int = 0, seq_id=None, rounds=None, round0: int = 0,
                        options: Optional[Options] = None, out: Optional[VerifyResult] = None) -> VerifyResult:
    """adasd_verify_shard_decide: the decisions of the round from the gathered records (no logits)."""
    _need(triples_all, torch.float32, "triples_all")
    _need(pos_all, torch.float32, "pos_all")
    if out is None:
        out = alloc_verify_result(B, k, draft_tokens.device)
    a = _meta_args(B, k, dtype, draft_tokens, workspace, shard, out, state, draft_len, seed, seq_id, rounds, round0)
    opt = options._c() if options is not None else None
    sh = shard._c()
    rc = load_library().adasd_verify_shard_decide(C.byref(a), C.byref(sh), triples_all.data_ptr(),
                                                  pos_all.data_ptr(),
                                                  C.byref(opt) if opt is not None else None, _stream())
    _check(rc, "adasd_verify_shard_decide")
    return out


def verify_shard_sample(target_local, draft_local, draft_tokens, workspace: Workspace, shard: Shard, draft_len=None,
                        seed: int = 0, seq_id=None, rounds=None, round0: int = 0, top_out=None):
    """adasd_verify_shard_sample: this holder's best / runner-up record of every sequence."""
    a = _local_args(target_local, draft_local, draft_tokens, workspace, draft_len, seed, seq_id, rounds, round0)
    if top_out is None:
        top_out = torch.empty(a.B, 4, dtype=torch.float32, device=target_local.device)
    sh = shard._c()
    _check(load_library().adasd_verify_shard_sample(C.byref(a), C.byref(sh), top_out.data_ptr(), _stream()),
           "adasd_verify_shard_sample")
    return top_out


def verify_shard_pick(B: int, k: int, dtype, draft_tokens, workspace: Workspace, shard: Shard, top_all: torch.Tensor,
                      out: VerifyResult, draft_len=None, tau_out=None):
    """adasd_verify_shard_pick: certain winners into out.next_token; returns tau [B] (+inf where settled)."""
    _need(top_all, torch.float32, "top_all")
    if tau_out is None:
        tau_out = torch.empty(B, dtype=torch.float32, device=draft_tokens.device)
    a = _meta_args(B, k, dtype, draft_tokens, workspace, shard, out, None, draft_len)
    sh = shard._c()
    _check(load_library().adasd_verify_shard_pick(C.byref(a), C.byref(sh), top_all.data_ptr(), tau_out.data_ptr(),
                                                  _stream()), "adasd_verify_shard_pick")
    return tau_out


def verify_shard_refine(target_local, draft_local, draft_tokens, workspace: Workspace, shard: Shard, tau: torch.Tensor,
                        draft_len=None, seed: int = 0, seq_id=None, rounds=None, round0: int = 0, cand_out=None,
                        exact_sums: int = 0):
    """adasd_verify_shard_refine: this holder's candidates and refined sums of the open sequences."""
    _need(tau, torch.float32, "tau")
    a = _local_args(target_local, draft_local, draft_tokens, workspace, draft_len, seed, seq_id, rounds, round0)
    if cand_out is None:
        cand_out = torch.empty(a.B, SHARD_CAND_BYTES, dtype=torch.uint8, device=target_local.device)
    sh = shard._c()
    _check(load_library().adasd_verify_shard_refine(C.byref(a), C.byref(sh), tau.data_ptr(), exact_sums, cand_out.data_ptr(),
                                                    _stream()), "adasd_verify_shard_refine")
    return cand_out


def verify_shard_settle(B: int, k: int, dtype, draft_tokens, workspace: Workspace, shard: Shard, tau: torch.Tensor,
                        cand_all: torch.Tensor, out: VerifyResult, draft_len=None, seed: int = 0, seq_id=None,
                        rounds=None, round0: int = 0):
    """adasd_verify_shard_settle: float64 decision of the open sequences into out.next_token / out.status."""
    _need(tau, torch.float32, "tau")
    _need(cand_all, torch.uint8, "cand_all")
    a = _meta_args(B, k, dtype, draft_tokens, workspace, shard, out, None, draft_len, seed, seq_id, rounds, round0)
    sh = shard._c()
    _check(load_library().adasd_verify_shard_settle(C.byref(a), C.byref(sh), tau.data_ptr(), cand_all.data_ptr(),
                                                    _stream()), "adasd_verify_shard_settle")


def update_thresholds(state: State, k_max: int, n_accept: torch.Tensor, H_q: torch.Tensor,
                      d_js: torch.Tensor, draft_len: Optional[torch.Tensor] = None,
                      options: Optional[Options] = None, status: Optional[torch.Tensor] = None):
    """adasd_update_thresholds: fold one verified round into the adaptive state."""
    _need(n_accept, torch.int32, "n_accept")
    _need(H_q, torch.float32, "H_q")
    _need(d_js, torch.float32, "d_js")
    _need(draft_len, torch.int32, "draft_len", optional=True)
    _need(status, torch.int32, "status", optional=True)
    st = state._c()
    opt = options._c() if options is not None else None
    rc = load_library().adasd_update_thresholds(
        C.byref(st), k_max, n_accept.data_ptr(), _p(draft_len), H_q.data_ptr(), d_js.data_ptr(),
        C.byref(opt) if opt is not None else None, _p(status), _stream())
    _check(rc, "adasd_update_thresholds")


def stream_read(src: torch.Tensor, sink: torch.Tensor):
    """adasd_stream_read on a contiguous device tensor; sink: int32 device tensor, one word per 32 KiB."""
    if not src.is_contiguous():
        raise ValueError("src must be contiguous")
    _need(sink, torch.int32, "sink")
    rc = load_library().adasd_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                          sink.numel(), _stream())
    _check(rc, "adasd_stream_read")


def profile_enable(max_launches: int):
    _check(load_library().adasd_profile_enable(max_launches), "adasd_profile_enable")


def profile_read(kernel_class: int):
    ms, n = C.c_double(), C.c_int()
    _check(load_library().adasd_profile_read(kernel_class, C.byref(ms), C.byref(n)), "adasd_profile_read")
    return ms.value, n.value


def profile_disable():
    _check(load_library().adasd_profile_disable(), "adasd_profile_disable")
