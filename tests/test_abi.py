"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything is enqueued (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "adasd.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2512_11280_amd import build as b
    path = b.build(force=False)
    return C.CDLL(path)


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adasd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"adasd_draft_entropy", "adasd_draft_step", "adasd_verify", "adasd_update_thresholds", "adasd_workspace_bytes",
            "adasd_workspace_init", "adasd_state_init", "adasd_strerror", "adasd_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_error_strings(lib):
    lib.adasd_version.restype = C.c_int
    lib.adasd_strerror.restype = C.c_char_p
    assert lib.adasd_version() >= 100
    assert lib.adasd_strerror(0) == b"ok"
    seen = {lib.adasd_strerror(c) for c in range(-6, 1)}
    assert len(seen) == 7 and b"unknown error code" not in seen
    assert lib.adasd_strerror(-99) == b"unknown error code"


def test_workspace_size_query(lib):
    n = C.c_size_t()
    f = lib.adasd_workspace_bytes
    f.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    assert f(32, 8, 128256, 1, C.byref(n)) == 0 and n.value > 0
    big = n.value
    assert f(1, 8, 128256, 1, C.byref(n)) == 0 and 0 < n.value < big
    assert f(32, 8, 128256, 1, None) == -1
    assert f(-1, 8, 128256, 1, C.byref(n)) == -1
    assert f(32, 8, 0, 1, C.byref(n)) == -1
    assert f(32, 8, 128256, 5, C.byref(n)) == -1
    assert f(32, 65, 128256, 1, C.byref(n)) == -5        # k_max above the compiled limit
    assert f(32, 8, (1 << 24) + 1, 1, C.byref(n)) == -5
    assert f(40000, 8, 128256, 1, C.byref(n)) == -5


def test_null_arguments_are_rejected_on_the_host(lib):
    lib.adasd_verify.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    assert lib.adasd_verify(None, None, None) == -1
    lib.adasd_state_init.argtypes = [C.c_void_p, C.c_void_p]
    assert lib.adasd_state_init(None, None) == -1
    lib.adasd_workspace_init.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.adasd_workspace_init(None, 0, None) == -4
    lib.adasd_draft_entropy.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_void_p,
                                        C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.adasd_draft_entropy(None, 1, 4, 128, 128, None, None, 0, 20, None, None, None, 0, None) == -1
    assert lib.adasd_draft_entropy(None, 1, 0, 128, 128, None, None, 0, 20, None, None, None, 0, None) == 0
    lib.adasd_update_thresholds.argtypes = [C.c_void_p] + [C.c_int] + [C.c_void_p] * 7
    assert lib.adasd_update_thresholds(None, 4, None, None, None, None, None, None, None) == -1
    lib.adasd_profile_read.argtypes = [C.c_int, C.c_void_p, C.c_void_p]
    assert lib.adasd_profile_read(0, None, None) == -1


def test_newer_entry_points_validate_on_the_host(lib):
    lib.adasd_state_refresh.argtypes = [C.c_void_p, C.c_void_p]
    assert lib.adasd_state_refresh(None, None) == -1
    lib.adasd_draft_step.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint32,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                     C.c_void_p]
    args = [None, 1, 4, 128, 128, None, None, 0, 20, 7, None, None, 0, None, None, None, None, None, 0, None]
    assert lib.adasd_draft_step(*args) == -1                    # no logits
    args[2] = 0
    assert lib.adasd_draft_step(*args) == 0                     # no rows: nothing to do
    for name, n_ptr in (("stats", 1), ("jsd", 2), ("sample", 1), ("pick", 2), ("settle", 2)):
        f = getattr(lib, "adasd_verify_shard_" + name)
        f.argtypes = [C.c_void_p] * (3 + n_ptr)
        assert f(*([None] * (3 + n_ptr))) == -1, name
    lib.adasd_verify_shard_decide.argtypes = [C.c_void_p] * 6
    assert lib.adasd_verify_shard_decide(None, None, None, None, None, None) == -1
    lib.adasd_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.adasd_stream_read(None, 0, None, 0, None) == 0          # nothing to read
    assert lib.adasd_stream_read(None, 64, None, 1, None) == -1
    assert lib.adasd_stream_read(256, 24, 256, 1, None) == -2            # not whole 128-bit vectors
    assert lib.adasd_stream_read(264, 64, 256, 1, None) == -2            # source below 16-byte alignment
    assert lib.adasd_stream_read(256, 65536, 256, 1, None) == -4         # two pieces, one word of room
    lib.adasd_verify_shard_refine.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    assert lib.adasd_verify_shard_refine(None, None, None, 0, None, None) == -1


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    import paper_2512_11280_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="missing"):
        b.load_library()
