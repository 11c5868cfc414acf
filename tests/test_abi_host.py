"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
declared in include/gbnn.h, sizes are right, and every argument error is reported before any
launch (no compute call is made here)."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_1303_7032_amd import binding as gb

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    if not gb._LIB_PATH.exists():
        from paper_1303_7032_amd import build
        build.build()
    return gb.lib()


def declared_functions():
    text = (ROOT / "include" / "gbnn.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gbnn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"gbnn_store", "gbnn_prepare", "gbnn_retrieve", "gbnn_retrieve_symbols", "gbnn_w_bytes", "gbnn_workspace_bytes", "gbnn_strerror"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None, name


def test_sizes(lib):
    assert gb.gbnn_w_row_words(8, 256) == 64 and gb.gbnn_w_bytes(8, 256) == 512 * 1024
    assert gb.gbnn_w_bytes(16, 512) == 8 * 1024 * 1024
    assert gb.gbnn_w_row_words(3, 3) == 1 and gb.gbnn_w_bytes(3, 3) == 36
    assert gb.gbnn_w_row_words(7, 33) == 8
    for bad in [(1, 16), (65, 4), (8, 0), (64, 257), (2, 8193)]:
        assert gb.gbnn_w_bytes(*bad) == 0 and gb.gbnn_w_row_words(*bad) == 0
    ws = gb.gbnn_workspace_bytes(8, 256, 65536, "sum_of_max")
    assert ws > 0 and ws % 256 == 0
    assert gb.gbnn_workspace_bytes(8, 256, -1, "sum_of_max") == 0
    assert gb.gbnn_workspace_bytes(8, 256, 1, 9) == 0


def test_retrieve_argument_errors(lib):
    E = gb.ERRORS
    fake = 0x1000  # never dereferenced on the host; nothing is launched when an error is returned
    ws = 1 << 24

    def call(W=fake, C=8, L=256, V0=fake, Vout=fake, K=4, rule=1, gamma=1, cap=20, it=0, wsp=fake * 16, wsb=ws):
        return lib.gbnn_retrieve(W, C, L, V0, Vout, K, rule, gamma, cap, it, wsp, wsb, 0)

    assert call(C=1) == E["SHAPE"] and call(C=65, L=1) == E["SHAPE"] and call(L=0) == E["SHAPE"]
    assert call(C=64, L=257) == E["SHAPE"] and call(K=-1) == E["SHAPE"] and call(K=2 ** 31) == E["SHAPE"]
    assert call(rule=3) == E["RULE"] and call(rule=-1) == E["RULE"]
    assert call(gamma=-1) == E["GAMMA"] and call(gamma=32768) == E["GAMMA"]
    assert call(cap=0) == E["ITERS"]
    assert call(W=0) == E["NULL"] and call(V0=0) == E["NULL"] and call(Vout=0) == E["NULL"]
    assert call(wsp=0) == E["WORKSPACE"] and call(wsp=fake * 16 + 8) == E["WORKSPACE"] and call(wsb=16) == E["WORKSPACE"]


def test_retrieve_symbols_argument_errors(lib):
    E = gb.ERRORS
    fake = 0x1000
    ws = 1 << 24

    def call(W=fake, C=8, L=256, P=fake, K=4, rule=1, gamma=1, cap=20, bits=fake, sym=fake, it=0, wsp=fake * 16, wsb=ws):
        return lib.gbnn_retrieve_symbols(W, C, L, P, K, rule, gamma, cap, bits, sym, it, wsp, wsb, 0)

    assert call(C=1) == E["SHAPE"] and call(L=0) == E["SHAPE"] and call(K=-1) == E["SHAPE"]
    assert call(rule=3) == E["RULE"]
    assert call(gamma=-1) == E["GAMMA"] and call(gamma=32768) == E["GAMMA"]
    assert call(cap=0) == E["ITERS"]
    assert call(W=0) == E["NULL"] and call(P=0) == E["NULL"]
    assert call(wsp=0) == E["WORKSPACE"] and call(wsb=16) == E["WORKSPACE"]
    assert call(K=0, P=0, bits=0, sym=0) == gb.GBNN_OK     # nothing to do, nothing launched


def test_store_argument_errors(lib):
    E = gb.ERRORS
    assert lib.gbnn_store(0x1000, 1, 4, 0x1000, 1, 0, 0) == E["SHAPE"]
    assert lib.gbnn_store(0x1000, 4, 4, 0x1000, -1, 0, 0) == E["SHAPE"]
    assert lib.gbnn_store(0, 4, 4, 0x1000, 1, 0, 0) == E["NULL"]
    assert lib.gbnn_store(0x1000, 4, 4, 0, 1, 0, 0) == E["NULL"]


def test_prepare_argument_errors(lib):
    E = gb.ERRORS
    need = gb.gbnn_workspace_bytes(8, 256, 0, "hybrid")
    assert need >= gb.gbnn_w_bytes(8, 256) + 8 * 64 * 4 and need % 256 == 0
    assert lib.gbnn_prepare(0x1000, 1, 4, 0x10000, 1 << 20, 0) == E["SHAPE"]
    assert lib.gbnn_prepare(0, 8, 256, 0x10000, need, 0) == E["NULL"]
    assert lib.gbnn_prepare(0x1000, 8, 256, 0, need, 0) == E["WORKSPACE"]
    assert lib.gbnn_prepare(0x1000, 8, 256, 0x10010, need, 0) == E["WORKSPACE"]
    assert lib.gbnn_prepare(0x1000, 8, 256, 0x10000, need - 1, 0) == E["WORKSPACE"]


def test_store_update_argument_errors(lib):
    E = gb.ERRORS
    need = gb.gbnn_workspace_bytes(8, 256, 0, "hybrid")
    assert lib.gbnn_store_update(0x1000, 1, 4, 0x1000, 1, 0, 0x10000, need, 0) == E["SHAPE"]
    assert lib.gbnn_store_update(0x1000, 8, 256, 0x1000, -1, 0, 0x10000, need, 0) == E["SHAPE"]
    assert lib.gbnn_store_update(0, 8, 256, 0x1000, 1, 0, 0x10000, need, 0) == E["NULL"]
    assert lib.gbnn_store_update(0x1000, 8, 256, 0, 1, 0, 0x10000, need, 0) == E["NULL"]
    assert lib.gbnn_store_update(0x1000, 8, 256, 0x1000, 1, 0, 0, need, 0) == E["WORKSPACE"]
    assert lib.gbnn_store_update(0x1000, 8, 256, 0x1000, 1, 0, 0x10010, need, 0) == E["WORKSPACE"]
    assert lib.gbnn_store_update(0x1000, 8, 256, 0x1000, 1, 0, 0x10000, need - 1, 0) == E["WORKSPACE"]


def test_sparse_sizes_and_argument_errors(lib):
    E = gb.ERRORS
    base = gb.gbnn_sparse_bytes(8, 256, 0)
    assert base % 256 == 0 and base >= (2048 + 1) * 4 + 8 * 64 * 4 + 256
    assert gb.gbnn_sparse_bytes(8, 256, 1) == base + 256 and gb.gbnn_sparse_bytes(8, 256, 129) == base + 512
    assert gb.gbnn_sparse_bytes(8, 100, 0) == 0          # L must be a multiple of 32
    assert gb.gbnn_sparse_bytes(8, 256, -1) == 0 and gb.gbnn_sparse_bytes(8, 256, 1 << 32) == 0
    assert gb.gbnn_sparse_bytes(1, 256, 0) == 0
    assert lib.gbnn_sparse_count(0, 8, 256, 0x1000, 0) == E["NULL"]
    assert lib.gbnn_sparse_count(0x1000, 8, 256, 0, 0) == E["NULL"]
    assert lib.gbnn_sparse_count(0x1000, 1, 256, 0x1000, 0) == E["SHAPE"]
    assert lib.gbnn_sparsify(0x1000, 8, 100, 0x10000, 1 << 20, 0, 0) == E["SHAPE"]
    assert lib.gbnn_sparsify(0, 8, 256, 0x10000, 1 << 20, 0, 0) == E["NULL"]
    assert lib.gbnn_sparsify(0x1000, 8, 256, 0, 1 << 20, 0, 0) == E["WORKSPACE"]
    assert lib.gbnn_sparsify(0x1000, 8, 256, 0x10010, 1 << 20, 0, 0) == E["WORKSPACE"]
    assert lib.gbnn_sparsify(0x1000, 8, 256, 0x10000, base - 1, 0, 0) == E["WORKSPACE"]
    ok = (0x10000, base, 8, 256, 0x1000, 1, 20, 0, 0, 0, 0)
    assert lib.gbnn_retrieve_sparse(0x10000, base, 8, 100, 0x1000, 1, 20, 0, 0, 0, 0) == E["SHAPE"]
    assert lib.gbnn_retrieve_sparse(0x10000, base, 8, 256, 0x1000, -1, 20, 0, 0, 0, 0) == E["SHAPE"]
    assert lib.gbnn_retrieve_sparse(0x10000, base, 8, 256, 0x1000, 1, 0, 0, 0, 0, 0) == E["ITERS"]
    assert lib.gbnn_retrieve_sparse(0x10000, base, 8, 256, 0, 1, 20, 0, 0, 0, 0) == E["NULL"]
    assert lib.gbnn_retrieve_sparse(0, base, 8, 256, 0x1000, 1, 20, 0, 0, 0, 0) == E["WORKSPACE"]
    assert lib.gbnn_retrieve_sparse(0x10000, base - 1, 8, 256, 0x1000, 1, 20, 0, 0, 0, 0) == E["WORKSPACE"]
    assert lib.gbnn_retrieve_sparse(0x10000, base, 8, 256, 0, 0, 20, 0, 0, 0, 0) == 0   # K = 0: nothing to do
    del ok


def test_strerror_and_path(lib):
    for code in range(-8, 1):
        assert gb.gbnn_strerror(code)
    assert gb.gbnn_strerror(0) == "ok"
    assert gb.gbnn_retrieve_path(8, 256, "sum_of_max") == "wave1"
    assert gb.gbnn_retrieve_path(8, 128, "sum_of_sum") == "half1"
    assert gb.gbnn_retrieve_path(32, 32, "hybrid") == "half1"
    assert gb.gbnn_retrieve_path(2, 512, "sum_of_max") == "half1"
    assert gb.gbnn_retrieve_path(64, 32, "sum_of_max") == "wave1"
    assert gb.gbnn_retrieve_path(16, 512, "hybrid") == "wave4"
    assert gb.gbnn_retrieve_path(12, 256, "hybrid") == "wave2"
    assert gb.gbnn_retrieve_path(4, 16, "sum_of_max") == "half1"       # clusters padded to 32 neurons
    assert gb.gbnn_retrieve_path(8, 100, "hybrid") == "half1"          # ... to 128
    assert gb.gbnn_retrieve_path(10, 300, "sum_of_sum") == "wave4"     # ... to 512
    assert gb.gbnn_retrieve_path(60, 270, "sum_of_max") == "generic"   # 60 x 512 neurons would exceed the limit
    assert gb.gbnn_retrieve_path(3, 2049, "sum_of_max") == "generic"   # no more than 2048 neurons per cluster
    assert gb.gbnn_retrieve_path(16, 1024, "sum_of_max") == "wave8"
    assert gb.gbnn_retrieve_path(8, 2048, "hybrid") == "wave8"
    assert gb.gbnn_retrieve_path(16, 1024, "sum_of_sum") == "wave8"
    assert gb.gbnn_retrieve_path(4, 4096, "sum_of_max") == "generic"
    assert gb.gbnn_retrieve_path(1, 16, "sum_of_max") == ""


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(gb, "_lib", None)
    monkeypatch.setattr(gb, "_LIB_PATH", tmp_path / "missing.so")
    with pytest.raises(FileNotFoundError):
        gb.lib()


def test_reference_copy_argument_errors(lib):
    E = gb.ERRORS
    assert lib.gbnn_reference_copy(0, 0, 0, 0, 0) == 0                      # nothing to do
    assert lib.gbnn_reference_copy(0, 0x1000, 16, 0, 0) == E["NULL"]
    assert lib.gbnn_reference_copy(0x1000, 0, 16, 1, 0) == E["NULL"]
    assert lib.gbnn_reference_copy(0x1000, 0x2000, 24, 0, 0) == E["SHAPE"]  # not a multiple of 16
    assert lib.gbnn_reference_copy(0x1008, 0x2000, 32, 0, 0) == E["SHAPE"]  # alignment
    assert lib.gbnn_reference_copy(0x1000, 0x2004, 32, 1, 0) == E["SHAPE"]

