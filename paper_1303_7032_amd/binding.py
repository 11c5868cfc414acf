"""Thin Python binding of the C ABI in include/gbnn.h (argument marshalling only).

Every step of storing and retrieval runs in the HIP kernels of libgbnn_hip.so; torch is
used for device memory and streams.  There is no CPU fallback: if the library has not been
built (python -m paper_1303_7032_amd.build) loading fails with an error.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libgbnn_hip.so"
_lib = None

SUM_OF_SUM, SUM_OF_MAX, HYBRID = 0, 1, 2
RULES = {"sum_of_sum": SUM_OF_SUM, "sum_of_max": SUM_OF_MAX, "hybrid": HYBRID}

GBNN_OK = 0
ERRORS = {"NULL": -1, "SHAPE": -2, "RULE": -3, "GAMMA": -4, "ITERS": -5, "WORKSPACE": -6, "DEVICE": -7,
          "TOO_LARGE": -8}


class GbnnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"gbnn status {code}: {message}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Load libgbnn_hip.so (once).  Raises if it is not built."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_1303_7032_amd.build` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(str(_LIB_PATH))
        vp, ci, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.gbnn_w_row_words.restype = sz
        L.gbnn_w_row_words.argtypes = [ci, ci]
        L.gbnn_w_bytes.restype = sz
        L.gbnn_w_bytes.argtypes = [ci, ci]
        L.gbnn_workspace_bytes.restype = sz
        L.gbnn_workspace_bytes.argtypes = [ci, ci, i64, ci]
        L.gbnn_store.restype = ci
        L.gbnn_store.argtypes = [vp, ci, ci, vp, i64, vp, vp]
        L.gbnn_prepare.restype = ci
        L.gbnn_prepare.argtypes = [vp, ci, ci, vp, sz, vp]
        L.gbnn_store_update.restype = ci
        L.gbnn_store_update.argtypes = [vp, ci, ci, vp, i64, vp, vp, sz, vp]
        L.gbnn_retrieve.restype = ci
        L.gbnn_retrieve.argtypes = [vp, ci, ci, vp, vp, i64, ci, ci, ci, vp, vp, sz, vp]
        L.gbnn_retrieve_static.restype = ci
        L.gbnn_retrieve_static.argtypes = [vp, ci, ci, vp, vp, i64, ci, ci, ci, vp, vp]
        L.gbnn_retrieve_symbols.restype = ci
        L.gbnn_retrieve_symbols.argtypes = [vp, ci, ci, vp, i64, ci, ci, ci, vp, vp, vp, vp, sz, vp]
        L.gbnn_sparse_bytes.restype = sz
        L.gbnn_sparse_bytes.argtypes = [ci, ci, i64]
        L.gbnn_sparse_count.restype = ci
        L.gbnn_sparse_count.argtypes = [vp, ci, ci, vp, vp]
        L.gbnn_sparsify.restype = ci
        L.gbnn_sparsify.argtypes = [vp, ci, ci, vp, sz, vp, vp]
        L.gbnn_retrieve_sparse.restype = ci
        L.gbnn_retrieve_sparse.argtypes = [vp, sz, ci, ci, vp, i64, ci, vp, vp, vp, vp]
        L.gbnn_strerror.restype = ctypes.c_char_p
        L.gbnn_strerror.argtypes = [ci]
        L.gbnn_retrieve_path.restype = ctypes.c_char_p
        L.gbnn_retrieve_path.argtypes = [ci, ci, ci, vp, vp]
        L.gbnn_set_kernel_choice.restype = ci
        L.gbnn_set_kernel_choice.argtypes = [ci, ci]
        L.gbnn_reference_copy.restype = ci
        L.gbnn_reference_copy.argtypes = [vp, vp, sz, ci, vp]
        _lib = L
    return _lib


def _check(code: int) -> None:
    if code != GBNN_OK:
        raise GbnnError(code, lib().gbnn_strerror(code).decode())


def _rule(rule) -> int:
    return RULES[rule] if isinstance(rule, str) else int(rule)


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> None:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous {dtype} tensor on the GPU")


def gbnn_w_row_words(C: int, L: int) -> int:
    return int(lib().gbnn_w_row_words(C, L))


def gbnn_w_bytes(C: int, L: int) -> int:
    return int(lib().gbnn_w_bytes(C, L))


def gbnn_workspace_bytes(C: int, L: int, K: int, rule) -> int:
    return int(lib().gbnn_workspace_bytes(C, L, K, _rule(rule)))


def gbnn_strerror(code: int) -> str:
    return lib().gbnn_strerror(code).decode()


def new_network(C: int, L: int, device="cuda") -> torch.Tensor:
    """An empty (all-zero) W in the canonical layout: int32[n][ceil(n/32)] on the device."""
    nw = gbnn_w_row_words(C, L)
    if nw == 0:
        _check(ERRORS["SHAPE"])
    return torch.zeros((C * L, nw), dtype=torch.int32, device=device)


def gbnn_store(W: torch.Tensor, C: int, L: int, msgs: torch.Tensor, status: torch.Tensor | None = None) -> None:
    """OR the cliques of msgs (int32[M][C] on the device) into W (enqueued on the current stream)."""
    _dev(W, torch.int32, "W")
    _dev(msgs, torch.int32, "msgs")
    if W.numel() * 4 != gbnn_w_bytes(C, L) or msgs.numel() % C:
        _check(ERRORS["SHAPE"])
    st = 0
    if status is not None:
        _dev(status, torch.int32, "status")
        st = status.data_ptr()
    M = msgs.numel() // C
    _check(lib().gbnn_store(W.data_ptr(), C, L, msgs.data_ptr() if M else 0, M, st, _stream(W)))


def gbnn_store_update(W: torch.Tensor, C: int, L: int, msgs: torch.Tensor, workspace: torch.Tensor,
                      status: torch.Tensor | None = None) -> None:
    """gbnn_store into W and into the workspace prepared for it, so that retrieval can follow at once."""
    _dev(W, torch.int32, "W")
    _dev(msgs, torch.int32, "msgs")
    _dev(workspace, torch.uint8, "workspace")
    if W.numel() * 4 != gbnn_w_bytes(C, L) or msgs.numel() % C:
        _check(ERRORS["SHAPE"])
    st = 0
    if status is not None:
        _dev(status, torch.int32, "status")
        st = status.data_ptr()
    M = msgs.numel() // C
    _check(lib().gbnn_store_update(W.data_ptr(), C, L, msgs.data_ptr() if M else 0, M, st, workspace.data_ptr(),
                                   workspace.numel(), _stream(W)))


def gbnn_prepare(W: torch.Tensor, C: int, L: int, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Fill (and, if not supplied, allocate) the workspace gbnn_retrieve reads: derived tables of W.
    Call again whenever W changes.  Returns the workspace (a uint8 tensor on W's device)."""
    _dev(W, torch.int32, "W")
    if W.numel() * 4 != gbnn_w_bytes(C, L):
        _check(ERRORS["SHAPE"])
    if workspace is None:
        workspace = torch.empty(gbnn_workspace_bytes(C, L, 0, SUM_OF_MAX), dtype=torch.uint8, device=W.device)
    _dev(workspace, torch.uint8, "workspace")
    _check(lib().gbnn_prepare(W.data_ptr(), C, L, workspace.data_ptr(), workspace.numel(), _stream(W)))
    return workspace


def gbnn_retrieve(W: torch.Tensor, C: int, L: int, V0: torch.Tensor, rule, gamma: int = 1, max_iters: int = 20,
                  V_out: torch.Tensor | None = None, iters_out: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None, want_iters: bool = True):
    """Retrieve the K probes of V0 (uint8[K][n]).  Returns (V_out, iters_out).

    `workspace` is what gbnn_prepare returned for this W; if it is None it is built here (one
    more pass over W per call: pass it in when retrieving repeatedly).  Output tensors are
    allocated with torch when not supplied.  Work is enqueued on the current stream.
    """
    r = _rule(rule)
    _dev(W, torch.int32, "W")
    _dev(V0, torch.uint8, "V0")
    n = C * L
    if W.numel() * 4 != gbnn_w_bytes(C, L) or V0.numel() % n:
        _check(ERRORS["SHAPE"])
    K = V0.numel() // n
    if V_out is None:
        V_out = torch.empty_like(V0)
    _dev(V_out, torch.uint8, "V_out")
    if V_out.numel() != V0.numel():
        _check(ERRORS["SHAPE"])
    if iters_out is None and want_iters:
        iters_out = torch.empty(K, dtype=torch.int32, device=V0.device)
    if iters_out is not None:
        _dev(iters_out, torch.int32, "iters_out")
        if iters_out.numel() != K:
            _check(ERRORS["SHAPE"])
    if workspace is None:
        workspace = gbnn_prepare(W, C, L)
    _dev(workspace, torch.uint8, "workspace")
    _check(lib().gbnn_retrieve(W.data_ptr(), C, L, V0.data_ptr() if K else 0, V_out.data_ptr() if K else 0, K, r,
                               gamma, max_iters, iters_out.data_ptr() if iters_out is not None else 0,
                               workspace.data_ptr(), workspace.numel(), _stream(V0)))
    return V_out, iters_out


def gbnn_retrieve_static(W: torch.Tensor, C: int, L: int, V0: torch.Tensor, rule, gamma: int, max_iters: int,
                         V_out: torch.Tensor, iters_out: torch.Tensor | None = None) -> None:
    """gbnn_retrieve without a workspace (the library's own static device array holds the prepared table);
    nothing is allocated here either: the caller passes every output."""
    _dev(W, torch.int32, "W")
    _dev(V0, torch.uint8, "V0")
    _dev(V_out, torch.uint8, "V_out")
    n = C * L
    if W.numel() * 4 != gbnn_w_bytes(C, L) or V0.numel() % n or V_out.numel() != V0.numel():
        _check(ERRORS["SHAPE"])
    K = V0.numel() // n
    it = 0
    if iters_out is not None:
        _dev(iters_out, torch.int32, "iters_out")
        if iters_out.numel() != K:
            _check(ERRORS["SHAPE"])
        it = iters_out.data_ptr()
    _check(lib().gbnn_retrieve_static(W.data_ptr(), C, L, V0.data_ptr() if K else 0, V_out.data_ptr() if K else 0, K,
                                      _rule(rule), gamma, max_iters, it, _stream(V0)))


SYM_NONE, SYM_AMBIGUOUS = -1, -2


def gbnn_retrieve_symbols(W: torch.Tensor, C: int, L: int, probes: torch.Tensor, rule, gamma: int = 1,
                          max_iters: int = 20, bits_out: torch.Tensor | None = None,
                          symbols_out: torch.Tensor | None = None, iters_out: torch.Tensor | None = None,
                          workspace: torch.Tensor | None = None, want_bits: bool = True, want_symbols: bool = True,
                          want_iters: bool = True):
    """Retrieve the K partially erased messages of probes (int32[K][C], -1 = erased).
    Returns (bits_out int32[K][nw] or None, symbols_out int32[K][C] or None, iters_out or None);
    outputs not supplied are allocated with torch unless switched off by the want_* flags."""
    r = _rule(rule)
    _dev(W, torch.int32, "W")
    _dev(probes, torch.int32, "probes")
    if W.numel() * 4 != gbnn_w_bytes(C, L) or probes.numel() % C:
        _check(ERRORS["SHAPE"])
    K = probes.numel() // C
    nw = gbnn_w_row_words(C, L)
    if bits_out is None and want_bits:
        bits_out = torch.empty((K, nw), dtype=torch.int32, device=probes.device)
    if symbols_out is None and want_symbols:
        symbols_out = torch.empty((K, C), dtype=torch.int32, device=probes.device)
    if iters_out is None and want_iters:
        iters_out = torch.empty(K, dtype=torch.int32, device=probes.device)
    for t, cnt, name in ((bits_out, K * nw, "bits_out"), (symbols_out, K * C, "symbols_out"), (iters_out, K, "iters_out")):
        if t is not None:
            _dev(t, torch.int32, name)
            if t.numel() != cnt:
                _check(ERRORS["SHAPE"])
    if workspace is None:
        workspace = gbnn_prepare(W, C, L)
    _dev(workspace, torch.uint8, "workspace")
    ptr = lambda t: t.data_ptr() if (t is not None and K) else 0
    _check(lib().gbnn_retrieve_symbols(W.data_ptr(), C, L, ptr(probes), K, r, gamma, max_iters, ptr(bits_out),
                                       ptr(symbols_out), ptr(iters_out), workspace.data_ptr(), workspace.numel(),
                                       _stream(probes)))
    return bits_out, symbols_out, iters_out


def gbnn_retrieve_path(C: int, L: int, rule, V0: torch.Tensor | None = None, V_out: torch.Tensor | None = None) -> str:
    p = lib().gbnn_retrieve_path(C, L, _rule(rule), V0.data_ptr() if V0 is not None else 0,
                                 V_out.data_ptr() if V_out is not None else 0)
    return p.decode() if p else ""


FAMILIES = {"auto": 0, "generic": 1, "wave": 2}
STORE_KERNELS = {"auto": 0, "atomic": 1, "rows": 2}


def gbnn_set_kernel_choice(retrieve_family="auto", store_kernel="auto") -> None:
    """Tests and A/B timing: the kernel that serves the following calls (process-wide; "auto" = the library's choice)."""
    f = FAMILIES[retrieve_family] if isinstance(retrieve_family, str) else int(retrieve_family)
    k = STORE_KERNELS[store_kernel] if isinstance(store_kernel, str) else int(store_kernel)
    _check(lib().gbnn_set_kernel_choice(f, k))


def gbnn_sparse_bytes(C: int, L: int, nnz: int) -> int:
    return int(lib().gbnn_sparse_bytes(C, L, nnz))


def gbnn_sparse_count(W: torch.Tensor, C: int, L: int) -> int:
    """Number of nonzero elements of W (synchronises: the count is read back)."""
    _dev(W, torch.int32, "W")
    if W.numel() * 4 != gbnn_w_bytes(C, L):
        _check(ERRORS["SHAPE"])
    out = torch.empty(1, dtype=torch.int64, device=W.device)
    _check(lib().gbnn_sparse_count(W.data_ptr(), C, L, out.data_ptr(), _stream(W)))
    return int(out.item())


def gbnn_sparsify(W: torch.Tensor, C: int, L: int, Wp: torch.Tensor | None = None,
                  status: torch.Tensor | None = None) -> torch.Tensor:
    """Fill (and, if not supplied, size and allocate) the sparse form W' of W; returns it (uint8 tensor)."""
    _dev(W, torch.int32, "W")
    if W.numel() * 4 != gbnn_w_bytes(C, L):
        _check(ERRORS["SHAPE"])
    if Wp is None:
        need = gbnn_sparse_bytes(C, L, gbnn_sparse_count(W, C, L))
        if need == 0:
            _check(ERRORS["SHAPE"])
        Wp = torch.empty(need, dtype=torch.uint8, device=W.device)
    _dev(Wp, torch.uint8, "Wp")
    st = 0
    if status is not None:
        _dev(status, torch.int32, "status")
        st = status.data_ptr()
    _check(lib().gbnn_sparsify(W.data_ptr(), C, L, Wp.data_ptr(), Wp.numel(), st, _stream(W)))
    return Wp


def gbnn_retrieve_sparse(Wp: torch.Tensor, C: int, L: int, probes: torch.Tensor, max_iters: int = 20,
                         bits_out: torch.Tensor | None = None, symbols_out: torch.Tensor | None = None,
                         iters_out: torch.Tensor | None = None):
    """Sum-of-max retrieval of probes (int32[K][C], -1 = erased) from the sparse W'.
    Returns (bits_out int32[K][nw], symbols_out int32[K][C], iters_out int32[K])."""
    _dev(Wp, torch.uint8, "Wp")
    _dev(probes, torch.int32, "probes")
    if probes.numel() % C:
        _check(ERRORS["SHAPE"])
    K = probes.numel() // C
    nw = gbnn_w_row_words(C, L)
    if bits_out is None:
        bits_out = torch.empty((K, nw), dtype=torch.int32, device=probes.device)
    if symbols_out is None:
        symbols_out = torch.empty((K, C), dtype=torch.int32, device=probes.device)
    if iters_out is None:
        iters_out = torch.empty(K, dtype=torch.int32, device=probes.device)
    for t, cnt, name in ((bits_out, K * nw, "bits_out"), (symbols_out, K * C, "symbols_out"), (iters_out, K, "iters_out")):
        _dev(t, torch.int32, name)
        if t.numel() != cnt:
            _check(ERRORS["SHAPE"])
    _check(lib().gbnn_retrieve_sparse(Wp.data_ptr(), Wp.numel(), C, L, probes.data_ptr() if K else 0, K, max_iters,
                                      bits_out.data_ptr() if K else 0, symbols_out.data_ptr() if K else 0,
                                      iters_out.data_ptr() if K else 0, _stream(Wp)))
    return bits_out, symbols_out, iters_out


def gbnn_reference_copy(dst: torch.Tensor, src: torch.Tensor, streaming: bool) -> None:
    """dst <- src (same number of bytes, a multiple of 16) by the library's reference copy kernel."""
    for t, name in ((dst, "dst"), (src, "src")):
        if not (t.is_cuda and t.is_contiguous()):
            raise TypeError(f"{name} must be a contiguous tensor on the GPU")
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src differ in size")
    _check(lib().gbnn_reference_copy(dst.data_ptr(), src.data_ptr(), nbytes, 1 if streaming else 0, _stream(src)))

