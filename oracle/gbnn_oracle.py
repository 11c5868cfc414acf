"""ctypes front end of the plain C oracle (oracle/gbnn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  Nothing in the product package imports it, and it imports nothing from
the product package.  All arrays are numpy, on the host; W is the full byte matrix
uint8[n][n] (W[j, i] = w_ji), activity is uint8[K][n].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "gbnn_oracle.c"
_LIB = _HERE / "libgbnn_oracle.so"

RULES = {"sum_of_sum": 0, "sum_of_max": 1, "hybrid": 2, "sum_of_max_eq": 3}


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (a second or two)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               str(_SRC), "-o", str(_LIB)]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        u8p, i32p = ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_int32)
        ci, i64 = ctypes.c_int, ctypes.c_int64
        L.gbnn_oracle_store.restype = i64
        L.gbnn_oracle_store.argtypes = [u8p, ci, ci, i32p, i64]
        L.gbnn_oracle_sos_scores.restype = None
        L.gbnn_oracle_sos_scores.argtypes = [u8p, ci, ci, u8p, ci, i32p]
        L.gbnn_oracle_sos_select.restype = None
        L.gbnn_oracle_sos_select.argtypes = [i32p, ci, ci, u8p]
        L.gbnn_oracle_som_init.restype = None
        L.gbnn_oracle_som_init.argtypes = [ci, ci, u8p]
        L.gbnn_oracle_som_scores_eq.restype = None
        L.gbnn_oracle_som_scores_eq.argtypes = [u8p, ci, ci, u8p, ci, i32p]
        L.gbnn_oracle_som_pass_eq.restype = None
        L.gbnn_oracle_som_pass_eq.argtypes = [u8p, ci, ci, u8p, ci, u8p]
        L.gbnn_oracle_som_pass_boe.restype = None
        L.gbnn_oracle_som_pass_boe.argtypes = [u8p, ci, ci, u8p, u8p, u8p]
        L.gbnn_oracle_retrieve.restype = ci
        L.gbnn_oracle_retrieve.argtypes = [u8p, ci, ci, u8p, u8p, i64, ci, ci, ci, i32p, ci]
        _lib = L
    return _lib


def _u8(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _i32(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def store(C: int, L: int, msgs: np.ndarray, W: np.ndarray | None = None):
    """OR the cliques of msgs (int32[M][C]) into W (fresh zero matrix if None).
    Returns (W uint8[n][n], number of skipped out-of-range messages)."""
    n = C * L
    if W is None:
        W = np.zeros((n, n), dtype=np.uint8)
    assert W.shape == (n, n) and W.dtype == np.uint8 and W.flags.c_contiguous
    msgs = np.ascontiguousarray(msgs, dtype=np.int32).reshape(-1, C)
    skipped = lib().gbnn_oracle_store(_u8(W), C, L, _i32(msgs), msgs.shape[0])
    return W, int(skipped)


def sos_scores(W, C, L, v, gamma):
    v = np.ascontiguousarray(v, dtype=np.uint8)
    s = np.zeros(C * L, dtype=np.int32)
    lib().gbnn_oracle_sos_scores(_u8(W), C, L, _u8(v), gamma, _i32(s))
    return s


def sos_select(s, C, L):
    s = np.ascontiguousarray(s, dtype=np.int32)
    v = np.zeros(C * L, dtype=np.uint8)
    lib().gbnn_oracle_sos_select(_i32(s), C, L, _u8(v))
    return v


def som_init(C, L, v):
    v = np.array(v, dtype=np.uint8, copy=True)
    lib().gbnn_oracle_som_init(C, L, _u8(v))
    return v


def som_scores_eq(W, C, L, v, gamma):
    v = np.ascontiguousarray(v, dtype=np.uint8)
    s = np.zeros(C * L, dtype=np.int32)
    lib().gbnn_oracle_som_scores_eq(_u8(W), C, L, _u8(v), gamma, _i32(s))
    return s


def som_pass_eq(W, C, L, v, gamma):
    v = np.ascontiguousarray(v, dtype=np.uint8)
    out = np.zeros(C * L, dtype=np.uint8)
    lib().gbnn_oracle_som_pass_eq(_u8(W), C, L, _u8(v), gamma, _u8(out))
    return out


def som_pass_boe(W, C, L, v, update_cluster=None):
    v = np.ascontiguousarray(v, dtype=np.uint8)
    out = np.zeros(C * L, dtype=np.uint8)
    uc = None
    if update_cluster is not None:
        uc_arr = np.ascontiguousarray(update_cluster, dtype=np.uint8)
        uc = _u8(uc_arr)
    lib().gbnn_oracle_som_pass_boe(_u8(W), C, L, _u8(v), _u8(out), uc)
    return out


def retrieve(W, C, L, V0, rule, gamma=1, max_iters=20, nthreads=0):
    """Retrieve K probes.  rule is a name from RULES.  Returns (V_out uint8[K][n],
    iters int32[K] (+p converged at pass p, -max_iters cap reached), threads used)."""
    n = C * L
    V0 = np.ascontiguousarray(V0, dtype=np.uint8).reshape(-1, n)
    K = V0.shape[0]
    assert W.shape == (n, n) and W.dtype == np.uint8 and W.flags.c_contiguous
    out = np.zeros_like(V0)
    iters = np.zeros(K, dtype=np.int32)
    if nthreads <= 0:
        nthreads = int(os.environ.get("OMP_NUM_THREADS", 0)) or (os.cpu_count() or 1)
    used = lib().gbnn_oracle_retrieve(_u8(W), C, L, _u8(V0), _u8(out), K, RULES[rule], gamma, max_iters,
                                      _i32(iters), nthreads)
    return out, iters, int(used)


def error_rate(V_out: np.ndarray, target_onehot: np.ndarray) -> float:
    """Fraction of probes whose final activity is not exactly the one-hot code of the
    message they were made from (retrieval rate of Section VII = 1 - this)."""
    ok = (V_out == target_onehot).all(axis=1)
    return 1.0 - float(ok.mean()) if len(ok) else 0.0


def pack_bits(Wfull: np.ndarray) -> np.ndarray:
    """Byte matrix -> the boundary's bit-packed layout uint32[n][ceil(n/32)] (bit j%32 of
    word j//32 of row i is W[i, j], least significant bit first).  Used only to compare a
    packed W coming from elsewhere with the oracle's."""
    n = Wfull.shape[0]
    nw = (n + 31) // 32
    padded = np.zeros((n, nw * 32), dtype=np.uint8)
    padded[:, :n] = Wfull
    b = np.packbits(padded.reshape(n, nw, 32), axis=2, bitorder="little")  # [n][nw][4] bytes, LSB first
    return b.view("<u4").reshape(n, nw)


# ------------------------------------------------------------------ symbols in, symbols / packed bits out
SYM_NONE, SYM_AMBIGUOUS = -1, -2


def encode_probes(C: int, L: int, probes: np.ndarray) -> np.ndarray:
    """Partially erased messages -> activity vectors (Section II-A: a message activates the neuron
    of its symbol in every cluster; an erased cluster has no active neuron).  probes is
    int32[K][C] with 0-based symbols; any entry outside [0, L) (-1 by convention) marks the
    cluster as erased.  Plain loops: this is the definition."""
    probes = np.asarray(probes, dtype=np.int64).reshape(-1, C)
    V = np.zeros((probes.shape[0], C * L), dtype=np.uint8)
    for k in range(probes.shape[0]):
        for c in range(C):
            s = int(probes[k, c])
            if 0 <= s < L:
                V[k, c * L + s] = 1
    return V


def decode(C: int, L: int, V: np.ndarray):
    """Activity vectors -> (packed bits uint32[K][ceil(n/32)], symbols int32[K][C]).  Bit i%32 of
    word i//32 is neuron i, least significant bit first.  The symbol of a cluster is the index of
    its active neuron if it has exactly one, SYM_NONE if it has none, SYM_AMBIGUOUS if it has
    several (Section V-B: several cliques may survive)."""
    V = np.asarray(V, dtype=np.uint8).reshape(-1, C * L)
    K, n = V.shape
    nw = (n + 31) // 32
    bits = np.zeros((K, nw), dtype=np.uint32)
    sym = np.zeros((K, C), dtype=np.int32)
    for k in range(K):
        for i in np.nonzero(V[k])[0]:
            bits[k, i // 32] |= np.uint32(1) << np.uint32(i % 32)
        for c in range(C):
            on = np.nonzero(V[k, c * L:(c + 1) * L])[0]
            sym[k, c] = int(on[0]) if len(on) == 1 else (SYM_NONE if len(on) == 0 else SYM_AMBIGUOUS)
    return bits, sym


def retrieve_symbols(W, C, L, probes, rule, gamma=1, max_iters=20, nthreads=0):
    """The retrieval of `retrieve` with messages at the boundary: encode, retrieve, decode.
    Returns (bits, symbols, iters)."""
    out, iters, _ = retrieve(W, C, L, encode_probes(C, L, probes), rule, gamma, max_iters, nthreads)
    bits, sym = decode(C, L, out)
    return bits, sym, iters


# ------------------------------------------------------------------ sparse W' (Section IV-B, "Sparsification")
def sparsify(W: np.ndarray):
    """W -> W': only the nonzero elements and their coordinates, row by row.  Returns
    (offsets int64[n+1], cols int64[nnz]): the neighbours of neuron i are cols[offsets[i]:offsets[i+1]],
    in ascending order."""
    n = W.shape[0]
    offsets = np.zeros(n + 1, dtype=np.int64)
    cols = []
    for i in range(n):
        nz = np.nonzero(W[i])[0]
        cols.append(nz)
        offsets[i + 1] = offsets[i] + len(nz)
    return offsets, (np.concatenate(cols) if cols else np.zeros(0, dtype=np.int64)).astype(np.int64)


def som_pass_lists(C: int, L: int, offsets: np.ndarray, cols: np.ndarray, v: np.ndarray) -> np.ndarray:
    """One sum-of-max pass (Eq. 6-7 with gamma = 1) computed from W' alone: an active neuron stays on
    iff each of the C-1 other clusters holds an active neuron of its neighbour list."""
    n = C * L
    out = np.zeros(n, dtype=np.uint8)
    for i in range(n):
        if not v[i]:
            continue
        seen = np.zeros(C, dtype=bool)
        for j in cols[offsets[i]:offsets[i + 1]]:
            if v[j]:
                seen[j // L] = True
        seen[i // L] = True
        out[i] = 1 if seen.all() else 0
    return out
