"""Sparse W' (Section IV-B, "Sparsification") on the GPU: gbnn_sparsify against the oracle's neighbour
lists, and sum-of-max retrieval from W' against the oracle's sum-of-max on the dense W (the two must
agree bit for bit: W' loses nothing)."""
import numpy as np
import pytest
import torch

from oracle import gbnn_oracle as orc
from paper_1303_7032_amd import binding as gb
from paper_1303_7032_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    gb.lib()


def parts(Wp, C, L, nnz):
    """offsets, summary rows, flags and cols of a W' buffer, as numpy arrays."""
    n, nw = C * L, gb.gbnn_w_row_words(C, L)
    raw = Wp.cpu().numpy()
    up = lambda x: (x + 255) // 256 * 256
    o_sum = up((n + 1) * 4)
    o_full = o_sum + up(C * nw * 4)
    o_cols = o_full + 256
    offsets = raw[: (n + 1) * 4].view(np.uint32)
    summary = raw[o_sum: o_sum + C * nw * 4].view(np.uint32).reshape(C, nw)
    flags = int(raw[o_full: o_full + 8].view(np.uint64)[0])
    cols = raw[o_cols: o_cols + nnz * 2].view(np.uint16)
    return offsets, summary, flags, cols


def network(C, L, M, seed):
    msgs = inputs.make_messages(C, L, M, seed) if M else np.zeros((0, C), dtype=np.int32)
    Wo, _ = orc.store(C, L, msgs)
    W = gb.new_network(C, L)
    if M:
        gb.gbnn_store(W, C, L, torch.from_numpy(msgs).cuda())
    return msgs, Wo, W


@pytest.mark.parametrize("C,L,M", [(4, 32, 100), (2, 32, 5), (3, 64, 50), (8, 128, 5000), (8, 256, 20000),
                                   (16, 512, 3000), (5, 96, 0), (64, 32, 400), (2, 8192, 3000)])
def test_sparsify_bit_exact(C, L, M):
    msgs, Wo, W = network(C, L, M, 41)
    off_ref, cols_ref = orc.sparsify(Wo)
    nnz = gb.gbnn_sparse_count(W, C, L)
    assert nnz == len(cols_ref) == int(Wo.sum())
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    Wp = gb.gbnn_sparsify(W, C, L, status=status)
    assert Wp.numel() == gb.gbnn_sparse_bytes(C, L, nnz) and int(status.item()) == 0
    offsets, summary, flags, cols = parts(Wp, C, L, nnz)
    assert (offsets == off_ref).all() and (cols == cols_ref).all()
    # summary row c, bit i: i is in c or has a neighbour in c -- from the definition, on the oracle's W
    n = C * L
    has = Wo.reshape(n, C, L).any(axis=2)
    has[np.arange(n), np.arange(n) // L] = True
    packed = np.ascontiguousarray(np.packbits(has.T.astype(np.uint8), axis=1, bitorder="little")).view("<u4")
    assert (summary == packed).all()
    assert flags == sum(1 << c for c in range(C) if has[:, c].all())


def test_sparsify_reports_a_buffer_that_is_too_small():
    C, L, M = 8, 128, 3000
    msgs, Wo, W = network(C, L, M, 43)
    nnz = int(Wo.sum())
    small = torch.zeros(gb.gbnn_sparse_bytes(C, L, nnz - 1000), dtype=torch.uint8, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    gb.gbnn_sparsify(W, C, L, small, status)
    assert int(status.item()) == 1
    room = (small.numel() - gb.gbnn_sparse_bytes(C, L, 0)) // 2
    offsets, _, _, cols = parts(small, C, L, room)
    off_ref, cols_ref = orc.sparsify(Wo)
    assert (offsets == off_ref).all() and (cols == cols_ref[:room]).all()   # what fits is right, nothing beyond is written


def make_probes(msgs, C, L, K, e, seed, wrong_every=0):
    rng = np.random.default_rng(seed)
    q, er = inputs.make_probe_plan(C, len(msgs), K, e, seed)
    probes = msgs[q].copy()
    probes[er] = -1
    if wrong_every:
        for k in range(0, K, wrong_every):
            probes[k, int(rng.integers(C))] = int(rng.integers(-3, L + 3))   # a wrong or out-of-range symbol
    return probes


def check(Wp, Wo, C, L, probes, cap):
    bits, sym, it = gb.gbnn_retrieve_sparse(Wp, C, L, torch.from_numpy(probes).cuda(), cap)
    rbits, rsym, rit = orc.retrieve_symbols(Wo, C, L, probes, "sum_of_max", 1, cap)
    got = bits.cpu().numpy().view(np.uint32)
    bad = np.nonzero((got != rbits).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} probes differ, first {bad[:5]}"
    assert (sym.cpu().numpy() == rsym).all()
    badi = np.nonzero(it.cpu().numpy() != rit)[0]
    assert badi.size == 0, f"iters differ at {badi[:5]}"


@pytest.mark.parametrize("C,L,M,K", [(4, 32, 100, 257), (8, 128, 5000, 700), (8, 256, 20000, 513), (3, 64, 50, 130),
                                     (16, 512, 3000, 200), (16, 512, 100000, 64), (64, 32, 400, 100),
                                     (8, 256, 200, 300)])
def test_retrieval_from_the_lists(C, L, M, K):
    msgs, Wo, W = network(C, L, M, 47)
    Wp = gb.gbnn_sparsify(W, C, L)
    for e in sorted({0, 1, C // 2, C - 1, C}):
        for cap in (1, 2, 20):
            check(Wp, Wo, C, L, make_probes(msgs, C, L, K, e, 100 * e + cap, wrong_every=3), cap)
    gb.gbnn_retrieve_sparse(Wp, C, L, torch.zeros((0, C), dtype=torch.int32, device="cuda"))   # K = 0


def test_empty_network_and_dying_clusters():
    C, L = 4, 64
    msgs, Wo, W = network(C, L, 0, 1)
    Wp = gb.gbnn_sparsify(W, C, L)
    probes = np.array([[1, 2, 3, 4], [-1, -1, -1, -1], [5, -1, -1, 7]], dtype=np.int32)
    check(Wp, Wo, C, L, probes, 20)
    # a sparse network where most probes lose a whole cluster after a pass or two
    msgs, Wo, W = network(6, 64, 40, 3)
    Wp = gb.gbnn_sparsify(W, 6, 64)
    rng = np.random.default_rng(0)
    probes = rng.integers(-1, 64, size=(400, 6)).astype(np.int32)
    probes[::2, :3] = msgs[rng.integers(0, 40, 200), :3]
    for cap in (1, 2, 3, 20):
        check(Wp, Wo, 6, 64, probes, cap)


def test_largest_network_low_density():
    """n = 16384 (the interface's limit), d about 0.01: the regime W' is meant for."""
    C, L, M, K = 8, 2048, 40000, 48
    msgs, Wo, W = network(C, L, M, 53)
    Wp = gb.gbnn_sparsify(W, C, L)
    check(Wp, Wo, C, L, make_probes(msgs, C, L, K, 4, 5, wrong_every=7), 20)
    check(Wp, Wo, C, L, make_probes(msgs, C, L, 16, 7, 6), 20)


@pytest.mark.parametrize("name", ["cfg3", "cfg5"])
def test_full_configurations_sampled_against_the_oracle_and_whole_against_the_packed_kernels(name):
    w = inputs.WORKLOADS[name]
    msgs = w.messages()
    Wo, _ = orc.store(w.C, w.L, msgs)
    W = gb.new_network(w.C, w.L)
    gb.gbnn_store(W, w.C, w.L, torch.from_numpy(msgs).cuda())
    Wp = gb.gbnn_sparsify(W, w.C, w.L)
    q, er = w.probe_plan()
    probes = msgs[q].copy()
    probes[er] = -1
    pd = torch.from_numpy(probes).cuda()
    bits, sym, it = gb.gbnn_retrieve_sparse(Wp, w.C, w.L, pd, 20)
    pick = np.random.default_rng(1).choice(w.K, 256, replace=False)
    rbits, rsym, rit = orc.retrieve_symbols(Wo, w.C, w.L, probes[pick], "sum_of_max", 1, 20)
    assert (bits.cpu().numpy().view(np.uint32)[pick] == rbits).all()
    assert (sym.cpu().numpy()[pick] == rsym).all() and (it.cpu().numpy()[pick] == rit).all()
    b2, s2, i2 = gb.gbnn_retrieve_symbols(W, w.C, w.L, pd, "sum_of_max", 1, 20)   # property at full size: same as the packed path
    assert torch.equal(bits, b2) and torch.equal(sym, s2) and torch.equal(it, i2)
