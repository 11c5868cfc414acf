"""Storing and retrieving in turn, a few messages at a time (the one-after-another use that Section
VII-C sets against batch decoding): gbnn_store_update keeps a prepared workspace in step with W, and a
captured HIP graph of store_update + retrieve replays correctly.  Everything is compared with the CPU
oracle, which stores the same messages incrementally and retrieves the same probes."""
import numpy as np
import pytest
import torch

from oracle import gbnn_oracle as orc
from paper_1303_7032_amd import binding as gb
from paper_1303_7032_amd import inputs

pytestmark = pytest.mark.gpu

RULES = ("sum_of_sum", "sum_of_max", "hybrid")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    gb.lib()


def table_regions(ws, C, L):
    """The defined bytes of a workspace: the table of (n + C + 2) rows and the word of flags."""
    nw = gb.gbnn_w_row_words(C, L)
    table = ws[: (C * L + C + 2) * nw * 4].cpu().numpy()
    flags = ws[ws.numel() - 256: ws.numel() - 248].cpu().numpy()
    return table, flags


@pytest.mark.parametrize("C,L,M0,M1", [(4, 16, 0, 40), (8, 128, 3000, 50), (8, 256, 0, 300), (5, 12, 30, 64),
                                       (16, 512, 2000, 20), (3, 3, 1, 5)])
def test_store_update_equals_store_then_prepare(C, L, M0, M1):
    msgs = inputs.make_messages(C, L, M0 + M1 + 2, 23)
    new = msgs[M0:].copy()
    new[1, 0] = L          # two messages with a bad symbol: skipped and reported
    new[M1 // 2, C - 1] = -1
    W = gb.new_network(C, L)
    if M0:
        gb.gbnn_store(W, C, L, torch.from_numpy(msgs[:M0].copy()).cuda())
    ws = gb.gbnn_prepare(W, C, L)       # also valid for the empty network
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    gb.gbnn_store_update(W, C, L, torch.from_numpy(new).cuda(), ws, status)
    gb.gbnn_store_update(W, C, L, torch.zeros((0, C), dtype=torch.int32, device="cuda"), ws)  # M = 0: no-op
    assert int(status.item()) == 1
    good = np.concatenate([msgs[:M0], new[(new >= 0).all(axis=1) & (new < L).all(axis=1)]])
    Wo, _ = orc.store(C, L, good)
    assert (W.cpu().numpy().view(np.uint32) == orc.pack_bits(Wo)).all()
    fresh = gb.gbnn_prepare(W, C, L)
    t0, f0 = table_regions(ws, C, L)
    t1, f1 = table_regions(fresh, C, L)
    assert (t0 == t1).all() and (f0 == f1).all()


@pytest.mark.parametrize("C,L", [(4, 16), (8, 128), (8, 256), (16, 512)])
def test_store_and_retrieve_in_turn(C, L):
    """Rounds of: store 1-3 messages, then retrieve 1-5 probes made from messages stored so far."""
    rng = np.random.default_rng(C * 1000 + L)
    msgs = inputs.make_messages(C, L, 120, 31)
    W = gb.new_network(C, L)
    ws = gb.gbnn_prepare(W, C, L)
    Wo = None
    stored = 0
    for step in range(30 if C * L <= 2048 else 9):
        add = int(rng.integers(1, 4))
        part = msgs[stored:stored + add]
        gb.gbnn_store_update(W, C, L, torch.from_numpy(part.copy()).cuda(), ws)
        Wo, _ = orc.store(C, L, part, Wo)
        stored += add
        K = int(rng.integers(1, 6))
        probes = msgs[rng.integers(0, stored, K)].copy()
        for k in range(K):
            probes[k, rng.choice(C, int(rng.integers(0, C)), replace=False)] = -1
        rule = RULES[step % 3]
        bits, sym, it = gb.gbnn_retrieve_symbols(W, C, L, torch.from_numpy(probes).cuda(), rule, 1, 20, workspace=ws)
        rbits, rsym, rit = orc.retrieve_symbols(Wo, C, L, probes, rule, 1, 20)
        assert (bits.cpu().numpy().view(np.uint32) == rbits).all(), (step, rule)
        assert (sym.cpu().numpy() == rsym).all() and (it.cpu().numpy() == rit).all(), (step, rule)
        V0 = orc.encode_probes(C, L, probes)
        out, it2 = gb.gbnn_retrieve(W, C, L, torch.from_numpy(V0).cuda(), rule, 1, 20, workspace=ws)
        ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, 1, 20)
        assert (out.cpu().numpy() == ref).all() and (it2.cpu().numpy() == itref).all(), (step, rule)


@pytest.mark.parametrize("C,L,rule", [(8, 256, "sum_of_max"), (8, 128, "sum_of_sum"), (16, 512, "hybrid")])
def test_graph_of_store_update_and_retrieve_replays(C, L, rule):
    """One captured graph = store 2 messages + retrieve 4 probes; replayed 6 times on fresh inputs with
    eager work and synchronisation in between, every replay checked against the oracle."""
    rng = np.random.default_rng(L + C)
    msgs = inputs.make_messages(C, L, 200, 37)
    nw = gb.gbnn_w_row_words(C, L)
    W = gb.new_network(C, L)
    gb.gbnn_store(W, C, L, torch.from_numpy(msgs[:100].copy()).cuda())
    ws = gb.gbnn_prepare(W, C, L)
    Wo, _ = orc.store(C, L, msgs[:100])
    new_d = torch.zeros((2, C), dtype=torch.int32, device="cuda")
    probes_d = torch.zeros((4, C), dtype=torch.int32, device="cuda")
    bits = torch.zeros((4, nw), dtype=torch.int32, device="cuda")
    sym = torch.zeros((4, C), dtype=torch.int32, device="cuda")
    it = torch.zeros(4, dtype=torch.int32, device="cuda")

    def one_round():
        gb.gbnn_store_update(W, C, L, new_d, ws)
        gb.gbnn_retrieve_symbols(W, C, L, probes_d, rule, 1, 20, bits_out=bits, symbols_out=sym, iters_out=it,
                                 workspace=ws)

    def fresh_inputs(r):
        new = msgs[100 + 2 * r: 102 + 2 * r].copy()
        probes = msgs[rng.integers(0, 100 + 2 * r + 2, 4)].copy()
        for k in range(4):
            probes[k, rng.choice(C, C // 2, replace=False)] = -1
        new_d.copy_(torch.from_numpy(new))
        probes_d.copy_(torch.from_numpy(probes))
        return new, probes

    side = torch.cuda.Stream()
    new, probes = fresh_inputs(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        one_round()                      # warm-up on the capture stream (also round 0 of the data)
    side.synchronize()
    Wo, _ = orc.store(C, L, new, Wo)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_round()
    for r in range(1, 7):
        new, probes = fresh_inputs(r)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        Wo, _ = orc.store(C, L, new, Wo)
        rbits, rsym, rit = orc.retrieve_symbols(Wo, C, L, probes, rule, 1, 20)
        assert (bits.cpu().numpy().view(np.uint32) == rbits).all(), r
        assert (sym.cpu().numpy() == rsym).all() and (it.cpu().numpy() == rit).all(), r
        # eager work between replays: the same retrieval outside the graph gives the same answer
        b2, s2, i2 = gb.gbnn_retrieve_symbols(W, C, L, probes_d, rule, 1, 20, workspace=ws)
        assert torch.equal(b2, bits) and torch.equal(s2, sym) and torch.equal(i2, it)
    assert (W.cpu().numpy().view(np.uint32) == orc.pack_bits(Wo)).all()
