"""The seeded input generator: determinism, ranges, and the paper's index convention."""
import numpy as np

from paper_1303_7032_amd import inputs
from conftest import read_golden


def test_rnd_is_a_pure_function():
    a = inputs.rnd(7, 0, np.arange(1000))
    b = inputs.rnd(7, 0, np.arange(1000))
    assert (a == b).all()
    assert (inputs.rnd(7, 1, np.arange(1000)) != a).any()
    assert (inputs.rnd(8, 0, np.arange(1000)) != a).any()
    # a subrange gives the same values: index-addressable
    assert (inputs.rnd(7, 0, np.arange(500, 600)) == a[500:600]).all()


def test_messages_uniform_in_range():
    m = inputs.make_messages(8, 128, 20000, 3)
    assert m.shape == (20000, 8) and m.dtype == np.int32
    assert m.min() == 0 and m.max() == 127
    counts = np.bincount(m.ravel(), minlength=128)
    exp = m.size / 128
    assert np.abs(counts - exp).max() < 6 * np.sqrt(exp)


def test_probe_plan():
    C, M, K, e = 8, 100, 5000, 3
    q, er = inputs.make_probe_plan(C, M, K, e, 11)
    assert q.min() >= 0 and q.max() < M
    assert (er.sum(axis=1) == e).all()
    # every cluster is erased about equally often
    f = er.mean(axis=0)
    assert np.abs(f - e / C).max() < 0.05
    # the plan of probe k does not depend on K
    q2, er2 = inputs.make_probe_plan(C, M, 100, e, 11)
    assert (q2 == q[:100]).all() and (er2 == er[:100]).all()
    for ee in (0, C):
        _, er3 = inputs.make_probe_plan(C, M, 10, ee, 1)
        assert (er3.sum(axis=1) == ee).all()


def test_one_hot_matches_printed_code():
    """Section II-A: the printed code of message (9,4,3,10) fixes neuron i = c*L + l."""
    g = read_golden("encoding_example.txt")
    C, L = int(g["C"][0]), int(g["L"][0])
    msg = np.array([int(x) - 1 for x in g["message_1based"][0].split()], dtype=np.int32)  # 0-based symbols
    code = np.array([int(ch) for ch in g["code"][0].replace(" ", "")], dtype=np.uint8)
    assert code.size == C * L and code.sum() == C
    v = inputs.one_hot(msg[None, :], L)[0]
    assert (v == code).all()
    assert list(inputs.active_neurons(msg, L)) == [8, 19, 34, 57]


def test_one_hot_erasure():
    msgs = inputs.make_messages(4, 16, 10, 1)
    er = np.zeros((10, 4), dtype=bool)
    er[:, 1] = True
    V = inputs.one_hot(msgs, 16, er)
    assert (V.reshape(10, 4, 16).sum(axis=2) == np.array([1, 0, 1, 1])).all()


def test_workload_table():
    w = inputs.WORKLOADS
    assert w["cfg3"].n == 2048 and w["cfg5"].n == 8192
    assert abs(w["cfg3"].density() - 0.263) < 2e-3
    assert abs(w["cfg2"].density() - 0.263) < 2e-3
    assert abs(w["cfg5"].density() - 0.317) < 2e-3
    seeds = [x.seed for x in w.values()]
    assert len(set(seeds)) == len(seeds)
