"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, bit for bit.

Everything here is integer / bit work, so the bar is exact equality: the packed W, every byte
of every final activity vector, every entry of iters_out, and the retrieval error rate.
"""
import numpy as np
import pytest
import torch

from oracle import gbnn_oracle as orc
from paper_1303_7032_amd import binding as gb
from paper_1303_7032_amd import inputs
from conftest import read_golden

pytestmark = pytest.mark.gpu

RULES = ("sum_of_sum", "sum_of_max", "hybrid")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    gb.lib()  # fails loudly if the HIP library is not built


@pytest.fixture(params=["auto", "atomic", "rows"])
def store_path(request):
    """Both storing kernels (one atomic OR per bit; rows built in LDS), and the library's own choice."""
    gb.gbnn_set_kernel_choice("auto", request.param)
    yield request.param
    gb.gbnn_set_kernel_choice("auto", "auto")


class family:
    """The kernel family the library picks, or the any-shape kernel for every shape, or one wavefront per
    probe also where two probes per wavefront would be picked (gbnn_set_kernel_choice around the calls)."""

    def __init__(self, force_generic=False, force_wave=False):
        self.name = "generic" if force_generic else "wave" if force_wave else "auto"

    def __enter__(self):
        gb.gbnn_set_kernel_choice(self.name, "auto")

    def __exit__(self, *exc):
        gb.gbnn_set_kernel_choice("auto", "auto")


def dev_store(C, L, msgs):
    W = gb.new_network(C, L)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    gb.gbnn_store(W, C, L, torch.from_numpy(np.ascontiguousarray(msgs, dtype=np.int32)).cuda(), status)
    return W, int(status.item())


def dev_retrieve(W, C, L, V0, rule, gamma, cap, force_generic=False, force_wave=False, **kw):
    """gbnn_retrieve on the kernel family the library picks, or with the any-shape kernel forced, or
    with the two-probes-per-wave kernel switched off."""
    with family(force_generic, force_wave):
        V0d = torch.from_numpy(V0).cuda() if isinstance(V0, np.ndarray) else V0
        out, it = gb.gbnn_retrieve(W, C, L, V0d, rule, gamma, cap, **kw)
        torch.cuda.synchronize()
    return out.cpu().numpy(), it.cpu().numpy()


def other_paths(C, L, rule):
    """Keyword sets that force every other kernel family able to serve the shape."""
    path = gb.gbnn_retrieve_path(C, L, rule, torch.zeros(1, device="cuda"))
    alts = []
    if path.startswith("half"):
        alts.append(("wave", {"force_wave": True}))
    if path != "generic":
        alts.append(("generic", {"force_generic": True}))
    return alts


def check_same(out, it, ref, itref, what):
    bad = np.nonzero((out != ref).any(axis=1))[0]
    assert bad.size == 0, f"{what}: {bad.size} probes differ, first {bad[:5]}"
    badi = np.nonzero(it != itref)[0]
    assert badi.size == 0, f"{what}: iters differ at {badi[:5]}: {it[badi[:5]]} vs {itref[badi[:5]]}"


# ------------------------------------------------------------------------------- storing
@pytest.mark.parametrize("name", list(inputs.WORKLOADS))
def test_store_bit_exact(name, store_path):
    w = inputs.WORKLOADS[name]
    msgs = w.messages()
    Wd, st = dev_store(w.C, w.L, msgs)
    Wo, skipped = orc.store(w.C, w.L, msgs)
    assert st == 0 and skipped == 0
    got = Wd.cpu().numpy().view(np.uint32)
    assert (got == orc.pack_bits(Wo)).all()


@pytest.mark.parametrize("C,L,M", [(3, 3, 4), (5, 12, 200), (7, 33, 500), (2, 1, 3), (64, 256, 3000), (6, 700, 9000),
                                   (4, 2048, 30000), (16, 1024, 2000)])
def test_store_odd_shapes_incremental_and_status(C, L, M, store_path):
    msgs = inputs.make_messages(C, L, M, 17)
    Wo, _ = orc.store(C, L, msgs)
    # two calls, second one overlapping the first, plus messages with bad symbols
    bad = msgs[:3].copy()
    bad[0, 0] = L
    bad[1, C - 1] = -1
    W = gb.new_network(C, L)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    h = M // 2
    for part in (msgs[:h], np.concatenate([msgs[h // 2:h], bad[:1], msgs[h:], bad[1:2]]), bad[:2]):
        gb.gbnn_store(W, C, L, torch.from_numpy(np.ascontiguousarray(part)).cuda(), status)
    assert int(status.item()) == 1
    assert (W.cpu().numpy().view(np.uint32) == orc.pack_bits(Wo)).all()
    gb.gbnn_store(W, C, L, torch.zeros((0, C), dtype=torch.int32, device="cuda"))  # M = 0 is a no-op


# ------------------------------------------------------------------------------- worked example
def test_oscillation_example_through_the_abi():
    """Section V-A on the GPU (n = 9, any-shape kernel): printed v^1..v^3 and the cap path."""
    g = read_golden("oscillation_example.txt")
    C, L = int(g["C"][0]), int(g["L"][0])
    msgs = np.array([[int(x) - 1 for x in m.split()] for m in g["messages_1based"][0].split("/")], dtype=np.int32)
    vec = {k: np.array([int(x) for x in g[k][0].split()], dtype=np.uint8) for k in ("v0", "v1", "v2", "v3")}
    W, _ = dev_store(C, L, msgs)
    for cap, want in {1: "v1", 2: "v2", 3: "v3", 4: "v2", 9: "v1"}.items():
        out, it = dev_retrieve(W, C, L, vec["v0"][None, :].copy(), "sum_of_sum", 1, cap)
        assert (out[0] == vec[want]).all() and it[0] == -cap
    out, it = dev_retrieve(W, C, L, vec["v0"][None, :].copy(), "sum_of_sum", 2, 20)
    assert (out[0] == vec["v2"]).all() and it[0] == 3
    out, it = dev_retrieve(W, C, L, vec["v0"][None, :].copy(), "sum_of_max", 1, 20)
    assert (out[0] == vec["v1"]).all() and it[0] == 1
    out, it = dev_retrieve(W, C, L, vec["v0"][None, :].copy(), "hybrid", 1, 20)
    assert (out[0] == vec["v1"]).all() and it[0] == 2
    # the same through the message boundary: probe "erased, erased, 1" as symbols
    probe = np.array([[int(x) - 1 for x in g["probe_1based"][0].split()]], dtype=np.int32)
    for cap, want in {1: "v1", 2: "v2", 3: "v3"}.items():
        bits, sym, it = dev_retrieve_symbols(W, C, L, probe, "sum_of_sum", 1, cap)
        assert int(bits.view(np.uint32)[0, 0]) == sum(int(b) << i for i, b in enumerate(vec[want])) and it[0] == -cap
        _, rsym = orc.decode(C, L, vec[want][None, :])
        assert (sym == rsym).all()


# ------------------------------------------------------------------------------- small / medium shapes
SHAPES = [
    # C, L, M, e, K
    (4, 16, 50, 2, 200),     # cfg1
    (3, 3, 4, 2, 37),        # clusters inside one word
    (5, 12, 200, 2, 101),    # clusters straddle words
    (7, 33, 400, 3, 64),     # n = 231, not a multiple of 32
    (8, 32, 300, 4, 259),    # one word per cluster, ragged K
    (8, 128, 5000, 4, 515),  # cfg2 shape: half the lanes idle
    (8, 256, 20000, 4, 1027),  # cfg3 shape: several workgroups and a ragged tail
    (3, 256, 3000, 1, 130),  # 24 of 64 lanes
    (12, 256, 20000, 6, 300),  # 96 words: two words per lane, second slot half empty
    (16, 512, 100000, 8, 260),  # cfg5 shape: four words per lane
    (2, 2048, 3000, 1, 70),  # a cluster is a whole wave
    (16, 1024, 60000, 8, 20),  # n = 16384, the largest: eight words per lane
    (8, 2048, 40000, 4, 40),   # ... a cluster is a whole slot
    (64, 256, 8000, 32, 36),   # ... eight lanes per cluster
    (9, 1024, 30000, 4, 33),   # 288 words: the fifth slot half empty
    (32, 32, 700, 16, 131),    # two probes per wave, a cluster is one lane, odd K
    (16, 64, 800, 8, 130),     # ... two lanes per cluster
    (2, 512, 30000, 1, 67),    # ... a cluster is half of the half-wave
    (32, 64, 3000, 16, 131),   # 64 words, two per cluster: one wave per probe
    (64, 32, 1000, 32, 45),    # 64 one-word clusters
    (8, 256, 300, 4, 130),     # a nearly empty network: no cluster summary is all ones (none may be skipped)
    (8, 128, 100, 5, 131),     # ... two probes per wave
    (8, 256, 3000, 4, 130),    # ... some summaries all ones, some not
    # cluster sizes that are not a power of two (or below 32): padded clusters in the register kernels
    (8, 100, 3000, 4, 301),    # 100 -> 128: two probes per wave; activity in 4-byte pieces
    (8, 200, 12000, 4, 203),   # 200 -> 256: one word per lane; 8-byte-aligned clusters
    (12, 96, 3000, 6, 150),    # 96 -> 128: whole words of the packed result change places
    (10, 300, 30000, 5, 77),   # 300 -> 512: four words per lane
    (6, 700, 90000, 3, 41),    # 700 -> 1024: four words per lane, odd alignment of the clusters (4 bytes)
    (5, 1501, 200000, 2, 23),  # 1501 -> 2048: eight words per lane, byte-wise activity
    (9, 17, 120, 4, 130),      # 17 -> 32: clusters share the words of the packed result
    (40, 50, 900, 20, 61),     # 50 -> 64: 80 words, two per lane
]


@pytest.fixture(scope="module")
def networks():
    cache = {}

    def get(C, L, M):
        key = (C, L, M)
        if key not in cache:
            msgs = inputs.make_messages(C, L, M, 1000 + C * L + M)
            Wo, _ = orc.store(C, L, msgs)
            Wd, _ = dev_store(C, L, msgs)
            assert (Wd.cpu().numpy().view(np.uint32) == orc.pack_bits(Wo)).all()
            cache[key] = (msgs, Wo, Wd)
        return cache[key]
    return get


@pytest.mark.parametrize("C,L,M,e,K", SHAPES)
@pytest.mark.parametrize("rule", RULES)
def test_probes_from_stored_messages(networks, C, L, M, e, K, rule):
    msgs, Wo, Wd = networks(C, L, M)
    q, er = inputs.make_probe_plan(C, M, K, e, 5 + C + L)
    V0 = inputs.one_hot(msgs[q], L, er)
    for gamma, cap in ((1, 20), (2, 3)):
        ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, gamma, cap)
        out, it = dev_retrieve(Wd, C, L, V0, rule, gamma, cap)
        check_same(out, it, ref, itref, f"{rule} gamma={gamma} cap={cap}")
        for nm, kw in other_paths(C, L, rule):
            if nm == "generic" and K > 300:
                continue
            out, it = dev_retrieve(Wd, C, L, V0, rule, gamma, cap, **kw)
            check_same(out, it, ref, itref, f"{rule} {nm} gamma={gamma} cap={cap}")
        if rule != "sum_of_sum":
            break  # gamma is ignored by the other rules


def dev_retrieve_symbols(W, C, L, probes, rule, gamma, cap, force_generic=False, force_wave=False, **kw):
    with family(force_generic, force_wave):
        bits, sym, it = gb.gbnn_retrieve_symbols(W, C, L, torch.from_numpy(probes).cuda(), rule, gamma, cap, **kw)
        torch.cuda.synchronize()
    return [None if t is None else t.cpu().numpy() for t in (bits, sym, it)]


@pytest.mark.parametrize("C,L,M,e,K", SHAPES)
@pytest.mark.parametrize("rule", RULES)
def test_messages_at_the_boundary(networks, C, L, M, e, K, rule):
    """gbnn_retrieve_symbols (symbols in; packed bits, symbols and pass counts out) against the
    oracle's encode -> retrieve -> decode, on every kernel family that serves the shape.  Besides
    erased clusters the probes hold wrong symbols (so that clusters end empty or ambiguous) and
    out-of-range entries (= erased)."""
    msgs, Wo, Wd = networks(C, L, M)
    q, er = inputs.make_probe_plan(C, M, K, e, 11 + C + L)
    probes = msgs[q].copy()
    probes[er] = -1
    rng = np.random.default_rng(C * 77 + L)
    for k in range(0, K, 5):                       # a wrong symbol in one known cluster
        c = int(rng.integers(C))
        probes[k, c] = int(rng.integers(L))
    probes[1::7, 0] = L + 3                        # outside [0, L): erased
    probes[2::9, C - 1] = -12345
    cap = 20 if rule != "sum_of_sum" else 4
    rbits, rsym, rit = orc.retrieve_symbols(Wo, C, L, probes, rule, 1, cap)
    for nm, kw in [("default", {})] + other_paths(C, L, rule):
        if nm == "generic" and K > 300:
            continue
        bits, sym, it = dev_retrieve_symbols(Wd, C, L, probes, rule, 1, cap, **kw)
        assert (bits.view(np.uint32) == rbits).all(), f"{rule} {nm}: packed bits differ"
        bad = np.nonzero((sym != rsym).any(axis=1))[0]
        assert bad.size == 0, f"{rule} {nm}: symbols differ at probes {bad[:5]}: {sym[bad[:2]]} vs {rsym[bad[:2]]}"
        assert (it == rit).all(), f"{rule} {nm}: iters differ"
    # each output alone, and none at all
    bits, sym, it = dev_retrieve_symbols(Wd, C, L, probes, rule, 1, cap, want_symbols=False, want_iters=False)
    assert sym is None and it is None and (bits.view(np.uint32) == rbits).all()
    bits, sym, it = dev_retrieve_symbols(Wd, C, L, probes, rule, 1, cap, want_bits=False)
    assert bits is None and (sym == rsym).all() and (it == rit).all()


def test_messages_at_the_boundary_edge_cases(networks):
    C, L, M = 8, 128, 5000
    msgs, Wo, Wd = networks(C, L, M)
    bits, sym, it = gb.gbnn_retrieve_symbols(Wd, C, L, torch.zeros((0, C), dtype=torch.int32, device="cuda"), "hybrid")
    assert bits.numel() == 0 and sym.numel() == 0 and it.numel() == 0
    for K in (1, 2, 3):                                   # fewer probes than a wave carries; odd K
        probes = msgs[:K].copy()
        probes[:, 1] = -1
        for rule in RULES:
            rbits, rsym, rit = orc.retrieve_symbols(Wo, C, L, probes, rule, 1, 6)
            bits, sym, it = dev_retrieve_symbols(Wd, C, L, probes, rule, 1, 6)
            assert (bits.view(np.uint32) == rbits).all() and (sym == rsym).all() and (it == rit).all()


@pytest.mark.parametrize("C,L,M", [(4, 16, 50), (5, 12, 200), (8, 32, 300), (8, 128, 5000), (8, 256, 20000),
                                    (16, 512, 100000), (32, 32, 700), (2, 512, 30000), (12, 256, 20000),
                                    # eight words per lane: sum-of-sum digits beyond the registers, the hybrid's
                                    # signal counter and the crowded-cluster walk at that width
                                    (16, 1024, 60000), (8, 2048, 40000), (64, 256, 8000), (9, 1024, 30000),
                                    # padded clusters
                                    (8, 100, 3000), (8, 200, 12000), (10, 300, 30000), (9, 17, 120), (3, 3, 12)])
@pytest.mark.parametrize("rule", RULES)
def test_arbitrary_binary_probes(networks, C, L, M, rule):
    """Probes outside the one-active-neuron-per-cluster contract: several active neurons in a
    cluster, corrupted symbols, empty and full probes, random dense activity."""
    msgs, Wo, Wd = networks(C, L, M)
    n = C * L
    rng = np.random.default_rng(C * 1000 + L)
    rows = []
    base = inputs.one_hot(msgs[:8], L)
    rows += [base[0], np.zeros(n, np.uint8), np.ones(n, np.uint8)]
    for k in range(8):                                  # two stored messages superposed, some clusters erased
        v = base[k] | base[(k + 3) % 8]
        v.reshape(C, L)[rng.permutation(C)[: C // 2]] = 0
        rows.append(v)
    for k in range(6):                                  # a corrupted symbol
        v = base[k].copy().reshape(C, L)
        c = int(rng.integers(C))
        v[c] = 0
        v[c, int(rng.integers(L))] = 1
        v[(c + 1) % C] = 0
        rows.append(v.reshape(-1))
    for dens in (1.0 / L, 4.0 / L, 0.2, 0.7):           # random activity
        for _ in range(3):
            rows.append((rng.random(n) < dens).astype(np.uint8))
    v = np.ones(n, np.uint8)                            # one cluster partly on, the rest full
    v[: L // 2] = 0
    rows.append(v)
    V0 = np.stack(rows)
    for gamma, cap in ((1, 6), (0, 4), (5, 4), (300, 3), (32767, 3)):  # scores beyond 8 and 15 binary digits too
        ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, gamma, cap)
        out, it = dev_retrieve(Wd, C, L, V0, rule, gamma, cap)
        check_same(out, it, ref, itref, f"{rule} gamma={gamma}")
        for nm, kw in other_paths(C, L, rule):
            out, it = dev_retrieve(Wd, C, L, V0, rule, gamma, cap, **kw)
            check_same(out, it, ref, itref, f"{rule} {nm} gamma={gamma}")
        if rule != "sum_of_sum":
            break


@pytest.mark.parametrize("M", [20000, 30000])
@pytest.mark.parametrize("rule", ["sum_of_max", "hybrid"])
def test_later_passes_many_caps_and_dying_clusters(networks, M, rule):
    """Passes after the first, at every cap, on probes that converge early, late, hit the cap, or lose
    a whole cluster (after which everything switches off): stored messages with 3-6 erased clusters,
    half of them with one wrong known symbol."""
    C, L, K = 8, 256, 600
    msgs, Wo, Wd = networks(C, L, M)
    rng = np.random.default_rng(M)
    parts = []
    for e in (3, 4, 5, 6):
        q, er = inputs.make_probe_plan(C, M, K // 4, e, 40 + e)
        sym = msgs[q].copy()
        for k in range(0, len(sym), 2):
            known = np.nonzero(~er[k])[0]
            sym[k, known[int(rng.integers(len(known)))]] = int(rng.integers(L))
        parts.append(inputs.one_hot(sym, L, er))
    V0 = np.concatenate(parts)
    seen_dead_late = seen_capped = 0
    for cap in (1, 2, 3, 4, 5, 20):
        ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, 1, cap)
        for nm, kw in [("default", {})] + other_paths(C, L, rule):
            out, it = dev_retrieve(Wd, C, L, V0, rule, 1, cap, **kw)
            check_same(out, it, ref, itref, f"{rule} M={M} cap={cap} {nm}")
        seen_capped += int((itref < 0).sum())
        if cap == 20:
            erased_part_dead = (ref.reshape(len(ref), C, L).sum(axis=2) == 0).any(axis=1)
            seen_dead_late += int((erased_part_dead & (itref >= 3)).sum())
    assert seen_capped > 0 and seen_dead_late > 0, "the sample must hold capped probes and probes that lose a cluster late"


@pytest.mark.parametrize("C,L,M,K", [(8, 128, 9000, 20000), (8, 256, 30000, 20000), (12, 256, 45000, 6000)])
@pytest.mark.parametrize("rule", ["sum_of_max", "hybrid"])
def test_many_probes_around_the_candidate_limit(networks, C, L, M, K, rule):
    """Networks dense enough that the number of candidates left by pass 1 straddles the limit of the
    candidate-matrix passes (28 per probe with two probes per wave, 32 with one), so that probes
    just below and just above it sit side by side, in both kernel families that serve the shape."""
    msgs, Wo, Wd = networks(C, L, M)
    e = C // 2
    q, er = inputs.make_probe_plan(C, M, K, e, 77)
    V0 = inputs.one_hot(msgs[q], L, er)
    ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, 1, 20)
    # candidates after pass 1 = what the hybrid's first pass leaves in the erased clusters
    first, _, _ = orc.retrieve(Wo, C, L, V0, "hybrid", 1, 1)
    cands = (first.astype(np.int32).sum(axis=1) - (C - e))
    assert (cands < 26).any() and (cands > 34).any(), f"candidates range {cands.min()}..{cands.max()}"
    for nm, kw in [("default", {})] + [a for a in other_paths(C, L, rule) if a[0] != "generic"]:
        out, it = dev_retrieve(Wd, C, L, V0, rule, 1, 20, **kw)
        check_same(out, it, ref, itref, f"{rule} {nm}")


def test_edge_cases(networks):
    C, L, M = 8, 256, 20000
    msgs, Wo, Wd = networks(C, L, M)
    n = C * L
    # K = 0
    out, it = gb.gbnn_retrieve(Wd, C, L, torch.zeros((0, n), dtype=torch.uint8, device="cuda"), "sum_of_max")
    assert out.numel() == 0 and it.numel() == 0
    for e in (0, 1, C - 1, C):
        q, er = inputs.make_probe_plan(C, M, 33, e, 9)
        V0 = inputs.one_hot(msgs[q], L, er)
        for rule in RULES:
            for cap in (1, 2, 20):
                ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, 1, cap)
                out, it = dev_retrieve(Wd, C, L, V0, rule, 1, cap)
                check_same(out, it, ref, itref, f"e={e} {rule} cap={cap}")
                out, it = dev_retrieve(Wd, C, L, V0, rule, 1, cap, force_wave=True)
                check_same(out, it, ref, itref, f"e={e} {rule} cap={cap} wave")
    # in place, without iters_out; then through an unaligned view
    q, er = inputs.make_probe_plan(C, M, 77, 4, 10)
    V0 = inputs.one_hot(msgs[q], L, er)
    ref, itref, _ = orc.retrieve(Wo, C, L, V0, "sum_of_max", 1, 20)
    buf = torch.from_numpy(V0).cuda()
    gb.gbnn_retrieve(Wd, C, L, buf, "sum_of_max", 1, 20, V_out=buf, want_iters=False)
    assert (buf.cpu().numpy() == ref).all()
    raw = torch.zeros(V0.size + 64, dtype=torch.uint8, device="cuda")
    view = raw[3:3 + V0.size].view(77, n)
    view.copy_(torch.from_numpy(V0))
    assert gb.gbnn_retrieve_path(C, L, "hybrid", view, view) == "wave1"   # (byte-wise loads and stores of the activity)
    refh, ith, _ = orc.retrieve(Wo, C, L, V0, "hybrid", 1, 20)
    out, it = gb.gbnn_retrieve(Wd, C, L, view, "hybrid", 1, 20, V_out=view)
    torch.cuda.synchronize()
    check_same(out.cpu().numpy(), it.cpu().numpy(), refh, ith, "unaligned in place")
    assert int(raw[:3].sum()) == 0 and int(raw[3 + V0.size:].sum()) == 0


def test_streams_share_a_workspace(networks):
    """Calls enqueue on the caller's stream and only read the prepared workspace, so two streams may run
    retrievals on the same network at the same time."""
    C, L, M = 8, 256, 20000
    msgs, Wo, Wd = networks(C, L, M)
    ws = gb.gbnn_prepare(Wd, C, L)
    torch.cuda.synchronize()
    jobs = []
    for i, rule in enumerate(("sum_of_max", "hybrid", "sum_of_sum", "sum_of_max")):
        q, er = inputs.make_probe_plan(C, M, 3000 + i, 4, 50 + i)
        V0 = inputs.one_hot(msgs[q], L, er)
        jobs.append((rule, V0, torch.from_numpy(V0).cuda(), torch.cuda.Stream()))
    torch.cuda.synchronize()
    results = []
    for _ in range(3):                      # several rounds in flight on every stream
        for rule, V0, V0d, st in jobs:
            with torch.cuda.stream(st):
                results.append((rule, V0, gb.gbnn_retrieve(Wd, C, L, V0d, rule, 1, 20, workspace=ws)))
    torch.cuda.synchronize()
    for rule, V0, (out, it) in results:
        ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, 1, 20)
        check_same(out.cpu().numpy(), it.cpu().numpy(), ref, itref, f"{rule} on its own stream")


def test_argument_errors_reach_python():
    W = gb.new_network(4, 16)
    V = torch.zeros((2, 64), dtype=torch.uint8, device="cuda")
    with pytest.raises(gb.GbnnError) as ei:
        gb.gbnn_retrieve(W, 4, 16, V, "sum_of_max", 1, 0)
    assert ei.value.code == gb.ERRORS["ITERS"]
    with pytest.raises(gb.GbnnError) as ei:
        gb.gbnn_retrieve(W, 4, 16, V, "sum_of_sum", -1, 4)
    assert ei.value.code == gb.ERRORS["GAMMA"]
    with pytest.raises(gb.GbnnError) as ei:
        gb.gbnn_retrieve(W, 4, 16, V, 7, 1, 4)
    assert ei.value.code == gb.ERRORS["RULE"]
    with pytest.raises(gb.GbnnError) as ei:
        gb.gbnn_retrieve(W, 4, 16, V, "hybrid", 1, 4, workspace=torch.zeros(256, dtype=torch.uint8, device="cuda")[:16])
    assert ei.value.code == gb.ERRORS["WORKSPACE"]


# ------------------------------------------------------------------------------- the five configurations, full size
@pytest.mark.parametrize("name", list(inputs.WORKLOADS))
def test_full_configuration(name):
    """BASELINE configurations at full K, in the launch configuration the benchmark times:
    identical W, identical final activity for every probe, identical iters and error rate."""
    w = inputs.WORKLOADS[name]
    msgs = w.messages()
    Wo, _ = orc.store(w.C, w.L, msgs)
    Wd, _ = dev_store(w.C, w.L, msgs)
    assert (Wd.cpu().numpy().view(np.uint32) == orc.pack_bits(Wo)).all()
    q, er, V0 = w.probes(msgs)
    target = inputs.one_hot(msgs[q], w.L)
    V0d = torch.from_numpy(V0).cuda()
    finals = {}
    for rule in w.rules:
        print(f"[{name}] {rule}: oracle on {w.K} probes", flush=True)
        ref, itref, _ = orc.retrieve(Wo, w.C, w.L, V0, rule, w.gamma, w.max_iters)
        out, it = dev_retrieve(Wd, w.C, w.L, V0d, rule, w.gamma, w.max_iters)
        check_same(out, it, ref, itref, f"{name} {rule}")
        assert orc.error_rate(out, target) == orc.error_rate(ref, target)
        finals[rule] = out
        del ref
        # the message boundary at full size: same final vectors, as packed bits and as symbols
        probes = msgs[q].copy()
        probes[er] = -1
        bits, sym, it2 = dev_retrieve_symbols(Wd, w.C, w.L, probes, rule, w.gamma, w.max_iters)
        assert (it2 == it).all()
        nw = (w.n + 31) // 32
        padded = np.zeros((w.K, nw * 32), dtype=np.uint8)
        padded[:, :w.n] = out
        assert (bits.view(np.uint32) == np.packbits(padded, axis=1, bitorder="little").view("<u4")).all()
        act = out.reshape(w.K, w.C, w.L)
        cnt = act.sum(axis=2)
        want = np.where(cnt == 1, act.argmax(axis=2), np.where(cnt == 0, -1, -2)).astype(np.int32)
        assert (sym == want).all()
        del padded, act
    if "hybrid" in finals and "sum_of_max" in finals:
        assert (finals["hybrid"] == finals["sum_of_max"]).all()      # Theorem 4


def test_streamed_probe_loads_with_a_partly_filled_slot():
    """A batch of more than 512 MiB on a table larger than an L2 is read with the streaming loads (two
    contiguous pieces per 64 words, lanes exchanging half words); here the last slot of a lane holds words
    only in 8 of 64 lanes (25 x 256: 200 packed words).  All probes against the any-shape kernel, the first
    1024 against the oracle."""
    C, L, M, e = 25, 256, 30000, 12
    K = (513 << 20) // (C * L) + 1
    assert K * C * L >= 512 << 20
    msgs = inputs.make_messages(C, L, M, 91)
    Wo, _ = orc.store(C, L, msgs)
    Wd, _ = dev_store(C, L, msgs)
    q, er = inputs.make_probe_plan(C, M, K, e, 92)
    idx = torch.from_numpy(inputs.active_neurons(msgs[q], L)).cuda()
    V0d = torch.zeros((K, C * L), dtype=torch.uint8, device="cuda")
    V0d.scatter_(1, idx, torch.from_numpy((~er).astype(np.uint8)).cuda())
    del idx
    host = V0d[:1024].cpu().numpy()
    for rule in ("sum_of_max", "hybrid"):
        assert gb.gbnn_retrieve_path(C, L, rule, V0d) == "wave4"
        out, it = gb.gbnn_retrieve(Wd, C, L, V0d, rule, 1, 20)
        with family(force_generic=True):
            out2, it2 = gb.gbnn_retrieve(Wd, C, L, V0d, rule, 1, 20)
        torch.cuda.synchronize()
        assert torch.equal(out, out2) and torch.equal(it, it2), rule
        ref, itref, _ = orc.retrieve(Wo, C, L, host, rule, 1, 20)
        check_same(out[:1024].cpu().numpy(), it[:1024].cpu().numpy(), ref, itref, f"streamed loads {rule}")
        del out, out2


@pytest.mark.parametrize("nbytes", [16, 1008, 2048, 2064, 8192 + 48, (1 << 20) + 16])
@pytest.mark.parametrize("streaming", [False, True])
def test_reference_copy(nbytes, streaming):
    """The benchmark's reference copy moves exactly the bytes it is given."""
    g = torch.Generator(device="cuda").manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes + 32,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.full((nbytes + 32,), 7, dtype=torch.uint8, device="cuda")
    gb.gbnn_reference_copy(dst[16:16 + nbytes], src[16:16 + nbytes], streaming)
    torch.cuda.synchronize()
    assert torch.equal(dst[16:16 + nbytes], src[16:16 + nbytes])
    assert (dst[:16] == 7).all() and (dst[16 + nbytes:] == 7).all()

