"""Seeded random shapes, networks, probes, rules and caps: every kernel family that can serve a shape
against the oracle (activity and message boundary), both storing kernels, gbnn_store_update, and the
sparse W'.  A bounded sample of a longer randomized comparison; each case prints what names it."""
import numpy as np
import pytest
import torch

from oracle import gbnn_oracle as orc
from paper_1303_7032_amd import binding as gb
from paper_1303_7032_amd import inputs

pytestmark = pytest.mark.gpu

RULES = ("sum_of_sum", "sum_of_max", "hybrid")
FAMILIES = ("auto", "wave", "generic")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    gb.lib()


@pytest.mark.parametrize("seed", [101, 202, 303])
def test_random_retrievals(seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        L = int(rng.choice([3, 4, 16, 20, 32, 48, 64, 100, 128, 200, 256, 300, 512, 700, 1024, 2048]))
        cmax = min(64, 16384 // L) if L >= 32 else min(64, 2048 // L)  # up to the interface's n = 16384
        C = int(rng.integers(2, max(3, cmax + 1)))
        dens = float(rng.choice([0.01, 0.1, 0.25, 0.4, 0.6]))
        M = min(200000, max(2, int(np.log(1 - dens) / np.log(1 - 1.0 / (L * L)))))
        K = int(rng.choice([1, 2, 63, 130, 257]))
        e = int(rng.integers(0, C + 1))
        print(f"seed {seed} case {case}: C={C} L={L} M={M} K={K} e={e}", flush=True)
        msgs = inputs.make_messages(C, L, M, int(rng.integers(1 << 30)))
        Wo, _ = orc.store(C, L, msgs)
        W = gb.new_network(C, L)
        gb.gbnn_store(W, C, L, torch.from_numpy(msgs).cuda())
        q, er = inputs.make_probe_plan(C, M, K, e, int(rng.integers(1 << 30)))
        probes = msgs[q].copy()
        probes[er] = -1
        for k in range(0, K, 3):
            if rng.random() < 0.5:
                probes[k, int(rng.integers(C))] = int(rng.integers(L))
        V0 = orc.encode_probes(C, L, probes)
        V0d, pd = torch.from_numpy(V0).cuda(), torch.from_numpy(probes).cuda()
        for rule in RULES:
            gamma, cap = int(rng.choice([0, 1, 2, 7])), int(rng.choice([1, 2, 3, 5, 20]))
            ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, gamma, cap)
            rbits, rsym = orc.decode(C, L, ref)
            for fam in FAMILIES:
                gb.gbnn_set_kernel_choice(fam, "auto")
                try:
                    out, it = gb.gbnn_retrieve(W, C, L, V0d, rule, gamma, cap)
                    bits, sym, it2 = gb.gbnn_retrieve_symbols(W, C, L, pd, rule, gamma, cap)
                    torch.cuda.synchronize()
                finally:
                    gb.gbnn_set_kernel_choice("auto", "auto")
                what = (rule, gamma, cap, fam)
                assert (out.cpu().numpy() == ref).all() and (it.cpu().numpy() == itref).all(), what
                assert (bits.cpu().numpy().view(np.uint32) == rbits).all() and (sym.cpu().numpy() == rsym).all(), what
                assert (it2.cpu().numpy() == itref).all(), what


@pytest.mark.parametrize("seed", [11, 22])
def test_random_stores_updates_and_lists(seed):
    rng = np.random.default_rng(seed)
    for case in range(60):
        lists = rng.random() < 0.6                      # the sparse W' needs L to be a multiple of 32
        if lists:
            L = int(rng.choice([32, 64, 96, 128, 256, 512, 1024]))
            cmax = min(64, 4096 // L)
        else:
            L = int(rng.integers(1, 300))
            cmax = min(64, 3000 // L)
        C = int(rng.integers(2, max(3, cmax + 1)))
        if C * L > 4096:
            continue
        M = int(rng.choice([1, 3, 63, 64, 65, 500, 3000, 20000]))
        print(f"seed {seed} case {case}: C={C} L={L} M={M} lists={lists}", flush=True)
        msgs = inputs.make_messages(C, L, M, int(rng.integers(1 << 30)))
        if rng.random() < 0.5:
            for _ in range(int(rng.integers(1, 4))):
                msgs[int(rng.integers(M)), int(rng.integers(C))] = int(rng.choice([-1, L, L + 7, -100]))
        good = msgs[((msgs >= 0) & (msgs < L)).all(axis=1)]
        Wo, skipped = orc.store(C, L, msgs)
        assert skipped == M - len(good)
        ref = orc.pack_bits(Wo)
        md = torch.from_numpy(msgs).cuda()
        for path in ("auto", "atomic", "rows"):
            gb.gbnn_set_kernel_choice("auto", path)
            try:
                W = gb.new_network(C, L)
                st = torch.zeros(1, dtype=torch.int32, device="cuda")
                h = int(rng.integers(0, M + 1))
                gb.gbnn_store(W, C, L, md[:h].contiguous(), st)
                gb.gbnn_store(W, C, L, md[h // 2:].contiguous(), st)
            finally:
                gb.gbnn_set_kernel_choice("auto", "auto")
                assert (W.cpu().numpy().view(np.uint32) == ref).all(), path
                assert int(st.item()) == (1 if len(good) < M else 0), path
        W = gb.new_network(C, L)
        gb.gbnn_store(W, C, L, md[:M // 2].contiguous())
        size = gb.gbnn_workspace_bytes(C, L, 0, "sum_of_max")
        ws = gb.gbnn_prepare(W, C, L, torch.zeros(size, dtype=torch.uint8, device="cuda"))
        gb.gbnn_store_update(W, C, L, md[M // 2:].contiguous(), ws)
        fresh = gb.gbnn_prepare(W, C, L, torch.zeros(size, dtype=torch.uint8, device="cuda"))
        assert (W.cpu().numpy().view(np.uint32) == ref).all()
        assert torch.equal(ws, fresh)   # (the bytes between the parts of a workspace are never written)
        if lists:
            Wp = gb.gbnn_sparsify(W, C, L)
            K, e, cap = int(rng.choice([1, 5, 64, 131])), int(rng.integers(0, C + 1)), int(rng.choice([1, 2, 3, 20]))
            src = good if len(good) else np.zeros((1, C), dtype=np.int32)
            q, er = inputs.make_probe_plan(C, len(src), K, e, int(rng.integers(1 << 30)))
            probes = src[q].copy()
            probes[er] = -1
            for k in range(0, K, 4):
                probes[k, int(rng.integers(C))] = int(rng.integers(-2, L + 2))
            bits, sym, it = gb.gbnn_retrieve_sparse(Wp, C, L, torch.from_numpy(probes).cuda(), cap)
            rb, rs, ri = orc.retrieve_symbols(Wo, C, L, probes, "sum_of_max", 1, cap)
            assert (bits.cpu().numpy().view(np.uint32) == rb).all() and (sym.cpu().numpy() == rs).all()
            assert (it.cpu().numpy() == ri).all()
