"""The entry point that allocates nothing (gbnn_retrieve_static: the prepared table lives in a device
array of the library) against gbnn_retrieve with a caller's workspace, through the C ABI: two calls
in a row on the same GPU, the second on a smaller network and batch, so that the shared array still
holds the first call's table when the second starts.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from oracle import gbnn_oracle as orc
from paper_1303_7032_amd import binding as gb
from paper_1303_7032_amd import inputs

RULES = {"sum_of_sum": 0, "sum_of_max": 1, "hybrid": 2}


@pytest.mark.gpu
def test_static_entry_point_matches_the_workspace_one():
    assert torch.cuda.is_available(), "needs the MI355X"
    lib = gb.lib()
    stream = torch.cuda.current_stream().cuda_stream
    # first a large network and batch, then a smaller one of another shape, then the first again
    for (C, L, M, e, K) in [(16, 512, 100000, 8, 1500), (8, 128, 5000, 4, 301), (8, 256, 20000, 4, 777),
                            (4, 16, 50, 2, 200)]:
        n = C * L
        msgs = inputs.make_messages(C, L, M, 7 + C)
        q, er = inputs.make_probe_plan(C, M, K, e, 9 + L)
        V0 = inputs.one_hot(msgs[q], L, er)
        Wo, _ = orc.store(C, L, msgs)
        W = gb.new_network(C, L)
        gb.gbnn_store(W, C, L, torch.from_numpy(msgs).cuda())
        V0d = torch.from_numpy(V0).cuda()
        ws = gb.gbnn_prepare(W, C, L)
        for rule, r in RULES.items():
            want, want_it = gb.gbnn_retrieve(W, C, L, V0d, rule, 1, 20, workspace=ws)
            out = torch.full_like(V0d, 7)
            it = torch.full((K,), 99, dtype=torch.int32, device="cuda")
            print(f"gbnn_retrieve_static C={C} L={L} K={K} {rule}", flush=True)
            rc = lib.gbnn_retrieve_static(W.data_ptr(), C, L, V0d.data_ptr(), out.data_ptr(), K, r, 1, 20,
                                          it.data_ptr(), stream)
            assert rc == gb.GBNN_OK, gb.gbnn_strerror(rc)
            torch.cuda.synchronize()
            assert torch.equal(out, want) and torch.equal(it, want_it), (C, L, rule)
            ref, itref, _ = orc.retrieve(Wo, C, L, V0, rule, 1, 20)
            assert (out.cpu().numpy() == ref).all() and (it.cpu().numpy() == itref).all(), (C, L, rule)


def test_static_entry_point_limits():
    lib = gb.lib()
    fake = 0x1000  # never dereferenced: errors are reported before anything is enqueued
    assert lib.gbnn_retrieve_static(fake, 16, 1024, fake, fake, 4, 1, 1, 20, 0, 0) == gb.ERRORS["TOO_LARGE"]
    assert lib.gbnn_retrieve_static(fake, 2, 8192, fake, fake, 4, 1, 1, 20, 0, 0) == gb.ERRORS["TOO_LARGE"]
    assert lib.gbnn_retrieve_static(fake, 8, 256, fake, fake, 4, 5, 1, 20, 0, 0) == gb.ERRORS["RULE"]
    assert lib.gbnn_retrieve_static(fake, 8, 256, 0, fake, 4, 1, 1, 20, 0, 0) == gb.ERRORS["NULL"]
    assert lib.gbnn_retrieve_static(fake, 8, 256, fake, fake, 4, 1, 1, 0, 0, 0) == gb.ERRORS["ITERS"]
    assert b"8192" in lib.gbnn_strerror(gb.ERRORS["TOO_LARGE"])
