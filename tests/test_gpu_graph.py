"""The whole step captured into a HIP graph and replayed (Section 5.3 of the paper runs its
steps from captured graphs): the library allocates nothing, clears nothing with memsets and
tags its workspace records per call, so a captured launch must give the eager result on
every replay, with the program's own eager work in between."""
import numpy as np
import pytest

from paper_2406_14066_amd import workloads as W
from paper_2406_14066_amd import spec_verify as sv
from parity_utils import check_attn, check_reject

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,kw,early_stop", [("c2", dict(B=4, L_scale=0.25), False),
                                                ("c4", dict(B=40, L_scale=0.5, V=8192), False),
                                                ("c4", dict(B=40, L_scale=0.5, V=8192), True),
                                                ("c5", dict(L_scale=0.1, V=16384), False)],
                         ids=["c2_small", "c4_small", "c4_small_early_stop", "c5_small"])
def test_step_replays_from_a_graph(tuning, name, kw, early_stop):
    import torch
    from paper_2406_14066_amd.harness import DeviceStep
    print("case graph", name, "early stop", early_stop, flush=True)
    if early_stop:   # the statistics pass in position order with placeholder records (large batches get it by themselves)
        tuning("SPEC_VERIFY_EARLY_STOP", 1)
    w = W.config(name, **kw)
    ds = DeviceStep(w, kv_layout=sv.KV_MFMA)
    ds.run_step()
    eager = ds.results()
    check_attn(w, eager["out"])
    check_reject(w, eager)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ds.run_step(side)          # warm-up on the capture stream
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        ds.run_step(torch.cuda.current_stream())
    torch.cuda.synchronize()

    scratch = torch.zeros(1 << 20, device="cuda")
    for replay in range(5):
        # the program's own eager work between the replays, and outputs reset to a sentinel
        ds.out.fill_(float("nan"))
        ds.accepted_len.fill_(-9)
        ds.next_token.fill_(-9)
        ds.out_tokens.fill_(-9)
        ds.counters.zero_()
        scratch.add_(1.0)
        if replay == 2:
            ds.run_step()           # an eager call on the same workspace between two replays
            ds.counters.zero_()
        torch.cuda.synchronize()
        graph.replay()
        got = ds.results()
        np.testing.assert_array_equal(got["out"], eager["out"])
        np.testing.assert_array_equal(got["accepted_len"], eager["accepted_len"])
        np.testing.assert_array_equal(got["next_token"], eager["next_token"])
        np.testing.assert_array_equal(got["out_tokens"], eager["out_tokens"])
        np.testing.assert_array_equal(got["counters"], eager["counters"])
