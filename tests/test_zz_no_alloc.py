"""The step on the library's own per-GPU scratch array (spec_verify_step_static: for callers
that cannot allocate) against the same step on a caller-owned workspace (spec_verify_step),
through the C ABI: bit-identical outputs on two calls in a row, the second with a smaller
input, and both against the CPU oracle.  (The refusal of a step that does not fit is a host-side
check, tested without a GPU in test_host_api.py.)"""
import numpy as np
import pytest

from paper_2406_14066_amd import workloads as W
from paper_2406_14066_amd import spec_verify as sv
from parity_utils import check_attn, check_reject

pytestmark = pytest.mark.gpu


def _both_ways(w):
    import torch
    from paper_2406_14066_amd.harness import DeviceStep
    ds = DeviceStep(w, kv_layout=sv.KV_MFMA)
    assert sv.spec_verify_workspace_bytes(ds.attn_args, ds.reject_args) <= sv.STATIC_SCRATCH_BYTES
    ds.run_step()                                   # caller-owned workspace
    ref = ds.results()
    ds.out.fill_(float("nan"))
    ds.accepted_len.fill_(-9)
    ds.next_token.fill_(-9)
    ds.out_tokens.fill_(-9)
    ds.counters.zero_()
    if ds.debug is not None:
        ds.debug.fill_(float("nan"))
    torch.cuda.synchronize()
    sv.spec_verify_step_static(ds.attn_args, ds.reject_args)
    got = ds.results()
    for key in ("out", "accepted_len", "next_token", "out_tokens", "counters"):
        np.testing.assert_array_equal(got[key], ref[key], err_msg=key)
    check_attn(w, got["out"])
    check_reject(w, got)
    return got


def test_static_scratch_step_matches_the_workspace_step_twice_in_a_row():
    import torch
    assert torch.cuda.is_available()
    print("case static scratch: split requests (partials, tickets, rejection records in the scratch)", flush=True)
    big = W.config("c5", L_scale=0.12, V=16384)          # long contexts: every request is split into chunks
    _both_ways(big)
    print("case static scratch: a smaller step right after, on the same array", flush=True)
    small = W.config("c4", B=12, L_scale=0.5, V=4096)
    _both_ways(small)
    # and the first shape again: whatever the smaller call left behind must not matter
    _both_ways(big)
