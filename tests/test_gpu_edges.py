"""Edge cases of the verification step on the GPU, against the CPU oracle: never-visible
cache slots holding NaN or infinity, the smallest possible inputs, more requests than the
request-order table holds, vocabulary sizes that do not divide into segments, and a
workspace reused across different shapes."""
import numpy as np
import pytest

import oracle
from paper_2406_14066_amd import workloads as W
from paper_2406_14066_amd import spec_verify as sv
from parity_utils import check_attn, check_reject

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def harness():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2406_14066_amd import harness as H
    return H


def _poison_invisible(w, bits_or_value):
    """Overwrite every slot no query may see (page tails past kv_len, spare pages) in place."""
    filler = W.f32_to_bf16_bits(np.float32(W.FILLER)) if w.dtype == "bf16" else np.float32(W.FILLER)
    for pool in (w.k_pages, w.v_pages):
        mask = pool == filler
        # only whole never-visible rows carry the filler in every element
        rows = mask.all(axis=-1)
        pool[rows] = bits_or_value


@pytest.mark.parametrize("layout", [sv.KV_TOKEN_MAJOR, sv.KV_MFMA], ids=["token_major", "tiles"])
@pytest.mark.parametrize("poison", [0x7FC0, 0x7F80, 0xFF80], ids=["nan", "plus_inf", "minus_inf"])
def test_invisible_slots_may_hold_anything(harness, layout, poison):
    print("case poison", hex(poison), layout, flush=True)
    w = W.make_workload("poison", B=4, Hq=8, Hkv=2, d=128, V=64, dtype="bf16", kv_len=[37, 5, 300, 130],
                        k=[3, 0, 8, 2], draft_std=2.0, sigma=1.0, data_seed=19, philox_seed=2)
    clean = oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len)
    _poison_invisible(w, np.uint16(poison))
    assert np.array_equal(oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len), clean)
    ds = harness.DeviceStep(w, kv_layout=layout)
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    check_reject(w, res)


def test_smallest_inputs(harness):
    """One request, one cached token, no draft token; and vocabularies of 4 and 8."""
    print("case smallest", flush=True)
    for V in (4, 8):
        w = W.make_workload("tiny", B=1, Hq=1, Hkv=1, d=128, V=V, dtype="bf16", kv_len=[1], k=[0], draft_std=1.0,
                            sigma=1.0, data_seed=3, philox_seed=4)
        for layout in (sv.KV_TOKEN_MAJOR, sv.KV_MFMA):
            ds = harness.DeviceStep(w, kv_layout=layout)
            ds.run_step()
            res = ds.results()
            check_attn(w, res["out"])
            check_reject(w, res)
            # one key: the output is that key's value row
            v0 = W.bf16_bits_to_f32(w.v_pages[w.block_table[0, 0], 0, 0, :])
            np.testing.assert_allclose(res["out"][0, 0], v0, rtol=0, atol=1e-6)


def test_more_requests_than_the_order_table(harness):
    """Ragged lengths with B above the table size: the attention items keep the given order."""
    print("case many requests", flush=True)
    B = 1100
    rng = np.random.default_rng(5)
    w = W.make_workload("many", B=B, Hq=2, Hkv=1, d=128, V=64, dtype="bf16", kv_len=rng.integers(2, 70, size=B),
                        k=rng.integers(0, 2, size=B), draft_std=2.0, sigma=1.0, data_seed=23, philox_seed=6)
    ds = harness.DeviceStep(w, kv_layout=sv.KV_MFMA)
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    check_reject(w, res)


@pytest.mark.parametrize("V", [12, 2052, 8196, 33000], ids=lambda v: "V%d" % v)
def test_vocabulary_sizes_that_do_not_divide_evenly(harness, V):
    print("case V", V, flush=True)
    w = W.make_workload("vocab", B=6, Hq=1, Hkv=1, d=64, V=V, dtype="f32", kv_len=[16] * 6, k=[0, 1, 3, 8, 5, 2],
                        draft_std=3.0, sigma=0.7, data_seed=V, philox_seed=7, with_kv=False)
    w.k_pages = w.v_pages = np.zeros((1, 1, 16, 64), np.float32)
    w.q = np.zeros((w.T, 1, 64), np.float32)
    for mode in (sv.ACCEPT_SAMPLE, sv.ACCEPT_GREEDY, sv.ACCEPT_POINT_DRAFT):
        ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR, accept_mode=mode)
        ds.run_reject()
        res = ds.results()
        if mode == sv.ACCEPT_SAMPLE:
            check_reject(w, res)
        elif mode == sv.ACCEPT_GREEDY:
            ref = oracle.reject_greedy(w.target_logits, w.draft_tokens, w.cu_q_len)
            np.testing.assert_array_equal(res["accepted_len"], ref.accepted_len)
            np.testing.assert_array_equal(res["next_token"], ref.next_token)
        else:
            ref = oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
            check_reject(w, res, ref=ref)


def test_workspace_reused_across_shapes(harness):
    """A big workspace used by steps of different shapes in turn: whatever one call leaves
    behind (tags, tickets, partials of another geometry) must not disturb the next."""
    import torch
    print("case workspace reuse", flush=True)
    ws = [W.config("c4", B=12, L_scale=0.5, V=4096), W.config("c5", L_scale=0.05, V=8192),
          W.config("c2", B=3, L_scale=0.25, V=4096)]
    steps = [harness.DeviceStep(w, kv_layout=sv.KV_MFMA) for w in ws]
    big = max(s.workspace.numel() for s in steps)
    shared = sv.alloc_workspace(big, "cuda")
    shared.random_(0, 255)      # arbitrary bytes
    first = None
    for rnd in range(3):
        for w, s in zip(ws, steps):
            s.counters.zero_()
            sv.spec_verify_step(s.attn_args, s.reject_args, shared)
            res = s.results()
            check_attn(w, res["out"])
            check_reject(w, res)


@pytest.mark.parametrize("kw,switch,value", [
    (dict(B=1, Hq=4, Hkv=1, d=128, kv_len=[8197], k=[3]), "SPEC_VERIFY_TARGET_BLOCKS", 256),   # one unit cut into a block per compute unit
    (dict(B=2, Hq=8, Hkv=2, d=128, kv_len=[4500, 300], k=[2, 5]), "SPEC_VERIFY_CHUNK", 64),    # short chunks, beside an unsplit request
], ids=["block_target", "chunk_size"])
def test_more_than_64_chunks_take_the_separate_merge_launch(harness, tuning, kw, switch, value):
    """The matrix kernel's last-arriver merge handles up to 64 chunks per request; beyond that the
    partials are merged by a launch of their own.  (The planner itself gets there only beyond
    64 x 4096 tokens in one request; the tuning switches force it at a size the oracle can check.)"""
    print("case many chunks", kw["kv_len"], switch, value, flush=True)
    tuning(switch, value)
    w = W.make_workload("chunks", V=64, dtype="bf16", draft_std=2.0, sigma=1.0, data_seed=31, philox_seed=8, **kw)
    ds = harness.DeviceStep(w, kv_layout=sv.KV_MFMA)
    plan = ds.plan()
    assert plan["attn_path"] == sv.PATH_MFMA and plan["max_chunks"] > 64 and plan["launches"] == 2, plan
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    check_reject(w, res)
    ds.out.fill_(float("nan"))
    ds.run_attn()
    check_attn(w, ds.results()["out"])
