"""What only the device can see -- lengths, block-table entries and draft tokens in device
memory -- is checked by the kernels before it is used: an entry out of range is never turned
into an address, the request or test it belongs to is left out or rejected, and the findings
are counted.  No test here makes the GPU read or write out of bounds: the point is that the
kernels do not, whatever the inputs hold.  Also: a bounded wait that runs out (forced from the
host by a spin limit of one poll) abandons the request cleanly while every block exits."""
import numpy as np
import pytest

import oracle
from paper_2406_14066_amd import workloads as W
from paper_2406_14066_amd import spec_verify as sv
from parity_utils import ATTN_TOL, check_attn, check_reject

pytestmark = pytest.mark.gpu


def _workload(name="robust", **kw):
    base = dict(B=5, Hq=8, Hkv=2, d=128, V=2048, dtype="bf16", kv_len=[300, 45, 1000, 129, 64], k=[3, 1, 4, 0, 2],
                draft_std=2.0, sigma=0.8, data_seed=77, philox_seed=9)
    base.update(kw)
    return W.make_workload(name, **base)


def _rows(w, b):
    return slice(int(w.cu_q_len[b]), int(w.cu_q_len[b + 1]))


@pytest.mark.parametrize("layout", [sv.KV_MFMA, sv.KV_TOKEN_MAJOR], ids=["tiles", "token_major"])
def test_request_with_impossible_lengths_is_left_out_and_counted(layout):
    """Device-side kv_len that the launch was not planned for (longer than the host said, beyond
    the block-table row, shorter than the request's own query rows)."""
    import torch
    from paper_2406_14066_amd.harness import DeviceStep
    print("case bad lengths", layout, flush=True)
    w = _workload()
    ref = oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len)
    for bad_b, bad_len in [(2, 5000), (1, 1), (4, 1 << 30), (0, -7)]:
        ds = DeviceStep(w, kv_layout=layout)
        ds.out.fill_(float("nan"))
        dev_len = w.kv_len.copy()
        dev_len[bad_b] = bad_len
        ds.kv_len.copy_(torch.from_numpy(dev_len))        # the device copy disagrees with the host copy
        ds.run_step()
        res = ds.results()
        assert res["counters"][6] == 1, res["counters"]
        assert np.isnan(res["out"][_rows(w, bad_b)]).all()                 # never written
        ok = np.ones(w.T, dtype=bool)
        ok[_rows(w, bad_b)] = False
        err = np.abs(res["out"][ok].astype(np.float64) - ref[ok]).max()
        assert err <= ATTN_TOL["bf16"], err
        check_reject(w, res, input_errors=1)                               # the other half does not depend on kv_len


@pytest.mark.parametrize("layout", [sv.KV_MFMA, sv.KV_TOKEN_MAJOR], ids=["tiles", "token_major"])
def test_block_table_entry_outside_the_pool_reads_as_zeros_and_is_counted(layout):
    import torch
    from paper_2406_14066_amd.harness import DeviceStep
    print("case bad page", layout, flush=True)
    w = _workload()
    ds = DeviceStep(w, kv_layout=layout)
    table = w.block_table.copy()
    table[2, 7] = w.num_blocks + 5          # request 2, tokens 112..127
    table[2, 30] = -3                       # tokens 480..495
    table[0, 18] = 1 << 30                  # request 0's last page (tokens 288..299)
    ds.block_table.copy_(torch.from_numpy(table))
    ds.run_step()
    res = ds.results()
    assert res["counters"][6] == 3, res["counters"]
    assert np.isfinite(res["out"]).all()
    # what the kernels computed: the same attention with those pages holding zeros
    wz = _workload()
    spare = [p for p in range(w.num_blocks) if p not in set(w.block_table.ravel().tolist())][:3]
    for (b, i), p in zip([(2, 7), (2, 30), (0, 18)], spare):
        wz.block_table[b, i] = p
        wz.k_pages[p] = 0
        wz.v_pages[p] = 0
    ref = oracle.verify_attn(wz.q, wz.k_pages, wz.v_pages, wz.block_table, wz.kv_len, wz.cu_q_len)
    err = np.abs(res["out"].astype(np.float64) - ref).max()
    assert err <= ATTN_TOL["bf16"], err


@pytest.mark.parametrize("mode", [sv.ACCEPT_SAMPLE, sv.ACCEPT_GREEDY, sv.ACCEPT_POINT_DRAFT],
                         ids=["sample", "greedy", "point_draft"])
def test_draft_token_outside_the_vocabulary_is_rejected_and_counted(mode):
    import torch
    from paper_2406_14066_amd.harness import DeviceStep
    print("case bad token", mode, flush=True)
    w = _workload(sigma=0.0 if mode == sv.ACCEPT_SAMPLE else 0.8)     # identical draft and target: everything else is accepted
    if mode != sv.ACCEPT_SAMPLE:
        w.draft_tokens = np.array([int(np.argmax(w.target_logits[int(w.cu_q_len[b]) + i]))
                                   for b in range(w.B) for i in range(int(w.q_len[b]) - 1)], dtype=np.int32)
    ds = DeviceStep(w, kv_layout=sv.KV_MFMA, accept_mode=mode, with_debug=False)
    tok = w.draft_tokens.copy()
    d0 = lambda b: int(w.cu_q_len[b]) - b
    tok[d0(0) + 1] = w.V            # request 0, position 1
    tok[d0(2) + 0] = -1             # request 2, position 0
    tok[d0(2) + 3] = 1 << 30        # request 2, position 3 (after the first rejection: counted all the same)
    ds.draft_tokens.copy_(torch.from_numpy(tok))
    ds.run_reject()
    res = ds.results()
    assert res["counters"][6] == 3, res["counters"]
    assert res["counters"][7] == 0
    if mode == sv.ACCEPT_GREEDY:
        ref = oracle.reject_greedy(w.target_logits, w.draft_tokens, w.cu_q_len)
    elif mode == sv.ACCEPT_POINT_DRAFT:
        ref = oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
    else:
        ref = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
    # requests without a bad token: exactly the oracle's result on the clean inputs
    for b in (1, 3, 4):
        assert res["accepted_len"][b] == ref.accepted_len[b] and res["next_token"][b] == ref.next_token[b]
    if mode != sv.ACCEPT_POINT_DRAFT:
        # (greedy: the drafts are the arg-max tokens; sample: draft == target, so p/q = 1 > u)
        np.testing.assert_array_equal(ref.accepted_len, w.k)
        assert res["accepted_len"][0] == 1 and res["accepted_len"][2] == 0     # the chain stops at the bad token
    else:
        assert res["accepted_len"][0] <= 1 and res["accepted_len"][2] == 0
    assert (res["next_token"] >= 0).all() and (res["next_token"] < w.V).all()
    for b in (0, 2):
        m = int(res["accepted_len"][b])
        assert (res["out_tokens"][b, :m] == w.draft_tokens[d0(b): d0(b) + m]).all()
        assert res["out_tokens"][b, m] == res["next_token"][b] and (res["out_tokens"][b, m + 1:] == -1).all()


def test_kv_append_skips_rows_that_would_land_outside():
    import torch
    print("case bad append", flush=True)
    w = _workload()
    dev = "cuda"
    rng = np.random.default_rng(3)
    new_k = W.f32_to_bf16_bits(rng.standard_normal((w.T, w.Hkv, w.d), dtype=np.float32))
    new_v = W.f32_to_bf16_bits(rng.standard_normal((w.T, w.Hkv, w.d), dtype=np.float32))
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    kc, vc = to_dev(w.k_pages), to_dev(w.v_pages)
    table = w.block_table.copy()
    last = lambda b: (int(w.kv_len[b]) - 1) // 16
    table[1, last(1)] = w.num_blocks              # request 1's q_len = 2 rows land in this page
    err = torch.zeros(1, dtype=torch.int64, device=dev)
    sv.spec_kv_append(to_dev(new_k), to_dev(new_v), kc, vc, torch.from_numpy(table).to(dev),
                      torch.from_numpy(w.kv_len).to(dev), torch.from_numpy(w.cu_q_len).to(dev), w.kv_len, w.cu_q_len,
                      kv_layout=sv.KV_TOKEN_MAJOR, error_count=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 2
    # every other row arrived; the page of the bad entry's rightful owner was not touched
    ek, ev = oracle.kv_append(new_k, new_v, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len, layout=0)
    gk = kc.view(torch.int16).cpu().numpy().view(np.uint16)
    gv = vc.view(torch.int16).cpu().numpy().view(np.uint16)
    keep = np.ones(w.num_blocks, dtype=bool)
    keep[w.block_table[1, last(1)]] = False
    np.testing.assert_array_equal(gk[keep], ek.reshape(gk.shape)[keep])
    np.testing.assert_array_equal(gv[keep], ev.reshape(gv.shape)[keep])
    np.testing.assert_array_equal(gk[~keep], w.k_pages[~keep])


def test_a_wait_that_runs_out_abandons_the_request_and_every_block_exits(tuning):
    """SPEC_VERIFY_SPIN_LIMIT=1 lets every bounded wait give up after one poll.  Whether a consumer
    block then finds its producers' records depends on timing; either way every request ends up
    with the oracle's result or with -1 in all its outputs and a count in counters[7], and the
    next call on the same workspace (normal limit) is not disturbed by what was left behind."""
    from paper_2406_14066_amd.harness import DeviceStep
    print("case spin limit", flush=True)
    w = W.make_workload("spin", B=48, Hq=1, Hkv=1, d=64, V=32000, dtype="f32", kv_len=[16] * 48, k=[4] * 48,
                        draft_std=3.0, sigma=0.8, data_seed=5, philox_seed=11, with_kv=False)
    w.k_pages = w.v_pages = np.zeros((1, 1, 16, 64), np.float32)
    w.q = np.zeros((w.T, 1, 64), np.float32)
    ref = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
    ds = DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR)
    tuning("SPEC_VERIFY_SPIN_LIMIT", 1)
    ds.run_reject()
    res = ds.results()
    gone = res["accepted_len"] < 0
    print("abandoned %d of %d requests" % (gone.sum(), w.B), flush=True)
    assert res["counters"][7] == gone.sum()
    assert (res["next_token"][gone] == -1).all() and (res["out_tokens"][gone] == -1).all()
    np.testing.assert_array_equal(res["accepted_len"][~gone], ref.accepted_len[~gone])
    np.testing.assert_array_equal(res["next_token"][~gone], ref.next_token[~gone])
    assert res["counters"][5] == (~gone).sum() and res["counters"][1] == ref.accepted_len[~gone].sum()
    tuning("SPEC_VERIFY_SPIN_LIMIT", 1 << 20)
    ds.counters.zero_()
    ds.run_reject()
    check_reject(w, ds.results(), ref=ref)
