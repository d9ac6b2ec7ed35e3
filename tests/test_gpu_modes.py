"""GPU parity of the two other acceptance rules against the CPU oracle: greedy acceptance
(Section 2.2 of the paper) and stochastic acceptance against a point-mass draft (proposers
without a distribution, Section 7).  Greedy results must be bit-exact; the stochastic
rule is bit-exact outside near-ties."""
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


def _logits_only(name, B, V, k, seed, step):
    w = W.make_workload(name, B=B, Hq=1, Hkv=1, d=64, V=V, dtype="f32", kv_len=[16] * B, k=k, draft_std=3.0,
                        sigma=0.8, data_seed=seed, philox_seed=0x1234567 + seed, philox_step=(3 << 32) + step,
                        with_kv=False)
    w.k_pages = w.v_pages = np.zeros((1, 1, 16, 64), np.float32)
    w.q = np.zeros((w.T, 1, 64), np.float32)
    return w


def _mostly_argmax_tokens(w, seed, hit=0.7):
    """Draft tokens that equal the target row's arg-max with probability `hit` (so that
    greedy acceptance produces runs of every length)."""
    rng = np.random.default_rng(seed)
    toks = w.draft_tokens.copy()
    for b in range(w.B):
        for i in range(int(w.q_len[b]) - 1):
            if rng.random() < hit:
                toks[int(w.cu_q_len[b]) - b + i] = int(np.argmax(w.target_logits[int(w.cu_q_len[b]) + i]))
    return toks


def _check_greedy(w, res):
    ref = oracle.reject_greedy(w.target_logits, w.draft_tokens, w.cu_q_len)
    np.testing.assert_array_equal(res["accepted_len"], ref.accepted_len)
    np.testing.assert_array_equal(res["next_token"], ref.next_token)
    np.testing.assert_array_equal(res["out_tokens"], ref.out_tokens)
    np.testing.assert_array_equal(res["counters"], ref.counters)
    return ref


CASES = [
    ("v8", 7, 8, [0, 1, 2, 3, 4, 8, 8]),
    ("v1024", 16, 1024, [4] * 16),
    ("v4100", 5, 4100, [8, 0, 3, 1, 6]),
    ("v32000_mixed", 12, 32000, [0, 1, 2, 3, 4, 5, 6, 7, 8, 8, 4, 2]),
    ("v128256", 3, 128256, [8, 2, 5]),
]


@pytest.mark.parametrize("name,B,V,k", CASES, ids=[c[0] for c in CASES])
def test_greedy_small(harness, name, B, V, k):
    print("case greedy", name, flush=True)
    seen = set()
    for step in range(3):
        w = _logits_only(name, B, V, k, 40 + step, step)
        w.draft_tokens = _mostly_argmax_tokens(w, 7 + step)
        ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR, accept_mode=sv.ACCEPT_GREEDY)
        ds.run_reject()
        ref = _check_greedy(w, ds.results())
        seen.update(ref.accepted_len.tolist())
    assert len(seen) > 1   # the cases exercise more than one accepted length


@pytest.mark.parametrize("B,V,k", [(16, 1024, 1), (7, 4100, 4), (5, 32000, 8), (3, 128256, 3)], ids=["k1", "k4", "k8", "v128256"])
def test_greedy_with_early_stop(harness, tuning, B, V, k):
    """Greedy acceptance with the arg-max pass in position order (rows after a request's first
    mismatch are skipped); the library picks that order for large batches only, the switch forces it."""
    print("case greedy early stop", B, V, k, flush=True)
    tuning("SPEC_VERIFY_EARLY_STOP", 1)
    seen = set()
    for step in range(3):
        w = _logits_only("ges_k%d" % k, B, V, [k] * B, 90 + step, step)
        w.draft_tokens = _mostly_argmax_tokens(w, 17 + step)
        ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR, accept_mode=sv.ACCEPT_GREEDY)
        ds.run_reject()
        ref = _check_greedy(w, ds.results())
        seen.update(ref.accepted_len.tolist())
        ds.counters.zero_()
        ds.run_reject()   # again on the same workspace
        _check_greedy(w, ds.results())
    assert len(seen) > 1


def test_greedy_equal_maxima_take_the_lowest_id(harness):
    print("case greedy ties", flush=True)
    w = _logits_only("ties", 4, 4096, [2, 2, 2, 2], 5, 0)
    # plant equal maxima far apart (different vocabulary segments) in every target row
    rng = np.random.default_rng(1)
    for r in range(w.T):
        ids = rng.choice(4096, size=3, replace=False)
        w.target_logits[r, ids] = 50.0
    w.draft_tokens = _mostly_argmax_tokens(w, 3, hit=0.8)
    ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR, accept_mode=sv.ACCEPT_GREEDY)
    ds.run_reject()
    _check_greedy(w, ds.results())


@pytest.mark.parametrize("name,B,V,k", CASES, ids=[c[0] for c in CASES])
def test_point_draft_small(harness, name, B, V, k):
    print("case point draft", name, flush=True)
    near = 0
    for step in range(3):
        w = _logits_only(name, B, V, k, 60 + step, step)
        if step == 1:   # likely tokens, so that acceptances occur at large V too
            w.draft_tokens = _mostly_argmax_tokens(w, 11, hit=0.9)
        ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR, accept_mode=sv.ACCEPT_POINT_DRAFT)
        ds.run_reject()
        ref = oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
        near += check_reject(w, ds.results(), ref=ref)["near_ties"]
    print("%s: near ties %d" % (name, near))


@pytest.mark.parametrize("B,V,k", [(16, 1024, 1), (7, 4100, 4), (5, 32000, 8)], ids=["k1", "k4", "k8"])
def test_point_draft_with_early_stop(harness, tuning, B, V, k):
    """Point-mass draft with the statistics pass in position order (rows after a request's first
    rejection are skipped); the library picks that order for large batches only, the switch forces it."""
    print("case point draft early stop", B, V, k, flush=True)
    tuning("SPEC_VERIFY_EARLY_STOP", 1)
    for step in range(2):
        w = _logits_only("es_k%d" % k, B, V, [k] * B, 80 + step, step)
        w.draft_tokens = _mostly_argmax_tokens(w, 13 + step, hit=0.8)
        ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR, accept_mode=sv.ACCEPT_POINT_DRAFT)
        ds.run_reject()
        ref = oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
        check_reject(w, ds.results(), ref=ref)


@pytest.mark.parametrize("mode", [sv.ACCEPT_GREEDY, sv.ACCEPT_POINT_DRAFT], ids=["greedy", "point_draft"])
def test_whole_step_in_each_mode(harness, mode):
    """The one-launch step (matrix-instruction attention + the mode's acceptance rule) on a
    GQA workload that spans several blocks per role."""
    print("case step mode", mode, flush=True)
    w = W.config("c4", B=24, L_scale=0.5, V=8192)
    w.draft_tokens = _mostly_argmax_tokens(w, 2, hit=0.6)
    ds = harness.DeviceStep(w, kv_layout=sv.KV_MFMA, accept_mode=mode)
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    if mode == sv.ACCEPT_GREEDY:
        _check_greedy(w, res)
    else:
        ref = oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
        check_reject(w, res, ref=ref)
    # a second call on the same workspace (stale tags of the first) gives the same result
    ds.run_step()
    res2 = ds.results()
    np.testing.assert_array_equal(res2["accepted_len"], res["accepted_len"])
    np.testing.assert_array_equal(res2["next_token"], res["next_token"])
