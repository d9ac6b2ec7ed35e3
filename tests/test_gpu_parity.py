"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Attention: max abs error <= 2e-3 (bf16 KV, fp32 accumulation) or
<= 1e-5 (fp32).  Accepted lengths and tokens: bit-exact outside near-ties."""
import zlib

import numpy as np
import pytest

import oracle
from paper_2406_14066_amd import workloads as W
from paper_2406_14066_amd import spec_verify as sv
from parity_utils import check_attn, check_reject, oracle_reject

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def harness():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2406_14066_amd import harness as H
    return H


def _run(harness, w, layout, what="step"):
    ds = harness.DeviceStep(w, kv_layout=layout)
    getattr(ds, "run_" + what)()
    return ds, ds.results()


def test_c1_tiny_fp32(harness):
    w = W.config("c1")
    print("case c1 fp32 token-major", flush=True)
    ds, res = _run(harness, w, sv.KV_TOKEN_MAJOR)
    err = check_attn(w, res["out"])
    info = check_reject(w, res)
    _assert_nothing_excluded(info)
    print("c1: attn err %.2e near ties %d" % (err, info["near_ties"]))


SMALL = [
    # name, kwargs of make_workload
    ("mha_ragged", dict(B=3, Hq=4, Hkv=4, d=128, kv_len=[37, 16, 300], k=[3, 0, 8])),
    ("gqa4", dict(B=4, Hq=8, Hkv=2, d=128, kv_len=[5, 130, 64, 257], k=[4, 1, 2, 7])),
    ("gqa8_k2", dict(B=5, Hq=16, Hkv=2, d=128, kv_len=[700, 3, 255, 256, 1025], k=[2, 2, 2, 2, 2])),
    ("decode_only", dict(B=3, Hq=4, Hkv=2, d=128, kv_len=[1, 17, 515], k=[0, 0, 0])),
    ("d64", dict(B=2, Hq=4, Hkv=2, d=64, kv_len=[90, 33], k=[5, 2])),
    ("many_rows", dict(B=2, Hq=16, Hkv=2, d=128, kv_len=[129, 400], k=[8, 6])),   # 72 rows per KV head
]

# more than 48 fused rows per KV head: the block's wavefronts split the rows (2 or 4 wave groups) on the matrix path
ROW_GROUP_CASES = [
    # name, kwargs, row tiles per wave group, wave groups per block
    ("g8_k8_k6", dict(B=2, Hq=16, Hkv=2, d=128, kv_len=[129, 400], k=[8, 6]), 3, 2),          # 72 and 56 rows
    ("g8_k7_split", dict(B=3, Hq=16, Hkv=2, d=128, kv_len=[3000, 517, 1999], k=[7, 7, 7]), 2, 2),   # 64 rows, requests split into chunks
    ("g16_k8", dict(B=2, Hq=16, Hkv=1, d=128, kv_len=[700, 90], k=[8, 8]), 3, 4),             # 144 rows
    ("g16_k6_long", dict(B=2, Hq=16, Hkv=1, d=128, kv_len=[5000, 1300], k=[6, 6]), 2, 4),     # 112 rows, chunks of at most 1024 tokens
    ("g16_ragged_k", dict(B=5, Hq=32, Hkv=2, d=128, kv_len=[64, 1500, 9, 333, 2048], k=[8, 0, 3, 5, 2]), 3, 4),  # requests that fill 1, 2 and 4 groups
    ("c4_shape_k7", dict(B=20, Hq=64, Hkv=8, d=128, kv_len=[256 + 37 * i for i in range(20)], k=[7] * 20), 2, 2),
]


@pytest.mark.parametrize("layout", [sv.KV_MFMA, sv.KV_TOKEN_MAJOR], ids=["mfma", "token_major"])
@pytest.mark.parametrize("name,kw,tiles,groups", ROW_GROUP_CASES, ids=[c[0] for c in ROW_GROUP_CASES])
def test_many_rows_stay_on_the_matrix_path(harness, name, kw, tiles, groups, layout):
    print("case row groups", name, "layout", layout, flush=True)
    w = W.make_workload(name, V=64, dtype="bf16", draft_std=2.0, sigma=1.0, data_seed=zlib.crc32(name.encode()) % 1000,
                        philox_seed=3, **kw)
    ds = harness.DeviceStep(w, kv_layout=layout)
    plan = ds.plan()
    assert plan["attn_path"] == sv.PATH_MFMA and plan["row_tiles"] == tiles and plan["row_groups"] == groups, plan
    ds.run_attn()
    err = check_attn(w, ds.results()["out"])
    # the whole step through the same path, and a second call on the same workspace
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    check_reject(w, res)
    print("%s: attn err %.2e, plan %s" % (name, err, plan))


@pytest.mark.parametrize("layout", [sv.KV_TOKEN_MAJOR, sv.KV_MFMA], ids=["token_major", "mfma"])
@pytest.mark.parametrize("name,kw", SMALL, ids=[s[0] for s in SMALL])
def test_small_bf16_attention(harness, name, kw, layout):
    print("case small bf16", name, "layout", layout, flush=True)
    w = W.make_workload(name, V=64, dtype="bf16", draft_std=2.0, sigma=1.0, data_seed=zlib.crc32(name.encode()) % 1000,
                        philox_seed=3, **kw)
    ds, res = _run(harness, w, layout, "attn")
    err = check_attn(w, res["out"])
    print("%s layout %d: attn err %.2e" % (name, layout, err))


@pytest.mark.parametrize("name,kw", [
    ("f32_gqa", dict(B=3, Hq=6, Hkv=2, d=64, kv_len=[37, 260, 16], k=[3, 8, 0])),
    ("f32_d128", dict(B=2, Hq=2, Hkv=2, d=128, kv_len=[513, 31], k=[1, 4])),
])
def test_small_fp32_attention(harness, name, kw):
    print("case small fp32", name, flush=True)
    w = W.make_workload(name, V=64, dtype="f32", draft_std=2.0, sigma=1.0, data_seed=5, philox_seed=3, **kw)
    ds, res = _run(harness, w, sv.KV_TOKEN_MAJOR, "attn")
    check_attn(w, res["out"])


REJECT_CASES = [
    ("v8", dict(B=7, V=8, k=[0, 1, 2, 3, 4, 8, 8], sigma=1.0)),
    ("v1024", dict(B=16, V=1024, k=[4] * 16, sigma=1.0)),
    ("v4100", dict(B=5, V=4100, k=[8, 0, 3, 1, 6], sigma=0.5)),
    ("v32000_mixed", dict(B=12, V=32000, k=[0, 1, 2, 3, 4, 5, 6, 7, 8, 8, 4, 2], sigma=0.8)),
    ("identical", dict(B=6, V=2048, k=[0, 2, 4, 6, 8, 5], sigma=0.0)),
    ("far_apart", dict(B=6, V=2048, k=[3] * 6, sigma=4.0)),
]


@pytest.mark.parametrize("name,kw", REJECT_CASES, ids=[c[0] for c in REJECT_CASES])
def test_reject_sample_small(harness, name, kw):
    print("case reject", name, flush=True)
    B = kw["B"]
    total_near = 0
    for step in range(3):
        w = W.make_workload(name, B=B, Hq=1, Hkv=1, d=64, V=kw["V"], dtype="f32", kv_len=[16] * B, k=kw["k"],
                            draft_std=3.0, sigma=kw["sigma"], data_seed=17 + step, philox_seed=0xABCDEF0123456789,
                            philox_step=(5 << 32) + step, with_kv=False)
        w.k_pages = w.v_pages = np.zeros((1, 1, 16, 64), np.float32)
        w.q = np.zeros((w.T, 1, 64), np.float32)
        ds, res = _run(harness, w, sv.KV_TOKEN_MAJOR, "reject")
        info = check_reject(w, res)
        total_near += info["near_ties"]
        if name == "identical":
            np.testing.assert_array_equal(res["accepted_len"], w.k)
    print("%s: near ties %d" % (name, total_near))


EARLY_STOP_CASES = [
    ("k1_v1024", dict(B=16, V=1024, k=1, sigma=1.0)),
    ("k4_v4100", dict(B=9, V=4100, k=4, sigma=0.8)),
    ("k8_v32000", dict(B=6, V=32000, k=8, sigma=0.6)),
    ("k3_identical", dict(B=5, V=2048, k=3, sigma=0.0)),
    ("k3_far_apart", dict(B=7, V=2048, k=3, sigma=4.0)),
]


@pytest.mark.parametrize("name,kw", EARLY_STOP_CASES, ids=[c[0] for c in EARLY_STOP_CASES])
def test_reject_sample_with_early_stop(harness, tuning, name, kw):
    """The statistics pass in position order, skipping the rows after a request's first rejection
    (the library chooses it for large batches only; the switch forces it here)."""
    print("case early stop", name, flush=True)
    tuning("SPEC_VERIFY_EARLY_STOP", 1)
    B = kw["B"]
    for step in range(3):
        w = W.make_workload(name, B=B, Hq=1, Hkv=1, d=64, V=kw["V"], dtype="f32", kv_len=[16] * B, k=[kw["k"]] * B,
                            draft_std=3.0, sigma=kw["sigma"], data_seed=29 + step, philox_seed=0x1234567,
                            philox_step=(9 << 32) + step, with_kv=False)
        w.k_pages = w.v_pages = np.zeros((1, 1, 16, 64), np.float32)
        w.q = np.zeros((w.T, 1, 64), np.float32)
        ds, res = _run(harness, w, sv.KV_TOKEN_MAJOR, "reject")
        check_reject(w, res)
        if name == "k3_identical":
            np.testing.assert_array_equal(res["accepted_len"], w.k)
        # a second call on the same workspace (the placeholder records were cleared)
        ds.counters.zero_()
        ds.run_reject()
        check_reject(w, ds.results())


def test_whole_step_with_early_stop(harness, tuning):
    print("case early stop, fused step", flush=True)
    tuning("SPEC_VERIFY_EARLY_STOP", 1)
    w = W.config("c4", B=24, L_scale=0.5)
    ds, res = _run(harness, w, sv.KV_MFMA)
    check_attn(w, res["out"])
    check_reject(w, res)


@pytest.mark.parametrize("name,kw,tiles", [("c2", dict(B=4, L_scale=0.5), 1), ("c4", dict(B=32, L_scale=0.5, V=4096), 2),
                                           ("c5", dict(L_scale=0.1, V=8192), 3)], ids=["c2_small", "c4_small", "c5_small"])
def test_token_major_pages_on_the_matrix_path(harness, name, kw, tiles):
    """bf16 token-major pages ([16 tokens][128 dims]): K loaded straight into operand order, V transposed
    through LDS; the whole step in one launch, one, two and three row tiles."""
    print("case token-major matrix path", name, flush=True)
    w = W.config(name, **kw)
    ds = harness.DeviceStep(w, kv_layout=sv.KV_TOKEN_MAJOR)
    plan = ds.plan()
    assert plan["attn_path"] == sv.PATH_MFMA and plan["row_tiles"] == tiles and plan["launches"] == 1, plan
    ds.run_step()
    res = ds.results()
    err = check_attn(w, res["out"])
    check_reject(w, res)
    ds.out.fill_(float("nan"))
    ds.run_attn()
    check_attn(w, ds.results()["out"])
    print("%s token-major: attn err %.2e" % (name, err))


@pytest.mark.parametrize("layout", [sv.KV_TOKEN_MAJOR, sv.KV_MFMA], ids=["token_major", "tiles"])
@pytest.mark.parametrize("name", ["gqa8_k2", "d64", "many_rows"])
def test_bf16_on_the_generic_kernels(harness, tuning, name, layout):
    """The scalar kernels read bf16 pages in both layouts too (the planner takes them for fp32 only; the
    switch forces them): unsplit and split requests, the whole step."""
    print("case forced generic", name, "layout", layout, flush=True)
    tuning("SPEC_VERIFY_FORCE_GENERIC", 1)
    kw = dict(SMALL)[name]
    w = W.make_workload(name, V=64, dtype="bf16", draft_std=2.0, sigma=1.0, data_seed=zlib.crc32(name.encode()) % 1000,
                        philox_seed=3, **kw)
    ds = harness.DeviceStep(w, kv_layout=layout)
    assert ds.plan()["attn_path"] == sv.PATH_GENERIC
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    check_reject(w, res)


D64_CASES = [
    # name, kwargs, row tiles, tuning switch
    ("d64_mha", dict(B=3, Hq=4, Hkv=4, d=64, kv_len=[37, 16, 300], k=[3, 0, 8]), 1, None),
    ("d64_gqa4_split", dict(B=3, Hq=8, Hkv=2, d=64, kv_len=[3000, 517, 1999], k=[7, 2, 5]), 2, None),
    ("d64_gqa8", dict(B=2, Hq=16, Hkv=2, d=64, kv_len=[700, 90], k=[5, 4]), 3, None),
    ("d64_many_chunks", dict(B=2, Hq=8, Hkv=2, d=64, kv_len=[1500, 260], k=[8, 1]), 3, ("SPEC_VERIFY_CHUNK", 64)),    # 24 chunks: three merge passes
    ("d64_merge_launch", dict(B=2, Hq=4, Hkv=2, d=64, kv_len=[4500, 300], k=[2, 5]), 1, ("SPEC_VERIFY_CHUNK", 64)),    # 71 chunks: merged by a launch of its own
    ("d64_two_groups", dict(B=3, Hq=16, Hkv=2, d=64, kv_len=[3000, 517, 1999], k=[7, 7, 6]), 2, None),                  # 64 rows: two wave groups, split requests
    ("d64_four_groups", dict(B=2, Hq=16, Hkv=1, d=64, kv_len=[700, 90], k=[8, 8]), 3, None),                           # 144 rows: four wave groups
]


@pytest.mark.parametrize("layout", [sv.KV_MFMA, sv.KV_TOKEN_MAJOR], ids=["tiles", "token_major"])
@pytest.mark.parametrize("name,kw,tiles,switch", D64_CASES, ids=[c[0] for c in D64_CASES])
def test_head_dim_64_on_the_matrix_path(harness, tuning, name, kw, tiles, switch, layout):
    """bf16 with a head dim of 64, in both page layouts: half the matrix instructions per page, 2 KB per
    (page, KV head); unsplit, split with the in-kernel merge, split with the merge launch, wave groups."""
    print("case head dim 64", name, "layout", layout, flush=True)
    if switch:
        tuning(*switch)
    w = W.make_workload(name, V=64, dtype="bf16", draft_std=2.0, sigma=1.0, data_seed=zlib.crc32(name.encode()) % 1000,
                        philox_seed=3, **kw)
    ds = harness.DeviceStep(w, kv_layout=layout)
    plan = ds.plan()
    assert plan["attn_path"] == sv.PATH_MFMA and plan["row_tiles"] == tiles, plan
    assert plan["row_groups"] == {"d64_two_groups": 2, "d64_four_groups": 4}.get(name, 1), plan
    ds.run_attn()
    err = check_attn(w, ds.results()["out"])
    ds.out.fill_(float("nan"))
    ds.run_step()
    res = ds.results()
    check_attn(w, res["out"])
    check_reject(w, res)
    print("%s: attn err %.2e, plan %s" % (name, err, plan))


def test_counters_accumulate_and_runs_are_deterministic(harness):
    print("case determinism", flush=True)
    w = W.config("c2", B=2, L_scale=0.25)
    ds, res1 = _run(harness, w, sv.KV_MFMA)
    ds.run_step()
    res2 = ds.results()
    np.testing.assert_array_equal(res1["out"], res2["out"])
    np.testing.assert_array_equal(res1["next_token"], res2["next_token"])
    np.testing.assert_array_equal(res1["accepted_len"], res2["accepted_len"])
    np.testing.assert_array_equal(res2["counters"], 2 * res1["counters"])


@pytest.mark.parametrize("switches", [
    {"SPEC_VERIFY_REJECT_FIRST_LIMIT": 0},                                      # attention blocks first (or mixed) instead of rejection first
    {"SPEC_VERIFY_ATTN_FIRST_LIMIT": 0, "SPEC_VERIFY_REJECT_FIRST_LIMIT": 0},   # rejection rows mixed among the attention rows
    {"SPEC_VERIFY_REJECT_EVEN": 0, "SPEC_VERIFY_REJECT_FIRST_LIMIT": 0},        # rejection blocks on all XCDs
    {"SPEC_VERIFY_TARGET_BLOCKS": 512},                                         # more, shorter chunks
], ids=["attention_first", "mixed", "all_xcds", "more_chunks"])
def test_the_grid_order_and_the_split_change_no_decision(harness, tuning, switches):
    """Where a block sits in the grid is a matter of speed only: with every order the planner can
    choose the step gives the same decisions, and the same output bits unless the split changes."""
    print("case grid order", switches, flush=True)
    w = W.config("c4", B=12, L_scale=0.5, V=4096)
    ds, base = _run(harness, w, sv.KV_MFMA)
    check_attn(w, base["out"])
    check_reject(w, base)
    for name, value in switches.items():
        tuning(name, value)
    ds2, res = _run(harness, w, sv.KV_MFMA)
    check_attn(w, res["out"])
    check_reject(w, res)
    for key in ("accepted_len", "next_token", "counters"):
        np.testing.assert_array_equal(res[key], base[key], err_msg=key)
    if "SPEC_VERIFY_TARGET_BLOCKS" not in switches:
        np.testing.assert_array_equal(res["out"], base["out"])


def test_c2_full(harness):
    w = W.config("c2")
    print("case c2 full", flush=True)
    ds, res = _run(harness, w, sv.KV_MFMA)
    err = check_attn(w, res["out"])
    info = check_reject(w, res)
    _assert_nothing_excluded(info)
    print("c2: attn err %.2e near ties %d min race margin %.2e" % (err, info["near_ties"], info["min_race_margin"]))


def _assert_nothing_excluded(info):
    # on the five named workloads no decision is a near tie: every request is compared bit for bit
    assert info["excluded"] == 0 and info["near_accept"] == 0 and info["near_race"] == 0, info


C3_POINTS = [(k, 0.7) for k in range(9)] + [(4, 0.5), (4, 0.9), (8, 0.9), (1, 0.5)]


@pytest.mark.parametrize("k,alpha", C3_POINTS, ids=["k%d_a%.1f" % p for p in C3_POINTS])
def test_c3_sweep_points(harness, k, alpha):
    """Every speculation length of the sweep at one acceptance level, and the three levels at one
    length: the whole attention output (all 32 requests) and every decision against the oracle."""
    w = W.config("c3", k=k, alpha=alpha)
    print("case c3 k=%d alpha=%.1f" % (k, alpha), flush=True)
    ds, res = _run(harness, w, sv.KV_MFMA)
    err = check_attn(w, res["out"])
    info = check_reject(w, res)
    _assert_nothing_excluded(info)
    # accepted-token count against Eq. 4's general form at the measured per-row acceptance probabilities
    if k > 0:
        expect = 0.0
        for b in range(w.B):
            prod = 1.0
            for i in range(k):
                prod *= oracle.accept_probability(w.target_logits[b * (k + 1) + i], w.draft_logits[b * k + i])
                expect += prod
        got = int(res["counters"][1])
        print("c3 k=%d alpha=%.1f: accepted %d, Eq.4 expectation %.1f, attn err %.2e" % (k, alpha, got, expect, err))
        assert abs(got - expect) < 5.0 * np.sqrt(w.B * k) + 1
    else:
        assert res["counters"][1] == 0 and res["counters"][3] == w.B


def test_c4_full(harness):
    """All 256 ragged requests: the whole attention output and every decision against the oracle."""
    w = W.config("c4")
    print("case c4 full", flush=True)
    ds, res = _run(harness, w, sv.KV_MFMA)
    err = check_attn(w, res["out"])
    info = check_reject(w, res)
    _assert_nothing_excluded(info)
    print("c4: attn err %.2e near ties %d min race margin %.2e" % (err, info["near_ties"], info["min_race_margin"]))


def test_c4_shape_at_k7_full(harness, layout=sv.KV_MFMA):
    """The c4 batch at k = 7 as bench.py times it (64 fused rows per KV head: two wave groups; statistics
    in position order): the whole attention output and every decision against the oracle."""
    w = W.config("c4", k=7)
    print("case c4 at k=7 full, layout", layout, flush=True)
    ds = harness.DeviceStep(w, kv_layout=layout)
    plan = ds.plan()
    assert (plan["attn_path"], plan["row_tiles"], plan["row_groups"], plan["launches"], plan["early_stop"]) == (sv.PATH_MFMA, 2, 2, 1, 1), plan
    ds.run_step()
    res = ds.results()
    err = check_attn(w, res["out"])
    info = check_reject(w, res)
    _assert_nothing_excluded(info)
    print("c4 at k=7: attn err %.2e near ties %d min race margin %.2e" % (err, info["near_ties"], info["min_race_margin"]))


def test_c5_full(harness):
    w = W.config("c5")
    print("case c5 full", w.kv_len, w.q_len, flush=True)
    ds, res = _run(harness, w, sv.KV_MFMA)
    err = check_attn(w, res["out"])
    info = check_reject(w, res)
    _assert_nothing_excluded(info)
    print("c5: attn err %.2e near ties %d min race margin %.2e" % (err, info["near_ties"], info["min_race_margin"]))
