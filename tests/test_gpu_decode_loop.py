"""A decode loop replayed from ONE captured HIP graph (the paper runs its steps from graphs
captured per batch shape, Section 5.3): KV append, lookahead attention and rejection sampling
are captured once under a length bucket (max_kv_len) and replayed step after step while every
request's kv_len advances by what the previous step accepted, across page and chunk boundaries.
The random numbers advance through a device-side step word.  Every replay is compared bit for
bit with the same calls made eagerly, and with the CPU oracle fed the same inputs."""
import numpy as np
import pytest

import oracle
from paper_2406_14066_amd import workloads as W
from paper_2406_14066_amd import spec_verify as sv
from parity_utils import ATTN_TOL

pytestmark = pytest.mark.gpu


def _bf16_dev(a, dev):
    import torch
    return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)


@pytest.mark.parametrize("Hq,Hkv,k,start", [
    (8, 2, 3, [60, 125, 250, 700, 1000, 62]),          # 16 rows per KV head: one wave group
    (32, 2, 4, [63, 1279, 15, 640]),                   # 80 rows per KV head: two wave groups per block
], ids=["gqa4_k3", "gqa16_k4_row_groups"])
def test_captured_step_survives_a_decode_loop(Hq, Hkv, k, start, tuning):
    import torch
    dev = "cuda"
    tuning("SPEC_VERIFY_CHUNK", 64)   # short chunks, so that the growing requests cross chunk boundaries within a few steps
    B, d, V = len(start), 128, 4096
    q_len = np.full(B, k + 1, dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    T = int(cu[-1])
    max_kv_len = 1408
    steps = 10
    seed = 0xC0FFEE
    print("case decode loop", Hq, Hkv, k, start, flush=True)
    rng = np.random.default_rng(123 + Hq)
    max_blocks = max_kv_len // 16
    num_blocks = B * max_blocks + 7
    table = rng.permutation(num_blocks)[: B * max_blocks].reshape(B, max_blocks).astype(np.int32)

    # host mirror of the paged cache (token-major bf16 bits): everything random, the appends overwrite what they cover
    k_host = W.f32_to_bf16_bits(rng.standard_normal((num_blocks, Hkv, 16, d), dtype=np.float32))
    v_host = W.f32_to_bf16_bits(rng.standard_normal((num_blocks, Hkv, 16, d), dtype=np.float32))
    k_tm, v_tm = _bf16_dev(k_host, dev), _bf16_dev(v_host, dev)
    k_cache, v_cache = torch.empty_like(k_tm), torch.empty_like(v_tm)
    sv.spec_kv_repack_mfma(k_tm, v_tm, k_cache, v_cache)

    lens = np.asarray(start, dtype=np.int32)
    # device buffers that the captured launches read; refilled before every step
    q_dev = torch.zeros((T, Hq, d), dtype=torch.bfloat16, device=dev)
    nk_dev = torch.zeros((T, Hkv, d), dtype=torch.bfloat16, device=dev)
    nv_dev = torch.zeros((T, Hkv, d), dtype=torch.bfloat16, device=dev)
    tl_dev = torch.zeros((T, V), dtype=torch.float32, device=dev)
    dl_dev = torch.zeros((T - B, V), dtype=torch.float32, device=dev)
    tok_dev = torch.zeros(T - B, dtype=torch.int32, device=dev)
    table_dev = torch.from_numpy(table).to(dev)
    len_dev = torch.from_numpy(lens).to(dev)
    cu_dev = torch.from_numpy(cu).to(dev)
    step_dev = torch.zeros(1, dtype=torch.int64, device=dev)
    out = torch.zeros((T, Hq, d), dtype=torch.float32, device=dev)
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    toks = torch.zeros((B, sv.K_MAX + 1), dtype=torch.int32, device=dev)
    new_len = torch.zeros(B, dtype=torch.int32, device=dev)
    draft_next = torch.zeros(B, dtype=torch.int32, device=dev)
    counters = torch.zeros(sv.NUM_COUNTERS, dtype=torch.int64, device=dev)
    append_err = torch.zeros(1, dtype=torch.int64, device=dev)

    # planned once: the bucket bound, the shapes, and the lengths of the moment as a hint
    attn, keep_a = sv.make_attn_args(q_dev, k_cache, v_cache, table_dev, len_dev, cu_dev, out, lens.copy(), cu,
                                     Hkv=Hkv, kv_layout=sv.KV_MFMA, max_kv_len=max_kv_len)
    rej, keep_r = sv.make_reject_args(tl_dev, dl_dev, tok_dev, cu_dev, cu, acc, nxt, counters, philox_seed=seed,
                                      philox_step=999999, out_tokens=toks, kv_len=len_dev, new_kv_len=new_len,
                                      draft_next_len=draft_next, philox_step_device=step_dev)
    plan = sv.spec_verify_plan(attn, rej)
    assert plan["attn_path"] == sv.PATH_MFMA and plan["launches"] == 1, plan
    assert plan["row_groups"] == (2 if Hq // Hkv * (k + 1) > 48 else 1), plan
    ws = sv.alloc_workspace(plan["workspace_bytes"], dev)
    hold_lens = lens.copy()   # (the append's host copies are for validation only)

    def enqueue(stream):
        sv.spec_kv_append(nk_dev, nv_dev, k_cache, v_cache, table_dev, len_dev, cu_dev, hold_lens, cu,
                          kv_layout=sv.KV_MFMA, stream=stream, error_count=append_err)
        sv.spec_verify_step(attn, rej, ws, stream)

    def reset_outputs():
        out.fill_(float("nan"))
        for t in (acc, nxt, toks, new_len, draft_next):
            t.fill_(-9)
        counters.zero_()

    def read():
        torch.cuda.synchronize()
        return dict(out=out.cpu().numpy(), acc=acc.cpu().numpy(), nxt=nxt.cpu().numpy(), toks=toks.cpu().numpy(),
                    new_len=new_len.cpu().numpy(), draft_next=draft_next.cpu().numpy(), counters=counters.cpu().numpy())

    graph = None
    crossed_chunk = crossed_page = 0
    chunk = plan["chunk_tokens"]
    for step in range(steps):
        # this step's inputs
        q = W.f32_to_bf16_bits(rng.standard_normal((T, Hq, d), dtype=np.float32))
        nk = W.f32_to_bf16_bits(rng.standard_normal((T, Hkv, d), dtype=np.float32))
        nv = W.f32_to_bf16_bits(rng.standard_normal((T, Hkv, d), dtype=np.float32))
        tl, dl, tok = W.make_logits(rng, q_len, V, 3.0, 0.5)
        q_dev.copy_(_bf16_dev(q, dev)); nk_dev.copy_(_bf16_dev(nk, dev)); nv_dev.copy_(_bf16_dev(nv, dev))
        tl_dev.copy_(torch.from_numpy(tl)); dl_dev.copy_(torch.from_numpy(dl)); tok_dev.copy_(torch.from_numpy(tok))
        len_dev.copy_(torch.from_numpy(lens))
        step_dev.fill_(step)

        # the oracle's side: append into the mirror, attend, accept
        k_host, v_host = oracle.kv_append(nk, nv, k_host, v_host, table, lens, cu, layout=0)
        ref_out = oracle.verify_attn(q, k_host.reshape(num_blocks, Hkv, 16, d), v_host.reshape(num_blocks, Hkv, 16, d),
                                     table, lens, cu)
        ref = oracle.reject_sample(tl, dl, tok, cu, seed, step)
        ref_new_len, ref_draft_next = oracle.kv_after_accept(lens, cu, ref.accepted_len)

        # eagerly, then from the graph (captured at the first step, after one eager pass)
        reset_outputs()
        enqueue(None)
        eager = read()
        if graph is None:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                enqueue(torch.cuda.current_stream())
            torch.cuda.synchronize()
        reset_outputs()
        graph.replay()
        got = read()

        for key in eager:
            np.testing.assert_array_equal(got[key], eager[key], err_msg="step %d: %s" % (step, key))
        err = np.abs(got["out"].astype(np.float64) - ref_out.astype(np.float64)).max()
        assert err <= ATTN_TOL["bf16"], (step, err)
        assert ref.race_margin.min() > 1e-5 and not np.any(np.abs(ref.dec_u - ref.dec_ratio) < 1e-6)   # nothing near a tie
        np.testing.assert_array_equal(got["acc"], ref.accepted_len, err_msg="step %d" % step)
        np.testing.assert_array_equal(got["nxt"], ref.next_token, err_msg="step %d" % step)
        np.testing.assert_array_equal(got["toks"], ref.out_tokens)
        np.testing.assert_array_equal(got["new_len"], ref_new_len)
        np.testing.assert_array_equal(got["draft_next"], ref_draft_next)
        np.testing.assert_array_equal(got["counters"][:6], ref.counters[:6])
        assert got["counters"][6] == 0 and got["counters"][7] == 0 and int(append_err.item()) == 0

        # the next step scores the emitted token and k new draft tokens on top of what was kept
        nxt_lens = ref_new_len + q_len
        crossed_chunk += int(((nxt_lens - 1) // chunk != (lens - 1) // chunk).sum())
        crossed_page += int(((nxt_lens - 1) // 16 != (lens - 1) // 16).sum())
        lens = nxt_lens.astype(np.int32)
        assert lens.max() <= max_kv_len
    print("decode loop: %d chunk and %d page boundaries crossed; final lengths %s" % (crossed_chunk, crossed_page, lens))
    assert crossed_chunk >= 2 and crossed_page >= 5
