#!/usr/bin/env python3
"""Benchmark of the speculative-verification step on one MI355X.

A "step" is one pass of the whole hot path -- lookahead attention over the paged KV
cache, then rejection sampling with bonus token -- over one batch of seeded synthetic
input that is already resident in HBM.  The headline workload is the largest of the
named configurations that fits one GPU: c4, the 70B-shaped GQA batch (B=256, L uniform
in [256,1024], k=2, 64/8 heads, d=128, bf16 paged KV, V=32000).  The other named
workloads (c1, c2, a c3 sweep point, c5), a c4-shaped batch at k=7 (more than 48 fused
query rows per KV head), the same steps on token-major pages and the 7B-shaped step with a
single request (bound by latencies) are timed in the same run and reported under "workloads".

KV pools and logits are rotated over several device copies so that consecutive steps
do not find their inputs in the 256 MB last-level cache.

Prints ONE JSON line:
  value      verified token positions per second, sum_b (k_b+1) / t_step
  roofline   achieved HBM rate of the step's kernel (the whole step is one launch):
             algorithmic bytes per launch / mean launch duration measured with HIP
             events attached to the launches of a timed region, against the 8 TB/s peak
             (a second region of K steps: the events cost wall clock, `value` is timed without)
  cpu_baseline  the CPU oracle timed in this same run on this host
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "c4_k7", "c2_one_request"],
                    help="the workload of the headline figures")
    ap.add_argument("--k", type=int, default=None, help="speculation length of the c3 sweep point")
    ap.add_argument("--alpha", type=float, default=None, help="acceptance level of the c3 sweep point")
    ap.add_argument("--rotate", type=int, default=0, help="device copies of KV/logits to cycle through (0 = auto)")
    ap.add_argument("--accept-mode", default="sample", choices=["sample", "greedy", "point"],
                    help="acceptance rule: the stochastic rule (headline), greedy, or stochastic against a point-mass draft")
    ap.add_argument("--setup-steps", type=int, default=300,
                    help="untimed steps before the W warm-up steps: the device needs some tens of milliseconds of "
                         "load to reach its sustained clocks (the first hundred steps of c4 run 2-3%% slower)")
    ap.add_argument("--only", action="store_true", help="time the headline workload only (no \"workloads\" entries)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the same steps")
    ap.add_argument("--events-in-value-region", action="store_true",
                    help="one timed region only: the K steps that give `value` also carry the kernel events "
                         "(an event pair attached to a launch costs about 4 us of wall clock per step)")
    return ap.parse_args()


def traffic_from_profile(workload):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary is committed."""
    path = os.path.join(ROOT, "profiles", "spec_step_kernel_%s_pmc.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def make_workload(name, k=None, alpha=None):
    from paper_2406_14066_amd import workloads as W
    if name == "c3":
        return W.config("c3", k=k, alpha=alpha)
    if name == "c4_k7":
        w = W.config("c4", k=7)
        w.name = "c4_k7"
        return w
    if name == "c2_one_request":   # the 7B-shaped step with a single request: bound by latencies, not by bytes
        w = W.config("c2", B=1)
        w.name = "c2_one_request"
        return w
    return W.config(name)


def describe(w):
    kv = "bf16 paged KV (block 16, shuffled table)" if w.dtype == "bf16" else "fp32 KV (8 consecutive pages of 16)"
    return ("%s: B=%d, L=%s, k=%s, Hq/Hkv=%d/%d, d=%d, %s, V=%d fp32 logits"
            % (w.name, w.B, _span(w.kv_len), _span(w.k), w.Hq, w.Hkv, w.d, kv, w.V))


def measure(w, args, mode, with_graph, token_major=False):
    """Times K steps of workload w: wall clock without events, kernel time with events attached."""
    import torch
    from paper_2406_14066_amd import spec_verify as sv
    from paper_2406_14066_amd.harness import DeviceStep

    # bf16 workloads keep their pages in the matrix-operand layout; the tiny fp32 one (c1) has token-major pages
    layout = sv.KV_MFMA if (w.dtype == "bf16" and not token_major) else sv.KV_TOKEN_MAJOR
    ds = DeviceStep(w, kv_layout=layout, with_debug=False, accept_mode=mode)
    plan = ds.plan()
    attn_bytes = w.attn_algorithmic_bytes()
    # without a draft distribution only the target rows are read
    rej_bytes = w.reject_algorithmic_bytes() if mode == sv.ACCEPT_SAMPLE else w.T * w.V * 4
    step_bytes = attn_bytes + rej_bytes
    kv_bytes = 2 * ds.k_cache.numel() * ds.k_cache.element_size()
    # at least four copies and 4 GB in all: with two copies of a 1 GB workload the 256 MB
    # last-level cache still served a few per cent of the (non-temporal) reads
    nrot = args.rotate or max(4, int(np.ceil(4.0e9 / max(kv_bytes + rej_bytes, 1))))
    nrot = min(nrot, 16)
    variants = ds.rotated(nrot)   # same bytes at different addresses
    stream = torch.cuda.current_stream()

    def run(n, first=0):
        for i in range(n):
            a, r = variants[(first + i) % nrot]
            sv.spec_verify_step(a, r, ds.workspace, stream)

    run(args.setup_steps)
    torch.cuda.synchronize()
    run(args.warmup)
    torch.cuda.synchronize()

    # Two timed regions of exactly K steps each, both bracketed by a device synchronisation.  The
    # first carries nothing but the steps and gives `value`; the second attaches an event pair to
    # every launch (the kernel's own begin and end time stamps) and gives the kernel time of the
    # roofline.  The events are measurement: they cost about 4 us of wall clock per step, which a
    # serving loop would not pay.  --events-in-value-region folds the two into one.
    events_in_region = args.events_in_value_region
    if events_in_region:
        sv.spec_profile_begin(args.steps * 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, first=args.warmup)
    t_enqueued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if events_in_region:
        kt = sv.spec_profile_end()
        sec_per_step_events = (t1 - t0) / args.steps
    else:
        sv.spec_profile_begin(args.steps * 2)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        run(args.steps, first=args.warmup)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        kt = sv.spec_profile_end()
        sec_per_step_events = (t3 - t2) / args.steps
    sec_per_step = (t1 - t0) / args.steps

    # The same steps replayed from one captured HIP graph (one step per rotated copy): what is
    # left of the launch gaps when the host is out of the loop.  Reported beside the eager figure.
    graph_info = None
    if with_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        per_graph = -(-max(args.steps, 1) // nrot) * nrot     # K steps rounded up to whole rounds of the rotated copies
        with torch.cuda.graph(graph, stream=side):
            for i in range(per_graph):
                a, r = variants[i % nrot]
                sv.spec_verify_step(a, r, ds.workspace, torch.cuda.current_stream())
        torch.cuda.synchronize()
        replays = 3
        graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        graph_sec = (g1 - g0) / (replays * per_graph)
        graph_info = {"ms_per_step": graph_sec * 1e3, "value": w.verified_tokens() / graph_sec,
                      "steps": replays * per_graph, "steps_per_graph": per_graph,
                      "achieved_GBps": step_bytes / graph_sec / 1e9}
        del graph
    # the step before the path: this step's K/V rows entering the paged cache (same positions every time)
    append_us = None
    if w.dtype == "bf16":
        nk = torch.randn((w.T, w.Hkv, w.d), device="cuda").to(torch.bfloat16)
        nv = torch.randn((w.T, w.Hkv, w.d), device="cuda").to(torch.bfloat16)
        reps = max(args.steps, 10)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        app, _keep_app = sv.make_kv_append_args(nk, nv, ds.k_cache, ds.v_cache, ds.block_table, ds.kv_len, ds.cu_q_len,
                                                w.kv_len, w.cu_q_len, kv_layout=layout)
        for i in range(reps + 3):
            if i == 3:
                e0.record()
            sv.spec_kv_append_args(app, stream)
        e1.record()
        torch.cuda.synchronize()
        append_us = e0.elapsed_time(e1) * 1e3 / reps
    res = ds.results()
    calls = max(int(res["counters"][5]) // w.B, 1)
    emitted_per_step = int(res["counters"][3]) // calls
    # logit bytes of the rows up to each request's first rejection: what the step needs at least
    # (the library reads no more than these when it takes the statistics pass in position order,
    # which it does for large batches with one draft length)
    m = res["accepted_len"].astype(np.int64)
    kk = w.k.astype(np.int64)
    rows_needed = (2 if mode == sv.ACCEPT_SAMPLE else 1) * np.minimum(m + 1, kk) + (m == kk)
    rej_bytes_needed = int(rows_needed.sum()) * w.V * 4

    kernel_us = {k: (1e3 * ms / n if n else None) for k, (ms, n) in kt.items()}
    # the step is the one launch of the step kernel (plus a merge launch only when a request has more than 64
    # chunks); on the generic path (fp32) it is two or three launches: attention, a merge if a request is split,
    # rejection sampling
    step_us = sum(kernel_us[k] or 0.0 for k in ("step", "attn_generic", "attn_combine", "reject"))
    achieved = step_bytes / (step_us * 1e-6) / 1e9
    out = dict(
        w=w, ds=ds, layout=layout, res=res, plan=plan, nrot=nrot, sec_per_step=sec_per_step, sec_per_step_events=sec_per_step_events,
        host_us_per_call=(t_enqueued - t0) / args.steps * 1e6, kernel_us=kernel_us, step_us=step_us, achieved=achieved,
        attn_bytes=attn_bytes, rej_bytes=rej_bytes, step_bytes=step_bytes, rej_bytes_needed=rej_bytes_needed,
        emitted_per_step=emitted_per_step, graph_info=graph_info, events_in_region=events_in_region,
        kv_append_us=append_us,
        near_tie_accept_tests_per_step=int(res["counters"][4]) // calls,
        input_errors=int(res["counters"][6]), abandoned=int(res["counters"][7]),
    )
    return out


def brief(mm, traffic):
    """One entry of "workloads"."""
    w = mm["w"]
    return {
        "workload": describe(w),
        "verified_tokens_per_step": w.verified_tokens(),
        "value": w.verified_tokens() / mm["sec_per_step"],
        "ms_per_step": mm["sec_per_step"] * 1e3,
        "kernel_us": mm["step_us"],
        "algorithmic_bytes": mm["step_bytes"],
        "achieved_GBps": mm["achieved"],
        "frac": mm["achieved"] / HBM_PEAK_GBS,
        "traffic": traffic,
        "attention_path": {1: "matrix instructions", 2: "generic"}[mm["plan"]["attn_path"]],
        "kv_layout": "token-major pages" if mm["layout"] == 0 else "matrix-operand tiles",
        "row_tiles": mm["plan"]["row_tiles"], "row_groups": mm["plan"]["row_groups"],
        "chunk_tokens": mm["plan"]["chunk_tokens"], "launches": mm["plan"]["launches"],
        "early_stop": mm["plan"]["early_stop"],
        "emitted_tokens_per_step": mm["emitted_per_step"],
        "near_tie_accept_tests_per_step": mm["near_tie_accept_tests_per_step"],
        "rotated_copies": mm["nrot"],
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the step has no multi-GPU path); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_14066_amd import spec_verify as sv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sv.lib()  # fail loudly if the HIP library is missing

    mode = {"sample": sv.ACCEPT_SAMPLE, "greedy": sv.ACCEPT_GREEDY, "point": sv.ACCEPT_POINT_DRAFT}[args.accept_mode]

    # the headline workload first, on a fresh device; then the others (each frees its device memory before the next)
    w = make_workload(args.workload, args.k, args.alpha)
    mm = measure(w, args, mode, with_graph=not args.no_graph)
    del mm["ds"]      # (frees the headline workload's device memory)
    torch.cuda.empty_cache()
    others = {}
    if not args.only:
        if w.dtype == "bf16" and w.d == 128:
            # the same step on token-major pages (V transposed through LDS inside the kernel)
            mo = measure(w, args, mode, with_graph=False, token_major=True)
            others[w.name + "_token_major_pages"] = brief(mo, None)
            del mo
            torch.cuda.empty_cache()
        for name, kw in [("c1", {}), ("c2", {}), ("c3", dict(k=4, alpha=0.7)), ("c5", {}), ("c4_k7", {}), ("c2_one_request", {})]:
            if name == args.workload:
                continue
            wo = make_workload(name, **kw)
            mo = measure(wo, args, mode, with_graph=False)
            others[name] = brief(mo, traffic_from_profile(name) if mode == sv.ACCEPT_SAMPLE else None)
            del mo
            torch.cuda.empty_cache()
            if name in ("c2", "c4_k7"):
                mo = measure(wo, args, mode, with_graph=False, token_major=True)
                others[name + "_token_major_pages"] = brief(mo, None)
                del mo
                torch.cuda.empty_cache()
            del wo
    res = mm["res"]
    sec_per_step = mm["sec_per_step"]
    traffic = traffic_from_profile(args.workload) if mode == sv.ACCEPT_SAMPLE else None

    out = {
        "metric": "verified tokens/s per MI355X for spec-verify step",
        "value": w.verified_tokens() / sec_per_step,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": describe(w),
            "kv_layout": "mfma-tiled pages",
            "accept_mode": args.accept_mode,
            "rotated_copies": mm["nrot"],
            "untimed_setup_steps_before_warmup": args.setup_steps,
            "verified_tokens_per_step": w.verified_tokens(),
            "emitted_tokens_per_step": mm["emitted_per_step"],
            "goodput_tokens_per_s": mm["emitted_per_step"] / sec_per_step,
            "plan": {k: v for k, v in mm["plan"].items()},
        },
        "step_hbm": {
            "algorithmic_bytes": mm["step_bytes"],
            "achieved_GBps": mm["step_bytes"] / sec_per_step / 1e9,
            "frac_of_peak": mm["step_bytes"] / sec_per_step / 1e9 / HBM_PEAK_GBS,
        },
        "kernel_us": mm["kernel_us"],
        "host_us_per_call": mm["host_us_per_call"],
        "kv_append_us_per_call": mm["kv_append_us"],   # back-to-back launches of spec_kv_append for this step's T rows
        "graph_replay": mm["graph_info"],
        "decisions": {
            # counters[4]: evaluated accept tests within 1e-6 of their uniform, per step (counted by the kernel)
            "near_tie_accept_tests_per_step": mm["near_tie_accept_tests_per_step"],
            "device_side_input_errors": mm["input_errors"],
            "abandoned_requests": mm["abandoned"],
        },
        "roofline": {
            "kernel": "spec_step_kernel (whole step in one launch: attention over the paged KV cache + rejection sampling)",
            "bound": "hbm",
            "achieved": mm["achieved"],
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": mm["achieved"] / HBM_PEAK_GBS,
            "traffic": traffic,
            "algorithmic_bytes_per_launch": mm["step_bytes"],
            "attention_bytes": mm["attn_bytes"],
            "rejection_bytes": mm["rej_bytes"],
            "rejection_bytes_up_to_first_rejection": mm["rej_bytes_needed"],
            "events_in_timed_region": True,
            "kernel_time_region": ("the K steps that give value" if mm["events_in_region"] else
                                   "a second timed region of K steps with an event pair attached to every launch"),
            "ms_per_step_with_events": mm["sec_per_step_events"] * 1e3,
        },
        "workloads": others,
    }

    if not args.no_cpu_baseline:
        import oracle
        # The oracle as it stands, single thread, on whole steps of the headline workload until about
        # ten seconds have passed (at least one step).  Its decisions are compared with the GPU's here,
        # and the decisions the oracle marks as near ties are counted.
        reps, t_attn, t_rej = 0, 0.0, 0.0
        ref = None
        while reps == 0 or (t_attn + t_rej < 10.0 and reps < 1000):
            t2 = time.perf_counter()
            oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len)
            t3 = time.perf_counter()
            if mode == sv.ACCEPT_SAMPLE:
                ref = oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, w.philox_seed,
                                           w.philox_step)
            elif mode == sv.ACCEPT_GREEDY:
                ref = oracle.reject_greedy(w.target_logits, w.draft_tokens, w.cu_q_len)
            else:
                ref = oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
            t4 = time.perf_counter()
            t_attn += t3 - t2
            t_rej += t4 - t3
            reps += 1
        out["cpu_baseline"] = {
            "value": reps * w.verified_tokens() / (t_attn + t_rej),
            "unit": "tokens/s",
            "cores": 1,
            "kind": "oracle",
            "sample": "the whole %s step %d times (attention %.2f s + rejection sampling %.2f s per step), single thread; host has %d cpus"
                      % (w.name, reps, t_attn / reps, t_rej / reps, os.cpu_count()),
        }
        near_accept = 0
        if ref.dec_u.size:
            with np.errstate(invalid="ignore"):
                near_accept = int((np.abs(ref.dec_u - ref.dec_ratio) < 1e-6).sum())
        near_race = int((ref.race_margin < 1e-5).sum())
        out["decisions"].update({
            "oracle_near_tie_accept_tests": near_accept,
            "oracle_near_tie_races": near_race,
            "requests_excluded_from_exact_comparison": near_accept + near_race,
            "accepted_len_equal_to_oracle": bool((res["accepted_len"] == ref.accepted_len).all()),
            "next_token_equal_to_oracle": bool((res["next_token"] == ref.next_token).all()),
        })
    print(json.dumps(out))


def _span(a):
    a = np.asarray(a)
    return str(int(a[0])) if (a == a[0]).all() else "%d..%d" % (a.min(), a.max())


if __name__ == "__main__":
    main()
