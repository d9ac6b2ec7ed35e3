#!/usr/bin/env python3
"""Benchmark of the speculative-verification step on one MI355X.

A "step" is one pass of the whole hot path -- lookahead attention over the paged KV
cache, then rejection sampling with bonus token -- over one batch of seeded synthetic
input that is already resident in HBM.  The default workload is the Llama-2-7B-shaped
single-layer verify (B=8, L=2048, k=4, 32/32 heads, d=128, bf16 paged KV, V=32000).

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
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--k", type=int, default=None, help="speculation length of the c3 sweep point")
    ap.add_argument("--alpha", type=float, default=None, help="acceptance level of the c3 sweep point")
    ap.add_argument("--rotate", type=int, default=0, help="device copies of KV/logits to cycle through (0 = auto)")
    ap.add_argument("--accept-mode", default="sample", choices=["sample", "greedy", "point"],
                    help="acceptance rule: the stochastic rule (headline), greedy, or stochastic against a point-mass draft")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the same steps")
    ap.add_argument("--events-in-value-region", action="store_true",
                    help="one timed region only: the K steps that give `value` also carry the kernel events "
                         "(an event pair attached to a launch costs about 4 us of wall clock per step)")
    return ap.parse_args()


def traffic_from_profile(workload):
    """HBM bytes per attention launch measured with rocprofv3 counters, if a summary is committed."""
    path = os.path.join(ROOT, "profiles", "spec_step_kernel_%s_pmc.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the step has no multi-GPU path); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_14066_amd import workloads as W
    from paper_2406_14066_amd import spec_verify as sv
    from paper_2406_14066_amd.harness import DeviceStep

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sv.lib()  # fail loudly if the HIP library is missing

    kw = {}
    if args.workload == "c3":
        kw = dict(k=args.k, alpha=args.alpha)
    w = W.config(args.workload, **kw)
    mode = {"sample": sv.ACCEPT_SAMPLE, "greedy": sv.ACCEPT_GREEDY, "point": sv.ACCEPT_POINT_DRAFT}[args.accept_mode]
    ds = DeviceStep(w, kv_layout=sv.KV_MFMA, with_debug=False, accept_mode=mode)

    attn_bytes = w.attn_algorithmic_bytes()
    # without a draft distribution only the target rows are read
    rej_bytes = w.reject_algorithmic_bytes() if mode == sv.ACCEPT_SAMPLE else w.T * w.V * 4
    step_bytes = attn_bytes + rej_bytes
    kv_bytes = 2 * ds.k_cache.numel() * ds.k_cache.element_size()
    # at least four copies and 4 GB in all: with two copies of a 1 GB workload the 256 MB
    # last-level cache still served a few per cent of the (non-temporal) reads
    nrot = args.rotate or max(4, int(np.ceil(4.0e9 / max(kv_bytes + rej_bytes, 1))))
    nrot = min(nrot, 16)

    # rotated copies: same bytes at different addresses
    variants = [(a, r, None) for a, r in ds.rotated(nrot)]

    stream = torch.cuda.current_stream()

    def run(n, first=0):
        for i in range(n):
            a, r, _ = variants[(first + i) % nrot]
            sv.spec_verify_step(a, r, ds.workspace, stream)

    run(args.warmup)
    torch.cuda.synchronize()

    # Two timed regions of exactly K steps each, both bracketed by a device synchronisation.  The
    # first carries nothing but the steps and gives `value`; the second attaches an event pair to
    # every launch (the kernel's own begin and end time stamps) and gives the kernel time of the
    # roofline.  The events are measurement: they cost about 4 us of wall clock per step, which a
    # serving loop would not pay.  --events-in-value-region folds the two into one.
    events_in_region = args.events_in_value_region
    if events_in_region:
        sv.spec_profile_begin(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, first=args.warmup)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if events_in_region:
        kt = sv.spec_profile_end()
        sec_per_step_events = (t1 - t0) / args.steps
    else:
        sv.spec_profile_begin(args.steps)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        run(args.steps, first=args.warmup)
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        kt = sv.spec_profile_end()
        sec_per_step_events = (t3 - t2) / args.steps

    sec_per_step = (t1 - t0) / args.steps
    value = w.verified_tokens() / sec_per_step

    # The same steps replayed from one captured HIP graph (one step per rotated copy): what is
    # left of the launch gaps when the host is out of the loop.  Reported beside the eager figure.
    graph_info = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(nrot):
                a, r, _ = variants[i]
                sv.spec_verify_step(a, r, ds.workspace, torch.cuda.current_stream())
        torch.cuda.synchronize()
        replays = max(args.steps // nrot, 1)
        for _ in range(max(args.warmup // nrot, 1)):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        graph_sec = (g1 - g0) / (replays * nrot)
        graph_info = {"ms_per_step": graph_sec * 1e3, "value": w.verified_tokens() / graph_sec,
                      "steps": replays * nrot, "steps_per_graph": nrot,
                      "achieved_GBps": step_bytes / graph_sec / 1e9}
    res = ds.results()
    emitted_per_step = int(res["counters"][3]) // max(int(res["counters"][5]) // w.B, 1)
    # logit bytes of the rows up to each request's first rejection: what the step needs at least
    # (the library reads no more than these when it takes the statistics pass in position order,
    # which it does for large batches with one draft length)
    m = res["accepted_len"].astype(np.int64)
    kk = w.k.astype(np.int64)
    rows_needed = (2 if mode == sv.ACCEPT_SAMPLE else 1) * np.minimum(m + 1, kk) + (m == kk)
    rej_bytes_needed = int(rows_needed.sum()) * w.V * 4

    kernel_us = {k: (1e3 * ms / n if n else None) for k, (ms, n) in kt.items()}
    step_us = kernel_us["step"]
    achieved = step_bytes / (step_us * 1e-6) / 1e9
    traffic = traffic_from_profile(args.workload) if mode == sv.ACCEPT_SAMPLE else None

    out = {
        "metric": "verified tokens/s per MI355X for spec-verify step",
        "value": value,
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
            "workload": "%s: B=%d, L=%s, k=%s, Hq/Hkv=%d/%d, d=%d, bf16 paged KV (block 16, shuffled table), V=%d fp32 logits"
                        % (w.name, w.B, _span(w.kv_len), _span(w.k), w.Hq, w.Hkv, w.d, w.V),
            "kv_layout": "mfma-tiled pages",
            "accept_mode": args.accept_mode,
            "rotated_copies": nrot,
            "verified_tokens_per_step": w.verified_tokens(),
            "emitted_tokens_per_step": emitted_per_step,
            "goodput_tokens_per_s": emitted_per_step / sec_per_step,
        },
        "step_hbm": {
            "algorithmic_bytes": step_bytes,
            "achieved_GBps": step_bytes / sec_per_step / 1e9,
            "frac_of_peak": step_bytes / sec_per_step / 1e9 / HBM_PEAK_GBS,
        },
        "kernel_us": kernel_us,
        "graph_replay": graph_info,
        "roofline": {
            "kernel": "spec_step_kernel (whole step in one launch: attention over the paged KV cache + rejection sampling)",
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "algorithmic_bytes_per_launch": step_bytes,
            "attention_bytes": attn_bytes,
            "rejection_bytes": rej_bytes,
            "rejection_bytes_up_to_first_rejection": rej_bytes_needed,
            "events_in_timed_region": True,
            "kernel_time_region": ("the K steps that give value" if events_in_region else
                                   "a second timed region of K steps with an event pair attached to every launch"),
            "ms_per_step_with_events": sec_per_step_events * 1e3,
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        # the oracle as it stands, single thread, on whole steps of this workload until about
        # ten seconds have passed (at least one step)
        reps, t_attn, t_rej = 0, 0.0, 0.0
        while reps == 0 or (t_attn + t_rej < 10.0 and reps < 1000):
            t2 = time.perf_counter()
            oracle.verify_attn(w.q, w.k_pages, w.v_pages, w.block_table, w.kv_len, w.cu_q_len)
            t3 = time.perf_counter()
            if mode == sv.ACCEPT_SAMPLE:
                oracle.reject_sample(w.target_logits, w.draft_logits, w.draft_tokens, w.cu_q_len, w.philox_seed,
                                     w.philox_step)
            elif mode == sv.ACCEPT_GREEDY:
                oracle.reject_greedy(w.target_logits, w.draft_tokens, w.cu_q_len)
            else:
                oracle.reject_onehot(w.target_logits, w.draft_tokens, w.cu_q_len, w.philox_seed, w.philox_step)
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
    print(json.dumps(out))


def _span(a):
    a = np.asarray(a)
    return str(int(a[0])) if (a == a[0]).all() else "%d..%d" % (a.min(), a.max())


if __name__ == "__main__":
    main()
